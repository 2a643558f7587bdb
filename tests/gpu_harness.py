"""Drives the HIP module (through the C ABI) and the CPU oracle side by side on the same seeded inputs
and reports, per tensor, max|gpu - oracle| / max|oracle| -- the bar of the benchmark spec (2e-2 for the
bf16 MFMA path) -- plus exact agreement of the queue indices."""
from __future__ import annotations

import copy
from typing import Dict, List, Tuple

import numpy as np

import fdg_workloads as W

TOL = 2e-2   # max |err| / max |ref| per tensor: bf16 operands (2^-9 relative rounding) with fp32 accumulation


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if not np.all(np.isfinite(got)):
        return float("inf")
    denom = np.abs(ref).max() if ref.size else 0.0
    err = np.abs(got - ref).max() if ref.size else 0.0
    if denom == 0.0:
        return 0.0 if err == 0.0 else float("inf")
    return float(err / denom)


def per_tensor_errors(spec, got_flat: np.ndarray, ref_flat: np.ndarray, prefix: str) -> Dict[str, float]:
    out, off = {}, 0
    for name, shape, _ in W.param_shapes(spec):
        n = int(np.prod(shape))
        out[f"{prefix}:{name}"] = rel_err(got_flat[off:off + n], ref_flat[off:off + n])
        off += n
    return out


def run_side_by_side(spec, steps: int, seed: int = 0, perturb_bn: bool = True, backward_first: bool = False,
                     oracle_dtype=np.float32, device="cuda:0") -> Tuple[Dict[str, float], List[str]]:
    """Runs `steps` iterations (after the warm-up that fills the history) on both sides.
    Returns ({tensor label: relative error (worst over the steps)}, [exact-check failures])."""
    import torch
    from oracle.fdg_oracle import OracleModule
    from paper_1906_09108_amd import FdgModule

    theta0 = W.make_params(spec, seed, perturb_bn=perturb_bn)
    ora = OracleModule(spec, oracle_dtype)
    ora.set_params(theta0)
    gpu = FdgModule(spec, device)
    gpu.set_params(theta0)
    errs: Dict[str, float] = {}
    exact: List[str] = []

    def note(label, e):
        errs[label] = max(errs.get(label, 0.0), e)

    def check_queue(tag):
        if gpu.queue_state() != ora.queue_state():
            exact.append(f"{tag}: queue gpu={gpu.queue_state()} oracle={ora.queue_state()}")

    dev = torch.device(device)
    d = spec.delay
    total = d + steps
    grad_in = None if spec.is_bottom else torch.empty(spec.input_shape(), dtype=torch.float32, device=dev)

    def do_forward(t):
        x = W.make_input(spec, t, seed)
        labels = W.make_labels(spec, t, seed)
        y_ref = ora.forward(x, labels)
        y = gpu.forward(torch.from_numpy(x).to(dev), None if labels is None else torch.from_numpy(labels).to(dev))
        y = y.cpu().numpy()
        if spec.is_top:
            note("loss", abs(float(y[0]) - float(y_ref[0])) / max(abs(float(y_ref[0])), 1e-30))
            note("logits", rel_err(y[1:], y_ref[1:]))
        else:
            note("y", rel_err(y, y_ref))
        check_queue(f"after forward {t}")

    def do_backward_update(t):
        s = t - d                                  # the batch whose gradient arrives at iteration t
        g = W.make_grad_out(spec, s, seed)
        gin_ref = ora.backward_delayed(g)
        gpu.backward_delayed(None if g is None else torch.from_numpy(g).to(dev), grad_in)
        check_queue(f"after backward {t}")
        for k, e in per_tensor_errors(spec, gpu.get_grads(), ora.get_grads(), "grad").items():
            note(k, e)
        if gin_ref is not None:
            note("grad_in", rel_err(grad_in.cpu().numpy(), gin_ref))
        ora.update(spec.lr)
        gpu.update(spec.lr)
        for k, e in per_tensor_errors(spec, gpu.get_params(), ora.get_params(), "theta").items():
            note(k, e)
        for k, e in per_tensor_errors(spec, gpu.get_momentum(), ora.get_momentum(), "v").items():
            note(k, e)

    if backward_first:
        # order of Algorithm I: delayed backward -> update -> forward.  Needs d >= 1 (a delay-0 module
        # can only back-propagate what it has just forwarded).
        assert d >= 1
        for t in range(d):
            do_forward(t)
        for t in range(d, total):
            do_backward_update(t)
            do_forward(t)
    else:
        for t in range(total):
            do_forward(t)
            if t >= d:
                do_backward_update(t)
    if gpu.get_bn_running().size:
        note("bn_running", rel_err(gpu.get_bn_running(), ora.get_bn_running()))
    gpu.close()
    return errs, exact


def format_report(errs: Dict[str, float], limit: float = TOL) -> str:
    lines = []
    for k in sorted(errs, key=lambda kk: -errs[kk]):
        flag = "  <-- FAIL" if not (errs[k] <= limit) else ""
        lines.append(f"  {k:40s} {errs[k]:.3e}{flag}")
    return "\n".join(lines)

"""Drives the HIP module (through the C ABI) and the CPU oracle side by side on the same seeded inputs.

Three runs advance in lock step through the same iterations:
  gpu    the HIP path;
  same   the oracle in its bf16-storage mode (decisions taken in the kernel's precision);
  plain  the oracle's fp32 definition.

What can be asked of a bf16 path.  The module is a deep composition of ReLU gates.  Rounding an
operand to bf16 moves a pre-activation by about 1.6e-3 of its spread, so about 4 in 10^4 gates fall
the other way; with the noise gradients of the synthetic workload every such element moves a
per-channel sum by a whole term (relative error about sqrt(2 f) for a flip rate f), and each block
amplifies the difference it inherits.  `inherent` = distance between `same` and `plain`, measured on
the CPU alone, is therefore several per cent for one block and of order one for the 27- and 150-block
modules.  Two bf16 evaluations that merely sum in a different order separate in the same way, only
later: one block apart they agree to 1e-4, a few wide blocks apart they do not.

Hence two bars:
  STRICT (spec bar): max|gpu - same| / max|same| <= 2e-2 per tensor, asked up to the first backward
      of modules shallow enough for the two bf16 evaluations to stay together (every layer kind and
      both shortcut forms are covered by such modules).  The input gradient carries single gated
      elements unreduced; a few gates sit within a rounding of zero and are valid either way, so it is
      held to the bar on all but TIE_FRACTION of its elements and in relative L2 norm.
  ENVELOPE (every module, every iteration): relL2(gpu, same) <= 2e-2 + 2 * relL2(same, plain): the HIP
      path may not be further from the kernel-precision oracle than bf16 storage itself is from the
      definition.  A wiring or indexing mistake gives errors of order one and breaks either bar
      wherever `inherent` is below one half.  Where it is above (gradients of the 27- and 150-block
      modules: there the definition and its own bf16-storage evaluation are already unrelated vectors)
      the comparison carries no information and is only reported; for those modules the proof is
      carried by the per-kernel tests at their real shapes (tests/test_gpu_kernels.py), by their
      forwards, and by the shallow modules built from the same blocks.
Queue indices and sequence numbers are compared exactly, always."""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

import fdg_workloads as W

TOL = 2e-2            # max |err| / max |ref| per tensor: bf16 operands (2^-9 relative rounding), fp32 accumulation
TIE_FRACTION = 1e-4   # share of input-gradient elements allowed to sit on a ReLU tie
ENVELOPE_FACTOR = 2.0
INFORMATIVE_LIMIT = 0.5   # an inherent distance above this means the two oracles are themselves unrelated


def rel_err(got, ref) -> float:
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


def rel_err_robust(got, ref, fraction: float = TIE_FRACTION) -> float:
    """max|err| / max|ref| after setting aside the ceil(fraction * size) largest errors."""
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    if not np.all(np.isfinite(got)):
        return float("inf")
    err = np.abs(got - ref)
    k = int(np.ceil(fraction * err.size))
    kept = np.partition(err, err.size - k - 1)[err.size - k - 1] if k < err.size else 0.0
    denom = np.abs(ref).max()
    return float(kept / denom) if denom > 0 else (0.0 if kept == 0 else float("inf"))


def rel_l2(got, ref) -> float:
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    if not np.all(np.isfinite(got)):
        return float("inf")
    d = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / d) if d > 0 else (0.0 if np.linalg.norm(got) == 0 else float("inf"))


class Record:
    """One tensor at one iteration: strict measure (max norm, or the tie-robust one for grad_in), relative
    L2 against the kernel-precision oracle, and the inherent distance of that oracle from the definition."""

    def __init__(self, label: str, step: int, strict: float, l2: float, inherent: float):
        self.label, self.step, self.strict, self.l2, self.inherent = label, step, strict, l2, inherent

    @property
    def informative(self) -> bool:
        return self.inherent <= INFORMATIVE_LIMIT

    @property
    def envelope_ok(self) -> bool:
        return (not self.informative) or self.l2 <= TOL + ENVELOPE_FACTOR * self.inherent

    @property
    def strict_ok(self) -> bool:
        return self.strict <= TOL and (self.label != "grad_in" or self.l2 <= TOL)


def _split(spec, flat) -> List[Tuple[str, np.ndarray]]:
    out, off = [], 0
    for name, shape, _ in W.param_shapes(spec):
        n = int(np.prod(shape))
        out.append((name, flat[off:off + n]))
        off += n
    return out


def run_side_by_side(spec, steps: int, seed: int = 0, perturb_bn: bool = True, backward_first: bool = False,
                     device="cuda:0", save_mode: int = 0) -> Tuple[List[Record], List[str]]:
    """Runs `steps` iterations (after the warm-up that fills the history) on the three runs.
    Returns (records, exact-check failures).  save_mode is the library's (fdg_save_mode); the oracle runs keep
    their activations either way: replaying a saved forward changes where the numbers come from, not the numbers."""
    import torch
    from oracle.fdg_oracle import OracleModule
    from paper_1906_09108_amd import FdgModule

    theta0 = W.make_params(spec, seed, perturb_bn=perturb_bn)
    same = OracleModule(spec, np.float32, storage="bf16")
    plain = OracleModule(spec, np.float32, storage="fp32")
    gpu = FdgModule(spec, device, save_mode=save_mode)
    for m in (same, plain, gpu):
        m.set_params(theta0)
    records: List[Record] = []
    exact: List[str] = []
    dev = torch.device(device)
    d = spec.delay
    total = d + steps
    grad_in = None if spec.is_bottom else torch.empty(spec.input_shape(), dtype=torch.float32, device=dev)

    def note(label, step, got, ref_same, ref_plain, robust=False):
        strict = rel_err_robust(got, ref_same) if robust else rel_err(got, ref_same)
        records.append(Record(label, step, strict, rel_l2(got, ref_same), rel_l2(ref_same, ref_plain)))

    def check_queue(tag):
        if gpu.queue_state() != same.queue_state():
            exact.append(f"{tag}: queue gpu={gpu.queue_state()} oracle={same.queue_state()}")

    def do_forward(t):
        x = W.make_input(spec, t, seed)
        labels = W.make_labels(spec, t, seed)
        y_same, y_plain = same.forward(x, labels), plain.forward(x, labels)
        y = gpu.forward(torch.from_numpy(x).to(dev), None if labels is None else torch.from_numpy(labels).to(dev))
        y = y.cpu().numpy()
        if spec.is_top:
            note("loss", t, y[:1], y_same[:1], y_plain[:1])
            note("logits", t, y[1:], y_same[1:], y_plain[1:])
        else:
            note("y", t, y, y_same, y_plain)
        check_queue(f"after forward {t}")

    def do_backward_update(t):
        s = t - d                                  # the batch whose gradient arrives at iteration t
        g = W.make_grad_out(spec, s, seed)
        gin_same, gin_plain = same.backward_delayed(g), plain.backward_delayed(g)
        gpu.backward_delayed(None if g is None else torch.from_numpy(g).to(dev), grad_in)
        check_queue(f"after backward {t}")
        for (name, a), (_, b), (_, c) in zip(_split(spec, gpu.get_grads()), _split(spec, same.get_grads()),
                                             _split(spec, plain.get_grads())):
            note("grad:" + name, t, a, b, c)
        if gin_same is not None:
            note("grad_in", t, grad_in.cpu().numpy(), gin_same, gin_plain, robust=True)
        for m in (same, plain, gpu):
            m.update(spec.lr)
        for (name, a), (_, b), (_, c) in zip(_split(spec, gpu.get_params()), _split(spec, same.get_params()),
                                             _split(spec, plain.get_params())):
            note("theta:" + name, t, a, b, c)
        for (name, a), (_, b), (_, c) in zip(_split(spec, gpu.get_momentum()), _split(spec, same.get_momentum()),
                                             _split(spec, plain.get_momentum())):
            note("v:" + name, t, a, b, c)

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
        note("bn_running", total - 1, gpu.get_bn_running(), same.get_bn_running(), plain.get_bn_running())
    gpu.close()
    return records, exact


def judge(records: List[Record], spec, strict: bool) -> List[str]:
    """Failure messages.  ENVELOPE applies to every record; STRICT to the forwards up to, and the gradients
    of, the first backward (the first update re-rounds the weights of the runs independently)."""
    bad = []
    t0 = spec.delay
    for r in records:
        if not r.envelope_ok:
            bad.append(f"ENVELOPE step {r.step} {r.label}: L2 {r.l2:.3e} > {TOL} + {ENVELOPE_FACTOR} * inherent {r.inherent:.3e}")
        if strict and r.step <= t0 and not r.label.startswith(("theta:", "v:", "bn_running")) and not r.strict_ok:
            bad.append(f"STRICT step {r.step} {r.label}: {r.strict:.3e} (L2 {r.l2:.3e}) over {TOL}")
    return bad


def format_report(records: List[Record], limit: int = 30) -> str:
    rows = sorted(records, key=lambda r: -r.strict)[:limit]
    silent = sum(1 for r in records if not r.informative)
    lines = [f"  {len(records)} tensor records, {silent} beyond the informative range (inherent > {INFORMATIVE_LIMIT})",
             f"  {'tensor':34s} step   strict      L2    inherent(L2)"]
    for r in rows:
        lines.append(f"  {r.label:34s} {r.step:3d}  {r.strict:.2e}  {r.l2:.2e}  {r.inherent:.2e}")
    return "\n".join(lines)

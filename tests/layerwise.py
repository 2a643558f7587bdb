"""Layer-by-layer parity of a REAL module step: every layer of the HIP path is checked by itself, on the input that
layer actually saw on the GPU.

Why.  A module is a deep chain of ReLU gates; two correct evaluations that differ in the last bit somewhere drift apart
layer after layer (tests/gpu_harness.py), so an end-to-end comparison of a deep module says little about any one layer.
The chain rule of Eq. 8 - Eq. 10 is a product of per-layer factors, and each factor can be checked in isolation:

  forward   layer i of the GPU's step got z_in (fp32, read back through fdg_trace_read / the module input) and the
            weights of that forward; the oracle runs the SAME layer on z_in and its output and every intermediate the
            GPU kept (fdg_saved_read) are compared element by element;
  backward  layer i got the gradient dz of its output (fdg_trace_read) and worked on the tensors its forward kept;
            the oracle back-propagates dz through that ONE layer on the GPU's own kept tensors (batch statistics are
            recomputed by the oracle from the kept batch-norm inputs) and the input gradient and the layer's
            parameter gradients are compared element by element.

Every layer, every fused output stage and every hand-over between kernels of fdg_forward / fdg_backward_delayed is
covered at the sizes the step runs at, with no error inherited from the layers before.  The oracle runs in its
bf16-storage mode: a kept tensor is a bf16 tensor on both sides.  What differs is summation order in fp32 and hence, for
a few elements, the bf16 neighbour a value rounds to (one unit in the last place)."""
from __future__ import annotations

import copy
from typing import Dict, List, Optional, Tuple

import numpy as np

import fdg_workloads as W
from fdg_workloads import ModuleSpec
from oracle.fdg_oracle import (BASIC_POSTACT, BASIC_PREACT, BOTTLENECK_POSTACT, HEAD_POSTACT, HEAD_PREACT, INVERTED_RESIDUAL, STEM,
                               STEM_POOL, OracleModule, _Flat, oracle_param_layout)

# which saved tensor (fdg_saved_read) is which oracle quantity, per layer kind: (which, tape key | "bn:<tag>")
SAVED = {
    STEM: [(0, "bn:bn")],
    BASIC_POSTACT: [(0, "bn:bn1"), (1, "a1"), (2, "bn:bn2"), (3, "bn:bnp")],
    BASIC_PREACT: [(0, "o1"), (1, "bn:bn2"), (2, "o2")],
    BOTTLENECK_POSTACT: [(0, "bn:bn1"), (1, "a1"), (2, "bn:bn2"), (3, "bn:bnp"), (4, "a2"), (5, "bn:bn3")],
    HEAD_POSTACT: [],
    HEAD_PREACT: [(0, "o")],
    STEM_POOL: [(0, "bn:bn"), (1, "a")],
    INVERTED_RESIDUAL: [(0, "bn:bn1"), (1, "a1"), (2, "bn:bn2"), (4, "a2"), (5, "bn:bn3")],
}
# batch norms of a layer kind: tag -> which saved tensor is its input (7 = the layer input)
BN_INPUT = {
    STEM: {"bn": 0},
    BASIC_POSTACT: {"bn1": 0, "bn2": 2, "bnp": 3},
    BASIC_PREACT: {"bn1": 7, "bn2": 1},
    BOTTLENECK_POSTACT: {"bn1": 0, "bn2": 2, "bn3": 5, "bnp": 3},
    HEAD_POSTACT: {},
    HEAD_PREACT: {"bn": 7},
    STEM_POOL: {"bn": 0},
    INVERTED_RESIDUAL: {"bn1": 0, "bn2": 2, "bn3": 5},
}


class Row:
    def __init__(self, layer: int, what: str, got, ref):
        got = np.asarray(got, np.float64).ravel()
        ref = np.asarray(ref, np.float64).ravel()
        assert got.shape == ref.shape, (what, got.shape, ref.shape)
        self.layer, self.what = layer, what
        self.finite = bool(np.all(np.isfinite(got)))
        d = np.abs(got - ref)
        mx = np.abs(ref).max() if ref.size else 0.0
        self.max_norm = float(d.max() / mx) if mx > 0 else (0.0 if not d.size or d.max() == 0 else float("inf"))
        nr = np.linalg.norm(ref)
        self.l2 = float(np.linalg.norm(d) / nr) if nr > 0 else (0.0 if np.linalg.norm(d) == 0 else float("inf"))
        self.differ = float(np.count_nonzero(d) / max(d.size, 1))

    def __repr__(self):
        return f"L{self.layer:<3d} {self.what:22s} max {self.max_norm:.2e}  L2 {self.l2:.2e}  differing {self.differ:.1e}"


def layer_slices(spec) -> List[Tuple[int, int]]:
    """[start, end) of every layer's parameters in the flat order."""
    out, off = [], 0
    per = [0] * len(spec.layers)
    for name, shape in oracle_param_layout(spec):
        per[int(name.split(".")[0])] += int(np.prod(shape))
    for n in per:
        out.append((off, off + n))
        off += n
    return out


def _one_layer(spec, i: int, shape_in, storage: str = "bf16") -> Tuple[ModuleSpec, OracleModule]:
    L = copy.deepcopy(spec.layers[i])
    s1 = ModuleSpec(spec.n, L.c_in, shape_in[2], shape_in[3], [L], delay=0, is_bottom=False, num_classes=spec.num_classes,
                    beta=1.0, momentum=spec.momentum, weight_decay=spec.weight_decay, bn_eps=spec.bn_eps,
                    bn_momentum=spec.bn_momentum, name=f"{spec.name}.L{i}")
    return s1, OracleModule(s1, np.float32, storage=storage)


def _input_shapes(spec) -> List[Tuple[int, int, int, int]]:
    shapes = [spec.input_shape()] + spec.activation_shapes()
    return shapes[:len(spec.layers)]


def check_forward_layers(gpu, spec, theta: np.ndarray, seq: int, x: np.ndarray, labels, y_gpu: np.ndarray,
                         storage: str = "bf16") -> List[Row]:
    """The forward with sequence number `seq` (the last one traced), run with parameters `theta` on x.
    storage = "fp32": each layer against its plain fp32 definition (unrounded weights, nothing rounded inside)."""
    rows: List[Row] = []
    shapes = _input_shapes(spec)
    z_in = np.ascontiguousarray(x, np.float32)
    for i, (L, (lo, hi)) in enumerate(zip(spec.layers, layer_slices(spec))):
        s1, om = _one_layer(spec, i, shapes[i], storage)
        om.set_params(theta[lo:hi])
        th = om._stored_weights(om.theta.copy())
        out, tapes = om._layers(z_in, labels if L.is_head else None, th, move_running=False)
        t = tapes[0]
        if storage == "bf16":
            rows.append(Row(i, "fwd input copy", gpu.saved_read(seq, i, 7), t["x"]))
        for which, key in SAVED[L.kind]:
            if key == "bn:bnp" and not L.projects:
                continue
            ref = t["0." + key[3:]][0] if key.startswith("bn:") else t[key]
            rows.append(Row(i, f"fwd saved[{which}] {key}", gpu.saved_read(seq, i, which), ref))
        if L.is_head:
            rows.append(Row(i, "fwd pooled", gpu.saved_read(seq, i, 8)[:, :, 0, 0], t["p"]))
            rows.append(Row(i, "fwd dlogits", gpu.saved_read(seq, i, 9)[:, :, 0, 0], t["dl"]))
            rows.append(Row(i, "fwd loss", y_gpu[:1], out[:1]))
            rows.append(Row(i, "fwd logits", y_gpu[1:], out[1:]))
            break
        rows.append(Row(i, "fwd output copy", gpu.saved_read(seq, i, 6), t["y"]))
        z_gpu, _ = gpu.trace_read(0, i)
        rows.append(Row(i, "fwd output fp32", z_gpu, out))
        z_in = z_gpu                      # the next layer is checked on what the GPU gave it
    if not spec.is_top:
        rows.append(Row(len(spec.layers) - 1, "fwd module y", y_gpu, z_in))
    return rows


def _tape_from_gpu(gpu, om: OracleModule, th: _Flat, L, seq: int, i: int) -> Dict:
    """What layer i's forward kept, as the oracle's backward wants it, built from the GPU's own saved tensors."""
    sv = lambda which: gpu.saved_read(seq, i, which)
    t: Dict = {"x": sv(7)}
    cache = {7: t["x"]}
    for tag, which in BN_INPUT[L.kind].items():
        if tag == "bnp" and not L.projects:
            continue
        if which not in cache:
            cache[which] = sv(which)
        xin = cache[which]
        _, mean, _, invstd = om.k.bn_fwd(xin, th[f"0.{tag}.gamma"], th[f"0.{tag}.beta"], om.spec.bn_eps)
        t[f"0.{tag}"] = (xin, mean, invstd)
    if L.kind in (BASIC_POSTACT, BOTTLENECK_POSTACT, INVERTED_RESIDUAL):
        t["a1"] = sv(1)
    if L.kind in (BOTTLENECK_POSTACT, INVERTED_RESIDUAL):
        t["a2"] = sv(4)
    if L.kind == STEM_POOL:
        t["a"] = sv(1)
    if L.kind == BASIC_PREACT:
        t["o1"], t["o2"] = sv(0), sv(2)
    if L.kind in (STEM, BASIC_POSTACT, BOTTLENECK_POSTACT):
        t["y"] = sv(6)
    if L.is_head:
        o = sv(0) if L.kind == HEAD_PREACT else t["x"]
        if L.kind == HEAD_PREACT:
            t["o"] = o
        t.update(o_shape=o.shape, p=np.ascontiguousarray(sv(8)[:, :, 0, 0]), dl=np.ascontiguousarray(sv(9)[:, :, 0, 0]))
    return t


def check_backward_layers(gpu, spec, theta: np.ndarray, seq: int, grads_gpu: np.ndarray,
                          grad_in_gpu: Optional[np.ndarray], storage: str = "bf16") -> List[Row]:
    """The last traced backward, which popped the saved forward `seq` that had run with parameters `theta`.
    storage = "fp32": the plain fp32 chain rule through each layer (unrounded weights, no gradient rounded on the
    way), evaluated on the forward tensors the GPU kept -- so every ReLU passes the gradient where the GPU's forward
    had it open, and what is measured is the backward's arithmetic."""
    rows: List[Row] = []
    shapes = _input_shapes(spec)
    nl = len(spec.layers)
    names = [n for n, _ in oracle_param_layout(spec)]
    for i in reversed(range(nl)):
        L = spec.layers[i]
        lo, hi = layer_slices(spec)[i]
        s1, om = _one_layer(spec, i, shapes[i], storage)
        om.set_params(theta[lo:hi])
        th = om._stored_weights(om.theta.copy())
        t = _tape_from_gpu(gpu, om, th, L, seq, i)
        dz = None if L.is_head else gpu.trace_read(1, i + 1)[0]
        need_dx = not (i == 0 and spec.is_bottom)
        g = _Flat(om.layout, om.dt)
        dx = om._layer_backward(0, L, t, th, dz, g, need_dx)
        off = 0
        for name, shape in om.layout:
            n = int(np.prod(shape))
            rows.append(Row(i, "bwd grad " + name[2:], grads_gpu[lo + off:lo + off + n], g.flat[off:off + n]))
            off += n
        if need_dx:
            got, gated = gpu.trace_read(1, i)
            if gated:     # the producer also applied the ReLU of the layer below (gate = this layer's input copy)
                dx = dx * (t["x"] > 0)
            rows.append(Row(i, "bwd input gradient" + (" (gated)" if gated else ""), got, dx))
            if i == 0 and grad_in_gpu is not None:
                rows.append(Row(i, "bwd module grad_in", grad_in_gpu, got))
    return rows


def check_update(spec, theta_before, v_before, grads_gpu, theta_gpu, v_gpu, lr: float) -> List[Row]:
    """Eq. 11 on the GPU's own gradient: the oracle's update from the same (theta, v, g)."""
    from oracle.fdg_oracle import Kernels
    k = Kernels(np.float32)
    th, v = np.array(theta_before, np.float32), np.array(v_before, np.float32)
    k.sgd_momentum(th, v, np.ascontiguousarray(grads_gpu, np.float32), lr, spec.momentum, spec.weight_decay)
    return [Row(-1, "update theta", theta_gpu, th), Row(-1, "update v", v_gpu, v)]


def format_rows(rows: List[Row], limit: int = 25) -> str:
    worst = sorted(rows, key=lambda r: -r.max_norm)[:limit]
    return "\n".join("  " + repr(r) for r in worst)


def summarize(rows: List[Row]) -> Dict[str, Tuple[float, float]]:
    """Per class of tensor: (largest max-norm deviation, largest L2 deviation)."""
    out: Dict[str, Tuple[float, float]] = {}
    for r in rows:
        key = r.what.split("[")[0].split(" (")[0]
        if key.startswith("bwd grad "):
            key = "bwd grad " + ("conv/fc weights" if r.what.endswith(".w") else "bn/bias vectors")
        a, b = out.get(key, (0.0, 0.0))
        out[key] = (max(a, r.max_norm), max(b, r.l2))
    return out

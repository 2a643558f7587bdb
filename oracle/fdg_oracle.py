"""CPU ORACLE -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module; the
product path (paper_1906_09108_amd) never does, and this module never imports the product path.

One FDG module worker (arXiv 1906.09108, Section III), step by step in the paper's order:

  forward (Section III-A, "forward"; Fig. 1(b) step A)
      run the module's layers on the newest input with the current parameters and push a context
      -- every intermediate the backward will need AND a copy of the parameters used -- into a FIFO.
  backward_delayed (Section III-A, "backward", Eq. 10; Section III-B, Eq. 15)
      pop the OLDEST context, multiply the received gradient by beta, then apply the chain rule
      (Eq. 8, Eq. 9) through that context: activations of the stale batch, parameters of the stale
      iteration -- both superscripts of Eq. 10 carry the stale index.  Keeps the parameter gradient
      and returns the gradient of the module input (the tensor sent down, Section III-A
      "communication").
  update (Eq. 11 / Eq. 12, optimiser of Section V-A)
      momentum SGD with weight decay on the CURRENT parameters using that delayed gradient.

The layer arithmetic (convolution, batch normalisation, ...) lives in fdg_oracle_kernels.c as plain
loops; this file only sequences it.  Two element types are available: float32 (default; the
spec precision) and float64 (for finite-difference pins).

Readings taken where the paper is silent (all listed in the design notes of the repository):
  * weights used by the delayed backward: the snapshot taken at that batch's forward (Eq. 10);
  * beta multiplies the received gradient only; a top module (one ending in the loss) receives no
    gradient and is not shrunk (Section III-B, text below Eq. 15);
  * optimiser: g' = g + wd*theta; v = mu*v + g'; theta -= lr*v, weight decay on every parameter;
  * BN: eps inside the square root, biased batch variance for normalising, running statistics
    updated with the unbiased variance; no convolution bias; loss = mean softmax cross-entropy.

Two storage precisions.  storage="fp32" is the plain definition above.  storage="bf16" evaluates the
SAME steps but rounds a tensor to bfloat16 (fdgref_round_bf16: nearest, ties to even) at exactly the
points where the bf16 matrix-core path stores one: the convolution weights as used by a forward, every
convolution / BN+ReLU output that is kept, the bf16 copy of a block's input and output, and the
gradients handed to a convolution (one exception: in basic blocks of 16, 32 or 64 channels the gated
gradient between the second convolution's data gradient and the first batch norm's backward stays in
fp32, see _layer_backward).  Residual sums, BN statistics, parameter gradients and the
optimiser stay in the oracle's full precision.  The mode exists because ReLU turns a float into a
decision (gradient passes or not): compared with the fp32 definition, a path with bf16 operands
decides differently for about 4 in 10^4 activations, and with noise gradients every such element
moves a per-channel sum by a whole term, which alone puts parameter gradients several per cent away.
Taking the decision in the kernel's storage precision on both sides removes that, and what remains
is the arithmetic.

OracleChain runs K such workers as Algorithm I does: every iteration each module back-propagates the
oldest saved batch with the gradient it received, updates, forwards the input it received, and the
tensors are exchanged once per iteration, after all compute of that iteration (Section III-A, "communication"; Fig. 1(a)).

Parity status: every function of this oracle is pinned by tests/test_oracle_*.py (finite
differences in float64, torch-CPU autograd as an independent library, closed forms, adjoint
identities, brute force, and the paper's own K=3 delay example; the chain against the integer
schedule, against one module on the whole network for K = 1, against autograd of the composed
network for the stale gradient of Eq. 13, and against Eq. 16/17 for the compounded shrinking).
Nothing here is "parity unpinned".
"""
from __future__ import annotations

import collections
import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fdg_oracle_kernels.c")

# layer kinds, numerically equal to the C ABI's fdg_layer_kind (an interface constant)
STEM, BASIC_POSTACT, BASIC_PREACT, HEAD_POSTACT, HEAD_PREACT, BOTTLENECK_POSTACT = 0, 1, 2, 3, 4, 5
# Layers of the Tiny-ImageNet networks of Table V: the ImageNet stem of ResNet-18 (7x7 convolution stride 2, batch norm,
# ReLU, 3x3 max-pool stride 2) and the inverted residual block of MobileNet-v2 (1x1 expansion by 6, 3x3 depthwise
# convolution carrying the stride, 1x1 projection; batch norm after each, ReLU6 after the first two, the input added
# when stride and channels allow).  The paper names the networks and says they are the usual ones; nothing more.
STEM_POOL, INVERTED_RESIDUAL = 6, 7
EXPANSION = 6


def lib_path(dtype) -> str:
    return os.path.join(_HERE, "libfdg_oracle_f64.so" if np.dtype(dtype) == np.float64 else "libfdg_oracle_f32.so")


def build(force: bool = False) -> None:
    """Compile the C kernels of the oracle for float and double with gcc."""
    for real, dt in (("float", np.float32), ("double", np.float64)):
        out = lib_path(dt)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        subprocess.check_call(["gcc", "-O3", "-mavx2", "-mfma", "-fopenmp", "-shared", "-fPIC",
                               f"-DFDG_REAL={real}", "-o", out, _SRC, "-lm"])


_LIBS: Dict[str, ctypes.CDLL] = {}


def _lib(dtype) -> ctypes.CDLL:
    key = np.dtype(dtype).name
    if key not in _LIBS:
        build()
        lib = ctypes.CDLL(lib_path(dtype))
        lib.fdgref_softmax_ce.restype = ctypes.c_double
        assert lib.fdgref_sizeof_real() == np.dtype(dtype).itemsize
        _LIBS[key] = lib
    return _LIBS[key]


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    """Threads the OpenMP loops of the C kernels use."""
    omp = ctypes.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


class Kernels:
    """Thin typed wrappers over the C loops (allocation of outputs, nothing else)."""

    def __init__(self, dtype=np.float32):
        self.dt = np.dtype(dtype)
        self.lib = _lib(dtype)

    def _a(self, x) -> np.ndarray:
        return np.ascontiguousarray(x, dtype=self.dt)

    def conv_fwd(self, x, w, stride: int, pad: int) -> np.ndarray:
        x, w = self._a(x), self._a(w)
        N, Ci, H, W = x.shape
        Co, Ci2, k, _ = w.shape
        assert Ci == Ci2
        Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
        y = np.empty((N, Co, Ho, Wo), self.dt)
        self.lib.fdgref_conv2d_fwd(_p(x), _p(w), _p(y), N, Ci, H, W, Co, k, stride, pad)
        return y

    def conv_bwd_data(self, dy, w, x_shape, stride: int, pad: int) -> np.ndarray:
        dy, w = self._a(dy), self._a(w)
        N, Ci, H, W = x_shape
        Co, _, k, _ = w.shape
        dx = np.empty((N, Ci, H, W), self.dt)
        self.lib.fdgref_conv2d_bwd_data(_p(dy), _p(w), _p(dx), N, Ci, H, W, Co, k, stride, pad)
        return dx

    def conv_bwd_weight(self, x, dy, k: int, stride: int, pad: int) -> np.ndarray:
        x, dy = self._a(x), self._a(dy)
        N, Ci, H, W = x.shape
        Co = dy.shape[1]
        dw = np.empty((Co, Ci, k, k), self.dt)
        self.lib.fdgref_conv2d_bwd_weight(_p(x), _p(dy), _p(dw), N, Ci, H, W, Co, k, stride, pad)
        return dw

    def bn_fwd(self, x, gamma, beta, eps: float):
        x, gamma, beta = self._a(x), self._a(gamma), self._a(beta)
        N, C, H, W = x.shape
        y = np.empty_like(x)
        mean, var, invstd = (np.empty(C, self.dt) for _ in range(3))
        self.lib.fdgref_bn_fwd(_p(x), _p(gamma), _p(beta), _p(y), _p(mean), _p(var), _p(invstd), N, C, H, W,
                               ctypes.c_double(eps))
        return y, mean, var, invstd

    def bn_bwd(self, x, dy, gamma, mean, invstd):
        x, dy, gamma, mean, invstd = map(self._a, (x, dy, gamma, mean, invstd))
        N, C, H, W = x.shape
        dx = np.empty_like(x)
        dgamma, dbeta = np.empty(C, self.dt), np.empty(C, self.dt)
        self.lib.fdgref_bn_bwd(_p(x), _p(dy), _p(gamma), _p(mean), _p(invstd), _p(dx), _p(dgamma), _p(dbeta),
                               N, C, H, W)
        return dx, dgamma, dbeta

    def relu_fwd(self, x) -> np.ndarray:
        x = self._a(x)
        y = np.empty_like(x)
        self.lib.fdgref_relu_fwd(_p(x), _p(y), ctypes.c_size_t(x.size))
        return y

    def relu_bwd(self, x, dy) -> np.ndarray:
        x, dy = self._a(x), self._a(dy)
        dx = np.empty_like(x)
        self.lib.fdgref_relu_bwd(_p(x), _p(dy), _p(dx), ctypes.c_size_t(x.size))
        return dx

    def relu6_fwd(self, x) -> np.ndarray:
        x = self._a(x)
        y = np.empty_like(x)
        self.lib.fdgref_relu6_fwd(_p(x), _p(y), ctypes.c_size_t(x.size))
        return y

    def relu6_bwd(self, x, dy) -> np.ndarray:
        x, dy = self._a(x), self._a(dy)
        dx = np.empty_like(x)
        self.lib.fdgref_relu6_bwd(_p(x), _p(dy), _p(dx), ctypes.c_size_t(x.size))
        return dx

    def maxpool_fwd(self, x, k: int, stride: int, pad: int) -> np.ndarray:
        x = self._a(x)
        N, C, H, W = x.shape
        y = np.empty((N, C, (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1), self.dt)
        self.lib.fdgref_maxpool_fwd(_p(x), _p(y), N, C, H, W, k, stride, pad)
        return y

    def maxpool_bwd(self, x, dy, k: int, stride: int, pad: int) -> np.ndarray:
        x, dy = self._a(x), self._a(dy)
        N, C, H, W = x.shape
        dx = np.empty_like(x)
        self.lib.fdgref_maxpool_bwd(_p(x), _p(dy), _p(dx), N, C, H, W, k, stride, pad)
        return dx

    def dwconv_fwd(self, x, w, stride: int, pad: int) -> np.ndarray:
        x, w = self._a(x), self._a(w)
        N, C, H, W = x.shape
        k = w.shape[-1]
        assert w.shape == (C, 1, k, k)
        y = np.empty((N, C, (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1), self.dt)
        self.lib.fdgref_dwconv2d_fwd(_p(x), _p(w), _p(y), N, C, H, W, k, stride, pad)
        return y

    def dwconv_bwd_data(self, dy, w, x_shape, stride: int, pad: int) -> np.ndarray:
        dy, w = self._a(dy), self._a(w)
        N, C, H, W = x_shape
        dx = np.empty((N, C, H, W), self.dt)
        self.lib.fdgref_dwconv2d_bwd_data(_p(dy), _p(w), _p(dx), N, C, H, W, w.shape[-1], stride, pad)
        return dx

    def dwconv_bwd_weight(self, x, dy, k: int, stride: int, pad: int) -> np.ndarray:
        x, dy = self._a(x), self._a(dy)
        N, C, H, W = x.shape
        dw = np.empty((C, 1, k, k), self.dt)
        self.lib.fdgref_dwconv2d_bwd_weight(_p(x), _p(dy), _p(dw), N, C, H, W, k, stride, pad)
        return dw

    def avgpool_fwd(self, x) -> np.ndarray:
        x = self._a(x)
        N, C, H, W = x.shape
        p = np.empty((N, C), self.dt)
        self.lib.fdgref_avgpool_fwd(_p(x), _p(p), N, C, H, W)
        return p

    def avgpool_bwd(self, dp, x_shape) -> np.ndarray:
        dp = self._a(dp)
        N, C, H, W = x_shape
        dx = np.empty((N, C, H, W), self.dt)
        self.lib.fdgref_avgpool_bwd(_p(dp), _p(dx), N, C, H, W)
        return dx

    def fc_fwd(self, p, Wt, b) -> np.ndarray:
        p, Wt, b = self._a(p), self._a(Wt), self._a(b)
        N, C = p.shape
        J = Wt.shape[0]
        logits = np.empty((N, J), self.dt)
        self.lib.fdgref_fc_fwd(_p(p), _p(Wt), _p(b), _p(logits), N, C, J)
        return logits

    def fc_bwd(self, p, Wt, dl):
        p, Wt, dl = self._a(p), self._a(Wt), self._a(dl)
        N, C = p.shape
        J = Wt.shape[0]
        dWt, db, dp = np.empty((J, C), self.dt), np.empty(J, self.dt), np.empty((N, C), self.dt)
        self.lib.fdgref_fc_bwd(_p(p), _p(Wt), _p(dl), _p(dWt), _p(db), _p(dp), N, C, J)
        return dWt, db, dp

    def softmax_ce(self, logits, labels):
        logits = self._a(logits)
        labels = np.ascontiguousarray(labels, np.int32)
        N, J = logits.shape
        dl = np.empty((N, J), self.dt)
        loss = self.lib.fdgref_softmax_ce(_p(logits), _p(labels), _p(dl), N, J)
        return float(loss), dl

    def round_bf16(self, x) -> np.ndarray:
        """A copy of x with every element rounded to the nearest bfloat16 (ties to even)."""
        y = np.array(x, dtype=self.dt, order="C", copy=True)
        self.lib.fdgref_round_bf16(_p(y), ctypes.c_size_t(y.size))
        return y

    def sgd_momentum(self, theta, v, g, lr: float, mu: float, wd: float) -> None:
        """In place on theta and v."""
        assert theta.dtype == self.dt and v.dtype == self.dt and g.dtype == self.dt
        self.lib.fdgref_sgd_momentum(_p(theta), _p(v), _p(g), ctypes.c_size_t(theta.size), ctypes.c_double(lr),
                                     ctypes.c_double(mu), ctypes.c_double(wd))


def _projects(L) -> bool:
    return L.kind in (BASIC_POSTACT, BASIC_PREACT, BOTTLENECK_POSTACT) and (L.stride != 1 or L.c_in != L.c_out)


def oracle_param_layout(spec) -> List[Tuple[str, Tuple[int, ...]]]:
    """(name, shape) of every parameter tensor in flat order (the order documented in the C header)."""
    out: List[Tuple[str, Tuple[int, ...]]] = []
    J = spec.num_classes
    for i, L in enumerate(spec.layers):
        def bn(tag, c):
            return [(f"{i}.{tag}.gamma", (c,)), (f"{i}.{tag}.beta", (c,))]
        if L.kind == STEM:
            out += [(f"{i}.conv.w", (L.c_out, L.c_in, 3, 3))] + bn("bn", L.c_out)
        elif L.kind == BASIC_POSTACT:
            out += [(f"{i}.conv1.w", (L.c_out, L.c_in, 3, 3))] + bn("bn1", L.c_out)
            out += [(f"{i}.conv2.w", (L.c_out, L.c_out, 3, 3))] + bn("bn2", L.c_out)
            if _projects(L):
                out += [(f"{i}.proj.w", (L.c_out, L.c_in, 1, 1))] + bn("bnp", L.c_out)
        elif L.kind == BOTTLENECK_POSTACT:
            cm = L.c_out // 4
            out += [(f"{i}.conv1.w", (cm, L.c_in, 1, 1))] + bn("bn1", cm)
            out += [(f"{i}.conv2.w", (cm, cm, 3, 3))] + bn("bn2", cm)
            out += [(f"{i}.conv3.w", (L.c_out, cm, 1, 1))] + bn("bn3", L.c_out)
            if _projects(L):
                out += [(f"{i}.proj.w", (L.c_out, L.c_in, 1, 1))] + bn("bnp", L.c_out)
        elif L.kind == BASIC_PREACT:
            out += bn("bn1", L.c_in) + [(f"{i}.conv1.w", (L.c_out, L.c_in, 3, 3))]
            out += bn("bn2", L.c_out) + [(f"{i}.conv2.w", (L.c_out, L.c_out, 3, 3))]
            if _projects(L):
                out += [(f"{i}.proj.w", (L.c_out, L.c_in, 1, 1))]
        elif L.kind == STEM_POOL:
            out += [(f"{i}.conv.w", (L.c_out, L.c_in, 7, 7))] + bn("bn", L.c_out)
        elif L.kind == INVERTED_RESIDUAL:
            cm = EXPANSION * L.c_in
            out += [(f"{i}.conv1.w", (cm, L.c_in, 1, 1))] + bn("bn1", cm)
            out += [(f"{i}.conv2.w", (cm, 1, 3, 3))] + bn("bn2", cm)
            out += [(f"{i}.conv3.w", (L.c_out, cm, 1, 1))] + bn("bn3", L.c_out)
        elif L.kind == HEAD_POSTACT:
            out += [(f"{i}.fc.w", (J, L.c_in)), (f"{i}.fc.b", (J,))]
        elif L.kind == HEAD_PREACT:
            out += bn("bn", L.c_in) + [(f"{i}.fc.w", (J, L.c_in)), (f"{i}.fc.b", (J,))]
        else:
            raise ValueError(f"unknown layer kind {L.kind}")
    return out


class _Flat:
    """A flat vector with named views, in the documented parameter order."""

    def __init__(self, layout, dtype, data: Optional[np.ndarray] = None):
        self.layout = layout
        total = int(sum(int(np.prod(s)) for _, s in layout))
        self.flat = np.zeros(total, dtype) if data is None else np.array(data, dtype=dtype, copy=True).reshape(-1)
        assert self.flat.size == total
        self.views: Dict[str, np.ndarray] = {}
        off = 0
        for name, shape in layout:
            n = int(np.prod(shape))
            self.views[name] = self.flat[off:off + n].reshape(shape)
            off += n

    def __getitem__(self, k: str) -> np.ndarray:
        return self.views[k]

    def copy(self) -> "_Flat":
        return _Flat(self.layout, self.flat.dtype, self.flat)


class QueueFull(Exception):
    pass


class QueueEmpty(Exception):
    pass


class NoGrad(Exception):
    pass


class OracleModule:
    """One FDG module worker on the CPU.  `spec` is any object with the fields of the C ABI's module
    descriptor (n, c_in, h_in, w_in, layers[kind,c_in,c_out,stride], delay, is_bottom, num_classes,
    beta, momentum, weight_decay, bn_eps, bn_momentum)."""

    def __init__(self, spec, dtype=np.float32, storage: str = "fp32", save: str = "activations", weights: str = "snapshot"):
        """weights = "snapshot": the delayed backward runs at the parameters of its own forward (the stale index on
        every factor of Eq. 10).  weights = "current" is the ablation in which a saved forward keeps no parameters:
        the backward takes whatever the parameters are when it runs (what a framework that updates weights in place
        and back-propagates through a saved graph would compute) -- stale activations and batch statistics, current
        convolution weights, batch-norm scales and classifier weights.
        save = "activations": a saved forward keeps every intermediate (the saved graph of Fig. 1(b)).
        save = "input": it keeps the module input, the labels and the parameters of that forward only, and
        the delayed backward first runs the same forward again (recomputation as in feature replay,
        Section II, but at the STALE parameters, so that Eq. 10 is evaluated as before); running
        statistics move only in forward()."""
        assert storage in ("fp32", "bf16") and save in ("activations", "input") and weights in ("snapshot", "current")
        assert not (save == "input" and weights == "current"), "a forward run again needs the parameters it ran with"
        self.save = save
        self.weights = weights
        self.spec = spec
        self.dt = np.dtype(dtype)
        self.k = Kernels(dtype)
        self.storage = storage
        self.layout = oracle_param_layout(spec)
        self.theta = _Flat(self.layout, self.dt)
        self.v = np.zeros_like(self.theta.flat)
        self.grad = _Flat(self.layout, self.dt)
        self.has_grad = False
        # running statistics per BN, keyed like the parameters ("<layer>.<tag>")
        self.running: "collections.OrderedDict[str, List[np.ndarray]]" = collections.OrderedDict()
        for name, shape in self.layout:
            if name.endswith(".gamma"):
                self.running[name[:-6]] = [np.zeros(shape, self.dt), np.ones(shape, self.dt)]
        self.fifo: "collections.deque[dict]" = collections.deque()
        self.seq_fwd = 0   # number of forwards done  = sequence number of the next forward
        self.seq_bwd = 0   # number of backwards done = sequence number of the next context to pop
        self.is_top = bool(spec.layers) and spec.layers[-1].kind in (HEAD_POSTACT, HEAD_PREACT)
        self._move_running = True

    # ---- accessors ---------------------------------------------------------------------------
    def param_count(self) -> int:
        return self.theta.flat.size

    def set_params(self, flat) -> None:
        self.theta = _Flat(self.layout, self.dt, flat)
        self.v = np.zeros_like(self.theta.flat)

    def get_params(self) -> np.ndarray:
        return self.theta.flat.copy()

    def get_grads(self) -> np.ndarray:
        return self.grad.flat.copy()

    def get_momentum(self) -> np.ndarray:
        return self.v.copy()

    def get_bn_running(self) -> np.ndarray:
        return np.concatenate([np.concatenate([m, v]) for m, v in self.running.values()]) if self.running \
            else np.zeros(0, self.dt)

    def queue_state(self) -> Tuple[int, int, int]:
        """(outstanding, oldest sequence number, newest sequence number), -1 when empty."""
        out = len(self.fifo)
        return (out, self.seq_bwd if out else -1, self.seq_fwd - 1 if out else -1)

    # ---- batch normalisation with running statistics -----------------------------------------
    def _bn(self, key: str, x, th: _Flat, tape: dict):
        y, mean, var, invstd = self.k.bn_fwd(x, th[key + ".gamma"], th[key + ".beta"], self.spec.bn_eps)
        if self._move_running:
            M = x.shape[0] * x.shape[2] * x.shape[3]
            mom = self.spec.bn_momentum
            rm, rv = self.running[key]
            unbiased = var * (M / (M - 1.0)) if M > 1 else var
            self.running[key] = [((1.0 - mom) * rm + mom * mean).astype(self.dt),
                                 ((1.0 - mom) * rv + mom * unbiased).astype(self.dt)]
        tape[key] = (x, mean, invstd)
        return y

    def _bn_back(self, key: str, dy, th: _Flat, tape: dict, g: _Flat):
        x, mean, invstd = tape[key]
        dx, dgamma, dbeta = self.k.bn_bwd(x, dy, th[key + ".gamma"], mean, invstd)
        g[key + ".gamma"][...] = dgamma
        g[key + ".beta"][...] = dbeta
        return dx

    # ---- storage precision ------------------------------------------------------------------------
    def _q(self, x):
        """Identity in fp32 storage; rounds to bfloat16 where the bf16 path stores bfloat16."""
        return self.k.round_bf16(x) if self.storage == "bf16" else x

    def _stored_weights(self, theta: _Flat) -> _Flat:
        """The parameters as a forward uses them: convolution weights in storage precision."""
        if self.storage != "bf16":
            return theta
        th = theta.copy()
        for name, shape in self.layout:
            if len(shape) == 4:
                th[name][...] = self.k.round_bf16(th[name])
        return th

    # ---- forward -------------------------------------------------------------------------------
    def forward(self, x, labels=None):
        """Section III-A forward step.  Returns the module output (top module: [loss, logits...]).
        z is the residual stream in full precision, zb its stored copy (conv / BN operand)."""
        if len(self.fifo) >= self.spec.delay + 1:
            raise QueueFull()
        th = self._stored_weights(self.theta.copy())   # parameters of THIS iteration, kept for the backward
        x = np.array(x, dtype=self.dt, order="C")
        out, tapes = self._layers(x, labels, th, move_running=True)
        if self.save == "input":
            self.fifo.append({"theta": th, "x": x, "labels": None if labels is None else np.array(labels), "seq": self.seq_fwd})
        else:
            self.fifo.append({"theta": th, "tapes": tapes, "seq": self.seq_fwd})
        self.seq_fwd += 1
        return out

    def _layers(self, x, labels, th: _Flat, move_running: bool):
        """The module's layers on x with parameters th: (output, what every layer keeps for its backward)."""
        self._move_running = move_running
        k, q = self.k, self._q
        tapes: List[dict] = []
        z = np.ascontiguousarray(x, dtype=self.dt)
        assert z.shape == (self.spec.n, self.spec.c_in, self.spec.h_in, self.spec.w_in)
        zb = q(z)
        out = None
        for i, L in enumerate(self.spec.layers):
            t: dict = {"x": zb}
            if L.kind == STEM:
                c = q(k.conv_fwd(zb, th[f"{i}.conv.w"], L.stride, 1))
                b = self._bn(f"{i}.bn", c, th, t)
                z = k.relu_fwd(b)
            elif L.kind == BASIC_POSTACT:
                c1 = q(k.conv_fwd(zb, th[f"{i}.conv1.w"], L.stride, 1))
                a1 = q(k.relu_fwd(self._bn(f"{i}.bn1", c1, th, t)))
                c2 = q(k.conv_fwd(a1, th[f"{i}.conv2.w"], 1, 1))
                b2 = self._bn(f"{i}.bn2", c2, th, t)
                if _projects(L):
                    sc = self._bn(f"{i}.bnp", q(k.conv_fwd(zb, th[f"{i}.proj.w"], L.stride, 0)), th, t)
                else:
                    sc = z
                t.update(a1=a1)
                z = k.relu_fwd(b2 + sc)
            elif L.kind == BOTTLENECK_POSTACT:
                # 1x1 down to a quarter of the output channels, 3x3 (which carries the stride), 1x1 up, each followed
                # by batch norm; ReLU after the first two and after the shortcut is added
                c1 = q(k.conv_fwd(zb, th[f"{i}.conv1.w"], 1, 0))
                a1 = q(k.relu_fwd(self._bn(f"{i}.bn1", c1, th, t)))
                c2 = q(k.conv_fwd(a1, th[f"{i}.conv2.w"], L.stride, 1))
                a2 = q(k.relu_fwd(self._bn(f"{i}.bn2", c2, th, t)))
                c3 = q(k.conv_fwd(a2, th[f"{i}.conv3.w"], 1, 0))
                b3 = self._bn(f"{i}.bn3", c3, th, t)
                if _projects(L):
                    sc = self._bn(f"{i}.bnp", q(k.conv_fwd(zb, th[f"{i}.proj.w"], L.stride, 0)), th, t)
                else:
                    sc = z
                t.update(a1=a1, a2=a2)
                z = k.relu_fwd(b3 + sc)
            elif L.kind == STEM_POOL:
                assert L.stride == 4, "a 7x7 convolution of stride 2 followed by a pool of stride 2"
                c = q(k.conv_fwd(zb, th[f"{i}.conv.w"], 2, 3))
                a = q(k.relu_fwd(self._bn(f"{i}.bn", c, th, t)))
                t.update(a=a)
                z = k.maxpool_fwd(a, 3, 2, 1)
            elif L.kind == INVERTED_RESIDUAL:
                c1 = q(k.conv_fwd(zb, th[f"{i}.conv1.w"], 1, 0))
                a1 = q(k.relu6_fwd(self._bn(f"{i}.bn1", c1, th, t)))
                c2 = q(k.dwconv_fwd(a1, th[f"{i}.conv2.w"], L.stride, 1))
                a2 = q(k.relu6_fwd(self._bn(f"{i}.bn2", c2, th, t)))
                c3 = q(k.conv_fwd(a2, th[f"{i}.conv3.w"], 1, 0))
                b3 = self._bn(f"{i}.bn3", c3, th, t)
                t.update(a1=a1, a2=a2)
                z = b3 + z if (L.stride == 1 and L.c_in == L.c_out) else b3
            elif L.kind == BASIC_PREACT:
                o1 = q(k.relu_fwd(self._bn(f"{i}.bn1", zb, th, t)))
                c1 = q(k.conv_fwd(o1, th[f"{i}.conv1.w"], L.stride, 1))
                o2 = q(k.relu_fwd(self._bn(f"{i}.bn2", c1, th, t)))
                c2 = k.conv_fwd(o2, th[f"{i}.conv2.w"], 1, 1)
                sc = k.conv_fwd(o1, th[f"{i}.proj.w"], L.stride, 0) if _projects(L) else z
                t.update(o1=o1, o2=o2)
                z = c2 + sc
            elif L.kind in (HEAD_POSTACT, HEAD_PREACT):
                assert i == len(self.spec.layers) - 1 and labels is not None
                if L.kind == HEAD_PREACT:
                    o = q(k.relu_fwd(self._bn(f"{i}.bn", zb, th, t)))
                    t["o"] = o
                else:
                    o = zb
                p = k.avgpool_fwd(o)
                logits = k.fc_fwd(p, th[f"{i}.fc.w"], th[f"{i}.fc.b"])
                loss, dl = k.softmax_ce(logits, labels)
                t.update(o_shape=o.shape, p=p, dl=dl)
                out = np.concatenate([np.array([loss], self.dt), logits.reshape(-1)])
                tapes.append(t)
                break
            zb = q(z)
            t["y"] = zb          # stored copy of the layer output: next operand and ReLU gate (y > 0)
            tapes.append(t)
        if out is None:
            out = z
        return out, tapes

    # ---- delayed backward ----------------------------------------------------------------------
    def backward_delayed(self, grad_out=None):
        """Eq. 10 with the shrinking of Eq. 15 on the oldest saved forward.  Returns the gradient of
        the module input (None for a bottom module).  A ReLU passes the gradient where its stored
        output is positive, which is where its input was."""
        if not self.fifo:
            raise QueueEmpty()
        ctx = self.fifo.popleft()
        assert ctx["seq"] == self.seq_bwd
        self.seq_bwd += 1
        k, q, th = self.k, self._q, ctx["theta"]
        if self.weights == "current":
            th = self._stored_weights(self.theta.copy())
        if self.save == "input":    # the saved forward again, on its input with its parameters
            _, tapes = self._layers(ctx["x"], ctx["labels"], th, move_running=False)
        else:
            tapes = ctx["tapes"]
        g = _Flat(self.layout, self.dt)
        if self.is_top:
            assert grad_out is None
            dz = None
        else:
            # gradient shrinking: multiply by beta BEFORE back-propagating (Eq. 15)
            dz = (np.asarray(self.spec.beta, self.dt) * np.ascontiguousarray(grad_out, dtype=self.dt)).astype(self.dt)
        for i in reversed(range(len(self.spec.layers))):
            dz = self._layer_backward(i, self.spec.layers[i], tapes[i], th, dz, g, not (i == 0 and self.spec.is_bottom))
        self.grad = g
        self.has_grad = True
        return dz

    def _layer_backward(self, i: int, L, t: dict, th: _Flat, dz, g: _Flat, need_dx: bool):
        """The chain rule (Eq. 8, Eq. 9) through ONE layer: given what the layer's forward kept (t), the parameters
        of that forward (th) and the gradient dz of its output, writes the layer's parameter gradients into g and
        returns the gradient of its input (None if not needed)."""
        k, q = self.k, self._q
        x = t["x"]
        if L.kind in (HEAD_POSTACT, HEAD_PREACT):
            dW, db, dp = k.fc_bwd(t["p"], th[f"{i}.fc.w"], t["dl"])
            g[f"{i}.fc.w"][...] = dW
            g[f"{i}.fc.b"][...] = db
            do = k.avgpool_bwd(dp, t["o_shape"])
            if L.kind == HEAD_PREACT:
                dz = self._bn_back(f"{i}.bn", k.relu_bwd(t["o"], do), th, t, g)
            else:
                dz = do
        elif L.kind == STEM:
            dc = q(self._bn_back(f"{i}.bn", k.relu_bwd(t["y"], dz), th, t, g))
            g[f"{i}.conv.w"][...] = k.conv_bwd_weight(x, dc, 3, L.stride, 1)
            dz = k.conv_bwd_data(dc, th[f"{i}.conv.w"], x.shape, L.stride, 1) if need_dx else None
        elif L.kind == BASIC_POSTACT:
            ds = k.relu_bwd(t["y"], dz)                 # through the final ReLU; feeds both branches
            dc2 = q(self._bn_back(f"{i}.bn2", ds, th, t, g))
            g[f"{i}.conv2.w"][...] = k.conv_bwd_weight(t["a1"], dc2, 3, 1, 1)
            da1 = k.conv_bwd_data(dc2, th[f"{i}.conv2.w"], t["a1"].shape, 1, 1)
            if L.c_out not in (16, 32, 64):
                # Storage map of the bf16 path: this gradient is a bf16 tensor, except in blocks of 16, 32 or 64 channels,
                # where it stays in fp32.  (A bf16 gradient whose batch-norm backward is rounded to bf16 again is rounded
                # twice; the second rounding is biased, and the pixel sum of conv1's weight gradient adds that bias up.)
                da1 = q(da1)
            dc1 = q(self._bn_back(f"{i}.bn1", k.relu_bwd(t["a1"], da1), th, t, g))
            g[f"{i}.conv1.w"][...] = k.conv_bwd_weight(x, dc1, 3, L.stride, 1)
            if _projects(L):
                dpr = q(self._bn_back(f"{i}.bnp", ds, th, t, g))
                g[f"{i}.proj.w"][...] = k.conv_bwd_weight(x, dpr, 1, L.stride, 0)
            if need_dx:
                dx = k.conv_bwd_data(dc1, th[f"{i}.conv1.w"], x.shape, L.stride, 1)
                if _projects(L):
                    dx = dx + k.conv_bwd_data(dpr, th[f"{i}.proj.w"], x.shape, L.stride, 0)
                else:
                    dx = dx + ds
                dz = dx
            else:
                dz = None
        elif L.kind == BOTTLENECK_POSTACT:
            ds = k.relu_bwd(t["y"], dz)                 # through the final ReLU; feeds both branches
            dc3 = q(self._bn_back(f"{i}.bn3", ds, th, t, g))
            g[f"{i}.conv3.w"][...] = k.conv_bwd_weight(t["a2"], dc3, 1, 1, 0)
            da2 = q(k.conv_bwd_data(dc3, th[f"{i}.conv3.w"], t["a2"].shape, 1, 0))
            dc2 = q(self._bn_back(f"{i}.bn2", k.relu_bwd(t["a2"], da2), th, t, g))
            g[f"{i}.conv2.w"][...] = k.conv_bwd_weight(t["a1"], dc2, 3, L.stride, 1)
            da1 = q(k.conv_bwd_data(dc2, th[f"{i}.conv2.w"], t["a1"].shape, L.stride, 1))
            dc1 = q(self._bn_back(f"{i}.bn1", k.relu_bwd(t["a1"], da1), th, t, g))
            g[f"{i}.conv1.w"][...] = k.conv_bwd_weight(x, dc1, 1, 1, 0)
            if _projects(L):
                dpr = q(self._bn_back(f"{i}.bnp", ds, th, t, g))
                g[f"{i}.proj.w"][...] = k.conv_bwd_weight(x, dpr, 1, L.stride, 0)
            if need_dx:
                dx = k.conv_bwd_data(dc1, th[f"{i}.conv1.w"], x.shape, 1, 0)
                if _projects(L):
                    dx = dx + k.conv_bwd_data(dpr, th[f"{i}.proj.w"], x.shape, L.stride, 0)
                else:
                    dx = dx + ds
                dz = dx
            else:
                dz = None
        elif L.kind == STEM_POOL:
            da = k.maxpool_bwd(t["a"], dz, 3, 2, 1)
            dc = q(self._bn_back(f"{i}.bn", k.relu_bwd(t["a"], da), th, t, g))
            g[f"{i}.conv.w"][...] = k.conv_bwd_weight(x, dc, 7, 2, 3)
            dz = k.conv_bwd_data(dc, th[f"{i}.conv.w"], x.shape, 2, 3) if need_dx else None
        elif L.kind == INVERTED_RESIDUAL:
            dc3 = q(self._bn_back(f"{i}.bn3", dz, th, t, g))        # no gate: the block ends in a batch norm
            g[f"{i}.conv3.w"][...] = k.conv_bwd_weight(t["a2"], dc3, 1, 1, 0)
            # storage map of the bf16 path: the two gradients that go into a gate and a batch-norm backward stay in fp32
            # (as in the narrow basic blocks: see there)
            da2 = k.conv_bwd_data(dc3, th[f"{i}.conv3.w"], t["a2"].shape, 1, 0)
            dc2 = q(self._bn_back(f"{i}.bn2", k.relu6_bwd(t["a2"], da2), th, t, g))
            g[f"{i}.conv2.w"][...] = k.dwconv_bwd_weight(t["a1"], dc2, 3, L.stride, 1)
            da1 = k.dwconv_bwd_data(dc2, th[f"{i}.conv2.w"], t["a1"].shape, L.stride, 1)
            dc1 = q(self._bn_back(f"{i}.bn1", k.relu6_bwd(t["a1"], da1), th, t, g))
            g[f"{i}.conv1.w"][...] = k.conv_bwd_weight(x, dc1, 1, 1, 0)
            if need_dx:
                dx = k.conv_bwd_data(dc1, th[f"{i}.conv1.w"], x.shape, 1, 0)
                dz = dx + dz if (L.stride == 1 and L.c_in == L.c_out) else dx
            else:
                dz = None
        elif L.kind == BASIC_PREACT:
            # y = conv2(o2) + shortcut; the convolutions take the stored copy of the gradient
            dzb = q(dz)
            g[f"{i}.conv2.w"][...] = k.conv_bwd_weight(t["o2"], dzb, 3, 1, 1)
            do2 = q(k.conv_bwd_data(dzb, th[f"{i}.conv2.w"], t["o2"].shape, 1, 1))
            dc1 = q(self._bn_back(f"{i}.bn2", k.relu_bwd(t["o2"], do2), th, t, g))
            g[f"{i}.conv1.w"][...] = k.conv_bwd_weight(t["o1"], dc1, 3, L.stride, 1)
            do1 = k.conv_bwd_data(dc1, th[f"{i}.conv1.w"], t["o1"].shape, L.stride, 1)
            if _projects(L):
                g[f"{i}.proj.w"][...] = k.conv_bwd_weight(t["o1"], dzb, 1, L.stride, 0)
                do1 = do1 + k.conv_bwd_data(dzb, th[f"{i}.proj.w"], t["o1"].shape, L.stride, 0)
            do1 = q(do1)
            dx = self._bn_back(f"{i}.bn1", k.relu_bwd(t["o1"], do1), th, t, g)   # BN1 needs this even at the bottom
            if not _projects(L):
                dx = dx + dz
            dz = dx if need_dx else None
        return dz

    # ---- update --------------------------------------------------------------------------------
    def update(self, lr: float) -> None:
        """Eq. 11 / Eq. 12: the delayed gradient moves the CURRENT parameters."""
        if not self.has_grad:
            raise NoGrad()
        self.k.sgd_momentum(self.theta.flat, self.v, self.grad.flat, lr, self.spec.momentum,
                            self.spec.weight_decay)
        self.has_grad = False


# ------------------------------------------------------------------------------------------------
# The iteration schedule of Fig. 1(a): which batch each module touches at each iteration.
# ------------------------------------------------------------------------------------------------
def fdg_schedule(K: int, T: int):
    """Integer simulation of K module workers exchanging tensors at the END of every iteration
    (Section III-A, "communication"; Fig. 1(a)).  Modules k = 1..K, iterations t = 1..T, batches
    numbered from 1.  Within an iteration a module first runs its forward on the input it holds,
    then a backward on the oldest forward for which a gradient has arrived; the top module k=K
    back-propagates the batch it has just forwarded (delay 0).

    Returns (fwd, bwd, depth): fwd[k][t] / bwd[k][t] = batch id processed (0 = idle) and
    depth[k] = the largest number of saved forwards module k ever held at once."""
    fwd = {k: {} for k in range(1, K + 1)}
    bwd = {k: {} for k in range(1, K + 1)}
    depth = {k: 0 for k in range(1, K + 1)}
    inbox_act = {k: None for k in range(1, K + 2)}    # activation waiting at module k's input
    inbox_grad = {k: None for k in range(0, K + 1)}   # gradient waiting at module k's output
    saved = {k: collections.deque() for k in range(1, K + 1)}
    for t in range(1, T + 1):
        inbox_act[1] = t                               # the data loader feeds module 1 with batch t
        send_act, send_grad = {}, {}
        for k in range(1, K + 1):
            b = inbox_act[k]
            fwd[k][t] = b or 0
            if b:
                saved[k].append(b)
                send_act[k + 1] = b
            depth[k] = max(depth[k], len(saved[k]))
            if k == K:
                gb = b                                 # loss gradient of the batch just forwarded
            else:
                gb = inbox_grad[k]
            bwd[k][t] = gb or 0
            if gb:
                assert saved[k][0] == gb, "gradients must arrive in forward order"
                saved[k].popleft()
                send_grad[k - 1] = gb
        # communication: the last thing an iteration does
        for k in range(1, K + 2):
            inbox_act[k] = send_act.get(k)
        for k in range(0, K + 1):
            inbox_grad[k] = send_grad.get(k)
    return fwd, bwd, depth


# ------------------------------------------------------------------------------------------------
# K modules run as Algorithm I
# ------------------------------------------------------------------------------------------------
class OracleChain:
    """K module workers and their mailboxes (Section III-A; Algorithm I).  `specs[k]`, k = 0..K-1 from
    the input side, describe the modules: the first is a bottom module, the last ends in the loss, the
    output shape of each is the input shape of the next, and module k can hold the 2(K-1-k) saved
    forwards that are waiting for their gradients plus the newest one (Fig. 1(a): the gradient of
    module k -- k counted from 1 there -- is 2(K-k) iterations late), i.e. specs[k].delay >= 2(K-1-k).

    One call of step() is one iteration t = 1, 2, ...: batch t enters module 0.  Per module, in the
    order of Algorithm I: (1) if a gradient was received at the end of the previous iteration,
    delayed backward (shrunk by that module's beta) and update; (2) if an input was received, forward;
    (3) what was produced is delivered at the end of the iteration.  The last module has delay 0:
    it forwards its input, takes the loss gradient of that same batch, back-propagates and updates
    (Section III-B: its gradient is not shrunk).  Until the first tensors arrive a module idles, which
    is the max{0, .} clamp of the batch indices in Section IV."""

    def __init__(self, specs, dtype=np.float32, storage: str = "fp32"):
        K = len(specs)
        assert K >= 1
        self.K = K
        self.mods = [OracleModule(sp, dtype, storage) for sp in specs]
        assert self.mods[-1].is_top and all(not m.is_top for m in self.mods[:-1])
        for k, sp in enumerate(specs):
            assert sp.delay >= 2 * (K - 1 - k), "module %d needs a history of %d forwards" % (k, 2 * (K - 1 - k))
            assert bool(sp.is_bottom) == (k == 0)
        self.t = 0
        self.inbox_act: List[Optional[tuple]] = [None] * K    # (batch, tensor) waiting at module k's input
        self.inbox_grad: List[Optional[tuple]] = [None] * K   # (batch, tensor) waiting at module k's output
        self.labels: Dict[int, np.ndarray] = {}
        self.fwd_batch = [0] * K      # what each module did in the last iteration (0 = idle)
        self.bwd_batch = [0] * K

    def step(self, x, labels, lr: float):
        """One iteration.  Returns (batch, loss, logits) of the batch the last module saw, or None
        while it is still idle."""
        K = self.K
        self.t += 1
        t = self.t
        self.labels[t] = np.asarray(labels)
        send_act: Dict[int, tuple] = {}
        send_grad: Dict[int, tuple] = {}
        self.fwd_batch, self.bwd_batch = [0] * K, [0] * K
        result = None
        for k, m in enumerate(self.mods):
            inp = (t, x) if k == 0 else self.inbox_act[k]
            if k == K - 1:
                if inp is not None:
                    b, z = inp
                    out = m.forward(z, self.labels.pop(b))
                    result = (b, float(out.ravel()[0]), np.array(out.ravel()[1:]).reshape(m.spec.n, -1))
                    gin = m.backward_delayed(None)
                    m.update(lr)
                    self.fwd_batch[k] = self.bwd_batch[k] = b
                    if k > 0:
                        send_grad[k - 1] = (b, gin)
            else:
                got = self.inbox_grad[k]
                if got is not None:
                    b, g = got
                    gin = m.backward_delayed(g)
                    m.update(lr)
                    self.bwd_batch[k] = b
                    if k > 0:
                        send_grad[k - 1] = (b, gin)
                if inp is not None:
                    b, z = inp
                    send_act[k + 1] = (b, m.forward(z))
                    self.fwd_batch[k] = b
        # communication, the last thing an iteration does
        self.inbox_act = [send_act.get(k) for k in range(K)]
        self.inbox_grad = [send_grad.get(k) for k in range(K)]
        return result

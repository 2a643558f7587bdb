"""Synthetic workloads for one FDG module worker: the module shapes and the seeded tensors.

This module holds NO arithmetic of the method.  It only says which layers a module has (plain
data), which shapes its tensors take, and how the synthetic inputs are drawn.  Both the CPU oracle's
tests and the GPU path's tests / benchmark take their inputs from here, so that the two sides see
bit-identical inputs while sharing no implementation code.

The shapes stand in for the paper's CIFAR-10 experiments (Section V-A: 32x32 colour images, 10
classes, batch 128; ResNet / WRN architectures named in Table III).  The dataset itself is not used:
images are N(0,1) noise, labels are uniform, the gradient arriving from the module above is
N(0, 1e-2) noise (variance 1e-2, i.e. sigma = 0.1).

Random numbers come from numpy's Philox counter-based generator keyed by (seed, stream id), so any
tensor can be regenerated on its own, in any order.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

# layer kinds (values are the C ABI's fdg_layer_kind)
STEM = 0
BASIC_POSTACT = 1
BASIC_PREACT = 2
HEAD_POSTACT = 3
HEAD_PREACT = 4
BOTTLENECK_POSTACT = 5
STEM_POOL = 6            # ImageNet-style stem: 7x7 convolution stride 2 + BN + ReLU + 3x3 max-pool stride 2 (stride field = 4)
INVERTED_RESIDUAL = 7    # MobileNet-v2 block: 1x1 expand (x6) + BN + ReLU6, 3x3 depthwise (stride) + BN + ReLU6, 1x1 + BN

KIND_NAMES = {STEM: "stem", BASIC_POSTACT: "basic_postact", BASIC_PREACT: "basic_preact",
              HEAD_POSTACT: "head_postact", HEAD_PREACT: "head_preact", BOTTLENECK_POSTACT: "bottleneck_postact",
              STEM_POOL: "stem_pool", INVERTED_RESIDUAL: "inverted_residual"}
EXPANSION = 6            # channels inside an inverted residual block per input channel (MobileNet-v2's t)


@dataclass(frozen=True)
class Layer:
    kind: int
    c_in: int
    c_out: int = 0
    stride: int = 1

    @property
    def is_head(self) -> bool:
        return self.kind in (HEAD_POSTACT, HEAD_PREACT)

    @property
    def projects(self) -> bool:
        return self.kind in (BASIC_POSTACT, BASIC_PREACT, BOTTLENECK_POSTACT) and (self.stride != 1 or self.c_in != self.c_out)

    @property
    def c_mid(self) -> int:
        """Channels inside a bottleneck block: a quarter of its output channels; inside an inverted residual block:
        EXPANSION times its input channels."""
        return EXPANSION * self.c_in if self.kind == INVERTED_RESIDUAL else self.c_out // 4

    @property
    def adds_input(self) -> bool:
        """An inverted residual block adds its input to its output when shapes allow (no projection otherwise)."""
        return self.kind == INVERTED_RESIDUAL and self.stride == 1 and self.c_in == self.c_out


@dataclass
class ModuleSpec:
    """Plain description of one module; mirrors the C ABI's fdg_module_desc field by field."""
    n: int
    c_in: int
    h_in: int
    w_in: int
    layers: List[Layer]
    delay: int = 0
    is_bottom: bool = False
    num_classes: int = 10
    beta: float = 1.0
    momentum: float = 0.9
    weight_decay: float = 5e-4
    bn_eps: float = 1e-5
    bn_momentum: float = 0.1
    lr: float = 0.1          # not part of the descriptor: passed to every update call
    name: str = ""

    @property
    def is_top(self) -> bool:
        return bool(self.layers) and self.layers[-1].is_head

    def input_shape(self) -> Tuple[int, int, int, int]:
        return (self.n, self.c_in, self.h_in, self.w_in)

    def activation_shapes(self) -> List[Tuple[int, int, int, int]]:
        """NCHW shape after every non-head layer, in order."""
        out = []
        c, h, w = self.c_in, self.h_in, self.w_in
        for L in self.layers:
            if L.is_head:
                break
            assert L.c_in == c, (L, c)
            h = (h - 1) // L.stride + 1
            w = (w - 1) // L.stride + 1
            c = L.c_out
            out.append((self.n, c, h, w))
        return out

    def output_shape(self) -> Tuple[int, ...]:
        if self.is_top:
            return (1 + self.n * self.num_classes,)
        return self.activation_shapes()[-1]


def param_shapes(spec: ModuleSpec) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, role) of every parameter tensor in the flat order of the C ABI.

    role is one of 'conv', 'gamma', 'beta', 'fc_w', 'fc_b' and only selects how the synthetic
    initial value is drawn."""
    out = []
    for i, L in enumerate(spec.layers):
        p = f"L{i}."
        if L.kind == STEM:
            out += [(p + "conv.w", (L.c_out, L.c_in, 3, 3), "conv"),
                    (p + "bn.gamma", (L.c_out,), "gamma"), (p + "bn.beta", (L.c_out,), "beta")]
        elif L.kind == BASIC_POSTACT:
            out += [(p + "conv1.w", (L.c_out, L.c_in, 3, 3), "conv"),
                    (p + "bn1.gamma", (L.c_out,), "gamma"), (p + "bn1.beta", (L.c_out,), "beta"),
                    (p + "conv2.w", (L.c_out, L.c_out, 3, 3), "conv"),
                    (p + "bn2.gamma", (L.c_out,), "gamma"), (p + "bn2.beta", (L.c_out,), "beta")]
            if L.projects:
                out += [(p + "proj.w", (L.c_out, L.c_in, 1, 1), "conv"),
                        (p + "bnp.gamma", (L.c_out,), "gamma"), (p + "bnp.beta", (L.c_out,), "beta")]
        elif L.kind == BOTTLENECK_POSTACT:
            cm = L.c_mid
            out += [(p + "conv1.w", (cm, L.c_in, 1, 1), "conv"),
                    (p + "bn1.gamma", (cm,), "gamma"), (p + "bn1.beta", (cm,), "beta"),
                    (p + "conv2.w", (cm, cm, 3, 3), "conv"),
                    (p + "bn2.gamma", (cm,), "gamma"), (p + "bn2.beta", (cm,), "beta"),
                    (p + "conv3.w", (L.c_out, cm, 1, 1), "conv"),
                    (p + "bn3.gamma", (L.c_out,), "gamma"), (p + "bn3.beta", (L.c_out,), "beta")]
            if L.projects:
                out += [(p + "proj.w", (L.c_out, L.c_in, 1, 1), "conv"),
                        (p + "bnp.gamma", (L.c_out,), "gamma"), (p + "bnp.beta", (L.c_out,), "beta")]
        elif L.kind == BASIC_PREACT:
            out += [(p + "bn1.gamma", (L.c_in,), "gamma"), (p + "bn1.beta", (L.c_in,), "beta"),
                    (p + "conv1.w", (L.c_out, L.c_in, 3, 3), "conv"),
                    (p + "bn2.gamma", (L.c_out,), "gamma"), (p + "bn2.beta", (L.c_out,), "beta"),
                    (p + "conv2.w", (L.c_out, L.c_out, 3, 3), "conv")]
            if L.projects:
                out += [(p + "proj.w", (L.c_out, L.c_in, 1, 1), "conv")]
        elif L.kind == STEM_POOL:
            out += [(p + "conv.w", (L.c_out, L.c_in, 7, 7), "conv"),
                    (p + "bn.gamma", (L.c_out,), "gamma"), (p + "bn.beta", (L.c_out,), "beta")]
        elif L.kind == INVERTED_RESIDUAL:
            cm = L.c_mid
            out += [(p + "conv1.w", (cm, L.c_in, 1, 1), "conv"),
                    (p + "bn1.gamma", (cm,), "gamma"), (p + "bn1.beta", (cm,), "beta"),
                    (p + "conv2.w", (cm, 1, 3, 3), "conv"),          # depthwise: one 3x3 filter per channel
                    (p + "bn2.gamma", (cm,), "gamma"), (p + "bn2.beta", (cm,), "beta"),
                    (p + "conv3.w", (L.c_out, cm, 1, 1), "conv"),
                    (p + "bn3.gamma", (L.c_out,), "gamma"), (p + "bn3.beta", (L.c_out,), "beta")]
        elif L.kind == HEAD_POSTACT:
            out += [(p + "fc.w", (spec.num_classes, L.c_in), "fc_w"), (p + "fc.b", (spec.num_classes,), "fc_b")]
        elif L.kind == HEAD_PREACT:
            out += [(p + "bn.gamma", (L.c_in,), "gamma"), (p + "bn.beta", (L.c_in,), "beta"),
                    (p + "fc.w", (spec.num_classes, L.c_in), "fc_w"), (p + "fc.b", (spec.num_classes,), "fc_b")]
        else:
            raise ValueError(f"unknown layer kind {L.kind}")
    return out


def param_count(spec: ModuleSpec) -> int:
    return int(sum(int(np.prod(s)) for _, s, _ in param_shapes(spec)))


# ----------------------------------------------------------------------------------------------
# seeded tensors
# ----------------------------------------------------------------------------------------------
_STREAM_PARAMS = 1 << 20      # + parameter tensor index
_STREAM_X = 2 << 20           # + step
_STREAM_G = 3 << 20           # + step
_STREAM_LABELS = 4 << 20      # + step


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def normal(seed: int, stream: int, shape: Sequence[int], sigma: float = 1.0) -> np.ndarray:
    """fp32 N(0, sigma^2) tensor of the given shape from stream (seed, stream)."""
    z = _rng(seed, stream).standard_normal(size=tuple(shape), dtype=np.float32)
    if sigma != 1.0:
        z *= np.float32(sigma)
    return z


def make_params(spec: ModuleSpec, seed: int = 0, perturb_bn: bool = False) -> np.ndarray:
    """Flat fp32 initial parameters: convolutions He-normal with fan-in (sigma = sqrt(2/(c_in*k*k))),
    FC weights N(0, 1/c_in), FC bias 0, BN gamma 1 and beta 0.  With perturb_bn the BN parameters are
    moved off their symmetric start (gamma ~ 1 + 0.2 N(0,1), beta ~ 0.2 N(0,1)) so that tests also
    see non-trivial scale and shift."""
    chunks = []
    for idx, (_, shape, role) in enumerate(param_shapes(spec)):
        stream = _STREAM_PARAMS + idx
        if role == "conv":
            fan_in = shape[1] * shape[2] * shape[3]
            t = normal(seed, stream, shape, float(np.sqrt(2.0 / fan_in)))
        elif role == "fc_w":
            t = normal(seed, stream, shape, float(np.sqrt(1.0 / shape[1])))
        elif role == "fc_b":
            t = np.zeros(shape, np.float32)
        elif role == "gamma":
            t = np.ones(shape, np.float32)
            if perturb_bn:
                t = t + normal(seed, stream, shape, 0.2)
        elif role == "beta":
            t = np.zeros(shape, np.float32)
            if perturb_bn:
                t = t + normal(seed, stream, shape, 0.2)
        else:
            raise ValueError(role)
        chunks.append(t.reshape(-1).astype(np.float32))
    return np.concatenate(chunks) if chunks else np.zeros(0, np.float32)


def make_input(spec: ModuleSpec, step: int, seed: int = 0) -> np.ndarray:
    """Module input of iteration `step`: fp32 N(0,1), NCHW."""
    return normal(seed, _STREAM_X + step, spec.input_shape())


def make_grad_out(spec: ModuleSpec, step: int, seed: int = 0) -> Optional[np.ndarray]:
    """Gradient received from the module above for the batch of iteration `step`: fp32 N(0, 1e-2)
    (sigma 0.1) in the shape of the module output; None for a top module."""
    if spec.is_top:
        return None
    return normal(seed, _STREAM_G + step, spec.output_shape(), 0.1)


def make_labels(spec: ModuleSpec, step: int, seed: int = 0) -> Optional[np.ndarray]:
    """int32 labels uniform in [0, num_classes) for a top module, else None."""
    if not spec.is_top:
        return None
    return _rng(seed, _STREAM_LABELS + step).integers(0, spec.num_classes, size=(spec.n,), dtype=np.int32)


# ----------------------------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------------------------
def _postact_stage(c_in: int, c_out: int, blocks: int, first_stride: int) -> List[Layer]:
    ls = [Layer(BASIC_POSTACT, c_in, c_out, first_stride)]
    ls += [Layer(BASIC_POSTACT, c_out, c_out, 1) for _ in range(blocks - 1)]
    return ls


def config(idx: int, n: Optional[int] = None) -> ModuleSpec:
    """Benchmark configuration idx in 1..10 (1..5: the CIFAR modules the metric is stated on; 6, 7: the two halves of
    ResNet-18 at Tiny-ImageNet resolution, channel counts that are powers of two; 8: bottleneck blocks of ResNet-101;
    9: ResNet-18's lower half with the 7x7 stem and max-pool; 10: inverted residual blocks of MobileNet-v2).  `n` overrides the batch size (for bounded CPU timing and
    small parity cases); everything else keeps its real shape."""
    hyper = dict(momentum=0.9, weight_decay=5e-4, bn_eps=1e-5, bn_momentum=0.1, lr=0.1)
    if idx == 1:
        # one post-activation basic block 16->16 on [16,16,32,32]; K=2, module 0, d=1, beta=0.2.
        # grad_in is computed here although the paper's bottom module has no use for it, so that the
        # parity test also covers the input gradient of a basic block.
        return ModuleSpec(n or 16, 16, 32, 32, [Layer(BASIC_POSTACT, 16, 16, 1)], delay=1, is_bottom=False,
                          beta=0.2, name="cfg1 basic block 16->16", **hyper)
    if idx == 2:
        # ResNet-56 module 0 (K=2): stem + all 27 blocks, widths 16/32/64.
        ls = [Layer(STEM, 3, 16, 1)] + _postact_stage(16, 16, 9, 1) + _postact_stage(16, 32, 9, 2) \
            + _postact_stage(32, 64, 9, 2)
        return ModuleSpec(n or 128, 3, 32, 32, ls, delay=1, is_bottom=True, beta=0.2,
                          name="cfg2 ResNet-56 module 0 (stem + 27 blocks)", **hyper)
    if idx == 3:
        # ResNet-110 K=4 module 0: stem + 13 blocks at 16 channels, history depth 3.
        ls = [Layer(STEM, 3, 16, 1)] + _postact_stage(16, 16, 13, 1)
        return ModuleSpec(n or 128, 3, 32, 32, ls, delay=3, is_bottom=True, beta=0.2,
                          name="cfg3 ResNet-110 K=4 module 0 (stem + 13 blocks)", **hyper)
    if idx == 4:
        # WRN-28-10 K=2 top module: pre-activation blocks 7..12 (2 x 320 at 16x16, then 320->640
        # stride 2 and 3 x 640 at 8x8) + BN/ReLU/avgpool/FC/softmax-CE.  d=0, gradient not shrunk.
        ls = [Layer(BASIC_PREACT, 320, 320, 1), Layer(BASIC_PREACT, 320, 320, 1),
              Layer(BASIC_PREACT, 320, 640, 2)] + [Layer(BASIC_PREACT, 640, 640, 1) for _ in range(3)] \
            + [Layer(HEAD_PREACT, 640)]
        return ModuleSpec(n or 128, 320, 16, 16, ls, delay=0, is_bottom=False, beta=1.0, num_classes=10,
                          name="cfg4 WRN-28-10 K=2 top module (blocks 7-12 + head)", **hyper)
    if idx == 5:
        # ResNet-1202 K=4 module 1: blocks 150..299 = 50 x 16ch at 32x32, 16->32 stride 2, 99 x 32ch.
        ls = [Layer(BASIC_POSTACT, 16, 16, 1) for _ in range(50)] + _postact_stage(16, 32, 100, 2)
        return ModuleSpec(n or 128, 16, 32, 32, ls, delay=2, is_bottom=False, beta=0.2,
                          name="cfg5 ResNet-1202 K=4 module 1 (blocks 150-299)", **hyper)
    if idx == 6:
        # ResNet-18 on Tiny-ImageNet (64x64 images, 200 classes; Table VI), K=2 top module: the upper four of the
        # eight basic blocks (128->256 stride 2, 256, 256->512 stride 2, 512) + avgpool/FC/softmax-CE.  d=0.
        ls = _postact_stage(128, 256, 2, 2) + _postact_stage(256, 512, 2, 2) + [Layer(HEAD_POSTACT, 512)]
        return ModuleSpec(n or 128, 128, 32, 32, ls, delay=0, is_bottom=False, beta=1.0, num_classes=200,
                          name="cfg6 ResNet-18 Tiny-ImageNet K=2 top module (blocks 5-8 + head)", **hyper)
    if idx == 7:
        # the module below it: 3x3 stem 3->64 at 64x64 + blocks 1-4 (64, 64, 64->128 stride 2, 128); beta = 0.5 (Table VI)
        ls = [Layer(STEM, 3, 64, 1)] + _postact_stage(64, 64, 2, 1) + _postact_stage(64, 128, 2, 2)
        return ModuleSpec(n or 128, 3, 64, 64, ls, delay=1, is_bottom=True, beta=0.5,
                          name="cfg7 ResNet-18 Tiny-ImageNet K=2 module 0 (stem + blocks 1-4)", **hyper)
    if idx == 8:
        # ResNet-101 at ImageNet resolution (Table VII's second network), K = 4, third module: eight bottleneck blocks of
        # the 1024-channel stage (256 inside) at 14x14
        ls = [Layer(BOTTLENECK_POSTACT, 1024, 1024, 1) for _ in range(8)]
        return ModuleSpec(n or 128, 1024, 14, 14, ls, delay=1, is_bottom=False, beta=0.5,
                          name="cfg8 ResNet-101 ImageNet K=4 module 2 (8 bottleneck blocks 1024/256 @14x14)", **hyper)
    if idx == 9:
        # ResNet-18 with the ImageNet stem at Tiny-ImageNet resolution, K = 2, module 0: 7x7 convolution stride 2 + BN + ReLU +
        # 3x3 max-pool stride 2 (64x64 -> 16x16), then blocks 1-4
        ls = [Layer(STEM_POOL, 3, 64, 4)] + _postact_stage(64, 64, 2, 1) + _postact_stage(64, 128, 2, 2)
        return ModuleSpec(n or 128, 3, 64, 64, ls, delay=1, is_bottom=True, beta=0.5,
                          name="cfg9 ResNet-18 (7x7 stem + max-pool) Tiny-ImageNet K=2 module 0", **hyper)
    if idx == 10:
        # MobileNet-v2 on Tiny-ImageNet (Table V), a middle module: the 64- and 96-channel stages (inverted residual blocks,
        # expansion 6), entered from the 32-channel stage at 32x32 through the stride-2 block
        ls = [Layer(INVERTED_RESIDUAL, 32, 64, 2)] + [Layer(INVERTED_RESIDUAL, 64, 64, 1) for _ in range(3)] \
            + [Layer(INVERTED_RESIDUAL, 64, 96, 1)] + [Layer(INVERTED_RESIDUAL, 96, 96, 1) for _ in range(2)]
        return ModuleSpec(n or 128, 32, 32, 32, ls, delay=1, is_bottom=False, beta=0.5,
                          name="cfg10 MobileNet-v2 Tiny-ImageNet module (7 inverted residual blocks 64/96)", **hyper)
    raise ValueError("config index must be 1..10")


def conv_flops(spec: ModuleSpec) -> int:
    """Useful multiply-add flops (2 per MAC) of one module step: forward + data gradient + weight
    gradient of every convolution and FC; the first layer's data gradient is not counted for a bottom
    module.  Counting only; no arithmetic of the method."""
    total = 0
    c, h, w = spec.c_in, spec.h_in, spec.w_in
    first = True
    for L in spec.layers:
        if L.is_head:
            total += 3 * 2 * spec.n * c * spec.num_classes
            break
        ho, wo = (h - 1) // L.stride + 1, (w - 1) // L.stride + 1
        m = spec.n * ho * wo
        convs = []
        if L.kind == BOTTLENECK_POSTACT:
            # the first 1x1 convolution runs at the input resolution; (ci, co, taps, reads the module input, pixels)
            f1 = 2 * spec.n * h * w * L.c_in * L.c_mid
            total += (2 if first and spec.is_bottom else 3) * f1
            convs.append((L.c_mid, L.c_mid, 9, False))
            convs.append((L.c_mid, L.c_out, 1, False))
            if L.projects:
                convs.append((L.c_in, L.c_out, 1, True))
        elif L.kind == STEM:
            convs.append((L.c_in, L.c_out, 9, True))
        elif L.kind == STEM_POOL:
            # the 7x7 convolution runs at half the input resolution; the pool halves it again
            hc, wc = (h - 1) // 2 + 1, (w - 1) // 2 + 1
            total += (2 if first and spec.is_bottom else 3) * 2 * spec.n * hc * wc * L.c_in * L.c_out * 49
        elif L.kind == INVERTED_RESIDUAL:
            f1 = 2 * spec.n * h * w * L.c_in * L.c_mid           # expansion at the input resolution
            total += (2 if first and spec.is_bottom else 3) * f1
            total += 3 * 2 * m * L.c_mid * 9                     # depthwise
            convs.append((L.c_mid, L.c_out, 1, False))
        else:
            convs.append((L.c_in, L.c_out, 9, True))
            convs.append((L.c_out, L.c_out, 9, False))
            if L.projects:
                convs.append((L.c_in, L.c_out, 1, True))
        for ci, co, taps, reads_module_input in convs:
            f = 2 * m * ci * co * taps
            passes = 3
            if first and reads_module_input and spec.is_bottom and L.kind in (STEM, BASIC_POSTACT, BOTTLENECK_POSTACT):
                passes = 2
            total += passes * f
        first = False
        c, h, w = L.c_out, ho, wo
    return total


# ------------------------------------------------------------------------------------------------
# A small network cut into K modules (for the K-module driver), and separable synthetic data
# ------------------------------------------------------------------------------------------------
def chain_specs(K: int, n: int = 16, width: int = 16, hw: int = 8, blocks: int = 1, beta: float = 0.5,
                num_classes: int = 10, lr: float = 0.05, weight_decay: float = 5e-4, momentum: float = 0.9) -> List[ModuleSpec]:
    """K module descriptions of a post-activation ResNet: stem 3 -> width, K * blocks basic blocks (the first block of
    the upper half doubles the width with stride 2 when K > 1), average pool + FC + softmax cross-entropy.  Module k
    (0 = input side) holds blocks [k * blocks, (k+1) * blocks); the stem goes to module 0 and the head to module
    K-1.  Delays are the 2(K-1-k) of Fig. 1(a); beta is given to every module except the last (Section III-B)."""
    layers: List[List[Layer]] = [[] for _ in range(K)]
    layers[0].append(Layer(STEM, 3, width, 1))
    c = width
    for k in range(K):
        for b in range(blocks):
            if K > 1 and k == (K + 1) // 2 and b == 0:
                layers[k].append(Layer(BASIC_POSTACT, c, 2 * c, 2))
                c = 2 * c
            else:
                layers[k].append(Layer(BASIC_POSTACT, c, c, 1))
    layers[K - 1].append(Layer(HEAD_POSTACT, c))
    specs = []
    cin, h = 3, hw
    for k in range(K):
        sp = ModuleSpec(n=n, c_in=cin, h_in=h, w_in=h, layers=layers[k], delay=2 * (K - 1 - k), is_bottom=(k == 0),
                        num_classes=num_classes, beta=(1.0 if k == K - 1 else beta), momentum=momentum,
                        weight_decay=weight_decay, lr=lr, name="chain%d_module%d" % (K, k))
        specs.append(sp)
        if not sp.is_top:
            _, cin, h, _ = sp.output_shape()
    return specs


def whole_network_spec(specs: Sequence[ModuleSpec]) -> ModuleSpec:
    """The same layers as one module (delay 0, no shrinking): the network the chain was cut from.  Its flat
    parameter vector is the concatenation of the modules' vectors."""
    layers = [L for sp in specs for L in sp.layers]
    s0 = specs[0]
    return ModuleSpec(n=s0.n, c_in=s0.c_in, h_in=s0.h_in, w_in=s0.w_in, layers=layers, delay=0, is_bottom=True,
                      num_classes=s0.num_classes, beta=1.0, momentum=s0.momentum, weight_decay=s0.weight_decay,
                      lr=s0.lr, name="whole_network")


def make_separable_batch(spec: ModuleSpec, step: int, seed: int = 0, noise: float = 0.5):
    """(x, labels) of a classification task a small network learns within tens of iterations: every class has a
    fixed random prototype image (seeded), a sample is its class prototype plus N(0, noise^2)."""
    protos = normal(seed, 900, (spec.num_classes, spec.c_in, spec.h_in, spec.w_in))
    labels = _rng(seed, 901 + 2 * step).integers(0, spec.num_classes, size=spec.n).astype(np.int32)
    x = protos[labels] + noise * normal(seed, 902 + 2 * step, (spec.n, spec.c_in, spec.h_in, spec.w_in))
    return x.astype(np.float32), labels


def wrn_28_10_chain(K: int = 2, n: int = 128, beta: float = 0.7) -> List[ModuleSpec]:
    """The whole WRN-28-10 of the paper's Table VII cut "evenly" into K modules of 12 / K pre-activation blocks
    (K in 1, 2, 3, 4, 6): stem 3 -> 16, 4 blocks of 160 channels at 32x32, 4 of 320 at 16x16, 4 of 640 at 8x8,
    BN/ReLU/average pool/FC.  The stem is this build's conv + BN + ReLU layer (the original has a bare
    convolution there).  Delays 2(K-1-k) as in Fig. 1(a); beta on every module but the last."""
    assert 12 % K == 0
    blocks: List[Layer] = []
    c = 16
    for width, stride in ((160, 1), (320, 2), (640, 2)):
        for b in range(4):
            blocks.append(Layer(BASIC_PREACT, c, width, stride if b == 0 else 1))
            c = width
    per = 12 // K
    hyper = dict(momentum=0.9, weight_decay=5e-4, bn_eps=1e-5, bn_momentum=0.1, lr=0.1)
    specs = []
    cin, h = 3, 32
    for k in range(K):
        ls = ([Layer(STEM, 3, 16, 1)] if k == 0 else []) + blocks[k * per:(k + 1) * per] \
            + ([Layer(HEAD_PREACT, 640)] if k == K - 1 else [])
        sp = ModuleSpec(n, cin, h, h, ls, delay=2 * (K - 1 - k), is_bottom=(k == 0), num_classes=10,
                        beta=(1.0 if k == K - 1 else beta), name="WRN-28-10 K=%d module %d" % (K, k), **hyper)
        specs.append(sp)
        if not sp.is_top:
            _, cin, h, _ = sp.output_shape()
    return specs

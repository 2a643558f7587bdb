"""Pins for the module-level oracle (oracle/fdg_oracle.py): what the paper fixes about one FDG module.

 * Eq. 8-10: inside a module the backward is the chain rule -> whole-module gradients against central
   finite differences in float64 and against torch.autograd on an independent torch model.
 * K=1 / d=0 / beta=1 is standard back-propagation: a net split into K lock-step modules gives the
   gradients and the post-update weights of the unsplit net.
 * Section III-A: the delayed backward uses the activations AND weights of the stale batch: it equals
   a fresh back-propagation at (x_stale, theta_snapshot), times beta (Eq. 15).
 * Eq. 15-17: beta enters linearly; a chain of modules compounds to beta^(K-k); beta=1 is a no-op.
 * Eq. 11/12: the update moves the CURRENT weights with the delayed gradient.
"""
import copy
import math

import numpy as np
import pytest
import torch

import fdg_workloads as W
from fdg_workloads import Layer, ModuleSpec
from oracle.fdg_oracle import NoGrad, OracleModule, QueueEmpty, QueueFull
from tests import torch_ref

TINY = {
    "stem": ModuleSpec(2, 3, 6, 6, [Layer(W.STEM, 3, 4, 1)], is_bottom=False),
    "postact_identity": ModuleSpec(2, 4, 5, 5, [Layer(W.BASIC_POSTACT, 4, 4, 1)]),
    "postact_project": ModuleSpec(2, 4, 6, 6, [Layer(W.BASIC_POSTACT, 4, 6, 2)]),
    "preact_identity": ModuleSpec(2, 4, 5, 5, [Layer(W.BASIC_PREACT, 4, 4, 1)]),
    "preact_project": ModuleSpec(2, 4, 6, 6, [Layer(W.BASIC_PREACT, 4, 6, 2)]),
    "preact_widen": ModuleSpec(2, 4, 5, 5, [Layer(W.BASIC_PREACT, 4, 6, 1)]),
    "head_preact": ModuleSpec(3, 4, 4, 4, [Layer(W.BASIC_PREACT, 4, 4, 1), Layer(W.HEAD_PREACT, 4)], num_classes=5),
    "head_postact": ModuleSpec(3, 4, 4, 4, [Layer(W.BASIC_POSTACT, 4, 4, 1), Layer(W.HEAD_POSTACT, 4)], num_classes=5),
    "bottleneck_identity": ModuleSpec(2, 8, 5, 5, [Layer(W.BOTTLENECK_POSTACT, 8, 8, 1)]),
    "bottleneck_project": ModuleSpec(2, 4, 6, 6, [Layer(W.BOTTLENECK_POSTACT, 4, 8, 2)]),
    "bottleneck_stack_head": ModuleSpec(3, 4, 6, 6, [Layer(W.BOTTLENECK_POSTACT, 4, 8, 1), Layer(W.BOTTLENECK_POSTACT, 8, 8, 2),
                                                    Layer(W.HEAD_POSTACT, 8)], num_classes=5),
    "stem_pool": ModuleSpec(2, 3, 13, 14, [Layer(W.STEM_POOL, 3, 4, 4)], is_bottom=False),
    "stem_pool_stack_head": ModuleSpec(3, 3, 16, 16, [Layer(W.STEM_POOL, 3, 8, 4), Layer(W.BASIC_POSTACT, 8, 8, 1), Layer(W.HEAD_POSTACT, 8)],
                                       num_classes=5),
    "inverted_residual_identity": ModuleSpec(2, 4, 5, 5, [Layer(W.INVERTED_RESIDUAL, 4, 4, 1)]),
    "inverted_residual_stride2": ModuleSpec(2, 4, 6, 7, [Layer(W.INVERTED_RESIDUAL, 4, 8, 2)]),
    "inverted_residual_stack": ModuleSpec(2, 4, 6, 6, [Layer(W.INVERTED_RESIDUAL, 4, 8, 1), Layer(W.INVERTED_RESIDUAL, 8, 8, 1),
                                                     Layer(W.INVERTED_RESIDUAL, 8, 8, 2)]),
    "stack": ModuleSpec(2, 3, 8, 8, [Layer(W.STEM, 3, 4, 1), Layer(W.BASIC_POSTACT, 4, 4, 1),
                                    Layer(W.BASIC_POSTACT, 4, 8, 2), Layer(W.BASIC_POSTACT, 8, 8, 1)]),
}


def _inputs(spec, seed=3):
    theta = W.make_params(spec, seed, perturb_bn=True).astype(np.float64)
    x = W.make_input(spec, 0, seed).astype(np.float64)
    g = W.make_grad_out(spec, 0, seed)
    g = None if g is None else g.astype(np.float64) * 10
    labels = W.make_labels(spec, 0, seed)
    return theta, x, g, labels


@pytest.mark.parametrize("name", list(TINY))
def test_layouts_agree(name):
    spec = TINY[name]
    m = OracleModule(spec)
    assert [(n.split(".", 1)[1], s) for n, s in m.layout] == [(n.split(".", 1)[1], s) for n, s, _ in W.param_shapes(spec)]
    assert m.param_count() == W.param_count(spec)


@pytest.mark.parametrize("name", list(TINY))
def test_module_gradient_against_torch_autograd(name):
    spec = TINY[name]
    theta, x, g, labels = _inputs(spec)
    m = OracleModule(spec, np.float64)
    m.set_params(theta)
    y = m.forward(x, labels)
    gin = m.backward_delayed(g)
    params = torch_ref.split_params(spec, W.param_shapes(spec), theta)
    xt = torch.tensor(x, requires_grad=True)
    out = torch_ref.forward(spec, params, xt, labels)
    if spec.is_top:
        loss, logits = out
        assert math.isclose(y[0], loss.item(), rel_tol=1e-10)
        np.testing.assert_allclose(y[1:], logits.detach().numpy().reshape(-1), rtol=1e-9, atol=1e-11)
        loss.backward()
    else:
        np.testing.assert_allclose(y, out.detach().numpy(), rtol=1e-9, atol=1e-11)
        out.backward(torch.tensor(g) * spec.beta)
    ref = np.concatenate([p.grad.numpy().reshape(-1) for p in params])
    np.testing.assert_allclose(m.get_grads(), ref, rtol=1e-7, atol=1e-10)
    np.testing.assert_allclose(gin, xt.grad.numpy(), rtol=1e-7, atol=1e-10)


@pytest.mark.parametrize("name", list(TINY))
def test_module_gradient_against_finite_differences(name):
    """L(theta, x) = <g, module(x; theta)> (loss for a top module); central differences in float64."""
    spec = TINY[name]
    theta, x, g, labels = _inputs(spec, seed=5)

    def L(th, xx):
        mm = OracleModule(spec, np.float64)
        mm.set_params(th)
        y = mm.forward(xx, labels)
        return float(y[0]) if spec.is_top else float((y * g).sum())

    m = OracleModule(spec, np.float64)
    m.set_params(theta)
    m.forward(x, labels)
    gin = m.backward_delayed(g)
    gth = m.get_grads()
    r = np.random.default_rng(0)
    h = 1e-6
    for i in r.choice(theta.size, size=min(25, theta.size), replace=False):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h
        tm[i] -= h
        fd = (L(tp, x) - L(tm, x)) / (2 * h)
        assert math.isclose(fd, gth[i], rel_tol=2e-5, abs_tol=2e-7), (name, i, fd, gth[i])
    xf = x.reshape(-1)
    for i in r.choice(xf.size, size=15, replace=False):
        xp, xm = xf.copy(), xf.copy()
        xp[i] += h
        xm[i] -= h
        fd = (L(theta, xp.reshape(x.shape)) - L(theta, xm.reshape(x.shape))) / (2 * h)
        assert math.isclose(fd, gin.reshape(-1)[i], rel_tol=2e-5, abs_tol=2e-7), (name, i, fd, gin.reshape(-1)[i])


def _split(spec, cuts, betas, delay=0):
    """Split spec.layers at the given layer indices into consecutive modules."""
    mods, shapes = [], [spec.input_shape()] + spec.activation_shapes()
    bounds = [0] + list(cuts) + [len(spec.layers)]
    for j in range(len(bounds) - 1):
        a, b = bounds[j], bounds[j + 1]
        n, c, h, w = shapes[a]
        mods.append(ModuleSpec(n, c, h, w, spec.layers[a:b], delay=delay, is_bottom=False, num_classes=spec.num_classes,
                               beta=betas[j], momentum=spec.momentum, weight_decay=spec.weight_decay))
    return mods


def _net():
    return ModuleSpec(4, 3, 8, 8, [Layer(W.STEM, 3, 4, 1), Layer(W.BASIC_POSTACT, 4, 4, 1),
                                   Layer(W.BASIC_POSTACT, 4, 8, 2), Layer(W.BASIC_PREACT, 8, 8, 1),
                                   Layer(W.HEAD_PREACT, 8)], num_classes=5)


@pytest.mark.parametrize("cuts", [(2,), (1, 3), (1, 2, 4)])
def test_lockstep_split_equals_standard_bp(cuts):
    """No delay and beta=1: module-wise BP is the chain rule (Eq. 8, Eq. 9), so the split network gives
    the unsplit network's gradient and, after the update, its weights."""
    net = _net()
    theta, x, _, labels = _inputs(net, seed=7)
    whole = OracleModule(net, np.float64)
    whole.set_params(theta)
    y = whole.forward(x, labels)
    gin = whole.backward_delayed(None)
    whole.update(0.1)
    specs = _split(net, cuts, [1.0] * (len(cuts) + 1))
    mods, off = [], 0
    for s in specs:
        m = OracleModule(s, np.float64)
        m.set_params(theta[off:off + m.param_count()])
        off += m.param_count()
        mods.append(m)
    z = x
    for m in mods[:-1]:
        z = m.forward(z)
    yk = mods[-1].forward(z, labels)
    np.testing.assert_allclose(yk, y, rtol=1e-12, atol=1e-13)
    g = mods[-1].backward_delayed(None)
    for m in reversed(mods[:-1]):
        g = m.backward_delayed(g)
    np.testing.assert_allclose(g, gin, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(np.concatenate([m.get_grads() for m in mods]), whole.get_grads(), rtol=1e-10, atol=1e-13)
    for m in mods:
        m.update(0.1)
    np.testing.assert_allclose(np.concatenate([m.get_params() for m in mods]), whole.get_params(), rtol=1e-12, atol=1e-14)


def test_beta_chain_compounds_to_power():
    """Eq. 16 / Eq. 17: with every non-top module shrinking by beta, module k of K sees beta^(K-k) times
    the true gradient; the top module is not shrunk."""
    net, beta = _net(), 0.5
    theta, x, _, labels = _inputs(net, seed=9)
    whole = OracleModule(net, np.float64)
    whole.set_params(theta)
    whole.forward(x, labels)
    whole.backward_delayed(None)
    cuts = (1, 3)
    K = 3
    specs = _split(net, cuts, [beta, beta, 1.0])
    mods, off, ranges = [], 0, []
    for s in specs:
        m = OracleModule(s, np.float64)
        m.set_params(theta[off:off + m.param_count()])
        ranges.append((off, off + m.param_count()))
        off += m.param_count()
        mods.append(m)
    z = x
    for m in mods[:-1]:
        z = m.forward(z)
    mods[-1].forward(z, labels)
    g = mods[-1].backward_delayed(None)
    for m in reversed(mods[:-1]):
        g = m.backward_delayed(g)
    for k1, (m, (a, b)) in enumerate(zip(mods, ranges), start=1):
        np.testing.assert_allclose(m.get_grads(), beta ** (K - k1) * whole.get_grads()[a:b], rtol=1e-10, atol=1e-14)


def test_beta_is_linear_and_exact_for_half():
    spec32 = copy.deepcopy(TINY["stack"])
    theta, x, g, _ = _inputs(spec32, seed=11)
    outs = {}
    for beta in (1.0, 0.5):
        spec32.beta = beta
        m = OracleModule(spec32, np.float32)
        m.set_params(theta)
        m.forward(x)
        gin = m.backward_delayed(g)
        outs[beta] = (m.get_grads(), gin)
    # multiplying by 0.5 is exact in binary floating point, so the whole linear backward scales exactly
    np.testing.assert_array_equal(outs[0.5][0], np.float32(0.5) * outs[1.0][0])
    np.testing.assert_array_equal(outs[0.5][1], np.float32(0.5) * outs[1.0][1])


@pytest.mark.parametrize("d", [1, 3])
def test_delayed_backward_is_fresh_bp_at_stale_batch_and_stale_weights(d):
    """After d further forwards and updates, the backward of the oldest context equals back-propagation
    evaluated at (x_stale, theta at that forward), times beta."""
    spec = copy.deepcopy(TINY["stack"])
    spec.delay, spec.beta = d, 0.2
    theta0 = W.make_params(spec, 1, perturb_bn=True).astype(np.float64)
    m = OracleModule(spec, np.float64)
    m.set_params(theta0)
    xs = [W.make_input(spec, t, 1).astype(np.float64) for t in range(d + 6)]
    gs = [W.make_grad_out(spec, t, 1).astype(np.float64) for t in range(d + 6)]
    snapshots = []
    for t in range(d + 6):
        snapshots.append(m.get_params())
        m.forward(xs[t])
        assert m.queue_state() == (min(t, d) + 1, max(0, t - d), t)
        if t >= d:                      # warm-up: no gradient has arrived before iteration d
            s = t - d                   # the batch whose gradient arrives now
            gin = m.backward_delayed(gs[s])
            fresh_spec = copy.deepcopy(spec)
            fresh_spec.delay, fresh_spec.beta = 0, 1.0
            fresh = OracleModule(fresh_spec, np.float64)
            fresh.set_params(snapshots[s])
            fresh.forward(xs[s])
            gin_fresh = fresh.backward_delayed(gs[s])
            np.testing.assert_allclose(m.get_grads(), spec.beta * fresh.get_grads(), rtol=1e-12, atol=1e-15)
            np.testing.assert_allclose(gin, spec.beta * gin_fresh, rtol=1e-12, atol=1e-15)
            if d > 0 and t > d:
                assert np.abs(snapshots[s] - m.get_params()).max() > 1e-6   # weights have moved meanwhile
            before, v_before = m.get_params(), m.get_momentum()
            m.update(spec.lr)
            # Eq. 11/12: current weights, delayed gradient
            gp = m.get_grads() + spec.weight_decay * before
            v = spec.momentum * v_before + gp
            np.testing.assert_allclose(m.get_params(), before - spec.lr * v, rtol=1e-12, atol=1e-15)


def test_queue_errors():
    spec = copy.deepcopy(TINY["postact_identity"])
    spec.delay = 1
    m = OracleModule(spec)
    theta, x, g, _ = _inputs(spec)
    m.set_params(theta)
    with pytest.raises(QueueEmpty):
        m.backward_delayed(g)
    with pytest.raises(NoGrad):
        m.update(0.1)
    m.forward(x)
    m.forward(x)
    with pytest.raises(QueueFull):
        m.forward(x)
    m.backward_delayed(g)
    m.update(0.1)
    with pytest.raises(NoGrad):
        m.update(0.1)
    assert m.queue_state() == (1, 1, 1)


def test_running_statistics():
    spec = TINY["postact_identity"]
    theta, x, _, _ = _inputs(spec)
    m = OracleModule(spec, np.float64)
    m.set_params(theta)
    m.forward(x)
    c1 = m.k.conv_fwd(x, m.theta["0.conv1.w"], 1, 1)
    M = c1.shape[0] * c1.shape[2] * c1.shape[3]
    rm, rv = m.running["0.bn1"]
    np.testing.assert_allclose(rm, 0.1 * c1.mean(axis=(0, 2, 3)), rtol=1e-12)
    np.testing.assert_allclose(rv, 0.9 + 0.1 * c1.var(axis=(0, 2, 3)) * M / (M - 1), rtol=1e-12)
    assert m.get_bn_running().size == 2 * 2 * 4


# ---- the bf16-storage mode of the oracle ----------------------------------------------------------
def test_round_bf16_against_torch_and_ties_to_even():
    from oracle.fdg_oracle import Kernels
    k = Kernels(np.float32)
    r = np.random.default_rng(0)
    a = np.concatenate([r.standard_normal(10000) * 10.0 ** r.integers(-20, 20, 10000), [0.0, -0.0, 1.0, 3.0e38]]).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(k.round_bf16(a), want)
    # 1 + 2^-8 lies exactly between 1 and 1 + 2^-7: ties go to the even significand (1); 1 + 3*2^-8 goes up
    np.testing.assert_array_equal(k.round_bf16(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8], np.float32)),
                                  np.array([1.0, 1 + 2.0 ** -6], np.float32))
    np.testing.assert_array_equal(k.round_bf16(k.round_bf16(a)), k.round_bf16(a))       # idempotent


def test_bf16_storage_stays_close_to_the_fp32_definition_in_the_forward():
    spec = W.config(1)
    theta, x = W.make_params(spec), W.make_input(spec, 0)
    ys = []
    for storage in ("fp32", "bf16"):
        m = OracleModule(spec, np.float32, storage=storage)
        m.set_params(theta)
        ys.append(m.forward(x))
    assert 0 < np.abs(ys[1] - ys[0]).max() / np.abs(ys[0]).max() < 1e-2


def test_bf16_storage_delayed_backward_equals_fresh_backward_bit_for_bit():
    spec = copy.deepcopy(TINY["stack"])
    spec.delay, spec.beta = 2, 0.2
    m = OracleModule(spec, np.float32, storage="bf16")
    m.set_params(W.make_params(spec, 1, perturb_bn=True))
    xs = [W.make_input(spec, t, 1) for t in range(4)]
    snaps = []
    for t in range(3):
        snaps.append(m.get_params())
        m.forward(xs[t])
        if t >= 1:      # move the weights between the forwards
            m.grad.flat[:] = 0.01
            m.has_grad = True
            m.update(0.1)
    g = W.make_grad_out(spec, 0, 1)
    gin = m.backward_delayed(g)
    fresh_spec = copy.deepcopy(spec)
    fresh_spec.delay = 0
    fresh = OracleModule(fresh_spec, np.float32, storage="bf16")
    fresh.set_params(snaps[0])
    fresh.forward(xs[0])
    gin_fresh = fresh.backward_delayed(g)
    np.testing.assert_array_equal(gin, gin_fresh)
    np.testing.assert_array_equal(m.get_grads(), fresh.get_grads())


def test_why_relu_decisions_are_taken_in_storage_precision():
    """With noise gradients, the fp32 definition and the same steps with bf16-stored operands differ
    by several per cent in the parameter gradients although their forwards agree to 3e-3: the
    difference is carried by the few activations whose ReLU falls the other way."""
    spec = W.config(1)
    theta, x, g = W.make_params(spec), W.make_input(spec, 0), W.make_grad_out(spec, 0)
    out = {}
    for storage in ("fp32", "bf16"):
        spec0 = copy.deepcopy(spec)
        spec0.delay = 0
        m = OracleModule(spec0, np.float32, storage=storage)
        m.set_params(theta)
        y = m.forward(x)
        m.backward_delayed(g)
        out[storage] = (y, m.get_grads())
    flips = np.mean((out["fp32"][0] > 0) != (out["bf16"][0] > 0))
    assert 1e-5 < flips < 2e-3
    gerr = np.abs(out["bf16"][1] - out["fp32"][1]).max() / np.abs(out["fp32"][1]).max()
    assert gerr > 2e-2


def test_bottleneck_gradients_follow_the_summation_order_of_its_convolutions():
    """Why the GPU parity of bottleneck blocks is held to the envelope bar and not to 2e-2 in max norm: noise of the size of a
    changed summation order (3e-7 of a convolution's output, before it is rounded to bf16) moves the kernel-precision
    oracle's own gradients of a bottleneck block (128 -> 32 -> 32 -> 128 channels, 4096 pixels per channel) by per
    cents, and those of a basic block of the same size thirty times less: a value that lands on the neighbouring bf16
    reaches, through the 1x1 convolution over 32 channels, thousands of pre-activations of the block's last ReLU."""
    H = dict(momentum=0.9, weight_decay=5e-4, lr=0.1)
    moved = {}
    for kind in ("bottleneck", "basic"):
        if kind == "bottleneck":
            spec = ModuleSpec(16, 128, 16, 16, [Layer(W.BOTTLENECK_POSTACT, 128, 128, 1)], delay=0, beta=0.5, **H)
        else:
            spec = ModuleSpec(16, 32, 16, 16, [Layer(W.BASIC_POSTACT, 32, 32, 1)], delay=0, beta=0.5, **H)
        theta = W.make_params(spec, 1, perturb_bn=True)
        x, g = W.make_input(spec, 0, 1), W.make_grad_out(spec, 0, 1)
        grads = []
        for trial in range(3):
            m = OracleModule(spec, np.float32, storage="bf16")
            m.set_params(theta)
            if trial:
                r = np.random.default_rng(trial)
                plain = m.k.conv_fwd

                def noisy(x_, w_, s_, p_, plain=plain, r=r):
                    y_ = plain(x_, w_, s_, p_)
                    scale = np.sqrt((y_.astype(np.float64) ** 2).mean())
                    return (y_ + (3e-7 * scale) * r.standard_normal(y_.shape)).astype(y_.dtype)
                m.k.conv_fwd = noisy
            m.forward(x)
            m.backward_delayed(g)
            grads.append(m.get_grads().astype(np.float64))
        moved[kind] = max(np.linalg.norm(grads[t] - grads[0]) / np.linalg.norm(grads[0]) for t in (1, 2))
    assert moved["basic"] < 1e-3
    assert moved["bottleneck"] > 3e-3


@pytest.mark.parametrize("n", [8, 16])
def test_summation_order_noise_saturates_over_the_depth_of_the_wide_module(n):
    """The floor of every end-to-end comparison of the bench workload (WRN-28-10 top module: six wide pre-activation
    blocks and the head), measured on the CPU alone.  Two runs of the SAME bf16-storage oracle that differ only by noise
    of the size of a changed summation order -- 3e-7 of the rms of every convolution result, added before the result is
    stored -- end up 7 .. 13 per cent apart (relative L2) in every 3x3 weight gradient and in the input gradient, while
    their logits agree to 2e-3.  Mechanism: the noise moves one rounding to bf16 in about 1.5e-4 of the elements, each
    block amplifies the difference it inherits, after six blocks the activations differ by about 1e-3, about that share
    of the ReLU gates is decided the other way, and with the loss gradients of random labels a weight gradient is a sum
    of random-sign terms, so a share f of flipped terms is a relative error of sqrt(f).  That floor is 0.6 .. 0.8 of the
    distance between the bf16-storage oracle and the fp32 definition -- the amplification has saturated -- which is why
    an implementation that is exact layer by layer (tests/test_gpu_layerwise.py: 1e-3) still sits about one floor away
    from the oracle end to end, and why the end-to-end envelope of tests/gpu_harness.py is built on this floor."""
    from tests.gpu_harness import _split, rel_l2, with_summation_noise
    spec = W.config(4, n=n)
    theta, x, labels = W.make_params(spec, 0), W.make_input(spec, 0), W.make_labels(spec, 0)
    runs = {}
    for name in ("same", "noisy", "plain"):
        m = OracleModule(spec, np.float32, storage="fp32" if name == "plain" else "bf16")
        if name == "noisy":
            with_summation_noise(m, 1)
        m.set_params(theta)
        y = m.forward(x, labels)
        gin = m.backward_delayed(None)
        runs[name] = (y, dict(_split(spec, m.get_grads())), gin)
    floor = {k: rel_l2(runs["noisy"][1][k], v) for k, v in runs["same"][1].items()}
    inherent = {k: rel_l2(v, runs["plain"][1][k]) for k, v in runs["same"][1].items()}
    assert rel_l2(runs["noisy"][0][1:], runs["same"][0][1:]) < 5e-3          # logits
    convs = [k for k in floor if k.endswith((".conv1.w", ".conv2.w"))]
    assert len(convs) == 12
    for k in convs:
        assert 0.03 < floor[k] < 0.3, (k, floor[k])
        assert floor[k] > 0.5 * inherent[k], (k, floor[k], inherent[k])      # saturated: the size of the fp32-vs-bf16 distance
        assert floor[k] < 1.2 * inherent[k], (k, floor[k], inherent[k])
    fc = [k for k in floor if k.endswith("fc.w")][0]
    assert floor[fc] < 1e-2                                                  # one layer from the loss: nothing to amplify
    assert floor["L0.conv1.w"] > floor["L5.conv2.w"]                         # grows with the depth passed through
    gin_floor = rel_l2(runs["noisy"][2], runs["same"][2])
    assert 0.03 < gin_floor < 0.3

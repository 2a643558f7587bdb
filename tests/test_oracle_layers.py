"""Pins for the layer arithmetic of the CPU oracle (oracle/fdg_oracle_kernels.c).

The paper names its layers only by architecture, so each routine is pinned to what mathematics and
independent libraries fix: scipy's correlate2d, torch's CPU operators and autograd, closed forms,
adjoint identities, finite differences in float64 and brute-force Python loops on tiny inputs."""
import itertools
import math

import numpy as np
import pytest
import scipy.signal
import torch
import torch.nn.functional as F

from oracle.fdg_oracle import Kernels

K64 = Kernels(np.float64)
K32 = Kernels(np.float32)
rng = np.random.default_rng(1234)


def rnd(*shape):
    return rng.standard_normal(shape)


CONV_CASES = [  # N, Ci, H, W, Co, k, stride, pad
    (2, 3, 5, 5, 4, 3, 1, 1),
    (2, 4, 6, 7, 3, 3, 2, 1),
    (1, 2, 5, 4, 5, 3, 2, 1),
    (3, 4, 6, 6, 2, 1, 1, 0),
    (2, 3, 7, 5, 4, 1, 2, 0),
    (2, 3, 8, 8, 4, 1, 2, 0),
]


def brute_conv(x, w, s, p):
    N, Ci, H, W = x.shape
    Co, _, k, _ = w.shape
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    y = np.zeros((N, Co, Ho, Wo))
    for n, co, ho, wo, ci, r, q in itertools.product(range(N), range(Co), range(Ho), range(Wo), range(Ci),
                                                    range(k), range(k)):
        h, ww = ho * s + r - p, wo * s + q - p
        if 0 <= h < H and 0 <= ww < W:
            y[n, co, ho, wo] += x[n, ci, h, ww] * w[co, ci, r, q]
    return y


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_brute_force(case):
    N, Ci, H, W, Co, k, s, p = case
    x, w = rnd(N, Ci, H, W), rnd(Co, Ci, k, k)
    np.testing.assert_allclose(K64.conv_fwd(x, w, s, p), brute_conv(x, w, s, p), rtol=1e-12, atol=1e-12)


def test_conv_fwd_is_scipy_correlation():
    """3x3, pad 1, stride 1 is a 'same' cross-correlation summed over input channels; stride 2 keeps
    every second output of it."""
    x, w = rnd(2, 3, 8, 6), rnd(4, 3, 3, 3)
    full = np.zeros((2, 4, 8, 6))
    for n, co, ci in itertools.product(range(2), range(4), range(3)):
        full[n, co] += scipy.signal.correlate2d(x[n, ci], w[co, ci], mode="same", boundary="fill")
    np.testing.assert_allclose(K64.conv_fwd(x, w, 1, 1), full, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(K64.conv_fwd(x, w, 2, 1), full[:, :, ::2, ::2], rtol=1e-12, atol=1e-12)


def test_conv_1x1_is_matmul():
    x, w = rnd(3, 5, 6, 4), rnd(7, 5, 1, 1)
    np.testing.assert_allclose(K64.conv_fwd(x, w, 1, 0), np.einsum("nchw,oc->nohw", x, w[:, :, 0, 0]), rtol=1e-12)
    np.testing.assert_allclose(K64.conv_fwd(x, w, 2, 0),
                               np.einsum("nchw,oc->nohw", x[:, :, ::2, ::2], w[:, :, 0, 0]), rtol=1e-12)


def test_conv_delta_kernel_shifts():
    """A kernel that is 1 at tap (r,q) of channel c->c copies the image shifted by (r-1, q-1)."""
    x = rnd(1, 2, 5, 5)
    for r, q in itertools.product(range(3), range(3)):
        w = np.zeros((2, 2, 3, 3))
        w[0, 0, r, q] = w[1, 1, r, q] = 1.0
        y = K64.conv_fwd(x, w, 1, 1)
        xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
        np.testing.assert_array_equal(y, xp[:, :, r:r + 5, q:q + 5])


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_adjoint_identities(case):
    """<conv(x,w), g> = <x, dgrad(g,w)> = <w, wgrad(x,g)> because conv is bilinear."""
    N, Ci, H, W, Co, k, s, p = case
    x, w = rnd(N, Ci, H, W), rnd(Co, Ci, k, k)
    y = K64.conv_fwd(x, w, s, p)
    g = rnd(*y.shape)
    lhs = float((y * g).sum())
    assert math.isclose(lhs, float((x * K64.conv_bwd_data(g, w, x.shape, s, p)).sum()), rel_tol=1e-11, abs_tol=1e-11)
    assert math.isclose(lhs, float((w * K64.conv_bwd_weight(x, g, k, s, p)).sum()), rel_tol=1e-11, abs_tol=1e-11)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_against_torch_autograd(case):
    N, Ci, H, W, Co, k, s, p = case
    x, w = rnd(N, Ci, H, W), rnd(Co, Ci, k, k)
    xt, wt = torch.tensor(x, requires_grad=True), torch.tensor(w, requires_grad=True)
    yt = F.conv2d(xt, wt, stride=s, padding=p)
    g = rnd(*yt.shape)
    yt.backward(torch.tensor(g))
    np.testing.assert_allclose(K64.conv_fwd(x, w, s, p), yt.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(K64.conv_bwd_data(g, w, x.shape, s, p), xt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(K64.conv_bwd_weight(x, g, k, s, p), wt.grad.numpy(), rtol=1e-11, atol=1e-12)


def test_bn_fwd_closed_form():
    """Per channel the output has mean beta and variance gamma^2 * var/(var+eps)."""
    x = rnd(4, 3, 5, 6) * np.array([0.5, 2.0, 7.0]).reshape(1, 3, 1, 1) + np.array([3.0, -1.0, 0.2]).reshape(1, 3, 1, 1)
    gamma, beta, eps = np.array([1.5, -0.7, 2.0]), np.array([0.3, 0.1, -2.0]), 1e-5
    y, mean, var, invstd = K64.bn_fwd(x, gamma, beta, eps)
    np.testing.assert_allclose(mean, x.mean(axis=(0, 2, 3)), rtol=1e-12)
    np.testing.assert_allclose(var, x.var(axis=(0, 2, 3)), rtol=1e-12)          # biased
    np.testing.assert_allclose(invstd, 1 / np.sqrt(var + eps), rtol=1e-12)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), beta, atol=1e-12)
    np.testing.assert_allclose(y.var(axis=(0, 2, 3)), gamma ** 2 * var / (var + eps), rtol=1e-11)


def test_bn_bwd_invariants_and_torch():
    x, dy = rnd(3, 4, 5, 5) * 2 + 1, rnd(3, 4, 5, 5)
    gamma, beta, eps = rnd(4) + 2, rnd(4), 1e-5
    _, mean, var, invstd = K64.bn_fwd(x, gamma, beta, eps)
    dx, dgamma, dbeta = K64.bn_bwd(x, dy, gamma, mean, invstd)
    xhat = (x - mean.reshape(1, -1, 1, 1)) * invstd.reshape(1, -1, 1, 1)
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-11)             # shift invariance
    # scale invariance, exact form: sum dx*xhat = gamma*invstd*dgamma * eps/(var+eps)
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 2, 3)), gamma * invstd * dgamma * eps * invstd ** 2,
                               rtol=1e-6, atol=1e-12)
    xt, gt, bt = (torch.tensor(a, requires_grad=True) for a in (x, gamma, beta))
    yt = F.batch_norm(xt, None, None, gt, bt, training=True, eps=eps)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dgamma, gt.grad.numpy(), rtol=1e-10)
    np.testing.assert_allclose(dbeta, bt.grad.numpy(), rtol=1e-10)


def test_bn_bwd_finite_differences():
    x, dy = rnd(2, 2, 3, 3), rnd(2, 2, 3, 3)
    gamma, beta, eps = np.array([1.3, 0.6]), np.array([0.1, -0.4]), 1e-5
    _, mean, var, invstd = K64.bn_fwd(x, gamma, beta, eps)
    dx, _, _ = K64.bn_bwd(x, dy, gamma, mean, invstd)

    def L(xx):
        return float((K64.bn_fwd(xx, gamma, beta, eps)[0] * dy).sum())
    h = 1e-6
    for idx in [(0, 0, 0, 0), (1, 1, 2, 1), (0, 1, 1, 2)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        assert math.isclose((L(xp) - L(xm)) / (2 * h), dx[idx], rel_tol=1e-6, abs_tol=1e-8)


def test_relu():
    x = np.array([-2.0, -0.0, 0.0, 1e-9, 3.0])
    np.testing.assert_array_equal(K64.relu_fwd(x), [0, 0, 0, 1e-9, 3.0])
    np.testing.assert_array_equal(K64.relu_bwd(x, np.ones(5)), [0, 0, 0, 1, 1])   # derivative 0 at 0


def test_avgpool_and_fc_against_numpy_and_torch():
    x = rnd(3, 4, 2, 5)
    np.testing.assert_allclose(K64.avgpool_fwd(x), x.mean(axis=(2, 3)), rtol=1e-12)
    dp = rnd(3, 4)
    np.testing.assert_allclose(K64.avgpool_bwd(dp, x.shape), np.broadcast_to(dp[:, :, None, None] / 10, x.shape), rtol=1e-12)
    p, Wt, b, dl = rnd(3, 4), rnd(6, 4), rnd(6), rnd(3, 6)
    np.testing.assert_allclose(K64.fc_fwd(p, Wt, b), p @ Wt.T + b, rtol=1e-12)
    dWt, db, dpp = K64.fc_bwd(p, Wt, dl)
    np.testing.assert_allclose(dWt, dl.T @ p, rtol=1e-12)
    np.testing.assert_allclose(db, dl.sum(0), rtol=1e-12)
    np.testing.assert_allclose(dpp, dl @ Wt, rtol=1e-12)


def test_softmax_ce_closed_forms():
    N, J = 5, 10
    labels = np.array([0, 3, 9, 3, 1], np.int32)
    loss, dl = K64.softmax_ce(np.full((N, J), 2.5), labels)      # uniform logits -> ln J
    assert math.isclose(loss, math.log(J), rel_tol=1e-12)
    logits = rnd(N, J) * 3
    loss, dl = K64.softmax_ce(logits, labels)
    np.testing.assert_allclose(dl.sum(axis=1), 0, atol=1e-15)    # rows of the gradient sum to zero
    lt = torch.tensor(logits, requires_grad=True)
    lo = F.cross_entropy(lt, torch.tensor(labels, dtype=torch.long))
    lo.backward()
    assert math.isclose(loss, lo.item(), rel_tol=1e-12)
    np.testing.assert_allclose(dl, lt.grad.numpy(), rtol=1e-10, atol=1e-14)
    # shift invariance and no overflow for huge logits
    loss2, _ = K64.softmax_ce(logits + 1000.0, labels)
    assert math.isclose(loss, loss2, rel_tol=1e-9)


def test_sgd_momentum_closed_forms():
    """Constant gradient c, no decay: v_n = c(1-mu^n)/(1-mu), theta_n = theta_0 - lr*sum v_i.
    Decay only, no momentum: theta_n = theta_0 (1 - lr*wd)^n."""
    mu, lr, c, n = 0.9, 0.1, 0.25, 7
    theta, v, g = np.array([1.0, -2.0]), np.zeros(2), np.full(2, c)
    for _ in range(n):
        K64.sgd_momentum(theta, v, g, lr, mu, 0.0)
    vs = [c * (1 - mu ** i) / (1 - mu) for i in range(1, n + 1)]
    np.testing.assert_allclose(v, vs[-1], rtol=1e-12)
    np.testing.assert_allclose(theta, np.array([1.0, -2.0]) - lr * sum(vs), rtol=1e-12)
    theta, v = np.array([1.0, -2.0]), np.zeros(2)
    for _ in range(n):
        K64.sgd_momentum(theta, v, np.zeros(2), lr, 0.0, 5e-4)
    np.testing.assert_allclose(theta, np.array([1.0, -2.0]) * (1 - lr * 5e-4) ** n, rtol=1e-12)


def test_sgd_against_torch_optimizer():
    p0, g = rnd(50), [rnd(50) for _ in range(4)]
    tp = torch.nn.Parameter(torch.tensor(p0))
    opt = torch.optim.SGD([tp], lr=0.1, momentum=0.9, weight_decay=5e-4)
    theta, v = p0.copy(), np.zeros(50)
    for gi in g:
        tp.grad = torch.tensor(gi)
        opt.step()
        K64.sgd_momentum(theta, v, gi, 0.1, 0.9, 5e-4)
    np.testing.assert_allclose(theta, tp.detach().numpy(), rtol=1e-12)


def test_float32_build_matches_float64_build():
    x, w = rnd(2, 8, 6, 6), rnd(8, 8, 3, 3)
    np.testing.assert_allclose(K32.conv_fwd(x, w, 1, 1), K64.conv_fwd(x, w, 1, 1), rtol=1e-4, atol=1e-5)
    g = rnd(2, 8, 6, 6)
    np.testing.assert_allclose(K32.conv_bwd_weight(x, g, 3, 1, 1), K64.conv_bwd_weight(x, g, 3, 1, 1), rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(K32.conv_bwd_data(g, w, x.shape, 1, 1), K64.conv_bwd_data(g, w, x.shape, 1, 1), rtol=1e-4, atol=1e-5)
    y32, y64 = K32.bn_fwd(x, np.ones(8), np.zeros(8), 1e-5)[0], K64.bn_fwd(x, np.ones(8), np.zeros(8), 1e-5)[0]
    np.testing.assert_allclose(y32, y64, rtol=1e-4, atol=1e-5)


# ---- layers of the Tiny-ImageNet networks (Table V): max-pool, depthwise convolution, ReLU6 -------------------------
@pytest.mark.parametrize("shape,k,s,p", [((2, 3, 7, 9), 3, 2, 1), ((1, 2, 8, 8), 3, 2, 1), ((2, 1, 5, 5), 2, 2, 0), ((1, 2, 6, 7), 3, 1, 1)])
def test_maxpool_brute_force_ties_and_torch(shape, k, s, p):
    rng = np.random.default_rng(sum(shape) + k)
    # few distinct values: windows with several equal maxima are the rule, so the tie rule is what is tested
    x = rng.integers(0, 4, shape).astype(np.float64)
    y = K64.maxpool_fwd(x, k, s, p)
    N, C, H, W = shape
    Ho, Wo = y.shape[2:]
    dy = rng.standard_normal(y.shape)
    want_y = np.full(y.shape, -np.inf)
    want_dx = np.zeros(shape)
    for n, c, ho, wo in itertools.product(range(N), range(C), range(Ho), range(Wo)):
        cells = [(ho * s + r - p, wo * s + q - p) for r in range(k) for q in range(k)]
        cells = [(h, w) for h, w in cells if 0 <= h < H and 0 <= w < W]
        vals = [x[n, c, h, w] for h, w in cells]
        m = max(vals)
        want_y[n, c, ho, wo] = m
        h, w = cells[vals.index(m)]          # the first one in scan order
        want_dx[n, c, h, w] += dy[n, c, ho, wo]
    np.testing.assert_array_equal(y, want_y)
    dx = K64.maxpool_bwd(x, dy, k, s, p)
    np.testing.assert_allclose(dx, want_dx, rtol=0, atol=1e-14)
    assert math.isclose(dx.sum(), dy.sum(), rel_tol=1e-12)      # every window hands its gradient to exactly one cell
    xt = torch.tensor(x, requires_grad=True)
    yt = F.max_pool2d(xt, k, stride=s, padding=p)
    np.testing.assert_array_equal(yt.detach().numpy(), y)
    # on inputs without ties torch's gradient is the same map
    x2 = rng.standard_normal(shape)
    xt = torch.tensor(x2, requires_grad=True)
    F.max_pool2d(xt, k, stride=s, padding=p).backward(torch.tensor(dy))
    np.testing.assert_allclose(K64.maxpool_bwd(x2, dy, k, s, p), xt.grad.numpy(), rtol=0, atol=1e-14)


@pytest.mark.parametrize("shape,s", [((2, 5, 7, 6), 1), ((2, 4, 8, 9), 2), ((1, 3, 5, 5), 2)])
def test_depthwise_convolution_is_a_convolution_per_channel(shape, s):
    rng = np.random.default_rng(11 + s)
    N, C, H, W = shape
    x, w = rng.standard_normal(shape), rng.standard_normal((C, 1, 3, 3))
    y = K64.dwconv_fwd(x, w, s, 1)
    # one ordinary single-channel convolution per channel (the dense routine is pinned above)
    for c in range(C):
        np.testing.assert_allclose(y[:, c:c + 1], K64.conv_fwd(x[:, c:c + 1], w[c:c + 1], s, 1), rtol=1e-13, atol=1e-13)
    dy = rng.standard_normal(y.shape)
    dx, dw = K64.dwconv_bwd_data(dy, w, shape, s, 1), K64.dwconv_bwd_weight(x, dy, 3, s, 1)
    # adjoint identities: <dy, conv(x, w)> = <dx, x> = <dw, w>
    assert math.isclose(float((dy * y).sum()), float((dx * x).sum()), rel_tol=1e-11)
    assert math.isclose(float((dy * y).sum()), float((dw * w).sum()), rel_tol=1e-11)
    xt, wt = torch.tensor(x, requires_grad=True), torch.tensor(w, requires_grad=True)
    yt = F.conv2d(xt, wt, stride=s, padding=1, groups=C)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-12, atol=1e-12)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_relu6():
    x = np.array([-1.0, 0.0, 1e-9, 3.0, 6.0 - 1e-9, 6.0, 7.5])
    np.testing.assert_array_equal(K64.relu6_fwd(x), np.array([0.0, 0.0, 1e-9, 3.0, 6.0 - 1e-9, 6.0, 6.0]))
    dy = np.arange(1.0, 8.0)
    want = np.array([0.0, 0.0, 3.0, 4.0, 5.0, 0.0, 0.0])
    np.testing.assert_array_equal(K64.relu6_bwd(x, dy), want)
    np.testing.assert_array_equal(K64.relu6_bwd(K64.relu6_fwd(x), dy), want)     # gated on the clamped output: the same map
    xt = torch.tensor(x, requires_grad=True)
    F.relu6(xt).backward(torch.tensor(dy))
    np.testing.assert_array_equal(xt.grad.numpy(), want)


def test_a_bf16_gradient_rounded_again_after_its_batch_norm_backward_is_rounded_with_a_bias():
    """Why the bf16 storage map keeps the gated gradient of a narrow block in fp32 (OracleModule._layer_backward): the
    batch-norm backward is dy = A g + (B x + C) with small per-channel terms B x + C.  If g already sits on the bf16 grid
    and A g does too (A a power of two here; any A close to a short binary fraction does it in part), rounding dy to bf16
    returns A g wherever |B x + C| is below half a step: the terms that make sum(dy) = 0 are dropped for all large
    elements at once, the rounding errors no longer cancel over the pixels, and a weight gradient -- a sum over all
    pixels against a non-negative input -- inherits an error that grows with the pixel count.  With g in fp32 the same
    rounding is unbiased."""
    K = Kernels(np.float32)
    r = np.random.default_rng(5)
    n, c, h, w = 32, 8, 16, 16
    x = np.maximum(r.standard_normal((n, c, h, w)), 0).astype(np.float32)           # the block input: non-negative
    c1 = (r.standard_normal((n, c, h, w)) * (0.5 + r.random((1, c, 1, 1))) + 0.3).astype(np.float32)
    _, mean, var, invstd = K.bn_fwd(c1, np.ones(c, np.float32), np.zeros(c, np.float32), 1e-5)
    gamma = (1.0 / invstd).astype(np.float32)                                       # A = gamma * invstd = 1
    g = (r.standard_normal((n, c, h, w)) * 1e-2).astype(np.float32) * (r.random((n, c, h, w)) < 0.5)
    pixels = n * h * w

    def bias_and_gradient(g_in):
        dy = K.bn_bwd(c1, g_in, gamma, mean, invstd)[0]
        err = K.round_bf16(dy).astype(np.float64) - dy
        z = err.sum((0, 2, 3)) / (np.sqrt((err ** 2).mean((0, 2, 3))) * np.sqrt(pixels))    # ~ N(0, 1) if unbiased
        return np.abs(z).max(), K.conv_bwd_weight(x, K.round_bf16(dy), 3, 1, 1), K.conv_bwd_weight(x, dy, 3, 1, 1)

    z32, dw32, ref32 = bias_and_gradient(g)
    z16, dw16, ref16 = bias_and_gradient(K.round_bf16(g))
    rel = lambda a, b: float(np.abs(a - b).max() / np.abs(b).max())
    assert z32 < 5.0                      # errors cancel like independent draws
    assert z16 > 8.0                      # they do not: the per-channel sum of the errors is many standard deviations out
    assert rel(dw16, ref16) > 1.5 * rel(dw32, ref32)     # 4.4e-3 against 2.0e-3 at these 8192 pixels; the gap widens with their number

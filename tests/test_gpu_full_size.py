"""The convolution and batch-norm kernels at the benchmarks' full sizes (batch 128: the layers of configuration 4,
and the narrow layers and stems of configurations 2, 3, 5 and 7), in the launch configuration bench.py times,
checked on sub-problems the oracle computes exactly:

  * forward and data gradient are independent per image, so the oracle runs on a few images of the batch
    and those images' outputs are compared element by element;
  * the weight gradient contracts over pixels only, so for a few output and input channels the oracle's
    weight gradient of the channel-restricted operands IS that block of the full gradient;
  * batch norm is independent per channel: the oracle runs on a few channels over all rows;
  * the fused statistics are compared with sums of the tensor the kernel wrote (holds at any size).

Inputs are bf16-representable and given to both sides, so only accumulation order and output rounding
differ (tolerances as in test_gpu_kernels.py)."""
import numpy as np
import pytest

from oracle.fdg_oracle import Kernels

pytestmark = pytest.mark.gpu

F32_TOL = 2e-4
B16_TOL = 2.0 ** -8
K32 = Kernels(np.float32)

# the layer shapes of configuration 4 (WRN-28-10 top module): n, h, w, ci, co, ksize, stride
FULL_CASES = [
    (128, 8, 8, 640, 640, 3, 1),
    (128, 16, 16, 320, 320, 3, 1),
    (128, 16, 16, 320, 640, 3, 2),
    (128, 16, 16, 320, 640, 1, 2),
    # narrow layers (ResNet-110 / ResNet-56 stages, the 64-channel stage at 64x64) and the stems (3 channels stored as 8)
    (128, 32, 32, 16, 16, 3, 1),
    (128, 16, 16, 32, 32, 3, 1),
    (128, 64, 64, 64, 64, 3, 1),
    (128, 32, 32, 3, 16, 3, 1),
    (128, 64, 64, 3, 64, 3, 1),
    # WRN-28-10's 160-channel stage at 32x32 (the lower module of the K = 2 chain): 256-pixel tiles with a partly filled
    # last channel block; the same with a ragged last tile; 128 channels on the 384-row patch
    (128, 32, 32, 160, 160, 3, 1),
    (61, 31, 32, 160, 160, 3, 1),
    (128, 32, 32, 128, 128, 3, 1),
    # the layers of a ResNet-101 bottleneck block of the 1024-channel stage at 14x14
    (128, 14, 14, 1024, 256, 1, 1),
    (128, 14, 14, 256, 256, 3, 1),
    (128, 14, 14, 256, 1024, 1, 1),
    (127, 14, 14, 256, 1024, 1, 1),   # a ragged last pixel tile in the two-workgroups-per-unit form of the short contraction
]
IMAGES = [0, 63, -1]   # first, one inside (modulo the batch), last


def _t():
    import torch
    return torch


def rel(got, ref):
    d = np.abs(ref).max()
    return float(np.abs(np.asarray(got, np.float64) - ref).max() / (d if d > 0 else 1.0))


def _sel(c, wanted):
    """The indices of `wanted` that exist among c channels (negative ones count from the end)."""
    return sorted({i % c for i in wanted if -c <= i < c})


def _pad_last(dev, to):
    """A device tensor with its last dimension zero-filled up to `to` (input channels are stored in eights)."""
    t = _t()
    return dev if dev.shape[-1] == to else t.nn.functional.pad(dev, (0, to - dev.shape[-1])).contiguous()


def _dev_bf16(shape, seed, scale=1.0):
    """A bf16 device tensor of N(0, scale^2) values and the same values on the host in fp32."""
    t = _t()
    g = t.Generator(device="cpu").manual_seed(seed)
    a = (t.randn(shape, generator=g) * scale).to(t.bfloat16)
    return a.cuda(), a.to(t.float32).numpy()


@pytest.mark.parametrize("case", FULL_CASES)
def test_conv_forward_and_data_gradient_on_sampled_images(case):
    from paper_1906_09108_amd import kernels as K
    t = _t()
    n, h, w, ci, co, k, s = case
    print("full-size conv fwd/dgrad", case, flush=True)
    pad = 1 if k == 3 else 0
    ho, wo = (h - 1) // s + 1, (w - 1) // s + 1
    cip = (ci + 7) // 8 * 8
    xd, x = _dev_bf16((n, h, w, ci), 1)                               # NHWC
    wd, wt = _dev_bf16((co, k * k, ci), 2, (2.0 / (ci * k * k)) ** 0.5)  # [co][tap][ci]
    xd, wd = _pad_last(xd, cip), _pad_last(wd, cip)
    w_oihw = wt.reshape(co, k, k, ci).transpose(0, 3, 1, 2).copy()
    y16 = t.zeros((n, ho, wo, co), dtype=t.bfloat16, device="cuda")
    y32 = t.full((n, ho, wo, co), float("nan"), dtype=t.float32, device="cuda")
    stats = K.new_sums(co)
    K.fdgk_conv_fwd(xd, wd, None, y32, y16, stats, n, h, w, ci, co, k, s)
    t.cuda.synchronize()
    imgs = sorted({i % n for i in IMAGES})
    x_sel = x[imgs].transpose(0, 3, 1, 2).copy()
    ref = K32.conv_fwd(x_sel, w_oihw, s, pad).astype(np.float64)       # [3, co, ho, wo]
    got32 = y32[imgs].cpu().numpy().transpose(0, 3, 1, 2)
    got16 = y16[imgs].to(t.float32).cpu().numpy().transpose(0, 3, 1, 2)
    assert rel(got32, ref) <= F32_TOL
    assert rel(got16, ref) <= B16_TOL
    yb = y16.to(t.float64).reshape(-1, co)
    st = K.fdgk_sums_read(stats, co)
    assert rel(st[:co], yb.sum(0).cpu().numpy()) <= 1e-5
    assert rel(st[co:], (yb * yb).sum(0).cpu().numpy()) <= 1e-5
    assert bool(t.isfinite(y32).all())

    # data gradient with the same weights stored [ci][tap][co]
    dyd, dy = _dev_bf16((n, ho, wo, co), 3)
    wtd = wd.permute(2, 1, 0).contiguous()
    dx32 = t.full((n, h, w, cip), float("nan"), dtype=t.float32, device="cuda")
    dx16 = t.zeros((n, h, w, cip), dtype=t.bfloat16, device="cuda")
    K.fdgk_conv_dgrad(dyd, wtd, None, None, dx32, dx16, n, h, w, ci, co, k, s)
    t.cuda.synchronize()
    dy_sel = dy[imgs].transpose(0, 3, 1, 2).copy()
    dref = K32.conv_bwd_data(dy_sel, w_oihw, (len(imgs), ci, h, w), s, pad).astype(np.float64)
    assert rel(dx32[imgs][..., :ci].cpu().numpy().transpose(0, 3, 1, 2), dref) <= F32_TOL
    assert rel(dx16[imgs][..., :ci].to(t.float32).cpu().numpy().transpose(0, 3, 1, 2), dref) <= B16_TOL
    assert bool((dx32[..., ci:] == 0).all())
    assert bool(t.isfinite(dx32).all())


@pytest.mark.parametrize("case", FULL_CASES)
def test_conv_weight_gradient_on_sampled_channels(case):
    from paper_1906_09108_amd import kernels as K
    t = _t()
    n, h, w, ci, co, k, s = case
    print("full-size conv wgrad", case, flush=True)
    pad = 1 if k == 3 else 0
    ho, wo = (h - 1) // s + 1, (w - 1) // s + 1
    xd, x = _dev_bf16((n, h, w, ci), 5)
    dyd, dy = _dev_bf16((n, ho, wo, co), 6)
    cip = (ci + 7) // 8 * 8
    co_sel = _sel(co, [0, 15, 16, 31, 32, 127, 128, co // 2 + 1, -33, -1])   # across MFMA blocks, tiles and both ends
    ci_sel = _sel(ci, [0, 2, 15, 16, 63, 64, ci // 2 - 1, -65, -1])
    x_sel = x[..., ci_sel].transpose(0, 3, 1, 2).copy()
    dy_sel = dy[..., co_sel].transpose(0, 3, 1, 2).copy()
    ref = K32.conv_bwd_weight(x_sel, dy_sel, k, s, pad).astype(np.float64)   # [len(co_sel), len(ci_sel), k, k]
    xd = _pad_last(xd, cip)
    nbytes = K.fdgk_conv_wgrad_scratch_bytes(n, h, w, ci, co, k, s)
    scratch = t.full((max(nbytes // 4, 4),), float("nan"), dtype=t.float32, device="cuda")
    dw = t.full((co, k * k, ci), 7.0, dtype=t.float32, device="cuda")   # unpadded: [co][tap][ci]
    K.fdgk_conv_wgrad(xd, dyd, dw, scratch if nbytes else None, n, h, w, ci, co, k, s, overwrite=True)
    t.cuda.synchronize()
    assert bool(t.isfinite(dw).all())
    got = dw.cpu().numpy().reshape(co, k, k, ci)[co_sel][:, :, :, ci_sel].transpose(0, 3, 1, 2)
    # fp32 accumulation over up to 524288 pixel products of unit-variance operands
    assert rel(got, ref) <= F32_TOL


@pytest.mark.parametrize("m,c", [(128 * 8 * 8, 640), (128 * 16 * 16, 320), (128 * 32 * 32, 16), (128 * 64 * 64, 64), (128 * 14 * 14, 1024), (128 * 14 * 14, 256)])
def test_batch_norm_on_sampled_channels(m, c):
    from paper_1906_09108_amd import kernels as K
    t = _t()
    print("full-size bn", m, c, flush=True)
    eps = 1e-5
    sel = _sel(c, [0, 7, 8, c // 2, -9, -1])
    r = np.random.default_rng(m + c)
    xd, x = _dev_bf16((m, c), 11, 1.5)
    gamma = (1 + 0.2 * r.standard_normal(c)).astype(np.float32)
    beta = (0.2 * r.standard_normal(c)).astype(np.float32)
    gd, bd = t.from_numpy(gamma).cuda(), t.from_numpy(beta).cuda()
    sums = K.new_sums(c)
    K.fdgk_bn_stats(xd, sums, m, c)
    y32 = t.empty((m, c), dtype=t.float32, device="cuda")
    y16 = t.empty((m, c), dtype=t.bfloat16, device="cuda")
    K.fdgk_bn_apply(xd, sums, gd, bd, None, y32, y16, m, c, eps, 1)
    t.cuda.synchronize()
    x4 = x[:, sel].T.reshape(1, len(sel), m, 1).copy()
    y_ref, mean, var, invstd = K32.bn_fwd(x4, gamma[sel], beta[sel], eps)
    out_ref = np.maximum(y_ref.reshape(len(sel), m).T.astype(np.float64), 0)
    assert rel(y32[:, sel].cpu().numpy(), out_ref) <= F32_TOL
    assert rel(y16[:, sel].to(t.float32).cpu().numpy(), out_ref) <= B16_TOL
    # backward through the ReLU gate, fp32 incoming gradient
    dyd = t.randn((m, c), generator=t.Generator(device="cpu").manual_seed(12)).cuda()
    gate = (y16[:, sel].to(t.float32).cpu().numpy() > 0)
    g = (dyd[:, sel].cpu().numpy() * gate).astype(np.float32)
    dx_ref, dgamma_ref, dbeta_ref = K32.bn_bwd(x4, g.T.reshape(1, len(sel), m, 1).copy(), gamma[sel], mean, invstd)
    scratch = K.new_sums(c)
    dx32 = t.empty((m, c), dtype=t.float32, device="cuda")
    dg, db = t.empty(c, dtype=t.float32, device="cuda"), t.empty(c, dtype=t.float32, device="cuda")
    K.fdgk_bn_bwd(dyd, True, y16, xd, sums, gd, scratch, None, dx32, None, dg, db, m, c, eps)
    t.cuda.synchronize()
    assert rel(db[sel].cpu().numpy(), dbeta_ref.astype(np.float64)) <= F32_TOL
    assert rel(dg[sel].cpu().numpy(), dgamma_ref.astype(np.float64)) <= F32_TOL
    assert rel(dx32[:, sel].cpu().numpy(), dx_ref.reshape(len(sel), m).T.astype(np.float64)) <= F32_TOL
    assert bool(t.isfinite(dx32).all())

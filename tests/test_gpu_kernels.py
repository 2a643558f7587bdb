"""Per-kernel GPU parity against the oracle's layer loops.  Inputs are rounded to bf16 first and the
oracle receives exactly those values, so only accumulation order and output rounding differ:
fp32 outputs must agree to 2e-4 of the tensor's largest magnitude, bf16 outputs to 2^-8."""
import numpy as np
import pytest

from oracle.fdg_oracle import Kernels

pytestmark = pytest.mark.gpu

F32_TOL = 2e-4
B16_TOL = 2.0 ** -8
K32 = Kernels(np.float32)


def _torch():
    import torch
    return torch


def bf16_round(a: np.ndarray) -> np.ndarray:
    t = _torch()
    return t.from_numpy(np.ascontiguousarray(a, np.float32)).to(t.bfloat16).to(t.float32).numpy()


def to_dev_nhwc_b16(a_nchw: np.ndarray, cpad: int = 0):
    """NCHW fp32 (already bf16-representable) -> device NHWC bf16, channels zero-padded to cpad."""
    t = _torch()
    x = t.from_numpy(np.ascontiguousarray(a_nchw.transpose(0, 2, 3, 1)))
    if cpad and cpad > x.shape[3]:
        x = t.nn.functional.pad(x, (0, cpad - x.shape[3]))
    return x.to(t.bfloat16).contiguous().cuda()


def to_dev_nhwc_f32(a_nchw: np.ndarray):
    t = _torch()
    return t.from_numpy(np.ascontiguousarray(a_nchw.transpose(0, 2, 3, 1))).contiguous().cuda()


def nhwc_to_nchw(tns) -> np.ndarray:
    t = _torch()
    return tns.to(t.float32).cpu().numpy().transpose(0, 3, 1, 2)


def rel(got, ref):
    d = np.abs(ref).max()
    return float(np.abs(np.asarray(got, np.float64) - ref).max() / (d if d > 0 else 1.0))


CONV_CASES = [  # n, h, w, ci, co, ksize, stride
    (3, 7, 5, 16, 16, 3, 1),
    (2, 8, 8, 16, 32, 3, 2),
    (2, 9, 7, 8, 24, 3, 2),
    (2, 6, 6, 96, 160, 3, 1),
    (3, 7, 5, 16, 160, 3, 1),      # the first block of a wide network: the narrow forward kernel with ten channel blocks
    (16, 32, 32, 16, 160, 3, 1),
    (4, 8, 8, 32, 32, 1, 2),
    (3, 7, 7, 16, 40, 1, 2),
    (2, 5, 5, 24, 16, 1, 1),
    (2, 6, 5, 3, 16, 3, 1),
    (2, 16, 16, 64, 64, 3, 1),
    (8, 8, 8, 320, 320, 3, 1),
    (4, 16, 16, 160, 320, 3, 2),
    (16, 32, 32, 16, 16, 3, 1),
    (4, 16, 16, 16, 160, 3, 1),     # many output channels from few inputs: the 128 x 32 weight-gradient tiles
    (2, 9, 9, 24, 136, 1, 1),
    # wide layers (input channels a multiple of 64): the direct-to-LDS kernel, both tile widths, ragged pixels
    (2, 8, 8, 64, 160, 3, 1),
    (3, 7, 5, 128, 128, 3, 1),
    (2, 8, 8, 320, 640, 3, 2),
    (3, 9, 7, 192, 320, 3, 2),
    (2, 8, 8, 320, 640, 1, 2),
    (5, 4, 4, 128, 192, 1, 1),
    (16, 8, 8, 640, 640, 3, 1),
    (3, 6, 6, 136, 128, 3, 1),      # input channels = 2 chunks of 64 + 8: the partly filled last chunk
    # the pipelined gather kernel at the short end: one step (forward), two steps, fewer steps than stages in flight
    (2, 8, 8, 64, 128, 1, 1),
    (3, 5, 7, 128, 160, 1, 1),
    (2, 6, 6, 64, 192, 1, 2),
    (1, 8, 40, 64, 128, 3, 1),      # rows longer than 32 pixels: nine steps through the gather form instead of the patch form
    (2, 4, 36, 136, 160, 3, 1),     # the same with a partly filled last chunk
    (2, 8, 8, 200, 160, 1, 2),
    # channel counts that are multiples of 160: the transposing direct-to-LDS weight-gradient kernel
    (3, 4, 4, 160, 160, 3, 1),
    (5, 8, 8, 160, 320, 3, 1),
    (3, 16, 16, 320, 160, 3, 2),
    # narrow layers (16 / 32 / 64 channels in and out, 3x3, unit stride): patch and filter on chip; ragged tiles,
    # odd widths, every tile size, a row wider than a tile
    (4, 16, 16, 32, 32, 3, 1),
    (2, 5, 9, 32, 32, 3, 1),
    (3, 8, 8, 64, 64, 3, 1),
    (1, 64, 64, 64, 64, 3, 1),
    (2, 33, 31, 16, 16, 3, 1),
    (40, 16, 16, 32, 32, 3, 1),
    (64, 16, 16, 32, 32, 3, 1),
    (9, 64, 64, 64, 64, 3, 1),
    # stems: 3 input channels (stored as 8) into a narrow layer
    (8, 32, 32, 3, 16, 3, 1),
    (2, 64, 64, 3, 64, 3, 1),
    (3, 9, 7, 3, 32, 3, 1),
    # degenerate images: one pixel, one row, one column (every tap but the centre falls outside)
    (1, 1, 1, 16, 16, 3, 1),
    (2, 1, 7, 32, 32, 3, 1),
    (2, 7, 1, 16, 16, 3, 1),
    (3, 2, 2, 64, 64, 3, 1),
    # the 1x1 convolutions of bottleneck blocks: down to a quarter of the channels and back up
    (16, 16, 16, 128, 32, 1, 1),
    (16, 16, 16, 32, 128, 1, 1),
    (4, 14, 14, 1024, 256, 1, 1),
    (4, 14, 14, 256, 1024, 1, 1),
    (4, 14, 14, 256, 256, 3, 1),
    (16, 14, 14, 256, 128, 1, 1),   # pixels a multiple of 64, width not a divisor of 64: the weight gradient sees rows of 32
    (16, 14, 14, 128, 256, 1, 1),
    # 3x3 at widths that do not divide 64 (and a 64-row image): the weight gradient's flat form
    (16, 14, 14, 128, 256, 3, 1),
    (64, 7, 7, 128, 128, 3, 1),
    (1, 64, 64, 128, 128, 3, 1),
    (48, 6, 10, 128, 128, 3, 1),
]


def _conv_data(case, seed):
    n, h, w, ci, co, k, s = case
    r = np.random.default_rng(seed)
    x = bf16_round(r.standard_normal((n, ci, h, w)))
    wt = bf16_round(r.standard_normal((co, ci, k, k)) * np.sqrt(2.0 / (ci * k * k)))
    ho, wo = (h - 1) // s + 1, (w - 1) // s + 1
    dy = bf16_round(r.standard_normal((n, co, ho, wo)))
    return x, wt, dy, ho, wo


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd(case):
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, ci, co, k, s = case
    print("conv_fwd", case, flush=True)
    x, wt, _, ho, wo = _conv_data(case, 1)
    cip = (ci + 7) // 8 * 8
    ref = K32.conv_fwd(x, wt, s, 1 if k == 3 else 0).astype(np.float64)
    xd = to_dev_nhwc_b16(x, cip)
    wd = t.nn.functional.pad(t.from_numpy(wt.transpose(0, 2, 3, 1).copy()), (0, cip - ci)).to(t.bfloat16).contiguous().cuda()
    add = np.random.default_rng(2).standard_normal(ref.shape).astype(np.float32)
    y32 = t.full((n, ho, wo, co), float("nan"), dtype=t.float32, device="cuda")
    y16 = t.zeros((n, ho, wo, co), dtype=t.bfloat16, device="cuda")
    stats = K.new_sums(co)
    K.fdgk_conv_fwd(xd, wd, None, y32, y16, stats, n, h, w, ci, co, k, s)
    t.cuda.synchronize()
    assert rel(nhwc_to_nchw(y32), ref) <= F32_TOL
    assert rel(nhwc_to_nchw(y16), ref) <= B16_TOL
    # fused batch-norm statistics: sums of the bf16 values just written
    yb = y16.to(t.float64).reshape(-1, co)
    got = K.fdgk_sums_read(stats, co)
    assert rel(got[:co], yb.sum(0).cpu().numpy()) <= 1e-5
    assert rel(got[co:], (yb * yb).sum(0).cpu().numpy()) <= 1e-5
    K.fdgk_conv_fwd(xd, wd, to_dev_nhwc_f32(add), y32, None, None, n, h, w, ci, co, k, s)
    t.cuda.synchronize()
    assert rel(nhwc_to_nchw(y32), ref + add) <= F32_TOL


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_dgrad(case):
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, ci, co, k, s = case
    print("conv_dgrad", case, flush=True)
    x, wt, dy, ho, wo = _conv_data(case, 3)
    cip = (ci + 7) // 8 * 8
    ref = K32.conv_bwd_data(dy, wt, x.shape, s, 1 if k == 3 else 0).astype(np.float64)
    dyd = to_dev_nhwc_b16(dy)
    # [cip][k*k][co]
    wtd = t.nn.functional.pad(t.from_numpy(wt.transpose(1, 2, 3, 0).copy()), (0, 0, 0, 0, 0, 0, 0, cip - ci))
    wtd = wtd.to(t.bfloat16).contiguous().cuda()
    dx32 = t.full((n, h, w, cip), float("nan"), dtype=t.float32, device="cuda")
    dx16 = t.zeros((n, h, w, cip), dtype=t.bfloat16, device="cuda")
    K.fdgk_conv_dgrad(dyd, wtd, None, None, dx32, dx16, n, h, w, ci, co, k, s)
    t.cuda.synchronize()
    got = nhwc_to_nchw(dx32)
    assert rel(got[:, :ci], ref) <= F32_TOL
    assert np.all(got[:, ci:] == 0)
    assert rel(nhwc_to_nchw(dx16)[:, :ci], ref) <= B16_TOL
    # masked addend (the identity shortcut through a ReLU)
    r = np.random.default_rng(4)
    add = r.standard_normal((n, cip, h, w)).astype(np.float32)
    mask = bf16_round(np.maximum(r.standard_normal((n, cip, h, w)), 0))
    K.fdgk_conv_dgrad(dyd, wtd, to_dev_nhwc_f32(add), to_dev_nhwc_b16(mask), dx32, None, n, h, w, ci, co, k, s)
    t.cuda.synchronize()
    full = np.zeros((n, cip, h, w))
    full[:, :ci] = ref
    assert rel(nhwc_to_nchw(dx32), full + add * (mask > 0)) <= F32_TOL


GATED_CASES = [  # data gradients the wide kernels run: output (= layer input) channels >= 128, co % 64 == 0
    (2, 8, 8, 128, 64, 3, 1),
    (3, 7, 5, 160, 128, 3, 1),      # ragged pixel tile, 160-wide tile
    (16, 8, 8, 640, 640, 3, 1),     # patch form
    (3, 9, 7, 192, 320, 3, 2),      # four parity classes, odd sizes
    (2, 8, 8, 320, 640, 1, 2),      # three of the four classes have no tap: zeros (plus addend) gated
    (5, 4, 4, 128, 192, 1, 1),
    (2, 8, 8, 160, 160, 3, 1),      # contraction over 160 channels: a partly filled last 64-channel chunk
    (2, 8, 8, 160, 136, 3, 2),      # the same with parity classes (136 = 2 chunks + 8 channels)
    # narrow layers: the gate and the sums in the output stage of the narrow kernel
    (3, 7, 5, 16, 16, 3, 1),
    (16, 32, 32, 16, 16, 3, 1),
    (4, 16, 16, 32, 32, 3, 1),
    (3, 8, 8, 64, 64, 3, 1),
]


@pytest.mark.parametrize("case", GATED_CASES)
def test_gated_data_gradient_feeds_the_batch_norm_backward(case):
    """conv_dgrad_gated leaves g = gate > 0 ? dgrad + addend : 0 and the sums [sum g, sum g*x] of its bf16 values;
    bn_bwd_gated turns them into dgamma, dbeta and dx.  Reference: the oracle's data gradient, the gate and the
    rounding applied in numpy, then the oracle's batch-norm backward on that rounded g."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, ci, co, k, s = case
    print("gated dgrad", case, flush=True)
    assert K.fdgk_conv_dgrad_gates(n, h, w, ci, co, k, s)
    x_unused, wt, dy, ho, wo = _conv_data(case, 11)
    r = np.random.default_rng(12)
    ref = K32.conv_bwd_data(dy, wt, x_unused.shape, s, 1 if k == 3 else 0).astype(np.float64)
    add = r.standard_normal(ref.shape).astype(np.float32) * 0.5
    gate = bf16_round(np.maximum(r.standard_normal(ref.shape), 0))            # a ReLU output: about half closed
    bnx = bf16_round(r.standard_normal(ref.shape) * (0.5 + r.random((1, ci, 1, 1))) + r.standard_normal((1, ci, 1, 1)))
    dyd = to_dev_nhwc_b16(dy)
    wtd = t.from_numpy(wt.transpose(1, 2, 3, 0).copy()).to(t.bfloat16).contiguous().cuda()
    gsums = K.new_sums(ci)
    g32 = t.full((n, h, w, ci), float("nan"), dtype=t.float32, device="cuda")
    g16 = t.zeros((n, h, w, ci), dtype=t.bfloat16, device="cuda")
    K.fdgk_conv_dgrad_gated(dyd, wtd, to_dev_nhwc_f32(add), to_dev_nhwc_b16(gate), to_dev_nhwc_b16(bnx), gsums, g32, g16,
                            n, h, w, ci, co, k, s)
    t.cuda.synchronize()
    g_ref = (ref + add) * (gate > 0)
    assert rel(nhwc_to_nchw(g32), g_ref) <= F32_TOL
    assert rel(nhwc_to_nchw(g16), g_ref) <= B16_TOL
    assert np.all(nhwc_to_nchw(g32)[gate <= 0] == 0)
    # the sums are those of the bf16 values written (holds exactly up to summation order)
    gb = g16.to(t.float64).reshape(-1, ci).cpu().numpy()
    xb = to_dev_nhwc_b16(bnx).to(t.float64).reshape(-1, ci).cpu().numpy()
    got = K.fdgk_sums_read(gsums, ci)
    assert rel(got[:ci], gb.sum(0)) <= 1e-5
    assert rel(got[ci:], (gb * xb).sum(0)) <= 1e-5
    # batch-norm backward from those sums against the oracle's on the same rounded g
    m = n * h * w
    eps = 1e-5
    gamma = (1 + 0.2 * r.standard_normal(ci)).astype(np.float32)
    x4 = xb.T.reshape(1, ci, m, 1).astype(np.float32)
    _, mean, var, invstd = K32.bn_fwd(x4, gamma, np.zeros(ci, np.float32), eps)
    dx_ref, dgamma_ref, dbeta_ref = K32.bn_bwd(x4, gb.T.reshape(1, ci, m, 1).astype(np.float32), gamma, mean, invstd)
    xd = to_dev_nhwc_b16(bnx).reshape(m, ci)
    sums = K.new_sums(ci)
    K.fdgk_bn_stats(xd, sums, m, ci)
    res = r.standard_normal((m, ci)).astype(np.float32)
    dx32 = t.empty((m, ci), dtype=t.float32, device="cuda")
    dx16 = t.empty((m, ci), dtype=t.bfloat16, device="cuda")
    dg, db = t.empty(ci, dtype=t.float32, device="cuda"), t.empty(ci, dtype=t.float32, device="cuda")
    K.fdgk_bn_bwd_gated(g16.reshape(m, ci), xd, sums, t.from_numpy(gamma).cuda(), gsums, t.from_numpy(res).cuda(), dx32, dx16,
                        dg, db, m, ci, eps)
    t.cuda.synchronize()
    assert rel(db.cpu().numpy(), dbeta_ref.astype(np.float64)) <= F32_TOL
    assert rel(dg.cpu().numpy(), dgamma_ref.astype(np.float64)) <= F32_TOL
    dref = dx_ref.reshape(ci, m).T.astype(np.float64) + res
    assert rel(dx32.cpu().numpy(), dref) <= F32_TOL
    assert rel(dx16.to(t.float32).cpu().numpy(), dref) <= B16_TOL


PAIR_CASES = [  # (n, h, w, ci, co): 3x3 stride-2 layer with a 1x1 stride-2 projection beside it
    (2, 8, 8, 128, 128),
    (3, 9, 7, 192, 320),       # odd sizes: parity classes of different extent, ragged pixel tiles
    (16, 16, 16, 320, 640),    # WRN-28-10's second transition at a reduced batch: several tiles per class
    (2, 6, 6, 160, 192),       # 160 output channels of the data gradient: one ragged 160-wide tile
]


@pytest.mark.parametrize("case", PAIR_CASES)
def test_gated_data_gradient_of_a_projecting_block(case):
    """conv_dgrad_gated_pair = gate > 0 ? dgrad of the 3x3 stride-2 convolution + dgrad of the 1x1 stride-2 projection : 0,
    with the sums of its bf16 values.  Reference: the oracle's two data gradients added, gated in numpy."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, ci, co = case
    print("gated dgrad pair", case, flush=True)
    assert K.fdgk_conv_dgrad_pair_applies(n, h, w, ci, co)
    x_unused, wt, dy, ho, wo = _conv_data((n, h, w, ci, co, 3, 2), 21)
    _, wt2, dy2, ho2, wo2 = _conv_data((n, h, w, ci, co, 1, 2), 22)
    assert (ho, wo) == (ho2, wo2)
    r = np.random.default_rng(23)
    ref = (K32.conv_bwd_data(dy, wt, x_unused.shape, 2, 1).astype(np.float64) +
           K32.conv_bwd_data(dy2, wt2, x_unused.shape, 2, 0).astype(np.float64))
    gate = bf16_round(np.maximum(r.standard_normal(ref.shape), 0))
    bnx = bf16_round(r.standard_normal(ref.shape) * (0.5 + r.random((1, ci, 1, 1))) + r.standard_normal((1, ci, 1, 1)))
    wtd = t.from_numpy(wt.transpose(1, 2, 3, 0).copy()).to(t.bfloat16).contiguous().cuda()
    wtd2 = t.from_numpy(wt2.transpose(1, 2, 3, 0).copy()).to(t.bfloat16).contiguous().cuda()
    gsums = K.new_sums(ci)
    g32 = t.full((n, h, w, ci), float("nan"), dtype=t.float32, device="cuda")
    g16 = t.zeros((n, h, w, ci), dtype=t.bfloat16, device="cuda")
    K.fdgk_conv_dgrad_gated_pair(to_dev_nhwc_b16(dy), wtd, to_dev_nhwc_b16(dy2), wtd2, to_dev_nhwc_b16(gate), to_dev_nhwc_b16(bnx),
                                 gsums, g32, g16, n, h, w, ci, co)
    t.cuda.synchronize()
    g_ref = ref * (gate > 0)
    assert rel(nhwc_to_nchw(g32), g_ref) <= F32_TOL
    assert rel(nhwc_to_nchw(g16), g_ref) <= B16_TOL
    assert np.all(nhwc_to_nchw(g32)[gate <= 0] == 0)
    # the projection reaches the even pixels only: elsewhere the result is the 3x3 data gradient alone
    only3 = K32.conv_bwd_data(dy, wt, x_unused.shape, 2, 1).astype(np.float64) * (gate > 0)
    odd = np.ones((h, w), bool)
    odd[::2, ::2] = False
    assert rel(nhwc_to_nchw(g32)[:, :, odd], only3[:, :, odd]) <= F32_TOL
    gb = g16.to(t.float64).reshape(-1, ci).cpu().numpy()
    xb = to_dev_nhwc_b16(bnx).to(t.float64).reshape(-1, ci).cpu().numpy()
    got = K.fdgk_sums_read(gsums, ci)
    assert rel(got[:ci], gb.sum(0)) <= 1e-5
    assert rel(got[ci:], (gb * xb).sum(0)) <= 1e-5
    # without a gate: the plain sum of the two data gradients (a post-activation block whose shortcut projects)
    p32 = t.full((n, h, w, ci), float("nan"), dtype=t.float32, device="cuda")
    K.fdgk_conv_dgrad_gated_pair(to_dev_nhwc_b16(dy), wtd, to_dev_nhwc_b16(dy2), wtd2, None, None, None, p32, None, n, h, w, ci, co)
    t.cuda.synchronize()
    assert rel(nhwc_to_nchw(p32), ref) <= F32_TOL


def test_gated_pair_refuses_what_it_does_not_cover():
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    assert not K.fdgk_conv_dgrad_pair_applies(2, 8, 8, 32, 64)     # narrow layer
    assert not K.fdgk_conv_dgrad_pair_applies(2, 1, 1, 128, 128)   # a single pixel
    z = t.zeros(16, dtype=t.bfloat16, device="cuda")
    st = K.new_sums(32)
    with pytest.raises(RuntimeError):
        K.fdgk_conv_dgrad_gated_pair(z, z, z, z, z, z, st, None, z, 2, 8, 8, 32, 64)


@pytest.mark.parametrize("case", [(3, 7, 5, 16, 16, 3, 1), (16, 32, 32, 16, 16, 3, 1), (4, 16, 16, 32, 32, 3, 1), (3, 8, 8, 64, 64, 3, 1),
                                  (9, 64, 64, 64, 64, 3, 1),
                                  (25, 14, 14, 1024, 256, 1, 1)])   # 1x1 of a bottleneck block: the two-workgroup wide kernel
def test_data_gradient_that_feeds_the_layer_below(case):
    """conv_dgrad_feeding_next: g = gate > 0 ? dgrad + addend * [addmask > 0] : 0 in fp32 (and its bf16 copy), and the
    sums [sum g, sum g * x] of the FP32 values.  Reference: the oracle's data gradient, gate and mask applied in numpy."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, ci, co, k, s = case
    print("dgrad feeding next", case, flush=True)
    x_unused, wt, dy, ho, wo = _conv_data(case, 21)
    r = np.random.default_rng(22)
    ref = K32.conv_bwd_data(dy, wt, x_unused.shape, s, 1 if k == 3 else 0).astype(np.float64)
    add = r.standard_normal(ref.shape).astype(np.float32) * 0.5
    mask = bf16_round(np.maximum(r.standard_normal(ref.shape), 0))
    gate = bf16_round(np.maximum(r.standard_normal(ref.shape), 0))
    bnx = bf16_round(r.standard_normal(ref.shape) * (0.5 + r.random((1, ci, 1, 1))) + r.standard_normal((1, ci, 1, 1)))
    wtd = t.from_numpy(wt.transpose(1, 2, 3, 0).copy()).to(t.bfloat16).contiguous().cuda()
    gsums = K.new_sums(ci)
    g32 = t.full((n, h, w, ci), float("nan"), dtype=t.float32, device="cuda")
    g16 = t.zeros((n, h, w, ci), dtype=t.bfloat16, device="cuda")
    K.fdgk_conv_dgrad_feeding_next(to_dev_nhwc_b16(dy), wtd, to_dev_nhwc_f32(add), to_dev_nhwc_b16(mask), to_dev_nhwc_b16(gate),
                                   to_dev_nhwc_b16(bnx), gsums, g32, g16, n, h, w, ci, co, k, s)
    t.cuda.synchronize()
    g_ref = (ref + add * (mask > 0)) * (gate > 0)
    got32 = nhwc_to_nchw(g32)
    assert rel(got32, g_ref) <= F32_TOL
    assert rel(nhwc_to_nchw(g16), g_ref) <= B16_TOL
    assert np.all(got32[gate <= 0] == 0)
    gf = g32.to(t.float64).reshape(-1, ci).cpu().numpy()
    xb = to_dev_nhwc_b16(bnx).to(t.float64).reshape(-1, ci).cpu().numpy()
    got = K.fdgk_sums_read(gsums, ci)
    assert rel(got[:ci], gf.sum(0)) <= 1e-5
    assert rel(got[ci:], (gf * xb).sum(0)) <= 1e-5
    # and they are NOT the sums of the bf16 copy wherever the two differ measurably
    gb = g16.to(t.float64).reshape(-1, ci).cpu().numpy()
    assert np.abs(got[ci:] - (gf * xb).sum(0)).max() <= np.abs(got[ci:] - (gb * xb).sum(0)).max() + 1e-3 * np.abs(got[ci:]).max()


def test_gated_data_gradient_refuses_layers_without_such_a_kernel():
    """Neither the wide kernels nor the narrow one take a 24 -> 40 layer or a stride-2 16 -> 32 layer."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    assert not K.fdgk_conv_dgrad_gates(2, 8, 8, 24, 40, 3, 1)
    assert not K.fdgk_conv_dgrad_gates(2, 8, 8, 16, 32, 3, 2)
    z = t.zeros(2 * 8 * 8 * 40, dtype=t.bfloat16, device="cuda")
    w = t.zeros(24 * 9 * 40, dtype=t.bfloat16, device="cuda")
    st = t.zeros(48, dtype=t.float32, device="cuda")
    with pytest.raises(RuntimeError):
        K.fdgk_conv_dgrad_gated(z, w, None, z, z, st, None, z, 2, 8, 8, 24, 40, 3, 1)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_wgrad(case):
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, ci, co, k, s = case
    print("conv_wgrad", case, flush=True)
    x, wt, dy, ho, wo = _conv_data(case, 5)
    cip = (ci + 7) // 8 * 8
    ref = K32.conv_bwd_weight(x, dy, k, s, 1 if k == 3 else 0).astype(np.float64)   # [co, ci, k, k]
    xd, dyd = to_dev_nhwc_b16(x, cip), to_dev_nhwc_b16(dy)
    dw = t.zeros((co, k * k, ci), dtype=t.float32, device="cuda")
    K.fdgk_conv_wgrad(xd, dyd, dw, None, n, h, w, ci, co, k, s)                     # splits added with atomics
    t.cuda.synchronize()
    got = dw.cpu().numpy().reshape(co, k, k, ci).transpose(0, 3, 1, 2)
    assert rel(got, ref) <= F32_TOL
    nbytes = K.fdgk_conv_wgrad_scratch_bytes(n, h, w, ci, co, k, s)
    if nbytes:                                                                      # splits through scratch
        scratch = t.full((nbytes // 4,), float("nan"), dtype=t.float32, device="cuda")
        dw2 = t.ones((co, k * k, ci), dtype=t.float32, device="cuda")               # the result is ADDED to dw
        K.fdgk_conv_wgrad(xd, dyd, dw2, scratch, n, h, w, ci, co, k, s)
        t.cuda.synchronize()
        got = dw2.cpu().numpy().reshape(co, k, k, ci).transpose(0, 3, 1, 2) - 1.0
        assert rel(got, ref) <= F32_TOL
    else:
        scratch = None
    for scr in (None, scratch):                                                     # overwrite: prior contents do not count
        dw3 = t.full((co, k * k, ci), 7.0, dtype=t.float32, device="cuda")
        K.fdgk_conv_wgrad(xd, dyd, dw3, scr, n, h, w, ci, co, k, s, overwrite=True)
        t.cuda.synchronize()
        got = dw3.cpu().numpy().reshape(co, k, k, ci).transpose(0, 3, 1, 2)
        assert rel(got, ref) <= F32_TOL


FWD_BN_CASES = [  # (n, h, w, c): narrow layers, unit stride
    (3, 7, 5, 16),        # ragged tile, odd image
    (16, 32, 32, 16),     # several tiles per image
    (128, 32, 32, 16),    # the ResNet-110 stage at the bench batch: 512 tiles of 256 pixels
    (8, 16, 16, 32),
    (128, 16, 16, 32),
    (5, 8, 8, 64),
    (128, 8, 8, 64),
]


@pytest.mark.parametrize("with_res", [False, True])
@pytest.mark.parametrize("case", FWD_BN_CASES)
def test_convolution_with_batch_norm_on_its_patch(case, with_res):
    """fdgk_conv_fwd_bn: act = relu(batchnorm(x_raw) [+ res]) written in bf16 (and fp32) and y = conv(act, w).  Reference: the
    oracle's batch norm (fp32 definition) on x_raw, the shortcut, ReLU, then the oracle's convolution of the bf16 values the
    kernel wrote; and the fused launch against the two launches it replaces (fdgk_bn_apply, then fdgk_conv_fwd), which must
    agree to a bf16 step of act."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, c = case
    print("conv_fwd_bn", case, with_res, flush=True)
    assert K.fdgk_conv_fwd_bn_applies(n, h, w, c, c, with_res)
    r = np.random.default_rng(31 + n + c)
    eps, mom = 1e-5, 0.1
    m = n * h * w
    x = bf16_round(r.standard_normal((n, c, h, w)) * (0.5 + r.random((1, c, 1, 1))) + r.standard_normal((1, c, 1, 1)))
    wt = bf16_round(r.standard_normal((c, c, 3, 3)) * np.sqrt(2.0 / (c * 9)))
    gamma = (1 + 0.2 * r.standard_normal(c)).astype(np.float32)
    beta = (0.2 * r.standard_normal(c)).astype(np.float32)
    y_bn, mean, var, invstd = K32.bn_fwd(x, gamma, beta, eps)
    res = r.standard_normal((n, c, h, w)).astype(np.float32) if with_res else None
    act_ref = np.maximum(y_bn.astype(np.float64) + (res if with_res else 0.0), 0)
    resd = to_dev_nhwc_f32(res) if with_res else None
    xd = to_dev_nhwc_b16(x)
    sums = K.new_sums(c)
    K.fdgk_bn_stats(xd.reshape(m, c), sums, m, c)
    wd = t.from_numpy(wt.transpose(0, 2, 3, 1).copy()).to(t.bfloat16).contiguous().cuda()
    gd, bd = t.from_numpy(gamma).cuda(), t.from_numpy(beta).cuda()
    rm0, rv0 = r.standard_normal(c).astype(np.float32), (1 + r.random(c)).astype(np.float32)
    rm, rv = t.from_numpy(rm0.copy()).cuda(), t.from_numpy(rv0.copy()).cuda()
    act = t.full((n, h, w, c), float("nan"), dtype=t.bfloat16, device="cuda")
    act32 = t.full((n, h, w, c), float("nan"), dtype=t.float32, device="cuda")
    y16 = t.full((n, h, w, c), float("nan"), dtype=t.bfloat16, device="cuda")
    st = K.new_sums(c)
    K.fdgk_conv_fwd_bn(xd, sums, gd, bd, eps, resd, act, act32, rm, rv, mom, wd, y16, st, n, h, w, c, c)
    t.cuda.synchronize()
    act_got = nhwc_to_nchw(act)
    assert rel(act_got, act_ref) <= B16_TOL
    assert rel(nhwc_to_nchw(act32), act_ref) <= F32_TOL
    assert np.all(act_got >= 0)
    # the convolution of exactly the values written
    y_ref = K32.conv_fwd(act_got.astype(np.float32), wt, 1, 1).astype(np.float64)
    y_got = nhwc_to_nchw(y16)
    assert rel(y_got, y_ref) <= B16_TOL
    yb = y16.to(t.float64).reshape(-1, c).cpu().numpy()
    got = K.fdgk_sums_read(st, c)
    assert rel(got[:c], yb.sum(0)) <= 1e-5
    assert rel(got[c:], (yb * yb).sum(0)) <= 1e-5
    # running statistics: one step with the unbiased variance
    unbias = m / (m - 1.0)
    assert rel(rm.cpu().numpy(), (1 - mom) * rm0 + mom * mean.astype(np.float64)) <= 1e-5
    assert rel(rv.cpu().numpy(), (1 - mom) * rv0 + mom * var.astype(np.float64) * unbias) <= 1e-4
    # the two launches it replaces
    act2 = t.empty((m, c), dtype=t.bfloat16, device="cuda")
    y2 = t.empty((n, h, w, c), dtype=t.bfloat16, device="cuda")
    K.fdgk_bn_apply(xd.reshape(m, c), sums, gd, bd, resd.reshape(m, c) if with_res else None, None, act2, m, c, eps, 1)
    K.fdgk_conv_fwd(act2, wd, None, None, y2, None, n, h, w, c, c, 3, 1)
    t.cuda.synchronize()
    assert rel(act.to(t.float32).reshape(m, c).cpu().numpy(), act2.to(t.float32).cpu().numpy().astype(np.float64)) <= 2.0 ** -8
    assert rel(nhwc_to_nchw(y16), nhwc_to_nchw(y2)) <= B16_TOL


@pytest.mark.parametrize("g_f32", [False, True])
@pytest.mark.parametrize("case", [(3, 7, 5, 16), (16, 32, 32, 16), (128, 16, 16, 32), (5, 8, 8, 64), (128, 8, 8, 64)])
def test_data_gradient_with_batch_norm_backward_on_its_patch(case, g_f32):
    """fdgk_conv_dgrad_bn on a gated gradient g with its sums, as the data gradient of the convolution ABOVE leaves them
    (fdgk_conv_dgrad_gated: bf16 g, sums of the bf16 values; fdgk_conv_dgrad_feeding_next: fp32 g, sums of the fp32 values).
    Reference: the oracle's batch-norm backward of that g, rounded to bf16 as the kernel writes it, then the oracle's data
    gradient; and the two launches it replaces (fdgk_bn_bwd_gated, fdgk_conv_dgrad)."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, c = case
    print("conv_dgrad_bn", case, g_f32, flush=True)
    assert K.fdgk_conv_dgrad_bn_applies(n, h, w, c, c, g_f32)
    m = n * h * w
    eps = 1e-5
    r = np.random.default_rng(41 + n + c)
    full = (n, h, w, c, c, 3, 1)
    _, w_up, dy_up, _, _ = _conv_data(full, 42)                      # the convolution above: its data gradient makes g
    _, wt, _, _, _ = _conv_data(full, 43)                            # the convolution whose data gradient is under test
    gate = bf16_round(np.maximum(r.standard_normal((n, c, h, w)), 0))
    x = bf16_round(r.standard_normal((n, c, h, w)) * (0.5 + r.random((1, c, 1, 1))) + r.standard_normal((1, c, 1, 1)))
    gamma = (1 + 0.2 * r.standard_normal(c)).astype(np.float32)
    tr = lambda a: t.from_numpy(a.transpose(1, 2, 3, 0).copy()).to(t.bfloat16).contiguous().cuda()
    gsums = K.new_sums(c)
    g32 = t.zeros((n, h, w, c), dtype=t.float32, device="cuda")
    g16 = t.zeros((n, h, w, c), dtype=t.bfloat16, device="cuda")
    xd, gated = to_dev_nhwc_b16(x), to_dev_nhwc_b16(gate)
    if g_f32:
        K.fdgk_conv_dgrad_feeding_next(to_dev_nhwc_b16(dy_up), tr(w_up), None, None, gated, xd, gsums, g32, g16, n, h, w, c, c, 3, 1)
    else:
        K.fdgk_conv_dgrad_gated(to_dev_nhwc_b16(dy_up), tr(w_up), None, gated, xd, gsums, None, g16, n, h, w, c, c, 3, 1)
    sums = K.new_sums(c)
    K.fdgk_bn_stats(xd.reshape(m, c), sums, m, c)
    gd = t.from_numpy(gamma).cuda()
    add = r.standard_normal((n, c, h, w)).astype(np.float32)
    mask = bf16_round(np.maximum(r.standard_normal((n, c, h, w)), 0))
    dy16 = t.full((n, h, w, c), float("nan"), dtype=t.bfloat16, device="cuda")
    dx32 = t.full((n, h, w, c), float("nan"), dtype=t.float32, device="cuda")
    dx16 = t.zeros((n, h, w, c), dtype=t.bfloat16, device="cuda")
    dg, db = t.empty(c, dtype=t.float32, device="cuda"), t.empty(c, dtype=t.float32, device="cuda")
    K.fdgk_conv_dgrad_bn(g32 if g_f32 else g16, g_f32, xd, sums, gsums, gd, eps, dy16, dg, db, tr(wt), to_dev_nhwc_f32(add),
                         to_dev_nhwc_b16(mask), dx32, dx16, n, h, w, c, c)
    t.cuda.synchronize()
    # oracle: batch-norm backward of the g the kernel read
    g_host = nhwc_to_nchw(g32 if g_f32 else g16).astype(np.float32)
    _, mean, var, invstd = K32.bn_fwd(x.astype(np.float32), gamma, np.zeros(c, np.float32), eps)
    dy_ref, dgamma_ref, dbeta_ref = K32.bn_bwd(x.astype(np.float32), g_host, gamma, mean, invstd)
    assert rel(db.cpu().numpy(), dbeta_ref.astype(np.float64)) <= F32_TOL
    assert rel(dg.cpu().numpy(), dgamma_ref.astype(np.float64)) <= F32_TOL
    dy_got = nhwc_to_nchw(dy16)
    assert rel(dy_got, dy_ref.astype(np.float64)) <= B16_TOL
    # the data gradient of exactly the values written, plus the masked addend
    dx_ref = K32.conv_bwd_data(dy_got.astype(np.float32), wt, x.shape, 1, 1).astype(np.float64) + add * (mask > 0)
    assert rel(nhwc_to_nchw(dx32), dx_ref) <= F32_TOL
    assert rel(nhwc_to_nchw(dx16), dx_ref) <= B16_TOL
    # the two launches it replaces
    dy2 = t.empty((m, c), dtype=t.bfloat16, device="cuda")
    dg2, db2 = t.empty(c, dtype=t.float32, device="cuda"), t.empty(c, dtype=t.float32, device="cuda")
    if not g_f32:
        K.fdgk_bn_bwd_gated(g16.reshape(m, c), xd.reshape(m, c), sums, gd, gsums, None, None, dy2, dg2, db2, m, c, eps)
        t.cuda.synchronize()
        assert rel(dy16.to(t.float32).reshape(m, c).cpu().numpy(), dy2.to(t.float32).cpu().numpy().astype(np.float64)) <= 2.0 ** -8
        assert rel(dg.cpu().numpy(), dg2.cpu().numpy().astype(np.float64)) <= 1e-5
        assert rel(db.cpu().numpy(), db2.cpu().numpy().astype(np.float64)) <= 1e-6


def test_conv_fwd_bn_refuses_what_it_does_not_cover():
    from paper_1906_09108_amd import kernels as K
    assert not K.fdgk_conv_fwd_bn_applies(2, 8, 8, 128, 128)      # wide layer
    assert not K.fdgk_conv_fwd_bn_applies(2, 8, 8, 16, 32)        # channels change
    assert not K.fdgk_conv_fwd_bn_applies(128, 64, 64, 64, 64)    # more tiles than a workgroup each may take
    assert not K.fdgk_conv_fwd_bn_applies(128, 64, 64, 64, 64, True)


BN_CASES = [(189, 16), (4096, 16), (1000, 40), (512, 640), (16384, 32), (77, 2048)]


@pytest.mark.parametrize("m,c", BN_CASES)
def test_bn_forward_and_backward(m, c):
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    print("bn", m, c, flush=True)
    r = np.random.default_rng(m + c)
    eps = 1e-5
    x = bf16_round(r.standard_normal((m, c)) * (0.5 + r.random(c)) + r.standard_normal(c))
    gamma = (1 + 0.2 * r.standard_normal(c)).astype(np.float32)
    beta = (0.2 * r.standard_normal(c)).astype(np.float32)
    res = r.standard_normal((m, c)).astype(np.float32)
    x4 = x.T.reshape(1, c, m, 1)                      # oracle layout: N=1, C, H=m, W=1
    y_ref, mean, var, invstd = K32.bn_fwd(x4, gamma, beta, eps)
    xd = t.from_numpy(x).to(t.bfloat16).cuda()
    sums = K.new_sums(c)
    K.fdgk_bn_stats(xd, sums, m, c)
    t.cuda.synchronize()
    s = K.fdgk_sums_read(sums, c)
    assert rel(s[:c] / m, mean.astype(np.float64)) <= 1e-5
    assert rel(s[c:] / m - (s[:c] / m) ** 2, var.astype(np.float64)) <= 1e-4
    gd, bd = t.from_numpy(gamma).cuda(), t.from_numpy(beta).cuda()
    y32 = t.empty((m, c), dtype=t.float32, device="cuda")
    y16 = t.empty((m, c), dtype=t.bfloat16, device="cuda")
    K.fdgk_bn_apply(xd, sums, gd, bd, None, y32, y16, m, c, eps, 0)
    t.cuda.synchronize()
    ref2d = y_ref.reshape(c, m).T.astype(np.float64)
    assert rel(y32.cpu().numpy(), ref2d) <= F32_TOL
    K.fdgk_bn_apply(xd, sums, gd, bd, t.from_numpy(res).cuda(), y32, y16, m, c, eps, 1)
    t.cuda.synchronize()
    out_ref = np.maximum(ref2d + res, 0)
    assert rel(y32.cpu().numpy(), out_ref) <= F32_TOL
    assert rel(y16.to(t.float32).cpu().numpy(), out_ref) <= B16_TOL
    # backward through the ReLU gate and the normalisation, for both gradient storage types
    mask = y16                                         # gate = ReLU output > 0, as the module uses it
    gate = (mask.to(t.float32).cpu().numpy() > 0)
    for dy_is_f32 in (True, False):
        dy = r.standard_normal((m, c)).astype(np.float32)
        if not dy_is_f32:
            dy = bf16_round(dy)
        g = (dy * gate).astype(np.float32)
        dx_ref, dgamma_ref, dbeta_ref = K32.bn_bwd(x4, g.T.reshape(1, c, m, 1), gamma, mean, invstd)
        add = r.standard_normal((m, c)).astype(np.float32)
        dyd = t.from_numpy(dy).cuda() if dy_is_f32 else t.from_numpy(dy).to(t.bfloat16).cuda()
        scratch = K.new_sums(c)
        dx32 = t.empty((m, c), dtype=t.float32, device="cuda")
        dx16 = t.empty((m, c), dtype=t.bfloat16, device="cuda")
        dg, db = t.empty(c, dtype=t.float32, device="cuda"), t.empty(c, dtype=t.float32, device="cuda")
        K.fdgk_bn_bwd(dyd, dy_is_f32, mask, xd, sums, gd, scratch, t.from_numpy(add).cuda(), dx32, dx16, dg, db, m, c, eps)
        t.cuda.synchronize()
        assert rel(db.cpu().numpy(), dbeta_ref.astype(np.float64)) <= F32_TOL
        assert rel(dg.cpu().numpy(), dgamma_ref.astype(np.float64)) <= F32_TOL
        dref = dx_ref.reshape(c, m).T.astype(np.float64) + add
        assert rel(dx32.cpu().numpy(), dref) <= F32_TOL
        assert rel(dx16.to(t.float32).cpu().numpy(), dref) <= B16_TOL


@pytest.mark.parametrize("count", [4, 1024, 4672, 1 << 20])
def test_sgd(count):
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    r = np.random.default_rng(count)
    theta, v, g = (r.standard_normal(count).astype(np.float32) for _ in range(3))
    td, vd, gd = (t.from_numpy(a.copy()).cuda() for a in (theta, v, g))
    for _ in range(3):
        K32.sgd_momentum(theta, v, g, 0.1, 0.9, 5e-4)
        K.fdgk_sgd(td, vd, gd, count, 0.1, 0.9, 5e-4)
    t.cuda.synchronize()
    assert rel(td.cpu().numpy(), theta.astype(np.float64)) <= 1e-6
    assert rel(vd.cpu().numpy(), v.astype(np.float64)) <= 1e-6


@pytest.mark.parametrize("ratio", [30.0, 300.0])
def test_batch_norm_with_a_mean_far_from_zero(ratio):
    """|mean| / sigma = 30 and 300 per channel.  The statistics are sum x and sum x^2; their totals are exact and the
    variance sum x^2 / m - mean^2 is taken in double, so the cancellation costs nothing beyond the fp32 rounding of a
    workgroup's partial sum of squares (1e-7 * ratio^2 of the variance); a plain fp32 evaluation of that formula
    loses ratio^2 * 6e-8 = 5e-3 (ratio 300) on top."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    m, c = 8192, 64
    eps = 1e-5
    r = np.random.default_rng(int(ratio))
    sigma = 0.5 + r.random(c)
    x = bf16_round(r.standard_normal((m, c)) * sigma + ratio * sigma * np.sign(r.standard_normal(c)))
    gamma = (1 + 0.2 * r.standard_normal(c)).astype(np.float32)
    beta = (0.2 * r.standard_normal(c)).astype(np.float32)
    x4 = x.T.reshape(1, c, m, 1)
    y_ref, mean, var, invstd = K32.bn_fwd(x4, gamma, beta, eps)          # two passes, double accumulation
    xd = t.from_numpy(x).to(t.bfloat16).cuda()
    sums = K.new_sums(c)
    K.fdgk_bn_stats(xd, sums, m, c)
    y32 = t.empty((m, c), dtype=t.float32, device="cuda")
    K.fdgk_bn_apply(xd, sums, t.from_numpy(gamma).cuda(), t.from_numpy(beta).cuda(), None, y32, None, m, c, eps, 0)
    t.cuda.synchronize()
    tol = 2e-4 if ratio <= 30 else 2e-2      # bf16 inputs this far from zero have only a few steps across their spread
    assert rel(y32.cpu().numpy(), y_ref.reshape(c, m).T) <= tol
    # backward through a ReLU gate
    dy = r.standard_normal((m, c)).astype(np.float32)
    mask = bf16_round(r.standard_normal((m, c)))
    g = (dy * (mask > 0)).astype(np.float32)
    dx_ref, dgamma_ref, dbeta_ref = K32.bn_bwd(x4, g.T.reshape(1, c, m, 1).copy(), gamma, mean, invstd)
    dx32 = t.empty((m, c), dtype=t.float32, device="cuda")
    dg, db = t.empty(c, dtype=t.float32, device="cuda"), t.empty(c, dtype=t.float32, device="cuda")
    K.fdgk_bn_bwd(t.from_numpy(dy).cuda(), True, t.from_numpy(mask).to(t.bfloat16).cuda(), xd, sums, t.from_numpy(gamma).cuda(),
                  K.new_sums(c), None, dx32, None, dg, db, m, c, eps)
    t.cuda.synchronize()
    assert rel(db.cpu().numpy(), dbeta_ref) <= 2e-4
    assert rel(dg.cpu().numpy(), dgamma_ref) <= tol
    assert rel(dx32.cpu().numpy(), dx_ref.reshape(c, m).T) <= tol


# ---- classifier head and layout kernels ---------------------------------------------------------------------------
HEAD_CASES = [  # n, h, w, c, classes
    (128, 8, 8, 640, 10),     # WRN-28-10 head at its full size (the bench workload)
    (16, 8, 8, 64, 10),       # ResNet-110 head
    (5, 7, 7, 2048, 200),     # ResNet-101 head, ragged batch
    (3, 4, 4, 512, 200),      # ResNet-18 head at Tiny-ImageNet resolution
    (1, 1, 1, 8, 2),
]


@pytest.mark.parametrize("case", HEAD_CASES)
def test_head_kernels_one_by_one(case):
    """Average pool, fully connected layer, softmax cross-entropy and their backward kernels, each on the same inputs as the
    oracle's loop for it (the head of a top module: it produces the loss and the first gradient of Eq. 8)."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, c, J = case
    print("head case", case, flush=True)
    rng = np.random.default_rng(100 + c + n)
    o = bf16_round(rng.standard_normal((n, c, h, w)).astype(np.float32) + 0.3)
    Wt = (rng.standard_normal((J, c)) / np.sqrt(c)).astype(np.float32)
    b = (0.1 * rng.standard_normal(J)).astype(np.float32)
    labels = rng.integers(0, J, n).astype(np.int32)
    dev = "cuda:0"
    # pool
    pooled = t.empty((n, c), dtype=t.float32, device=dev)
    K.fdgk_avgpool(to_dev_nhwc_b16(o), pooled, n, h * w, c)
    p_ref = K32.avgpool_fwd(o)
    assert rel(pooled.cpu().numpy(), p_ref) <= 1e-5
    # fully connected, on the oracle's pooled features
    p_dev = t.from_numpy(p_ref).to(dev)
    W_dev, b_dev = t.from_numpy(Wt).to(dev), t.from_numpy(b).to(dev)
    logits = t.empty((n, J), dtype=t.float32, device=dev)
    K.fdgk_fc_fwd(p_dev, W_dev, b_dev, logits, n, c, J)
    l_ref = K32.fc_fwd(p_ref, Wt, b)
    assert rel(logits.cpu().numpy(), l_ref) <= 1e-5
    # loss
    y = t.empty(1 + n * J, dtype=t.float32, device=dev)
    dl = t.empty((n, J), dtype=t.float32, device=dev)
    K.fdgk_softmax_ce(t.from_numpy(l_ref).to(dev), t.from_numpy(labels).to(dev), y, dl, n, J)
    loss_ref, dl_ref = K32.softmax_ce(l_ref, labels)
    yh = y.cpu().numpy()
    assert abs(float(yh[0]) - loss_ref) <= 1e-5 * max(1.0, abs(loss_ref))
    assert np.array_equal(yh[1:].reshape(n, J), l_ref)            # the logits are handed through unchanged
    assert rel(dl.cpu().numpy(), dl_ref) <= 1e-5
    # backward of the fully connected layer
    dW, db, dp = t.empty((J, c), dtype=t.float32, device=dev), t.empty(J, dtype=t.float32, device=dev), t.empty((n, c), dtype=t.float32, device=dev)
    K.fdgk_fc_bwd(p_dev, W_dev, t.from_numpy(dl_ref).to(dev), dW, db, dp, n, c, J)
    dW_ref, db_ref, dp_ref = K32.fc_bwd(p_ref, Wt, dl_ref)
    assert rel(dW.cpu().numpy(), dW_ref) <= 1e-5
    # db[j] = sum_n dl[n, j] is a sum of terms of both signs that nearly cancel (a softmax row sums to one): absolute bar
    assert np.abs(db.cpu().numpy() - db_ref).max() <= 1e-6
    assert rel(dp.cpu().numpy(), dp_ref) <= 1e-5
    # backward of the pool: both outputs
    g32 = t.empty((n, h, w, c), dtype=t.float32, device=dev)
    g16 = t.empty((n, h, w, c), dtype=t.bfloat16, device=dev)
    K.fdgk_pool_bwd(t.from_numpy(dp_ref).to(dev), g32, g16, n, h * w, c)
    g_ref = K32.avgpool_bwd(dp_ref, (n, c, h, w))
    assert rel(nhwc_to_nchw(g32), g_ref) <= 1e-6
    assert np.array_equal(nhwc_to_nchw(g16), bf16_round(nhwc_to_nchw(g32)))   # the bf16 copy is the rounded fp32 value


def test_avgpool_refuses_a_channel_count_it_has_no_vector_loads_for():
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    o = t.zeros((2, 4, 12), dtype=t.bfloat16, device="cuda:0")
    pooled = t.zeros((2, 12), dtype=t.float32, device="cuda:0")
    assert K.fdgk_avgpool(o, pooled, 2, 4, 12, check=False) != 0


LAYOUT_CASES = [  # n, c, h, w, channel pitch
    (128, 320, 16, 16, 320),   # the input of the bench workload's module
    (4, 3, 32, 32, 8),         # an image batch: 3 channels padded to 8
    (3, 24, 17, 15, 24),       # ragged tiles both ways
    (2, 10, 5, 7, 16),
    (1, 1, 1, 1, 8),
]


@pytest.mark.parametrize("case", LAYOUT_CASES)
def test_layout_kernels(case):
    """NCHW fp32 -> NHWC (fp32 and bf16, scaled by beta of Eq. 15, padding channels zero) and back: moves and one rounding,
    so the results are exact."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, c, h, w, cp = case
    print("layout case", case, flush=True)
    rng = np.random.default_rng(7 + c)
    x = rng.standard_normal((n, c, h, w)).astype(np.float32)
    src = t.from_numpy(x).cuda()
    for scale in (1.0, 0.5, 0.2):
        d32 = t.full((n, h, w, cp), 7.0, dtype=t.float32, device="cuda:0")
        d16 = t.full((n, h, w, cp), 7.0, dtype=t.bfloat16, device="cuda:0")
        K.fdgk_nchw_to_nhwc(src, d32, d16, n, c, h * w, cp, scale)
        want = np.zeros((n, h, w, cp), np.float32)
        want[..., :c] = (x * np.float32(scale)).transpose(0, 2, 3, 1)
        got32 = d32.cpu().numpy()
        assert np.array_equal(got32, want)
        assert np.array_equal(d16.to(t.float32).cpu().numpy(), bf16_round(want))
        back = t.full((n, c, h, w), 7.0, dtype=t.float32, device="cuda:0")
        K.fdgk_nhwc_to_nchw(d32, back, n, c, h * w, cp)
        assert np.array_equal(back.cpu().numpy(), x * np.float32(scale))
    # only one of the two outputs
    d16 = t.full((n, h, w, cp), 7.0, dtype=t.bfloat16, device="cuda:0")
    K.fdgk_nchw_to_nhwc(src, None, d16, n, c, h * w, cp, 1.0)
    assert np.array_equal(d16.to(t.float32).cpu().numpy()[..., :c], bf16_round(x.transpose(0, 2, 3, 1)))
    assert K.fdgk_nchw_to_nhwc(src, None, None, n, c, h * w, cp, 1.0, check=False) != 0
    assert K.fdgk_nchw_to_nhwc(src, None, d16, n, c, h * w, c - 1, 1.0, check=False) != 0


# ---- layers of the Tiny-ImageNet networks: 7x7 stem as gathered rows, max-pool, depthwise convolution ----------------
@pytest.mark.parametrize("case", [(4, 64, 64, 3, 64), (3, 13, 14, 3, 16), (2, 9, 7, 5, 8)])
def test_stem7_as_gathered_rows_and_a_1x1_contraction(case):
    """conv7x7 / stride 2 / padding 3 = fdgk_im2col7 followed by fdgk_conv_fwd with ksize 1 over 448 elements, and its weight
    gradient fdgk_conv_wgrad on the same rows; compared with the oracle's 7x7 convolution."""
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, ci, co = case
    print("stem7 case", case, flush=True)
    rng = np.random.default_rng(70 + h)
    x = bf16_round(rng.standard_normal((n, ci, h, w)).astype(np.float32))
    wgt = bf16_round((rng.standard_normal((co, ci, 7, 7)) * np.sqrt(2.0 / (49 * ci))).astype(np.float32))
    ho, wo = (h - 1) // 2 + 1, (w - 1) // 2 + 1
    x8 = to_dev_nhwc_b16(x, 8)
    col = t.full((n, ho, wo, 448), 3.0, dtype=t.bfloat16, device="cuda:0")
    K.fdgk_im2col7(x8, col, n, h, w)
    # the rows themselves: exact copies
    colh = col.to(t.float32).cpu().numpy().reshape(n, ho, wo, 7, 8, 8)
    xp = np.zeros((n, h + 6, w + 8, 8), np.float32)
    xp[:, 3:3 + h, 3:3 + w, :ci] = x.transpose(0, 2, 3, 1)
    for kh in range(7):
        for kw in range(8):
            want = xp[:, kh:kh + 2 * ho:2, kw:kw + 2 * wo:2, :] if kw < 7 else 0.0
            assert np.array_equal(colh[:, :, :, kh, kw, :], np.broadcast_to(want, (n, ho, wo, 8))), (kh, kw)
    # weights in the same order: [co][kh][kw of 8][c of 8]
    w448 = np.zeros((co, 7, 8, 8), np.float32)
    w448[:, :, :7, :ci] = wgt.transpose(0, 2, 3, 1)
    w_dev = t.from_numpy(w448.reshape(co, 448)).to(t.bfloat16).cuda()
    y = t.empty((n, ho, wo, co), dtype=t.float32, device="cuda:0")
    K.fdgk_conv_fwd(col, w_dev, None, y, None, None, n, ho, wo, 448, co, 1, 1)
    ref = K32.conv_fwd(x, wgt, 2, 3)
    assert rel(nhwc_to_nchw(y), ref) <= F32_TOL
    dy = bf16_round(rng.standard_normal(ref.shape).astype(np.float32))
    dw = t.empty((co, 448), dtype=t.float32, device="cuda:0")
    nb = K.fdgk_conv_wgrad_scratch_bytes(n, ho, wo, 448, co, 1, 1)
    scratch = t.empty(max(nb // 4, 1), dtype=t.float32, device="cuda:0")
    K.fdgk_conv_wgrad(col, to_dev_nhwc_b16(dy), dw, scratch, n, ho, wo, 448, co, 1, 1, overwrite=True)
    dwh = dw.cpu().numpy().reshape(co, 7, 8, 8)
    ref_dw = K32.conv_bwd_weight(x, dy, 7, 2, 3)
    assert rel(dwh[:, :, :7, :ci].transpose(0, 3, 1, 2), ref_dw) <= F32_TOL
    assert not dwh[:, :, 7, :].any() and not dwh[:, :, :, ci:].any()       # the padding of the layout gets no gradient


@pytest.mark.parametrize("case", [(8, 32, 32, 64), (3, 7, 9, 16), (2, 8, 8, 24), (1, 1, 1, 8), (2, 33, 32, 64)])
def test_maxpool_forward_and_backward(case):
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, c = case
    print("maxpool case", case, flush=True)
    rng = np.random.default_rng(80 + h + c)
    # a ReLU output in bf16: many zeros and many equal values, so ties are common and the tie rule matters
    x = bf16_round(np.maximum(rng.standard_normal((n, c, h, w)), 0).astype(np.float32))
    x = bf16_round(np.round(x * 4) / 4)
    ho, wo = (h - 1) // 2 + 1, (w - 1) // 2 + 1
    xd = to_dev_nhwc_b16(x)
    y32 = t.empty((n, ho, wo, c), dtype=t.float32, device="cuda:0")
    y16 = t.empty((n, ho, wo, c), dtype=t.bfloat16, device="cuda:0")
    K.fdgk_maxpool3s2(xd, y32, y16, n, h, w, c)
    ref = K32.maxpool_fwd(x, 3, 2, 1)
    assert np.array_equal(nhwc_to_nchw(y32), ref)
    assert np.array_equal(nhwc_to_nchw(y16), ref)
    dy = rng.standard_normal(ref.shape).astype(np.float32)
    dx = t.full((n, h, w, c), 9.0, dtype=t.float32, device="cuda:0")
    K.fdgk_maxpool3s2_bwd(xd, to_dev_nhwc_f32(dy), dx, n, h, w, c)
    ref_dx = K32.maxpool_bwd(x, dy, 3, 2, 1)
    assert rel(nhwc_to_nchw(dx), ref_dx) <= 1e-6          # sums of at most four terms


@pytest.mark.parametrize("case", [(8, 16, 16, 192, 1), (8, 32, 32, 192, 2), (3, 7, 9, 24, 1), (2, 9, 7, 40, 2), (16, 8, 8, 576, 1), (1, 1, 1, 8, 1)])
def test_depthwise_convolution_kernels(case):
    from paper_1906_09108_amd import kernels as K
    t = _torch()
    n, h, w, c, s = case
    print("depthwise case", case, flush=True)
    rng = np.random.default_rng(90 + h + c + s)
    x = bf16_round(rng.standard_normal((n, c, h, w)).astype(np.float32))
    wgt = bf16_round((rng.standard_normal((c, 1, 3, 3)) * np.sqrt(2.0 / 9)).astype(np.float32))
    wt = t.from_numpy(np.ascontiguousarray(wgt.reshape(c, 9).T)).to(t.bfloat16).cuda()     # [9][c]
    ho, wo = (h - 1) // s + 1, (w - 1) // s + 1
    xd = to_dev_nhwc_b16(x)
    y = t.empty((n, ho, wo, c), dtype=t.bfloat16, device="cuda:0")
    K.fdgk_dwconv3_fwd(xd, wt, y, n, h, w, c, s)
    ref = K32.dwconv_fwd(x, wgt, s, 1)
    assert rel(nhwc_to_nchw(y), ref) <= B16_TOL
    dy = bf16_round(rng.standard_normal(ref.shape).astype(np.float32))
    dyd = to_dev_nhwc_b16(dy)
    dx = t.empty((n, h, w, c), dtype=t.bfloat16, device="cuda:0")
    K.fdgk_dwconv3_dgrad(dyd, wt, dx, n, h, w, c, s)
    assert rel(nhwc_to_nchw(dx), K32.dwconv_bwd_data(dy, wgt, x.shape, s, 1)) <= B16_TOL
    nb = K.fdgk_dwconv3_wgrad_scratch_bytes(n, h, w, c, s)
    assert nb > 0
    dws = []
    for _ in range(2):
        scratch = t.full((nb // 4,), 5.0, dtype=t.float32, device="cuda:0")
        dw = t.full((c, 9), 5.0, dtype=t.float32, device="cuda:0")
        K.fdgk_dwconv3_wgrad(xd, dyd, dw, scratch, n, h, w, c, s)
        dws.append(dw.cpu().numpy())
    assert rel(dws[0].reshape(c, 1, 3, 3), K32.dwconv_bwd_weight(x, dy, 3, s, 1)) <= F32_TOL
    assert np.array_equal(dws[0], dws[1])                  # fixed-order sums: the same bits every time

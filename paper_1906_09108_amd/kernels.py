"""Marshalling for the per-kernel C entry points of include/fdg_kernels.h (same names).  Arguments are
torch CUDA tensors (bf16 tensors for the *_b16 buffers) or None; nothing is computed here."""
from __future__ import annotations

import ctypes

from .binding import _ptr, _stream_handle, load

KERNEL_EXPORTS = ["fdgk_conv_fwd", "fdgk_conv_fwd_bn_applies", "fdgk_conv_fwd_bn", "fdgk_conv_dgrad_bn_applies", "fdgk_conv_dgrad_bn", "fdgk_conv_dgrad", "fdgk_conv_dgrad_gated", "fdgk_conv_dgrad_feeding_next", "fdgk_conv_dgrad_gates", "fdgk_conv_dgrad_pair_applies", "fdgk_conv_dgrad_gated_pair", "fdgk_bn_bwd_gated", "fdgk_conv_wgrad", "fdgk_conv_wgrad_scratch_bytes", "fdgk_bn_stats", "fdgk_bn_apply",
                  "fdgk_bn_bwd", "fdgk_sgd", "fdgk_bn_bwd_static", "fdgk_bn_bwd_static_max_c", "fdgk_sums_bytes", "fdgk_sums_read",
                  "fdgk_avgpool", "fdgk_fc_fwd", "fdgk_softmax_ce", "fdgk_fc_bwd", "fdgk_pool_bwd", "fdgk_nchw_to_nhwc", "fdgk_nhwc_to_nchw",
                  "fdgk_im2col7", "fdgk_maxpool3s2", "fdgk_maxpool3s2_bwd", "fdgk_dwconv3_fwd", "fdgk_dwconv3_dgrad",
                  "fdgk_dwconv3_wgrad_scratch_bytes", "fdgk_dwconv3_wgrad"]
_ready = False


def _lib():
    global _ready
    lib = load()
    if not _ready:
        vp, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        lib.fdgk_conv_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        lib.fdgk_conv_dgrad.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        lib.fdgk_conv_fwd_bn_applies.argtypes = [i, i, i, i, i, i]
        lib.fdgk_conv_dgrad_bn_applies.argtypes = [i, i, i, i, i, i]
        lib.fdgk_conv_dgrad_bn.argtypes = [vp, i, vp, vp, vp, vp, f, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp]
        lib.fdgk_conv_fwd_bn.argtypes = [vp, vp, vp, vp, f, vp, vp, vp, vp, vp, f, vp, vp, vp, i, i, i, i, i, vp]
        lib.fdgk_conv_dgrad_gated.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        lib.fdgk_conv_dgrad_feeding_next.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
        lib.fdgk_conv_dgrad_gates.argtypes = [i, i, i, i, i, i, i]
        lib.fdgk_conv_dgrad_pair_applies.argtypes = [i, i, i, i, i]
        lib.fdgk_conv_dgrad_gated_pair.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp]
        lib.fdgk_bn_bwd_gated.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, f, vp]
        lib.fdgk_conv_wgrad.argtypes = [vp, vp, vp, vp, sz, i, i, i, i, i, i, i, i, vp]
        lib.fdgk_conv_wgrad_scratch_bytes.argtypes = [i, i, i, i, i, i, i]
        lib.fdgk_bn_stats.argtypes = [vp, vp, i, i, vp]
        lib.fdgk_bn_apply.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, f, i, vp]
        lib.fdgk_bn_bwd.argtypes = [vp, i, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, f, vp]
        lib.fdgk_sgd.argtypes = [vp, vp, vp, sz, f, f, f, vp]
        lib.fdgk_bn_bwd_static.argtypes = [vp, i, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, f, vp]
        lib.fdgk_bn_bwd_static_max_c.argtypes = []
        lib.fdgk_sums_bytes.argtypes = [i]
        lib.fdgk_sums_read.argtypes = [vp, i, vp, vp]
        lib.fdgk_avgpool.argtypes = [vp, vp, i, i, i, vp]
        lib.fdgk_fc_fwd.argtypes = [vp, vp, vp, vp, i, i, i, vp]
        lib.fdgk_softmax_ce.argtypes = [vp, vp, vp, vp, i, i, vp]
        lib.fdgk_fc_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, vp]
        lib.fdgk_pool_bwd.argtypes = [vp, vp, vp, i, i, i, vp]
        lib.fdgk_nchw_to_nhwc.argtypes = [vp, vp, vp, i, i, i, i, f, vp]
        lib.fdgk_nhwc_to_nchw.argtypes = [vp, vp, i, i, i, i, vp]
        lib.fdgk_im2col7.argtypes = [vp, vp, i, i, i, vp]
        lib.fdgk_maxpool3s2.argtypes = [vp, vp, vp, i, i, i, i, vp]
        lib.fdgk_maxpool3s2_bwd.argtypes = [vp, vp, vp, i, i, i, i, vp]
        lib.fdgk_dwconv3_fwd.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        lib.fdgk_dwconv3_dgrad.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        lib.fdgk_dwconv3_wgrad_scratch_bytes.argtypes = [i, i, i, i, i]
        lib.fdgk_dwconv3_wgrad.argtypes = [vp, vp, vp, vp, sz, i, i, i, i, i, vp]
        for n in KERNEL_EXPORTS:
            if getattr(lib, n).argtypes is None:   # a pointer passed without a declared type would be cut to 32 bits
                raise RuntimeError(f"{n}: argument types not declared")
            getattr(lib, n).restype = i
        lib.fdgk_conv_wgrad_scratch_bytes.restype = sz
        lib.fdgk_sums_bytes.restype = sz
        lib.fdgk_dwconv3_wgrad_scratch_bytes.restype = sz
        _ready = True
    return lib


def _ok(rc: int, name: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{name} failed with hipError_t {rc}")


def fdgk_sums_bytes(c: int) -> int:
    return int(_lib().fdgk_sums_bytes(int(c)))


def new_sums(c: int, device="cuda:0"):
    """A zeroed sums array for c channels (torch owns the memory; the format is the library's)."""
    import torch
    return torch.zeros(fdgk_sums_bytes(c) // 8, dtype=torch.int64, device=device)


def fdgk_sums_read(sums, c: int, stream=None):
    """Totals of a sums array as a host float64 array [2c]: first sums, then second sums."""
    import numpy as np
    out = np.empty(2 * c, np.float64)
    _ok(_lib().fdgk_sums_read(_ptr(sums), int(c), out.ctypes.data, _stream_handle(stream)), "fdgk_sums_read")
    return out


def fdgk_conv_fwd(x_b16, w_b16, addend_f32, y_f32, y_b16, stats_f32, n, h, w, ci, co, ksize, stride, stream=None):
    _ok(_lib().fdgk_conv_fwd(_ptr(x_b16), _ptr(w_b16), _ptr(addend_f32), _ptr(y_f32), _ptr(y_b16), _ptr(stats_f32),
                             n, h, w, ci, co, ksize, stride, _stream_handle(stream)), "fdgk_conv_fwd")


def fdgk_conv_fwd_bn_applies(n, h, w, ci, co, with_residual=False) -> bool:
    return bool(_lib().fdgk_conv_fwd_bn_applies(n, h, w, ci, co, 1 if with_residual else 0))


def fdgk_conv_fwd_bn(x_raw_b16, x_sums, gamma, beta, eps, res_f32, act_b16, act_f32, run_mean, run_var, momentum, w_b16, y_b16,
                     stats_sums, n, h, w, ci, co, stream=None):
    _ok(_lib().fdgk_conv_fwd_bn(_ptr(x_raw_b16), _ptr(x_sums), _ptr(gamma), _ptr(beta), eps, _ptr(res_f32), _ptr(act_b16),
                                _ptr(act_f32), _ptr(run_mean), _ptr(run_var), momentum, _ptr(w_b16), _ptr(y_b16), _ptr(stats_sums),
                                n, h, w, ci, co, _stream_handle(stream)), "fdgk_conv_fwd_bn")


def fdgk_conv_dgrad_bn_applies(n, h, w, ci, co, g_is_f32) -> bool:
    return bool(_lib().fdgk_conv_dgrad_bn_applies(n, h, w, ci, co, 1 if g_is_f32 else 0))


def fdgk_conv_dgrad_bn(g, g_is_f32, x_b16, x_sums, gsums, gamma, eps, dy_b16, dgamma, dbeta, wt_b16, addend_f32, addmask_b16, dx_f32,
                       dx_b16, n, h, w, ci, co, stream=None):
    _ok(_lib().fdgk_conv_dgrad_bn(_ptr(g), 1 if g_is_f32 else 0, _ptr(x_b16), _ptr(x_sums), _ptr(gsums), _ptr(gamma), eps,
                                  _ptr(dy_b16), _ptr(dgamma), _ptr(dbeta), _ptr(wt_b16), _ptr(addend_f32), _ptr(addmask_b16),
                                  _ptr(dx_f32), _ptr(dx_b16), n, h, w, ci, co, _stream_handle(stream)), "fdgk_conv_dgrad_bn")


def fdgk_conv_dgrad(dy_b16, wt_b16, addend_f32, addmask_b16, dx_f32, dx_b16, n, h, w, ci, co, ksize, stride, stream=None):
    _ok(_lib().fdgk_conv_dgrad(_ptr(dy_b16), _ptr(wt_b16), _ptr(addend_f32), _ptr(addmask_b16), _ptr(dx_f32),
                               _ptr(dx_b16), n, h, w, ci, co, ksize, stride, _stream_handle(stream)), "fdgk_conv_dgrad")


def fdgk_conv_dgrad_gates(n, h, w, ci, co, ksize, stride) -> bool:
    return bool(_lib().fdgk_conv_dgrad_gates(n, h, w, ci, co, ksize, stride))


def fdgk_conv_dgrad_gated(dy_b16, wt_b16, addend_f32, gate_b16, bnx_b16, gsums_f32, dx_f32, dx_b16, n, h, w, ci, co, ksize,
                          stride, stream=None):
    _ok(_lib().fdgk_conv_dgrad_gated(_ptr(dy_b16), _ptr(wt_b16), _ptr(addend_f32), _ptr(gate_b16), _ptr(bnx_b16),
                                     _ptr(gsums_f32), _ptr(dx_f32), _ptr(dx_b16), n, h, w, ci, co, ksize, stride,
                                     _stream_handle(stream)), "fdgk_conv_dgrad_gated")


def fdgk_conv_dgrad_pair_applies(n, h, w, ci, co) -> bool:
    return bool(_lib().fdgk_conv_dgrad_pair_applies(n, h, w, ci, co))


def fdgk_conv_dgrad_gated_pair(dy_b16, wt_b16, dy2_b16, wt2_b16, gate_b16, bnx_b16, gsums_f32, dx_f32, dx_b16, n, h, w, ci, co,
                               stream=None):
    _ok(_lib().fdgk_conv_dgrad_gated_pair(_ptr(dy_b16), _ptr(wt_b16), _ptr(dy2_b16), _ptr(wt2_b16), _ptr(gate_b16), _ptr(bnx_b16),
                                          _ptr(gsums_f32), _ptr(dx_f32), _ptr(dx_b16), n, h, w, ci, co, _stream_handle(stream)),
        "fdgk_conv_dgrad_gated_pair")


def fdgk_conv_dgrad_feeding_next(dy_b16, wt_b16, addend_f32, addmask_b16, gate_b16, bnx_b16, gsums_f32, dx_f32, dx_b16, n, h, w,
                                 ci, co, ksize, stride, stream=None):
    _ok(_lib().fdgk_conv_dgrad_feeding_next(_ptr(dy_b16), _ptr(wt_b16), _ptr(addend_f32), _ptr(addmask_b16), _ptr(gate_b16),
                                            _ptr(bnx_b16), _ptr(gsums_f32), _ptr(dx_f32), _ptr(dx_b16), n, h, w, ci, co, ksize,
                                            stride, _stream_handle(stream)), "fdgk_conv_dgrad_feeding_next")


def fdgk_bn_bwd_gated(g_b16, x_b16, sums_f32, gamma, gsums_f32, addend_f32, dx_f32, dx_b16, dgamma, dbeta, m, c, eps,
                      stream=None):
    _ok(_lib().fdgk_bn_bwd_gated(_ptr(g_b16), _ptr(x_b16), _ptr(sums_f32), _ptr(gamma), _ptr(gsums_f32), _ptr(addend_f32),
                                 _ptr(dx_f32), _ptr(dx_b16), _ptr(dgamma), _ptr(dbeta), m, c, eps, _stream_handle(stream)),
        "fdgk_bn_bwd_gated")


def fdgk_conv_wgrad_scratch_bytes(n, h, w, ci, co, ksize, stride) -> int:
    return int(_lib().fdgk_conv_wgrad_scratch_bytes(n, h, w, ci, co, ksize, stride))


def fdgk_conv_wgrad(x_b16, dy_b16, dw_f32, scratch_f32, n, h, w, ci, co, ksize, stride, overwrite=False, stream=None):
    """scratch_f32: a float32 CUDA tensor (any contents) or None.  overwrite: write dw instead of adding to it."""
    nbytes = 0 if scratch_f32 is None else scratch_f32.numel() * scratch_f32.element_size()
    _ok(_lib().fdgk_conv_wgrad(_ptr(x_b16), _ptr(dy_b16), _ptr(dw_f32), _ptr(scratch_f32), nbytes, int(bool(overwrite)),
                               n, h, w, ci, co,
                               ksize, stride, _stream_handle(stream)), "fdgk_conv_wgrad")


def fdgk_bn_stats(x_b16, sums_f32, m, c, stream=None):
    _ok(_lib().fdgk_bn_stats(_ptr(x_b16), _ptr(sums_f32), m, c, _stream_handle(stream)), "fdgk_bn_stats")


def fdgk_bn_apply(x_b16, sums_f32, gamma, beta, res_f32, y_f32, y_b16, m, c, eps, relu, stream=None):
    _ok(_lib().fdgk_bn_apply(_ptr(x_b16), _ptr(sums_f32), _ptr(gamma), _ptr(beta), _ptr(res_f32), _ptr(y_f32),
                             _ptr(y_b16), m, c, eps, int(relu), _stream_handle(stream)), "fdgk_bn_apply")


def fdgk_bn_bwd(dy, dy_is_f32, mask_b16, x_b16, sums_f32, gamma, scratch_f32, addend_f32, dx_f32, dx_b16, dgamma,
                dbeta, m, c, eps, stream=None):
    _ok(_lib().fdgk_bn_bwd(_ptr(dy), int(dy_is_f32), _ptr(mask_b16), _ptr(x_b16), _ptr(sums_f32), _ptr(gamma),
                           _ptr(scratch_f32), _ptr(addend_f32), _ptr(dx_f32), _ptr(dx_b16), _ptr(dgamma), _ptr(dbeta),
                           m, c, eps, _stream_handle(stream)), "fdgk_bn_bwd")


def fdgk_bn_bwd_static_max_c() -> int:
    return int(_lib().fdgk_bn_bwd_static_max_c())


def fdgk_bn_bwd_static(dy, dy_is_f32, mask_b16, x_b16, sums_f32, gamma, addend_f32, dx_f32, dx_b16, dgamma, dbeta, m, c, eps,
                       stream=None, check=True) -> int:
    """fdgk_bn_bwd without a scratch argument: the sums live in the library's own per-GPU array."""
    rc = int(_lib().fdgk_bn_bwd_static(_ptr(dy), int(dy_is_f32), _ptr(mask_b16), _ptr(x_b16), _ptr(sums_f32), _ptr(gamma),
                                       _ptr(addend_f32), _ptr(dx_f32), _ptr(dx_b16), _ptr(dgamma), _ptr(dbeta), m, c, eps,
                                       _stream_handle(stream)))
    if check:
        _ok(rc, "fdgk_bn_bwd_static")
    return rc


def fdgk_sgd(theta, v, g, count, lr, mu, wd, stream=None):
    _ok(_lib().fdgk_sgd(_ptr(theta), _ptr(v), _ptr(g), count, lr, mu, wd, _stream_handle(stream)), "fdgk_sgd")


def fdgk_avgpool(o_b16, pooled, n, hw, c, stream=None, check=True):
    rc = int(_lib().fdgk_avgpool(_ptr(o_b16), _ptr(pooled), n, hw, c, _stream_handle(stream)))
    if check:
        _ok(rc, "fdgk_avgpool")
    return rc


def fdgk_fc_fwd(pooled, w, b, logits, n, c, j, stream=None):
    _ok(_lib().fdgk_fc_fwd(_ptr(pooled), _ptr(w), _ptr(b), _ptr(logits), n, c, j, _stream_handle(stream)), "fdgk_fc_fwd")


def fdgk_softmax_ce(logits, labels, y, dlogits, n, j, stream=None):
    _ok(_lib().fdgk_softmax_ce(_ptr(logits), _ptr(labels), _ptr(y), _ptr(dlogits), n, j, _stream_handle(stream)), "fdgk_softmax_ce")


def fdgk_fc_bwd(pooled, w, dlogits, dw, db, dpooled, n, c, j, stream=None):
    _ok(_lib().fdgk_fc_bwd(_ptr(pooled), _ptr(w), _ptr(dlogits), _ptr(dw), _ptr(db), _ptr(dpooled), n, c, j,
                           _stream_handle(stream)), "fdgk_fc_bwd")


def fdgk_pool_bwd(dpooled, g_f32, g_b16, n, hw, c, stream=None):
    _ok(_lib().fdgk_pool_bwd(_ptr(dpooled), _ptr(g_f32), _ptr(g_b16), n, hw, c, _stream_handle(stream)), "fdgk_pool_bwd")


def fdgk_nchw_to_nhwc(src, dst_f32, dst_b16, n, c, hw, cp, scale=1.0, stream=None, check=True):
    rc = int(_lib().fdgk_nchw_to_nhwc(_ptr(src), _ptr(dst_f32), _ptr(dst_b16), n, c, hw, cp, scale, _stream_handle(stream)))
    if check:
        _ok(rc, "fdgk_nchw_to_nhwc")
    return rc


def fdgk_nhwc_to_nchw(src, dst, n, c, hw, cp, stream=None):
    _ok(_lib().fdgk_nhwc_to_nchw(_ptr(src), _ptr(dst), n, c, hw, cp, _stream_handle(stream)), "fdgk_nhwc_to_nchw")


def fdgk_im2col7(x8_b16, col_b16, n, h, w, stream=None):
    _ok(_lib().fdgk_im2col7(_ptr(x8_b16), _ptr(col_b16), n, h, w, _stream_handle(stream)), "fdgk_im2col7")


def fdgk_maxpool3s2(x_b16, y_f32, y_b16, n, h, w, c, stream=None):
    _ok(_lib().fdgk_maxpool3s2(_ptr(x_b16), _ptr(y_f32), _ptr(y_b16), n, h, w, c, _stream_handle(stream)), "fdgk_maxpool3s2")


def fdgk_maxpool3s2_bwd(x_b16, dy_f32, dx_f32, n, h, w, c, stream=None):
    _ok(_lib().fdgk_maxpool3s2_bwd(_ptr(x_b16), _ptr(dy_f32), _ptr(dx_f32), n, h, w, c, _stream_handle(stream)), "fdgk_maxpool3s2_bwd")


def fdgk_dwconv3_fwd(x_b16, wt_b16, y_b16, n, h, w, c, stride, stream=None):
    _ok(_lib().fdgk_dwconv3_fwd(_ptr(x_b16), _ptr(wt_b16), _ptr(y_b16), n, h, w, c, stride, _stream_handle(stream)), "fdgk_dwconv3_fwd")


def fdgk_dwconv3_dgrad(dy_b16, wt_b16, dx_b16, n, h, w, c, stride, stream=None):
    _ok(_lib().fdgk_dwconv3_dgrad(_ptr(dy_b16), _ptr(wt_b16), _ptr(dx_b16), n, h, w, c, stride, _stream_handle(stream)),
        "fdgk_dwconv3_dgrad")


def fdgk_dwconv3_wgrad_scratch_bytes(n, h, w, c, stride) -> int:
    return int(_lib().fdgk_dwconv3_wgrad_scratch_bytes(n, h, w, c, stride))


def fdgk_dwconv3_wgrad(x_b16, dy_b16, dw_f32, scratch_f32, n, h, w, c, stride, stream=None):
    nbytes = 0 if scratch_f32 is None else scratch_f32.numel() * scratch_f32.element_size()
    _ok(_lib().fdgk_dwconv3_wgrad(_ptr(x_b16), _ptr(dy_b16), _ptr(dw_f32), _ptr(scratch_f32), nbytes, n, h, w, c, stride,
                                  _stream_handle(stream)), "fdgk_dwconv3_wgrad")

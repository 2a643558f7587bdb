"""The entry point for callers that cannot allocate device memory (fdgk_bn_bwd_static: the sums of the batch-norm
backward in the library's own per-GPU array) against the entry point it is a variant of (fdgk_bn_bwd, scratch given
by the caller), through the C ABI: two calls in a row, the second on a smaller input, so that what the first call
left in the array would show.  Both run the same kernels and the sums are exact (integer) totals of the same
workgroup partial sums, so the two entry points agree bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

F32_TOL = 2e-4
B16_TOL = 2.0 ** -8


def rel(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    d = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (d if d > 0 else 1.0))


def _case(t, K, m, c, seed, dy_is_f32):
    g = t.Generator(device="cpu").manual_seed(seed)
    x = (t.randn((m, c), generator=g) * 1.5 + 0.3).to(t.bfloat16).cuda()
    mask = t.randn((m, c), generator=g).to(t.bfloat16).cuda()
    dy = t.randn((m, c), generator=g)
    dy = dy.cuda() if dy_is_f32 else dy.to(t.bfloat16).cuda()
    gamma = (1 + 0.2 * t.randn(c, generator=g)).cuda()
    addend = t.randn((m, c), generator=g).cuda()
    sums = K.new_sums(c)
    K.fdgk_bn_stats(x, sums, m, c)
    return x, mask, dy, gamma, addend, sums


def _outputs(t, m, c):
    return (t.full((m, c), float("nan"), dtype=t.float32, device="cuda"), t.zeros((m, c), dtype=t.bfloat16, device="cuda"),
            t.full((c,), float("nan"), dtype=t.float32, device="cuda"), t.full((c,), float("nan"), dtype=t.float32, device="cuda"))


def test_two_calls_in_a_row_match_the_entry_point_with_caller_scratch():
    import torch as t
    from paper_1906_09108_amd import kernels as K
    eps = 1e-5
    assert K.fdgk_bn_bwd_static_max_c() == 2048
    # the second call is smaller in rows and in channels: stale sums of the first would land in its channels
    for i, (m, c, dy_is_f32) in enumerate([(4 * 33 * 31, 320, True), (2 * 9 * 7, 48, False)]):
        print("no-alloc bn backward", m, c, dy_is_f32, flush=True)
        x, mask, dy, gamma, addend, sums = _case(t, K, m, c, 100 + i, dy_is_f32)
        dx32, dx16, dg, db = _outputs(t, m, c)
        K.fdgk_bn_bwd_static(dy, dy_is_f32, mask, x, sums, gamma, addend, dx32, dx16, dg, db, m, c, eps)
        r32, r16, rg, rb = _outputs(t, m, c)
        scratch = K.new_sums(c)
        K.fdgk_bn_bwd(dy, dy_is_f32, mask, x, sums, gamma, scratch, addend, r32, r16, rg, rb, m, c, eps)
        t.cuda.synchronize()
        assert bool(t.isfinite(dx32).all())
        assert t.equal(dx32, r32) and t.equal(dx16, r16) and t.equal(dg, rg) and t.equal(db, rb)


def test_sizes_beyond_the_array_are_refused():
    import torch as t
    from paper_1906_09108_amd import kernels as K
    m, c = 16, 2048 + 8
    z32 = t.zeros((m, c), dtype=t.float32, device="cuda")
    z16 = t.zeros((m, c), dtype=t.bfloat16, device="cuda")
    v = t.zeros(2 * c, dtype=t.float32, device="cuda")
    out = t.full((m, c), 7.0, dtype=t.float32, device="cuda")
    rc = K.fdgk_bn_bwd_static(z32, True, z16, z16, K.new_sums(c), v, None, out, None, v[:c], v[c:], m, c, 1e-5, check=False)
    t.cuda.synchronize()
    assert rc == 1                      # hipErrorInvalidValue, nothing enqueued
    assert bool((out == 7.0).all())

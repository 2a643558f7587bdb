"""K modules on one GPU run as Algorithm I (include/fdg_chain.h) against the K-module oracle
(oracle.fdg_oracle.OracleChain) on the same seeded batches.

Three runs advance in lock step, as in tests/gpu_harness.py: the HIP chain, the oracle with bf16 storage
("same": ReLU decisions taken in the kernel's precision) and the oracle's fp32 definition ("plain").
  * which batch every module forwards and back-propagates, and every module's queue state: exact;
  * the first loss and logits (no weight has moved yet) and the last module's first gradient: the 2e-2 bar
    (max|err| / max|ref| per tensor; relative L2 for the gradient);
  * everything later -- losses, every module's gradients at every iteration, the final weights: the envelope
    relL2(gpu, same) <= 2e-2 + 2 relL2(same, plain), since after the first update the two bf16 evaluations
    round their weights independently;
  * Eq. 16 / Eq. 17 on the device: with frozen weights the gradient of module k under beta is beta^(K-k) times
    the gradient under beta = 1 (up to what the unfixed order of atomic sums can move: see that test);
  * the loss goes down on separable data.
"""
import numpy as np
import pytest

import fdg_workloads as W
from tests.gpu_harness import ENVELOPE_FACTOR, TOL, Record, format_report, rel_err, rel_l2

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def FdgChain_workspace(spec):
    from paper_1906_09108_amd import binding
    return binding.fdg_module_workspace_bytes(spec)


def _set_params(chain, specs, seed=0):
    thetas = [W.make_params(sp, seed + 17 * k, perturb_bn=True) for k, sp in enumerate(specs)]
    mods = chain.modules if hasattr(chain, "modules") else chain.mods
    for m, th in zip(mods, thetas):
        m.set_params(th)
    return thetas


@pytest.mark.parametrize("K,save_mode", [(1, 0), (2, 0), (3, 0), (3, 1)])
def test_chain_against_the_oracle(K, save_mode):
    """save_mode 1: every module keeps a saved forward as input + weight snapshot and replays it (include/fdg.h); the
    lower modules hold 2(K-1-k) of them, which is where that form saves memory."""
    t = _torch()
    from oracle.fdg_oracle import OracleChain
    from paper_1906_09108_amd import FdgChain
    print("chain parity K =", K, "save mode", save_mode, flush=True)
    specs = W.chain_specs(K, n=16, width=16, hw=8, blocks=1, beta=0.5)
    gpu = FdgChain(specs, save_mode=save_mode)
    if save_mode:
        assert sum(m.workspace_bytes for m in gpu.modules) < sum(
            FdgChain_workspace(sp) for sp in specs)
    same, plain = OracleChain(specs, np.float32, storage="bf16"), OracleChain(specs, np.float32, storage="fp32")
    for ch in (gpu, same, plain):
        _set_params(ch, specs)
    records, exact, strict_bad = [], [], []

    def note(label, step, got, a, b, strict=False):
        # end-to-end bar of the chain: the distance between the oracle's two storage precisions (the layers of its
        # modules are covered one by one in tests/test_gpu_layerwise.py)
        r = Record(label, step, rel_err(got, a), rel_l2(got, a), rel_l2(a, b), floor=rel_l2(a, b))
        records.append(r)
        # gradients of these small layers: one ReLU gate decided the other way (an activation within rounding of
        # zero) is several per cent of single elements, so their bar is taken in relative L2
        worst = r.l2 if label.startswith("grads") else r.strict
        if strict and worst > TOL:
            strict_bad.append(f"{label} at iteration {step}: {worst:.3e}")

    T = 2 * K + 3
    lr = 0.05
    for it in range(1, T + 1):
        x, labels = W.make_separable_batch(specs[0], it)
        ra, rb = same.step(x, labels, lr), plain.step(x, labels, lr)
        b = gpu.step(t.from_numpy(x).cuda(), t.from_numpy(labels).cuda(), lr)
        t.cuda.synchronize()
        tt, fwd, bwd = gpu.state()
        if (tt, fwd, bwd) != (it, same.fwd_batch, same.bwd_batch):
            exact.append(f"iteration {it}: gpu {(tt, fwd, bwd)} oracle {(it, same.fwd_batch, same.bwd_batch)}")
        for k in range(K):
            if fwd[k] != max(0, it - k) or bwd[k] != max(0, it - 2 * K + k + 2):     # Section III-A, k from 0
                exact.append(f"iteration {it} module {k}: batches {fwd[k]}, {bwd[k]}")
            if gpu.modules[k].queue_state() != same.mods[k].queue_state():
                exact.append(f"iteration {it} module {k}: queue {gpu.modules[k].queue_state()} {same.mods[k].queue_state()}")
        if (b != 0) != (ra is not None) or (ra is not None and b != ra[0]):
            exact.append(f"iteration {it}: top batch {b} vs {ra and ra[0]}")
        if ra is not None:
            y = gpu.top_y.cpu().numpy()
            first = it == K
            note("loss", it, y[:1], np.array([ra[1]]), np.array([rb[1]]), strict=first)
            note("logits", it, y[1:], ra[2].reshape(-1), rb[2].reshape(-1), strict=first)
        for k in range(K):
            if bwd[k]:
                note(f"grads[{k}]", it, gpu.modules[k].get_grads(), same.mods[k].get_grads(), plain.mods[k].get_grads(),
                     strict=(k == K - 1 and it == K))
    for k in range(K):
        note(f"theta[{k}]", T, gpu.modules[k].get_params(), same.mods[k].get_params(), plain.mods[k].get_params())
    gpu.close()
    print(format_report(records, 12), flush=True)
    assert not exact, exact
    assert not strict_bad, strict_bad
    bad = [f"{r.label}@{r.step}: L2 {r.l2:.3e} > {TOL} + {ENVELOPE_FACTOR} * {r.inherent:.3e}" for r in records
           if not r.envelope_ok]
    assert not bad, bad
    assert all(r.informative for r in records), "the test network is shallow enough for every comparison to count"


def test_chain_compounds_the_shrinking_factor():
    """Eq. 16 / Eq. 17 on the device, weights frozen (lr = 0): g_hat(module k; beta) = beta^(K-1-k) g_hat(module k; 1),
    k counted from 0.  beta = 0.5 scales every intermediate of the backward by a power of two; every operation of the
    backward is linear in the gradient, powers of two commute with every rounding, and the sums over workgroups are exact
    integers (order independent), so the relation holds BIT FOR BIT."""
    t = _torch()
    from paper_1906_09108_amd import FdgChain
    K = 3
    runs = {}
    for beta in (1.0, 0.5):
        specs = W.chain_specs(K, n=16, width=16, hw=8, blocks=1, beta=beta)
        ch = FdgChain(specs)
        _set_params(ch, specs)
        got = {}
        for it in range(1, 2 * K + 1):
            x, labels = W.make_separable_batch(specs[0], it)
            ch.step(t.from_numpy(x).cuda(), t.from_numpy(labels).cuda(), 0.0)
            t.cuda.synchronize()
            _, _, bwd = ch.state()
            for k in range(K):
                if bwd[k] == 1:
                    got[k] = ch.modules[k].get_grads()
        ch.close()
        assert sorted(got) == list(range(K))
        runs[beta] = got
    for k in range(K):
        ref = runs[1.0][k] * 0.5 ** (K - 1 - k)
        assert np.abs(ref).max() > 0
        assert np.array_equal(runs[0.5][k], ref), (k, rel_err(runs[0.5][k], ref), rel_l2(runs[0.5][k], ref))
        if k < K - 1:   # and the factor is there at all
            assert rel_l2(runs[0.5][k], runs[1.0][k]) > 0.4


def test_chain_learns_separable_data():
    t = _torch()
    from paper_1906_09108_amd import FdgChain
    specs = W.chain_specs(3, n=32, width=16, hw=8, blocks=1, beta=0.5, num_classes=4)
    ch = FdgChain(specs)
    for k, m in enumerate(ch.modules):
        m.set_params(W.make_params(specs[k], k))
    losses = []
    for it in range(1, 61):
        x, labels = W.make_separable_batch(specs[0], it, noise=0.3)
        b = ch.step(t.from_numpy(x).cuda(), t.from_numpy(labels).cuda(), 0.05)
        if b:
            losses.append(float(ch.top_y[0].item()))
    ch.close()
    print("first losses", np.round(losses[:5], 3), "last", np.round(losses[-5:], 3), flush=True)
    assert np.isfinite(losses).all()
    assert np.mean(losses[-5:]) < 0.5 * np.mean(losses[:5])


def test_chain_create_checks_its_modules():
    t = _torch()
    import ctypes
    from paper_1906_09108_amd import FdgModule, binding
    lib = binding.load()
    specs = W.chain_specs(2, n=16, width=16, hw=8, blocks=1)
    a, b = FdgModule(specs[0]), FdgModule(specs[1])
    out = ctypes.c_void_p()
    # wrong order: the top module first
    arr = (ctypes.c_void_p * 2)(b.handle, a.handle)
    assert lib.fdg_chain_mailbox_bytes(arr, 2) == 0
    assert lib.fdg_chain_create(arr, 2, None, 0, ctypes.byref(out)) == binding.FDG_ERR_INVALID_ARG
    # a lower module that cannot hold 2(K-1-k) waiting forwards
    shallow = W.chain_specs(2, n=16, width=16, hw=8, blocks=1)[0]
    shallow.delay = 1
    c = FdgModule(shallow)
    arr = (ctypes.c_void_p * 2)(c.handle, b.handle)
    assert lib.fdg_chain_mailbox_bytes(arr, 2) == 0
    # a good pair, but too little mailbox memory
    arr = (ctypes.c_void_p * 2)(a.handle, b.handle)
    need = lib.fdg_chain_mailbox_bytes(arr, 2)
    assert need > 0 and need % 256 == 0
    buf = t.empty(need, dtype=t.uint8, device="cuda")
    assert lib.fdg_chain_create(arr, 2, buf.data_ptr(), need - 256, ctypes.byref(out)) == binding.FDG_ERR_WORKSPACE_TOO_SMALL
    for m in (a, b, c):
        m.close()

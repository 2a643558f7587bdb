"""FDG_SAVE_ACTIVATIONS_CURRENT_WEIGHTS on the GPU (include/fdg.h): the ablation in which a saved forward keeps no weight
snapshot and the delayed backward reads the module's one copy of the weights as it is when it runs.  The oracle's
weights="current" mode (pinned on the CPU against autograd on a saved graph, tests/test_oracle_ablation.py) is the
reference; the method's own mode must NOT fit the same numbers, which each case checks on the oracle's side."""
import copy

import numpy as np
import pytest

import fdg_workloads as W
from tests.gpu_harness import TOL, format_report, judge, rel_err, rel_l2, run_side_by_side
from tests.test_gpu_parity import ENVELOPE, STRICT

pytestmark = pytest.mark.gpu

CURRENT = 2


@pytest.mark.parametrize("name", ["postact_identity_delay1", "preact_project", "stem_d1", "head_d1"])
def test_backward_reads_the_weights_of_the_moment(name):
    """forward(batch 0) at theta0; the parameters are then SET to a distant theta1; forward(batch 1); the delayed backward of
    batch 0 must use batch 0's activations and statistics with theta1's convolution weights, scales and classifier."""
    import torch as t
    from oracle.fdg_oracle import OracleModule
    from paper_1906_09108_amd import FdgModule
    if name == "stem_d1":
        spec = copy.deepcopy(STRICT["stem_with_grad_in"])
    elif name == "head_d1":
        spec = copy.deepcopy(STRICT["head_postact"])
    else:
        spec = copy.deepcopy({**STRICT, **ENVELOPE}[name])
    spec.delay = 1
    print("current-weights case", name, flush=True)
    dev = t.device("cuda:0")
    seed = 6
    theta0 = W.make_params(spec, seed, perturb_bn=True)
    theta1 = (theta0 + np.float32(0.3) * W.make_params(spec, seed + 1, perturb_bn=True)).astype(np.float32)
    xs = [W.make_input(spec, i, seed) for i in range(2)]
    labs = [W.make_labels(spec, i, seed) for i in range(2)]
    g0 = W.make_grad_out(spec, 0, seed)

    def oracle(weights):
        m = OracleModule(spec, np.float32, storage="bf16", weights=weights)
        m.set_params(theta0)
        m.forward(xs[0], labs[0])
        v = m.get_momentum()
        m.set_params(theta1)
        m.v[...] = v
        m.forward(xs[1], labs[1])
        gin = m.backward_delayed(g0)
        return m.get_grads(), gin
    ref_g, ref_in = oracle("current")
    oth_g, oth_in = oracle("snapshot")

    gpu = FdgModule(spec, dev, save_mode=CURRENT)
    gpu.set_params(theta0)
    gpu.forward(t.from_numpy(xs[0]).to(dev), None if labs[0] is None else t.from_numpy(labs[0]).to(dev))
    gpu.set_params(theta1)
    gpu.forward(t.from_numpy(xs[1]).to(dev), None if labs[1] is None else t.from_numpy(labs[1]).to(dev))
    gin = None if spec.is_bottom else t.empty(spec.input_shape(), dtype=t.float32, device=dev)
    gpu.backward_delayed(None if g0 is None else t.from_numpy(g0).to(dev), gin)
    got = gpu.get_grads()
    gpu.close()
    off = 0
    worst = 0.0
    for pname, shape, _ in W.param_shapes(spec):
        n = int(np.prod(shape))
        a, b = got[off:off + n], ref_g[off:off + n]
        off += n
        e = rel_err(a, b)
        worst = max(worst, e)
        assert e <= TOL, (pname, e, rel_l2(a, b))
    if gin is not None:
        e = rel_err(gin.cpu().numpy(), ref_in)
        assert e <= TOL, ("grad_in", e)
        assert rel_l2(oth_in, ref_in) > 5 * TOL      # the method's own mode gives another input gradient ...
        assert rel_l2(gin.cpu().numpy(), oth_in) > 4 * TOL   # ... and the GPU did not compute that one
    else:
        assert rel_l2(oth_g, ref_g) > 5 * TOL
    print(f"  worst parameter gradient {worst:.2e}; snapshot-mode oracle is {rel_l2(oth_g, ref_g):.2e} away in L2", flush=True)


@pytest.mark.parametrize("name", ["postact_identity_delay1", "bottom_stack_delay2", "bottleneck_project_delay1"])
def test_ablation_steps_against_the_oracle(name):
    spec = copy.deepcopy({**STRICT, **ENVELOPE}[name])
    spec.name = name + " current weights"
    print("current-weights steps", name, flush=True)
    records, exact = run_side_by_side(spec, 3, save_mode=CURRENT, seed=1)
    print(format_report(records), flush=True)
    assert not exact, exact
    bad = judge(records, spec, strict=False)
    assert not bad, "\n".join(bad[:40])


def test_ablation_backward_first_order():
    spec = copy.deepcopy(ENVELOPE["bottom_stack_delay2"])
    spec.name = "current weights, backward first"
    records, exact = run_side_by_side(spec, 3, save_mode=CURRENT, seed=2, backward_first=True)
    print(format_report(records), flush=True)
    assert not exact, exact
    bad = judge(records, spec, strict=False)
    assert not bad, "\n".join(bad[:40])


@pytest.mark.parametrize("idx,n", [(1, 16), (4, 8)])
def test_without_delay_the_ablation_is_the_method_bit_for_bit(idx, n):
    import torch as t
    from paper_1906_09108_amd import FdgModule
    spec = W.config(idx, n=n)
    spec.delay = 0
    print(f"current-weights identity cfg{idx}", flush=True)
    dev = t.device("cuda:0")

    def run(mode):
        m = FdgModule(spec, dev, save_mode=mode)
        m.set_params(W.make_params(spec, 2, perturb_bn=True))
        gin = None if spec.is_bottom else t.empty(spec.input_shape(), dtype=t.float32, device=dev)
        out = []
        for it in range(3):
            x, lab = W.make_input(spec, it, 2), W.make_labels(spec, it, 2)
            out.append(m.forward(t.from_numpy(x).to(dev), None if lab is None else t.from_numpy(lab).to(dev)).cpu().numpy())
            g = W.make_grad_out(spec, it, 2)
            m.backward_delayed(None if g is None else t.from_numpy(g).to(dev), gin)
            out.append(m.get_grads())
            m.update(0.01)
            out.append(m.get_params())
        m.close()
        return out
    a, b = run(0), run(CURRENT)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))


def test_the_ablation_saves_the_weight_snapshots():
    from paper_1906_09108_amd.binding import fdg_module_workspace_bytes_ex
    spec = W.config(3, n=16)          # delay 3: four saved forwards
    stored, shared = fdg_module_workspace_bytes_ex(spec, 0), fdg_module_workspace_bytes_ex(spec, CURRENT)
    assert 0 < shared < stored
    # four snapshots of both bf16 layouts against one: at least 3 x 2 layouts x 2 bytes per convolution weight
    conv_weights = sum(int(np.prod(s)) for _, s, _ in W.param_shapes(spec) if len(s) == 4)
    assert stored - shared >= 3 * 2 * 2 * conv_weights

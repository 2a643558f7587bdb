"""Two runs of the same steps on the same inputs give the same BITS.

Every sum that is taken over many workgroups is order independent by construction: the batch-norm statistics and the
two sums of a batch-norm backward are 128-bit fixed-point totals added with integer atomics (include/fdg_kernels.h,
"sums arrays"), weight gradients whose pixel range is split store their parts and a second kernel adds them in a fixed
order, and inside a workgroup partial sums are combined in a fixed order.  So a module step is a function of its
inputs: no tolerance is needed to compare two runs, and a difference between two runs is a bug."""
import numpy as np
import pytest

import fdg_workloads as W
from fdg_workloads import Layer, ModuleSpec

pytestmark = pytest.mark.gpu

H = dict(momentum=0.9, weight_decay=5e-4, lr=0.1)
CASES = {
    "cfg1": lambda: W.config(1),
    "cfg2_n8": lambda: W.config(2, n=8),            # narrow stages and their stride-2 transitions (generic kernels)
    "cfg3_n16": lambda: W.config(3, n=16),          # narrow kernels, replicated sums, delay 3
    "cfg4_n8": lambda: W.config(4, n=8),            # wide kernels, gated data gradients, head
    "cfg7_n2": lambda: W.config(7, n=2),
    "cfg8_n25": lambda: W.config(8, n=25),          # bottleneck blocks, the feeding 1x1 data gradient
    "ragged": lambda: ModuleSpec(3, 24, 17, 15, [Layer(W.BASIC_PREACT, 24, 40, 1), Layer(W.BASIC_POSTACT, 40, 40, 2)],
                                 delay=1, beta=0.5, name="ragged", **H),
}


def _run(spec, seed, iterations):
    import torch as t
    from paper_1906_09108_amd import FdgModule
    dev = t.device("cuda:0")
    m = FdgModule(spec)
    m.set_params(W.make_params(spec, seed, perturb_bn=True))
    gin = None if spec.is_bottom else t.empty(spec.input_shape(), dtype=t.float32, device=dev)
    out = []
    d = spec.delay
    for it in range(d + iterations):
        x, lab = W.make_input(spec, it, seed), W.make_labels(spec, it, seed)
        y = m.forward(t.from_numpy(x).to(dev), None if lab is None else t.from_numpy(lab).to(dev))
        out.append(("y", it, y.cpu().numpy()))
        if it < d:
            continue
        g = W.make_grad_out(spec, it - d, seed)
        m.backward_delayed(None if g is None else t.from_numpy(g).to(dev), gin)
        out.append(("grads", it, m.get_grads()))
        if gin is not None:
            out.append(("grad_in", it, gin.cpu().numpy()))
        m.update(spec.lr)
        out.append(("theta", it, m.get_params()))
    out.append(("running", -1, m.get_bn_running()))
    m.close()
    return out


@pytest.mark.parametrize("name", list(CASES))
def test_two_runs_give_the_same_bits(name):
    spec = CASES[name]()
    print("determinism case", name, flush=True)
    a, b = _run(spec, 5, 2), _run(spec, 5, 2)
    assert len(a) == len(b)
    bad = [f"{la} at iteration {ia}: {np.count_nonzero(va != vb)} of {va.size} elements differ"
           for (la, ia, va), (_, _, vb) in zip(a, b) if not np.array_equal(va, vb)]
    assert not bad, "\n".join(bad)
    assert all(np.all(np.isfinite(v)) for _, _, v in a)


@pytest.mark.parametrize("name", ["cfg4_n8", "cfg8_n25", "ragged"])
def test_weight_gradients_on_the_callers_stream_give_the_same_bits(name):
    """fdg_overlap_enable(m, 0) keeps the weight gradients on the caller's stream instead of the module's second one:
    the same kernels on the same operands, so the same bits."""
    spec = CASES[name]()
    print("overlap on/off case", name, flush=True)

    def run(overlap):
        import torch as t
        from paper_1906_09108_amd import FdgModule
        dev = t.device("cuda:0")
        m = FdgModule(spec)
        m.overlap_enable(overlap)
        m.set_params(W.make_params(spec, 3, perturb_bn=True))
        gin = None if spec.is_bottom else t.empty(spec.input_shape(), dtype=t.float32, device=dev)
        out = []
        for it in range(spec.delay + 2):
            x, lab = W.make_input(spec, it, 3), W.make_labels(spec, it, 3)
            m.forward(t.from_numpy(x).to(dev), None if lab is None else t.from_numpy(lab).to(dev))
            if it < spec.delay:
                continue
            g = W.make_grad_out(spec, it - spec.delay, 3)
            m.backward_delayed(None if g is None else t.from_numpy(g).to(dev), gin)
            out.append(m.get_grads())
            m.update(spec.lr)
            out.append(m.get_params())
        m.close()
        return out
    a, b = run(True), run(False)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    assert all(np.all(np.isfinite(u)) for u in a)

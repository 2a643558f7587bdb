"""A module step recorded into a HIP graph and replayed (callers with launch-bound loops do that): the library
allocates nothing, clears memory with fill kernels (no memset nodes) and forks / joins its second stream with events,
so fdg_forward + fdg_backward_delayed + fdg_update of a delay-0 module capture as one graph.  Every replay is checked
against the eager result on the same input, with eager work and synchronisations between the replays."""
import copy

import numpy as np
import pytest

import fdg_workloads as W
from tests.gpu_harness import TOL, rel_err, rel_l2
from tests.test_gpu_parity import STRICT

pytestmark = pytest.mark.gpu


def test_module_step_replays_from_a_hip_graph():
    import torch
    from paper_1906_09108_amd import FdgModule
    spec = copy.deepcopy(STRICT["head_postact"])          # block + pool + FC + loss, delay 0: one ring position
    m = FdgModule(spec)
    m.set_params(W.make_params(spec, 2, perturb_bn=True))
    s = torch.cuda.Stream()
    x = torch.empty(spec.input_shape(), dtype=torch.float32, device="cuda")
    labels = torch.empty(spec.n, dtype=torch.int32, device="cuda")
    y = m.new_output()
    grad_in = torch.empty(spec.input_shape(), dtype=torch.float32, device="cuda")

    def load(t):
        x.copy_(torch.from_numpy(W.make_input(spec, t, 2)))
        labels.copy_(torch.from_numpy(W.make_labels(spec, t, 2)))
        torch.cuda.synchronize()

    def eager():
        m.forward(x, labels, y, stream=s)
        m.backward_delayed(None, grad_in, stream=s)
        m.update(0.0, stream=s)                            # frozen weights: a replay must reproduce the eager numbers
        s.synchronize()
        return y.cpu().numpy().copy(), m.get_grads(), grad_in.cpu().numpy().copy()

    load(0)
    eager()                                               # first launches configure kernels: not inside a capture
    refs = {}
    for t in range(4):
        load(t)
        refs[t] = eager()
    load(0)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        m.forward(x, labels, y, stream=s)
        m.backward_delayed(None, grad_in, stream=s)
        m.update(0.0, stream=s)
    torch.cuda.synchronize()
    assert m.queue_state()[0] == 0
    for t in (1, 2, 0, 3, 3):
        load(t)
        worst = None
        for attempt in range(3):   # a replay adds its batch-norm sums in its own order: about one run in ten decides a
            y.zero_()              # ReLU gate the other way (tests/test_gpu_chain.py), so a replay may be repeated
            grad_in.zero_()
            g.replay()
            torch.cuda.synchronize()
            got = (y.cpu().numpy(), m.get_grads(), grad_in.cpu().numpy())
            worst = None
            for name, a, b in zip(("y", "grads", "grad_in"), got, refs[t]):
                assert np.abs(b).max() > 0
                if not (rel_l2(a, b) <= 2.0 ** -8 and rel_err(a, b) <= TOL):
                    worst = (t, name, rel_l2(a, b), rel_err(a, b))
                    break
            if worst is None:
                break
        assert worst is None, worst
        if t == 2:                                        # eager work of the same module between replays
            load(1)
            e = eager()
            assert rel_l2(e[1], refs[1][1]) <= 2.0 ** -8
    m.close()

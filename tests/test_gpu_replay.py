"""FDG_SAVE_INPUT_AND_REPLAY on the GPU (include/fdg.h): a saved forward is its input and its weight snapshot, and
the delayed backward runs the forward again before back-propagating.

  * against the oracle, on the same bars as the stored form (tests/gpu_harness.py), with delays, both call
    orders, a head, wide layers and benchmark modules at reduced batch;
  * against the stored form of the library itself with frozen weights: same outputs and gradients up to the order
    of fp32 atomic sums.  A last-bit difference in a batch-norm sum can move one bf16 rounding of an intermediate
    (2^-9 of that element) or, where an activation sits on the ReLU threshold, one gate (in the module with the
    pooling head one gate carries the same loss gradient to 64 pixels); two runs of the SAME form differ in the
    same way.  Bars: 2^-8 in relative L2 and the 2e-2 parity bar in max norm;
  * running statistics move in fdg_forward only: a backward leaves them bit for bit as they were.
"""
import copy

import numpy as np
import pytest

import fdg_workloads as W
from tests.gpu_harness import TOL, format_report, judge, rel_err, rel_l2, run_side_by_side
from tests.test_gpu_parity import ENVELOPE, STRICT

pytestmark = pytest.mark.gpu

REPLAY = 1


def _check(spec, steps, strict, deep=False, **kw):
    records, exact = run_side_by_side(spec, steps, save_mode=REPLAY, **kw)
    print(f"\n[{spec.name}] replay: largest deviations from the kernel-precision oracle\n{format_report(records)}", flush=True)
    assert not exact, exact
    bad = judge(records, spec, strict, deep=deep)
    assert not bad, "\n".join(bad[:40])


@pytest.mark.parametrize("name", ["postact_identity_delay1", "preact_project", "head_postact", "stem_with_grad_in"])
def test_replay_shallow_modules_meet_the_strict_bar(name):
    spec = copy.deepcopy(STRICT[name])
    spec.name = name
    print(f"replay case {name}", flush=True)
    _check(spec, steps=2, strict=True, seed=1)


@pytest.mark.parametrize("name", ["head_preact", "postact_project_ragged", "preact_wide", "bottom_stack_delay2", "bottleneck_project_delay1"])
def test_replay_ragged_wide_and_stacked_modules(name):
    spec = copy.deepcopy(ENVELOPE[name])
    spec.name = name
    print(f"replay case {name}", flush=True)
    _check(spec, steps=3, strict=False, seed=1)


def test_replay_backward_first_order_of_algorithm_1():
    spec = copy.deepcopy(ENVELOPE["bottom_stack_delay2"])
    spec.name = "replay backward-first"
    _check(spec, steps=3, strict=False, seed=2, backward_first=True)


@pytest.mark.parametrize("idx,n,steps", [(3, 16, 2), (4, 8, 1), (5, 8, 1), (8, 25, 1)])
def test_replay_configs_reduced_batch(idx, n, steps):
    spec = W.config(idx, n=n)
    print(f"replay case cfg{idx} n={n}", flush=True)
    _check(spec, steps=steps, strict=False, deep=idx == 5, perturb_bn=False)


def _forms_agree(run, forms):
    """run(form) -> list of (label, array).  Two forms of the same iteration run the same kernels on the same numbers, and
    every sum over workgroups is order independent (tests/test_gpu_determinism.py), so they must agree BIT FOR BIT."""
    ra, rb = run(forms[0]), run(forms[1])
    assert len(ra) == len(rb)
    for (k, a), (_, b) in zip(ra, rb):
        assert np.abs(a).max() > 0, k
        assert np.array_equal(a, b), (k, rel_l2(b, a), rel_err(b, a), int(np.count_nonzero(a != b)), a.size)


@pytest.mark.parametrize("name", ["postact_identity_delay1", "bottom_stack_delay2", "head_preact"])
def test_replay_equals_the_stored_form_with_frozen_weights(name):
    import torch
    from paper_1906_09108_amd import FdgModule
    spec = copy.deepcopy({**STRICT, **ENVELOPE}[name])
    print(f"replay vs stored {name}", flush=True)
    theta = W.make_params(spec, 4, perturb_bn=True)
    d = spec.delay
    def run(mode):
        m = FdgModule(spec, save_mode=mode)
        m.set_params(theta)
        grad_in = None if spec.is_bottom else torch.empty(spec.input_shape(), dtype=torch.float32, device="cuda")
        got = []
        for t in range(d + 3):
            x = torch.from_numpy(W.make_input(spec, t, 4)).cuda()
            labels = W.make_labels(spec, t, 4)
            y = m.forward(x, None if labels is None else torch.from_numpy(labels).cuda())
            got.append(("y", y.cpu().numpy()))
            if t >= d:
                before = m.get_bn_running()
                g = W.make_grad_out(spec, t - d, 4)
                m.backward_delayed(None if g is None else torch.from_numpy(g).cuda(), grad_in)
                got.append(("grads", m.get_grads()))
                if grad_in is not None:
                    got.append(("grad_in", grad_in.cpu().numpy()))
                np.testing.assert_array_equal(m.get_bn_running(), before)
                m.update(0.0)
        got.append(("running", m.get_bn_running()))
        assert m.queue_state()[0] == d
        m.close()
        return got

    _forms_agree(run, (0, REPLAY))


def test_replay_workspace_is_smaller():
    from paper_1906_09108_amd import FdgModule
    spec = W.config(3, n=16)
    a, b = FdgModule(spec, save_mode=0), FdgModule(spec, save_mode=REPLAY)
    assert b.workspace_bytes < a.workspace_bytes
    a.close()
    b.close()


@pytest.mark.parametrize("name", ["postact_identity_delay1", "bottom_stack_delay2"])
def test_forward_and_delayed_backward_on_two_streams(name):
    """include/fdg.h, "Two streams": with delay >= 1 the forward (newest context) and the delayed backward (oldest
    context) share no temporary and may overlap on the GPU; the caller orders the update after both and the next
    forward after the update.  The same iterations as on one stream, bit for bit, with moving weights: the events order
    every snapshot of the weights against every update."""
    import torch
    from paper_1906_09108_amd import FdgModule
    spec = copy.deepcopy({**STRICT, **ENVELOPE}[name])
    print(f"two streams {name}", flush=True)
    theta = W.make_params(spec, 6, perturb_bn=True)
    d = spec.delay
    def run(two):
        m = FdgModule(spec)
        m.set_params(theta)
        grad_in = None if spec.is_bottom else torch.empty(spec.input_shape(), dtype=torch.float32, device="cuda")
        s_f, s_b = (torch.cuda.Stream(), torch.cuda.Stream()) if two else (torch.cuda.current_stream(),) * 2
        ev_f, ev_u = torch.cuda.Event(), torch.cuda.Event()
        torch.cuda.synchronize()
        ev_u.record(s_b)
        got = []
        ys = []
        for t in range(d + 3):
            x = torch.from_numpy(W.make_input(spec, t, 6)).cuda()
            torch.cuda.synchronize()                       # x is ready for whichever stream reads it
            s_f.wait_event(ev_u)
            ys.append(m.forward(x, None, stream=s_f))
            ev_f.record(s_f)
            if t >= d:
                g = torch.from_numpy(W.make_grad_out(spec, t - d, 6)).cuda(non_blocking=False)
                m.backward_delayed(g, grad_in, stream=s_b)
                s_b.wait_event(ev_f)
                m.update(0.01, stream=s_b)
                ev_u.record(s_b)
                torch.cuda.synchronize()
                got.append(("grads", m.get_grads()))
                if grad_in is not None:
                    got.append(("grad_in", grad_in.cpu().numpy()))
            torch.cuda.synchronize()                       # the forward's stream is not the one the copy below runs on
            got.append(("y", ys[-1].cpu().numpy()))
        got.append(("theta", m.get_params()))
        got.append(("running", m.get_bn_running()))
        m.close()
        return got

    _forms_agree(run, (False, True))

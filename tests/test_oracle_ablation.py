"""Pins of the oracle's "current weights" ablation (OracleModule(weights="current")): the delayed backward works on
the activations and batch statistics its forward kept, but takes the parameters as they are when it runs -- what a
framework that updates weights in place and back-propagates through a saved graph computes.  (The method itself,
Eq. 10, evaluates every factor at the forward's parameters: weights="snapshot", pinned in test_oracle_module.py.)

The independent reference is torch.autograd used exactly in that way: forward at the old parameters with the graph kept,
the leaf tensors overwritten through .data (which autograd does not see), then backward."""
import copy

import numpy as np
import pytest
import torch

import fdg_workloads as W
from oracle.fdg_oracle import OracleModule
from tests import torch_ref
from tests.test_oracle_module import TINY


def _run(spec, weights, steps, seed=2, lr=None, dtype=np.float64):
    m = OracleModule(spec, dtype, weights=weights)
    m.set_params(W.make_params(spec, seed, perturb_bn=True).astype(dtype))
    out = []
    for t in range(spec.delay + steps):
        x = W.make_input(spec, t, seed).astype(dtype)
        m.forward(x, W.make_labels(spec, t, seed))
        if t < spec.delay:
            continue
        g = W.make_grad_out(spec, t - spec.delay, seed)
        gin = m.backward_delayed(None if g is None else g.astype(dtype))
        out.append((m.get_grads(), gin))
        m.update(spec.lr if lr is None else lr)
    return out, m.get_params()


@pytest.mark.parametrize("name", ["stack", "head_preact", "bottleneck_stack_head", "preact_project"])
def test_without_delay_the_current_weights_are_the_forwards(name):
    """Forward, backward, update in this order with delay 0: nothing moves the parameters between a forward and its
    backward, so the ablation is the method, bit for bit."""
    spec = copy.deepcopy(TINY[name])
    spec.delay = 0
    a, ta = _run(spec, "snapshot", 3, dtype=np.float32)
    b, tb = _run(spec, "current", 3, dtype=np.float32)
    for (ga, ia), (gb, ib) in zip(a, b):
        np.testing.assert_array_equal(ga, gb)
        if ia is not None:
            np.testing.assert_array_equal(ia, ib)
    np.testing.assert_array_equal(ta, tb)


def test_with_a_zero_step_size_the_ablation_is_the_method():
    spec = copy.deepcopy(TINY["stack"])
    spec.delay, spec.beta, spec.weight_decay = 2, 0.5, 0.0
    a, _ = _run(spec, "snapshot", 3, lr=0.0)
    b, _ = _run(spec, "current", 3, lr=0.0)
    for (ga, ia), (gb, ib) in zip(a, b):
        np.testing.assert_array_equal(ga, gb)
        np.testing.assert_array_equal(ia, ib)


@pytest.mark.parametrize("name", ["stem", "stack", "postact_project", "preact_identity", "preact_project", "head_preact", "head_postact",
                                  "bottleneck_project", "bottleneck_stack_head"])
def test_against_autograd_on_a_saved_graph_with_weights_overwritten_in_place(name):
    spec = copy.deepcopy(TINY[name])
    spec.delay, spec.beta = 1, (1.0 if spec.is_top else 0.5)
    seed = 4
    theta0 = W.make_params(spec, seed, perturb_bn=True).astype(np.float64)
    m = OracleModule(spec, np.float64, weights="current")
    m.set_params(theta0)
    xs = [W.make_input(spec, t, seed).astype(np.float64) for t in range(2)]
    labs = [W.make_labels(spec, t, seed) for t in range(2)]
    g0 = W.make_grad_out(spec, 0, seed)
    g0 = None if g0 is None else g0.astype(np.float64)
    m.forward(xs[0], labs[0])
    # move the parameters as an update would, but far enough to matter: an arbitrary other point
    theta1 = theta0 + 0.3 * W.make_params(spec, seed + 1, perturb_bn=True).astype(np.float64)
    m.theta.flat[...] = theta1
    m.forward(xs[1], labs[1])
    gin = m.backward_delayed(g0)            # the oldest saved forward: batch 0, run at theta0

    params = torch_ref.split_params(spec, W.param_shapes(spec), theta0)
    xt = torch.tensor(xs[0], requires_grad=True)
    out = torch_ref.forward(spec, params, xt, labs[0])
    off = 0
    for p in params:                        # in place, unseen by autograd
        p.data.copy_(torch.tensor(theta1[off:off + p.numel()]).reshape(p.shape))
        off += p.numel()
    if spec.is_top:
        out[0].backward()
    else:
        out.backward(torch.tensor(g0) * spec.beta)
    ref = np.concatenate([p.grad.numpy().reshape(-1) for p in params])
    np.testing.assert_allclose(m.get_grads(), ref, rtol=1e-7, atol=1e-10)
    if gin is not None:
        np.testing.assert_allclose(gin, xt.grad.numpy(), rtol=1e-7, atol=1e-10)

    # and it is NOT the method: Eq. 10 at theta0 gives something else wherever a parameter sits between the loss and a gradient
    s = OracleModule(spec, np.float64)
    s.set_params(theta0)
    s.forward(xs[0], labs[0])
    s.theta.flat[...] = theta1
    s.forward(xs[1], labs[1])
    s.backward_delayed(g0)
    if len(spec.layers) > 1 or spec.layers[0].kind != W.HEAD_POSTACT:
        assert np.abs(s.get_grads() - m.get_grads()).max() > 1e-6

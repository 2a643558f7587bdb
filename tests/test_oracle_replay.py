"""Pins of the oracle's save="input" mode (a saved forward keeps its input and its parameters; the delayed
backward runs that forward again -- recomputation as in feature replay, Section II, at FDG's stale parameters):

  * it is the same iteration: over several steps with moving weights, delay d and beta < 1, every output,
    gradient, parameter and running statistic equals the save="activations" run bit for bit (both element
    types and both storage precisions) -- the replay adds no arithmetic of its own;
  * independently of that run: the backward of the oldest context equals a fresh back-propagation by
    torch autograd at (x_stale, theta at that forward), times beta (Eq. 10, Eq. 15);
  * the context really holds no intermediate, and the running statistics move once per forward, not once
    more per replay (closed form of one step from the batch moments).
"""
import copy

import numpy as np
import pytest
import torch

import fdg_workloads as W
from oracle.fdg_oracle import OracleModule
from tests import torch_ref
from tests.test_oracle_module import TINY


def _run(spec, dtype, storage, save, steps, seed=2):
    m = OracleModule(spec, dtype, storage=storage, save=save)
    m.set_params(W.make_params(spec, seed, perturb_bn=True).astype(dtype))
    d, out = spec.delay, []
    for t in range(d + steps):
        x = W.make_input(spec, t, seed).astype(dtype)
        labels = W.make_labels(spec, t, seed)
        out.append(("y", m.forward(x, labels)))
        if t >= d:
            g = W.make_grad_out(spec, t - d, seed)
            gin = m.backward_delayed(None if g is None else g.astype(dtype))
            out.append(("grads", m.get_grads()))
            if gin is not None:
                out.append(("grad_in", gin))
            m.update(spec.lr)
            out.append(("theta", m.get_params()))
    out.append(("running", m.get_bn_running()))
    return m, out


@pytest.mark.parametrize("name,d", [("stack", 2), ("preact_project", 1), ("head_preact", 0), ("head_postact", 0), ("postact_project", 3)])
@pytest.mark.parametrize("dtype,storage", [(np.float64, "fp32"), (np.float32, "fp32"), (np.float32, "bf16")])
def test_replay_is_the_same_iteration_bit_for_bit(name, d, dtype, storage):
    spec = copy.deepcopy(TINY[name])
    spec.delay = d
    spec.beta = 1.0 if spec.is_top else 0.3
    _, a = _run(spec, dtype, storage, "activations", steps=4)
    _, b = _run(spec, dtype, storage, "input", steps=4)
    assert [k for k, _ in a] == [k for k, _ in b]
    for (k, u), (_, v) in zip(a, b):
        np.testing.assert_array_equal(u, v, err_msg=k)
    assert any(k == "grads" and np.abs(u).max() > 0 for k, u in a)


@pytest.mark.parametrize("d", [1, 2])
def test_replayed_backward_is_autograd_at_the_stale_batch_and_stale_weights(d):
    spec = copy.deepcopy(TINY["stack"])
    spec.delay, spec.beta = d, 0.4
    m = OracleModule(spec, np.float64, save="input")
    m.set_params(W.make_params(spec, 5, perturb_bn=True).astype(np.float64))
    xs = [W.make_input(spec, t, 5).astype(np.float64) for t in range(d + 4)]
    gs = [W.make_grad_out(spec, t, 5).astype(np.float64) for t in range(d + 4)]
    snaps = []
    for t in range(d + 4):
        snaps.append(m.get_params())
        m.forward(xs[t])
        if t < d:
            continue
        s = t - d
        gin = m.backward_delayed(gs[s])
        params = torch_ref.split_params(spec, W.param_shapes(spec), snaps[s])
        xt = torch.tensor(xs[s], requires_grad=True)
        y = torch_ref.forward(spec, params, xt)
        y.backward(torch.tensor(spec.beta * gs[s]))
        ref = np.concatenate([p.grad.numpy().reshape(-1) for p in params])
        np.testing.assert_allclose(m.get_grads(), ref, rtol=1e-8, atol=1e-11)
        np.testing.assert_allclose(gin, xt.grad.numpy(), rtol=1e-8, atol=1e-11)
        m.update(0.1)
        if t > d:
            assert np.abs(snaps[s] - snaps[t]).max() > 1e-6     # the weights did move between that forward and now


def test_a_saved_forward_holds_no_intermediate_and_statistics_move_once():
    spec = copy.deepcopy(TINY["stem"])
    spec.delay = 1
    m = OracleModule(spec, np.float64, save="input")
    theta = W.make_params(spec, 0, perturb_bn=True).astype(np.float64)
    m.set_params(theta)
    x = W.make_input(spec, 0, 0).astype(np.float64)
    m.forward(x)
    ctx = m.fifo[0]
    assert sorted(ctx) == ["labels", "seq", "theta", "x"]
    after_forward = m.get_bn_running()
    m.backward_delayed(W.make_grad_out(spec, 0, 0).astype(np.float64))
    np.testing.assert_array_equal(m.get_bn_running(), after_forward)
    # one step of the running statistics from the batch moments of the convolution output (momentum 0.1, unbiased variance)
    w = torch_ref.split_params(spec, W.param_shapes(spec), theta)[0].detach()
    c = torch.nn.functional.conv2d(torch.tensor(x), w, padding=1).numpy()
    mean = c.mean(axis=(0, 2, 3))
    var = c.var(axis=(0, 2, 3), ddof=1)
    C = mean.size
    np.testing.assert_allclose(after_forward[:C], 0.1 * mean, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(after_forward[C:], 0.9 + 0.1 * var, rtol=1e-10)

"""Pins of the K-module oracle (oracle.fdg_oracle.OracleChain: Algorithm I with the communication of
Section III-A) against things that are not the oracle:

  * the batch indices of Section III-A (module k forwards batch t-k+1 and back-propagates batch
    t-2K+k+1, k counted from 1) -- closed forms;
  * Eq. 13 with Eq. 16/17: with frozen weights the gradient a module computes is beta^(K-k) times the
    gradient of the WHOLE network on the stale batch -- torch autograd of the composed network, float64;
  * the full iteration with moving weights, momentum and weight decay -- an independent simulation
    written with torch tensors that RECOMPUTES every stale forward at the weights that forward used
    (mathematically the saved graph of Fig. 1(b)), float64;
  * K = 1 is ordinary back-propagation with momentum SGD (torch, float64);
  * the loss goes down on separable data (the point of running the algorithm at all).
"""
import numpy as np
import pytest
import torch

import fdg_workloads as W
from oracle.fdg_oracle import OracleChain
from tests import torch_ref


def _tiny(K, beta=0.5, **kw):
    return W.chain_specs(K, n=4, width=4, hw=4, blocks=1, beta=beta, num_classes=3, **kw)


def _params(specs, seed=0):
    return [W.make_params(sp, seed + 17 * k, perturb_bn=True).astype(np.float64) for k, sp in enumerate(specs)]


def _chain(specs, thetas, dtype=np.float64):
    ch = OracleChain(specs, dtype)
    for m, th in zip(ch.mods, thetas):
        m.set_params(th)
    return ch


@pytest.mark.parametrize("K", [1, 2, 3, 4])
def test_batch_indices_of_section_3a(K):
    specs = _tiny(K)
    ch = _chain(specs, _params(specs))
    for t in range(1, 13):
        x, labels = W.make_separable_batch(specs[0], t)
        res = ch.step(x.astype(np.float64), labels, 0.01)
        for k1 in range(1, K + 1):                     # the paper counts modules from 1
            assert ch.fwd_batch[k1 - 1] == max(0, t - k1 + 1)
            assert ch.bwd_batch[k1 - 1] == max(0, t - 2 * K + k1 + 1)
        assert (res is None) == (t - K + 1 < 1)
        if res is not None:
            assert res[0] == t - K + 1
    for k, m in enumerate(ch.mods):                    # saved forwards still waiting for their gradient
        assert m.queue_state()[0] == 2 * (K - 1 - k)


@pytest.mark.parametrize("K,beta", [(2, 0.5), (3, 0.3), (4, 0.7)])
def test_frozen_weights_give_the_shrunk_stale_gradient_of_the_whole_network(K, beta):
    """Eq. 13 / Eq. 17: g_hat(module k, iteration t) = beta^(K-k) * dLoss(batch d_kt)/dtheta_k."""
    specs = _tiny(K, beta=beta)
    thetas = _params(specs)
    ch = _chain(specs, thetas)
    whole = W.whole_network_spec(specs)
    flat = np.concatenate(thetas)
    batches = {}
    T = 2 * K + 2
    checked = 0
    for t in range(1, T + 1):
        x, labels = W.make_separable_batch(specs[0], t)
        batches[t] = (x.astype(np.float64), labels)
        ch.step(batches[t][0], labels, 0.0)            # lr = 0: the weights never move
        for k in range(K):
            b = ch.bwd_batch[k]
            if not b:
                continue
            params = torch_ref.split_params(whole, W.param_shapes(whole), flat)
            loss, _ = torch_ref.forward(whole, params, torch.tensor(batches[b][0]), batches[b][1])
            loss.backward()
            ref = np.concatenate([p.grad.numpy().reshape(-1) for p in params])
            off = sum(th.size for th in thetas[:k])
            ref_k = ref[off:off + thetas[k].size] * beta ** (K - 1 - k)
            np.testing.assert_allclose(ch.mods[k].get_grads(), ref_k, rtol=1e-6, atol=1e-10)
            checked += 1
    assert checked >= K + 2


def _torch_algorithm_1(specs, thetas, batches, lr):
    """Algorithm I written independently: per module a parameter list, a momentum list and a FIFO of
    (input, parameters as of that forward); a backward RECOMPUTES the stale forward at those stale
    parameters with autograd and feeds it beta * received gradient."""
    K = len(specs)
    P = [[p.detach().clone() for p in torch_ref.split_params(sp, W.param_shapes(sp), th)] for sp, th in zip(specs, thetas)]
    V = [[torch.zeros_like(p) for p in ps] for ps in P]
    fifo = [[] for _ in range(K)]
    inbox_act, inbox_grad = [None] * K, [None] * K
    losses = []

    def backprop(k, grad_out, labels=None):
        z_in, stale = fifo[k].pop(0)
        leaves = [p.clone().requires_grad_(True) for p in stale]
        zi = z_in.clone().requires_grad_(True)
        out = torch_ref.forward(specs[k], leaves, zi, labels)
        if labels is not None:
            out[0].backward()
        else:
            out.backward(specs[k].beta * grad_out)
        for p, v, leaf in zip(P[k], V[k], leaves):
            g = leaf.grad + specs[k].weight_decay * p
            v.mul_(specs[k].momentum).add_(g)
            p.sub_(lr * v)
        return zi.grad

    for t in range(1, len(batches) + 1):
        x, labels_t = batches[t]
        send_act, send_grad = {}, {}
        for k in range(K):
            inp = (t, torch.tensor(x)) if k == 0 else inbox_act[k]
            if k == K - 1:
                if inp is not None:
                    b, z = inp
                    fifo[k].append((z, [p.clone() for p in P[k]]))
                    with torch.no_grad():
                        losses.append((b, torch_ref.forward(specs[k], P[k], z, batches[b][1])[0].item()))
                    gin = backprop(k, None, batches[b][1])
                    if k > 0:
                        send_grad[k - 1] = gin
            else:
                if inbox_grad[k] is not None:
                    gin = backprop(k, inbox_grad[k])
                    if k > 0:
                        send_grad[k - 1] = gin
                if inp is not None:
                    b, z = inp
                    fifo[k].append((z, [p.clone() for p in P[k]]))
                    with torch.no_grad():
                        send_act[k + 1] = (b, torch_ref.forward(specs[k], P[k], z))
        inbox_act = [send_act.get(k) for k in range(K)]
        inbox_grad = [send_grad.get(k) for k in range(K)]
    return [np.concatenate([p.numpy().reshape(-1) for p in ps]) for ps in P], losses


@pytest.mark.parametrize("K", [1, 2, 3])
def test_algorithm_1_against_an_independent_torch_simulation(K):
    specs = _tiny(K, beta=0.4)
    thetas = _params(specs, seed=3)
    T = 2 * K + 4
    batches = {}
    for t in range(1, T + 1):
        x, labels = W.make_separable_batch(specs[0], t, seed=5)
        batches[t] = (x.astype(np.float64), labels)
    ch = _chain(specs, thetas)
    got_losses = []
    for t in range(1, T + 1):
        res = ch.step(batches[t][0], batches[t][1], 0.05)
        if res is not None:
            got_losses.append((res[0], res[1]))
    ref_params, ref_losses = _torch_algorithm_1(specs, thetas, batches, 0.05)
    assert [b for b, _ in got_losses] == [b for b, _ in ref_losses]
    np.testing.assert_allclose([l for _, l in got_losses], [l for _, l in ref_losses], rtol=1e-8)
    for m, ref in zip(ch.mods, ref_params):
        np.testing.assert_allclose(m.get_params(), ref, rtol=1e-6, atol=1e-9)
    if K > 1:   # and the weights did move, differently from module to module
        assert np.abs(ch.mods[0].get_params() - thetas[0]).max() > 1e-4


def test_k1_is_backpropagation_with_momentum_sgd():
    specs = _tiny(1)
    thetas = _params(specs, seed=1)
    sp = specs[0]
    ch = _chain(specs, thetas)
    params = [p.detach().clone().requires_grad_(True) for p in torch_ref.split_params(sp, W.param_shapes(sp), thetas[0])]
    opt = torch.optim.SGD(params, lr=0.05, momentum=sp.momentum, weight_decay=sp.weight_decay)
    for t in range(1, 5):
        x, labels = W.make_separable_batch(sp, t)
        res = ch.step(x.astype(np.float64), labels, 0.05)
        opt.zero_grad()
        loss, _ = torch_ref.forward(sp, params, torch.tensor(x.astype(np.float64)), labels)
        loss.backward()
        opt.step()
        assert res[0] == t and abs(res[1] - loss.item()) < 1e-9 * max(1.0, abs(loss.item()))
    ref = np.concatenate([p.detach().numpy().reshape(-1) for p in params])
    np.testing.assert_allclose(ch.mods[0].get_params(), ref, rtol=1e-7, atol=1e-10)


def test_loss_goes_down_on_separable_data():
    specs = W.chain_specs(3, n=16, width=8, hw=8, blocks=1, beta=0.5, num_classes=4, lr=0.05)
    ch = OracleChain(specs, np.float32)
    for k, m in enumerate(ch.mods):
        m.set_params(W.make_params(specs[k], k))
    losses = []
    for t in range(1, 41):
        x, labels = W.make_separable_batch(specs[0], t, noise=0.3)
        res = ch.step(x, labels, 0.05)
        if res is not None:
            losses.append(res[1])
    assert np.mean(losses[-5:]) < 0.5 * np.mean(losses[:5])

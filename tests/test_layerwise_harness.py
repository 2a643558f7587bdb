"""CPU check of the layer-by-layer parity harness (tests/layerwise.py) itself: a stand-in for the GPU module that
answers the parity accessors from a whole-module run of the ORACLE must pass the per-layer checks with zero deviation
(the per-layer factors of Eq. 8 - Eq. 10 multiply up to the whole module's backward), and a planted mistake in what
the stand-in reports must be found in the layer it was planted in and nowhere else."""
import numpy as np
import pytest

import fdg_workloads as W
from fdg_workloads import Layer, ModuleSpec
from oracle.fdg_oracle import OracleModule, _Flat
from tests import layerwise as LW

H = dict(momentum=0.9, weight_decay=5e-4, lr=0.1)


class OracleAsGpu:
    """Answers saved_read / trace_read from one forward and one backward of the bf16-storage oracle."""

    def __init__(self, spec, theta, x, labels, grad_out):
        om = OracleModule(spec, np.float32, storage="bf16")
        om.set_params(theta)
        self.spec = spec
        th = om._stored_weights(om.theta.copy())
        self.y, self.tapes = om._layers(np.ascontiguousarray(x, np.float32), labels, th, move_running=False)
        # residual stream after every layer: run the layers one after the other, as the module does
        self.z, z = [], np.ascontiguousarray(x, np.float32)
        shapes = LW._input_shapes(spec)
        for i, L in enumerate(spec.layers):
            if L.is_head:
                break
            _, o1 = LW._one_layer(spec, i, shapes[i])
            lo, hi = LW.layer_slices(spec)[i]
            o1.set_params(theta[lo:hi])
            z, _ = o1._layers(z, None, o1._stored_weights(o1.theta.copy()), move_running=False)
            self.z.append(z)
        g = _Flat(om.layout, om.dt)
        dz = None if spec.is_top else (np.float32(spec.beta) * grad_out).astype(np.float32)
        self.dz = {len(spec.layers): dz}
        for i in reversed(range(len(spec.layers))):
            dz = om._layer_backward(i, spec.layers[i], self.tapes[i], th, dz, g, not (i == 0 and spec.is_bottom))
            self.dz[i] = dz
        self.grads = g.flat.copy()

    def saved_read(self, seq, layer, which):
        t, L = self.tapes[layer], self.spec.layers[layer]
        if which == 7:
            return t["x"]
        if which == 6:
            return t["y"]
        if which == 8:
            return t["p"][:, :, None, None]
        if which == 9:
            return t["dl"][:, :, None, None]
        key = dict(LW.SAVED[L.kind])[which]
        return t[f"{layer}.{key[3:]}"][0] if key.startswith("bn:") else t[key]

    def trace_read(self, direction, layer):
        return (self.z[layer] if direction == 0 else self.dz[layer]), False


CASES = {
    "postact_stack": ModuleSpec(4, 3, 12, 12, [Layer(W.STEM, 3, 16, 1), Layer(W.BASIC_POSTACT, 16, 16, 1),
                                               Layer(W.BASIC_POSTACT, 16, 32, 2)], beta=0.5, **H),
    "preact_head": ModuleSpec(6, 16, 8, 8, [Layer(W.BASIC_PREACT, 16, 16, 1), Layer(W.BASIC_PREACT, 16, 32, 2),
                                            Layer(W.HEAD_PREACT, 32)], num_classes=5, **H),
    "bottleneck_head": ModuleSpec(4, 32, 8, 8, [Layer(W.BOTTLENECK_POSTACT, 32, 64, 2), Layer(W.BOTTLENECK_POSTACT, 64, 64, 1),
                                                Layer(W.HEAD_POSTACT, 64)], num_classes=5, **H),
}


def _stand_in(spec, seed=3):
    theta = W.make_params(spec, seed, perturb_bn=True)
    x, labels, g = W.make_input(spec, 0, seed), W.make_labels(spec, 0, seed), W.make_grad_out(spec, 0, seed)
    return theta, x, labels, OracleAsGpu(spec, theta, x, labels, g)


@pytest.mark.parametrize("name", list(CASES))
def test_the_oracle_passes_its_own_layerwise_check_exactly(name):
    spec = CASES[name]
    theta, x, labels, fake = _stand_in(spec)
    rows = LW.check_forward_layers(fake, spec, theta, 0, x, labels, fake.y)
    rows += LW.check_backward_layers(fake, spec, theta, 0, fake.grads, None if spec.is_bottom else fake.dz[0])
    assert len(rows) > 10
    # the backward's batch statistics are recomputed from the kept tensors by the same routine: identical bits
    assert max(r.max_norm for r in rows) == 0.0, LW.format_rows(rows, 5)


def test_a_planted_mistake_is_found_where_it_was_planted():
    spec = CASES["postact_stack"]
    theta, x, labels, fake = _stand_in(spec)
    names = [n for n, _ in LW.oracle_param_layout(spec)]
    lo, hi = LW.layer_slices(spec)[1]
    fake.grads[lo + 5] *= 1.5                       # one element of layer 1's first weight gradient
    fake.dz[2] = fake.dz[2].copy()
    fake.dz[2][1, 3, 2, 2] += 0.05 * np.abs(fake.dz[2]).max()   # and the gradient layer 2 hands to layer 1
    rows = LW.check_backward_layers(fake, spec, theta, 0, fake.grads, None)
    wrong = [(r.layer, r.what) for r in rows if r.max_norm > 1e-4]
    # layer 2's reported input gradient is off; layer 1, fed with it, is consistent with it except for the planted weight
    assert (2, "bwd input gradient") in wrong
    assert (1, "bwd grad conv1.w") in wrong
    assert all(layer in (1, 2) for layer, _ in wrong), wrong
    assert names[0].startswith("0.")

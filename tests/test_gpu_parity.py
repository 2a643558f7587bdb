"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Every test needs a real MI355X."""
import copy

import numpy as np
import pytest

import fdg_workloads as W
from fdg_workloads import Layer, ModuleSpec
from tests.gpu_harness import TOL, format_report, run_side_by_side

pytestmark = pytest.mark.gpu

H = dict(momentum=0.9, weight_decay=5e-4, lr=0.1)

# small modules: every layer kind, both shortcut forms, strides, ragged sizes that leave partial tiles
SMALL = {
    "stem": ModuleSpec(3, 3, 9, 7, [Layer(W.STEM, 3, 16, 1)], delay=0, is_bottom=True, beta=0.5, **H),
    "stem_with_grad_in": ModuleSpec(2, 3, 8, 8, [Layer(W.STEM, 3, 16, 1)], delay=0, is_bottom=False, beta=0.5, **H),
    "postact_identity": ModuleSpec(3, 16, 7, 5, [Layer(W.BASIC_POSTACT, 16, 16, 1)], delay=0, beta=0.2, **H),
    "postact_identity_fast_rows": ModuleSpec(4, 16, 8, 8, [Layer(W.BASIC_POSTACT, 16, 16, 1)], delay=1, beta=0.2, **H),
    "postact_project": ModuleSpec(3, 16, 8, 6, [Layer(W.BASIC_POSTACT, 16, 32, 2)], delay=0, beta=0.2, **H),
    "postact_project_odd": ModuleSpec(2, 16, 7, 9, [Layer(W.BASIC_POSTACT, 16, 32, 2)], delay=0, beta=0.2, **H),
    "postact_wide": ModuleSpec(2, 96, 6, 6, [Layer(W.BASIC_POSTACT, 96, 160, 1)], delay=0, beta=1.0, **H),
    "preact_identity": ModuleSpec(3, 16, 5, 7, [Layer(W.BASIC_PREACT, 16, 16, 1)], delay=0, beta=0.7, **H),
    "preact_project": ModuleSpec(3, 16, 8, 8, [Layer(W.BASIC_PREACT, 16, 32, 2)], delay=0, beta=0.7, **H),
    "preact_widen": ModuleSpec(2, 24, 6, 5, [Layer(W.BASIC_PREACT, 24, 40, 1)], delay=0, beta=0.7, **H),
    "preact_wide": ModuleSpec(2, 160, 8, 8, [Layer(W.BASIC_PREACT, 160, 320, 2), Layer(W.BASIC_PREACT, 320, 320, 1)],
                              delay=0, beta=1.0, **H),
    "head_preact": ModuleSpec(5, 32, 4, 4, [Layer(W.BASIC_PREACT, 32, 32, 1), Layer(W.HEAD_PREACT, 32)], delay=0,
                              num_classes=10, **H),
    "head_postact": ModuleSpec(5, 32, 4, 4, [Layer(W.BASIC_POSTACT, 32, 32, 1), Layer(W.HEAD_POSTACT, 32)], delay=0,
                               num_classes=7, **H),
    "bottom_stack_delay2": ModuleSpec(4, 3, 16, 16, [Layer(W.STEM, 3, 16, 1), Layer(W.BASIC_POSTACT, 16, 16, 1),
                                                     Layer(W.BASIC_POSTACT, 16, 32, 2), Layer(W.BASIC_POSTACT, 32, 32, 1)],
                                      delay=2, is_bottom=True, beta=0.2, **H),
}


def _check(spec, steps, **kw):
    errs, exact = run_side_by_side(spec, steps, **kw)
    report = format_report(errs)
    print(f"\n[{spec.name or 'module'}] per-tensor max|err|/max|ref| (worst over {steps} steps)\n{report}", flush=True)
    assert not exact, exact
    bad = {k: v for k, v in errs.items() if not (v <= TOL)}
    assert not bad, "tensors over the 2e-2 bar:\n" + format_report(bad)


@pytest.mark.parametrize("name", list(SMALL))
def test_small_modules(name):
    spec = copy.deepcopy(SMALL[name])
    spec.name = name
    print(f"case {name}", flush=True)
    _check(spec, steps=2, seed=1)


def test_backward_first_order_of_algorithm_1():
    spec = copy.deepcopy(SMALL["bottom_stack_delay2"])
    spec.name = "backward-first"
    _check(spec, steps=3, seed=2, backward_first=True)


def test_config1_basic_block():
    _check(W.config(1), steps=3, perturb_bn=False)


@pytest.mark.parametrize("idx,n,steps", [(2, 16, 2), (3, 16, 2), (4, 8, 1), (5, 8, 1)])
def test_configs_reduced_batch(idx, n, steps):
    """The benchmark modules at their real layer shapes, with a batch the oracle finishes in seconds."""
    spec = W.config(idx, n=n)
    print(f"case cfg{idx} n={n}", flush=True)
    _check(spec, steps=steps, perturb_bn=False)

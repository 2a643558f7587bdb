"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and its
host logic (descriptor validation, workspace sizing) behaves; no kernel is launched here."""
import ctypes
import os
import re

import pytest

import fdg_workloads as W
from fdg_workloads import Layer, ModuleSpec
from paper_1906_09108_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header, prefix):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_1906_09108_amd import kernels
    lib = binding.load()
    names = sorted(set(_declared("fdg.h", "fdg_") + _declared("fdg_chain.h", "fdg_")))
    assert set(names) == set(binding.EXPORTS)
    knames = _declared("fdg_kernels.h", "fdgk_")
    assert set(knames) == set(kernels.KERNEL_EXPORTS)
    kernels._lib()   # raises if an exported kernel entry has no declared argument types (pointers would be cut to 32 bits)
    for n in names + knames:
        assert getattr(lib, n) is not None


def test_status_strings():
    lib = binding.load()
    assert lib.fdg_status_string(0) == b"ok"
    assert b"queue" in lib.fdg_status_string(4)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10])
def test_workspace_bytes_of_benchmark_configs(idx):
    spec = W.config(idx)
    b = binding.fdg_module_workspace_bytes(spec)
    assert b > 0 and b % 256 == 0
    deeper = W.config(idx)
    deeper.delay += 1
    assert binding.fdg_module_workspace_bytes(deeper) > b      # one more ring slot


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6, 7, 8])
def test_workspace_bytes_when_a_saved_forward_is_its_input(idx):
    """FDG_SAVE_INPUT_AND_REPLAY: one set of intermediates for the module instead of one per ring slot; a slot is the
    weight snapshot plus the fp32 input."""
    spec = W.config(idx)
    full = binding.fdg_module_workspace_bytes_ex(spec, binding.FDG_SAVE_ACTIVATIONS)
    assert full == binding.fdg_module_workspace_bytes(spec)
    replay = binding.fdg_module_workspace_bytes_ex(spec, binding.FDG_SAVE_INPUT_AND_REPLAY)
    assert replay > 0 and replay % 256 == 0
    x_bytes = 4 * spec.n * spec.c_in * spec.h_in * spec.w_in
    if spec.delay >= 1:
        assert replay < full
    else:
        assert replay <= full + x_bytes + 512          # nothing to share with a single slot: only the input copy is added
    deeper = W.config(idx)
    deeper.delay += 1
    step_full = binding.fdg_module_workspace_bytes(deeper) - full
    step_replay = binding.fdg_module_workspace_bytes_ex(deeper, binding.FDG_SAVE_INPUT_AND_REPLAY) - replay
    assert 0 < step_replay < step_full
    shared = binding.fdg_module_workspace_bytes_ex(spec, binding.FDG_SAVE_ACTIVATIONS_CURRENT_WEIGHTS)
    assert shared > 0 and shared % 256 == 0
    assert (shared < full) if spec.delay >= 1 else (shared <= full + 512)   # one weight copy instead of delay + 1
    for bad_mode in (-1, 3, 7):
        assert binding.fdg_module_workspace_bytes_ex(spec, bad_mode) == 0
    lib = binding.load()
    out = ctypes.c_void_p()
    d, keep = binding.make_desc(spec)
    assert lib.fdg_module_create_ex(ctypes.byref(d), 5, None, 0, None, ctypes.byref(out)) == binding.FDG_ERR_INVALID_ARG


def test_invalid_descriptors_are_rejected():
    ok = ModuleSpec(2, 16, 8, 8, [Layer(W.BASIC_POSTACT, 16, 16, 1)])
    assert binding.fdg_module_workspace_bytes(ok) > 0
    for bad in (ModuleSpec(2, 16, 8, 8, [Layer(W.BASIC_POSTACT, 8, 16, 1)]),          # channel mismatch
                ModuleSpec(2, 16, 8, 8, [Layer(W.BASIC_POSTACT, 16, 16, 3)]),         # stride
                ModuleSpec(2, 16, 8, 8, [Layer(W.BASIC_POSTACT, 16, 16, 1)], beta=0.0),
                ModuleSpec(2, 16, 8, 8, [Layer(W.BASIC_POSTACT, 16, 16, 1)], delay=-1),
                ModuleSpec(2, 16, 8, 8, [Layer(W.HEAD_POSTACT, 16), Layer(W.BASIC_POSTACT, 16, 16, 1)]),  # head not last
                ModuleSpec(2, 16, 8, 8, [Layer(W.BASIC_POSTACT, 16, 12, 1)]),         # channels not a multiple of 8
                ModuleSpec(0, 16, 8, 8, [Layer(W.BASIC_POSTACT, 16, 16, 1)]),
                ModuleSpec(2, 16, 8, 8, [Layer(W.BOTTLENECK_POSTACT, 16, 48, 1)]),    # a quarter of 48 is not a multiple of 8
                ModuleSpec(2, 16, 8, 8, [Layer(8, 16, 16, 1)]),                       # no such layer kind
                ModuleSpec(2, 3, 8, 8, [Layer(W.STEM_POOL, 3, 16, 2)], is_bottom=True),  # the stem halves twice: stride 4
                ModuleSpec(2, 3, 8, 8, [Layer(W.STEM_POOL, 3, 16, 4)], is_bottom=False),  # it has no input gradient
                ModuleSpec(2, 16, 8, 8, [Layer(W.INVERTED_RESIDUAL, 16, 16, 4)])):
        assert binding.fdg_module_workspace_bytes(bad) == 0
    bottleneck = ModuleSpec(2, 16, 8, 8, [Layer(W.BOTTLENECK_POSTACT, 16, 64, 2), Layer(W.BOTTLENECK_POSTACT, 64, 64, 1)])
    plain = ModuleSpec(2, 16, 8, 8, [Layer(W.BOTTLENECK_POSTACT, 16, 64, 2)])
    assert binding.fdg_module_workspace_bytes(bottleneck) > binding.fdg_module_workspace_bytes(plain) > 0
    lib = binding.load()
    assert lib.fdg_module_workspace_bytes(None) == 0
    out = ctypes.c_void_p()
    d, keep = binding.make_desc(ok)
    assert lib.fdg_module_create(ctypes.byref(d), None, 0, None, ctypes.byref(out)) == binding.FDG_ERR_INVALID_ARG
    assert lib.fdg_forward(None, None, None, None, None) == binding.FDG_ERR_INVALID_ARG
    assert lib.fdg_update(None, 0.1, None) == binding.FDG_ERR_INVALID_ARG
    lib.fdg_destroy(None)


def test_chain_rejects_bad_arguments_without_a_gpu():
    """No module can be created here (no device memory), so only the argument checks that come first."""
    lib = binding.load()
    assert lib.fdg_chain_mailbox_bytes(None, 2) == 0
    arr = (ctypes.c_void_p * 2)(None, None)
    assert lib.fdg_chain_mailbox_bytes(arr, 2) == 0
    out = ctypes.c_void_p()
    assert lib.fdg_chain_create(arr, 2, None, 0, ctypes.byref(out)) == binding.FDG_ERR_INVALID_ARG
    assert lib.fdg_chain_create(arr, 0, None, 0, ctypes.byref(out)) == binding.FDG_ERR_INVALID_ARG
    assert lib.fdg_chain_step(None, None, None, 0.1, None, None, None) == binding.FDG_ERR_INVALID_ARG
    assert lib.fdg_chain_state(None, None, None, None) == binding.FDG_ERR_INVALID_ARG
    lib.fdg_chain_destroy(None)


def test_learning_rate_schedule_of_section_5a():
    """Section V-A: lr 0.1, divided by 10 at epochs 150, 225 and 275 of 300; 0.01 for the first 3 epochs where the
    paper warms up.  The expected values are the paper's, typed in."""
    f = binding.fdg_lr_schedule
    for epoch, lr in ((0, 0.1), (1, 0.1), (149, 0.1), (150, 0.01), (224, 0.01), (225, 0.001), (274, 0.001), (275, 0.0001),
                      (299, 0.0001)):
        assert f(epoch) == pytest.approx(lr, rel=1e-6), epoch
    for epoch, lr in ((0, 0.01), (2, 0.01), (3, 0.1), (149, 0.1), (150, 0.01), (299, 0.0001)):
        assert f(epoch, 3) == pytest.approx(lr, rel=1e-6), epoch
    assert f(-5) == pytest.approx(0.1, rel=1e-6)



def test_build_refuses_scratch_in_kernels_with_hand_counted_waits():
    """The build reads the compiler's resource-usage remarks and fails when a kernel whose vmcnt waits are counted by hand
    uses scratch memory beyond what is listed for it (a spill or a table moved to memory inside the counted loop adds loads
    to that count); the parser on a sample."""
    from paper_1906_09108_amd.build import NO_SCRATCH, scratch_users
    sample = """x.hip:1:1: remark: Function Name: _ZN3fdg23conv_gather_pipe_kernelILi160ELi4ELb0EEEvNS_14GatherConvArgsEii [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     ScratchSize [bytes/lane]: 64 [-Rpass-analysis=kernel-resource-usage]
x.hip:9:1: remark: Function Name: _ZN3fdg17conv_patch_kernelILi160ELi160ELi5ELb0EEEvNS_14GatherConvArgsEii [-Rpass-analysis=kernel-resource-usage]
x.hip:9:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
x.hip:20:1: remark: Function Name: _ZN3fdg19wgrad_reduce_kernelEP15HIP_vector_typeIfLj4EE [-Rpass-analysis=kernel-resource-usage]
x.hip:20:1: remark:     ScratchSize [bytes/lane]: 16 [-Rpass-analysis=kernel-resource-usage]
"""
    bad = scratch_users(sample, NO_SCRATCH["conv_wide_kernels.hip"])
    assert bad == [("_ZN3fdg23conv_gather_pipe_kernelILi160ELi4ELb0EEEvNS_14GatherConvArgsEii", 64)]

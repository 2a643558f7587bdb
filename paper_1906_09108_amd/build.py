"""Builds libfdg.so (the C-ABI library) from the HIP sources with hipcc for gfx950."""
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfdg.so")
SOURCES = ["conv_kernels.hip", "conv_wide_kernels.hip", "conv_narrow_kernels.hip", "stream_kernels.hip", "layer_kernels.hip", "fdg_module.hip", "fdg_chain.hip", "kernel_api.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


# Kernels whose main loops count outstanding loads by hand (s_waitcnt vmcnt(n), n worked out from the loads issued after the
# one waited for): a register spill or a table the compiler moves to scratch memory inside such a loop adds scratch loads to
# the count, every wait then holds for longer than intended and the pipeline the loop was built for is gone -- without any
# error (it happened once: a select between two per-lane tables became a table in scratch, five scratch loads per step).
# The build therefore asks the compiler for each kernel's resource usage and fails if one of these uses more scratch than
# listed here (conv_patch256_kernel spills a few registers in its output stage, after the counted loop: known and harmless).
NO_SCRATCH = {"conv_wide_kernels.hip": {"conv_patch_kernel": 0, "conv_patch256_kernel": 32, "conv_gather_pipe_kernel": 0,
                                        "conv_wgrad128w8_kernel": 0, "conv_wgrad_tall_kernel": 0, "conv_wgrad_dma_kernel": 0}}


def scratch_users(remarks: str, allowed: dict) -> list:
    """(kernel, bytes per lane) of the kernels named in `allowed` (name -> bytes per lane it may use) that the compiler's
    resource-usage remarks give more scratch than that."""
    bad, current = [], None
    for line in remarks.splitlines():
        if "remark: Function Name:" in line:
            current = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line and current:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            for name, limit in allowed.items():
                if re.search(r"\d" + name + "I", current) and size > limit:   # mangled: <length><name>I<template arguments>
                    bad.append((current, size))
    return bad


def build(verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        objs.append(obj)
        extra = ["-Rpass-analysis=kernel-resource-usage"] if src in NO_SCRATCH else []
        cmd = [hipcc] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, cmd, pr in procs:
        out, _ = pr.communicate()
        if src in NO_SCRATCH:
            bad = scratch_users(out, NO_SCRATCH[src])
            if bad:
                raise RuntimeError(f"{src}: scratch memory in kernels with hand-counted waits (kernel, bytes per lane): {bad}")
            out = "\n".join(l for l in out.splitlines() if "kernel-resource-usage" not in l and not l.lstrip().startswith(("|", "^")) and
                            not (l[:1].isspace() and l.strip()[:1].isdigit()))
        out = "\n".join(l for l in out.splitlines() if "not a recognized feature" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))

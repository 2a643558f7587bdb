#!/usr/bin/env python3
"""Throughput of one FDG module step on one MI355X.

A step is one pass of the whole hot path of a module worker: forward on the newest batch, delayed
backward (with gradient shrinking) on the oldest saved batch, momentum-SGD update -- the three calls of
the C ABI -- with the history ring in steady state and every input already resident in HBM.

Prints ONE JSON line: images/s of the step, the roofline position of the kernel class that takes most of
the step (timed with HIP events on the stream the kernels run on, during a second pass over the same
steps), and the CPU oracle timed on this machine's host cores on a bounded sample (a reported baseline).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E



# the sources that define the kernels whose traffic profiles/hbm_traffic.json holds (the wide convolution kernels and
# their output stage)
TRAFFIC_SOURCES = ("conv_wide_kernels.hip", "conv_common.h")


def library_source_sha() -> str:
    """sha256 over the sources of the measured kernels: what a stored counter measurement is valid for."""
    import hashlib
    h = hashlib.sha256()
    for name in TRAFFIC_SOURCES:
        h.update(name.encode())
        h.update(open(os.path.join(ROOT, "paper_1906_09108_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(config: int, kernel: str):
    """HBM-side bytes per launch of `kernel` (FETCH_SIZE + WRITE_SIZE of rocprofv3 --pmc, each scaled by what the same
    counter reads for a plain copy of known size) from profiles/hbm_traffic.json -- or None when that file was measured
    on other sources than the ones this run uses (it is then stale and says nothing about this build)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        return None, "not measured"
    if rec.get("library_source_sha") != library_source_sha():
        return None, "stale: profiles/hbm_traffic.json was measured on other kernel sources"
    v = rec.get("bytes_per_launch", {}).get(f"cfg{config}|{kernel}")
    return (v, rec.get("how", "")) if v is not None else (None, "not measured for this kernel")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)     # about half a second of the headline step: the clock under load has settled
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 1..10 (default 4: WRN-28-10 top module)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--two-streams", action="store_true",
                    help="forward on one stream, delayed backward + update on another: the default for modules with delay >= 1 "
                         "in the stored form (the two touch different saved forwards and overlap on the GPU: the decoupling "
                         "the method is about); an error where it does not apply")
    ap.add_argument("--one-stream", action="store_true", help="everything on one stream also where the delay is >= 1")
    ap.add_argument("--graph", action="store_true",
                    help="record the step into HIP graphs (one per position of the history ring) and time their replay")
    ap.add_argument("--replay", action="store_true",
                    help="FDG_SAVE_INPUT_AND_REPLAY: a saved forward is its input and weight snapshot; the backward runs the forward again")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run 3 plain device copies of 1 GiB (float32): the known traffic a profiler's HBM counters "
                         "are scaled by")
    ap.add_argument("--no-overlap", action="store_true",
                    help="weight gradients on the caller's stream (fdg_overlap_enable(0)): for an external profiler's kernel "
                         "trace, in which a kernel's duration should be its own")
    ap.add_argument("--copy-reference", action="store_true",
                    help="instead of the module step: time plain device copies (torch's copy kernel) of the sizes the "
                         "batch-norm passes of the configuration move; what a pass over a tensor of that size can reach")
    ap.add_argument("--cpu-sample-batch", type=int, default=0, help="batch of the oracle sample (0 = pick by config)")
    ap.add_argument("--chain", type=int, default=0, metavar="K",
                    help="instead of the module step: time one iteration of Algorithm I for the whole WRN-28-10 cut "
                         "into K modules that share this GPU (one stream each); prints its own JSON line")
    return ap.parse_args()


def cpu_baseline(idx: int, sample_batch: int):
    """The oracle as it stands (fp32 definition), one step of the same layers at a reduced batch."""
    import numpy as np
    import fdg_workloads as W
    from oracle import fdg_oracle
    n = sample_batch or {1: 128, 2: 128, 3: 128, 4: 128, 5: 32, 6: 64, 7: 32, 8: 32, 9: 32, 10: 64}[idx]   # about 10-30 s of oracle time
    spec = W.config(idx, n=n)
    spec.delay = 0
    m = fdg_oracle.OracleModule(spec, np.float32, storage="fp32")
    m.set_params(W.make_params(spec))
    x, labels, g = W.make_input(spec, 0), W.make_labels(spec, 0), W.make_grad_out(spec, 0)
    t0 = time.perf_counter()
    m.forward(x, labels)
    m.backward_delayed(g)
    m.update(spec.lr)
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "images/s", "cores": fdg_oracle.num_threads(), "kind": "oracle",
            "sample": f"same layers at batch {n} (of {W.config(idx).n}), 1 step forward+backward+update, {dt:.1f} s"}


def copy_reference(args):
    """A batch-norm pass reads a tensor and writes one of the same size; these tensors are small against the chip (10 to
    40 MB), so the time of a launch is mostly ramp-up and the latency of one round of memory accesses.  A plain copy of
    the same bytes is the yardstick: what the memory system gives ANY kernel that moves so little."""
    import torch
    import fdg_workloads as W
    spec = W.config(args.config)
    dev = torch.device("cuda:0")
    sizes = sorted({2 * n * c * h * w for (n, c, h, w) in spec.activation_shapes()})   # bf16 NHWC activations
    sizes += [4 * sizes[-1], 16 * sizes[-1]]
    out = []
    for nbytes in sizes:
        n = nbytes // 2
        # a ring of buffers, so that a copy does not find its source in L2 from the copy before
        ring = [(torch.ones(n, dtype=torch.bfloat16, device=dev), torch.empty(n, dtype=torch.bfloat16, device=dev)) for _ in range(8)]
        for s, d in ring:
            d.copy_(s)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(40)]
        for i, (a, b) in enumerate(evs):
            s, d = ring[i % 8]
            a.record()
            d.copy_(s)
            b.record()
        torch.cuda.synchronize()
        us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)[20]
        out.append({"read_MB": nbytes / 1e6, "written_MB": nbytes / 1e6, "median_us": us, "GB/s": 2 * nbytes / us * 1e-3})
        del ring
    print(json.dumps({"what": "plain device copies of the sizes of %s's activations (bf16), event-timed" % spec.name, "copies": out}))


def chain_bench(args):
    """Whole-network iteration of Algorithm I, K modules on K streams of this one GPU (the paper runs them on K
    GPUs).  Not the headline metric: a second, reported figure."""
    import torch
    import fdg_workloads as W
    from paper_1906_09108_amd import FdgChain
    specs = W.wrn_28_10_chain(args.chain)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    chain = FdgChain(specs, dev)
    for k, m in enumerate(chain.modules):
        m.set_params(W.make_params(specs[k], k))
    pool = 4
    xs = [torch.from_numpy(W.make_input(specs[0], t)).to(dev) for t in range(pool)]
    labels = [torch.from_numpy(W.make_labels(specs[-1], t)).to(dev) for t in range(pool)]
    lr = 0.01
    warm = max(args.warmup, 2 * args.chain)            # every module's history is in steady state after 2K iterations
    for i in range(warm):
        chain.step(xs[i % pool], labels[i % pool], lr)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        chain.step(xs[(warm + i) % pool], labels[(warm + i) % pool], lr)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    loss = float(chain.top_y[0].item())
    flops = sum(W.conv_flops(sp) for sp in specs)
    chain.close()
    if not (loss == loss and abs(loss) < 1e30):
        print("non-finite loss", file=sys.stderr)
        sys.exit(1)
    print(json.dumps({
        "metric": "images/sec, one iteration of Algorithm I over all K modules (whole network) on one GPU",
        "value": specs[0].n * args.steps / elapsed, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": warm,
        "ms_per_step": 1e3 * elapsed / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "WRN-28-10, K=%d modules sharing one GPU" % args.chain, "batch": specs[0].n,
                   "delays": [sp.delay for sp in specs], "params": sum(W.param_count(sp) for sp in specs),
                   "useful_conv_gflop_per_step": flops / 1e9},
        "step_tflops": flops / (elapsed / args.steps) / 1e12,
        "paper_context": "FDG K=2 WRN-28-10: 354.56 images/s on 2x 1080Ti, BP 188.16 on 1x (Table VII); other hardware",
    }))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one module worker on ONE GPU; this build has no multi-GPU path "
              f"(got --gpus {args.gpus}). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if args.chain:
        return chain_bench(args)
    if args.copy_reference:
        return copy_reference(args)
    import numpy as np
    import torch
    import fdg_workloads as W
    from paper_1906_09108_amd import FdgModule

    spec = W.config(args.config)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    mod = FdgModule(spec, dev, save_mode=1 if args.replay else 0)
    mod.set_params(W.make_params(spec))
    if args.no_overlap:
        mod.overlap_enable(False)

    # a small pool of resident inputs, cycled, so consecutive steps do not re-read the same lines
    pool = 4
    xs = [torch.from_numpy(W.make_input(spec, t)).to(dev) for t in range(pool)]
    labels = [None if not spec.is_top else torch.from_numpy(W.make_labels(spec, t)).to(dev) for t in range(pool)]
    gs = [None if spec.is_top else torch.from_numpy(W.make_grad_out(spec, t)).to(dev) for t in range(pool)]
    y = mod.new_output()
    grad_in = None if spec.is_bottom else torch.empty(spec.input_shape(), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    lr = 0.01   # small enough that the synthetic noise gradients do not blow the weights up over many steps

    for t in range(spec.delay):                       # fill the history ring
        mod.forward(xs[t % pool], labels[t % pool], y, stream)

    two = bool(args.two_streams) or (spec.delay >= 1 and not args.replay and not args.graph and not args.one_stream)
    if two and (spec.delay < 1 or args.replay):
        print("--two-streams needs a module with delay >= 1 in the stored form", file=sys.stderr)
        sys.exit(2)
    if two and args.graph:
        print("--graph records a step on one stream; it is not combined with --two-streams", file=sys.stderr)
        sys.exit(2)
    if two:
        s_fwd, s_bwd = torch.cuda.Stream(), torch.cuda.Stream()
        ev_fwd, ev_upd = torch.cuda.Event(), torch.cuda.Event()
        torch.cuda.synchronize()
        ev_upd.record(s_bwd)

    def step_one(i):
        mod.forward(xs[i % pool], labels[i % pool], y, stream)
        mod.backward_delayed(gs[i % pool], grad_in, stream)
        mod.update(lr, stream)

    def step(i):
        if two:
            s_fwd.wait_event(ev_upd)                      # the forward reads the weights of the last update
            mod.forward(xs[i % pool], labels[i % pool], y, s_fwd)
            ev_fwd.record(s_fwd)
            mod.backward_delayed(gs[i % pool], grad_in, s_bwd)   # the oldest saved forward: independent of the one above
            s_bwd.wait_event(ev_fwd)                      # the update must not move the weights under the forward's snapshot
            mod.update(lr, s_bwd)
            ev_upd.record(s_bwd)
            return
        mod.forward(xs[i % pool], labels[i % pool], y, stream)
        mod.backward_delayed(gs[i % pool], grad_in, stream)
        mod.update(lr, stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.graph:
        # One graph per ring position (the slot pointers of a step are fixed in it); the replays continue the cycle
        # the recording went through.  The library allocates nothing, clears memory with kernels (no memset nodes)
        # and forks / joins its own second stream with events, so a whole step records as it is.
        period = spec.delay + 1
        s_main = torch.cuda.Stream()
        graphs = []
        for ph in range(period):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s_main):
                i = args.warmup + ph
                mod.forward(xs[i % pool], labels[i % pool], y, s_main)
                mod.backward_delayed(gs[i % pool], grad_in, s_main)
                mod.update(lr, s_main)
            graphs.append(g)
        torch.cuda.synchronize()

        def step(i):   # noqa: F811 -- from here on a step is a replay
            graphs[(i - args.warmup) % period].replay()
        for i in range(args.warmup, args.warmup + period):
            step(i)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    value = spec.n * args.steps / elapsed
    if not bool(torch.isfinite(y).all()):
        print("non-finite module output", file=sys.stderr)
        sys.exit(1)

    # second pass (at most 40 steps) with per-class HIP events (eager: the profiler's events are not part of a
    # recorded graph)
    step = step_one         # per-kernel times are taken with everything on one stream: a kernel's time is then its own
    torch.cuda.synchronize()
    prof_steps = min(args.steps, 40)
    if args.graph:
        # The replays advanced the ring on the device while the library's host counters stayed where the recording
        # left them: an eager step of THIS module would pop a slot that is not the oldest saved forward.  The
        # profile is therefore taken on a fresh module of the same shape (same kernels, same sizes).
        ws_bytes = mod.workspace_bytes
        mod.close()
        mod = FdgModule(spec, dev, save_mode=1 if args.replay else 0)
        mod.set_params(W.make_params(spec))
        for t in range(spec.delay):
            mod.forward(xs[t % pool], labels[t % pool], y, stream)
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
    mod.profile_enable(True)
    for i in range(prof_steps):
        step(args.warmup + args.steps + i)
    entries = mod.profile_read()
    mod.profile_enable(False)
    total_ms = sum(e["total_ms"] for e in entries)

    def merged(key):
        out = {}
        for e in entries:
            k = key(e)
            acc = out.setdefault(k, dict(calls=0, total_ms=0.0, flops=0.0, bytes=0.0))
            for f in ("calls", "total_ms", "flops", "bytes"):
                acc[f] += e[f]
        return out

    prof = merged(lambda e: e["name"])                       # per kernel class
    kernels = merged(lambda e: e["kernel"] or e["name"])     # per kernel and layer shape (forward and data
    #                                                          gradient of a stride-1 3x3 layer run the same kernel)
    name, dom = max(kernels.items(), key=lambda kv: kv[1]["total_ms"])
    avg_ms = dom["total_ms"] / dom["calls"]
    if dom["flops"] > 0:
        achieved = dom["flops"] / dom["calls"] / (avg_ms * 1e-3) / 1e12
        roofline = {"kernel": name, "bound": "mfma", "achieved": achieved, "peak": PEAK_MFMA_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / PEAK_MFMA_BF16_TFLOPS}
    else:
        achieved = dom["bytes"] / dom["calls"] / (avg_ms * 1e-3) / 1e9
        roofline = {"kernel": name, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS}
    roofline.update({"avg_launch_ms": avg_ms, "calls_per_step": dom["calls"] / prof_steps,
                     "share_of_step": dom["total_ms"] / total_ms,
                     "algorithmic_flops_per_launch": dom["flops"] / dom["calls"],
                     "algorithmic_bytes_per_launch": dom["bytes"] / dom["calls"]})
    roofline["traffic"], roofline["traffic_source"] = measured_traffic(args.config, name)
    classes = {k: {"ms_per_step": v["total_ms"] / prof_steps, "calls_per_step": v["calls"] / prof_steps,
                   "TFLOP/s": (v["flops"] / (v["total_ms"] * 1e-3) / 1e12) if v["flops"] else None,
                   "GB/s": v["bytes"] / (v["total_ms"] * 1e-3) / 1e9}
               for k, v in sorted(prof.items(), key=lambda kv: -kv[1]["total_ms"])}
    per_kernel = {k: {"ms_per_step": v["total_ms"] / prof_steps, "calls_per_step": v["calls"] / prof_steps,
                      "avg_us": 1e3 * v["total_ms"] / v["calls"],
                      "TFLOP/s": (v["flops"] / (v["total_ms"] * 1e-3) / 1e12) if v["flops"] else None}
                  for k, v in sorted(kernels.items(), key=lambda kv: -kv[1]["total_ms"]) if v["flops"]}
    mod.close()

    out = {
        "metric": "images/sec per FDG module step (fwd+delayed bwd+update)",
        "value": value, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": spec.name, "batch": spec.n, "delay": spec.delay, "beta": spec.beta,
                   "saved_forward": "input + weight snapshot, replayed by the backward" if args.replay else "activations",
                   "streams": "forward on one, delayed backward + update on another" if two else "one",
                   "launch": "HIP graph replay" if args.graph else "eager", "profiled_steps": prof_steps,
                   "workspace_MiB": mod.workspace_bytes / 2 ** 20,
                   "params": W.param_count(spec), "useful_conv_gflop_per_step": W.conv_flops(spec) / 1e9},
        "step_tflops": W.conv_flops(spec) / (ms_per_step * 1e-3) / 1e12,
        "roofline": roofline,
        "kernel_classes": classes,
        "conv_kernels": per_kernel,
        "paper_context": "FDG K=2 WRN-28-10: 354.56 images/s on 2x 1080Ti, BP 188.16 on 1x (Table VII); other hardware, whole system",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, args.cpu_sample_batch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

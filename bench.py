#!/usr/bin/env python3
"""Benchmark of the per-block fused mixed-precision Adam step on one MI355X.

A "step" is one pass of the whole hot path over one block whose inputs are already resident in
HBM: lohan_grad_sqnorm (one 2 B/element read of the fp16 gradients giving the overflow flag and
the squared norm) followed by lohan_adam_block_step with LOHAN_FLAG_PRECHECKED (the 28 B/element
stream: unscale, Adam/AdamW with bias correction, fp32 write-back, bf16 copy).  The metric is
Adam-updated elements per second; the roofline object prices the dominant kernel
(k_adam_block_step, 28 algorithmic bytes per element) against the 8 TB/s HBM peak using HIP events
recorded on the launch stream inside the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gpt13b|gpt175b|gpt_h768|
                     stream13b|offload13b|shapes|models|gpt13b_oop|gpt175b_oop|ring13b]

The *_oop workloads time lohan_adam_block_step_out_of_place instead: the overflow test fused into
a single 28 B/element pass between two sets of state (not the default: it doubles the state).

Prints ONE JSON line.  There is no multi-GPU path: the step is elementwise and would shard by
contiguous element ranges, but this build runs on one GPU only.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
ADAM_BYTES_PER_ELEM = 28        # read g16 2 + p 4 + m 4 + v 4, write p 4 + m 4 + v 4 + bf16 2
REDUCE_BYTES_PER_ELEM = 2       # one read of g16

# HBM bytes per k_adam_block_step launch measured with two rocprofv3 --pmc runs of this script
# (FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for a plain 1 GiB copy:
# factor 2.000 and 1.000 on gfx950).  Summary: profiles/k_adam_block_step_gpt13b_hbm_traffic.md.
MEASURED_TRAFFIC_BYTES = {"gpt13b": 8601691 * 1024,      # profiles/..._gpt13b_hbm_traffic.md
                          "gpt175b": 49545515 * 1024,    # profiles/..._gpt175b_trace_and_traffic.md
                          "gpt13b_oop": 8601956 * 1024}  # profiles/k_adam_block_step_oop_gpt13b_...


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="gpt13b",
                    choices=["gpt13b", "gpt175b", "gpt_h768", "stream13b", "offload13b", "shapes",
                             "gpt13b_oop", "gpt175b_oop", "models", "ring13b"])
    ap.add_argument("--variant", type=int, default=None, help="kernel launch-shape override")
    ap.add_argument("--wgs-per-cu", type=int, default=0)
    ap.add_argument("--waves-per-cu", type=int, default=-1,
                    help="occupancy throttle override (0 = none, -1 = built-in default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--compare-allocator", action="store_true",
                    help="also time the update kernel on the five separate torch allocations "
                         "before the block is moved into the library's placement")
    ap.add_argument("--placement", choices=["library", "allocator"], default="library",
                    help="gpt13b/gpt175b/gpt_h768/shapes/models: where the blocks' arrays sit -- at "
                         "the offsets lohan_model_placement gives inside one slab (default), or "
                         "in five separate torch allocations")
    ap.add_argument("--blocks", type=int, default=None,
                    help="stream13b: number of blocks (default 40); offload13b: default 6; "
                         "ring13b: default 8")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy before the steps, so that a "
                         "rocprofv3 --pmc run of this command holds a kernel of known traffic")
    return ap.parse_args()


def cpu_baseline(block, wl, sample_elems=1 << 27):
    """Time the CPU oracle, as it stands, on the first `sample_elems` elements of the same block
    (copied to the host before the timed GPU region)."""
    import numpy as np
    from oracle import reference as oracle
    from paper_2403_06504_amd import synthetic_inputs as synth

    k = min(sample_elems, wl.n)
    host = {name: synth.to_numpy_bits(block[name][:k]) for name in ("p", "m", "v", "g", "p16")}
    hy = wl.hyper()
    threads = min(oracle.max_threads(), 16 if os.environ.get("OMP_NUM_THREADS") is None
                  else int(os.environ["OMP_NUM_THREADS"]))
    threads = max(1, threads)

    def time_step(nthreads, reps):
        best = float("inf")
        for r in range(reps):
            t0 = time.perf_counter()
            f = oracle.adam_block_step(host["p"], host["m"], host["v"], host["g"], host["p16"],
                                       nthreads=nthreads, **dict(hy, step=hy["step"] + r))
            best = min(best, time.perf_counter() - t0)
            assert f == 0
        return best

    t_multi = time_step(threads, 5)
    t_single = time_step(1, 3)
    t0 = time.perf_counter()
    oracle.grad_sqnorm(host["g"], wl.loss_scale)
    t_norm = time.perf_counter() - t0
    return {
        "value": k / t_multi, "unit": "elements/s", "cores": threads, "kind": "oracle",
        "sample": f"first {k} elements of the {wl.name} block; oracle Adam block step (overflow "
                  f"check + update + bf16 copy), best of 5 on {threads} OpenMP threads",
        "single_thread_value": k / t_single,
        "single_thread_with_sqnorm_value": k / (t_single + t_norm),
        "host_cpus": os.cpu_count(),
    }


def placed_views(n, torch, lohan, dev):
    """One slab with room for a full group of n-element blocks at the offsets
    lohan_model_placement gives (the layout a framework holding the whole model would use), and
    views of block 0's five arrays in it.  Allocate it before anything else, as a framework
    would: a slab carved out of fresh memory keeps the lanes' relative position physically.
    Returns (views, slab, description)."""
    gib = 1 << 30
    offsets, slab_bytes, align, group = lohan.lohan_model_placement(n)     # one full group
    slab = torch.empty(slab_bytes + align, dtype=torch.uint8, device=dev)
    start = (-slab.data_ptr()) % align
    spec = {"p": ("param_fp32", torch.float32), "m": ("exp_avg", torch.float32),
            "v": ("exp_avg_sq", torch.float32), "g": ("grad_fp16", torch.float16),
            "p16": ("param_bf16", torch.bfloat16)}
    views = {}
    for k, (field, dtype) in spec.items():
        off = start + offsets[0][field]
        nbytes = n * torch.empty(0, dtype=dtype).element_size()
        views[k] = slab[off: off + nbytes].view(dtype)
    what = (f"block 0 of a {group}-block group laid out by lohan_model_placement "
            f"({slab_bytes / gib:.2f} GiB slab)")
    return views, slab, what


def adam_kernel_only_ms(block, wl, torch, lohan, reps):
    """Average duration of the update kernel alone on `block` (prechecked, flag 0)."""
    flag = torch.zeros(1, dtype=torch.int32, device=block["p"].device)
    hy = wl.hyper()

    def call(t):
        lohan.lohan_adam_block_step(block["p"], block["m"], block["v"], block["g"], block["p16"],
                                    wl.n, hy["lr"], hy["beta1"], hy["beta2"], hy["eps"],
                                    hy["weight_decay"], t, hy["loss_scale"], flag,
                                    lohan.LOHAN_FLAG_PRECHECKED, None)

    for w in range(3):
        call(hy["step"] + w)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for k in range(reps):
        call(hy["step"] + 3 + k)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def bench_block(args, torch, lohan, synth):
    wl = synth.WORKLOADS[args.workload]
    dev = "cuda:0"
    n = wl.n
    placement = "five separate allocations of torch's caching allocator"
    allocator_ms = None
    if args.placement == "library":
        views, slab, placement = placed_views(n, torch, lohan, dev)
    block = synth.make_block(wl, seed=0, device=dev)
    if args.placement == "library":
        if args.compare_allocator:
            allocator_ms = adam_kernel_only_ms(block, wl, torch, lohan, min(args.steps, 20))
        for k in views:
            views[k].copy_(block[k])
        block = views
        torch.cuda.empty_cache()
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    sqnorm = torch.zeros(1, dtype=torch.float64, device=dev)
    ws = lohan.new_workspace(dev)
    hy = wl.hyper()

    base = None if args.no_cpu_baseline else cpu_baseline(block, wl)

    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)        # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def one_step(t, ev=None):
        lohan.lohan_grad_sqnorm(block["g"], n, wl.loss_scale, sqnorm, flag, ws)
        if ev is not None:
            ev[0].record()
        lohan.lohan_adam_block_step(block["p"], block["m"], block["v"], block["g"], block["p16"],
                                    n, hy["lr"], hy["beta1"], hy["beta2"], hy["eps"],
                                    hy["weight_decay"], t, hy["loss_scale"], flag,
                                    lohan.LOHAN_FLAG_PRECHECKED, None)
        if ev is not None:
            ev[1].record()

    for w in range(args.warmup):
        one_step(hy["step"] + w)
    torch.cuda.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True),
               torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        events[k][2].record()
        one_step(hy["step"] + args.warmup + k, events[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    assert int(flag.cpu().item()) == 0, "synthetic gradients must not overflow"
    adam_all = sorted(e[0].elapsed_time(e[1]) for e in events)
    adam_ms = sum(adam_all) / args.steps
    reduce_ms = sum(e[2].elapsed_time(e[0]) for e in events) / args.steps
    ms_per_step = elapsed * 1e3 / args.steps
    achieved = ADAM_BYTES_PER_ELEM * n / (adam_ms * 1e-3) / 1e9
    out = {
        "metric": "adam_updated_elements_per_sec",
        "value": n / (elapsed / args.steps),
        "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: one GPT block, n={n} elements "
                               f"(fp32 p/m/v, fp16 grads x loss scale {wl.loss_scale:g}, "
                               f"bf16 copy), AdamW step {wl.step}",
                   "elements": n, "bytes_per_element_step": 30, "placement": placement,
                   "launch_config": list(lohan.lohan_tuning_get_launch_config())},
        "step_hbm_gbps": (ADAM_BYTES_PER_ELEM + REDUCE_BYTES_PER_ELEM) * n /
                         (elapsed / args.steps) / 1e9,
        "roofline": {"kernel": "k_adam_block_step", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name), "avg_launch_ms": adam_ms,
                     "median_launch_ms": adam_all[len(adam_all) // 2],
                     "min_launch_ms": adam_all[0],
                     "algorithmic_bytes_per_launch": ADAM_BYTES_PER_ELEM * n},
        "reduce_kernel": {"kernel": "k_grad_reduce+k_grad_finalize", "avg_ms": reduce_ms,
                          "achieved_gbps": REDUCE_BYTES_PER_ELEM * n / (reduce_ms * 1e-3) / 1e9},
        "cpu_baseline": base,
    }
    if allocator_ms is not None:
        gbps = ADAM_BYTES_PER_ELEM * n / (allocator_ms * 1e-3) / 1e9
        out["allocator_placement"] = {
            "note": "the same kernel on five separate torch allocations, measured in this run "
                    "before the block was moved into the library's placement",
            "avg_launch_ms": allocator_ms, "achieved": gbps, "frac": gbps / HBM_PEAK_GBPS}
    return out


def bench_block_oop(args, torch, lohan, synth):
    """One call of the out-of-place step per "step"; the two state sets swap roles every step, as
    a caller does after reading flag == 0."""
    wl = synth.WORKLOADS[args.workload[:-len("_oop")]]
    dev = "cuda:0"
    block = synth.make_block(wl, seed=0, device=dev)
    n = wl.n
    sets = [{k: block[k] for k in ("p", "m", "v", "p16")},
            {k: torch.empty_like(block[k]) for k in ("p", "m", "v", "p16")}]
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    hy = wl.hyper()

    def one_step(k, t):
        a, b = sets[k & 1], sets[(k & 1) ^ 1]
        lohan.lohan_adam_block_step_out_of_place(
            a["p"], a["m"], a["v"], block["g"], b["p"], b["m"], b["v"], b["p16"], n, hy["lr"],
            hy["beta1"], hy["beta2"], hy["eps"], hy["weight_decay"], t, hy["loss_scale"], flag, 0)

    for w in range(args.warmup):
        one_step(w, hy["step"] + w)
    torch.cuda.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        events[k][0].record()
        one_step(args.warmup + k, hy["step"] + args.warmup + k)
        events[k][1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert int(flag.cpu().item()) == 0, "synthetic gradients must not overflow"
    all_ms = sorted(e[0].elapsed_time(e[1]) for e in events)
    call_ms = sum(all_ms) / args.steps
    achieved = ADAM_BYTES_PER_ELEM * n / (call_ms * 1e-3) / 1e9
    return {
        "metric": "adam_updated_elements_per_sec",
        "value": n / (elapsed / args.steps), "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}, out-of-place step with the overflow test fused in: "
                               f"n={n} elements, two sets of fp32 p/m/v and of the bf16 copy",
                   "elements": n, "bytes_per_element_step": 28,
                   "launch_config": list(lohan.lohan_tuning_get_launch_config())},
        "step_hbm_gbps": ADAM_BYTES_PER_ELEM * n / (elapsed / args.steps) / 1e9,
        "roofline": {"kernel": "k_adam_block_step_oop (events also span the one-lane flag clear)",
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload),
                     "avg_launch_ms": call_ms, "median_launch_ms": all_ms[len(all_ms) // 2],
                     "min_launch_ms": all_ms[0],
                     "algorithmic_bytes_per_launch": ADAM_BYTES_PER_ELEM * n},
        "cpu_baseline": None,
    }


def bench_ring(args, torch, lohan, synth):
    """Eight 13B-shaped blocks in nine slots (lohan_ring_*): every step is one single-pass
    out-of-place update from the block's slot into the spare slot, committed on the device.  A
    "step" is one block; the blocks are taken round robin, highest index first."""
    wl = synth.WORKLOADS["gpt13b"]
    dev = "cuda:0"
    n, nblocks = wl.n, args.blocks or 8
    offsets, slab_bytes, align, _ = lohan.lohan_model_placement(n, nblocks + 1)
    slab = torch.empty(slab_bytes + align, dtype=torch.uint8, device=dev)
    start = (-slab.data_ptr()) % align

    def view(slot, field, dtype, width):
        off = start + offsets[slot][field]
        return slab[off: off + n * width].view(dtype)

    slots, grads = [], []
    for s_ in range(nblocks + 1):
        slot = (view(s_, "param_fp32", torch.float32, 4), view(s_, "exp_avg", torch.float32, 4),
                view(s_, "exp_avg_sq", torch.float32, 4), view(s_, "param_bf16", torch.bfloat16, 2))
        slots.append(slot)
        if s_ < nblocks:
            src = synth.make_block(wl, seed=s_, device=dev)
            for dst, k in zip(slot, ("p", "m", "v", "p16")):
                dst.copy_(src[k])
            g = view(s_, "grad_fp16", torch.float16, 2)
            g.copy_(src["g"])
            grads.append(g)
            del src
    ring = torch.empty(lohan.lohan_ring_bytes(nblocks), dtype=torch.uint8, device=dev)
    lohan.lohan_ring_init(ring, slots, n)
    hy = wl.hyper()

    def one_step(k):
        b = nblocks - 1 - (k % nblocks)
        lohan.lohan_ring_adam_block_step(ring, nblocks, b, grads[b], n, hy["lr"], hy["beta1"],
                                         hy["beta2"], hy["eps"], hy["weight_decay"],
                                         hy["step"] + k // nblocks, hy["loss_scale"], 0)

    for w in range(args.warmup):
        one_step(w)
    torch.cuda.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        events[k][0].record()
        one_step(args.warmup + k)
        events[k][1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    slot_of, spare, skipped = lohan.lohan_ring_read(ring, nblocks)
    assert skipped == [0] * nblocks, "synthetic gradients must not overflow"
    assert sorted(slot_of + [spare]) == list(range(nblocks + 1))
    all_ms = sorted(e[0].elapsed_time(e[1]) for e in events)
    call_ms = sum(all_ms) / args.steps
    achieved = ADAM_BYTES_PER_ELEM * n / (call_ms * 1e-3) / 1e9
    return {
        "metric": "adam_updated_elements_per_sec",
        "value": n / (elapsed / args.steps), "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"ring13b: {nblocks} blocks of n={n} elements in {nblocks + 1} "
                               "slots, single-pass out-of-place steps committed on the device",
                   "elements": n, "bytes_per_element_step": 28,
                   "extra_state_fraction": 1.0 / nblocks,
                   "launch_config": list(lohan.lohan_tuning_get_launch_config())},
        "step_hbm_gbps": ADAM_BYTES_PER_ELEM * n / (elapsed / args.steps) / 1e9,
        "roofline": {"kernel": "k_adam_ring_step (events also span the one-lane commit)",
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                     "avg_launch_ms": call_ms, "median_launch_ms": all_ms[len(all_ms) // 2],
                     "min_launch_ms": all_ms[0],
                     "algorithmic_bytes_per_launch": ADAM_BYTES_PER_ELEM * n},
        "cpu_baseline": None,
    }


def bench_stream(args, torch, lohan, synth):
    """13B-shaped model stream: blocks issued one at a time, last block first, alternating two
    side streams, each behind the event of a synthetic bf16 backward GEMM on the main stream."""
    wl = synth.WORKLOADS["gpt13b"]
    dev = "cuda:0"
    nblocks = args.blocks or 40
    n = wl.n
    blocks = [synth.make_block(wl, seed=i, device=dev) for i in range(nblocks)]
    flags = [torch.zeros(1, dtype=torch.int32, device=dev) for _ in range(nblocks)]
    norms = [torch.zeros(1, dtype=torch.float64, device=dev) for _ in range(nblocks)]
    wss = [lohan.new_workspace(dev)
           for _ in range(2)]
    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    a = torch.randn(2048, 5120, device=dev, dtype=torch.bfloat16)
    b = torch.randn(5120, 20480, device=dev, dtype=torch.bfloat16)
    hy = wl.hyper()
    main = torch.cuda.current_stream()

    def gemm_only():
        for _ in range(nblocks):
            torch.matmul(a, b)

    def one_pass(t, gemm=True):
        for i in reversed(range(nblocks)):
            if gemm:
                torch.matmul(a, b)
            ev = torch.cuda.Event()
            ev.record(main)
            s = side[i % 2]
            s.wait_event(ev)
            blk = blocks[i]
            lohan.lohan_grad_sqnorm(blk["g"], n, wl.loss_scale, norms[i], flags[i], wss[i % 2],
                                    stream=s)
            lohan.lohan_adam_block_step(blk["p"], blk["m"], blk["v"], blk["g"], blk["p16"], n,
                                        hy["lr"], hy["beta1"], hy["beta2"], hy["eps"],
                                        hy["weight_decay"], t, hy["loss_scale"], flags[i],
                                        lohan.LOHAN_FLAG_PRECHECKED, None, stream=s)
        for s in side:
            main.wait_stream(s)

    for w in range(args.warmup):
        one_pass(hy["step"] + w)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        gemm_only()
    torch.cuda.synchronize()
    gemm_s = (time.perf_counter() - t0) / args.steps
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_pass(hy["step"] + args.warmup + k, gemm=False)
    torch.cuda.synchronize()
    steps_only_s = (time.perf_counter() - t0) / args.steps
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_pass(hy["step"] + args.warmup + args.steps + k)
    torch.cuda.synchronize()
    elapsed = (time.perf_counter() - t0) / args.steps
    assert all(int(f.cpu().item()) == 0 for f in flags)
    total = n * nblocks

    # The same pass with the ring form: the blocks' own arrays are slots 0..B-1, one more slot
    # is the spare; every step is the single-pass out-of-place update, committed on the device.
    # A ring's steps must be ordered, so they all go to one side stream.
    spare = {k: torch.empty_like(blocks[0][k]) for k in ("p", "m", "v", "p16")}
    slot_list = [(blk["p"], blk["m"], blk["v"], blk["p16"]) for blk in blocks]
    slot_list.append((spare["p"], spare["m"], spare["v"], spare["p16"]))
    ring = torch.empty(lohan.lohan_ring_bytes(nblocks), dtype=torch.uint8, device=dev)
    lohan.lohan_ring_init(ring, slot_list, n)

    def ring_pass(t):
        s = side[0]
        for i in reversed(range(nblocks)):
            torch.matmul(a, b)
            ev = torch.cuda.Event()
            ev.record(main)
            s.wait_event(ev)
            lohan.lohan_ring_adam_block_step(ring, nblocks, i, blocks[i]["g"], n, hy["lr"],
                                             hy["beta1"], hy["beta2"], hy["eps"],
                                             hy["weight_decay"], t, hy["loss_scale"], 0, stream=s)
        main.wait_stream(s)

    t_ring0 = hy["step"] + args.warmup + 2 * args.steps
    ring_pass(t_ring0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        ring_pass(t_ring0 + 1 + k)
    torch.cuda.synchronize()
    ring_elapsed = (time.perf_counter() - t0) / args.steps
    assert lohan.lohan_ring_read(ring, nblocks)[2] == [0] * nblocks
    return {
        "metric": "adam_updated_elements_per_sec", "value": total / elapsed,
        "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"stream13b: {nblocks} blocks of n={n}, 2 side streams, one bf16 "
                               "GEMM 2048x5120x20480 per block on the main stream",
                   "elements": total, "blocks": nblocks},
        "step_hbm_gbps": 30 * total / elapsed / 1e9,
        "ms_per_block": elapsed * 1e3 / nblocks,
        "gemm_only_ms": gemm_s * 1e3, "steps_only_ms": steps_only_s * 1e3,
        "pass_over_sum_of_parts": elapsed / (gemm_s + steps_only_s),
        "ring_form": {"note": "same pass with lohan_ring_adam_block_step (one spare slot, "
                              "single-pass steps on one side stream)",
                      "ms_per_step": ring_elapsed * 1e3, "value": total / ring_elapsed,
                      "over_in_place": elapsed / ring_elapsed},
        "roofline": {"kernel": "k_adam_block_step", "bound": "hbm",
                     "achieved": 28 * total / elapsed / 1e9, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": 28 * total / elapsed / 1e9 / HBM_PEAK_GBPS,
                     "traffic": None,
                     "note": "whole-pass figure (GEMMs and reductions overlapped), not a "
                             "per-kernel event timing"},
        "cpu_baseline": None,
    }


def bench_offload(args, torch, lohan, synth):
    """Active gradient offloading with the fp32 state in pinned host memory (the paper's far tier
    re-cast for this machine): per block H2D p,m,v -> flag/norm + Adam step in a device slot ->
    D2H p,m,v, serialised (the paper's naive schedule) and overlapped (its optimized schedule)."""
    wl = synth.WORKLOADS["gpt13b"]
    dev = "cuda:0"
    nblocks = args.blocks or 6
    n = wl.n
    hy = wl.hyper()
    host, grads, p16s, flags, norms = [], [], [], [], []
    for i in range(nblocks):
        t = synth.make_block(wl, seed=i, device=dev)
        host.append(tuple(torch.empty(n, dtype=torch.float32, pin_memory=True).copy_(t[k])
                          for k in ("p", "m", "v")))
        grads.append(t["g"])
        p16s.append(t["p16"])
        flags.append(torch.zeros(1, dtype=torch.int32, device=dev))
        norms.append(torch.zeros(1, dtype=torch.float64, device=dev))
        del t
    slots = 3
    slab = torch.empty(lohan.lohan_offload_slab_bytes(n, slots), dtype=torch.uint8, device=dev)

    def run(mode, passes, first_step):
        h = lohan.lohan_offload_create(slab, n, slots, mode)
        try:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(passes):
                for i in reversed(range(nblocks)):
                    p, m, v = host[i]
                    lohan.lohan_offload_submit(h, p, m, v, grads[i], p16s[i], n, flags[i],
                                               norms[i], hy["lr"], hy["beta1"], hy["beta2"],
                                               hy["eps"], hy["weight_decay"], first_step + k,
                                               hy["loss_scale"], 0.0, 0)
            lohan.lohan_offload_drain(h)
            return (time.perf_counter() - t0) / passes
        finally:
            lohan.lohan_offload_destroy(h)

    steps = max(1, min(args.steps, 5))
    warm = max(1, min(args.warmup, 2))
    run(lohan.LOHAN_OFFLOAD_OVERLAPPED, warm, hy["step"])
    t_ser = run(lohan.LOHAN_OFFLOAD_SERIALIZED, steps, hy["step"] + warm)
    t_ovl = run(lohan.LOHAN_OFFLOAD_OVERLAPPED, steps, hy["step"] + warm + steps)
    assert all(int(f.cpu().item()) == 0 for f in flags)

    # Zero-copy alternative: pinned host memory is device-accessible, so the same two calls can
    # run with p, m, v left in host memory; every access of the kernel then crosses PCIe.
    ws = lohan.new_workspace(dev)

    def zero_copy_pass(t):
        for i in reversed(range(nblocks)):
            p, m, v = host[i]
            lohan.lohan_grad_sqnorm(grads[i], n, wl.loss_scale, norms[i], flags[i], ws)
            lohan.lohan_adam_block_step(p, m, v, grads[i], p16s[i], n, hy["lr"], hy["beta1"],
                                        hy["beta2"], hy["eps"], hy["weight_decay"], t,
                                        hy["loss_scale"], flags[i], lohan.LOHAN_FLAG_PRECHECKED,
                                        None)

    zero_copy_pass(hy["step"] + warm + 2 * steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        zero_copy_pass(hy["step"] + warm + 2 * steps + 1 + k)
    torch.cuda.synchronize()
    t_zc = (time.perf_counter() - t0) / steps
    total = n * nblocks
    return {
        "metric": "adam_updated_elements_per_sec", "value": total / t_ovl, "unit": "elements/s",
        "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": t_ovl * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"offload13b: {nblocks} blocks of n={n}, fp32 state in pinned host "
                               f"memory, {slots} device staging slots, overlapped schedule",
                   "elements": total, "blocks": nblocks},
        "serialized_value": total / t_ser, "serialized_ms_per_step": t_ser * 1e3,
        "overlapped_over_serialized": t_ser / t_ovl,
        "zero_copy_value": total / t_zc, "zero_copy_ms_per_step": t_zc * 1e3,
        "zero_copy_pcie_gbps_each_direction": 12 * total / t_zc / 1e9,
        "pcie_gbps_each_direction": 12 * total / t_ovl / 1e9,
        "roofline": {"kernel": "H2D/D2H copies around k_adam_block_step", "bound": "pcie",
                     "achieved": 12 * total / t_ovl / 1e9, "peak": 64.0, "unit": "GB/s",
                     "frac": 12 * total / t_ovl / 1e9 / 64.0, "traffic": None,
                     "note": "12 B/element cross PCIe in each direction; peak = PCIe Gen5 x16 "
                             "per direction; the HBM-side step is ~50x faster than the link"},
        "cpu_baseline": None,
    }


def bench_shapes(args, torch, lohan, synth):
    """Size-versus-bandwidth curve over the block shapes of the paper's evaluation models
    (Table IV GPT-style, Table VI DiT): one block of each shape through the same two calls."""
    dev = "cuda:0"
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    sqnorm = torch.zeros(1, dtype=torch.float64, device=dev)
    ws = lohan.new_workspace(dev)
    rows = []
    for wl in synth.shape_workloads():
        n = wl.n
        if args.placement == "library":
            views, slab, _ = placed_views(n, torch, lohan, dev)
        block = synth.make_block(wl, seed=0, device=dev)
        hy = wl.hyper()
        reps = max(3, min(args.steps, int(2e10 // n)))
        if args.placement == "library":
            for k in views:
                views[k].copy_(block[k])
            block = views
            torch.cuda.empty_cache()

        def one_step(t, ev=None):
            lohan.lohan_grad_sqnorm(block["g"], n, wl.loss_scale, sqnorm, flag, ws)
            if ev is not None:
                ev[0].record()
            lohan.lohan_adam_block_step(block["p"], block["m"], block["v"], block["g"],
                                        block["p16"], n, hy["lr"], hy["beta1"], hy["beta2"],
                                        hy["eps"], hy["weight_decay"], t, hy["loss_scale"], flag,
                                        lohan.LOHAN_FLAG_PRECHECKED, None)
            if ev is not None:
                ev[1].record()

        for w in range(2):
            one_step(hy["step"] + w)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(reps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(reps):
            one_step(hy["step"] + 2 + k, evs[k])
        torch.cuda.synchronize()
        step_s = (time.perf_counter() - t0) / reps
        adam_ms = sum(a.elapsed_time(b) for a, b in evs) / reps
        assert int(flag.cpu().item()) == 0
        rows.append({"shape": wl.name, "elements": n, "resident_gb": 16 * n / 1e9,
                     "ms_per_step": step_s * 1e3, "elements_per_s": n / step_s,
                     "adam_kernel_ms": adam_ms,
                     "adam_kernel_gbps": ADAM_BYTES_PER_ELEM * n / adam_ms / 1e6,
                     "adam_kernel_frac_of_peak": ADAM_BYTES_PER_ELEM * n / adam_ms / 1e6 /
                                                 HBM_PEAK_GBPS})
        del block
        views = slab = None
        torch.cuda.empty_cache()
    total = sum(r["elements"] for r in rows)
    total_s = sum(r["ms_per_step"] for r in rows) / 1e3
    worst = min(rows, key=lambda r: r["adam_kernel_frac_of_peak"])
    return {
        "metric": "adam_updated_elements_per_sec", "value": total / total_s,
        "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": 2,
        "ms_per_step": total_s * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "shapes: one block of every Table IV (12*h^2) and Table VI "
                               "(18*h^2) model shape", "elements": total},
        "roofline": {"kernel": "k_adam_block_step", "bound": "hbm",
                     "achieved": worst["adam_kernel_gbps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": worst["adam_kernel_frac_of_peak"], "traffic": None,
                     "note": f"worst shape of the sweep ({worst['shape']})"},
        "shapes": rows, "cpu_baseline": None,
    }


def bench_models(args, torch, lohan, synth):
    """Whole small models, all blocks' gradients present: the step of every block issued (a) block
    by block (lohan_grad_sqnorm + lohan_adam_block_step per block) and (b) through one
    lohan_adam_multi_block_step call.  One "step" = one pass over all blocks of one model."""
    dev = "cuda:0"
    models = [("gpt_h768_12blocks", 12, 12 * 768 ** 2)]
    models += [(f"dit{name}_{layers}blocks", layers, 18 * h * h)
               for name, layers, h in synth.TABLE_VI_DIT[:4]]
    models += [("gpt6B_28blocks", 28, 12 * 4096 ** 2)]
    rows = []
    for name, layers, n in models:
        wl = synth.Workload(name, n, 100, 65536.0, False)
        hy = wl.hyper()
        if args.placement == "library":
            # the whole model in one slab, every block where lohan_model_placement puts it
            offsets, slab_bytes, align, _ = lohan.lohan_model_placement(n, layers)
            slab = torch.empty(slab_bytes + align, dtype=torch.uint8, device=dev)
            start = (-slab.data_ptr()) % align
            spec = {"p": ("param_fp32", torch.float32, 4), "m": ("exp_avg", torch.float32, 4),
                    "v": ("exp_avg_sq", torch.float32, 4), "g": ("grad_fp16", torch.float16, 2),
                    "p16": ("param_bf16", torch.bfloat16, 2)}
            blocks = []
            for i in range(layers):
                src = synth.make_block(wl, seed=i, device=dev)
                views = {}
                for k, (field, dtype, width) in spec.items():
                    off = start + offsets[i][field]
                    views[k] = slab[off: off + n * width].view(dtype)
                    views[k].copy_(src[k])
                blocks.append(views)
                del src
        else:
            slab = None
            blocks = [synth.make_block(wl, seed=i, device=dev) for i in range(layers)]
        flags = torch.zeros(layers, dtype=torch.int32, device=dev)
        norms = torch.zeros(layers, dtype=torch.float64, device=dev)
        ws = lohan.new_workspace(dev)
        array = lohan.make_block_array([(b["p"], b["m"], b["v"], b["g"], b["p16"], n)
                                        for b in blocks])
        reps = max(3, min(args.steps, int(4e10 // (n * layers))))

        def per_block(t):
            for i, b in enumerate(blocks):
                lohan.lohan_grad_sqnorm(b["g"], n, wl.loss_scale, norms[i:i + 1],
                                        flags[i:i + 1], ws)
                lohan.lohan_adam_block_step(b["p"], b["m"], b["v"], b["g"], b["p16"], n,
                                            hy["lr"], hy["beta1"], hy["beta2"], hy["eps"],
                                            hy["weight_decay"], t, hy["loss_scale"],
                                            flags[i:i + 1], lohan.LOHAN_FLAG_PRECHECKED, None)

        def multi(t):
            lohan.lohan_adam_multi_block_step(array, hy["lr"], hy["beta1"], hy["beta2"],
                                              hy["eps"], hy["weight_decay"], t,
                                              hy["loss_scale"], 0.0, flags, norms, 0, ws,
                                              num_blocks=layers)

        def timed(fn, t_first):
            fn(t_first)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(reps):
                fn(t_first + 1 + k)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps

        t_blk = timed(per_block, hy["step"])
        t_multi = timed(multi, hy["step"] + reps + 1)
        assert int(flags.max().cpu().item()) == 0
        total = n * layers
        rows.append({"model": name, "blocks": layers, "elements_per_block": n,
                     "per_block_calls_ms": t_blk * 1e3, "multi_block_call_ms": t_multi * 1e3,
                     "per_block_calls_elements_per_s": total / t_blk,
                     "multi_block_call_elements_per_s": total / t_multi,
                     "multi_block_call_step_hbm_gbps":
                         (ADAM_BYTES_PER_ELEM + REDUCE_BYTES_PER_ELEM) * total / t_multi / 1e9,
                     "speedup": t_blk / t_multi})
        del blocks, array, slab
        torch.cuda.empty_cache()
    total = sum(r["blocks"] * r["elements_per_block"] for r in rows)
    total_s = sum(r["multi_block_call_ms"] for r in rows) / 1e3
    worst = min(rows, key=lambda r: r["multi_block_call_step_hbm_gbps"])
    return {
        "metric": "adam_updated_elements_per_sec", "value": total / total_s,
        "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": 1,
        "ms_per_step": total_s * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "models: all blocks of six small models (h=768 x12, the four "
                               "smallest DiT shapes of Table VI, GPT 6B), one multi-block call "
                               "per model", "elements": total},
        "roofline": {"kernel": "whole multi-block call (reduction + update), 30 B/element",
                     "bound": "hbm", "achieved": worst["multi_block_call_step_hbm_gbps"],
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": worst["multi_block_call_step_hbm_gbps"] / HBM_PEAK_GBPS,
                     "traffic": None, "note": f"worst model of the sweep ({worst['model']})"},
        "models": rows, "cpu_baseline": None,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); the step is "
              "elementwise and would shard by contiguous element ranges, but no multi-GPU path "
              "exists here", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2403_06504_amd as lohan
    from paper_2403_06504_amd import synthetic_inputs as synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    lohan.load_library()
    if args.variant is not None or args.wgs_per_cu or args.waves_per_cu >= 0:
        lohan.lohan_tuning_set_launch_config(-1 if args.variant is None else args.variant,
                                      args.wgs_per_cu, args.waves_per_cu, 0)
    if args.workload == "stream13b":
        out = bench_stream(args, torch, lohan, synth)
    elif args.workload == "offload13b":
        out = bench_offload(args, torch, lohan, synth)
    elif args.workload == "shapes":
        out = bench_shapes(args, torch, lohan, synth)
    elif args.workload == "models":
        out = bench_models(args, torch, lohan, synth)
    elif args.workload == "ring13b":
        out = bench_ring(args, torch, lohan, synth)
    elif args.workload.endswith("_oop"):
        out = bench_block_oop(args, torch, lohan, synth)
    else:
        out = bench_block(args, torch, lohan, synth)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

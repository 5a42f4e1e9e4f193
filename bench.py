#!/usr/bin/env python3
"""Benchmark of the RGC hot path on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input:
  rgc_compress_layers on the VGG16-shaped layer set (16 tensors, 138.3 M fp32 elements,
  momentum-corrected variant, density 0.1 %)  followed by
  rgc_decompress_accumulate of 128 virtual workers' messages (0.1 % each, 80 % from a shared
  hot set) into a VGG16-shaped dense buffer, averaged by 128.
All inputs are resident in HBM before the timed region.  The residual and velocity evolve
from step to step (steady-state RGC) while the gradient rotates through 4 pre-generated sets.

Prints ONE JSON line: `value` = gradient bytes through the whole step per second (wall-clock mean of the K
timed steps); `compress`, `decompress`, `local_clipping`, `alternating_signs`, `threshold_search`,
`threshold_to_decompress`, `warmup_densities` (and the same with 16 gradient sets in rotation) and `other_workloads` time the parts and the variants; `roofline` is the streaming
accumulate kernel against the HBM peak, timed with HIP events inside the timed steps; `cpu_baseline` is the CPU
oracle timed on the same step.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
NUM_GRAD_SETS = 4


def kernel_source_digest():
    """sha256 over the kernel sources of the compression path: what profiles/hbm_traffic.json is stamped with."""
    import hashlib
    h = hashlib.sha256()
    for name in ("rgc_compress.hip", "rgc_device.h", "rgc_internal.h"):
        with open(os.path.join(ROOT, "paper_1808_04357_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def upload(torch, arrays, dev):
    return [torch.from_numpy(a).to(dev) for a in arrays]


class CompressWorkload:
    def __init__(self, torch, rgc, cfg, dev, ppm=1000):
        self.torch, self.rgc = torch, rgc
        self.name = cfg["name"]
        self.m = float(cfg["momentum"])
        self.sizes = [int(v.size) for v in cfg["V"]]
        self.total = sum(self.sizes)
        self.ks = [rgc.rgc_k_for_density(n, ppm) for n in self.sizes]
        self.V = upload(torch, cfg["V"], dev)
        self.U = upload(torch, cfg["U"], dev) if cfg["U"] is not None else None
        self.G = [upload(torch, g, dev) for g in cfg["G"]]
        self.out_idx = [torch.empty(k, dtype=torch.int32, device=dev) for k in self.ks]
        self.out_val = [torch.empty(k, dtype=torch.float32, device=dev) for k in self.ks]
        self.out_count = torch.zeros(len(self.ks), dtype=torch.int32, device=dev)
        self.lists = [rgc.LayerList(g, self.V, self.ks, self.out_idx, self.out_val, self.out_count, self.U)
                      for g in self.G]
        per_elem = 20 if self.U is not None else 12      # read G,V(,u); write V(,u)
        self.alg_bytes_stream = per_elem * self.total
        self.alg_bytes = per_elem * self.total + (16 if self.U is not None else 12) * sum(self.ks)
        self.t = 0

    def step(self, ctx, stream, flags=0):
        self.rgc.rgc_compress_layers(ctx, self.lists[self.t % len(self.lists)], self.m, flags, stream)
        self.t += 1


class DecompressWorkload:
    def __init__(self, torch, rgc, sizes, workers, dev, synth):
        self.torch, self.rgc = torch, rgc
        self.sizes = sizes
        self.workers = workers
        idx, val = synth.decompress_messages(sizes, num_workers=workers)
        self.entries = sum(int(a.size) for row in idx for a in row)
        # the messages sit back to back, worker after worker, as an Allgather leaves them
        self.recv_idx = torch.empty(self.entries, dtype=torch.int32, device=dev)
        self.recv_val = torch.empty(self.entries, dtype=torch.float32, device=dev)
        self.d_idx, self.d_val, o = [], [], 0
        for w in range(workers):
            ri, rv = [], []
            for l in range(len(sizes)):
                c = int(idx[w][l].size)
                ri.append(self.recv_idx[o:o + c])
                rv.append(self.recv_val[o:o + c])
                ri[-1].copy_(torch.from_numpy(idx[w][l]))
                rv[-1].copy_(torch.from_numpy(val[w][l]))
                o += c
            self.d_idx.append(ri)
            self.d_val.append(rv)
        self.dense = [torch.empty(n, dtype=torch.float32, device=dev) for n in sizes]
        self.msgs = rgc.MessageList(self.d_idx, self.d_val, self.dense)
        self.scale = 1.0 / workers
        self.alg_bytes = 8 * self.entries + 4 * sum(sizes)

    def step(self, ctx, stream):
        self.rgc.rgc_decompress_accumulate(ctx, self.msgs, self.scale, self.rgc.RGC_OVERWRITE, stream)


def time_loop(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def measure_yardstick(torch, rgc, ctx, wl, dec, stream, dev, reps):
    """rgc_stream_yardstick on tensors of the workload's total size: u = m u + g, V += u and nothing else."""
    g = torch.randn(wl.total, dtype=torch.float32, device=dev) * 1e-3
    v = torch.zeros(wl.total, dtype=torch.float32, device=dev)
    u = torch.zeros(wl.total, dtype=torch.float32, device=dev)
    calls = [0]

    def bare():
        rgc.rgc_stream_yardstick(g, v, u, wl.m, calls[0] & 1, stream)     # alternating direction, like the compress calls
        calls[0] += 1

    for _ in range(5):
        bare()
    ms_b2b = time_loop(torch, bare, reps)
    evs = []
    for _ in range(reps):
        dec.step(ctx, stream)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        bare()
        b.record(stream)
        evs.append((a, b))
    torch.cuda.synchronize()
    ms_after = sum(a.elapsed_time(b) for a, b in evs) / reps
    bytes_ = 20.0 * wl.total
    return {"kernel": "yardstick_kernel (reads G, V, u and writes V, u of the same total size; no selection work)",
            "back_to_back_ms": ms_b2b, "back_to_back_GBps": bytes_ / ms_b2b / 1e6,
            "after_decompress_ms": ms_after, "after_decompress_GBps": bytes_ / ms_after / 1e6,
            "frac_of_peak_after_decompress": bytes_ / (ms_after * 1e-3) / (HBM_PEAK_GBPS * 1e9)}


def measure_threshold(torch, rgc, ctx, wl, stream, steps, dev):
    """A call that searches the thresholds, a call that reuses them, and the paper's schedule (search every
    fifth call) on the workload's tensors; message buffers of 2k entries."""
    out_idx2 = [torch.empty(2 * k, dtype=torch.int32, device=dev) for k in wl.ks]
    out_val2 = [torch.empty(2 * k, dtype=torch.float32, device=dev) for k in wl.ks]
    lists2 = [rgc.LayerList(g, wl.V, wl.ks, out_idx2, out_val2, wl.out_count, wl.U) for g in wl.G]
    thr = torch.zeros(len(wl.sizes), dtype=torch.float32, device=dev)
    nnz = torch.zeros(len(wl.sizes), dtype=torch.int32, device=dev)
    calls = [0]

    def tbs(search):
        rgc.rgc_compress_layers_threshold(ctx, lists2[calls[0] % len(lists2)], wl.m, thr, nnz,
                                          rgc.RGC_THRESHOLD_SEARCH if search else 0, stream)
        calls[0] += 1

    for _ in range(5):
        tbs(True)
    reps = min(steps, 50)
    ms_search = time_loop(torch, lambda: tbs(True), reps)
    ms_reuse = time_loop(torch, lambda: tbs(False), reps)
    ms_sampled = time_loop(torch, lambda: tbs(calls[0] % 5 == 0), 5 * max(1, reps // 5))
    sent = nnz.cpu().numpy()
    return {"search_call_ms": ms_search, "reuse_call_ms": ms_reuse, "sampled_every_5_ms": ms_sampled,
            "sent_over_k_last_call": float(sent.sum()) / float(sum(wl.ks)),
            "search_call_alg_bytes": wl.alg_bytes_stream + 3 * 4 * wl.total,
            "reuse_call_alg_bytes": wl.alg_bytes_stream}


def measure_threshold_flow(torch, rgc, ctx, wl, dec, stream, steps, dev):
    """Threshold binary search selection feeding decompression (Sections 2.1 + 2.3): the messages' lengths vary from
    step to step, and rgc_msg.count is a host value, so every step runs the selection (a search every fifth step),
    brings the 16 length elements to the host (a synchronisation), and decompresses 128 workers' messages of which
    worker 0's are the ones just produced (the other 127 are the fixed synthetic ones).  Reported: the whole step,
    how long the host waits for the lengths, and how long the decompression call keeps the host (its descriptor
    tables are rebuilt and uploaded whenever a length changes)."""
    L = len(wl.sizes)
    out_idx2 = [torch.empty(2 * k, dtype=torch.int32, device=dev) for k in wl.ks]
    out_val2 = [torch.empty(2 * k, dtype=torch.float32, device=dev) for k in wl.ks]
    count = torch.zeros(L, dtype=torch.int32, device=dev)
    lists2 = [rgc.LayerList(g, wl.V, wl.ks, out_idx2, out_val2, count, wl.U) for g in wl.G]
    thr = torch.zeros(L, dtype=torch.float32, device=dev)
    host_count = torch.zeros(L, dtype=torch.int32).pin_memory()
    d_idx = [list(row) for row in dec.d_idx]
    d_val = [list(row) for row in dec.d_val]
    d_idx[0], d_val[0] = out_idx2, out_val2
    msgs = rgc.MessageList(d_idx, d_val, dec.dense)
    calls = [0]
    wait_ms, host_ms = [], []

    def step():
        rgc.rgc_compress_layers_threshold(ctx, lists2[calls[0] % len(lists2)], wl.m, thr, None,
                                          rgc.RGC_THRESHOLD_SEARCH if calls[0] % 5 == 0 else 0, stream)
        calls[0] += 1
        t0 = time.perf_counter()
        host_count.copy_(count, non_blocking=True)
        stream.synchronize()
        t1 = time.perf_counter()
        for l in range(L):
            msgs.msgs[l].count = int(host_count[l])
        t2 = time.perf_counter()
        rgc.rgc_decompress_accumulate(ctx, msgs, dec.scale, rgc.RGC_OVERWRITE, stream)
        t3 = time.perf_counter()
        wait_ms.append((t1 - t0) * 1e3)
        host_ms.append((t3 - t2) * 1e3)

    for _ in range(10):
        step()
    del wait_ms[:], host_ms[:]
    reps = 5 * max(1, min(steps, 50) // 5)
    ms = time_loop(torch, step, reps)
    sent = int(host_count.sum())
    return {"ms_per_step": ms, "steps": reps, "gradient_GBps": 4.0 * wl.total / ms / 1e6,
            "host_waits_for_lengths_ms": sum(wait_ms) / len(wait_ms),
            "decompress_call_host_ms": sum(host_ms) / len(host_ms),
            "decompress_call_host_ms_max": max(host_ms),
            "sent_over_k_last_step": sent / float(sum(wl.ks))}


def measure_compress(torch, rgc, ctx, wl, stream, steps, warmup):
    """Steady-state ms/iter plus first-call and hint-free timings of one compress workload."""
    out = {"elements": wl.total, "tensors": len(wl.sizes), "sum_k": sum(wl.ks)}
    ctx.reset_hints()
    out["first_call_ms"] = time_loop(torch, lambda: wl.step(ctx, stream), 1)
    # After a reset the threshold hints (and their drift estimate) take a few dozen calls to settle:
    # the embedding-like tensor of the LSTM set misses on every other call until about the 30th.
    # Training runs for thousands of iterations, so the steady state is what is timed: at least
    # 40 warm-up calls here, and the hint misses inside the timed calls are counted and reported.
    settle = max(warmup, 40)
    for _ in range(settle):
        wl.step(ctx, stream)
    misses0 = sum(r[4] for r in ctx.last_stats(len(wl.sizes), stream))
    ms = time_loop(torch, lambda: wl.step(ctx, stream), steps)
    out["ms_per_iter"] = ms
    out["warmup_calls"] = settle
    out["hint_misses_in_timed_calls"] = sum(r[4] for r in ctx.last_stats(len(wl.sizes), stream)) - misses0
    # the same iterations once more, each bracketed by its own pair of events on the stream (median and minimum)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in evs:
        a.record(stream)
        wl.step(ctx, stream)
        b.record(stream)
    torch.cuda.synchronize()
    per = sorted(a.elapsed_time(b) for a, b in evs)
    out["ms_median"] = per[len(per) // 2]
    out["ms_min"] = per[0]
    out["gradient_GBps"] = 4.0 * wl.total / ms / 1e6
    out["alg_bytes"] = wl.alg_bytes
    out["hbm_frac_algorithmic"] = wl.alg_bytes / (ms * 1e-3) / (HBM_PEAK_GBPS * 1e9)
    # kernel split and path statistics with the library's event timing switched on
    ctx.profile_enable(True)
    slow = 0
    psteps = min(steps, 20)
    for _ in range(psteps):
        wl.step(ctx, stream)
        slow += sum(1 for p in ctx.last_paths(len(wl.sizes), stream) if p != 0)
    ms4, calls = ctx.profile_read()
    ctx.profile_enable(False)
    out["accumulate_kernel_ms"] = ms4[0] / max(calls[0], 1)
    out["phase_launches_ms"] = ms4[1] / max(calls[0], 1)
    out["layers_off_one_pass_path_per_iter"] = slow / psteps
    out["hint_free_ms"] = time_loop(torch, lambda: wl.step(ctx, stream, rgc.RGC_NO_HINTS), 3)
    # a call whose hints all miss (thresholds set far too high before every call: the streaming pass collects too
    # few candidates, notices, and every layer takes the multi-pass path on the updated residual)

    def forced_miss():
        ctx.poison_hints(0, stream)
        wl.step(ctx, stream)

    out["forced_miss_ms"] = time_loop(torch, forced_miss, 5)
    out["forced_miss_layers_on_fallback"] = sum(1 for p in ctx.last_paths(len(wl.sizes), stream) if p == 2)
    return out


def measure_step_on(torch, rgc, ctx, wl, stream, steps, dev, synth):
    """The whole step (compression + decompression of 128 workers' messages of the same shape) on a layer set."""
    dec = DecompressWorkload(torch, rgc, wl.sizes, 128, dev, synth)

    def step():
        wl.step(ctx, stream)
        dec.step(ctx, stream)

    for _ in range(40):
        step()
    ms = time_loop(torch, step, steps)
    ms_d = time_loop(torch, lambda: dec.step(ctx, stream), steps)
    nbytes = wl.alg_bytes + dec.alg_bytes
    return {"ms_per_step": ms, "gradient_GBps": 4.0 * wl.total / ms / 1e6, "alg_bytes": nbytes,
            "hbm_frac_step_algorithmic": nbytes / (ms * 1e-3) / (HBM_PEAK_GBPS * 1e9),
            "decompress_alone_ms": ms_d, "decompress_entries": dec.entries}


def more_gradient_sets(torch, wl, count, dev, seed=20180804):
    """`count` further gradient sets for the workload's tensors, drawn on the device from the headline recipe's law
    (Laplace(0, 1e-3), inverse-CDF of a seeded uniform stream)."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)

    def laplace(n, b):
        u = torch.rand(n, device=dev, generator=gen) - 0.5
        return (-b * torch.sign(u) * torch.log1p(-2.0 * u.abs())).to(torch.float32)

    return [[laplace(n, 1e-3) for n in wl.sizes] for _ in range(count)]


def measure_density(torch, rgc, ctx, vgg, ppm, stream, steps, dev, grads=None):
    """The compression call on the headline tensors at another density (Section 2.5: the warm-up period's):
    message buffers of its own, residual and velocity shared with the headline workload."""
    ks = [rgc.rgc_k_for_density(n, ppm) for n in vgg.sizes]
    oi = [torch.empty(k, dtype=torch.int32, device=dev) for k in ks]
    ov = [torch.empty(k, dtype=torch.float32, device=dev) for k in ks]
    lists = [rgc.LayerList(g, vgg.V, ks, oi, ov, vgg.out_count, vgg.U) for g in (grads if grads is not None else vgg.G)]
    calls = [0]

    def warm_step():
        rgc.rgc_compress_layers(ctx, lists[calls[0] % len(lists)], vgg.m, 0, stream)
        calls[0] += 1

    for _ in range(40):                           # the hints and margins of the dense layers settle within a few dozen calls
        warm_step()
    misses0 = sum(r[4] for r in ctx.last_stats(len(vgg.sizes), stream))
    ms = time_loop(torch, warm_step, min(steps, 20))
    alg = vgg.alg_bytes_stream + 16 * sum(ks)
    return {"sum_k": sum(ks), "ms_per_iter": ms, "alg_bytes": alg,
            "hbm_frac_algorithmic": alg / (ms * 1e-3) / (HBM_PEAK_GBPS * 1e9),
            "hint_misses_in_timed_calls": sum(r[4] for r in ctx.last_stats(len(vgg.sizes), stream)) - misses0,
            "layers_on_multi_pass_path_last_call": sum(1 for p in ctx.last_paths(len(vgg.sizes), stream) if p != 0)}


def cpu_baseline(torch, wl, dec):
    """The oracle as it stands, timed on the host over one whole step of the headline workload: one
    compress step of the layer set on one thread (about 10 s for the VGG16 set: the largest tensor
    alone is a 103 M-pair sort) plus the decompression of the same messages the GPU step consumes
    (sequential scatter-add, one thread).  The compress step once more with the layers spread over
    the host's threads (layers are independent; the largest one bounds the gain)."""
    import oracle
    torch.cuda.synchronize()
    G = [g.cpu().numpy() for g in wl.G[0]]
    V0 = [v.cpu().numpy() for v in wl.V]
    U0 = [u.cpu().numpy() for u in wl.U] if wl.U is not None else None

    def run(threads):
        V = [v.copy() for v in V0]
        U = [u.copy() for u in U0] if U0 is not None else None
        t0 = time.perf_counter()
        oracle.compress_layers(G, V, wl.ks, momenta=U, m=wl.m, threads=threads)
        return time.perf_counter() - t0

    dt1 = run(1)
    T = min(oracle.hardware_threads(), len(wl.sizes), 16)
    dtT = run(T)
    h_idx = [[a.cpu().numpy() for a in row] for row in dec.d_idx]
    h_val = [[a.cpu().numpy() for a in row] for row in dec.d_val]
    t0 = time.perf_counter()
    for l, n in enumerate(dec.sizes):
        oracle.decompress([h_idx[w][l] for w in range(dec.workers)], [h_val[w][l] for w in range(dec.workers)],
                          n, dec.scale)
    dt_dec = time.perf_counter() - t0
    return {"value": 4.0 * wl.total / (dt1 + dt_dec) / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "one whole step: compress of all %d %s tensors (%d elements, plain C++ full-sort oracle, %.1f s) "
                      "+ decompress of %d workers' messages (%d entries, %.2f s), 1 thread"
                      % (len(wl.sizes), wl.name, wl.total, dt1, dec.workers, dec.entries, dt_dec),
            "compress_seconds": dt1, "decompress_seconds": dt_dec,
            "compress_only_GBps": 4.0 * wl.total / dt1 / 1e9,
            "layer_parallel_compress": {"value": 4.0 * wl.total / dtT / 1e9, "unit": "GB/s", "cores": T, "seconds": dtT},
            "host_threads_available": oracle.hardware_threads()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--skip-others", action="store_true", help="only the headline VGG16 step")
    ap.add_argument("--skip-cpu", action="store_true", help="leave out the oracle timing")
    ap.add_argument("--step-only", action="store_true",
                    help="only the step loops (warm-up, K steps, K timed steps): what a profiler should see when its "
                         "per-kernel averages are to be those of the timed region")
    ap.add_argument("--workload", choices=["lstm", "resnet50", "single_1Mi", "uniform_1Mi", "uniform_64Mi"],
                    help="time only the compression call on this layer set and print its block (for a profiler: "
                         "the per-kernel averages are then those of this workload)")
    ap.add_argument("--with-step", action="store_true",
                    help="with --workload: also time the whole step (compression + decompression of 128 workers' "
                         "messages of the same shape) on that layer set")
    ap.add_argument("--density-ppm", type=int,
                    help="time only the compression call on the headline tensors at this density (parts per million; "
                         "the warm-up period's densities of Section 2.5) and print its block (for a profiler)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain device copies of 4*138,344,128 bytes (a yardstick of known "
                         "size for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1")

    import torch
    import paper_1808_04357_amd as rgc
    from paper_1808_04357_amd import synth
    rgc.load_library()             # raises if the HIP library is missing: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()

    makers = {"lstm": lambda: synth.config_lstm(num_grads=NUM_GRAD_SETS),
              "resnet50": lambda: synth.config_resnet50(num_grads=NUM_GRAD_SETS),
              "single_1Mi": lambda: synth.config_single(1 << 20, num_grads=NUM_GRAD_SETS),
              "uniform_1Mi": lambda: synth.config_uniform(1 << 20, num_grads=NUM_GRAD_SETS),
              # the value law of the paper's own selection benchmark (Figure 2), 64 Mi elements
              "uniform_64Mi": lambda: synth.config_uniform(1 << 26, num_grads=NUM_GRAD_SETS)}
    if args.workload:
        wl = CompressWorkload(torch, rgc, makers[args.workload](), dev)
        ctx = rgc.Context(wl.total, 256)
        out = measure_compress(torch, rgc, ctx, wl, stream, args.steps, args.warmup)
        out["workload"] = args.workload
        if args.with_step:
            out["step"] = measure_step_on(torch, rgc, ctx, wl, stream, args.steps, dev, synth)
        print(json.dumps(out))
        return

    log("generating VGG16-shaped inputs (138.3 M elements, %d gradient sets)..." % NUM_GRAD_SETS)
    t0 = time.perf_counter()
    vgg = CompressWorkload(torch, rgc, synth.config_vgg16(num_grads=NUM_GRAD_SETS), dev)
    if args.density_ppm:
        ctx = rgc.Context(vgg.total, 256)
        for _ in range(20):                        # the state the densities meet in the default run: a residual in use
            vgg.step(ctx, stream)
        out = measure_density(torch, rgc, ctx, vgg, args.density_ppm, stream, args.steps, dev)
        out["density_ppm"] = args.density_ppm
        print(json.dumps(out))
        return
    log("  %.1f s; generating 128 workers' messages..." % (time.perf_counter() - t0))
    dec = DecompressWorkload(torch, rgc, vgg.sizes, 128, dev, synth)
    ctx = rgc.Context(vgg.total, 256)
    log("  done (%.1f s)" % (time.perf_counter() - t0))

    def step():
        vgg.step(ctx, stream)
        dec.step(ctx, stream)

    # ---- headline: whole step, inputs resident, W warmup + exactly K timed steps.  The threshold hints take a few
    # dozen calls to settle after a context is created (see measure_compress): at least 40 untimed steps,
    # whatever --warmup says; the hint misses that still fall into the timed steps are reported.
    settle = max(args.warmup, 40)
    for _ in range(settle):
        step()
    ms_step_plain = time_loop(torch, step, args.steps)   # the same loop without the library's events (reported beside)
    # the timed region: the library records HIP events around its kernels on the caller's stream,
    # so the dominant kernel's launch duration comes from these very K steps
    ctx.profile_enable(True)
    misses0 = sum(r[4] for r in ctx.last_stats(len(vgg.sizes), stream))
    ms_step = time_loop(torch, step, args.steps)
    step_misses = sum(r[4] for r in ctx.last_stats(len(vgg.sizes), stream)) - misses0
    step_ms4, step_calls = ctx.profile_read()
    ctx.profile_enable(False)
    step_bytes = vgg.alg_bytes + dec.alg_bytes
    value = 4.0 * vgg.total / ms_step / 1e6          # gradient GB/s through the whole step
    # the same step K more times, each bracketed by its own pair of events on the stream (median and minimum)
    per_step = [None]
    if not args.step_only:
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for a, b in evs:
            a.record(stream)
            step()
            b.record(stream)
        torch.cuda.synchronize()
        per_step = sorted(a.elapsed_time(b) for a, b in evs)

    # ---- the two halves and the dominant kernel, measured live with HIP events
    comp = dec_info = None
    if not args.step_only:
        ms_dec = time_loop(torch, lambda: dec.step(ctx, stream), args.steps)
        comp = measure_compress(torch, rgc, ctx, vgg, stream, args.steps, args.warmup)
        ctx.profile_enable(True)
        for _ in range(min(args.steps, 20)):
            dec.step(ctx, stream)
        ms4, calls = ctx.profile_read()
        ctx.profile_enable(False)
        dec_info = {"ms_per_iter": ms_dec, "entries": dec.entries, "workers": dec.workers,
                    "alg_bytes": dec.alg_bytes,
                    "hbm_frac_algorithmic": dec.alg_bytes / (ms_dec * 1e-3) / (HBM_PEAK_GBPS * 1e9),
                    "table_kernel_ms": ms4[2] / max(calls[1], 1), "tile_kernel_ms": ms4[3] / max(calls[1], 1)}
        # what writing the dense output costs by itself in the step's position: a plain fill of one tensor of the
        # same size (PyTorch's kernel) between two compression calls, and when fills follow each other
        fill_out = torch.empty(vgg.total, dtype=torch.float32, device=dev)
        for _ in range(3):
            fill_out.fill_(0.0)
        ms_fill = time_loop(torch, lambda: fill_out.fill_(0.0), min(args.steps, 20))
        evs = []
        for _ in range(min(args.steps, 20)):
            vgg.step(ctx, stream)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            fill_out.fill_(0.0)
            b.record(stream)
            evs.append((a, b))
        torch.cuda.synchronize()

        def step_with_fill():
            vgg.step(ctx, stream)
            fill_out.fill_(0.0)

        ms_step_fill = time_loop(torch, step_with_fill, min(args.steps, 20))
        dec_info["plain_fill_of_output_size"] = {"back_to_back_ms": ms_fill,
                                                 "after_compress_ms": sum(a.elapsed_time(b) for a, b in evs) / len(evs),
                                                 "step_with_fill_in_place_of_decompress_ms": ms_step_fill,
                                                 "bytes": 4 * vgg.total}
        del fill_out
    k_ms = step_ms4[0] / max(step_calls[0], 1)          # accumulate_kernel inside the timed steps
    achieved = vgg.alg_bytes_stream / (k_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "accumulate_kernel (fused residual/momentum accumulate + candidate collect)",
                "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                "traffic": None, "bytes_per_launch": vgg.alg_bytes_stream, "avg_launch_ms": k_ms}
    # HBM bytes per launch of that kernel as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE, scaled by a
    # copy of known size): a counter run cannot share a process with the timed run, so the figure
    # comes from the committed summary of the same command -- and only while the kernel sources are the
    # ones it was taken with (the file names their digest); otherwise null
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            t = json.load(f)
        if t.get("kernel_source_sha256") == kernel_source_digest():
            roofline["traffic"] = t["fetch_bytes_per_launch"] + t["write_bytes_per_launch"]
            roofline["traffic_source"] = t["source"]
            roofline["frac_measured_traffic"] = roofline["traffic"] / (k_ms * 1e-3) / (HBM_PEAK_GBPS * 1e9)
        else:
            roofline["traffic_source"] = "profiles/hbm_traffic.json was taken with other kernel sources: not used"
    except (OSError, ValueError, KeyError):
        pass

    # what the dominant kernel's traffic costs by itself on this device: the library's bare kernel of the same
    # reads and writes (no selection work), back to back like the compress loop above and, like the kernel in
    # the step, after a decompression call each time
    if not args.step_only:
        roofline["bare_kernel_same_traffic"] = measure_yardstick(torch, rgc, ctx, vgg, dec, stream, dev, min(args.steps, 30))
        bare = roofline["bare_kernel_same_traffic"]
        roofline["time_vs_bare_kernel"] = k_ms / bare["after_decompress_ms"]     # 1.03: 3 % more time than the traffic alone

    # the step before the accumulate when gradients are clipped locally (Section 2.4): one read of all gradients
    clip_info = None
    if not args.step_only:
        coef = torch.zeros(1, dtype=torch.float32, device=dev)
        ms_clip = time_loop(torch, lambda: rgc.rgc_clip_coefficient(ctx, vgg.lists[0], 1.0, 128, coef, stream), args.steps)
        ms_scaled = time_loop(torch, lambda: rgc.rgc_compress_layers_scaled(ctx, vgg.lists[0], vgg.m, coef, rgc.RGC_NESTEROV, stream),
                              min(args.steps, 20))
        clip_info = {"clip_coefficient_ms": ms_clip, "gradient_read_GBps": 4.0 * vgg.total / ms_clip / 1e6,
                     "hbm_frac": 4.0 * vgg.total / (ms_clip * 1e-3) / (HBM_PEAK_GBPS * 1e9),
                     "coefficient": float(coef.cpu()[0]),
                     "scaled_nesterov_compress_ms": ms_scaled}

    # Alternating Signs Quantization (Section 2.2): the k largest and the k smallest elements in turn, one
    # average per message, decompression of one-value messages; the same tensors and index sets as the headline step
    asq_info = None
    if not args.step_only:
        means = torch.zeros(len(vgg.sizes), dtype=torch.float32, device=dev)
        one_value = rgc.RGC_OVERWRITE | rgc.RGC_ONE_VALUE

        def asq_compress():
            vgg.step(ctx, stream, rgc.RGC_SELECT_LARGEST if vgg.t % 2 == 0 else rgc.RGC_SELECT_SMALLEST)

        def asq_step():
            asq_compress()
            rgc.rgc_message_means(ctx, vgg.lists[0], means, stream)
            rgc.rgc_decompress_accumulate(ctx, dec.msgs, dec.scale, one_value, stream)

        for _ in range(60):                               # each sign keeps hints of its own: both settle
            asq_step()
        misses0 = sum(r[4] for r in ctx.last_stats(len(vgg.sizes), stream))
        ms_asq = time_loop(torch, asq_step, args.steps)
        asq_misses = sum(r[4] for r in ctx.last_stats(len(vgg.sizes), stream)) - misses0
        ms_asq_comp = time_loop(torch, asq_compress, args.steps)
        ms_means = time_loop(torch, lambda: rgc.rgc_message_means(ctx, vgg.lists[0], means, stream), args.steps)
        ms_dec1 = time_loop(torch, lambda: rgc.rgc_decompress_accumulate(ctx, dec.msgs, dec.scale, one_value, stream),
                            args.steps)
        asq_info = {"ms_per_step": ms_asq, "gradient_GBps": 4.0 * vgg.total / ms_asq / 1e6,
                    "hint_misses_in_timed_steps": asq_misses, "compress_ms": ms_asq_comp,
                    "message_means_ms": ms_means, "decompress_one_value_ms": ms_dec1,
                    "decompress_alg_bytes": 4 * dec.entries + 4 * sum(dec.sizes)}

    # Threshold binary search selection (Section 2.1, Algorithm 3) and its sampled variant on the same tensors
    tbs_info = None
    if not args.step_only:
        tbs_info = measure_threshold(torch, rgc, ctx, vgg, stream, args.steps, dev)

    flow_info = None
    if not args.step_only:
        flow_info = measure_threshold_flow(torch, rgc, ctx, vgg, dec, stream, args.steps, dev)

    # The densities of a warm-up period (Section 2.5: 25 %, 6.25 %, 1.5625 %, 0.4 % before 0.1 %) on the same
    # tensors: message buffers of their own, residual and velocity shared with the headline workload
    # At these densities a quarter of the residual leaves with every call, and a gradient set that comes round again
    # after four calls meets what is left of its own last contribution: the k-th magnitude then swings from call to
    # call in a way no fresh gradient produces, and the dense layers' hints (which expect it where it last was) pay
    # for that in fix-up writes.  The second block rotates through 16 independent sets instead of 4.
    warm_info = warm_info16 = None
    if not args.step_only:
        warm_info = {}
        for ppm in (250_000, 62_500, 15_625, 4_000):
            warm_info["%g%%" % (ppm / 1e4)] = measure_density(torch, rgc, ctx, vgg, ppm, stream, args.steps, dev)
        torch.cuda.empty_cache()
        grads16 = vgg.G + more_gradient_sets(torch, vgg, 16 - len(vgg.G), dev)
        warm_info16 = {}
        for ppm in (250_000, 62_500, 15_625, 4_000):
            warm_info16["%g%%" % (ppm / 1e4)] = measure_density(torch, rgc, ctx, vgg, ppm, stream, args.steps, dev, grads16)
        del grads16
        torch.cuda.empty_cache()

    if args.calibrate_copy:
        src = torch.zeros(vgg.total, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    others = {}
    if not (args.skip_others or args.step_only):
        del step
        for name, make in makers.items():
            log("workload %s..." % name)
            wl = CompressWorkload(torch, rgc, make(), dev)
            others[name] = measure_compress(torch, rgc, ctx, wl, stream, args.steps, args.warmup)
            if name == "lstm":      # the paper selects the large layers of its recurrent models this way
                others[name]["threshold_search"] = measure_threshold(torch, rgc, ctx, wl, stream, args.steps, dev)
                # the whole step on this layer set too: compression + decompression of 128 workers' messages
                others[name]["step"] = measure_step_on(torch, rgc, ctx, wl, stream, args.steps, dev, synth)
            del wl
            torch.cuda.empty_cache()

    cpu = None
    if not args.skip_cpu:
        log("timing the CPU oracle on one whole step (compress on 1 thread, then layer-parallel, decompress; about 20 s)...")
        cpu = cpu_baseline(torch, vgg, dec)

    line = {
        "metric": "gradient GB/s through accumulate+top-k+pack (% HBM peak); ms/iter per layer set",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "VGG16-shaped layer set: compress (16 tensors, 138,344,128 elements, momentum 0.9, "
                               "density 0.1 %) + decompress of 128 virtual workers into the same shape",
                   "step": "rgc_compress_layers + rgc_decompress_accumulate", "gradient_sets_rotated": NUM_GRAD_SETS,
                   "kernel_launches_per_step": {"compress": 6, "decompress": 1}},
        "hbm_frac_step_algorithmic": step_bytes / (ms_step * 1e-3) / (HBM_PEAK_GBPS * 1e9),
        "ms_per_step_without_kernel_events": ms_step_plain,
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "hint_misses_in_timed_steps": step_misses, "untimed_steps_before": settle,
        "step_kernels_ms": {"accumulate_kernel": step_ms4[0] / max(step_calls[0], 1),
                            "phase_launches": step_ms4[1] / max(step_calls[0], 1),
                            "decompress_tiles_kernel": step_ms4[3] / max(step_calls[1], 1)},
        "compress": comp, "decompress": dec_info, "local_clipping": clip_info, "alternating_signs": asq_info, "threshold_search": tbs_info,
        "threshold_to_decompress": flow_info,
        "warmup_densities": warm_info, "warmup_densities_16_gradient_sets": warm_info16, "other_workloads": others,
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the fused OptiReduce node path (RHT encode -> masked aggregate -> mean -> decode).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extra] [--no-cpu]

One step = one pass of the whole path (sign flip, blockwise Hadamard, masked sum and count, mean,
inverse transform) over one synthetic batch: the N workers' raw slices of the shard this node owns,
already resident in HBM.  The headline workload is the largest configuration, Llama-8B-sized (bf16, 8 workers,
blocks of 2^16 entries, a 1.0e9-entry shard: 20 GB per step); the other four are reported beside it under
`other_workloads`.  Input sets of the small workloads are rotated so that consecutive steps do not find their
inputs in the 256 MB last-level cache.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
LLC_BYTES = 256 << 20       # last-level (Infinity) cache the rotation has to defeat


def build_sets(wl, b, cfg, device, nsets, entries=None, first=0):
    """nsets independent input sets for one launch shape: (grads, masks, out, count, workspace)."""
    sets = []
    L = cfg.shard_len(entries)
    for s in range(nsets):
        g = wl.make_grads(cfg, device, shard=s % cfg.workers, entries=entries, first=first)
        m = wl.make_masks(cfg, device, shard=s % cfg.workers, entries=entries, salt=s)
        out = torch.empty(L, dtype=g.dtype, device=device)
        cnt = torch.empty(L, dtype=torch.uint8, device=device)
        nws = b.or_workspace_bytes(L, cfg.block_log2)
        ws = torch.empty(nws, dtype=torch.uint8, device=device) if nws else None
        sets.append((g, m, out, cnt, ws))
    return sets


def launch(b, cfg, L, st, shard, stream=None):
    g, m, out, cnt, ws = st
    fn = b.or_fused_path if cfg.dtype == "f32" else b.or_fused_path_bf16
    fn(g, m, cfg.workers, L, cfg.block_log2, cfg.seed, shard * L, out, cnt, ws, stream)


class HipEvents:
    """Raw hipEvent_t pairs (ctypes on the HIP runtime torch already loaded).  The library attaches
    them to its kernel dispatch (or_time_next_call), so elapsed time is the kernel's own duration on
    the stream it runs on, as rocprofv3's kernel trace reports it."""

    def __init__(self, n):
        import ctypes
        self.c = ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, z = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0 and self.hip.hipEventCreate(ctypes.byref(z)) == 0
            self.pairs.append((a, z))

    def seconds(self):
        out = []
        for a, z in self.pairs:
            ms = self.c.c_float()
            rc = self.hip.hipEventElapsedTime(self.c.byref(ms), a, z)
            assert rc == 0, "hipEventElapsedTime failed: %d" % rc
            out.append(ms.value * 1e-3)
        return out

    def destroy(self):
        for a, z in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(z)


def time_fused(wl, b, cfg, device, steps, warmup, entries=None, launches_per_step=1, max_bytes=24 << 30, info=None):
    """Times `steps` steps; a step is `launches_per_step` launches (buckets) of one shape, one after the
    other on one stream.  The launches of the timed region are recorded into ONE HIP graph beforehand
    (the entry points only enqueue kernels, so they can be captured) and the timed region is one replay of
    it: the same kernels in the same strict order as plain launches, without the few microseconds that the
    runtime leaves between two dependent plain launches.  `info`, if given, also receives the plain-launch
    timing.  Returns (seconds per step by wall clock, mean seconds per launch by two HIP events on the
    launch stream, bytes per launch, number of input sets, the sets)."""
    L = cfg.shard_len(entries)
    es = 4 if cfg.dtype == "f32" else 2
    per_launch = wl.bytes_fused(cfg.workers, L, es)
    footprint = cfg.workers * L * es + cfg.workers * L // 8 + L * (es + 1) + b.or_workspace_bytes(L, cfg.block_log2)
    nsets = max(2, min(-(-3 * LLC_BYTES // footprint), 64))
    nsets = max(1, min(nsets, max_bytes // footprint))
    sets = build_sets(wl, b, cfg, device, nsets, entries)
    torch.cuda.synchronize()
    it = 0
    for _ in range(warmup * launches_per_step):
        launch(b, cfg, L, sets[it % nsets], it % nsets % cfg.workers)
        it += 1
    torch.cuda.synchronize()
    total = steps * launches_per_step

    def enqueue_all(first):
        for j in range(first, first + total):
            launch(b, cfg, L, sets[j % nsets], j % nsets % cfg.workers)

    if info is not None:   # plain launches back to back, for reference
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        enqueue_all(it)
        torch.cuda.synchronize()
        info["plain_launches_ms_per_step"] = (time.perf_counter() - t0) / steps * 1e3
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue_all(it)
    graph.replay()            # untimed: the first replay uploads the graph (and is `steps` more warm-up steps)
    torch.cuda.synchronize()
    # The timed region: exactly `total` launches, bracketed by a synchronise on both sides (wall clock ->
    # `value`) and by two HIP events recorded on the launch stream (-> mean time per launch for the roofline).
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    graph.replay()
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern = e0.elapsed_time(e1) * 1e-3 / total
    del graph
    return (t1 - t0) / steps, kern, per_launch, nsets, sets


def kernel_only_seconds(b, cfg, L, sets, launches=32):
    """Cross-check outside the timed region: events attached to single dispatches (kernel begin/end
    timestamps, what rocprofv3's kernel trace reports).  Slower to enqueue, so not used for `value`."""
    ev = HipEvents(launches)
    nsets = len(sets)
    for j in range(launches):
        b.or_time_next_call(ev.pairs[j][0], ev.pairs[j][1])
        launch(b, cfg, L, sets[j % nsets], j % nsets % cfg.workers)
    torch.cuda.synchronize()
    secs = ev.seconds()
    ev.destroy()
    return float(np.median(secs)), float(np.min(secs))


def time_three_calls(wl, b, cfg, sets, iters=20, L=None):
    """The same shard through the separate calls: encode (this node's own full gradient, N*L entries),
    masked reduce of the N encoded shards, finalize+decode of the shard.  Returns GB/s per call by the
    algorithmic bytes of each."""
    N, L, k = cfg.workers, (cfg.shard_len() if L is None else L), cfg.block_log2
    es = 4 if cfg.dtype == "f32" else 2
    bf = cfg.dtype != "f32"
    ns = len(sets)
    enc = torch.empty_like(sets[0][0])
    total = torch.empty(L, dtype=torch.float32, device=enc.device)
    cnt = torch.empty(L, dtype=torch.uint8, device=enc.device)
    out = torch.empty(L, dtype=enc.dtype, device=enc.device)

    def run(fn, nbytes):
        for j in range(2):
            fn(j)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for j in range(iters):
            fn(j)
        e1.record()
        torch.cuda.synchronize()
        return nbytes / (e0.elapsed_time(e1) * 1e-3 / iters) / 1e9

    if bf:
        f_enc = lambda j: b.or_rht_encode_bf16(sets[j % ns][0].view(-1), N * L, k, cfg.seed, 0, enc.view(-1))
        f_red = lambda j: b.or_masked_reduce_bf16(sets[j % ns][0], sets[j % ns][1], N, L, total, cnt)
        f_dec = lambda j: b.or_finalize_decode_bf16(total, cnt, L, k, cfg.seed, 0, out)
    else:
        f_enc = lambda j: b.or_rht_encode(sets[j % ns][0].view(-1), N * L, k, cfg.seed, enc.view(-1))
        f_red = lambda j: b.or_masked_reduce(sets[j % ns][0], sets[j % ns][1], N, L, total, cnt)
        f_dec = lambda j: b.or_finalize_decode(total, cnt, L, k, cfg.seed, 0, out)
    return {"encode_full_gradient_GB_per_s": run(f_enc, 2 * N * L * es),
            "masked_reduce_GB_per_s": run(f_red, N * L * es + N * L // 8 + 5 * L),
            "finalize_decode_shard_GB_per_s": run(f_dec, L * (5 + es))}


def cpu_baseline(wl, b, cfg, sets, target_seconds=12.0):
    """The oracle, single-threaded on this host, on the first blocks of the same workload; also
    checks the GPU result of those blocks against it."""
    import oracle
    g, m, out, cnt, _ = sets[0]
    B, N, k = cfg.block, cfg.workers, cfg.block_log2
    L = g.shape[1]

    def run(nblocks):
        n = nblocks * B
        gh = g[:, :n].contiguous().cpu()
        gh = gh.view(torch.int16).numpy().view(np.uint16) if gh.dtype == torch.bfloat16 else gh.numpy()
        mh = m[:, : n // 32].contiguous().cpu().numpy().view(np.uint32)
        t0 = time.perf_counter()
        want, wcnt = oracle.fused_path(gh, mh, k, cfg.seed, 0)
        return time.perf_counter() - t0, want, wcnt

    probe = max(1, min(4, L // B))
    t_probe, _, _ = run(probe)
    nblocks = int(max(probe, min(L // B, target_seconds / max(t_probe / probe, 1e-9))))
    secs, want, wcnt = run(nblocks)
    # a sample that the oracle finishes in well under the target is timed over several passes
    passes = 1
    if secs < target_seconds / 2:
        extra = min(64, int(target_seconds / max(secs, 1e-9)) - 1)
        total = secs
        for _ in range(extra):
            total += run(nblocks)[0]
        passes += extra
        secs = total / passes
    n = nblocks * B
    got = out[:n].cpu()
    got = (got.view(torch.int16).numpy().view(np.uint16).astype(np.uint32) << 16).view(np.float32) \
        if got.dtype == torch.bfloat16 else got.numpy()
    wantf = (want.astype(np.uint32) << 16).view(np.float32) if want.dtype == np.uint16 else want
    rel = float(np.linalg.norm(got.astype(np.float64) - wantf) / np.linalg.norm(wantf.astype(np.float64)))
    counts_equal = bool(np.array_equal(cnt[:n].cpu().numpy(), wcnt))
    es = 4 if cfg.dtype == "f32" else 2
    return {
        "value": wl.bytes_fused(N, n, es) / secs / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "host_cores": os.cpu_count(), "entries_per_s": N * n / secs, "seconds": secs, "passes": passes,
        "sample": "first %d blocks of 2^%d entries x %d workers of the %s workload (%d of %d input entries), "
                  "mean of %d passes" % (nblocks, k, N, cfg.name, N * n, N * L, passes),
        "gpu_vs_oracle_rel_l2_on_sample": rel, "counts_bit_exact_on_sample": counts_equal,
    }


def profiled_traffic(workload):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (scaled by a known-size copy); taken from the committed summary under profiles/, null if there is none."""
    import re
    path = os.path.join(ROOT, "profiles", "fused_path_%s.md" % workload)
    try:
        m = re.search(r"traffic = (\d+) bytes per (?:launch|step)", open(path).read())
        return int(m.group(1)) if m else None
    except OSError:
        return None


def roofline(cfg, L, nbytes, kern):
    """Which roof: the path's minimum work per input entry is es + 1/8 + (es + 1)/N bytes and
    k (N + 1)/N + 1 additions.  At the chip's peaks (8 TB/s; 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz = 78.6e12
    fp32 additions per second: an addition is half of the fused multiply-add that the published 157.3 TFLOP/s
    counts) the bytes take longer than the additions for all five workloads, so HBM is the roof.  The second
    figure is reported beside it because the kernels for 2^15 / 2^16 blocks spend several times that minimum in
    instructions (sign flips, conversions, rounding, exchanges through LDS) and sit far below the HBM roof."""
    N, k = cfg.workers, cfg.block_log2
    adds = (k * (N + 1) / N + 1.0) * N * L
    peak_adds = 256 * 4 * 32 * 2.4e9
    names = {True: "k_fused (one launch per step)",
             False: "k_sign_table + k_fused_mx (one step; the fused kernel is 99 % of it)" if cfg.dtype != "f32"
             else "k_sign_table + k_fused_pairs (+ k_decode_block for 2^16 blocks), one step"}
    return {"bound": "hbm", "achieved": nbytes / kern / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": nbytes / kern / 1e9 / HBM_PEAK_GBPS, "traffic": profiled_traffic(cfg.name),
            "kernel": names[cfg.block_log2 <= 14], "avg_launch_us": kern * 1e6,
            "ideal_ms_hbm": nbytes / (HBM_PEAK_GBPS * 1e9) * 1e3, "ideal_ms_alu": adds / peak_adds * 1e3,
            "alu": {"algorithmic_fp32_additions": adds, "achieved_Tadd_per_s": adds / kern / 1e12,
                    "peak_Tadd_per_s": peak_adds / 1e12, "frac": adds / kern / peak_adds}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="default: 20 for llama_8b, 300 for the small workloads")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--no-extra", action="store_true", help="skip the other model-sized workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--workload", default="llama_8b")
    ap.add_argument("--timed-region-only", action="store_true",
                    help="only the warm-up and the timed region (for a profiler: every launch of the run is then "
                         "one of the serialized launches that `value` and `roofline` are about)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 512 MiB device-to-device copies (a known-size reference for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the node path has no collective); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    import paper_2310_06993_amd.binding as b
    from paper_2310_06993_amd import workloads as wl

    device = torch.device("cuda:0")
    torch.cuda.set_device(device)
    cfg = wl.CONFIGS[args.workload]
    es = 4 if cfg.dtype == "f32" else 2
    big = cfg.shard_len() * cfg.workers * es > (1 << 30)
    if args.steps is None:
        args.steps = 20 if big else 300
    if args.warmup is None:
        args.warmup = 3 if big else 20

    if args.calibrate_copy:
        src = torch.zeros(512 << 20, dtype=torch.uint8, device=device)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    only = args.timed_region_only
    info = None if only else {}
    per_step, kern, nbytes, nsets, sets = time_fused(wl, b, cfg, device, args.steps, args.warmup, info=info)
    L = cfg.shard_len()
    # make sure the set the oracle is compared with holds this run's output
    if not only:
        launch(b, cfg, L, sets[0], 0)
        torch.cuda.synchronize()

    result = {
        "metric": "GB/s and gradient entries/s, fused RHT+masked reduce; % of HBM peak",
        "value": nbytes / per_step / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": per_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if cfg.dtype == "f32" else "bf16 in/out, f32 arithmetic",
        "data": "synthetic",
        "entries_per_s": cfg.workers * L / per_step,
        "pct_hbm_peak": 100.0 * nbytes / per_step / 1e9 / HBM_PEAK_GBPS,
        "config": {"workload": "%s-sized: N=%d workers, %s, P=%d, shard_len=%d, block 2^%d, %s drops %.0f%%"
                               % (cfg.name, cfg.workers, cfg.dtype, cfg.entries, L, cfg.block_log2, cfg.drops,
                                  cfg.loss * 100),
                   "entry_point": "or_fused_path" if cfg.dtype == "f32" else "or_fused_path_bf16",
                   "input_sets_rotated": nsets, "bytes_per_step": nbytes},
        "roofline": roofline(cfg, L, nbytes, kern),
        "timed_region": "one replay of a HIP graph holding the %d launches, in order, on one stream" % args.steps,
        "plain_launches_ms_per_step": None if only else info["plain_launches_ms_per_step"],
    }
    if only:
        print(json.dumps(result))
        return
    # The same launches when consecutive steps may overlap (independent buckets issued round-robin on
    # four streams): the ramp, tail and gap of single launches then hide under the neighbours.  Reported
    # beside `value`, which keeps the strict one-after-the-other order.
    streams = [torch.cuda.Stream() for _ in range(4)]
    def overlapped(n):
        for j in range(n):
            launch(b, cfg, L, sets[j % nsets], j % nsets % cfg.workers, streams[j % 4])
    overlapped(max(args.steps, 200))   # streams that are new to the runtime need a few hundred launches to settle
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    overlapped(args.steps)
    torch.cuda.synchronize()
    t4 = (time.perf_counter() - t0) / args.steps
    result["four_streams"] = {"GB_per_s": nbytes / t4 / 1e9, "ms_per_step": t4 * 1e3,
                              "frac_hbm_peak": nbytes / t4 / 1e9 / HBM_PEAK_GBPS,
                              "note": "steps issued round-robin on four streams, same inputs and launches"}
    result["three_call_path"] = time_three_calls(wl, b, cfg, sets)
    # last of the measurements on these inputs: dispatches that carry events switch the runtime's queues to a
    # slower, profiled mode for the rest of the process
    med, lo = kernel_only_seconds(b, cfg, L, sets)
    result["roofline"]["kernel_only_us_dispatch_events"] = med * 1e6      # median of 32 single dispatches
    result["roofline"]["kernel_only_us_dispatch_events_min"] = lo * 1e6
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl, b, cfg, sets)
    del sets
    torch.cuda.empty_cache()

    if not args.no_extra:
        extra = []
        for name, steps in (("tiny", 300), ("resnet50", 300), ("bert_large", 20), ("gpt2_xl", 3), ("llama_8b", 5)):
            if name == args.workload:
                continue
            c = wl.CONFIGS[name]
            try:
                if c.bucket_entries:
                    nb = len(c.buckets())
                    ps, kn, by, ns, st = time_fused(wl, b, c, device, steps, 1, entries=c.bucket_entries,
                                                    launches_per_step=nb)
                    by_step = by * nb   # the short last bucket is counted as a full one: a few % high on bytes AND time
                    ent = c.workers * c.shard_len(c.bucket_entries) * nb
                    note = "%d back-to-back launches of one 25 MiB bucket shape per step" % nb
                    extra.append({"workload": name + " (one launch per bucket)", "GB_per_s": by_step / ps / 1e9,
                                  "entries_per_s": ent / ps, "ms_per_step": ps * 1e3, "avg_launch_us": kn * 1e6,
                                  "launch_GB_per_s": by / kn / 1e9, "frac_hbm_peak": by / kn / 1e9 / HBM_PEAK_GBPS,
                                  "input_sets_rotated": ns, "note": note,
                                  "three_call_path_one_bucket": time_three_calls(
                                      wl, b, c, st, iters=20, L=c.shard_len(c.bucket_entries))})
                    # the same per-bucket launches spread over four streams: a bucket alone is ~100
                    # workgroups, so kernels of different buckets share the GPU (what a DDP hook that
                    # fires per bucket can do without waiting for the other buckets)
                    streams = [torch.cuda.Stream() for _ in range(4)]
                    Lb = c.shard_len(c.bucket_entries)
                    def spread(nsteps):
                        for j in range(nsteps * nb):
                            launch(b, c, Lb, st[j % ns], j % ns % c.workers, streams[j % 4])
                    spread(1)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    spread(steps)
                    torch.cuda.synchronize()
                    ps4 = (time.perf_counter() - t0) / steps
                    extra.append({"workload": name + " (one launch per bucket, four streams)",
                                  "GB_per_s": by_step / ps4 / 1e9, "entries_per_s": ent / ps4, "ms_per_step": ps4 * 1e3,
                                  "frac_hbm_peak": by_step / ps4 / 1e9 / HBM_PEAK_GBPS, "input_sets_rotated": ns,
                                  "note": "%d launches per step, round-robin over 4 streams" % nb})
                    # the same buckets through the batched entry points: up to 64 buckets per launch.  Inputs are
                    # the rotated sets; every bucket has outputs of its own (buckets of a call must not share any)
                    outs = torch.empty((nb, Lb), dtype=torch.float32, device=device)
                    cnts = torch.empty((nb, Lb), dtype=torch.uint8, device=device)
                    sums = torch.empty((nb, Lb), dtype=torch.float32, device=device)
                    arr = b.make_buckets([(st[j % ns][0], st[j % ns][1], outs[j], cnts[j], Lb, c.seed,
                                           (j % ns % c.workers) * Lb) for j in range(nb)])
                    sarr = b.make_stage_buckets([(st[j % ns][0], st[j % ns][1], sums[j], cnts[j], outs[j], Lb, c.seed,
                                                  (j % ns % c.workers) * Lb) for j in range(nb)])
                    reps = max(steps, 10)   # 1.5 ms a step: a few more for a steadier figure

                    def timed(fn):
                        for _ in range(2):
                            fn()
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        for _ in range(reps):
                            fn()
                        torch.cuda.synchronize()
                        return (time.perf_counter() - t0) / reps

                    N_, k_, Lall = c.workers, c.block_log2, Lb * nb
                    t_red = timed(lambda: b.or_masked_reduce_batched(sarr, nb, N_, False))
                    t_fdec = timed(lambda: b.or_finalize_decode_batched(sarr, nb, k_, False))
                    t_rdec = timed(lambda: b.or_reduce_decode_batched(arr, nb, N_, k_, False))
                    extra.append({"workload": name + " (separate calls, batched)",
                                  "masked_reduce_GB_per_s": (N_ * Lall * 4 + N_ * Lall // 8 + 5 * Lall) / t_red / 1e9,
                                  "finalize_decode_GB_per_s": Lall * 9 / t_fdec / 1e9,
                                  "reduce_decode_GB_per_s": by_step / t_rdec / 1e9,
                                  "note": "all %d buckets per call: or_masked_reduce_batched, or_finalize_decode_batched, "
                                          "or_reduce_decode_batched (%d launches each)" % (nb, -(-nb // 64))})
                    ps = timed(lambda: b.or_fused_path_batched(arr, nb, c.workers, c.block_log2, False))
                    kn = ps / -(-nb // 64)
                    by = by_step / -(-nb // 64)
                    note = "all %d buckets per step through or_fused_path_batched (%d launches)" % (nb, -(-nb // 64))
                    name = name + " (batched)"
                    del outs, cnts, sums
                else:
                    ps, kn, by, ns, st = time_fused(wl, b, c, device, steps, 2)
                    by_step, ent, note = by, c.workers * c.shard_len(), "one launch per step"
                row = {"workload": name, "GB_per_s": by_step / ps / 1e9, "entries_per_s": ent / ps,
                       "ms_per_step": ps * 1e3, "avg_launch_us": kn * 1e6,
                       "launch_GB_per_s": by / kn / 1e9, "frac_hbm_peak": by / kn / 1e9 / HBM_PEAK_GBPS,
                       "input_sets_rotated": ns, "note": note}
                if name == "tiny":
                    row["note"] = ("correctness configuration: %d input sets of %.1f MB stay in the 256 MB last-level "
                                   "cache, so this is not an HBM figure" % (ns, by / 1e6))
                    row["cache_resident"] = True
                if not c.bucket_entries:
                    row["three_call_path"] = time_three_calls(wl, b, c, st, iters=5 if by > (1 << 28) else 50)
                extra.append(row)
                del st
                torch.cuda.empty_cache()
            except Exception as exc:  # an extra workload must not take the headline down with it
                extra.append({"workload": name, "error": repr(exc)})
        result["other_workloads"] = extra

    print(json.dumps(result))


if __name__ == "__main__":
    main()

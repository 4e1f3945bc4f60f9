#!/usr/bin/env python3
"""Benchmark of the preemptible paged-KV decode + KV reclamation path on one MI355X.

One step = one pass of the whole path over one synthetic batch:
  for every layer: attention slices through the slice scheduler (+ merge) -> plan (host) and
  upload for the next decode step, overlapping the last layers in flight
  -> reclaim the highest-address range (relocation plan, chunked block copy, table
  rewrite, hand-over; enqueued behind the decode on the same stream) -> the online tenant
  returns the range and the pool bookkeeping is rewound so that every step does the same work
  (host-only, microseconds; the KV bytes themselves never move back because the copy leaves
  the sources intact).

With no --workload the run covers every timed configuration, one after the other in one
process: the largest single-GPU one (stress, 200 GiB pool) is the headline of the JSON line and
the others (llama8b, llama70b_tp8, offline_batch) are records of the same shape under
"workloads".  Prints ONE JSON line.  `value` is the algorithmic HBM bytes of a step (K+V bytes
read by attention in all layers + bytes read and written by the relocation) divided by the
wall time of a step, inputs resident in HBM.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published
HEADLINE = "stress"
EVENT_STRIDE = 8         # every so many launches inside the timed steps carry timing events (every 2nd: whole step -1..2 %)
CPU_SAMPLE_HEADLINE_FACTOR = 8.0 / 3.0   # the headline workload's oracle sample against the others'
# Run order of the default run, smallest pool first: a 40 or 64 GiB pool allocated after a 200 GiB one has
# been freed in the same process ran its kernels 5-6 % slower than in a fresh process (the same
# kernels, the same inputs); in this order every configuration measures what it does on its own.
ALL_WORKLOADS = ["llama8b", "llama70b_tp8", "offline_batch", "stress"]
T_BEGIN = time.time()


def progress(msg):
    """Phase marker on stderr (stdout carries the one JSON line only)."""
    print(f"[bench {time.time() - T_BEGIN:7.1f}s] {msg}", file=sys.stderr, flush=True)


def measured_traffic(workload: str):
    """(attention HBM bytes / algorithmic bytes, relocation HBM bytes / algorithmic bytes) from the
    committed counter run of this workload; an entry is None when there is no run or the kernel's
    source has changed since it was taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None, None
    kv = dict(l.split(":", 1) for l in open(path) if l.startswith(("attn_", "reloc_")))

    def sha(rel):
        return hashlib.sha256(open(os.path.join(ROOT, "paper_2604_07874_amd", "csrc", rel), "rb").read()).hexdigest()

    attn = reloc = None
    try:
        if kv.get("attn_source_sha256", "").strip() == sha("attn_kernel.inc"):
            attn = float(kv["attn_traffic_ratio"])
        if kv.get("reloc_source_sha256", "").strip() == sha("reclaim.hip"):
            reloc = float(kv["reloc_traffic_ratio"])
    except (KeyError, ValueError, OSError):
        pass
    return attn, reloc


def percentile(a, q):
    return float(np.percentile(np.asarray(a, dtype=np.float64), q)) if len(a) else None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="all",
                    help="one of the configurations, or 'all': the headline one and then the others as sub-records")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--chunk-tokens", type=int, default=None)
    ap.add_argument("--slice-bytes", type=int, default=None)
    ap.add_argument("--reclaim-chunk-bytes", type=int, default=None)
    ap.add_argument("--max-inflight", type=int, default=2)
    ap.add_argument("--yield-injections", type=int, default=1000)
    ap.add_argument("--concurrent-reclaim", dest="concurrent_reclaim", action="store_true", default=None,
                    help="extra leg: rate-capped, chunked reclamation on a second stream while decode runs "
                         "(default: on for workloads that define a rate cap)")
    ap.add_argument("--no-concurrent-reclaim", dest="concurrent_reclaim", action="store_false")
    ap.add_argument("--rate-cap", type=float, default=None, help="bytes/s for the concurrent leg")
    ap.add_argument("--overlap-slices", dest="overlap", action="store_true", default=None,
                    help="alternate the slices of a layer between two streams (default: on when a layer has more "
                         "than one slice)")
    ap.add_argument("--no-overlap-slices", dest="overlap", action="store_false")
    ap.add_argument("--arena", action="store_true",
                    help="pool memory from a handle-backed arena; the burst leg then unmaps the handed-over range "
                         "(physical memory back to the driver) and maps it again when the range is returned")
    ap.add_argument("--bursts", type=int, default=None,
                    help="extra leg: this many online bursts (yield, reclaim, hold, return) at exponential "
                         "inter-arrival times while decode runs continuously (default: 25 for the stress workload)")
    ap.add_argument("--burst-mean-s", type=float, default=0.2)
    ap.add_argument("--burst-hold-ms", type=float, default=20.0, help="mean time a burst keeps its memory")
    ap.add_argument("--burst-target-rate", type=float, default=4.0,
                    help="pressure events per second the MIAD controller is asked to stay under")
    ap.add_argument("--prefill-leg", dest="prefill_leg", action="store_true", default=None,
                    help="extra leg: causal prefill of the newest --prefill-tokens tokens of every sequence "
                         "(default: on for the llama8b workload)")
    ap.add_argument("--no-prefill-leg", dest="prefill_leg", action="store_false")
    ap.add_argument("--prefill-tokens", type=int, default=2048)
    ap.add_argument("--prefill-slice-bytes", type=int, default=768 << 20)
    ap.add_argument("--prefill-one-stream", action="store_true",
                    help="prefill leg without overlapped slices (then per-launch durations are additive)")
    ap.add_argument("--prefill-yield-injections", type=int, default=100)
    ap.add_argument("--prefill-chunk-tokens", type=int, default=8192)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-bytes", type=float, default=1.5e9,
                    help="K+V bytes of the sample the oracle is timed on, per workload (about 2.7 s of one core per GB); "
                         "the headline workload's sample is this times 8/3 (about 11 s)")
    ap.add_argument("--cpu-workers", type=int, default=min(16, os.cpu_count() or 1),
                    help="worker processes for the all-cores timing of the oracle (0 = skip it)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the bandwidth yardsticks")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    # The oracle's worker processes are started before anything touches the GPU: they are plain CPU
    # interpreters and must not be children forked from a process that has initialised it.
    workers = None
    if not args.no_cpu_baseline and args.cpu_workers > 1:
        import multiprocessing as mp
        try:
            workers = mp.get_context("spawn").Pool(args.cpu_workers, initializer=_oracle_worker_init)
            workers.map(_oracle_worker_ready, range(args.cpu_workers))
        except Exception as e:      # no worker processes here: the one-thread timing still runs
            print(f"bench.py: all-cores oracle timing skipped ({type(e).__name__}: {e})", file=sys.stderr)
            workers = None

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(torch.device("cuda:0"))

    names = ALL_WORKLOADS if args.workload == "all" else [args.workload]
    head_name = HEADLINE if args.workload == "all" else args.workload
    records = {}
    for name in names:
        progress(f"==== workload {name} ====")
        try:
            records[name] = run_workload(name, args, workers, headline=(name == head_name))
        except Exception as e:      # one configuration failing must not take the others' figures with it
            if name == head_name:
                raise
            records[name] = {"error": f"{type(e).__name__}: {e}"}
        import gc
        gc.collect()
        torch.cuda.empty_cache()
    if workers is not None:
        workers.close()
        workers.join()

    head = records[head_name]
    line = {
        "metric": "reclaim GB/s & paged-decode GB/s (% HBM peak); p99 yield latency us",
        "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
    }
    line.update({k: v for k, v in head.items() if k not in line})
    if len(names) > 1:
        line["workloads"] = {n: records[n] for n in names if n != head_name}
        line["summary"] = {n: {k: records[n].get(k) for k in
                               ("value", "frac_of_hbm_peak", "decode_GBps", "decode_frac_of_peak", "reclaim_traffic_GBps",
                                "reclaim_frac_of_peak", "yield_latency_us_p99")}
                           | {"attn_kernel_frac": (records[n].get("roofline") or {}).get("frac"),
                              "relocate_kernel_frac": (records[n].get("roofline_reclaim") or {}).get("frac")}
                           for n in names if "error" not in records[n]}
    print(json.dumps(line), flush=True)


def run_workload(name, args, workers, headline=True):
    """Everything for one configuration: inputs, timed steps, per-kernel figures, legs, oracle timing.
    Returns the record (the fields of the JSON line that belong to one workload)."""
    import torch
    import synth
    import paper_2604_07874_amd as vkv

    dev = torch.device("cuda:0")
    wl = synth.workload(name)
    g = wl.geom
    chunk_tokens = args.chunk_tokens or wl.chunk_tokens
    slice_bytes = args.slice_bytes or wl.slice_bytes
    rc_chunk = wl.chunk_bytes if args.reclaim_chunk_bytes is None else args.reclaim_chunk_bytes
    L, S = g.num_layers, wl.num_seqs
    prefill_leg = (wl.name == "llama8b") if args.prefill_leg is None else args.prefill_leg
    concurrent_leg = (wl.rate_cap > 0) if args.concurrent_reclaim is None else args.concurrent_reclaim
    n_bursts = (25 if wl.name == "stress" else 0) if args.bursts is None else args.bursts

    # ---- inputs, resident in HBM before anything is timed --------------------------
    t_setup = time.time()
    st = synth.build_state(wl, args.seed, materialize_pool=False)
    arena = None
    if args.arena:
        arena, span = vkv.kv_arena_create(0, g.blocks_per_handle * g.block_bytes, g.num_blocks // g.blocks_per_handle)
        pool_t = torch.as_tensor(span, device=dev)          # aliases the arena's address range, no copy
        assert pool_t.data_ptr() == span.address and pool_t.numel() == g.pool_elems
    else:
        pool_t = torch.empty(g.pool_elems, dtype=torch.int16, device=dev)
    progress(f"filling the {g.pool_bytes / 2**30:.0f} GiB pool on the device")
    fill_step = 1 << 34                                   # elements per progress line (32 GiB)
    for lo_e in range(0, g.pool_elems, fill_step):
        hi_e = min(g.pool_elems, lo_e + fill_step)
        synth.fill_pool_range_torch(pool_t, g, args.seed, lo_e, hi_e)
        torch.cuda.synchronize()
        progress(f"  filled {hi_e * 2 / 2**30:.0f} GiB")
    synth.poison_unused_slots(st, pool_t)
    q_all = torch.stack([torch.from_numpy(synth.query_bits(wl, args.seed, l).view(np.int16)) for l in range(L)]).to(dev)
    tables0 = torch.from_numpy(st.tables).to(dev)
    tables = tables0.clone()
    remap = torch.empty(g.num_blocks, dtype=torch.int32, device=dev)
    out = torch.empty((L, S, g.num_q_heads, g.head_dim), dtype=torch.float32, device=dev)
    pool = vkv.kv_pool_init(g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks,
                            g.blocks_per_handle, base=pool_t)
    vkv.kv_pool_adopt(pool, np.flatnonzero(st.live).astype(np.int32))
    if arena is not None:
        vkv.kv_pool_attach_arena(pool, arena)
    info = vkv.kv_attn_plan(pool, st.ctx_len, slice_bytes, chunk_tokens)
    overlap = (info.n_slices > 1) if args.overlap is None else bool(args.overlap)
    vkv.kv_sched_set_overlap(pool, overlap)
    ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device=dev)
    lo, hi = wl.reclaim_range
    remap_plan, plan_stats = vkv.kv_reclaim_plan(pool, lo, hi, g.num_blocks)
    src_ids = np.flatnonzero(remap_plan != np.arange(g.num_blocks)).astype(np.int32)
    dst_ids = remap_plan[src_ids].astype(np.int32)
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    stream = torch.cuda.current_stream()
    reclaim_launches = (len(src_ids) // max(1, rc_chunk // g.block_bytes) + 1) if rc_chunk else 1
    launches_per_step = L * info.n_slices + 2 + reclaim_launches
    # launches overlapped on two streams have durations that are not additive: they are timed in a
    # one-stream pass of their own after the timed steps
    events_in_steps = not overlap
    if events_in_steps:
        # every eighth launch carries timing events (the dispatch's own start and end: nothing is enqueued
        # around it), so the timed steps run as an untimed caller's would
        vkv.kv_profile_enable(pool, launches_per_step * (args.steps + 1) + 16)
        vkv.kv_profile_sample(pool, EVENT_STRIDE)

    def decode_pass():
        for layer in range(L):
            s_, cur = vkv.kv_attn_run_layer(pool, layer, 0, q_all[layer], tables, ws, out[layer],
                                            max_inflight=args.max_inflight, stream=stream)
            assert s_ == vkv.VKV_OK

    def rewind():
        # the online tenant gives the range back; rewind the bookkeeping so that every step does the same work
        vkv.kv_pool_return_range(pool, lo, hi)
        vkv.kv_pool_free(pool, dst_ids)
        vkv.kv_pool_adopt(pool, src_ids)
        tables.copy_(tables0, non_blocking=True)

    vkv.kv_attn_bind(pool, ws, stream)      # the plan made above, for the first step

    def step():
        decode_pass()
        # the plan of the next decode step is made and uploaded while the last layers of this one are
        # still running (the upload is ordered after them on the stream): one plan + bind per step
        vkv.kv_attn_plan(pool, st.ctx_len, slice_bytes, chunk_tokens)
        vkv.kv_attn_bind(pool, ws, stream)
        # the reclamation is enqueued behind the decode on the same stream, so every slice has finished
        # before the first block moves and nothing has to be waited for on the host: the next step's
        # slices are ordered behind the copy and the table rewrite in turn
        rs = vkv.kv_reclaim_range(pool, lo, hi, tables, remap, chunk_bytes=rc_chunk, copy_stream=stream,
                                  flags=vkv.VKV_RECLAIM_ASYNC)
        rewind()
        return rs

    progress("inputs resident; warm-up steps")
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if events_in_steps:
        vkv.kv_profile_read(pool, 1 << 20)   # drop warm-up records

    progress("timed steps")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        rs = step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    decode_bytes_layer = int(info.kv_bytes_per_layer)
    decode_bytes = decode_bytes_layer * L
    reclaim_traffic = 2 * int(rs.bytes_moved)
    step_bytes = decode_bytes + reclaim_traffic
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel figures from events recorded around every launch on its stream ----------
    if not events_in_steps:
        progress("one-stream pass with launch events (kernel durations)")
        vkv.kv_sched_set_overlap(pool, False)
        vkv.kv_profile_enable(pool, 3 * launches_per_step + 16)
        vkv.kv_profile_sample(pool, 1)
        decode_pass()
        decode_pass()
        vkv.kv_reclaim_range(pool, lo, hi, tables, remap, chunk_bytes=rc_chunk, copy_stream=stream)
        rewind()
        torch.cuda.synchronize()
    rec = vkv.kv_profile_read(pool, 1 << 20)
    vkv.kv_profile_enable(pool, 0)
    vkv.kv_sched_set_overlap(pool, overlap)
    sl = rec[rec["kind"] == vkv.VKV_PROF_SLICE]
    rl = rec[rec["kind"] == vkv.VKV_PROF_RELOCATE]
    rw = rec[rec["kind"] == vkv.VKV_PROF_REWRITE]
    slice_ms_avg = float(sl["ms"].mean())
    bytes_per_launch = decode_bytes_layer / info.n_slices
    ach = bytes_per_launch / (slice_ms_avg * 1e-3) / 1e9
    attn_ratio, reloc_ratio = measured_traffic(wl.name)
    roofline = {"kernel": "paged_decode_attn_slice_kernel", "bound": "hbm", "achieved": round(ach, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
                "traffic": None if attn_ratio is None else int(attn_ratio * bytes_per_launch),
                "avg_launch_us": round(slice_ms_avg * 1e3, 2),
                "bytes_per_launch": int(bytes_per_launch), "launches": int(len(sl)),
                "method": ((f"HIP events carried by every {EVENT_STRIDE}th launch inside the timed steps" if events_in_steps else
                            "HIP events carried by every launch of two one-stream passes after the timed steps (the timed "
                            "steps alternate slices between two streams, where durations are not additive)")
                           + "; hipExtLaunchKernelGGL start/stop events = the dispatch's own start and end")}
    roofline_reclaim = None
    if len(rl) and int(rl["index"].sum()) > 0:
        n_launches = int(rl["index"].sum())
        rl_ms = float(rl["ms"].sum())                    # all copy launches, gaps between them included
        per_launch_ms = rl_ms / n_launches
        per_launch_bytes = reclaim_traffic * len(rl) / n_launches
        rach = per_launch_bytes / (per_launch_ms * 1e-3) / 1e9
        roofline_reclaim = {"kernel": "kv_block_relocate_kernel", "bound": "hbm", "achieved": round(rach, 1),
                            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(rach / HBM_PEAK_GBPS, 4),
                            "traffic": None if reloc_ratio is None else int(reloc_ratio * per_launch_bytes),
                            "avg_launch_us": round(per_launch_ms * 1e3, 2),
                            "bytes_per_launch": int(per_launch_bytes), "launches": n_launches}
    extra = {
        "slice_us_p50": round(percentile(sl["ms"], 50) * 1e3, 1),
        "slice_us_p99": round(percentile(sl["ms"], 99) * 1e3, 1),
        "slice_us_max": round(float(sl["ms"].max()) * 1e3, 1),
        "rewrite_us_avg": round(float(rw["ms"].mean()) * 1e3, 2) if len(rw) else None,
    }

    # ---- yardsticks: what the memory system gives a sequential read and the runtime's own copy
    ceilings = None
    if not args.no_ceilings:
        progress("bandwidth yardsticks")

        def timed_ms(fn, reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fn(0)
            torch.cuda.synchronize()
            e0.record(stream)
            for i in range(reps):
                fn(i + 1)
            e1.record(stream)
            e1.synchronize()
            return e0.elapsed_time(e1) / reps

        pool_bytes = g.pool_elems * 2
        sink = torch.zeros(256, dtype=torch.uint8, device=dev)
        big = min(pool_bytes, 8 << 30) // 65536 * 65536
        launch_sized = int(bytes_per_launch) // 65536 * 65536
        n_regions = max(1, pool_bytes // launch_sized)
        base_addr = pool_t.data_ptr()
        read_big_ms = timed_ms(lambda i: vkv.kv_probe_read(base_addr, big, sink, stream), 4)
        read_launch_ms = timed_ms(lambda i: vkv.kv_probe_read(base_addr + (i % n_regions) * launch_sized, launch_sized,
                                                              sink, stream), 16)
        # the attention kernel's own reads without its arithmetic: slices of (up to 4) layers in turn
        probe_layers = min(L, 4)
        n_probe = probe_layers * info.n_slices
        probe_ms = timed_ms(lambda i: [vkv.kv_probe_attn_reads(pool, (i * 3 + l) % L, s_, tables, ws, sink, stream)
                                       for l in range(probe_layers) for s_ in range(info.n_slices)], 2) / n_probe
        cp_bytes = 1 << 30
        cp_a = torch.empty(cp_bytes, dtype=torch.uint8, device=dev)
        cp_b = torch.empty(cp_bytes, dtype=torch.uint8, device=dev)
        copy_ms = timed_ms(lambda i: vkv.kv_probe_copy(cp_b, cp_a, cp_bytes, stream), 4)
        del cp_a, cp_b
        # what a pair of timing events around one launch reads when the launch itself is next to nothing
        # (a 64 KiB read): the share of every per-launch figure above that is not the kernel
        br = []
        for _ in range(20):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            vkv.kv_probe_read(base_addr, 65536, sink, stream)
            e1.record(stream)
            e1.synchronize()
            br.append(e0.elapsed_time(e1) * 1e3)
        ceilings = {
            "event_pair_around_64KiB_read_us": round(float(np.median(br)), 2),
            "sequential_read_GBps": round(big / read_big_ms / 1e6, 1), "sequential_read_bytes": int(big),
            "sequential_read_at_launch_size_GBps": round(launch_sized / read_launch_ms / 1e6, 1),
            "launch_size_bytes": int(launch_sized),
            "attention_reads_only_GBps": round(bytes_per_launch / probe_ms / 1e6, 1),
            "runtime_copy_traffic_GBps": round(2 * cp_bytes / copy_ms / 1e6, 1), "copy_bytes": cp_bytes,
        }
        roofline["frac_of_read_ceiling_at_launch_size"] = round(
            roofline["achieved"] / ceilings["sequential_read_at_launch_size_GBps"], 4)
        roofline["frac_of_own_reads_only"] = round(roofline["achieved"] / ceilings["attention_reads_only_GBps"], 4)
        if roofline_reclaim is not None:
            roofline_reclaim["frac_of_runtime_copy"] = round(
                roofline_reclaim["achieved"] / ceilings["runtime_copy_traffic_GBps"], 4)

    progress("decode-only and reclaim-only legs")
    # ---- separate legs: decode only, reclaim only (wall clock, no launch events) ----
    reps = max(3, min(args.steps, 10))
    decode_pass()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        decode_pass()
    torch.cuda.synchronize()
    decode_ms = (time.perf_counter() - t0) * 1e3 / reps
    reclaim_ms = []
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        vkv.kv_reclaim_range(pool, lo, hi, tables, remap, chunk_bytes=rc_chunk, copy_stream=stream)
        reclaim_ms.append((time.perf_counter() - t0) * 1e3)
        rewind()
    torch.cuda.synchronize()
    reclaim_ms_med = float(np.median(reclaim_ms))
    extra.update({
        "decode_GBps": round(decode_bytes / (decode_ms * 1e-3) / 1e9, 1),
        "decode_frac_of_peak": round(decode_bytes / (decode_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "decode_ms_all_layers": round(decode_ms, 3),
        "decode_tokens_per_s": round(S / (decode_ms * 1e-3), 1),
        "reclaim_traffic_GBps": round(reclaim_traffic / (reclaim_ms_med * 1e-3) / 1e9, 1),
        "reclaim_frac_of_peak": round(reclaim_traffic / (reclaim_ms_med * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "reclaimed_GBps": round((hi - lo) * g.block_bytes / (reclaim_ms_med * 1e-3) / 1e9, 1),
        "reclaim_ms": round(reclaim_ms_med, 3),
        "reclaim_blocks_moved": int(rs.blocks_moved),
    })

    # ---- end-to-end yield latency: request at a random instant, until compute is off the GPU
    if args.yield_injections > 0:
        progress("yield injections")
        rng = np.random.default_rng(args.seed)
        lat = []
        req_t = [0.0]

        def requester(delay):
            time.sleep(delay)
            req_t[0] = time.perf_counter()
            vkv.kv_yield_request(pool)

        layer = 0
        cur = 0
        budget_s = 20.0
        t_begin = time.time()
        for i in range(args.yield_injections):
            if time.time() - t_begin > budget_s:
                break
            delay = float(rng.uniform(0.0, min(decode_ms, 10.0) * 1e-3))
            th = threading.Thread(target=requester, args=(delay,))
            th.start()
            landed = None
            while landed is None:
                s_, cur = vkv.kv_attn_run_layer(pool, layer, cur, q_all[layer], tables, ws, out[layer],
                                                max_inflight=args.max_inflight, stream=stream)
                if s_ == vkv.VKV_YIELDED:
                    landed = time.perf_counter()
                else:
                    layer = (layer + 1) % L
                    cur = 0
            th.join()
            lat.append((landed - req_t[0]) * 1e6)
            vkv.kv_yield_clear(pool)
        torch.cuda.synchronize()
        # finish the layer the last injection interrupted (a started layer must be finished or rebound)
        vkv.kv_attn_bind(pool, ws, stream)
        extra.update({"yield_latency_us_p50": round(percentile(lat, 50), 1),
                      "yield_latency_us_p99": round(percentile(lat, 99), 1),
                      "yield_latency_us_max": round(max(lat), 1), "yield_injections": len(lat)})

    # ---- optional: reclamation under a rate cap on a second stream while decode keeps running
    def concurrent_leg_run():
        progress("concurrent rate-capped reclamation leg")
        cap = args.rate_cap or wl.rate_cap or 20e9
        cchunk = rc_chunk or (64 << 20)
        decode_stream, copy_stream = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        stop = threading.Event()
        marks = []          # (time, layers finished) samples from the decode thread

        thread_error = []

        def decode_forever():
            n = 0
            try:
                while not stop.is_set():
                    for layer in range(L):
                        vkv.kv_attn_run_layer(pool, layer, 0, q_all[layer], tables, ws, out[layer],
                                              max_inflight=args.max_inflight, stream=decode_stream)
                        n += 1
                    decode_stream.synchronize()
                    marks.append((time.perf_counter(), n))
            except BaseException as e:      # the main thread polls `marks`: it must learn that none will come
                thread_error.append(e)

        def wait_for(cond):
            while not cond():
                if thread_error:
                    raise RuntimeError(f"decode thread failed: {thread_error[0]!r}")
                time.sleep(0.001)

        th = threading.Thread(target=decode_forever)
        th.start()
        try:
            wait_for(lambda: len(marks) >= 2)
            t_a, n_a = marks[-1]
            crs = vkv.kv_reclaim_range(pool, lo, hi, tables, remap, chunk_bytes=cchunk, rate_cap_bytes_per_s=int(cap),
                                       copy_stream=copy_stream, decode_stream=decode_stream)
            wait_for(lambda: marks[-1][0] >= t_a + crs.host_seconds)
            t_b, n_b = marks[-1]
        finally:
            stop.set()
            th.join()
        torch.cuda.synchronize()
        rewind()
        torch.cuda.synchronize()
        extra.update({
            "concurrent_rate_cap_GBps": cap / 1e9,
            "concurrent_reclaim_achieved_GBps": round(crs.bytes_moved / crs.host_seconds / 1e9, 2),
            "concurrent_reclaim_ms": round(crs.host_seconds * 1e3, 2),
            "concurrent_reclaim_launches": int(crs.n_chunks),
            "concurrent_decode_GBps": round((n_b - n_a) * decode_bytes_layer / (t_b - t_a) / 1e9, 1),
            "concurrent_decode_frac_of_peak": round((n_b - n_a) * decode_bytes_layer / (t_b - t_a) / 1e9 / HBM_PEAK_GBPS, 4),
        })

    if concurrent_leg:
        try:
            concurrent_leg_run()
        except Exception as e:      # an extra leg must not take the workload's record down with it
            extra["concurrent_error"] = f"{type(e).__name__}: {e}"
            torch.cuda.synchronize()

    # ---- optional: online bursts against a continuous offline decode loop --------------------
    if n_bursts > 0:
        try:
            extra.update(burst_leg(vkv, args, wl, pool, pool_t, arena, st, q_all, tables, tables0, ws, out, remap, lo, hi,
                                   rc_chunk, src_ids, dst_ids, decode_bytes_layer, int(rs.bytes_moved), n_bursts))
        except Exception as e:      # an extra leg must not take the headline line down with it
            extra["burst_error"] = f"{type(e).__name__}: {e}"
            vkv.kv_yield_clear(pool)
            torch.cuda.synchronize()

    # ---- optional: preemptible causal prefill over the same pool (MFMA-bound) -------------
    if prefill_leg:
        progress("prefill leg")
        try:
            extra.update(prefill_leg_run(vkv, args, wl, pool, pool_t, st, tables, stream, overlap))
        except Exception as e:      # an extra leg must not take the headline line down with it
            extra["prefill_error"] = f"{type(e).__name__}: {e}"
            vkv.kv_yield_clear(pool)

    # ---- the CPU oracle on a bounded sample of the same workload --------------------
    cpu_baseline = None
    if not args.no_cpu_baseline:
        progress("CPU oracle baseline")
        try:
            cpu_baseline = cpu_oracle_baseline(wl, st, pool_t, q_all, decode_bytes, reclaim_traffic,
                                               args.cpu_baseline_bytes * (CPU_SAMPLE_HEADLINE_FACTOR if headline else 1.0),
                                               workers, args.cpu_workers)
        except Exception as e:      # the GPU figures above stand on their own
            cpu_baseline = {"error": f"{type(e).__name__}: {e}", "kind": "oracle"}

    vkv.kv_pool_destroy(pool)
    if arena is not None:
        del pool_t
        vkv.kv_arena_destroy(arena)
    record = {
        "value": round(value, 1), "unit": "GB/s", "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": (f"{wl.name}: L={L} Hq={g.num_q_heads} Hkv={g.num_kv_heads} D={g.head_dim} "
                                f"block={g.block_tokens} batch={S} ctx={wl.ctx_dist} pool={g.pool_bytes / 2**30:.1f}GiB "
                                f"occupancy={wl.occupancy} reclaim_top={(hi - lo) * g.block_bytes / 2**30:.2f}GiB"),
                   "chunk_tokens": chunk_tokens, "slice_bytes": slice_bytes, "n_slices_per_layer": info.n_slices,
                   "n_items_per_layer": info.n_items, "reclaim_chunk_bytes": rc_chunk,
                   "max_inflight": args.max_inflight, "overlap_slices": bool(overlap),
                   "arena": bool(args.arena), "seed": args.seed},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "step_bytes": step_bytes, "decode_bytes": decode_bytes, "reclaim_traffic_bytes": reclaim_traffic,
        "setup_s": round(setup_s, 1),
        "roofline": roofline, "roofline_reclaim": roofline_reclaim, "cpu_baseline": cpu_baseline,
        "ceilings": ceilings,
    }
    record.update(extra)
    return record


def burst_leg(vkv, args, wl, pool, pool_t, arena, st, q_all, tables, tables0, ws, out, remap, lo, hi, rc_chunk,
              src_ids, dst_ids, decode_bytes_layer, moved_bytes, n_bursts):
    """Online bursts against a continuous offline decode loop, with the online tenant's headroom kept by
    the MIAD controller (Section 5): bursts of 16 GiB-style demand arrive at exponential gaps and last
    an exponential time; at every arrival, departure and tick the controller sees the handles in use.
    A pressure event (use >= 90 % of the headroom) grows the headroom: offline compute yields, the
    highest run of handles still with the offline job is emptied by relocation or, when no room is
    left, the handles Algorithm 1 picks are evicted, and offline resumes.  Without pressure the
    controller gives one handle back per interval; the offline job moves back into it (the moves
    out of that handle are undone in the block tables; the copy had left the sources intact)."""
    import torch
    g = wl.geom
    L, S = g.num_layers, wl.num_seqs
    dev = pool_t.device
    bph, nb = g.blocks_per_handle, g.num_blocks
    n_handles = nb // bph
    burst_handles = (hi - lo) // bph
    progress(f"burst leg: {n_bursts} bursts of {burst_handles} handles, headroom by the MIAD controller")
    brng = np.random.default_rng(args.seed + 1)
    arrivals = np.cumsum(brng.exponential(args.burst_mean_s, size=n_bursts))
    holds = brng.exponential(args.burst_hold_ms * 1e-3, size=n_bursts)
    miad_cfg = dict(h_init=burst_handles + burst_handles // 8, h_min=max(1, burst_handles // 8),
                    h_max=min(n_handles // 2, 3 * burst_handles), alpha=1.25, pressure_frac=0.9,
                    t_init=0.004, t_min=0.001, t_max=0.25, t_up=2.0, t_down=0.001, window_s=2.0,
                    target_rate=float(args.burst_target_rate))
    miad = vkv.kv_miad_init(**miad_cfg)
    decode_stream, copy_stream = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    stop = threading.Event()
    cv = threading.Condition()
    gate = {"want_pause": False, "paused": False, "restart_layer": False}    # only change under cv
    layers_done = [0]
    ctx = st.ctx_len.copy()
    tables_host = st.tables.copy()
    cost = np.array([int((tables_host[r] >= 0).sum()) * 16 for r in range(tables_host.shape[0])], dtype=np.int64)
    cost[:S] = ctx
    plan_box = [vkv.kv_attn_plan(pool, ctx, args.slice_bytes or wl.slice_bytes, args.chunk_tokens or wl.chunk_tokens)]
    vkv.kv_attn_bind(pool, ws, decode_stream)
    vkv.kv_attn_run_layer(pool, 0, 0, q_all[0], tables, ws, out[0], max_inflight=args.max_inflight, stream=decode_stream)
    decode_stream.synchronize()
    before = out[0].clone()
    bytes_layer = [int(plan_box[0].kv_bytes_per_layer)]
    decoded_bytes = [0]

    offline_error = []

    def offline():
        try:
            offline_loop()
        except BaseException as e:      # the main thread must not wait for a thread that is gone
            offline_error.append(e)
            with cv:
                gate["paused"] = True
                cv.notify_all()

    def offline_loop():
        layer, cur = 0, 0
        while not stop.is_set():
            with cv:
                while gate["want_pause"] and not stop.is_set():
                    gate["paused"] = True          # nothing of ours is on the GPU: every call below
                    cv.notify_all()                # returns only after its launches have drained
                    cv.wait(0.05)
                gate["paused"] = False
                if gate["restart_layer"]:          # the batch was planned anew while we were off the GPU
                    gate["restart_layer"] = False
                    cur = 0
            if plan_box[0].n_slices == 0:
                time.sleep(0.001)
                continue
            s_, cur = vkv.kv_attn_run_layer(pool, layer, cur, q_all[layer], tables, ws, out[layer],
                                            max_inflight=args.max_inflight, stream=decode_stream)
            if s_ != vkv.VKV_YIELDED:
                layers_done[0] += 1
                decoded_bytes[0] += bytes_layer[0]
                layer, cur = (layer + 1) % L, 0
        decode_stream.synchronize()

    reserved = np.zeros(n_handles, dtype=bool)      # handles with the online tenant
    units = []                                      # handed-over handles, newest last: (handle, src ids, dst ids)
    stats = {"grow_events": 0, "relocations": 0, "evictions": 0, "evicted_requests": 0, "evicted_cost": 0,
             "fifo_cost": 0, "moved_bytes": 0, "released_handles": 0}
    grow_ms, idle_ms, paused_s = [], [], [0.0]
    reloc_ms, evict_ms, reloc_handles, evict_handles, all_gone = [], [], [], [], []
    pending = []                                    # evicted requests of the batch waiting to be taken back
    readmit = {"events": 0, "requests": 0, "tokens_to_recompute": 0, "last_t": 0.0}
    nblk_of = -(-st.ctx_len.astype(np.int64) // g.block_tokens)
    ident = torch.arange(nb, dtype=torch.int32, device=dev)

    def pause_offline():
        t_req = time.perf_counter()
        with cv:
            gate["want_pause"] = True
        vkv.kv_yield_request(pool)
        with cv:
            while not gate["paused"]:
                cv.wait(1.0)
                if offline_error:
                    raise RuntimeError(f"offline decode thread failed: {offline_error[0]!r}")
        if offline_error:
            raise RuntimeError(f"offline decode thread failed: {offline_error[0]!r}")
        return t_req, time.perf_counter()

    def resume_offline(t_req):
        vkv.kv_yield_clear(pool)
        paused_s[0] += time.perf_counter() - t_req
        with cv:
            gate["want_pause"] = False
            cv.notify_all()

    def top_run(n):
        """Highest run of n consecutive handles still with the offline job, as a block range."""
        run = 0
        for h in range(n_handles - 1, -1, -1):
            run = run + 1 if not reserved[h] else 0
            if run == n:
                return h * bph, (h + n) * bph
        return None

    def grow(n, timed=True):
        rng_ = top_run(n)
        if rng_ is None:
            return False
        rlo, rhi = rng_
        t_req, t_idle = pause_offline() if timed else (time.perf_counter(),) * 2
        try:
            remap_plan = None
            try:
                remap_plan, _ = vkv.kv_reclaim_plan(pool, rlo, rhi, nb)
            except vkv.VkvError as e:
                if e.code != vkv.VKV_E_NOSPACE:
                    raise
                # what first-in-first-out eviction of as many handles would have cost (Section 7.2)
                fifo = np.flatnonzero(~reserved)[:n].astype(np.int32)
                stats["fifo_cost"] += vkv.kv_handles_cost(pool, tables_host, cost, fifo)[1]
            info, rs, handles, evicted, _ = vkv.kv_reclaim_or_evict(
                pool, rlo, rhi, tables, tables_host, cost, remap, chunk_bytes=rc_chunk, copy_stream=copy_stream,
                decode_stream=decode_stream)
            if info.mode == 0:
                src = np.flatnonzero(remap_plan != np.arange(nb)).astype(np.int32)
                dst = remap_plan[src].astype(np.int32)
                for h in range(rhi // bph - 1, rlo // bph - 1, -1):     # top handle first, so that giving back
                    m = (src // bph) == h                                  # starts at the boundary
                    # with the arena the handle's memory really goes away: its blocks stay where they were moved
                    units.append((h, src[m], dst[m]) if arena is None else (h, None, None))
                    reserved[h] = True
                stats["relocations"] += 1
                stats["moved_bytes"] += int(rs.bytes_moved)
            else:
                for h in handles.tolist():
                    units.append((int(h), None, None))
                    reserved[int(h)] = True
                stats["evictions"] += 1
                stats["evicted_requests"] += int(info.n_evicted)
                stats["evicted_cost"] += int(info.total_cost)
                gone = [r for r in evicted.tolist() if r < S]
                all_gone.extend(gone)
                pending.extend(gone)
                if gone:
                    # the evicted requests leave the batch; the next slices follow a new plan
                    ctx[gone] = 0
                    plan_box[0] = vkv.kv_attn_plan(pool, ctx, args.slice_bytes or wl.slice_bytes,
                                                   args.chunk_tokens or wl.chunk_tokens)
                    bytes_layer[0] = int(plan_box[0].kv_bytes_per_layer)
                    vkv.kv_attn_bind(pool, ws, decode_stream)
                    with cv:
                        gate["restart_layer"] = True
            t_done = time.perf_counter()
            if timed:
                grow_ms.append((t_done - t_req) * 1e3)
                idle_ms.append((t_idle - t_req) * 1e3)
                stats["grow_events"] += 1
                (evict_ms if info.mode else reloc_ms).append((t_done - t_idle) * 1e3)
                (evict_handles if info.mode else reloc_handles).append(n)
            if arena is not None:
                for h, _, _ in units[-n:]:
                    vkv.kv_arena_release(arena, pool, h * bph, (h + 1) * bph)
        finally:
            if timed:
                resume_offline(t_req)
        return True

    def release_one():
        """The newest handed-over handle goes back; the offline job's blocks return to it."""
        if not units:
            return
        h, src, dst = units.pop()
        if arena is not None:
            vkv.kv_arena_restore(arena, pool, h * bph, (h + 1) * bph)
        vkv.kv_pool_return_range(pool, h * bph, (h + 1) * bph)
        reserved[h] = False
        stats["released_handles"] += 1
        if src is not None and len(src):
            # a request evicted since then took its blocks with it: nothing of it moves back
            kept = np.isin(dst, tables_host[tables_host >= 0])
            src, dst = src[kept], dst[kept]
        if src is not None and len(src):
            # undo the moves out of this handle: the sources were left intact, so only bookkeeping and tables change.
            # Slices in flight may read either copy (same bytes); the old destinations are freed, not overwritten.
            vkv.kv_pool_free(pool, dst)
            vkv.kv_pool_adopt(pool, src)
            inv = ident.clone()
            inv[torch.from_numpy(dst).to(dev).long()] = torch.from_numpy(src).to(dev)
            with torch.cuda.stream(copy_stream):
                vkv.block_table_rewrite(tables, inv, nb, stream=copy_stream)
            back = np.arange(nb, dtype=np.int32)
            back[dst] = src
            used = tables_host >= 0
            tables_host[used] = back[tables_host[used]]
            copy_stream.synchronize()

    def readmit_some(now):
        """Evicted requests come back once the online tenant has let go of enough memory: fresh blocks, their
        table rows filled in, the plan made anew.  Their KV has to be recomputed (the paper's cost of an
        eviction); here only its size is counted."""
        if not pending or now - readmit["last_t"] < 0.010:
            return
        readmit["last_t"] = now
        live_now, _ = vkv.kv_pool_state(pool, nb, max_ranges=1)
        free = int(((live_now == 0) & ~np.repeat(reserved, bph)).sum())
        room = free - nb // 50                       # two per cent of the pool stay free
        take, need = [], 0
        for r in pending[:64]:
            if need + int(nblk_of[r]) > room:
                break
            take.append(r)
            need += int(nblk_of[r])
        if not take:
            return
        t_req, _ = pause_offline()
        try:
            ids = vkv.kv_pool_alloc(pool, need)
            at = 0
            for r in take:
                n = int(nblk_of[r])
                tables_host[r, :n] = ids[at:at + n]
                at += n
                ctx[r] = st.ctx_len[r]
                cost[r] = ctx[r]
            rows_t = torch.tensor(take, device=dev)
            tables[rows_t] = torch.from_numpy(tables_host[take]).to(dev)
            torch.cuda.synchronize()
            del pending[:len(take)]
            plan_box[0] = vkv.kv_attn_plan(pool, ctx, args.slice_bytes or wl.slice_bytes,
                                           args.chunk_tokens or wl.chunk_tokens)
            bytes_layer[0] = int(plan_box[0].kv_bytes_per_layer)
            vkv.kv_attn_bind(pool, ws, decode_stream)
            with cv:
                gate["restart_layer"] = True
            readmit["events"] += 1
            readmit["requests"] += len(take)
            readmit["tokens_to_recompute"] += int(st.ctx_len[take].sum())
        finally:
            resume_offline(t_req)

    # the initial headroom is taken before anything is timed (also creates the queues of the two new streams)
    h0 = vkv.kv_miad_observe(miad, 0.0, 0)[0]
    grow(h0, timed=False)
    th = threading.Thread(target=offline)
    t_start = time.perf_counter()
    th.start()
    timeline = sorted([(float(a), +1) for a in arrivals] + [(float(a + h), -1) for a, h in zip(arrivals, holds)])
    tick_s = 0.002
    active, k_ev, n_pressure, headroom_trace = 0, 0, 0, []
    served_late = 0
    t_end = timeline[-1][0] + 0.05
    try:
        while True:
            now = time.perf_counter() - t_start
            if now >= t_end or offline_error:
                break
            nxt = timeline[k_ev][0] if k_ev < len(timeline) else t_end
            wait = min(nxt, now + tick_s) - now
            if wait > 0:
                time.sleep(wait)
            now = time.perf_counter() - t_start
            while k_ev < len(timeline) and timeline[k_ev][0] <= now:
                active += timeline[k_ev][1]
                k_ev += 1
            used_h = active * burst_handles
            for _ in range(32):                       # the controller until it has nothing more to ask for
                H, grow_by, release, event, T = vkv.kv_miad_observe(miad, time.perf_counter() - t_start, used_h)
                n_pressure += event
                if grow_by > 0:
                    if not grow(grow_by):
                        break
                    continue                          # pressure may persist: the next observation decides
                if release:
                    release_one()
                break
            headroom_trace.append(H)
            if used_h > H:
                served_late += 1
            if active == 0:
                readmit_some(time.perf_counter() - t_start)
    finally:
        # whatever happened, the decode thread is stopped and nothing of it is left on the GPU
        stop.set()
        vkv.kv_yield_clear(pool)
        with cv:
            gate["want_pause"] = False
            cv.notify_all()
        th.join()
    if offline_error:
        raise RuntimeError(f"offline decode thread failed: {offline_error[0]!r}")
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t_start
    # everything goes back, newest first, so that the pool ends as it began (bar the evicted requests)
    while units:
        release_one()
    vkv.kv_miad_destroy(miad)
    if arena is None:
        # requests that were evicted and taken back sit in blocks of their own: those go first
        for r in sorted(set(all_gone)):
            mine = tables_host[r][tables_host[r] >= 0]
            if len(mine):
                vkv.kv_pool_free(pool, mine)
                tables_host[r] = -1
        # the evicted requests come back for the legs that follow: their blocks were freed, never overwritten
        live_now, _ = vkv.kv_pool_state(pool, nb)
        vkv.kv_pool_adopt(pool, np.flatnonzero(st.live.astype(bool) & ~live_now.astype(bool)).astype(np.int32))
        tables.copy_(tables0)
        vkv.kv_attn_plan(pool, st.ctx_len, args.slice_bytes or wl.slice_bytes, args.chunk_tokens or wl.chunk_tokens)
    else:
        # handles that were unmapped came back as fresh memory: the blocks stay where the relocations put
        # them, the tables say so, and the evicted requests stay out
        vkv.kv_attn_plan(pool, ctx, args.slice_bytes or wl.slice_bytes, args.chunk_tokens or wl.chunk_tokens)
    vkv.kv_attn_bind(pool, ws, torch.cuda.current_stream())
    vkv.kv_attn_run_layer(pool, 0, 0, q_all[0], tables, ws, out[0], max_inflight=args.max_inflight,
                          stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    # the requests that stayed compute the same bits as before the bursts; the evicted ones lost their KV for good
    stayed = torch.ones(S, dtype=torch.bool, device=dev)
    if all_gone:
        stayed[torch.tensor(sorted(set(all_gone)), device=dev)] = False
    same_bits = bool(torch.equal(out[0][stayed].view(torch.int32), before[stayed].view(torch.int32)))
    run_s = max(1e-9, total_s - paused_s[0])
    res = {
        "bursts": int(n_bursts), "burst_handles": int(burst_handles), "burst_bytes": int((hi - lo) * g.block_bytes),
        "burst_mean_interarrival_s": args.burst_mean_s, "burst_mean_hold_ms": args.burst_hold_ms,
        "burst_run_s": round(total_s, 2), "burst_survivors_bits_unchanged_afterwards": same_bits,
        "miad": {**miad_cfg, "pressure_events": int(n_pressure),
                 "pressure_events_per_s": round(n_pressure / total_s, 3),
                 "headroom_handles_mean": round(float(np.mean(headroom_trace)), 1) if headroom_trace else None,
                 "headroom_handles_max": int(max(headroom_trace)) if headroom_trace else None,
                 "observations_with_use_above_headroom": int(served_late)},
        "burst_grow_events": stats["grow_events"], "burst_relocations": stats["relocations"],
        "burst_evictions": stats["evictions"], "burst_evicted_requests": stats["evicted_requests"],
        "burst_evicted_cost_tokens": stats["evicted_cost"], "burst_fifo_cost_tokens": stats["fifo_cost"],
        "burst_moved_bytes_total": stats["moved_bytes"], "burst_released_handles": stats["released_handles"],
        "burst_requests_taken_back": readmit["requests"], "burst_take_back_events": readmit["events"],
        "burst_tokens_to_recompute": readmit["tokens_to_recompute"], "burst_requests_still_out": len(pending),
        "burst_yield_to_idle_ms_p50": round(percentile(idle_ms, 50), 3) if idle_ms else None,
        "burst_yield_to_idle_ms_p99": round(percentile(idle_ms, 99), 3) if idle_ms else None,
        "burst_request_to_handed_over_ms_p50": round(percentile(grow_ms, 50), 3) if grow_ms else None,
        "burst_request_to_handed_over_ms_p99": round(percentile(grow_ms, 99), 3) if grow_ms else None,
        "burst_request_to_handed_over_ms_max": round(max(grow_ms), 3) if grow_ms else None,
        "burst_relocation_ms_max": round(max(reloc_ms), 3) if reloc_ms else None,
        "burst_relocation_handles_max": int(max(reloc_handles)) if reloc_handles else None,
        "burst_eviction_ms": [round(x, 3) for x in evict_ms], "burst_eviction_handles": [int(x) for x in evict_handles],
        "burst_offline_paused_frac": round(paused_s[0] / total_s, 4),
        "burst_decode_GBps_whole_run": round(decoded_bytes[0] / total_s / 1e9, 1),
        "burst_decode_GBps_while_running": round(decoded_bytes[0] / run_s / 1e9, 1),
    }
    return res


def prefill_leg_run(vkv, args, wl, pool, pool_t, st, tables, stream, decode_overlap):
    """Preemptible causal prefill of the newest tokens of every sequence over the same pool."""
    import torch
    g = wl.geom
    L = g.num_layers
    dev = pool_t.device
    res = {}
    q_len = np.minimum(st.ctx_len, args.prefill_tokens).astype(np.int32)
    pinfo = vkv.kv_prefill_plan(pool, st.ctx_len, q_len, args.prefill_slice_bytes, args.prefill_chunk_tokens)
    pws = torch.empty(pinfo.workspace_bytes, dtype=torch.uint8, device=dev)
    vkv.kv_prefill_bind(pool, pws, stream)
    pq = torch.empty((pinfo.total_q, g.num_q_heads, g.head_dim), dtype=torch.int16, device=dev)
    # query values: the generator's bits at the start of the pool serve as well as any
    pq.view(-1).copy_(pool_t[:pq.numel()])
    pout = torch.empty((pinfo.total_q, g.num_q_heads, g.head_dim), dtype=torch.float32, device=dev)
    p_overlap = not args.prefill_one_stream
    vkv.kv_sched_set_overlap(pool, p_overlap)
    vkv.kv_profile_enable(pool, (pinfo.n_slices + pinfo.n_merge_steps) * 8 + 16)
    n_layers_p = min(L, 2)
    # warm-up: the first passes over a layer's K/V run 5-7 % slower than the later ones
    for _ in range(4):
        for layer in range(n_layers_p):
            vkv.kv_prefill_run_layer(pool, layer, 0, pq, tables, pws, pout, max_inflight=args.max_inflight, stream=stream)
    torch.cuda.synchronize()
    vkv.kv_profile_read(pool, 1 << 20)
    reps = 3
    t0 = time.perf_counter()
    for _ in range(reps):
        for layer in range(n_layers_p):
            vkv.kv_prefill_run_layer(pool, layer, 0, pq, tables, pws, pout, max_inflight=args.max_inflight, stream=stream)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / (n_layers_p * reps)
    rec = vkv.kv_profile_read(pool, 1 << 20)
    psl = rec[rec["kind"] == vkv.VKV_PROF_PREFILL]
    pmg = rec[rec["kind"] == vkv.VKV_PROF_PREFILL_MERGE]
    vkv.kv_profile_enable(pool, 0)
    # overlapped launches: per-launch durations are not additive, rate by the wall clock instead
    kern_s = dt if p_overlap else float(psl["ms"].sum()) * 1e-3 / (n_layers_p * reps)
    res.update({
        "prefill_rows": int(pinfo.total_q), "prefill_slices_per_layer": int(pinfo.n_slices),
        "prefill_items_per_layer": int(pinfo.n_items), "prefill_merge_steps_per_layer": int(pinfo.n_merge_steps),
        "prefill_overlapped_slices": p_overlap,
        "prefill_slice_bytes": args.prefill_slice_bytes, "prefill_chunk_tokens": args.prefill_chunk_tokens,
        "prefill_TFLOPs_wall": round(pinfo.flops_per_layer / dt / 1e12, 1),
        "prefill_TFLOPs_kernel": None if p_overlap else round(pinfo.flops_per_layer / kern_s / 1e12, 1),
        "prefill_frac_of_mfma_bf16_peak": round(pinfo.flops_per_layer / kern_s / 2.5e15, 4),
        "prefill_ms_per_layer": round(dt * 1e3, 3),
        "prefill_slice_us_p50": round(percentile(psl["ms"], 50) * 1e3, 1),
        "prefill_slice_us_p99": round(percentile(psl["ms"], 99) * 1e3, 1),
        "prefill_kv_GBps": round(pinfo.kv_bytes_per_layer / kern_s / 1e9, 1),
        "prefill_merge_us_per_layer": round(float(pmg["ms"].sum()) * 1e3 / (n_layers_p * reps), 1),
        "prefill_merge_step_us_max": round(float(pmg["ms"].max()) * 1e3, 1) if len(pmg) else None,
    })
    # yield latency of a prefill: request at a random instant of a layer, until compute is off the GPU
    if args.prefill_yield_injections > 0:
        prng = np.random.default_rng(args.seed + 2)
        plat, preq = [], [0.0]

        def prequester(delay):
            time.sleep(delay)
            preq[0] = time.perf_counter()
            vkv.kv_yield_request(pool)

        layer, cur, t_begin = 0, 0, time.time()
        for _ in range(args.prefill_yield_injections):
            if time.time() - t_begin > 20.0:
                break
            th = threading.Thread(target=prequester, args=(float(prng.uniform(0.0, dt)),))
            th.start()
            landed = None
            while landed is None:
                s_, cur = vkv.kv_prefill_run_layer(pool, layer, cur, pq, tables, pws, pout,
                                                   max_inflight=args.max_inflight, stream=stream)
                if s_ == vkv.VKV_YIELDED:
                    landed = time.perf_counter()
                else:
                    layer, cur = (layer + 1) % n_layers_p, 0
            th.join()
            plat.append((landed - preq[0]) * 1e6)
            vkv.kv_yield_clear(pool)
        torch.cuda.synchronize()
        res.update({"prefill_yield_latency_us_p50": round(percentile(plat, 50), 1),
                    "prefill_yield_latency_us_p99": round(percentile(plat, 99), 1),
                    "prefill_yield_latency_us_max": round(max(plat), 1), "prefill_yield_injections": len(plat)})
    vkv.kv_prefill_check(pool, pws, stream)
    vkv.kv_sched_set_overlap(pool, bool(decode_overlap))
    return res


def _oracle_worker_init():
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(limits=1)
    except Exception:   # pragma: no cover
        pass


def _oracle_worker_ready(i):
    import oracle.attention   # noqa: F401  (pay the import before anything is timed)
    return i


def _oracle_worker_task(task):
    """One (layer file, sequence) unit of the oracle's attention; returns nothing of interest."""
    path, geom, seq = task
    from oracle.attention import PoolLayout, paged_decode_attention
    z = np.load(path, mmap_mode="r")
    meta = np.load(path + ".meta.npz")
    lay = PoolLayout(1, geom[0], geom[1], geom[2])
    paged_decode_attention(z, lay, meta["q"], meta["tables"], meta["ctx"], 0, seqs=[seq])
    return seq


def cpu_oracle_baseline(wl, st, pool_t, q_all, decode_bytes, reclaim_traffic, sample_bytes, workers, n_workers):
    """Times the oracle as it stands on a bounded sample of this workload (the first sequences of the
    batch, as many as give about sample_bytes of K+V per layer, over as many layers as that takes; plus
    a reclamation of a 1024-block pool) with one thread, and again over worker processes, and scales
    both to one step's byte mix."""
    import contextlib
    import tempfile
    import torch
    from oracle.attention import PoolLayout, paged_decode_attention
    from oracle.reclaim import ReclaimOracle
    try:
        from threadpoolctl import threadpool_limits
    except Exception:   # pragma: no cover
        threadpool_limits = None
    g = wl.geom
    # sample: sequences 0..n_seq-1 (all of them if one layer of the batch is below the byte target), layers 0..n_layers-1
    per_seq_layer = st.ctx_len[:wl.num_seqs].astype(np.int64) * g.kv_bytes_per_token_layer
    cum = np.cumsum(per_seq_layer)
    n_seq = int(min(wl.num_seqs, max(2, np.searchsorted(cum, sample_bytes) + 1)))
    layer_bytes = int(cum[n_seq - 1])
    n_layers = int(max(1, min(g.num_layers, round(sample_bytes / layer_bytes))))
    # compact one-layer pools holding only the sample's blocks (ids renumbered; the attention result
    # does not depend on block ids)
    rows = st.tables[:n_seq]
    ids = np.unique(rows[rows >= 0])
    renum = np.full(g.num_blocks, -1, dtype=np.int32)
    renum[ids] = np.arange(len(ids), dtype=np.int32)
    layer_elems = 2 * g.num_kv_heads * g.block_tokens * g.head_dim
    ids_t = torch.from_numpy(ids).to(pool_t.device).long()
    sample_tables = np.where(rows >= 0, renum[np.maximum(rows, 0)], -1).astype(np.int32)
    lay = PoolLayout(1, g.num_kv_heads, g.head_dim, g.block_tokens)
    ctx = st.ctx_len[:n_seq]
    attn_bytes = int(ctx.astype(np.int64).sum()) * g.kv_bytes_per_token_layer * n_layers
    tmpdir = tempfile.mkdtemp(prefix="vkv_bench_", dir="/dev/shm" if os.path.isdir("/dev/shm") else None)
    files = []
    t_attn = 0.0
    try:
        with (threadpool_limits(limits=1) if threadpool_limits else contextlib.nullcontext()):
            for layer in range(n_layers):
                blocks = pool_t.view(g.num_blocks, g.block_elems)[ids_t, layer * layer_elems:(layer + 1) * layer_elems]
                sample_pool = blocks.cpu().numpy().view(np.uint16).reshape(-1)
                q = q_all[layer, :n_seq].cpu().numpy().view(np.uint16)
                if workers is not None:
                    try:
                        path = os.path.join(tmpdir, f"layer{layer}.npy")
                        np.save(path, sample_pool)
                        np.savez(path + ".meta.npz", q=q, tables=sample_tables, ctx=ctx)
                        files.append(path)
                    except OSError as e:     # no room for the sample files: skip the all-cores timing
                        progress(f"  cannot stage the sample for the worker processes: {e}")
                        workers = None
                t0 = time.perf_counter()
                paged_decode_attention(sample_pool, lay, q, sample_tables, ctx, 0)
                t_attn += time.perf_counter() - t0
                del sample_pool, blocks
            progress(f"  oracle, one thread: {n_layers} layer(s) of {n_seq} sequences in {t_attn:.1f} s")
            # reclamation: the top 1024 blocks of the pool as a pool of their own, upper quarter reclaimed
            nb_s = min(1024, g.num_blocks) // g.blocks_per_handle * g.blocks_per_handle
            base = g.num_blocks - nb_s
            rc = max(g.blocks_per_handle, nb_s // 4 // g.blocks_per_handle * g.blocks_per_handle)
            live = st.live[base:].copy()
            if (live[:nb_s - rc] == 0).sum() < live[nb_s - rc:].sum():
                live[:nb_s - rc] = 0            # crowded sample: make room, the copy cost is what is timed
            pool_s = pool_t.view(g.num_blocks, g.block_elems)[base:].cpu().numpy().view(np.uint16)
            tabs = np.flatnonzero(live).astype(np.int32).reshape(1, -1)
            orc = ReclaimOracle(nb_s, g.blocks_per_handle, live, tabs, pool_s)
            t0 = time.perf_counter()
            status, src, dst, _ = orc.reclaim(nb_s - rc, nb_s)
            t_rec = time.perf_counter() - t0
            assert status == 0
            rec_bytes = 2 * len(src) * g.block_bytes
            del pool_s
        attn_rate = attn_bytes / t_attn
        rec_rate = rec_bytes / t_rec if t_rec > 0 and rec_bytes else float("inf")
        step_s = decode_bytes / attn_rate + (reclaim_traffic / rec_rate if rec_bytes else 0.0)
        result = {"value": round((decode_bytes + reclaim_traffic) / step_s / 1e9, 4), "unit": "GB/s", "cores": 1,
                  "kind": "oracle",
                  "sample": (f"attention: layers 0..{n_layers - 1} of sequences 0..{n_seq - 1} ({attn_bytes / 1e6:.0f} MB of "
                             f"K+V, {t_attn:.1f} s); reclamation: top {nb_s} blocks as a pool, {len(src)} blocks moved "
                             f"({rec_bytes / 1e6:.0f} MB read+written, {t_rec:.2f} s); scaled to one step's byte mix"),
                  "attention_GBps": round(attn_rate / 1e9, 4), "reclaim_GBps": round(rec_rate / 1e9, 3)}
        if workers is not None:
            # the same attention sample over worker processes, one (layer, sequence) unit at a time,
            # longest first; the reclamation oracle is one memory copy per block and stays as timed
            geom = (g.num_kv_heads, g.head_dim, g.block_tokens)
            tasks = [(f, geom, int(s_)) for f in files for s_ in np.argsort(-ctx)]
            t0 = time.perf_counter()
            try:
                workers.map(_oracle_worker_task, tasks, chunksize=1)
                t_mp = time.perf_counter() - t0
                mp_rate = attn_bytes / t_mp
                mp_step = decode_bytes / mp_rate + (reclaim_traffic / rec_rate if rec_bytes else 0.0)
                result["all_cores"] = {"value": round((decode_bytes + reclaim_traffic) / mp_step / 1e9, 4),
                                       "unit": "GB/s", "cores": n_workers, "attention_GBps": round(mp_rate / 1e9, 4),
                                       "attention_seconds": round(t_mp, 2), "host_cpu_count": os.cpu_count()}
            except Exception as e:
                result["all_cores"] = {"error": f"{type(e).__name__}: {e}"}
        return result
    finally:
        import shutil
        shutil.rmtree(tmpdir, ignore_errors=True)


if __name__ == "__main__":
    main()

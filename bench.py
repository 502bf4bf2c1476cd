#!/usr/bin/env python3
"""Benchmark of the KV-reclaim hot path on one MI355X.

A step is one pass of the whole path over one seeded synthetic workload:
kv_plan_reclaim -> kv_compact -> kv_remap_tables, back to back on one HIP
stream with no host synchronisation in between (the block tables are restored
from a pristine device copy at the start of each step, a 2 MiB device copy, so
that every step does identical work; replaying the block copy needs no
restore because source blocks are never written).

Prints ONE JSON line.  `value` is read+write GB/s of the whole step with
inputs resident in HBM; `roofline` prices the block-copy kernel alone against
the 8 TB/s HBM peak using HIP-event times taken on the launch stream;
`cpu_baseline` is the single-threaded CPU oracle timed on a bounded sample of
the same workload; `materialize` adds the weight-streaming leg of the third
configuration (pinned host -> reclaimed region) serial and overlapped, and
checks pool, tables and weight region byte for byte after one more (untimed)
run of each overlapped path on a freshly generated pool; `must_fail` records
the infeasible variants (they must change nothing).
`roofline.ceiling_contiguous_GBps` is the same block-copy kernel on the one
plan that is a plain memmove (a full upper half onto an empty lower half, same
byte count), measured outside the timed region: the empirical ceiling of this
copy on this machine.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
LINK_PEAK_GBPS = 63.0           # PCIe 5.0 x16, one direction, theoretical

# HBM bytes per launch of the block-copy kernel from two rocprofv3 --pmc runs (FETCH_SIZE, then
# WRITE_SIZE, each scaled by what the counter shows for a plain 1 GiB copy: x2.0 and x1.0), for
# configs[1], [3] and [4] with the default launch shape.  Profiler figures cannot be taken
# inside this process; other workloads or launch shapes report null.
MEASURED_TRAFFIC_BYTES = {(1, 4687): 19_668_716_536, (3, 3415): 35_828_382_869, (4, 15425): 32_366_820_165}
TRAFFIC_SOURCE = {1: "profiles/pmc_hbm_bytes_compact_cfg2_8b.md", 3: "profiles/pmc_hbm_bytes_compact_cfg4_70b_cfg5_frag.md",
                  4: "profiles/pmc_hbm_bytes_compact_cfg4_70b_cfg5_frag.md"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="index into the benchmark config list (default 1: 8B-shaped)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-materialize", action="store_true")
    ap.add_argument("--no-must-fail", action="store_true")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the contiguous-plan ceiling (profiler runs: keeps its launches out of the kernel's statistics)")
    ap.add_argument("--workgroups", type=int, default=0)
    ap.add_argument("--chunk-bytes", type=int, default=0)
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--calibration-copy", type=int, default=0, metavar="MiB",
                    help="also run one plain device copy of this many MiB before the timed region "
                         "(a known-size reference for profiler byte counters)")
    ap.add_argument("--comparators", action="store_true",
                    help="also time a plain contiguous device-to-device copy of the same byte count "
                         "(hipMemcpy DtoD through torch) as a reference point")
    ap.add_argument("--layout", choices=("block", "layer"), default="block",
                    help="pool layout: block-major (default) or layer-major (one slab per layer)")
    ap.add_argument("--kv-heads", type=int, default=0,
                    help="override the config's KV heads per block (a tensor-parallel share has fewer: smaller "
                         "tiles, same block count); 0 = as the config says")
    ap.add_argument("--ceiling", action="store_true",
                    help="only the empirical ceiling: the block-copy kernel on the plan that is one plain memmove "
                         "(full upper half onto an empty lower half, the config's moved byte count); one JSON line")
    ap.add_argument("--size-sweep", action="store_true",
                    help="instead of the benchmark: time the block copy alone on one-layer pools of 8 GiB whose "
                         "block size runs from 256 B to 5 MiB (45 %% live, half reclaimed) and print one line per size")
    ap.add_argument("--vmm-compare", type=int, default=0, metavar="BLOCKS",
                    help="also time the no-move variant (HIP virtual-memory remapping of unused blocks' pages) on a "
                         "pool of this many blocks of the config's shape; 20480 = the full 8B-shaped pool, which "
                         "takes about half a minute, most of it tearing the pool down")
    return ap.parse_args()


def assignment_from_bitmap(live_words, num_blocks: int, boundary: int):
    """The relocation rule written out with numpy, for the benchmark's own byte check (neither the
    library's plan nor the oracle is consulted): the live ids at or above the boundary, ascending,
    take the smallest free ids below it, ascending.  Returns (src, dst, new_id)."""
    bits = np.unpackbits(live_words.view(np.uint8), bitorder="little")[:num_blocks].astype(bool)
    src = boundary + np.flatnonzero(bits[boundary:])
    dst = np.flatnonzero(~bits[:boundary])[:src.size]
    assert dst.size == src.size, "infeasible"
    new_id = np.where(bits, np.arange(num_blocks), -1).astype(np.int32)
    new_id[boundary:] = -1
    new_id[src] = dst
    return src.astype(np.int32), dst.astype(np.int32), new_id


def contiguous_ceiling(wk, torch, pool_t, cfg, n_moves: int, stream, tuning, reps: int = 10, layer_stride: int = 0):
    """kv_compact on the closed-form contiguous plan: a pool of 2n blocks (the first 2n of pool_t)
    whose upper half is full and lower half empty, boundary n, so that the n moves are one memmove
    of n*block_bytes.  Overwrites those blocks.  Returns (GB/s r+w, avg ms, min ms)."""
    dev = pool_t.device
    n = min(n_moves, cfg.num_blocks // 2)
    bits = np.zeros(2 * n, dtype=np.uint8)
    bits[n:] = 1
    words = np.packbits(bits, bitorder="little")
    words = np.concatenate([words, np.zeros((-len(words)) % 8, np.uint8)]).view(np.int64)
    live_d = torch.from_numpy(words).to(dev)
    n_ws = wk.kv_plan_workspace_bytes(2 * n, n)
    ws = torch.zeros(n_ws, dtype=torch.uint8, device=dev)
    plan = wk.kv_plan_bind(ws, n_ws, 2 * n, n)
    pool = wk.pool_desc(pool_t, 2 * n, cfg.num_layers, cfg.tile_bytes, layer_stride)   # layer-major: one memmove per slab
    s = stream.cuda_stream
    wk.kv_plan_reclaim(live_d, plan, s)
    st = wk.kv_plan_fetch(plan, s)
    assert st.status == wk.KV_OK and st.n_moves == n
    for _ in range(3):
        wk.kv_compact_launch(pool, plan, s, **tuning)
    ms = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        wk.kv_compact_launch(pool, plan, s, **tuning)
        e1.record(stream)
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1))
    avg = sum(ms) / len(ms)
    return 2 * n * cfg.block_bytes / avg / 1e6, avg, min(ms)


def cpu_baseline(cfg, w, sample_moves: int, weights=None):
    """The oracle as it stands, one thread, on the first `sample_moves` moves of this workload."""
    import oracle
    t0 = time.perf_counter()
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    t_plan = time.perf_counter() - t0
    m = min(sample_moves, p.n_moves)
    bb = cfg.block_bytes
    pool = np.empty(cfg.pool_bytes, dtype=np.uint8)       # virtual; only sampled blocks get touched
    blocks = pool.reshape(cfg.num_blocks, bb)
    pattern = np.random.default_rng(cfg.seed).integers(0, 256, bb, dtype=np.uint8)
    for k in range(m):
        blocks[p.src[k]] = pattern                         # sources hold bytes, destinations are faulted in
        blocks[p.dst[k]] = 0
    sample = oracle.Plan(0, p.src[:m], p.dst[:m], p.new_id, p.live_out, m, cfg.num_blocks, cfg.boundary)
    t0 = time.perf_counter()
    oracle.compact(pool, bb, sample)
    t_compact = time.perf_counter() - t0
    for k in sorted({0, m // 2, m - 1}):                  # the copy did happen: destinations hold the sources' bytes
        assert np.array_equal(blocks[p.dst[k]], pattern), "oracle.compact left a destination unwritten"
    tables = w.tables.copy()
    t0 = time.perf_counter()
    oracle.remap(tables, p)
    t_remap = time.perf_counter() - t0
    total = t_plan + t_compact + t_remap
    parallel = None
    try:                                   # bench-only: the same sampled move list on every host core
        import ctypes
        import subprocess
        so = os.path.join(ROOT, "bench_hostcopy.so")
        src_cpp = os.path.join(ROOT, "bench_hostcopy.cpp")
        if not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src_cpp):
            subprocess.run(["g++", "-O2", "-std=c++17", "-pthread", "-fPIC", "-shared", src_cpp, "-o", so], check=True)
        lib = ctypes.CDLL(so)
        lib.hostcopy_moves.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_uint32, ctypes.c_uint32]
        lib.hostcopy_moves.restype = None
        cores = len(os.sched_getaffinity(0))
        src_a, dst_a = np.ascontiguousarray(p.src[:m]), np.ascontiguousarray(p.dst[:m])
        t_pars = []
        for _ in range(5):
            t0 = time.perf_counter()
            lib.hostcopy_moves(pool.ctypes.data, bb, src_a.ctypes.data, dst_a.ctypes.data, m, cores)
            t_pars.append(time.perf_counter() - t0)
        rates = sorted(2 * m * bb / t / 1e9 for t in t_pars)
        parallel = {"value": round(statistics.median(rates), 3), "unit": "GB/s", "cores": cores,
                    "kind": "threaded memcpy of the same move list (bench-only code, not the oracle)",
                    "repetitions": len(rates), "min": round(rates[0], 3), "max": round(rates[-1], 3),
                    "ms_median": round(statistics.median(t_pars) * 1e3, 3)}
    except Exception as e:                 # a missing compiler must not cost the benchmark line
        parallel = {"error": str(e)[:200]}
    del pool, blocks
    out = {"value": round(2 * m * bb / total / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "all_cores_copy": parallel,
           "host_cores_available": os.cpu_count(),
           "sample": f"oracle plan (all {cfg.num_blocks} blocks) + block copy of the first {m} of {p.n_moves} moves "
                     f"({m * bb / 2**30:.2f} GiB moved) + table remap (all {tables.size} entries), one thread",
           "ms": {"plan": round(t_plan * 1e3, 3), "compact_sample": round(t_compact * 1e3, 3),
                  "remap": round(t_remap * 1e3, 3)}}
    if weights is not None:
        # the weight copy of the third configuration (one memcpy per tensor into a host stand-in for
        # the reclaimed region, pre-faulted), one thread: the oracle's last step on this workload
        host, starts, sizes, offs = weights
        region = np.empty(offs[-1] + sizes[-1], dtype=np.uint8)
        region.fill(0)                                    # touch every page before the timed copy
        views = [(host[st:st + sz].numpy(), off) for st, sz, off in zip(starts, sizes, offs)]
        t0 = time.perf_counter()
        rc = oracle.materialize(region, 0, views)
        t_mat = time.perf_counter() - t0
        assert rc == 0 and np.array_equal(region[offs[-1]:offs[-1] + 4096], views[-1][0][:4096])
        total_w = sum(sizes)
        out["materialize"] = {"ms": round(t_mat * 1e3, 2), "GBps": round(total_w / t_mat / 1e9, 3),
                              "sample": f"oracle weight copy of all {len(sizes)} tensors ({total_w} B), pinned host "
                                        "memory (the weights as parked for the GPU) to pageable host memory, one thread"}
    return out


SWEEP_SIZES = [256, 512, 1040, 2048, 3072, 4096, 6144, 8192, 12288, 16384, 20480, 24576, 28672, 32768, 36864, 40960,
               45056, 49152, 53248, 57344, 61440, 65536, 69632, 73728, 77824, 86016, 94208, 102400, 114688, 131072,
               147456, 180224, 196608, 262144, 278528, 327680, 393216, 458752, 524288, 1048576 + 4096, 2097152, 5242880]


def size_sweep(args):
    """Block copy alone across block sizes (which kernel shape each size gets is the library's choice)."""
    import torch
    import paper_2512_09472_amd as wk
    from synth import content
    wk.binding.load()
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()
    s = stream.cuda_stream
    rows = []
    for tile in SWEEP_SIZES:
        nb = min(1 << 22, max(2048, (8 << 30) // tile))
        b = nb // 2
        bits = np.random.default_rng(nb).random(nb) < 0.45
        words = np.packbits(bits, bitorder="little")
        words = np.concatenate([words, np.zeros((-len(words)) % 8, np.uint8)]).view(np.int64)
        live_d = torch.from_numpy(words).to(dev)
        pool_t = torch.empty(nb * tile, dtype=torch.uint8, device=dev)
        content.fill_device(pool_t.data_ptr(), nb, tile, 1)
        n_ws = wk.kv_plan_workspace_bytes(nb, b)
        ws = torch.zeros(n_ws, dtype=torch.uint8, device=dev)
        plan = wk.kv_plan_bind(ws, n_ws, nb, b)
        pool = wk.pool_desc(pool_t, nb, 1, tile)
        torch.cuda.synchronize()
        wk.kv_plan_reclaim(live_d, plan, s)
        n_moves = wk.kv_plan_fetch(plan, s).n_moves
        tuning = dict(workgroups=args.workgroups, chunk_bytes=args.chunk_bytes, flags=args.flags)
        for _ in range(2):
            wk.kv_compact_launch(pool, plan, s, **tuning)
        ms = []
        for _ in range(7):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            wk.kv_compact_launch(pool, plan, s, **tuning)
            e1.record(stream)
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        st = wk.kv_plan_fetch(plan, s)
        assert st.status == wk.KV_OK and st.ticket == 0 and st.finished == 0
        gbps = 2 * n_moves * tile / min(ms) / 1e6
        rows.append({"block_bytes": tile, "blocks": nb, "moved": n_moves, "kernel_ms_min": round(min(ms), 4),
                     "GBps_rw": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)})
        print(f"block {tile:>8} B x {nb:>8} blocks, {n_moves:>7} moved: {min(ms):.3f} ms  {gbps:7.0f} GB/s r+w  "
              f"{100 * gbps / HBM_PEAK_GBPS:.1f} % of peak", file=sys.stderr, flush=True)
        del pool_t
    print(json.dumps({"metric": "block copy GB/s (read+write) by block size", "unit": "GB/s", "n_gpus": 1,
                      "data": "synthetic", "peak": HBM_PEAK_GBPS, "sizes": rows}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "there is no multi-GPU path to measure. Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    if args.size_sweep:
        size_sweep(args)
        return

    import torch
    import paper_2512_09472_amd as wk
    from synth import CONFIGS, content, dense_offsets, make_workload, weight_shapes_8b

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    wk.binding.load()
    dev = torch.device("cuda:0")
    cfg = CONFIGS[args.config]
    if args.kv_heads:
        cfg = cfg.scaled(kv_heads=args.kv_heads)
    w = make_workload(cfg)
    bb = cfg.block_bytes

    # ---- device-resident inputs
    pool_t = torch.empty(cfg.pool_bytes, dtype=torch.uint8, device=dev)
    table = content.normal_bf16_table(1.0) if cfg.content == "bf16_normal" else None
    table_d = torch.from_numpy(table.view(np.int16)).to(dev) if table is not None else None
    layer_stride = cfg.num_blocks * cfg.tile_bytes if args.layout == "layer" else 0

    def fill_pool():
        """Block i holds content id i; in a layer-major pool slab l holds bytes [l*tile, (l+1)*tile) of each."""
        tp = table_d.data_ptr() if table_d is not None else 0
        if not layer_stride:
            content.fill_device(pool_t.data_ptr(), cfg.num_blocks, bb, cfg.seed, table_ptr=tp)
        else:
            for l in range(cfg.num_layers):
                content.fill_device(pool_t.data_ptr() + l * layer_stride, cfg.num_blocks, cfg.tile_bytes, cfg.seed,
                                    table_ptr=tp, byte_offset=l * cfg.tile_bytes)

    fill_pool()
    live_d = torch.from_numpy(w.live.view(np.int64)).to(dev)
    tables0_d = torch.from_numpy(w.tables).to(dev)
    tables_d = tables0_d.clone()
    ws_bytes = wk.kv_plan_workspace_bytes(cfg.num_blocks, cfg.boundary)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=dev)
    plan = wk.kv_plan_bind(ws, ws_bytes, cfg.num_blocks, cfg.boundary)
    pool = wk.pool_desc(pool_t, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes, layer_stride)
    stream = torch.cuda.Stream()
    s = stream.cuda_stream
    tuning = dict(workgroups=args.workgroups, chunk_bytes=args.chunk_bytes, flags=args.flags)

    def step(ev=None):
        with torch.cuda.stream(stream):
            tables_d.copy_(tables0_d, non_blocking=True)
        wk.kv_plan_reclaim(live_d, plan, s)
        if ev is not None:
            ev[0].record(stream)
        wk.kv_compact_launch(pool, plan, s, **tuning)
        if ev is not None:
            ev[1].record(stream)
        wk.kv_remap_tables(tables_d, w.tables.shape[0], w.tables.shape[1], plan, s)

    if args.calibration_copy:
        n_cal = args.calibration_copy << 20
        cal_src = torch.empty(n_cal, dtype=torch.uint8, device=dev)
        cal_dst = torch.empty(n_cal, dtype=torch.uint8, device=dev)
        content.fill_device(cal_src.data_ptr(), 1, n_cal, 7)
        torch.cuda.synchronize()
        cal_dst.copy_(cal_src)          # one elementwise copy kernel: reads n_cal bytes, writes n_cal bytes
        torch.cuda.synchronize()
        del cal_src, cal_dst

    if args.ceiling:       # the planner alone tells how many blocks the workload moves; no block copy but the ceiling's
        wk.kv_plan_reclaim(live_d, plan, s)
        n_moves = wk.kv_plan_fetch(plan, s).n_moves
        bb = cfg.block_bytes
        gbps, avg, mn = contiguous_ceiling(wk, torch, pool_t, cfg, n_moves, stream, tuning, reps=max(10, args.steps),
                                           layer_stride=layer_stride)
        print(json.dumps({"metric": "block copy of one contiguous range GB/s (read+write)", "value": round(gbps, 2),
                          "unit": "GB/s", "n_gpus": 1, "data": "synthetic", "kernel_ms_avg": round(avg, 4),
                          "kernel_ms_min": round(mn, 4), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
                          "workload": f"{min(n_moves, cfg.num_blocks // 2)} blocks of {bb} B, upper half of a "
                                      f"2n-block {args.layout}-major pool onto its empty lower half (one memmove"
                                      f"{' per layer slab' if layer_stride else ''})"}), flush=True)
        return

    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    st = wk.kv_plan_fetch(plan, s)
    if st.status != wk.KV_OK:
        print(f"bench.py: plan status {st.status}", file=sys.stderr)
        sys.exit(1)
    n_moves = st.n_moves
    rw_bytes = 2 * n_moves * bb

    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    compact_ms = [a.elapsed_time(b) for a, b in events]
    compact_avg = sum(compact_ms) / len(compact_ms)
    st = wk.kv_plan_fetch(plan, s)
    assert st.status == wk.KV_OK and st.n_moves == n_moves and st.n_bad_entries == 0

    # the same step through kv_reclaim (one call; a single kernel launch on small pools), outside the timed region
    def step_one_call():
        with torch.cuda.stream(stream):
            tables_d.copy_(tables0_d, non_blocking=True)
        wk.kv_reclaim(pool, plan, live_d, tables_d, w.tables.shape[0], w.tables.shape[1], s)

    for _ in range(args.warmup):
        step_one_call()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step_one_call()
    torch.cuda.synchronize()
    one_call_ms = (time.perf_counter() - t2) * 1e3 / args.steps
    st1 = wk.kv_plan_fetch(plan, s)
    assert st1.status == wk.KV_OK and st1.n_moves == n_moves and st1.n_bad_entries == 0

    reclaimed_bytes = (cfg.num_blocks - cfg.boundary) * bb
    # which block-copy kernel the library picked: units of half a ticket or less share tickets
    unit_bytes = cfg.tile_bytes if args.layout == "layer" else bb
    ticket_bytes = min(args.chunk_bytes, 65536) if args.chunk_bytes else 86016   # pairs of up to 42 KiB by default
    copy_kernel = ("compact_packed_kernel" if 2 * unit_bytes <= ticket_bytes and not args.flags & 8
                   else "compact_ticket_kernel")
    out = {
        "metric": "KV compaction GB/s (read+write)",
        "value": round(rw_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name}: {cfg.num_layers} layers, block {bb} B, "
                               f"{cfg.num_blocks} blocks ({cfg.pool_bytes / 2**30:.0f} GiB pool), boundary {cfg.boundary}, "
                               f"{w.live_count} live, {n_moves} moved",
                   "step": "kv_plan_reclaim + kv_compact + kv_remap_tables on one stream",
                   "moved_GiB": round(n_moves * bb / 2**30, 3),
                   "reclaimed_GiB": round(reclaimed_bytes / 2**30, 3),
                   "ms_to_reclaim": round(ms_per_step, 4),
                   "ms_to_reclaim_kv_reclaim_one_call": round(one_call_ms, 4),
                   "pct_of_hbm_peak_whole_step": round(100 * rw_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
                   "layout": args.layout + "-major", "tuning": tuning,
                   "inputs_sha256": hashlib.sha256(w.live.tobytes() + w.tables.tobytes()).hexdigest()[:16]},
        "roofline": {"bound": "hbm", "kernel": copy_kernel,
                     "achieved": round(rw_bytes / (compact_avg * 1e-3) / 1e9, 2), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(rw_bytes / (compact_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                     "traffic": (MEASURED_TRAFFIC_BYTES.get((cfg.index, n_moves))
                                 if not any(tuning.values()) and args.layout == "block" and not args.kv_heads
                                 else None),
                     "traffic_source": (f"{TRAFFIC_SOURCE[cfg.index]}: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of "
                                        "this command, scaled by a plain copy; a profiler figure, not measured by this run"
                                        if not any(tuning.values()) and args.layout == "block" and not args.kv_heads
                                        and (cfg.index, n_moves) in MEASURED_TRAFFIC_BYTES else None),
                     "kernel_ms_avg": round(compact_avg, 4), "kernel_ms_min": round(min(compact_ms), 4),
                     "kernel_ms_median": round(statistics.median(compact_ms), 4),
                     "algorithmic_bytes_per_launch": rw_bytes},
    }

    if args.comparators:
        half = n_moves * bb
        a_, b_ = pool_t[:half], pool_t[cfg.pool_bytes - half:]
        ts = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            a_.copy_(b_)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        out["comparators"] = {"contiguous_hipMemcpyDtoD_GBps_rw": round(2 * half / min(ts[1:]) / 1e6, 1),
                              "note": f"one contiguous copy of {half / 2**30:.2f} GiB, top of the pool to its bottom"}
        fill_pool()
        torch.cuda.synchronize()

    tptr = table_d.data_ptr() if table_d is not None else 0

    def pool_blocks_equal(cid, first, end, skip_below=0):
        """Blocks [first, end) of the pool hold the content ids in cid (device generator, 1 GiB at a
        time); bytes below skip_below are not looked at.  Block-major pools."""
        slab = max(1, (1 << 30) // bb)
        scratch = torch.empty(slab * bb, dtype=torch.uint8, device=dev)
        cid_d = torch.from_numpy(np.ascontiguousarray(cid, dtype=np.int32)).to(dev)
        ok = True
        for j0 in range(first, end, slab):
            n = min(slab, end - j0)
            content.fill_device(scratch.data_ptr(), n, bb, cfg.seed, cids_ptr=cid_d.data_ptr() + 4 * j0, table_ptr=tptr)
            lo = max(skip_below, j0 * bb)
            ok = ok and torch.equal(pool_t[lo:(j0 + n) * bb], scratch[lo - j0 * bb:n * bb])
        return ok

    # ---- must-fail variants: an infeasible request has to leave every pool byte and table entry as it was
    if args.layout == "block" and not args.kv_heads and not args.no_must_fail:
        import dataclasses
        variants = {}
        if cfg.occupancy is not None and int(round(cfg.occupancy * cfg.num_blocks)) > cfg.boundary:
            variants[f"stated occupancy taken literally ({int(round(cfg.occupancy * cfg.num_blocks))} live blocks, "
                     f"boundary {cfg.boundary})"] = (dataclasses.replace(cfg, live_budget_override=int(
                         round(cfg.occupancy * cfg.num_blocks))), cfg.boundary)
        variants[f"boundary = live count - 1 ({w.live_count - 1})"] = (cfg, w.live_count - 1)
        fill_pool()
        torch.cuda.synchronize()
        out["must_fail"] = {}
        for name, (vcfg, vb) in variants.items():
            vw = make_workload(vcfg) if vcfg is not cfg else w
            v_ws_bytes = wk.kv_plan_workspace_bytes(cfg.num_blocks, vb)
            v_ws = torch.zeros(v_ws_bytes, dtype=torch.uint8, device=dev)
            v_plan = wk.kv_plan_bind(v_ws, v_ws_bytes, cfg.num_blocks, vb)
            v_live = torch.from_numpy(vw.live.view(np.int64)).to(dev)
            v_tables = torch.from_numpy(vw.tables).to(dev)
            wk.kv_plan_reclaim(v_live, v_plan, s)
            wk.kv_compact_launch(pool, v_plan, s, **tuning)
            wk.kv_remap_tables(v_tables, vw.tables.shape[0], vw.tables.shape[1], v_plan, s)
            v_st = wk.kv_plan_fetch(v_plan, s)
            unchanged = (pool_blocks_equal(np.arange(cfg.num_blocks), 0, cfg.num_blocks)
                         and np.array_equal(v_tables.cpu().numpy(), vw.tables))
            out["must_fail"][name] = {"status": wk.binding._NAMES.get(v_st.status, v_st.status), "n_moves": v_st.n_moves,
                                      "pool_and_tables_unchanged": bool(unchanged)}
            if v_st.status != wk.KV_E_NOSPACE or not unchanged:
                print(f"bench.py: must-fail variant did not fail cleanly: {name}: {out['must_fail'][name]}", file=sys.stderr)
                sys.exit(1)

    # ---- weight materialisation leg (third configuration: same pool plus weights)
    weights_for_oracle = host_weights = None
    if not args.no_materialize and cfg.index in (1, 2) and not args.kv_heads:
        shapes = weight_shapes_8b()
        sizes = [2 * a * b for _, (a, b) in shapes]
        offs = dense_offsets(sizes)
        total = sum(sizes)
        host = torch.empty(total, dtype=torch.uint8, pin_memory=True)
        wtab = torch.from_numpy(content.normal_bf16_table(0.02).view(np.int16)).to(dev)
        stage = torch.empty(max(sizes), dtype=torch.uint8, device=dev)
        pos = 0
        for i, sz in enumerate(sizes):       # seeded N(0, 0.02) bf16, generated on the device, parked in pinned memory
            content.fill_device(stage.data_ptr(), 1, sz, 0x5EED0002, cid0=i, table_ptr=wtab.data_ptr())
            host[pos:pos + sz].copy_(stage[:sz])
            pos += sz
        torch.cuda.synchronize()
        del stage
        starts = np.concatenate([[0], np.cumsum(sizes)[:-1]]).tolist()
        region0 = cfg.boundary * bb
        tile, strip = cfg.tile_bytes, (cfg.num_blocks - cfg.boundary) * cfg.tile_bytes
        # pieces: (offset in the pinned buffer, bytes, region offset, content id, byte offset in that content)
        if not layer_stride:
            pieces = [(st_, sz, off, i, 0) for i, (st_, sz, off) in enumerate(zip(starts, sizes, offs))]
        else:
            # strip l takes layer l's seven matrices and the l-th of L row slices of the embedding matrix
            # (1.05 GB: it fits no 512 MiB strip whole)
            emb, emb_slice = len(sizes) - 1, sizes[-1] // cfg.num_layers
            pieces = []
            for l in range(cfg.num_layers):
                at = l * strip
                for i in range(7 * l, 7 * l + 7):
                    pieces.append((starts[i], sizes[i], at, i, 0))
                    at += sizes[i]
                pieces.append((starts[emb] + l * emb_slice, emb_slice, at, emb, l * emb_slice))
                assert at + emb_slice <= (l + 1) * strip
        tensors = [(host.data_ptr() + st_, sz, off) for st_, sz, off, _, _ in pieces]

        def device_offset(region_offset):
            if not layer_stride:
                return region0 + region_offset
            l, within = divmod(region_offset, strip)
            return l * layer_stride + cfg.boundary * tile + within
        weights_for_oracle = (host, starts, sizes, offs)
        copy_stream = torch.cuda.Stream()
        cs = copy_stream.cuda_stream

        def timed(fn, reps=3):
            ts = []
            for _ in range(reps):
                torch.cuda.synchronize()
                a = time.perf_counter()
                fn()
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - a) * 1e3)
            return min(ts)

        def only_copy():
            wk.weights_materialize(pool, cfg.boundary, tensors, cs, None)

        def serial():
            step()
            torch.cuda.synchronize()
            wk.weights_materialize(pool, cfg.boundary, tensors, cs, None)

        done = torch.cuda.Event()

        def overlapped():
            with torch.cuda.stream(stream):
                tables_d.copy_(tables0_d, non_blocking=True)
            wk.kv_plan_reclaim(live_d, plan, s)
            wk.kv_compact_launch(pool, plan, s, **tuning)
            done.record(stream)
            wk.weights_materialize(pool, cfg.boundary, tensors, cs, done.cuda_event)
            wk.kv_remap_tables(tables_d, w.tables.shape[0], w.tables.shape[1], plan, s)

        def pipelined():
            with torch.cuda.stream(stream):
                tables_d.copy_(tables0_d, non_blocking=True)
            wk.kv_plan_reclaim(live_d, plan, s)
            wk.kv_compact_launch(pool, plan, s, **tuning)
            done.record(stream)
            wk.weights_materialize_pipelined(pool, cfg.boundary, w.live, tensors, 0, cs, done.cuda_event)
            wk.kv_remap_tables(tables_d, w.tables.shape[0], w.tables.shape[1], plan, s)

        def one_call():
            with torch.cuda.stream(stream):
                tables_d.copy_(tables0_d, non_blocking=True)
            wk.kv_switch(pool, plan, live_d, tables_d, w.tables.shape[0], w.tables.shape[1], tensors, s, cs,
                         done.cuda_event, live_host=w.live, front_done=front_done.cuda_event)

        copy_stream2 = torch.cuda.Stream()

        def one_call_two_streams():
            with torch.cuda.stream(stream):
                tables_d.copy_(tables0_d, non_blocking=True)
            wk.kv_switch(pool, plan, live_d, tables_d, w.tables.shape[0], w.tables.shape[1], tensors, s, cs,
                         done.cuda_event, live_host=w.live, front_done=front_done.cuda_event,
                         copy_stream2=copy_stream2.cuda_stream)

        # a checkpoint whose tensors do not continue each other in host memory: every tensor (cut at
        # 64 MiB) is a request of its own, listed so that neighbours never merge
        split = []
        for a_, n_, o_ in tensors:
            for c0 in range(0, n_, 64 << 20):
                split.append((a_ + c0, min(64 << 20, n_ - c0), o_ + c0))
        split = split[0::2] + split[1::2]

        def copy_split_one_stream():
            wk.weights_materialize(pool, cfg.boundary, split, cs, None)

        def copy_split_two_streams():
            wk.weights_materialize_streams(pool, cfg.boundary, split, [cs, copy_stream2.cuda_stream])

        # the link's measured ceiling: one plain pinned-to-device copy of 4 GiB into the same region
        n_plain = min(4 << 30, total)

        def plain_copy():
            with torch.cuda.stream(copy_stream):
                pool_t[region0:region0 + n_plain].copy_(host[:n_plain], non_blocking=True)

        plain_copy()
        t_plain = timed(plain_copy)
        only_copy()
        t_copy = timed(only_copy)
        t_serial = timed(serial)
        t_overlap = timed(overlapped)
        t_pipe = timed(pipelined)
        front_done = torch.cuda.Event()
        done.record(stream)                # torch creates a HIP event on its first record
        front_done.record(stream)
        t_switch = timed(one_call)
        t_switch2 = timed(one_call_two_streams)
        t_split1 = timed(copy_split_one_stream)
        t_split2 = timed(copy_split_two_streams)

        # Byte check of the overlapped paths, outside every timed region: each runs once more on a
        # freshly generated pool (the timed replays above had weights where KV should be), then
        # pool, tables and weight region are compared with what the relocation rule says.
        src_x, dst_x, new_id_x = assignment_from_bitmap(w.live, cfg.num_blocks, cfg.boundary)
        cid_x = np.arange(cfg.num_blocks, dtype=np.int32)
        cid_x[dst_x] = src_x
        tables_x = np.where(w.tables >= 0, new_id_x[np.maximum(w.tables, 0)], w.tables).astype(np.int32)
        stage = torch.empty(max(sizes), dtype=torch.uint8, device=dev)

        def verified(fn):
            fill_pool()
            torch.cuda.synchronize()
            fn()
            torch.cuda.synchronize()
            ok = np.array_equal(tables_d.cpu().numpy(), tables_x)
            used = {}                                                              # weight bytes per strip (one strip if block-major)
            for st_, sz, off, cid, coff in pieces:                                 # every tensor
                content.fill_device(stage.data_ptr(), 1, sz, 0x5EED0002, cid0=cid, table_ptr=wtab.data_ptr(), byte_offset=coff)
                at = device_offset(off)
                ok = ok and torch.equal(pool_t[at:at + sz], stage[:sz])
                l = off // strip if layer_stride else 0
                used[l] = max(used.get(l, 0), off - l * strip * bool(layer_stride) + sz)
            if not layer_stride:
                ok = ok and pool_blocks_equal(cid_x, 0, cfg.boundary)              # moved and kept KV
                end = region0 + used[0]                                            # the region past the last tensor
                ok = ok and pool_blocks_equal(np.arange(cfg.num_blocks), end // bb, cfg.num_blocks, skip_below=end)
            else:
                scratch = torch.empty(layer_stride, dtype=torch.uint8, device=dev)
                cid_d = torch.from_numpy(cid_x).to(dev)
                for l in range(cfg.num_layers):                                    # slab by slab: KV below b, the strip's tail
                    content.fill_device(scratch.data_ptr(), cfg.num_blocks, tile, cfg.seed, cids_ptr=cid_d.data_ptr(),
                                        table_ptr=tptr, byte_offset=l * tile)
                    slab = pool_t[l * layer_stride:(l + 1) * layer_stride]
                    tail = cfg.boundary * tile + used.get(l, 0)
                    ok = ok and torch.equal(slab[:cfg.boundary * tile], scratch[:cfg.boundary * tile])
                    ok = ok and torch.equal(slab[tail:], scratch[tail:])
                del scratch
            return bool(ok)

        checks = {"weights_materialize (gated)": verified(overlapped),
                  "weights_materialize_pipelined": verified(pipelined),
                  "kv_switch (front first)": verified(one_call),
                  "kv_switch (front first, two copy streams)": verified(one_call_two_streams)}
        del stage
        if not all(checks.values()):
            print(f"bench.py: byte check of the overlapped weight paths failed: {checks}", file=sys.stderr)
            sys.exit(1)
        out["materialize"] = {"workload": f"configs[2]: {len(pieces)} bf16 tensors, 15,009,316,864 B from pinned host memory"
                                          + (" (layer-major pool: placed strip by strip, embedding rows in 32 slices)"
                                             if layer_stride else ""),
                              "h2d_ms": round(t_copy, 2), "h2d_GBps": round(total / t_copy / 1e6, 2),
                              "link_peak_GBps": LINK_PEAK_GBPS,
                              "link_measured_plain_copy_GBps": round(n_plain / t_plain / 1e6, 2),
                              "frac_of_link_peak": round(total / t_copy / 1e6 / LINK_PEAK_GBPS, 4),
                              "serial_reclaim_then_copy_ms": round(t_serial, 2),
                              "overlapped_ms": round(t_overlap, 2),
                              "block_pipelined_ms": round(t_pipe, 2),
                              "kv_switch_one_call_ms": round(t_switch, 2),
                              "kv_switch_one_call_two_copy_streams_ms": round(t_switch2, 2),
                              "h2d_unmergeable_requests": {"requests": len(split), "one_stream_ms": round(t_split1, 2),
                                                           "two_streams_ms": round(t_split2, 2)},
                              "verified": True,
                              "verified_paths": sorted(checks),
                              "verified_how": "one more untimed run of each path on a freshly generated pool; tables, every "
                                              "block below the boundary, every tensor and the region's tail compared "
                                              "byte for byte with the relocation rule written out in numpy"}
        host_weights = (host, starts, sizes, offs)
        if args.no_cpu_baseline:
            weights_for_oracle = None
        del host

    if not args.no_ceiling:
        # empirical ceiling, outside the timed region: the same kernel on the plan that is one memmove
        # (one memmove per slab in a layer-major pool)
        gbps, avg, mn = contiguous_ceiling(wk, torch, pool_t, cfg, n_moves, stream, tuning, layer_stride=layer_stride)
        out["roofline"]["ceiling_contiguous_GBps"] = round(gbps, 2)
        out["roofline"]["ceiling_kernel_ms_avg"] = round(avg, 4)
        out["roofline"]["frac_of_ceiling"] = round(out["roofline"]["achieved"] / gbps, 4)

    if args.vmm_compare:
        del pool_t
        torch.cuda.empty_cache()
        vcfg = cfg.scaled(num_blocks=args.vmm_compare)
        vw = make_workload(vcfg)
        want = vcfg.num_blocks - vcfg.boundary
        t0 = time.perf_counter()
        vp = wk.kv_vmm_pool_create(vcfg.num_blocks, vcfg.block_bytes)
        t1 = time.perf_counter()
        wk.kv_vmm_reclaim(vp, vw.live, want)
        t2 = time.perf_counter()
        wk.kv_vmm_restore(vp)
        t3 = time.perf_counter()
        piped = None
        if host_weights is not None and want * vcfg.block_bytes >= host_weights[3][-1] + host_weights[2][-1]:
            # the paper's way of hiding the mapping cost: weight copies pipelined behind the mapping
            h_t, h_starts, h_sizes, h_offs = host_weights
            h_tensors = [(h_t.data_ptr() + a, b_, c) for a, b_, c in zip(h_starts, h_sizes, h_offs)]
            vs = torch.cuda.Stream()
            torch.cuda.synchronize()
            t4 = time.perf_counter()
            wk.kv_vmm_reclaim_load(vp, vw.live, want, h_tensors, vs.cuda_stream, 0)
            t5 = time.perf_counter()
            torch.cuda.synchronize()
            t6 = time.perf_counter()
            wk.kv_vmm_restore(vp)
            piped = {"mapping_with_copies_enqueued_ms": round((t5 - t4) * 1e3, 1),
                     "until_last_weight_byte_ms": round((t6 - t4) * 1e3, 1),
                     "note": "kv_vmm_reclaim_load: 64 blocks mapped at a time, the weight bytes under each chunk enqueued "
                             "on a copy stream as soon as it is mapped (225 tensors, 15,009,316,864 B)"}
        wk.kv_vmm_pool_destroy(vp)
        out["vmm_compare"] = {"workload": f"{vcfg.num_blocks} blocks of {vcfg.block_bytes} B, pages of the {want} highest "
                                          f"free blocks ({want * vcfg.block_bytes / 2**30:.2f} GiB) remapped into the slot",
                              "create_ms": round((t1 - t0) * 1e3, 1), "reclaim_ms": round((t2 - t1) * 1e3, 1),
                              "reclaim_us_per_block": round((t2 - t1) * 1e6 / want, 1),
                              "restore_ms": round((t3 - t2) * 1e3, 1),
                              "pipelined_with_weight_stream": piped}

    if not args.no_cpu_baseline:
        # bounded sample: every move of this workload, capped at 12 GiB moved (24 GiB of host memory touched)
        out["cpu_baseline"] = cpu_baseline(cfg, w, sample_moves=max(1, (12 << 30) // bb), weights=weights_for_oracle)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

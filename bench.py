#!/usr/bin/env python3
"""Benchmark of the hashed-embedding hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: bag offsets -> ID hashing -> pooled lookup (forward)
-> sort / unique / segment-reduce -> row-wise Adagrad (backward), on the
16-table workload (16 x 1e7 rows x 64 fp32, 8192 bags per table, Poisson(20)
bag lengths, Zipf(1.05) raw IDs, mean pooling).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 3]
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

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak

METRIC = "pooled lookups/sec and achieved HBM GB/s (EmbeddingBag fwd + sparse Adagrad bwd)"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# HBM traffic per launch, from rocprofv3 --pmc (FETCH_SIZE in one run, WRITE_SIZE in another; KiB per
# dispatch, averaged over the dispatches of a run of this script), for the kernel sources whose digest
# is recorded with them: once a source file under csrc/ changes, `traffic` is reported as null until
# the counters are taken again.  The scale factors come from kernels of known traffic in the same
# runs: the 512 MiB device copy of --pmc-calibration reads 524288 KiB and FETCH_SIZE shows 262172
# (factor 2.0: the counter prices this part's 128-byte read requests as 64 bytes); the copy's and the
# table fill's writes (524288 and 2500000 KiB) are counted exactly (factor 1.0).  Read requests of 64
# bytes or less are counted at their true size, so for kernels that issue those (4-byte accumulators,
# 48-byte quantised rows) the scaled figure is an upper bound.
PMC_TRAFFIC = {
    "sources": "b73ec1126545090a",
    "fetch_scale": 2.0,
    "write_scale": 1.0,
    "kib_per_launch": {     # workload -> kernel -> (FETCH_SIZE, WRITE_SIZE)
        "3": {"bag_forward_train_kernel": (177568.9, 68960.1), "update_kernel": (240525.8, 324005.4)},
        "3b": {"bag_forward_train_kernel": (94766.7, 83182.2), "update_kernel": (169998.0, 220262.5)},
        "2": {"bag_forward_hashed_kernel": (176278.2, 33800.9), "bag_forward_kernel": (177913.7, 32768.0)},
        "2u": {"bag_forward_hashed_kernel": (338181.9, 33793.6), "bag_forward_kernel": (338144.8, 32768.0)},
        "2un": {"bag_forward_kernel": (346124.6, 32768.0)},
        "2q4": {"bag_forward_quant_kernel": (122247.6, 33832.7)},
        "2uq4": {"bag_forward_quant_kernel": (232535.4, 33926.1)},
        "2uq4r": {"bag_forward_quant_kernel": (190417.8, 33872.1)},
        "4": {"bag_forward_hashed_kernel": (52665.0, 8704.2)},
    },
}


def kernel_sources_digest() -> str:
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2508_05700_amd", "csrc", "*"))):
        with open(f, "rb") as fh:
            h.update(os.path.basename(f).encode() + b"\0" + fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` on `workload` (see PMC_TRAFFIC), or None."""
    kib = PMC_TRAFFIC["kib_per_launch"].get(workload, {}).get(kernel)
    if kib is None or PMC_TRAFFIC["sources"] != kernel_sources_digest():
        return None
    return int(round((kib[0] * PMC_TRAFFIC["fetch_scale"] + kib[1] * PMC_TRAFFIC["write_scale"]) * 1024))


def traffic_source(traffic):
    """Where a `traffic` figure comes from (it is never measured by the run that prints it)."""
    if traffic is None:
        return ("none: no counter run exists for this kernel and workload with the kernel sources as they are "
                "(digest %s)" % kernel_sources_digest())
    return ("carried from earlier rocprofv3 --pmc runs of this command (FETCH_SIZE x %.1f + WRITE_SIZE x %.1f, KiB per "
            "dispatch; profiles/hbm_traffic_pmc.md), taken with kernel sources of digest %s, which are the ones built "
            "now; not re-measured in this run" % (PMC_TRAFFIC["fetch_scale"], PMC_TRAFFIC["write_scale"],
                                                   PMC_TRAFFIC["sources"]))


def forward_bytes(nnz: int, bags: int, D: int, row_bytes: int) -> int:
    """Algorithmic bytes of one gather-pool launch: per lookup one table row and
    one 8-byte index; per bag one fp32 output row and one 8-byte offset."""
    return nnz * (row_bytes + 8) + bags * (4 * D + 8) + 8


def backward_bytes(nnz: int, bags: int, uniq: int, D: int, esz: int, passes: int) -> int:
    """Algorithmic bytes of one backward: per lookup its index (8) and 16 bytes
    (key+payload read and written) per radix pass; per bag its gradient row once;
    per distinct row one read and one write of the row plus its accumulator."""
    return nnz * (8 + 16 * passes) + bags * 4 * D + uniq * (2 * D * esz + 8)


def _oracle_batch_inputs(w, b, seed):
    """Index stage of one batch by the oracle (timed by the caller) is separate; this builds what
    the pooled lookup and the backward read: hashed rows, offsets and the host tables (untimed)."""
    import numpy as np

    from oracle import emb_oracle as oracle
    from paper_2508_05700_amd import workloads as wl

    t0 = time.perf_counter()
    off, _ = oracle.lengths_to_offsets(b["lengths"])
    if b["raw"] is not None:
        rows_np = np.concatenate([oracle.hash_ids(b["raw"][off[t * w.B]:off[(t + 1) * w.B]], w.salt(t), w.R)
                                  for t in range(w.T)])
    else:
        rows_np = b["rows"]
    t_index = time.perf_counter() - t0
    if w.quant:
        # compact quantised tables holding the touched rows only (the oracle's own quantiser, not
        # timed), lookups renumbered to match: denser than a full table, which flatters the CPU
        tables, parts = [], []
        for t in range(w.T):
            seg = rows_np[off[t * w.B]:off[(t + 1) * w.B]]
            touched = np.unique(seg)
            tables.append(oracle.quantize_rows(wl.table_values(w.table_seed(t, seed), touched, w.D), w.codes))
            parts.append(np.searchsorted(touched, seg))
        rows_np = np.concatenate(parts).astype(np.int64)
    else:
        tables = [wl.sparse_host_table(w.table_seed(t, seed), w.R, w.D, w.dtype,
                                       rows_np[off[t * w.B]:off[(t + 1) * w.B]]) for t in range(w.T)]
    return off, rows_np, tables, t_index


def _oracle_one_table(w, t, off, rows_np, tables, acc, dout):
    """The oracle's forward (and backward) over table t alone: the tables of a batch are independent."""
    from oracle import emb_oracle as oracle

    s, e = int(off[t * w.B]), int(off[(t + 1) * w.B])
    off_t = off[t * w.B:(t + 1) * w.B + 1] - s
    store = w.codes if w.quant else w.dtype     # the oracle reads the codes; row padding is layout only
    kw = {"D": w.D} if w.quant else {}
    oracle.bag_forward([tables[t]], store, rows_np[s:e], off_t, w.B, w.pool, want_absum=False, **kw)
    if w.backward:
        oracle.bag_backward_rowwise_adagrad([tables[t]], [acc[t]], w.dtype, rows_np[s:e], off_t, w.B, w.pool,
                                            dout[t:t + 1], w.lr, w.eps, want_G=False)


def cpu_baseline(w, batches_np, seed, min_seconds=10.0, max_batches=8):
    """The oracle, untuned, on whole batches of the same workload until about ``min_seconds`` of
    oracle time have been spent: first on one thread (the figure reported as ``value``), then the
    same oracle functions on all host cores, one table per call and one call per thread (the tables
    of a batch are independent; nothing in the oracle changes).  Host tables are full-size virtual
    arrays in which only the rows a batch touches are materialised (building them is not timed); the
    oracle's gathers then hit the same scattered addresses a fully materialised table would."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor

    from oracle import emb_oracle as oracle

    t_index = t_f = t_b = 0.0
    lookups = 0
    used = 0
    for b in batches_np[:max_batches]:
        off, rows_np, tables, ti = _oracle_batch_inputs(w, b, seed)
        t_index += ti
        store = w.codes if w.quant else w.dtype
        kw = {"D": w.D} if w.quant else {}
        t0 = time.perf_counter()
        oracle.bag_forward(tables, store, rows_np, off, w.B, w.pool, want_absum=False, **kw)
        t_f += time.perf_counter() - t0
        if w.backward:
            acc = [np.zeros(w.R, dtype=np.float32) for _ in range(w.T)]
            t0 = time.perf_counter()
            oracle.bag_backward_rowwise_adagrad(tables, acc, w.dtype, rows_np, off, w.B, w.pool, b["dout"], w.lr,
                                                w.eps, want_G=False)
            t_b += time.perf_counter() - t0
        lookups += int(b["nnz"])
        used += 1
        del tables
        if t_index + t_f + t_b >= min_seconds:
            break
    t_all = t_index + t_f + t_b
    log("cpu oracle: %d batches, %.2f s -> %.3g lookups/s on 1 core" % (used, t_all, lookups / t_all))
    result = {"value": round(lookups / t_all, 1), "unit": "lookups/s", "cores": 1, "kind": "oracle",
              "sample": "%d full batches of the same workload (%d lookups, all %d tables): offsets+hash %.2f s, "
                        "forward %.2f s, backward %.2f s of oracle time; single thread; host tables hold only "
                        "the touched rows" % (used, lookups, w.T, t_index, t_f, t_b)}

    # ---- the same oracle on all host cores: one table per call, one call per thread
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    threads = max(1, min(cores, w.T, 16))     # a one-GPU machine's share of the host is 16 cores
    if threads > 1:
        t_par = 0.0
        lookups_par = 0
        with ThreadPoolExecutor(max_workers=threads) as pool:
            for b in batches_np[:used]:
                off, rows_np, tables, ti = _oracle_batch_inputs(w, b, seed)
                acc = [np.zeros(w.R, dtype=np.float32) for _ in range(w.T)] if w.backward else None
                t0 = time.perf_counter()
                list(pool.map(lambda t: _oracle_one_table(w, t, off, rows_np, tables, acc, b.get("dout")), range(w.T)))
                t_par += ti + time.perf_counter() - t0      # the index stage stays on one thread
                lookups_par += int(b["nnz"])
                del tables
        log("cpu oracle: the same %d batches with %d threads (one table per call; %d cores visible) -> %.3g lookups/s" % (
            used, threads, cores, lookups_par / t_par))
        result["all_cores"] = {"value": round(lookups_par / t_par, 1), "unit": "lookups/s", "cores": threads,
                               "cores_visible": cores, "kind": "oracle",
                               "how": "the same oracle functions called once per table from %d threads (the tables of a "
                                      "batch are independent); offsets and hashing stay on one thread" % threads}
    return result


def stream_read_rate(data, nbytes=None, reps=5):
    """GB/s of emb_checksum (a plain streaming read) over ``data``: a device tensor, or a device-visible
    pointer with ``nbytes``."""
    import torch

    from paper_2508_05700_amd import binding as emb

    n = nbytes if isinstance(data, int) else data.numel() * data.element_size()
    out = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    emb.emb_checksum(data, out, nbytes)
    ev = [emb.Event(timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(reps):
        emb.emb_checksum(data, out, nbytes)
    ev[1].record()
    torch.cuda.synchronize()
    return reps * n / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9


def stream_copy_rate(nbytes=1 << 30, reps=5):
    """GB/s (bytes read + bytes written) of a plain device-to-device copy of ``nbytes``: what this
    part delivers to a kernel whose traffic is half reads, half writes."""
    import torch

    from paper_2508_05700_amd import binding as emb

    src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0").fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev = [emb.Event(timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(reps):
        dst.copy_(src)
    ev[1].record()
    torch.cuda.synchronize()
    return reps * 2 * nbytes / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9


def bench_hybrid(args) -> int:
    """Workload 5: pooled lookup over a table in pinned host memory fronted by an HBM cache of the
    hottest 5 % of rows.  A step is offsets + hashing + the cached forward; misses cross PCIe."""
    import numpy as np
    import psutil
    import torch

    from paper_2508_05700_amd import binding as emb
    from paper_2508_05700_amd import pipeline, workloads as wl

    seed = wl.DEFAULT_SEED if args.seed is None else args.seed
    w = wl.WORKLOADS[args.workload]
    store = w.storage
    rowb = emb.emb_row_bytes(w.D, store)
    need = w.R * rowb + (26 << 30)
    if args.scale_rows:
        w = w.scaled(rows=args.scale_rows)
    elif psutil.virtual_memory().available < need:
        w = w.scaled(rows=w.R // 4)
        log("workload %s scaled to %d rows: not enough host memory to pin %.0f GB" % (args.workload, w.R, need / 2 ** 30))
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, W = args.steps, args.warmup
    t_setup = time.time()
    if w.quant:
        # the fp32 table is filled in HBM, quantised row by row into the pinned host table, and dropped
        host = torch.empty((w.R, rowb), dtype=torch.uint8, pin_memory=True)
        ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
        src = torch.empty((w.R, w.D), dtype=torch.float32, device=dev)
        emb.emb_table_fill(src, w.R, w.D, "f32", w.table_seed(0, seed))
        emb.emb_quantize_rows(src, store, ptr)
        torch.cuda.synchronize()
        del src
        torch.cuda.empty_cache()
    else:
        host = torch.empty((w.R, w.D), dtype=torch.float32, pin_memory=True)
        ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
        emb.emb_table_fill(ptr, w.R, w.D, "f32", w.table_seed(0, seed))
    n_hot = int(round(w.hot_fraction * w.R))
    n_ranks = int(n_hot * 1.06) + 1000
    hot_raw = torch.from_numpy(wl.hot_raw_ids(w, 0, n_ranks, seed).view(np.int64)).to(dev)
    hot_rows = torch.empty(n_ranks, dtype=torch.int64, device=dev)
    emb.emb_hash_ids(hot_raw, w.salt(0), w.R, hot_rows)
    hot = torch.from_numpy(wl.first_k_distinct_sorted(hot_rows.cpu().numpy(), n_hot)).to(dev)
    n_hot = hot.numel()
    del hot_raw, hot_rows
    index = torch.empty(emb.emb_cache_index_bytes(w.R), dtype=torch.uint8, device=dev)
    cache = (torch.empty((n_hot, rowb), dtype=torch.uint8, device=dev) if w.quant
             else torch.empty((n_hot, w.D), dtype=torch.float32, device=dev))
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    emb.emb_cache_build(ptr, w.R, w.D, store, hot, cache, index, status)
    dbs = [pipeline.DeviceBatch(w, wl.make_batch(w, i, seed), dev) for i in range(args.batches)]
    max_nnz = max(d.nnz for d in dbs)
    offsets = torch.empty(w.B + 1, dtype=torch.int64, device=dev)
    rows = torch.empty(max_nnz, dtype=torch.int64, device=dev)
    out = torch.empty((1, w.B, w.D), dtype=torch.float32, device=dev)
    hm = torch.zeros(2, dtype=torch.int64, device=dev)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    log("setup: host table %d x %d %s (%.1f GB pinned), cache %d rows (%.2f GB), %.1f s" % (
        w.R, w.D, store, w.R * rowb / 1e9, n_hot, n_hot * rowb / 1e9, time.time() - t_setup))

    from_lengths = (not args.no_fused_forward and not args.separate_offsets
                    and w.B <= pipeline.LENGTHS_ROUTE_MAX_BAGS)
    off_scratch = torch.empty(emb.emb_offsets_scratch_bytes(w.B), dtype=torch.uint8, device=dev)

    def step(db, e=None):
        if e:
            e[0].record()
        if from_lengths:   # bag lengths in: the sums within tiles, then the lookup, which the library brackets itself
            emb.emb_bag_forward_cached_hashed_lengths(ptr, w.R, w.D, store, cache, index, n_hot, w.salt(0), db.raw,
                                                      db.lengths, w.B, w.pool, out, offsets, off_scratch, hm, status,
                                                      lookup_events=(e[1], e[2]) if e else None)
            return
        emb.emb_lengths_to_offsets(db.lengths, offsets, status)
        if args.no_fused_forward:
            r = rows[:db.nnz]
            emb.emb_hash_ids(db.raw, w.salt(0), w.R, r)
        if e:
            e[1].record()
        if args.no_fused_forward:
            emb.emb_bag_forward_cached(ptr, w.R, w.D, store, cache, index, n_hot, r, offsets, w.B, w.pool, out, hm,
                                       status)
        else:    # hashing inside the lookup
            emb.emb_bag_forward_cached_hashed(ptr, w.R, w.D, store, cache, index, n_hot, w.salt(0), db.raw, offsets,
                                              w.B, w.pool, out, hm, status)
        if e:
            e[2].record()

    E = args.event_every        # stages are bracketed by events on every E-th step only (an event costs microseconds)
    ev = [[emb.Event(timing=True) for _ in range(3)] for _ in range((K + E - 1) // E)]
    for i in range(W):          # the first warm-up step carries the event brackets too (their first use is not timed)
        step(dbs[i % len(dbs)], ev[0] if i == 0 else None)
    torch.cuda.synchronize()
    hm.zero_()
    t0 = time.perf_counter()
    for k in range(K):
        step(dbs[(W + k) % len(dbs)], ev[k // E] if k % E == 0 else None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert int(status.item()) == 0
    lookups = sum(dbs[(W + k) % len(dbs)].nnz for k in range(K))
    hits, misses = [int(x) for x in hm.cpu().tolist()]
    ms_index = sum(e[0].elapsed_time(e[1]) for e in ev) / len(ev)
    ms_fwd = sum(e[1].elapsed_time(e[2]) for e in ev) / len(ev)
    pcie_gbs = misses / K * rowb / (ms_fwd * 1e-3) / 1e9
    hbm_gbs = (hits / K * rowb + lookups / K * 24 + w.B * (4 * w.D + 8)) / (ms_fwd * 1e-3) / 1e9

    # what the link delivers to a plain DMA copy from the same pinned buffer (context for the PCIe rate)
    n_copy = min(w.R, (1 << 30) // rowb)
    staging = torch.empty((n_copy, host.shape[1]), dtype=host.dtype, device=dev)
    staging.copy_(host[:n_copy], non_blocking=True)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(3):
        staging.copy_(host[:n_copy], non_blocking=True)
    c1.record()
    torch.cuda.synchronize()
    dma_gbs = 3 * n_copy * rowb / (c0.elapsed_time(c1) * 1e-3) / 1e9
    zc_gbs = stream_read_rate(ptr, nbytes=min(w.R * rowb, 4 << 30) // 16 * 16, reps=2)   # a kernel streaming the pinned table
    log("step %.3f ms: index %.3f, cached forward %.3f; hit rate %.2f %%; misses %.1f GB/s over PCIe "
        "(DMA copy from the same buffer: %.1f GB/s, streaming zero-copy read: %.1f GB/s); HBM side %.0f GB/s" % (
            elapsed / K * 1e3, ms_index, ms_fwd, 100.0 * hits / max(1, hits + misses), pcie_gbs, dma_gbs, zc_gbs,
            hbm_gbs))
    policy = cache_policy_study(args, w, seed, ptr, store, n_hot, hot, dbs, offsets, out, W, K) \
        if args.cache_policy == "dynamic" else None
    PCIE_PEAK = 64.0   # PCIe Gen5 x16, nominal, one direction

    # ---- the same batches with the misses of several batches fetched ahead, in one launch -------------
    # A step is still one batch: its share of the staging launch plus its own offsets and pooled lookup.
    G = max(1, min(args.stage_batches, len(dbs)))
    groups = [dbs[i:i + G] for i in range(0, len(dbs) - G + 1, G)]
    graw = [torch.cat([d.raw for d in g]) for g in groups]
    gnnz = [[d.nnz for d in g] for g in groups]
    cap = int(max(sum(n) for n in gnnz) * 0.2) + 1024          # room for a miss rate of 20 %
    stage = (torch.empty((cap, rowb), dtype=torch.uint8, device=dev) if w.quant
             else torch.empty((cap, w.D), dtype=torch.float32, device=dev))
    loc = torch.empty(max(sum(n) for n in gnnz), dtype=torch.int64, device=dev)
    count = torch.zeros(1, dtype=torch.int64, device=dev)
    goff = [torch.empty(w.B + 1, dtype=torch.int64, device=dev) for _ in range(G)]
    hm2 = torch.zeros(2, dtype=torch.int64, device=dev)

    def staged_group(gi, e=None, counts=None):
        count.zero_()
        if e:
            e[0].record()
        emb.emb_cache_stage_misses(ptr, w.R, w.D, store, index, n_hot, graw[gi], stage, cap, loc, count, status,
                                   salt=w.salt(0))
        if e:
            e[1].record()
        at = 0
        for k, d in enumerate(groups[gi]):
            emb.emb_lengths_to_offsets(d.lengths, goff[k], status)
            emb.emb_bag_forward_staged(ptr, w.R, w.D, store, cache, n_hot, stage, cap, loc[at:at + d.nnz], goff[k], w.B,
                                       w.pool, out, counts, status)
            at += d.nnz
        if e:
            e[2].record()

    for i in range(max(1, W // G)):
        staged_group(i % len(groups))
    torch.cuda.synchronize()
    hm2.zero_()
    n_groups = max(1, K // G)
    gev = [[emb.Event(timing=True) for _ in range(3)] for _ in range(n_groups)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n_groups):
        staged_group(i % len(groups), gev[i] if i % E == 0 else None)
    torch.cuda.synchronize()
    el2 = time.perf_counter() - t0
    assert int(status.item()) == 0
    timed = [e for i, e in enumerate(gev) if i % E == 0]
    ms_stage = sum(e[0].elapsed_time(e[1]) for e in timed) / len(timed)
    ms_lookups = sum(e[1].elapsed_time(e[2]) for e in timed) / len(timed)
    # hits and misses are counted in a pass of their own (the timed lookups do not ask for them: thousands of
    # wavefronts adding to the same two counters cost more than such a lookup over HBM takes)
    for i in range(n_groups):
        staged_group(i % len(groups), None, hm2)
    torch.cuda.synchronize()
    h2, m2 = [int(x) for x in hm2.cpu().tolist()]
    lookups2 = sum(sum(gnnz[i % len(groups)]) for i in range(n_groups))
    stage_gbs = m2 / n_groups * rowb / (ms_stage * 1e-3) / 1e9
    staged = {"batches_per_staging_launch": G, "ms_per_batch": round(el2 / (n_groups * G) * 1e3, 4),
              "lookups_per_s": round(lookups2 / el2, 1), "stage_launch_ms": round(ms_stage, 4),
              "offsets_and_lookups_ms_per_group": round(ms_lookups, 4), "misses_per_launch": round(m2 / n_groups, 1),
              "hit_rate": round(h2 / max(1, h2 + m2), 5), "pcie_GBps": round(stage_gbs, 2),
              "pcie_frac_of_nominal": round(stage_gbs / PCIE_PEAK, 4),
              "kernel": "stage_misses_kernel (resolves the lookups of %d batches, copies every missed row into HBM)" % G}
    log("misses of %d batches staged by one launch: %.3f ms per batch (staging launch %.3f ms: %.0f misses, %.1f GB/s over "
        "PCIe = %.0f %% of nominal; %d x (offsets + lookup over HBM) %.3f ms)" % (
            G, staged["ms_per_batch"], ms_stage, m2 / n_groups, stage_gbs, 100 * stage_gbs / PCIE_PEAK, G, ms_lookups))
    out_json = {
        "metric": METRIC, "value": round(lookups / elapsed, 1), "unit": "lookups/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": round(elapsed / K * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: host-resident table %d rows x dim %d %s (%d B per row, pinned) + HBM cache of %d "
                               "hot rows, %d bags, poisson bag lengths (mean %g), zipf IDs alpha=%g over %.0e keys, "
                               "%s pooling, forward only" % (w.name, w.R, w.D, store, rowb, n_hot, w.B, w.mean_len,
                                                             w.alpha, w.n_keys, w.pool),
                   "lookups_per_step": round(lookups / K, 1), "resident_batches": len(dbs), "seed": seed},
        "stages": {"index_ms": round(ms_index, 4), "forward_cached_ms": round(ms_fwd, 4),
                   "hit_rate": round(hits / max(1, hits + misses), 5), "misses_per_step": round(misses / K, 1)},
        "roofline": {"kernel": "bag_forward_cached_quant_kernel" if w.quant else "bag_forward_cached_kernel",
                     "bag_offsets": ("made inside the lookup's call (the kernel is bracketed by events the library "
                                     "records)" if from_lengths else "separate launches"),
                     "bound": "pcie", "achieved": round(pcie_gbs, 2),
                     "peak": PCIE_PEAK, "unit": "GB/s", "frac": round(pcie_gbs / PCIE_PEAK, 4), "traffic": None,
                     "avg_ms": round(ms_fwd, 4), "algorithmic_bytes": int(misses / K * rowb),
                     "bytes_are": "one table row per miss, read zero-copy from pinned host memory",
                     "dma_copy_same_buffer_GBps": round(dma_gbs, 1), "zero_copy_stream_read_GBps": round(zc_gbs, 1),
                     "hbm_side_GBps": round(hbm_gbs, 1)},
        "staged": staged,
        "cpu_baseline": None,
    }
    if policy is not None:
        out_json["cache_policy"] = policy
    print(json.dumps(out_json), flush=True)
    return 0


def bench_hybrid_tables(args) -> int:
    """Workloads 5m / 5mq4: several hosted tables, each with its HBM cache.  A step is offsets + ONE cached
    lookup over all tables (hashing inside); the same step with one cached lookup per table is timed beside
    it."""
    import numpy as np
    import psutil
    import torch

    from paper_2508_05700_amd import binding as emb
    from paper_2508_05700_amd import pipeline, workloads as wl

    seed = wl.DEFAULT_SEED if args.seed is None else args.seed
    w = wl.WORKLOADS[args.workload]
    store = w.storage
    rowb = emb.emb_row_bytes(w.D, store)
    if args.scale_rows:
        w = w.scaled(rows=args.scale_rows)
    elif psutil.virtual_memory().available < w.T * w.R * rowb + (26 << 30):
        w = w.scaled(rows=w.R // 4)
        log("workload %s scaled to %d rows per table: not enough host memory to pin the tables" % (args.workload, w.R))
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, W = args.steps, args.warmup
    t_setup = time.time()
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    n_hot = int(round(w.hot_fraction * w.R))
    hosts, entries = [], []
    for t in range(w.T):
        if w.quant:
            host = torch.empty((w.R, rowb), dtype=torch.uint8, pin_memory=True)
            ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
            src = torch.empty((w.R, w.D), dtype=torch.float32, device=dev)
            emb.emb_table_fill(src, w.R, w.D, "f32", w.table_seed(t, seed))
            emb.emb_quantize_rows(src, store, ptr)
            torch.cuda.synchronize()
            del src
        else:
            host = torch.empty((w.R, w.D), dtype=torch.float32, pin_memory=True)
            ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
            emb.emb_table_fill(ptr, w.R, w.D, "f32", w.table_seed(t, seed))
        n_ranks = int(n_hot * 1.06) + 1000
        hot_raw = torch.from_numpy(wl.hot_raw_ids(w, t, n_ranks, seed).view(np.int64)).to(dev)
        hot_rows = torch.empty(n_ranks, dtype=torch.int64, device=dev)
        emb.emb_hash_ids(hot_raw, w.salt(t), w.R, hot_rows)
        hot = torch.from_numpy(wl.first_k_distinct_sorted(hot_rows.cpu().numpy(), n_hot)).to(dev)
        index = torch.empty(emb.emb_cache_index_bytes(w.R), dtype=torch.uint8, device=dev)
        cache = (torch.empty((hot.numel(), rowb), dtype=torch.uint8, device=dev) if w.quant
                 else torch.empty((hot.numel(), w.D), dtype=torch.float32, device=dev))
        emb.emb_cache_build(ptr, w.R, w.D, store, hot, cache, index, status)
        hosts.append(host)
        entries.append((ptr, w.R, cache, index, hot.numel(), w.salt(t)))
    torch.cuda.empty_cache()
    ct = emb.CachedTables(entries, w.D, store, device=dev)
    dbs = [pipeline.DeviceBatch(w, wl.make_batch(w, i, seed), dev) for i in range(args.batches)]
    offsets = torch.empty(w.T * w.B + 1, dtype=torch.int64, device=dev)
    out = torch.empty((w.T, w.B, w.D), dtype=torch.float32, device=dev)
    hm = torch.zeros(2, dtype=torch.int64, device=dev)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    log("setup: %d host tables %d x %d %s (%.1f GB pinned in all), caches of %d rows each, %.1f s" % (
        w.T, w.R, w.D, store, w.T * w.R * rowb / 1e9, n_hot, time.time() - t_setup))

    from_lengths = not args.separate_offsets and w.T * w.B <= pipeline.LENGTHS_ROUTE_MAX_BAGS
    off_scratch = torch.empty(emb.emb_offsets_scratch_bytes(w.T * w.B), dtype=torch.uint8, device=dev)

    def step_one_launch(db, e=None):
        if from_lengths:   # bag lengths in: the library brackets the lookup kernel itself
            emb.emb_bag_forward_cached_tables_hashed_lengths(ct, db.raw, db.lengths, w.B, w.pool, out, offsets,
                                                             off_scratch, hm, status,
                                                             lookup_events=(e[0], e[1]) if e else None)
            return
        emb.emb_lengths_to_offsets(db.lengths, offsets, status)
        if e:
            e[0].record()
        emb.emb_bag_forward_cached_tables_hashed(ct, db.raw, offsets, w.B, w.pool, out, hm, status)
        if e:
            e[1].record()

    def step_per_table(db, e=None):
        emb.emb_lengths_to_offsets(db.lengths, offsets, status)
        if e:
            e[0].record()
        for t, (ptr, R, cache, index, nh, salt) in enumerate(entries):
            # the table's B+1 offsets index the whole ID array
            emb.emb_bag_forward_cached_hashed(ptr, R, w.D, store, cache, index, nh, salt, db.raw,
                                              offsets[t * w.B:(t + 1) * w.B + 1], w.B, w.pool, out[t:t + 1], hm, status)
        if e:
            e[1].record()

    def run(step):
        E = args.event_every    # the lookups are bracketed by events on every E-th step only
        ev = [[emb.Event(timing=True) for _ in range(2)] for _ in range((K + E - 1) // E)]
        for i in range(W):      # the first warm-up step carries the event brackets too
            step(dbs[i % len(dbs)], ev[0] if i == 0 else None)
        torch.cuda.synchronize()
        hm.zero_()
        t0 = time.perf_counter()
        for k in range(K):
            step(dbs[(W + k) % len(dbs)], ev[k // E] if k % E == 0 else None)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        hits, misses = [int(x) for x in hm.cpu().tolist()]
        return dt, sum(e[0].elapsed_time(e[1]) for e in ev) / len(ev), hits, misses

    dt_pt, ms_pt, _, _ = run(step_per_table)
    elapsed, ms_fwd, hits, misses = run(step_one_launch)
    assert int(status.item()) == 0
    lookups = sum(dbs[(W + k) % len(dbs)].nnz for k in range(K))
    pcie_gbs = misses / K * rowb / (ms_fwd * 1e-3) / 1e9
    log("step %.3f ms: one cached lookup over %d tables %.3f ms (one lookup per table: step %.3f ms, lookups %.3f ms); "
        "hit rate %.2f %%; misses %.1f GB/s over PCIe" % (elapsed / K * 1e3, w.T, ms_fwd, dt_pt / K * 1e3, ms_pt,
                                                         100.0 * hits / max(1, hits + misses), pcie_gbs))
    PCIE_PEAK = 64.0
    print(json.dumps({
        "metric": METRIC, "value": round(lookups / elapsed, 1), "unit": "lookups/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": round(elapsed / K * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d host-resident tables of %d rows x dim %d %s (%d B per row, pinned), each with an HBM "
                               "cache of %d hot rows, %d bags per table, poisson bag lengths (mean %g), zipf IDs alpha=%g "
                               "over %.0e keys, %s pooling, forward only, one launch for all tables" % (
                                   w.name, w.T, w.R, w.D, store, rowb, n_hot, w.B, w.mean_len, w.alpha, w.n_keys, w.pool),
                   "lookups_per_step": round(lookups / K, 1), "resident_batches": len(dbs), "seed": seed},
        "stages": {"forward_cached_tables_ms": round(ms_fwd, 4), "hit_rate": round(hits / max(1, hits + misses), 5),
                   "misses_per_step": round(misses / K, 1),
                   "one_lookup_per_table": {"ms_per_step": round(dt_pt / K * 1e3, 4), "lookups_ms": round(ms_pt, 4)}},
        "roofline": {"kernel": "bag_forward_cached_tables_quant_kernel" if w.quant else "bag_forward_cached_tables_kernel",
                     "bag_offsets": ("made inside the lookup's call (the kernel is bracketed by events the library "
                                     "records)" if from_lengths else "separate launches"),
                     "bound": "pcie", "achieved": round(pcie_gbs, 2), "peak": PCIE_PEAK, "unit": "GB/s",
                     "frac": round(pcie_gbs / PCIE_PEAK, 4), "traffic": None, "avg_ms": round(ms_fwd, 4),
                     "algorithmic_bytes": int(misses / K * rowb),
                     "bytes_are": "one table row per miss, read zero-copy from pinned host memory"},
        "cpu_baseline": None,
    }), flush=True)
    return 0


def cache_policy_study(args, w, seed, ptr, store, n_hot, static_hot, dbs, offsets, out, W, K):
    """The frequency-based policy against the static hot set of the benchmark, on the same batches: the
    cache starts empty, watches a growing amount of traffic (lookups drawn like the batches'), and is
    refreshed after each stage; then the popularity moves to other IDs and it has to follow.  Reports hit
    rates, step times and what a refresh costs.  Not part of ``value``."""
    import torch

    from paper_2508_05700_amd import binding as emb
    from paper_2508_05700_amd import pipeline, workloads as wl

    dev = torch.device("cuda:0")
    cache = pipeline.HotRowCache(ptr, w.R, w.D, store, n_hot, w.salt(0), dev, decay_shift=1)
    status = cache.status
    chunk = 10_000_000
    next_chunk = [0]

    def watch(n, s):
        done = 0
        while done < n:
            m = min(chunk, n - done)
            raw = torch.from_numpy(wl.traffic_raw_ids(w, 0, m, next_chunk[0], s).view("int64")).to(dev)
            cache.observe(raw)
            next_chunk[0] += 1
            done += m
        torch.cuda.synchronize()

    def refresh():
        ev = [emb.Event(timing=True) for _ in range(3)]
        cache.moved.zero_()
        ev[0].record()
        emb.emb_cache_select(cache.freq, cache.capacity, cache.decay_shift, cache.workspace, cache.hot, cache.info)
        ev[1].record()
        new = 1 - cache.active
        emb.emb_cache_rebuild(ptr, w.R, w.D, store, cache.rows[cache.active], cache.index[cache.active], cache.num_hot,
                              cache.hot[:cache.capacity], cache.rows[new], cache.index[new], cache.moved, status)
        ev[2].record()
        cache.active, cache.num_hot = new, cache.capacity
        torch.cuda.synchronize()
        kept, fetched = [int(x) for x in cache.moved.cpu().tolist()]
        thr, tied = [int(x) for x in cache.info.cpu().tolist()]
        return {"select_ms": round(ev[0].elapsed_time(ev[1]), 3), "rebuild_ms": round(ev[1].elapsed_time(ev[2]), 3),
                "rows_kept_in_hbm": kept, "rows_fetched_from_table": fetched, "threshold_count": thr,
                "rows_at_threshold": tied}

    def measure(batches, fwd):
        """Hit rate and time per step of offsets + cached lookup over ``batches``."""
        for i in range(W):
            fwd(batches[i % len(batches)])
        torch.cuda.synchronize()
        cache.hit_miss.zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(K):
            fwd(batches[(W + k) % len(batches)])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        h, m = [int(x) for x in cache.hit_miss.cpu().tolist()]
        return round(h / max(1, h + m), 5), round(dt / K * 1e3, 4)

    def fwd_dynamic(db):
        emb.emb_lengths_to_offsets(db.lengths, offsets, status)
        cache.forward_hashed(db.raw, offsets, w.B, w.pool, out)

    static_index = torch.empty_like(cache.index[0])
    static_rows = torch.empty_like(cache.rows[0][:static_hot.numel()])
    emb.emb_cache_build(ptr, w.R, w.D, store, static_hot, static_rows, static_index, status)

    def fwd_static(db):
        emb.emb_lengths_to_offsets(db.lengths, offsets, status)
        emb.emb_bag_forward_cached_hashed(ptr, w.R, w.D, store, static_rows, static_index, static_hot.numel(), w.salt(0),
                                          db.raw, offsets, w.B, w.pool, out, cache.hit_miss, status)

    result = {"policy": "per-row u32 access counters; at a refresh the %d rows with the largest counters are kept "
                        "(ties to the smaller row), counters halved" % n_hot, "stages": []}
    hr, ms = measure(dbs, fwd_static)
    result["static"] = {"hit_rate": hr, "ms_per_step": ms}
    hr, ms = measure(dbs, fwd_dynamic)
    result["stages"].append({"watched_lookups": 0, "hit_rate": hr, "ms_per_step": ms})
    log("cache policy: static set %.2f %% hits (%.3f ms); empty cache %.2f %% (%.3f ms)" % (
        100 * result["static"]["hit_rate"], result["static"]["ms_per_step"], 100 * hr, ms))
    watched = 0
    for target in [int(float(x)) for x in args.watch_lookups.split(",")]:
        t0 = time.time()
        watch(target - watched, seed)
        watched = target
        st = {"watched_lookups": watched}
        st.update(refresh())
        st["hit_rate"], st["ms_per_step"] = measure(dbs, fwd_dynamic)
        result["stages"].append(st)
        log("cache policy: %.0e lookups watched (%.0f s): %.2f %% hits, step %.3f ms; refresh = select %.2f ms + "
            "rebuild %.2f ms (%d rows kept in HBM, %d fetched)" % (
                watched, time.time() - t0, 100 * st["hit_rate"], st["ms_per_step"], st["select_ms"], st["rebuild_ms"],
                st["rows_kept_in_hbm"], st["rows_fetched_from_table"]))
    # popularity moves: the same law over other IDs (another seed gives another rank -> ID map)
    seed2 = seed + 1
    moved_batches = [pipeline.DeviceBatch(w, wl.make_batch(w, i, seed2), dev) for i in range(len(dbs))]
    drift = {"static": dict(zip(("hit_rate", "ms_per_step"), measure(moved_batches, fwd_static))),
             "before_refresh": dict(zip(("hit_rate", "ms_per_step"), measure(moved_batches, fwd_dynamic))), "stages": []}
    watched = 0
    for target in [int(float(x)) for x in args.watch_lookups.split(",")][:2]:
        watch(target - watched, seed2)
        watched = target
        st = {"watched_lookups": watched}
        st.update(refresh())
        st["hit_rate"], st["ms_per_step"] = measure(moved_batches, fwd_dynamic)
        drift["stages"].append(st)
    result["after_popularity_moved"] = drift
    log("cache policy, popularity moved: static set %.2f %% hits, dynamic before refresh %.2f %%, after %s" % (
        100 * drift["static"]["hit_rate"], 100 * drift["before_refresh"]["hit_rate"],
        ", ".join("%.0e lookups: %.2f %%" % (s["watched_lookups"], 100 * s["hit_rate"]) for s in drift["stages"])))
    assert int(status.item()) == 0
    return result


def bench_mixed(args) -> int:
    """Workload "mix": offsets + hashing + ONE pooled-lookup launch over 24 tables of four widths and
    two storage types, output concatenated per sample."""
    import numpy as np
    import torch

    from paper_2508_05700_amd import binding as emb
    from paper_2508_05700_amd import pipeline, workloads as wl

    seed = wl.DEFAULT_SEED if args.seed is None else args.seed
    w = wl.WORKLOADS["mix"]
    spec = wl.MIX_SPEC
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, W = args.steps, args.warmup
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16}
    weights = []
    for t, (D, dt, R) in enumerate(spec):
        wt = torch.empty((R, D), dtype=tdt[dt], device=dev)
        emb.emb_table_fill(wt, R, D, dt, w.table_seed(t, seed))
        weights.append(wt)
    mt = emb.MixedTables(weights, w.B, "concat", salts=[w.salt(t) for t in range(w.T)], device=dev)
    dbs = [pipeline.DeviceBatch(w, wl.make_batch(w, i, seed), dev) for i in range(args.batches)]
    max_nnz = max(d.nnz for d in dbs)
    offsets = torch.empty(w.T * w.B + 1, dtype=torch.int64, device=dev)
    rows = torch.empty(max_nnz, dtype=torch.int64, device=dev)
    out = torch.empty(mt.out_floats, dtype=torch.float32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()

    def step(db, e=None):
        emb.emb_lengths_to_offsets(db.lengths, offsets, status)
        r = rows[:db.nnz]
        emb.emb_hash_ids_tables(mt.tables, db.raw, offsets, w.B, r, status)
        if e:
            e[0].record()
        emb.emb_bag_forward_mixed(mt, r, offsets, w.pool, out, status)
        if e:
            e[1].record()

    E = args.event_every        # the lookup is bracketed by events on every E-th step only
    ev = [[emb.Event(timing=True) for _ in range(2)] for _ in range((K + E - 1) // E)]
    for i in range(W):          # the first warm-up step carries the event brackets too
        step(dbs[i % len(dbs)], ev[0] if i == 0 else None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        step(dbs[(W + k) % len(dbs)], ev[k // E] if k % E == 0 else None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert int(status.item()) == 0
    lookups = sum(dbs[(W + k) % len(dbs)].nnz for k in range(K))
    ms_fwd = sum(e[0].elapsed_time(e[1]) for e in ev) / len(ev)
    # algorithmic bytes of the lookup: per lookup its table's row + 8 B index; per bag its output row + 8 B offset
    per_table = np.mean([b_["nnz_per_table"] for b_ in [wl.make_batch(w, i, seed) for i in range(1)]], axis=0)
    nbytes = sum(per_table[t] * (emb.emb_row_bytes(D, dt) + 8) + w.B * (4 * D + 8) for t, (D, dt, R) in enumerate(spec))
    gbs = nbytes / (ms_fwd * 1e-3) / 1e9
    log("step %.3f ms: mixed forward %.3f ms, %.0f GB/s algorithmic (%.1f %% of HBM peak)" % (
        elapsed / K * 1e3, ms_fwd, gbs, 100 * gbs / HBM_PEAK_GBS))
    print(json.dumps({
        "metric": METRIC, "value": round(lookups / elapsed, 1), "unit": "lookups/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": round(elapsed / K * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "mix: 24 tables (6 x dim 16 fp32 x 2e6 rows, 6 x dim 32 bf16 x 5e6, 8 x dim 64 fp32 x 1e7, "
                               "4 x dim 128 fp32 x 2e6), %d bags/table, poisson bag lengths (mean %g), zipf IDs "
                               "alpha=%g, %s pooling, one launch, output concatenated per sample, forward only" % (
                                   w.B, w.mean_len, w.alpha, w.pool),
                   "lookups_per_step": round(lookups / K, 1), "resident_batches": len(dbs), "seed": seed},
        "roofline": {"kernel": "bag_forward_mixed_kernel", "bound": "hbm", "achieved": round(gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "avg_ms": round(ms_fwd, 4), "algorithmic_bytes": int(nbytes),
                     "bytes_are": "row + 8 B index per lookup, fp32 output row + 8 B offset per bag"},
        "cpu_baseline": None}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="3",
                    help="3 (fwd+bwd, default), 3b (the same over bf16 tables), 1, 2, 2u or 4 (forward only), 2q4 / 2q8 / 2uq4 (forward over INT4 / "
                         "INT8 row-quantised tables), 5 / 5q4 (host table + HBM cache), 5m / 5mq4 (four hosted tables, one "
                         "launch), mix (tables of different width)")
    ap.add_argument("--batches", type=int, default=8, help="distinct resident batches cycled through")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--scale-rows", type=int, default=None, help="rows per table (debug: smaller tables)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--event-every", type=int, default=4,
                    help="bracket the dominant kernel with HIP events on every N-th timed step (1 = every step)")
    ap.add_argument("--versioned", action="store_true",
                    help="forward-only workloads: look up through a version handle (latch + lookup), returning (E, V)")
    ap.add_argument("--cache-policy", choices=["static", "dynamic"], default="static",
                    help="workloads 5/5q4: 'dynamic' adds the study of the frequency-based cache policy")
    ap.add_argument("--watch-lookups", default="1e6,1e7,1e8",
                    help="cumulative lookups the dynamic policy has watched at each refresh")
    ap.add_argument("--stage-batches", type=int, default=4,
                    help="workloads 5/5q4: batches whose misses one staging launch fetches ahead of their lookups")
    ap.add_argument("--no-extra", action="store_true", help="skip the forward-only side measurements")
    ap.add_argument("--no-fused-forward", action="store_true",
                    help="hash the IDs in a kernel of their own instead of inside the forward lookup")
    ap.add_argument("--separate-offsets", action="store_true",
                    help="bag offsets by emb_lengths_to_offsets (three launches) before the lookup, instead of inside "
                         "emb_bag_forward_train_lengths / emb_bag_forward_hashed_lengths")
    ap.add_argument("--overlap-sort", action="store_true",
                    help="enqueue the backward's sort on a second stream beside the forward (measured: no gain "
                         "here, the forward saturates HBM and the sort's small kernels only get slower)")
    ap.add_argument("--no-defer-join", action="store_true",
                    help="the backward makes the step's stream wait for its side stream at its own end, not in "
                         "the next step's lookup call")
    ap.add_argument("--no-side-stream", action="store_true",
                    help="run the backward's long-run path after the short-run update instead of beside it")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 512 MB device copy (a kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters by)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this library runs on ONE GPU only (no sharding, no collectives); use --gpus 1")
        return 2

    import numpy as np
    import torch

    from paper_2508_05700_amd import binding as emb
    from paper_2508_05700_amd import pipeline, workloads as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 2
    emb.lib()
    if wl.WORKLOADS[args.workload].hybrid:
        return bench_hybrid_tables(args) if wl.WORKLOADS[args.workload].T > 1 else bench_hybrid(args)
    if args.workload == "mix":
        return bench_mixed(args)
    seed = wl.DEFAULT_SEED if args.seed is None else args.seed
    w = wl.WORKLOADS[args.workload]
    if args.scale_rows:
        w = w.scaled(rows=args.scale_rows)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t_setup = time.time()
    tabs = pipeline.DeviceTables(w, seed)
    batches_np = [wl.make_batch(w, i, seed) for i in range(args.batches)]
    dbs = [pipeline.DeviceBatch(w, b, dev) for b in batches_np]
    max_nnz = max(d.nnz for d in dbs)
    buf = pipeline.StepBuffers(w, max_nnz, tabs.set.total_rows, dev, side_stream=not args.no_side_stream)
    torch.cuda.synchronize()
    log("setup: %d tables x %d rows x %d %s, %d batches of ~%d lookups, %.1f s" % (
        w.T, w.R, w.D, w.dtype, len(dbs), max_nnz, time.time() - t_setup))

    if args.pmc_calibration:
        cal_rowb = tabs.weights[0].shape[1] * tabs.weights[0].element_size()
        n_cal = min(w.R, (512 << 20) // cal_rowb)
        cal = tabs.weights[0][:n_cal].clone()      # plain copy kernel: reads and writes n_cal rows
        torch.cuda.synchronize()
        log("calibration copy: %d bytes read, %d bytes written" % (n_cal * cal_rowb, n_cal * cal_rowb))
        del cal

    K, W = args.steps, args.warmup
    fused = not args.no_fused_forward and not args.overlap_sort and dbs[0].raw is not None

    train_route = fused and w.backward     # the lookup also writes the backward's records
    offsets_inside = train_route and not args.separate_offsets   # ... and makes the bag offsets on the way
    # forward-only with hashing inside the lookup: the lookup also takes the bag lengths (up to 2^20 bags)
    lengths_route = (fused and not w.backward and not args.separate_offsets and not args.versioned
                     and w.T * w.B <= (1 << 20))
    off_scratch = (torch.empty(emb.emb_offsets_scratch_bytes(w.T * w.B), dtype=torch.uint8, device=dev)
                   if lengths_route else None)

    # The long-run half of a backward runs on a side stream.  The step's stream does not wait for it at the
    # end of the backward but in the next step, between that step's set-up launches (which touch neither
    # the tables nor the previous workspace) and its lookup: a wait met after the awaited work has ended
    # costs the stream almost nothing, one met before costs some 10 us.  Steps then alternate between two
    # workspaces.  All of it is work of the timed steps; the last join is waited for before the clock stops.
    defer_join = (offsets_inside and buf.side is not None and not args.no_defer_join)
    pair = [buf]
    if defer_join:
        second = pipeline.StepBuffers(w, max_nnz, tabs.set.total_rows, dev, side_stream=False)
        second.side, second.status = buf.side, buf.status
        buf.side.defer_join = True
        pair.append(second)
    steps_run = [0]

    def do_index(db):
        """Bag offsets, and the hashing unless it is fused into the forward.  Returns the rows (or None)."""
        if offsets_inside or lengths_route:
            return None
        if fused:
            emb.emb_lengths_to_offsets(db.lengths, buf.offsets, buf.status)
            return None
        return pipeline.run_index_stage(w, tabs.set, db, buf)

    versioned = args.versioned
    if versioned:
        if w.backward or not fused:
            log("--versioned applies to the forward-only workloads with hashing inside the lookup")
            return 2
        ver_record = torch.empty(emb.emb_version_record_bytes(w.T), dtype=torch.uint8, device=dev)
        ver_latch = torch.empty(emb.emb_version_latch_bytes(w.T), dtype=torch.uint8, device=dev)
        ver_handle = torch.zeros(1, dtype=torch.int64, device=dev)
        emb.emb_version_record_write(ver_record, tabs.set, 1)
        emb.emb_version_publish(ver_handle, ver_record)

    def do_forward(db, rows):
        if offsets_inside:
            emb.emb_bag_forward_train_lengths_after(tabs.set, db.raw, db.lengths, w.B, w.pool, buf.out, buf.offsets,
                                                    buf.workspace, buf.side if defer_join else None, None,
                                                    buf.num_unique, buf.status)
            return None
        if train_route:
            emb.emb_bag_forward_train(tabs.set, db.raw, buf.offsets, w.B, w.pool, buf.out, buf.workspace, None,
                                      buf.num_unique, buf.status)
            return None
        if versioned:
            # the lookup latches the current version record and reads only the latched copy: (E, V)
            emb.emb_version_latch(ver_handle, w.T, ver_latch, buf.status)
            emb.emb_bag_forward_latched_hashed(ver_latch, w.T, w.D, w.dtype, db.raw, buf.offsets, w.B, w.pool, buf.out,
                                               buf.status, streaming=w.streaming)
            return None
        if lengths_route:
            emb.emb_bag_forward_hashed_lengths(tabs.set, db.raw, db.lengths, w.B, w.pool, buf.out, buf.offsets,
                                               off_scratch, None, buf.status, streaming=w.streaming)
            return None
        if fused:
            rows = buf.rows[:db.nnz]
            emb.emb_bag_forward_hashed(tabs.set, db.raw, buf.offsets, w.B, w.pool, buf.out,
                                       rows if w.backward else None, buf.status, streaming=w.streaming)
            return rows
        pipeline.run_forward(w, tabs.set, rows, buf)
        return rows

    def index_and_forward(db):
        return do_forward(db, do_index(db))

    def do_backward(db, rows, sev):
        if train_route:
            emb.emb_bag_backward_sort_prepared(tabs.set, w.B, db.nnz, buf.workspace, buf.unique_keys,
                                               buf.unique_counts, buf.num_unique, buf.status, sev)
            emb.emb_bag_backward_update(tabs.set, w.B, db.nnz, db.dout, w.lr, w.eps, buf.workspace, buf.num_unique,
                                        sev, buf.side)
        else:
            pipeline.run_backward(w, tabs.set, rows, db, buf, stage_events=sev)

    # ---- timed region: exactly K steps --------------------------------------
    # Inside the timed region only the kernel with the largest share of the step is bracketed by two
    # events (the short-run update kernel of the backward, recorded by the library itself on the
    # launch stream; the forward kernel when the workload has no backward), and only on every
    # EVENT_EVERY-th step: an event pair costs the stream about 10 us (2 % of a 0.45 ms step).  The
    # full per-stage breakdown comes from a second, instrumented pass outside the timed region.
    EVENT_EVERY = args.event_every
    NS = emb.BWD_STAGE_EVENTS

    def new_events(n):
        # HIP events that release to device scope: a record does not write caches back to system
        # memory (a default event's record costs the stream several microseconds)
        return [emb.Event(timing=True) for _ in range(n)]

    dom = [new_events(2) for _ in range((K + EVENT_EVERY - 1) // EVENT_EVERY)]

    def next_buffers():
        nonlocal buf
        buf = pair[steps_run[0] % len(pair)]
        steps_run[0] += 1

    def timed_step(db, ev_k):
        next_buffers()
        if w.backward:
            sev = [None, None, None, ev_k[0], ev_k[1], None] if ev_k else None
            if args.overlap_sort:
                pipeline.run_step_overlapped(w, tabs.set, db, buf, stage_events=sev)
            else:
                rows = index_and_forward(db)
                do_backward(db, rows, sev)
        else:
            rows = do_index(db)
            if ev_k:
                ev_k[0].record()
            do_forward(db, rows)
            if ev_k:
                ev_k[1].record()

    # W untimed warm-up steps, the same code as the timed ones; the first of them carries the event
    # bracket, so the first use of that path (38 ms in the first GPU process on a machine: code pages
    # of the runtime read from disk) is not timed.  Nothing but the synchronisation stands between
    # them and the timed steps (the events were created above).
    for i in range(W):
        timed_step(dbs[i % len(dbs)], dom[0] if i == 0 else None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        timed_step(dbs[(W + k) % len(dbs)], dom[k // EVENT_EVERY] if k % EVENT_EVERY == 0 else None)
    if defer_join:
        buf.side.join()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    assert int(buf.status.item()) == 0, "device status word set during the timed steps"
    dom_ms = sorted(e[0].elapsed_time(e[1]) for e in dom)
    ms_dom = sum(dom_ms) / len(dom_ms)

    # ---- instrumented pass (not part of `value`): every stage bracketed ------
    KI = min(K, 20)
    ev = [new_events(3) for _ in range(KI)]
    bev = [new_events(NS) for _ in range(KI)]
    torch.cuda.synchronize()
    for k in range(KI):
        db = dbs[(W + k) % len(dbs)]
        next_buffers()
        ev[k][0].record()
        rows = do_index(db)
        ev[k][1].record()
        rows = do_forward(db, rows)
        ev[k][2].record()
        if w.backward:
            do_backward(db, rows, bev[k])
    if defer_join:
        buf.side.join()
    torch.cuda.synchronize()

    lookups = sum(dbs[(W + k) % len(dbs)].nnz for k in range(K))
    nnz_avg = lookups / K
    nnz_i = int(nnz_avg)
    bags = w.T * w.B
    def median(xs):
        # the instrumented pass reports medians: one stalled iteration (a page fault, a clock ramp) must not
        # decide which kernel counts as the dominant one
        xs = sorted(xs)
        return xs[len(xs) // 2]

    ms_index = median(e[0].elapsed_time(e[1]) for e in ev)
    ms_fwd = median(e[1].elapsed_time(e[2]) for e in ev)
    uniq = int(buf.num_unique.item()) if w.backward else 0   # of the last batch; all batches are alike
    passes = (max(1, int(w.R).bit_length()) + 7) // 8     # the sort works table by table on row numbers
    rowb = emb.emb_row_bytes(w.D, w.storage)

    def entry(name, ms, nbytes, what, pmc_kernel=None, cache_fed=False):
        gbs = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        traffic = measured_traffic(args.workload, pmc_kernel) if pmc_kernel and not args.scale_rows else None
        e = {"kernel": name, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
             "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_source(traffic),
             "avg_ms": round(ms, 4), "algorithmic_bytes": int(nbytes), "bytes_are": what}
        if traffic is not None and ms > 0:
            e["measured_traffic_GBps"] = round(traffic / (ms * 1e-3) / 1e9, 1)
            e["frac_measured_traffic"] = round(traffic / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        if cache_fed:
            # popular rows repeat within a batch and are served from L2 / the memory-side cache: the
            # algorithmic bytes are not HBM bytes and `frac` is not a fraction of an HBM roofline
            e["cache_fed"] = True
            e["frac_is"] = ("algorithmic GB/s over the HBM peak; rows that repeat come from cache, so this can "
                            "exceed 1; frac_measured_traffic (when present) is the HBM-side figure")
        return e

    if fused:
        fwd_name, fwd_pmc = "bag_forward_hashed_kernel (hash + gather-pool)", "bag_forward_hashed_kernel"
        if w.quant:
            fwd_name = "bag_forward_quant_kernel (hash + gather-dequantise-pool, %s rows of %d B)" % (w.quant, rowb)
            fwd_pmc = "bag_forward_quant_kernel"
        fwd_extra = 0
        if train_route:
            fwd_name = "bwd_init + bag_forward_train_kernel (hash + gather-pool + the backward's records)"
            fwd_pmc = "bag_forward_train_kernel"
            fwd_extra = nnz_i * 8 + bags * 4          # one 8-byte record per lookup, one scale per bag
        index_entry = entry("offsets_* (index stage, 3 launches; hashing is done inside the forward)", ms_index,
                            bags * 12, "12 B per bag (length in, offset out)")
        if lengths_route:
            fwd_name = "offsets_tile_scan + " + fwd_name.replace("(hash", "(bag offsets + hash")
            fwd_extra += bags * 28                   # length in, sum within the tile out and in, offset out
            index_entry = entry("(index stage: the bag offsets are made inside the lookup)", ms_index, 1,
                                "not priced: counted under the lookup")
        if offsets_inside:
            fwd_name = ("offsets_tile_scan + bwd_init + bag_forward_train_kernel (bag offsets + hash + gather-pool + "
                        "the backward's records)")
            fwd_extra += bags * 28                   # length in, sum within the tile out and in, offset out
            index_entry = entry("(index stage: the bag offsets are made inside the training lookup)", ms_index, 1,
                                "not priced: counted under the lookup")
    else:
        fwd_name = ("bag_forward_quant_kernel (gather-dequantise-pool, %s rows of %d B)" % (w.quant, rowb) if w.quant
                    else "bag_forward_kernel (gather-pool)")
        fwd_pmc = "bag_forward_quant_kernel" if w.quant else "bag_forward_kernel"
        fwd_extra = 0
        index_entry = entry("offsets_* + hash_ids_tables_kernel (index stage, 4 launches)", ms_index,
                            nnz_i * 16 + bags * 12,
                            "16 B per lookup (raw ID in, row out) + 12 B per bag (length in, offset out)")
    kernels = [
        index_entry,
        entry(fwd_name, ms_fwd if w.backward else ms_dom, forward_bytes(nnz_i, bags, w.D, rowb) + fwd_extra,
              "row + 8 B index per lookup (+ 8 B record out when a backward follows), fp32 output row + 8 B "
              "offset per bag", fwd_pmc, cache_fed=(w.ids == "zipf")),
    ]
    ms_bwd = 0.0
    if w.backward:
        st = [median(r[i].elapsed_time(r[i + 1]) for r in bev) for i in range(NS - 1)]
        st[3] = ms_dom      # the dominant kernel's time is the one measured inside the timed region
        ms_bwd = median(r[0].elapsed_time(r[NS - 1]) for r in bev)
        kernels += [
            entry("bwd_init + bwd_keys_kernel (key build)" if not train_route
                  else "(key build: done by the training lookup)", st[0], (nnz_i * 16 + bags * 20) if not train_route else 1,
                  "8 B row in + 8 B record out per lookup; 16 B offsets in + 4 B scale out per bag"),
            entry("sort_hist/scan/scatter x %d passes (radix sort)" % passes, st[1], nnz_i * 16 * passes,
                  "8 B record read + 8 B written per lookup and pass"),
            entry("update_kernel (segment reduce + row-wise Adagrad, short runs)", st[3] if st[3] > 0 else 1e-9,
                  uniq * (2 * rowb + 8) + nnz_i * 8 + bags * 4 * w.D,
                  "row read + row written + 8 B accumulator per distinct row, 8 B record per lookup, "
                  "gradient row once per bag (all distinct rows counted here; the few queued ones are "
                  "updated by the next stage)", "update_kernel"),
            entry("long_prepare/reduce/combine (queued long runs)", st[4], 1,
                  "not priced: its rows are counted under update_kernel"),
        ]
    # the roofline object is for the kernel with the largest share of the step
    roofline = max(kernels, key=lambda e: e["avg_ms"])
    stages = {"index_ms": round(ms_index, 4), "forward_ms": round(ms_fwd, 4), "backward_ms": round(ms_bwd, 4)}
    step_bytes = sum(e["algorithmic_bytes"] for e in kernels)
    if w.backward:
        stages.update({"bwd_keys_ms": round(st[0], 4), "bwd_sort_ms": round(st[1], 4),
                       "bwd_unique_list_ms": round(st[2], 4), "bwd_update_ms": round(st[3], 4),
                       "bwd_long_runs_ms": round(st[4], 4), "unique_rows_last_batch": uniq,
                       "backward_algorithmic_bytes": backward_bytes(nnz_i, bags, uniq, w.D, w.esz, passes)})
        stages["side_stream_join"] = ("in the next step's lookup call, after its set-up launches (two workspaces "
                                      "alternate; bwd_long_runs_ms no longer contains the wait)" if defer_join
                                      else ("at the end of the backward" if buf.side is not None else "no side stream"))
    log("step %.3f ms: index %.3f, forward %.3f, backward %.3f %s" % (
        elapsed / K * 1e3, ms_index, ms_fwd, ms_bwd,
        ("(keys %.3f, sort %.3f, update %.3f, long runs %.3f)" % (st[0], st[1], st[3], st[4])) if w.backward else ""))
    # what a plain streaming read gets on this part: the checksum kernel over one table (not part of `value`)
    stream_gbs = stream_read_rate(tabs.weights[0])
    roofline = dict(roofline, stream_read_GBps=round(stream_gbs, 1),
                    frac_of_stream_read=round(roofline["achieved"] / stream_gbs, 4))
    if w.backward:
        # the update kernel writes as much as it reads: a plain copy is the nearer yardstick
        copy_gbs = stream_copy_rate()
        roofline["stream_copy_GBps"] = round(copy_gbs, 1)
        if roofline.get("measured_traffic_GBps"):
            roofline["measured_traffic_frac_of_stream_copy"] = round(roofline["measured_traffic_GBps"] / copy_gbs, 4)
        log("a plain device copy moves %.0f GB/s (read + written)" % copy_gbs)
    if abs(roofline["avg_ms"] - round(ms_dom, 4)) < 1e-9:
        # the kernel bracketed by events inside the timed region: its spread over the K steps
        roofline.update(median_ms=round(dom_ms[len(dom_ms) // 2], 4), min_ms=round(dom_ms[0], 4),
                        max_ms=round(dom_ms[-1], 4), launches_timed=len(dom_ms),
                        timed_how="HIP events around this kernel on every %d-th of the %d timed steps" % (EVENT_EVERY, K))
    log("dominant: %s: %.3f ms, %.0f GB/s algorithmic = %.1f %% of HBM peak (a streaming read of one table gets "
        "%.0f GB/s)" % (roofline["kernel"], roofline["avg_ms"], roofline["achieved"], 100 * roofline["frac"],
                        stream_gbs))

    # ---- side measurements: the forward kernel alone on workloads 2 and 2u, and over INT4 copies
    # of the same tables (2q4, 2uq4; 2uq4r: the INT4 rows padded to 64 bytes)
    extra = {}
    if not args.no_extra and w.backward and not args.overlap_sort:
        # the step when the trainer also wants the ordered list of distinct rows and their counts (optional
        # outputs of the sort, not written in the timed steps)
        for b_ in pair:
            b_.unique_keys = torch.empty(max(max_nnz, 1), dtype=torch.int64, device=dev)
            b_.unique_counts = torch.empty(max(max_nnz, 1), dtype=torch.int32, device=dev)
        KU = min(K, 50)
        for i in range(3):
            timed_step(dbs[i % len(dbs)], None)
        torch.cuda.synchronize()
        tu = time.perf_counter()
        for k in range(KU):
            timed_step(dbs[(W + k) % len(dbs)], None)
        if defer_join:
            buf.side.join()
        torch.cuda.synchronize()
        ms_u = (time.perf_counter() - tu) / KU * 1e3
        assert int(buf.status.item()) == 0
        for b_ in pair:
            b_.unique_keys = b_.unique_counts = None
        extra["step_with_distinct_row_list"] = {"ms_per_step": round(ms_u, 4), "steps": KU,
                                                "adds_ms": round(ms_u - elapsed / K * 1e3, 4)}
        log("with the list of distinct rows written: step %.3f ms (+%.3f)" % (ms_u, ms_u - elapsed / K * 1e3))
    if not args.no_extra and args.workload == "3" and not args.scale_rows:
        qsets = {}
        for name in ("2", "2un", "2u", "2q4", "2uq4", "2uq4r"):
            wf = wl.WORKLOADS[name]
            tset = tabs.set
            if wf.quant:
                if wf.quant not in qsets:
                    qsets[wf.quant] = pipeline.quantized_tableset(tabs, wf.quant)
                tset = qsets[wf.quant][1]
            fb = [pipeline.DeviceBatch(wf, wl.make_batch(wf, i, seed), dev) for i in range(args.batches)]
            fbuf = pipeline.StepBuffers(wf, max(d.nnz for d in fb), tabs.set.total_rows, dev)
            rows_v = []
            for d in fb:                      # index stage once per batch, rows kept resident
                r = pipeline.run_index_stage(wf, tset, d, fbuf).clone()
                rows_v.append((r, fbuf.offsets.clone()))
            torch.cuda.synchronize()
            for i in range(3):
                fbuf.offsets.copy_(rows_v[i % len(fb)][1])
                pipeline.run_forward(wf, tset, rows_v[i % len(fb)][0], fbuf)
            torch.cuda.synchronize()
            n_it = 40
            e0 = [emb.Event(timing=True) for _ in range(n_it)]
            e1 = [emb.Event(timing=True) for _ in range(n_it)]
            tot = 0
            for i in range(n_it):
                r, o = rows_v[i % len(fb)]
                fbuf.offsets.copy_(o)
                e0[i].record()
                pipeline.run_forward(wf, tset, r, fbuf)
                e1[i].record()
                tot += r.numel()
            torch.cuda.synchronize()
            ms = sum(a.elapsed_time(b) for a, b in zip(e0, e1)) / n_it
            nb = forward_bytes(tot // n_it, wf.T * wf.B, wf.D, emb.emb_row_bytes(wf.D, wf.storage))
            gbs = nb / (ms * 1e-3) / 1e9
            kern = "bag_forward_quant_kernel" if wf.quant else "bag_forward_kernel"
            tr = measured_traffic(name, kern)
            ex = {"kernel": kern, "row_bytes": emb.emb_row_bytes(wf.D, wf.storage),
                  "avg_ms": round(ms, 4), "lookups_per_s": round(tot / n_it / (ms * 1e-3), 1),
                  "algorithmic_GBps": round(gbs, 1), "algorithmic_bytes": int(nb), "traffic": tr,
                  "traffic_source": traffic_source(tr)}
            if tr is not None:
                ex["measured_traffic_GBps"] = round(tr / (ms * 1e-3) / 1e9, 1)
                ex["frac_of_hbm_peak_measured_traffic"] = round(tr / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
            if wf.ids == "zipf":
                # rows repeat and come from cache: algorithmic GB/s is not an HBM rate, no roofline fraction from it
                ex["cache_fed"] = True
                log("forward only, workload %s: %.3f ms, %.3g lookups/s, %.0f GB/s algorithmic (cache-fed: popular rows "
                    "repeat)%s" % (name, ms, tot / n_it / (ms * 1e-3), gbs,
                                   "" if tr is None else "; %.0f GB/s of measured HBM traffic = %.1f %% of peak" % (
                                       ex["measured_traffic_GBps"], 100 * ex["frac_of_hbm_peak_measured_traffic"])))
            else:
                ex["frac_of_hbm_peak"] = round(gbs / HBM_PEAK_GBS, 4)
                log("forward only, workload %s: %.3f ms, %.3g lookups/s, %.0f GB/s (%.1f %% of HBM peak)" % (
                    name, ms, tot / n_it / (ms * 1e-3), gbs, 100 * gbs / HBM_PEAK_GBS))
            extra["forward_only_" + name] = ex
            del fb, fbuf, rows_v
        del qsets

    # ---- CPU baseline: the oracle, as it stands, on this host ----------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, batches_np, seed)

    value = lookups / elapsed
    out = {
        "metric": METRIC,
        "value": round(value, 1),
        "unit": "lookups/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(elapsed / K * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": ("%s: %d tables x %d rows x dim %d %s, %d bags/table, %s bag lengths (mean %g), %s IDs%s, "
                         "%s pooling, %s" % (
                             w.name, w.T, w.R, w.D,
                             w.dtype if not w.quant else "(fp32 quantised row-wise to %s, %d B per row)" % (w.quant, rowb),
                             w.B, w.length, w.mean_len, w.ids,
                             (" alpha=%g over %.0e keys" % (w.alpha, w.n_keys)) if w.ids == "zipf" else "", w.pool,
                             ("forward + sparse row-wise Adagrad backward" if w.backward else "forward only") +
                             (", rows read with the streaming hint" if w.streaming else "") +
                             (", through a version handle (latch + lookup)" if versioned else ""))),
            "lookups_per_step": round(nnz_avg, 1),
            "resident_batches": len(dbs),
            "seed": seed,
        },
        "achieved_GBps_whole_step": round(step_bytes / (elapsed / K) / 1e9, 1),
        "stages": stages,
        "roofline": roofline,
        "kernels": kernels,
        "cpu_baseline": cpu,
        "kernel_sources_digest": kernel_sources_digest(),   # of csrc/* as they are on disk (the library is rebuilt when stale)
    }
    if extra:
        out["extra"] = extra
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

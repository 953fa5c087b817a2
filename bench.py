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


def forward_bytes(nnz: int, bags: int, D: int, esz: int) -> int:
    """Algorithmic bytes of one gather-pool launch: per lookup one table row and
    one 8-byte index; per bag one fp32 output row and one 8-byte offset."""
    return nnz * (D * esz + 8) + bags * (4 * D + 8) + 8


def backward_bytes(nnz: int, bags: int, uniq: int, D: int, esz: int, passes: int) -> int:
    """Algorithmic bytes of one backward: per lookup its index (8) and 16 bytes
    (key+payload read and written) per radix pass; per bag its gradient row once;
    per distinct row one read and one write of the row plus its accumulator."""
    return nnz * (8 + 16 * passes) + bags * 4 * D + uniq * (2 * D * esz + 8)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="3", help="3 (fwd+bwd, default), 2 or 2u (forward only), 4")
    ap.add_argument("--batches", type=int, default=8, help="distinct resident batches cycled through")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--scale-rows", type=int, default=None, help="rows per table (debug: smaller tables)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the forward-only side measurements")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")
        return 2

    import numpy as np
    import torch

    from paper_2508_05700_amd import binding as emb
    from paper_2508_05700_amd import pipeline, workloads as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 2
    emb.lib()
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
    buf = pipeline.StepBuffers(w, max_nnz, tabs.set.total_rows, dev)
    torch.cuda.synchronize()
    log("setup: %d tables x %d rows x %d %s, %d batches of ~%d lookups, %.1f s" % (
        w.T, w.R, w.D, w.dtype, len(dbs), max_nnz, time.time() - t_setup))

    K, W = args.steps, args.warmup
    for i in range(W):
        pipeline.run_step(w, tabs.set, dbs[i % len(dbs)], buf)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps --------------------------------------
    # events on the launch stream: around the index stage and the forward kernel, and (recorded by
    # the library itself) between the stages of the backward
    NS = emb.BWD_STAGE_EVENTS
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    bev = [[torch.cuda.Event(enable_timing=True) for _ in range(NS)] for _ in range(K)]
    for row in bev:
        for e in row:
            e.record()          # creates the HIP event behind the torch object
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        db = dbs[(W + k) % len(dbs)]
        ev[k][0].record()
        rows = pipeline.run_index_stage(w, tabs.set, db, buf)
        ev[k][1].record()
        pipeline.run_forward(w, tabs.set, rows, buf)
        ev[k][2].record()
        if w.backward:
            pipeline.run_backward(w, tabs.set, rows, db, buf, stage_events=bev[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    assert int(buf.status.item()) == 0, "device status word set during the timed steps"

    lookups = sum(dbs[(W + k) % len(dbs)].nnz for k in range(K))
    nnz_avg = lookups / K
    nnz_i = int(nnz_avg)
    bags = w.T * w.B
    ms_index = sum(e[0].elapsed_time(e[1]) for e in ev) / K
    ms_fwd = sum(e[1].elapsed_time(e[2]) for e in ev) / K
    uniq = int(buf.num_unique.item()) if w.backward else 0   # of the last batch; all batches are alike
    passes = (max(1, int(tabs.set.total_rows).bit_length()) + 7) // 8
    rowb = w.D * w.esz

    def entry(name, ms, nbytes, what):
        gbs = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        return {"kernel": name, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "avg_ms": round(ms, 4),
                "algorithmic_bytes": int(nbytes), "bytes_are": what}

    kernels = [
        entry("offsets_* + hash_ids_tables_kernel (index stage, 4 launches)", ms_index, nnz_i * 16 + bags * 12,
              "16 B per lookup (raw ID in, row out) + 12 B per bag (length in, offset out)"),
        entry("bag_forward_kernel (gather-pool)", ms_fwd, forward_bytes(nnz_i, bags, w.D, w.esz),
              "row + 8 B index per lookup, fp32 output row + 8 B offset per bag"),
    ]
    ms_bwd = 0.0
    if w.backward:
        st = [sum(r[i].elapsed_time(r[i + 1]) for r in bev) / K for i in range(NS - 1)]
        ms_bwd = sum(bev[k][0].elapsed_time(bev[k][NS - 1]) for k in range(K)) / K
        kernels += [
            entry("bwd_init + bwd_keys_kernel (key build)", st[0], nnz_i * 16 + bags * 20,
                  "8 B row in + 8 B record out per lookup; 16 B offsets in + 4 B scale out per bag"),
            entry("sort_hist/scan/scatter x %d passes (radix sort)" % passes, st[1], nnz_i * 16 * passes,
                  "8 B record read + 8 B written per lookup and pass"),
            entry("update_kernel (segment reduce + row-wise Adagrad, short runs)", st[3] if st[3] > 0 else 1e-9,
                  uniq * (2 * rowb + 8) + nnz_i * 8 + bags * 4 * w.D,
                  "row read + row written + 8 B accumulator per distinct row, 8 B record per lookup, "
                  "gradient row once per bag (all distinct rows counted here; the few queued ones are "
                  "updated by the next stage)"),
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
    log("step %.3f ms: index %.3f, forward %.3f, backward %.3f %s" % (
        elapsed / K * 1e3, ms_index, ms_fwd, ms_bwd,
        ("(keys %.3f, sort %.3f, update %.3f, long runs %.3f)" % (st[0], st[1], st[3], st[4])) if w.backward else ""))
    log("dominant: %s: %.3f ms, %.0f GB/s algorithmic = %.1f %% of HBM peak" % (
        roofline["kernel"], roofline["avg_ms"], roofline["achieved"], 100 * roofline["frac"]))

    # ---- side measurements: the forward kernel alone on workloads 2 and 2u ---
    extra = {}
    if not args.no_extra and args.workload == "3" and not args.scale_rows:
        for name in ("2", "2u"):
            wf = wl.WORKLOADS[name]
            fb = [pipeline.DeviceBatch(wf, wl.make_batch(wf, i, seed), dev) for i in range(args.batches)]
            fbuf = pipeline.StepBuffers(wf, max(d.nnz for d in fb), tabs.set.total_rows, dev)
            rows_v = []
            for d in fb:                      # index stage once per batch, rows kept resident
                r = pipeline.run_index_stage(wf, tabs.set, d, fbuf).clone()
                rows_v.append((r, fbuf.offsets.clone()))
            torch.cuda.synchronize()
            for i in range(3):
                fbuf.offsets.copy_(rows_v[i % len(fb)][1])
                pipeline.run_forward(wf, tabs.set, rows_v[i % len(fb)][0], fbuf)
            torch.cuda.synchronize()
            n_it = 40
            e0 = [torch.cuda.Event(enable_timing=True) for _ in range(n_it)]
            e1 = [torch.cuda.Event(enable_timing=True) for _ in range(n_it)]
            tot = 0
            for i in range(n_it):
                r, o = rows_v[i % len(fb)]
                fbuf.offsets.copy_(o)
                e0[i].record()
                pipeline.run_forward(wf, tabs.set, r, fbuf)
                e1[i].record()
                tot += r.numel()
            torch.cuda.synchronize()
            ms = sum(a.elapsed_time(b) for a, b in zip(e0, e1)) / n_it
            nb = forward_bytes(tot // n_it, wf.T * wf.B, wf.D, wf.esz)
            gbs = nb / (ms * 1e-3) / 1e9
            extra["forward_only_" + name] = {
                "avg_ms": round(ms, 4), "lookups_per_s": round(tot / n_it / (ms * 1e-3), 1),
                "algorithmic_GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
            log("forward only, workload %s: %.3f ms, %.0f GB/s (%.1f %% of HBM peak)" % (
                name, ms, gbs, 100 * gbs / HBM_PEAK_GBS))
            del fb, fbuf, rows_v

    # ---- CPU baseline: the oracle, as it stands, on this host ----------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import emb_oracle as oracle
        b = batches_np[0]
        t_cpu = time.perf_counter()
        off, _ = oracle.lengths_to_offsets(b["lengths"])
        if b["raw"] is not None:
            rows_np = np.concatenate([oracle.hash_ids(b["raw"][off[t * w.B]:off[(t + 1) * w.B]], w.salt(t), w.R)
                                      for t in range(w.T)])
        else:
            rows_np = b["rows"]
        t_hash = time.perf_counter() - t_cpu
        # host tables: full-size virtual arrays in which only the rows this batch touches are
        # materialised (untimed); the oracle's gathers then hit the same scattered addresses
        tables = [wl.sparse_host_table(w.table_seed(t, seed), w.R, w.D, w.dtype,
                                       rows_np[off[t * w.B]:off[(t + 1) * w.B]]) for t in range(w.T)]
        t_cpu = time.perf_counter()
        oracle.bag_forward(tables, w.dtype, rows_np, off, w.B, w.pool, want_absum=False)
        t_f = time.perf_counter() - t_cpu
        t_b = 0.0
        if w.backward:
            acc = [np.zeros(w.R, dtype=np.float32) for _ in range(w.T)]
            t_cpu = time.perf_counter()
            oracle.bag_backward_rowwise_adagrad(tables, acc, w.dtype, rows_np, off, w.B, w.pool, b["dout"], w.lr,
                                                w.eps, want_G=False)
            t_b = time.perf_counter() - t_cpu
        t_all = t_hash + t_f + t_b
        cpu = {"value": round(int(b["nnz"]) / t_all, 1), "unit": "lookups/s", "cores": 1, "kind": "oracle",
               "sample": "one full batch of the same workload (%d lookups, all %d tables): offsets+hash %.2f s, "
                         "forward %.2f s, backward %.2f s; single thread; host tables hold only the touched rows"
                         % (int(b["nnz"]), w.T, t_hash, t_f, t_b)}
        log("cpu oracle: %.2f s per step -> %.3g lookups/s on 1 core" % (t_all, cpu["value"]))

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
                             w.name, w.T, w.R, w.D, w.dtype, w.B, w.length, w.mean_len, w.ids,
                             (" alpha=%g over %.0e keys" % (w.alpha, w.n_keys)) if w.ids == "zipf" else "", w.pool,
                             "forward + sparse row-wise Adagrad backward" if w.backward else "forward only")),
            "lookups_per_step": round(nnz_avg, 1),
            "resident_batches": len(dbs),
            "seed": seed,
        },
        "achieved_GBps_whole_step": round(step_bytes / (elapsed / K) / 1e9, 1),
        "stages": stages,
        "roofline": roofline,
        "kernels": kernels,
        "cpu_baseline": cpu,
    }
    if extra:
        out["extra"] = extra
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

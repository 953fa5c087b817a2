"""GPU parity at the full sizes of the five workloads, in the launch configuration the
benchmark times.  Tables are 13 MB - 64 GB and are filled procedurally on the device;
the oracle gets full-size host arrays in which only the rows a batch touches are
materialised (from the numpy generator), so it sees the very same row numbers.
Outputs are small (<= 34 MB) and are compared in full."""
import sys
import time

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import emb_oracle as oracle  # noqa: E402
from paper_2508_05700_amd import binding as emb  # noqa: E402
from paper_2508_05700_amd import pipeline, workloads as wl  # noqa: E402
from tests import harness as H  # noqa: E402


def say(*a):
    print("[%s]" % time.strftime("%H:%M:%S"), *a, file=sys.stderr, flush=True)


def _oracle_index(w, batch):
    off, st = oracle.lengths_to_offsets(batch["lengths"])
    assert st == 0
    if batch["raw"] is None:
        return off, batch["rows"]
    rows = np.concatenate([oracle.hash_ids(batch["raw"][off[t * w.B]:off[(t + 1) * w.B]], w.salt(t), w.R)
                           for t in range(w.T)])
    return off, rows


def _host_tables(w, rows, off):
    return [wl.sparse_host_table(w.table_seed(t), w.R, w.D, w.dtype, rows[off[t * w.B]:off[(t + 1) * w.B]])
            for t in range(w.T)]


def _check_fill_sample(w, tabs, rng, n=20_000):
    """The device tables hold exactly the generator's values (sampled rows)."""
    for t in (0, w.T - 1):
        r = np.sort(rng.integers(0, w.R, size=n))
        got = H.host_table(tabs.weights[t][torch.from_numpy(r).to(H.DEV)])
        assert np.array_equal(got, wl.table_rows(w.table_seed(t), r, w.D, w.dtype))


def _forward_parity(w, tabs, batch_index=0):
    batch = wl.make_batch(w, batch_index)
    dev = tabs.device
    db = pipeline.DeviceBatch(w, batch, dev)
    buf = pipeline.StepBuffers(w, db.nnz, tabs.set.total_rows, dev, want_unique=True)
    say("workload %s: %d lookups, index + forward on the device" % (w.name, db.nnz))
    rows_dev = pipeline.run_index_stage(w, tabs.set, db, buf)
    pipeline.run_forward(w, tabs.set, rows_dev, buf)
    torch.cuda.synchronize()
    assert int(buf.status.item()) == 0
    off, rows = _oracle_index(w, batch)
    assert np.array_equal(buf.offsets.cpu().numpy(), off)              # bit-exact offsets
    assert np.array_equal(rows_dev.cpu().numpy(), rows)                # bit-exact hashed rows
    say("workload %s: oracle forward" % w.name)
    tables = _host_tables(w, rows, off)
    ref, absum, st = oracle.bag_forward(tables, w.dtype, rows, off, w.B, w.pool)
    assert st == 0
    H.assert_pooled_close(buf.out.cpu().numpy(), ref, absum, what="workload " + w.name)
    if db.raw is not None:
        # the route the benchmark times: hashing inside the lookup; same bits, same row numbers
        two_step = buf.out.clone()
        rows_two_step = rows_dev.clone()
        buf.rows.fill_(-1)
        fused_rows = pipeline.run_index_and_forward_fused(w, tabs.set, db, buf)
        torch.cuda.synchronize()
        assert int(buf.status.item()) == 0 and torch.equal(buf.out, two_step)
        if w.backward:
            assert torch.equal(fused_rows, rows_two_step)
        else:
            buf.rows[:db.nnz].copy_(rows_two_step)
        rows_dev = buf.rows[:db.nnz]
        if True:
            # and through a version handle (latch + lookup over the latched descriptors): same bits, version returned
            record = torch.empty(emb.emb_version_record_bytes(w.T), dtype=torch.uint8, device=dev)
            latch = torch.empty(emb.emb_version_latch_bytes(w.T), dtype=torch.uint8, device=dev)
            handle = torch.zeros(1, dtype=torch.int64, device=dev)
            emb.emb_version_record_write(record, tabs.set, 7)
            emb.emb_version_publish(handle, record)
            buf.out.fill_(float("nan"))
            emb.emb_version_latch(handle, w.T, latch, buf.status)
            emb.emb_bag_forward_latched_hashed(latch, w.T, w.D, w.storage, db.raw, buf.offsets, w.B, w.pool, buf.out,
                                               buf.status, streaming=w.streaming)
            torch.cuda.synchronize()
            assert int(buf.status.item()) == 0 and int(emb.latched_version(latch).item()) == 7
            assert torch.equal(buf.out, two_step)
    return batch, db, buf, rows_dev, off, rows, tables


def test_workload_1_small_single_table():
    w = wl.WORKLOADS["1"]
    tabs = pipeline.DeviceTables(w)
    _check_fill_sample(w, tabs, np.random.default_rng(1))
    _forward_parity(w, tabs)


@pytest.fixture(scope="module")
def tables16():
    w = wl.WORKLOADS["3"]
    say("filling 16 tables x 1e7 x 64 fp32 (41 GB) on the device")
    tabs = pipeline.DeviceTables(w)
    torch.cuda.synchronize()
    _check_fill_sample(w, tabs, np.random.default_rng(2))
    yield tabs
    del tabs
    torch.cuda.empty_cache()


def test_workload_2_zipf_forward(tables16):
    _forward_parity(wl.WORKLOADS["2"], tables16)


def test_workload_2u_uniform_forward(tables16):
    w = wl.WORKLOADS["2u"]
    batch, *_ = _forward_parity(w, tables16)
    # uniform IDs: practically no row is looked up twice
    assert np.unique(batch["raw"]).size > 0.999 * batch["raw"].size


@pytest.mark.parametrize("name", ["2q4", "2q8"])
def test_workload_2_over_quantized_tables(tables16, name):
    # Runs before the backward test below changes the tables.  The fp32 tables are quantised on the
    # device; the oracle quantises the generator's values of the rows the batch touches and pools
    # them (lookups renumbered into that compact table: plumbing, the values are the same).
    w = wl.WORKLOADS[name]
    tabs = tables16
    say("workload %s: quantising 16 tables on the device" % name)
    qkeep, qset = pipeline.quantized_tableset(tabs, w.quant)
    batch = wl.make_batch(w, 0)
    db = pipeline.DeviceBatch(w, batch, tabs.device)
    buf = pipeline.StepBuffers(w, db.nnz, tabs.set.total_rows, tabs.device)
    rows_dev = pipeline.run_index_stage(w, qset, db, buf)
    pipeline.run_forward(w, qset, rows_dev, buf)
    torch.cuda.synchronize()
    assert int(buf.status.item()) == 0
    off, rows = _oracle_index(w, batch)
    assert np.array_equal(rows_dev.cpu().numpy(), rows)
    say("workload %s: oracle quantiser and forward" % name)
    qt, parts = [], []
    for t in range(w.T):
        seg = rows[off[t * w.B]:off[(t + 1) * w.B]]
        touched = np.unique(seg)
        packed = oracle.quantize_rows(wl.table_values(w.table_seed(t), touched, w.D), w.quant)
        got = qkeep[t][torch.from_numpy(touched).to(H.DEV)].cpu().numpy()
        assert np.array_equal(got, packed), "quantised rows of table %d differ" % t       # bit-exact codes
        qt.append(packed)
        parts.append(np.searchsorted(touched, seg))
    ref, absum, st = oracle.bag_forward(qt, w.quant, np.concatenate(parts).astype(np.int64), off, w.B, w.pool, D=w.D)
    assert st == 0
    H.assert_pooled_close(buf.out.cpu().numpy(), ref, absum, what="workload " + name)
    del qkeep, qset
    torch.cuda.empty_cache()


def test_workload_3_forward_and_backward(tables16):
    w = wl.WORKLOADS["3"]
    tabs = tables16
    batch, db, buf, rows_dev, off, rows, tables = _forward_parity(w, tabs)
    say("workload 3: training lookup + backward on the device (the route the benchmark times)")
    pooled = buf.out.clone()
    buf.out.fill_(float("nan"))
    pipeline.run_train_step(w, tabs.set, db, buf)
    torch.cuda.synchronize()
    assert int(buf.status.item()) == 0
    assert torch.equal(buf.out, pooled)                       # the training lookup pools the same bits
    say("workload 3: oracle backward")
    old = [None] * w.T
    acc = [np.zeros(w.R, dtype=np.float32) for _ in range(w.T)]
    base = np.arange(w.T + 1, dtype=np.int64) * w.R
    touched = [np.unique(rows[off[t * w.B]:off[(t + 1) * w.B]]) for t in range(w.T)]
    for t in range(w.T):
        old[t] = tables[t][touched[t]].copy()
    r = oracle.bag_backward_rowwise_adagrad(tables, acc, w.dtype, rows, off, w.B, w.pool, batch["dout"], w.lr, w.eps)
    assert r["status"] == 0
    U = int(buf.num_unique.item())
    assert np.array_equal(buf.unique_keys[:U].cpu().numpy(), r["unique_keys"])       # bit-exact unique-row set
    assert np.array_equal(buf.unique_counts[:U].cpu().numpy(), r["unique_counts"])
    assert np.array_equal(r["unique_keys"], np.concatenate([base[t] + touched[t] for t in range(w.T)]))
    say("workload 3: %d distinct rows; comparing updated rows and accumulators" % U)
    rng = np.random.default_rng(3)
    for t in range(w.T):
        idx = torch.from_numpy(touched[t]).to(H.DEV)
        got = tabs.weights[t][idx].cpu().numpy()
        H.assert_rows_close(got, tables[t][touched[t]], old[t], w.lr, what="workload 3 rows t=%d" % t)
        sel = (r["unique_keys"] >= base[t]) & (r["unique_keys"] < base[t + 1])
        H.assert_accum_close(tabs.accum[t][idx].cpu().numpy(), acc[t][touched[t]], r["Gabs"][sel],
                             what="workload 3 accum t=%d" % t)
        # first Adagrad step from S = 0: every touched row moves by lr * sqrt(D) (closed form)
        step = np.sqrt(((got.astype(np.float64) - old[t]) ** 2).sum(1))
        nz = np.abs(r["G"][sel]).sum(1) > 0
        np.testing.assert_allclose(step[nz], w.lr * np.sqrt(w.D), rtol=2e-3)
        # rows outside the batch keep the generator's values bit for bit, accumulators stay zero
        probe = np.setdiff1d(rng.integers(0, w.R, size=100_000), touched[t])
        pidx = torch.from_numpy(probe).to(H.DEV)
        assert np.array_equal(tabs.weights[t][pidx].cpu().numpy(), wl.table_values(w.table_seed(t), probe, w.D))
        assert float(tabs.accum[t].sum().item()) == pytest.approx(float(acc[t].sum(dtype=np.float64)), rel=1e-4)
        assert int((tabs.accum[t] != 0).sum().item()) == int((acc[t] != 0).sum())


def test_workload_3_steps_with_the_deferred_join_as_the_benchmark_runs_them(tables16):
    # The benchmark's loop defers the wait for the backward's side stream into the next step's lookup call
    # and alternates between two workspaces.  At full size: a step on batch 1 followed by the lookup of
    # batch 2, once joining at the end of the backward (the route the test above checks against the
    # oracle) and once deferred, from the same table state: pooled outputs of both lookups and every row and
    # accumulator the two batches touch, bit for bit.
    w = wl.WORKLOADS["3"]
    tabs = tables16
    dev = tabs.device
    b1, b2 = wl.make_batch(w, 1), wl.make_batch(w, 2)
    d1, d2 = pipeline.DeviceBatch(w, b1, dev), pipeline.DeviceBatch(w, b2, dev)
    n = max(d1.nnz, d2.nnz)
    buf_a = pipeline.StepBuffers(w, n, tabs.set.total_rows, dev)
    buf_b = pipeline.StepBuffers(w, n, tabs.set.total_rows, dev, side_stream=False)
    side = buf_a.side
    (off1, rows1), (off2, rows2) = _oracle_index(w, b1), _oracle_index(w, b2)
    touched = [torch.from_numpy(np.unique(np.concatenate([rows1[off1[t * w.B]:off1[(t + 1) * w.B]],
                                                          rows2[off2[t * w.B]:off2[(t + 1) * w.B]]]))).to(dev)
               for t in range(w.T)]
    saved = [(tabs.weights[t][touched[t]].clone(), tabs.accum[t][touched[t]].clone()) for t in range(w.T)]

    def route(defer):
        side.defer_join = defer
        pipeline.run_train_step(w, tabs.set, d1, buf_a)
        # the next step's lookup alone (its backward would only repeat what the first step showed)
        emb.emb_bag_forward_train_lengths_after(tabs.set, d2.raw, d2.lengths, w.B, w.pool, buf_b.out, buf_b.offsets,
                                                buf_b.workspace, side if defer else None, None, buf_b.num_unique,
                                                buf_a.status)
        torch.cuda.synchronize()
        assert int(buf_a.status.item()) == 0
        state = [(tabs.weights[t][touched[t]].clone(), tabs.accum[t][touched[t]].clone()) for t in range(w.T)]
        outs = (buf_a.out.clone(), buf_b.out.clone(), buf_b.offsets.clone())
        for t in range(w.T):                      # back to the state both routes start from
            tabs.weights[t][touched[t]] = saved[t][0]
            tabs.accum[t][touched[t]] = saved[t][1]
        torch.cuda.synchronize()
        return outs, state

    say("workload 3: step + next lookup, join at the end of the backward")
    outs_a, state_a = route(False)
    say("workload 3: the same with the join deferred into the next lookup")
    outs_b, state_b = route(True)
    side.defer_join = False
    assert all(torch.equal(x, y) for x, y in zip(outs_a, outs_b))
    changed = 0
    for t in range(w.T):
        assert torch.equal(state_a[t][0], state_b[t][0]) and torch.equal(state_a[t][1], state_b[t][1]), t
        changed += int((state_a[t][0] != saved[t][0]).any(dim=1).sum().item())
    assert changed > 500_000                      # the step did change rows, and the second lookup read some of them
    del buf_a, buf_b, saved, state_a, state_b
    torch.cuda.empty_cache()


def test_workload_3b_bf16_tables_forward_and_backward():
    # Workload 3 with bf16 rows at full size, by the route the benchmark times.  Pooled values see no bf16
    # rounding (rows are widened exactly, sums are fp32): 1e-5.  Updated rows are written as bf16: 1e-2.
    w = wl.WORKLOADS["3b"]
    say("filling 16 tables x 1e7 x 64 bf16 (20 GB) on the device")
    tabs = pipeline.DeviceTables(w)
    torch.cuda.synchronize()
    _check_fill_sample(w, tabs, np.random.default_rng(12))
    batch, db, buf, rows_dev, off, rows, tables = _forward_parity(w, tabs)
    pooled = buf.out.clone()
    buf.out.fill_(float("nan"))
    pipeline.run_train_step(w, tabs.set, db, buf)
    torch.cuda.synchronize()
    assert int(buf.status.item()) == 0
    assert torch.equal(buf.out, pooled)
    say("workload 3b: oracle backward")
    acc = [np.zeros(w.R, dtype=np.float32) for _ in range(w.T)]
    base = np.arange(w.T + 1, dtype=np.int64) * w.R
    touched = [np.unique(rows[off[t * w.B]:off[(t + 1) * w.B]]) for t in range(w.T)]
    old = [H.as_f32(tables[t][touched[t]]) for t in range(w.T)]
    r = oracle.bag_backward_rowwise_adagrad(tables, acc, w.dtype, rows, off, w.B, w.pool, batch["dout"], w.lr, w.eps)
    assert r["status"] == 0
    U = int(buf.num_unique.item())
    assert np.array_equal(buf.unique_keys[:U].cpu().numpy(), r["unique_keys"])
    assert np.array_equal(buf.unique_counts[:U].cpu().numpy(), r["unique_counts"])
    rng = np.random.default_rng(13)
    for t in range(w.T):
        idx = torch.from_numpy(touched[t]).to(H.DEV)
        got = H.as_f32(H.host_table(tabs.weights[t][idx]))
        H.assert_rows_close(got, H.as_f32(tables[t][touched[t]]), old[t], w.lr, H.EPS_BF16, what="workload 3b rows t=%d" % t)
        sel = (r["unique_keys"] >= base[t]) & (r["unique_keys"] < base[t + 1])
        H.assert_accum_close(tabs.accum[t][idx].cpu().numpy(), acc[t][touched[t]], r["Gabs"][sel],
                             what="workload 3b accum t=%d" % t)
        probe = np.setdiff1d(rng.integers(0, w.R, size=100_000), touched[t])
        pidx = torch.from_numpy(probe).to(H.DEV)
        assert np.array_equal(H.host_table(tabs.weights[t][pidx]), wl.table_rows(w.table_seed(t), probe, w.D, w.dtype))
        assert int((tabs.accum[t] != 0).sum().item()) == int((acc[t] != 0).sum())
    del tabs
    torch.cuda.empty_cache()


def test_workload_4_one_billion_row_bf16_table():
    w = wl.WORKLOADS["4"]
    free, total = torch.cuda.mem_get_info()
    if free < 70 * 2 ** 30:
        pytest.skip("workload 4 at full size needs 70 GB of free HBM; %.0f GB free" % (free / 2 ** 30))
    assert w.R == 1_000_000_000 and w.D == 32
    say("filling 1e9 x 32 bf16 (64 GB) on the device")
    tabs = pipeline.DeviceTables(w)
    torch.cuda.synchronize()
    _check_fill_sample(w, tabs, np.random.default_rng(4))
    _forward_parity(w, tabs)
    del tabs
    torch.cuda.empty_cache()


def _full_size_or_skip(name, host_bytes):
    """The workload at exactly its stated size, or a skip that says why: these tests never run on a
    smaller table under the same name."""
    import psutil
    w = wl.WORKLOADS[name]
    avail = psutil.virtual_memory().available
    if avail < host_bytes:
        pytest.skip("workload %s at full size needs %.0f GB of free host memory to pin its table(s); %.0f GB available"
                    % (name, host_bytes / 2 ** 30, avail / 2 ** 30))
    say("workload %s at full size: %d table(s) x %d rows (%.0f GB of host memory available)"
        % (name, w.T, w.R, avail / 2 ** 30))
    return w


def _release_pinned_cache():
    """torch keeps freed pinned blocks (here: tens of GB) for reuse; hand them back to the system
    so that the next test can pin its own table."""
    import gc
    gc.collect()
    torch.cuda.synchronize()
    torch._C._host_emptyCache()


def _hybrid_parity(w, say_name):
    _release_pinned_cache()
    rng = np.random.default_rng(5)
    K = int(round(w.hot_fraction * w.R))
    say("%s: pinning %.1f GB of host memory" % (say_name, w.R * w.D * 4 / 2 ** 30))
    host = torch.empty((w.R, w.D), dtype=torch.float32, pin_memory=True)
    ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
    say("%s: filling the host table from the device" % say_name)
    emb.emb_table_fill(ptr, w.R, w.D, "f32", w.table_seed(0))
    torch.cuda.synchronize()
    host_np = host.numpy()
    probe = np.sort(rng.integers(0, w.R, size=20_000))
    assert np.array_equal(host_np[probe], wl.table_values(w.table_seed(0), probe, w.D))

    # hot set: rows of the most popular IDs, most popular first, first K distinct
    n_ranks = int(K * 1.06) + 1000
    hot_raw = wl.hot_raw_ids(w, 0, n_ranks)
    say("%s: hashing %d popular IDs (device and oracle)" % (say_name, n_ranks))
    hot_rows_dev = torch.empty(n_ranks, dtype=torch.int64, device=H.DEV)
    emb.emb_hash_ids(H.dev(hot_raw), w.salt(0), w.R, hot_rows_dev)
    hot_rows_ref = oracle.hash_ids(hot_raw, w.salt(0), w.R)
    assert np.array_equal(hot_rows_dev.cpu().numpy(), hot_rows_ref)
    hot = wl.first_k_distinct_sorted(hot_rows_ref, K)
    assert hot.size == K
    del hot_rows_dev

    say("%s: building the cache (%d rows, %.2f GB)" % (say_name, K, K * w.D * 4 / 2 ** 30))
    index = torch.empty(emb.emb_cache_index_bytes(w.R), dtype=torch.uint8, device=H.DEV)
    cache = torch.empty((K, w.D), dtype=torch.float32, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    hot_dev = H.dev(hot)
    emb.emb_cache_build(ptr, w.R, w.D, "f32", hot_dev, cache, index, status)
    torch.cuda.synchronize()
    assert status.item() == 0
    sample = np.sort(rng.integers(0, K, size=20_000))
    assert np.array_equal(cache[torch.from_numpy(sample).to(H.DEV)].cpu().numpy(),
                          wl.table_values(w.table_seed(0), hot[sample], w.D))

    batch = wl.make_batch(w, 0)
    db = pipeline.DeviceBatch(w, batch, torch.device(H.DEV))
    off_dev = torch.empty(w.B + 1, dtype=torch.int64, device=H.DEV)
    rows_dev = torch.empty(db.nnz, dtype=torch.int64, device=H.DEV)
    out = torch.empty((1, w.B, w.D), dtype=torch.float32, device=H.DEV)
    hm = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    emb.emb_lengths_to_offsets(db.lengths, off_dev, status)
    emb.emb_hash_ids(db.raw, w.salt(0), w.R, rows_dev)
    emb.emb_bag_forward_cached(ptr, w.R, w.D, "f32", cache, index, K, rows_dev, off_dev, w.B, w.pool, out, hm, status)
    torch.cuda.synchronize()
    assert status.item() == 0
    off, rows = _oracle_index(w, batch)
    assert np.array_equal(off_dev.cpu().numpy(), off) and np.array_equal(rows_dev.cpu().numpy(), rows)
    say("%s: oracle forward over %d lookups" % (say_name, rows.size))
    table = wl.sparse_host_table(w.table_seed(0), w.R, w.D, "f32", rows)
    ref, absum, (hits, misses), st = oracle.bag_forward_cached(table, "f32", hot, rows, off, w.B, w.pool)
    assert st == 0
    assert hm.cpu().tolist() == [hits, misses]                         # bit-exact hit/miss counts
    H.assert_pooled_close(out.cpu().numpy(), ref, absum, what=say_name)
    say("%s: %d hits, %d misses (%.1f %% hit rate)" % (say_name, hits, misses, 100.0 * hits / max(1, hits + misses)))
    _check_cached_from_lengths(w, "f32", ptr, cache, index, K, db, off, out, hm, say_name)

    # the route with the misses fetched ahead: three batches staged by one launch (raw IDs), then one pooled lookup
    # per batch over HBM only; every batch against the oracle's cached lookup of that batch
    batches = [batch] + [wl.make_batch(w, i) for i in (1, 2)]
    raws = torch.cat([torch.from_numpy(b["raw"].view(np.int64)) for b in batches]).to(H.DEV)
    n_all = raws.numel()
    cap = n_all // 8
    stage = torch.empty((cap, w.D), dtype=torch.float32, device=H.DEV)
    loc = torch.empty(n_all, dtype=torch.int64, device=H.DEV)
    count = torch.zeros(1, dtype=torch.int64, device=H.DEV)
    emb.emb_cache_stage_misses(ptr, w.R, w.D, "f32", index, K, raws, stage, cap, loc, count, status, salt=w.salt(0))
    at = 0
    total_misses = 0
    for i, b in enumerate(batches):
        off_b, rows_b = _oracle_index(w, b)
        n = rows_b.size
        hm.zero_()
        emb.emb_bag_forward_staged(ptr, w.R, w.D, "f32", cache, K, stage, cap, loc[at:at + n], H.dev(off_b), w.B, w.pool,
                                   out, hm, status)
        torch.cuda.synchronize()
        assert status.item() == 0
        tb = wl.sparse_host_table(w.table_seed(0), w.R, w.D, "f32", rows_b)
        ref_b, absum_b, (h_b, m_b), st = oracle.bag_forward_cached(tb, "f32", hot, rows_b, off_b, w.B, w.pool)
        assert st == 0 and hm.cpu().tolist() == [h_b, m_b]
        H.assert_pooled_close(out.cpu().numpy(), ref_b, absum_b, what="%s staged batch %d" % (say_name, i))
        total_misses += m_b
        at += n
        del tb
    assert int(count.item()) == total_misses and total_misses <= cap
    say("%s: %d misses of 3 batches staged by one launch, lookups over HBM match the oracle" % (say_name, total_misses))
    return hits / max(1, hits + misses)


def test_workload_5_host_table_with_hbm_cache():
    w = _full_size_or_skip("5", 90 * 2 ** 30)
    assert w.R == 250_000_000 and w.D == 64                  # 64 GB of fp32 rows in pinned host memory
    rate = _hybrid_parity(w, "workload " + w.name)
    assert 0.85 < rate < 0.97            # Zipf(1.1) over 1e9 keys: the top 5 % of rows carry ~92 % of lookups


def test_workload_5q4_int4_host_table_with_hbm_cache():
    # Workload 5 with the hosted table stored as INT4 rows (the paper quantises exactly these tables).
    # The fp32 table is filled in HBM and quantised into pinned host memory by the device; the oracle
    # quantises the generator's values of the rows the batch and the checks touch.
    rb = emb.emb_row_bytes(wl.WORKLOADS["5q4"].D, wl.WORKLOADS["5q4"].quant)
    w = _full_size_or_skip("5q4", wl.WORKLOADS["5q4"].R * rb + (26 << 30))
    assert w.R == 250_000_000
    _release_pinned_cache()
    rng = np.random.default_rng(6)
    K = int(round(w.hot_fraction * w.R))
    say("5q4: filling %.0f GB of fp32 rows in HBM, quantising into %.1f GB of pinned host memory" % (
        w.R * w.D * 4 / 2 ** 30, w.R * rb / 2 ** 30))
    host = torch.empty((w.R, rb), dtype=torch.uint8, pin_memory=True)
    ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
    src = torch.empty((w.R, w.D), dtype=torch.float32, device=H.DEV)
    emb.emb_table_fill(src, w.R, w.D, "f32", w.table_seed(0))
    emb.emb_quantize_rows(src, w.quant, ptr)
    torch.cuda.synchronize()
    del src
    torch.cuda.empty_cache()
    probe = np.sort(rng.integers(0, w.R, size=20_000))
    assert np.array_equal(host.numpy()[probe],
                          oracle.quantize_rows(wl.table_values(w.table_seed(0), probe, w.D), w.quant))

    n_ranks = int(K * 1.06) + 1000
    hot = wl.first_k_distinct_sorted(oracle.hash_ids(wl.hot_raw_ids(w, 0, n_ranks), w.salt(0), w.R), K)
    assert hot.size == K
    index = torch.empty(emb.emb_cache_index_bytes(w.R), dtype=torch.uint8, device=H.DEV)
    cache = torch.empty((K, rb), dtype=torch.uint8, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_cache_build(ptr, w.R, w.D, w.quant, H.dev(hot), cache, index, status)
    torch.cuda.synchronize()
    assert status.item() == 0
    sample = np.sort(rng.integers(0, K, size=20_000))
    assert np.array_equal(cache[torch.from_numpy(sample).to(H.DEV)].cpu().numpy(),
                          oracle.quantize_rows(wl.table_values(w.table_seed(0), hot[sample], w.D), w.quant))

    batch = wl.make_batch(w, 0)
    db = pipeline.DeviceBatch(w, batch, torch.device(H.DEV))
    off_dev = torch.empty(w.B + 1, dtype=torch.int64, device=H.DEV)
    rows_dev = torch.empty(db.nnz, dtype=torch.int64, device=H.DEV)
    out = torch.empty((1, w.B, w.D), dtype=torch.float32, device=H.DEV)
    hm = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    emb.emb_lengths_to_offsets(db.lengths, off_dev, status)
    emb.emb_hash_ids(db.raw, w.salt(0), w.R, rows_dev)
    emb.emb_bag_forward_cached(ptr, w.R, w.D, w.quant, cache, index, K, rows_dev, off_dev, w.B, w.pool, out, hm, status)
    torch.cuda.synchronize()
    assert status.item() == 0
    off, rows = _oracle_index(w, batch)
    assert np.array_equal(rows_dev.cpu().numpy(), rows)
    say("5q4: oracle quantiser and forward over %d lookups" % rows.size)
    # compact table of the touched rows; lookups and hot rows renumbered into it (plumbing only)
    touched = np.unique(rows)
    packed = oracle.quantize_rows(wl.table_values(w.table_seed(0), touched, w.D), w.quant)
    hot_compact = np.flatnonzero(np.isin(touched, hot, assume_unique=True)).astype(np.int64)
    ref, absum, (hits, misses), st = oracle.bag_forward_cached(packed, w.quant, hot_compact,
                                                               np.searchsorted(touched, rows).astype(np.int64), off,
                                                               w.B, w.pool, D=w.D)
    assert st == 0
    assert hm.cpu().tolist() == [hits, misses]
    H.assert_pooled_close(out.cpu().numpy(), ref, absum, what="workload 5q4")
    _check_cached_from_lengths(w, w.quant, ptr, cache, index, K, db, off, out, hm, "5q4")
    assert 0.85 < hits / max(1, hits + misses) < 0.97


def _check_cached_from_lengths(w, store, ptr, cache, index, K, db, off, out, hm, name):
    """The call the bench times for a hosted table: raw IDs and bag lengths in.  Offsets against the oracle's,
    pooled output and hit/miss counts bit for bit against the (oracle-checked) lookup over hashed rows."""
    out2 = torch.full_like(out, float("nan"))
    hm2 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    off2 = torch.full((w.B + 1,), -1, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    scratch = torch.empty(emb.emb_offsets_scratch_bytes(w.B), dtype=torch.uint8, device=H.DEV)
    emb.emb_bag_forward_cached_hashed_lengths(ptr, w.R, w.D, store, cache, index, K, w.salt(0), db.raw, db.lengths, w.B,
                                              w.pool, out2, off2, scratch, hm2, status)
    torch.cuda.synchronize()
    assert status.item() == 0 and np.array_equal(off2.cpu().numpy(), off), name
    assert torch.equal(out2, out) and torch.equal(hm2, hm), name


def test_workload_5q4_cache_policy_at_full_size():
    # The frequency-based policy on the full-size hosted INT4 table: counters against the oracle's over the
    # whole table; the selected hot set row for row against the oracle's rule evaluated by selection instead
    # of a full sort (the sorting definition takes minutes over 2.5e8 rows; the two are pinned to each other
    # on the CPU); the refreshed cache's rows and the lookup through it against the oracle.
    rb = emb.emb_row_bytes(wl.WORKLOADS["5q4"].D, wl.WORKLOADS["5q4"].quant)
    w = _full_size_or_skip("5q4", wl.WORKLOADS["5q4"].R * rb + (30 << 30))
    assert w.R == 250_000_000
    _release_pinned_cache()
    rng = np.random.default_rng(7)
    K = int(round(w.hot_fraction * w.R))
    host = torch.empty((w.R, rb), dtype=torch.uint8, pin_memory=True)
    ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
    src = torch.empty((w.R, w.D), dtype=torch.float32, device=H.DEV)
    emb.emb_table_fill(src, w.R, w.D, "f32", w.table_seed(0))
    emb.emb_quantize_rows(src, w.quant, ptr)
    torch.cuda.synchronize()
    del src
    torch.cuda.empty_cache()
    cache = pipeline.HotRowCache(ptr, w.R, w.D, w.quant, K, w.salt(0), torch.device(H.DEV), decay_shift=1)
    ref_freq = np.zeros(w.R, np.uint32)

    def watch(chunks):
        for c in chunks:
            raw = wl.traffic_raw_ids(w, 0, 5_000_000, c)
            cache.observe(H.dev(raw))
            assert oracle.cache_observe(ref_freq, oracle.hash_ids(raw, w.salt(0), w.R)) == 0
        torch.cuda.synchronize()
        say("cache policy: %d lookups watched" % (5_000_000 * len(chunks)))

    def check_refresh(old_hot):
        counts = ref_freq.copy()
        assert np.array_equal(cache.freq.cpu().numpy().view(np.uint32), counts)      # every counter, exactly
        cache.moved.zero_()
        cache.refresh()
        torch.cuda.synchronize()
        thr, tied_taken = [int(x) for x in cache.info.cpu().tolist()]
        hot = H.cache_select_large(ref_freq, K, 1)                               # also ages ref_freq
        assert np.array_equal(cache.hot[:K].cpu().numpy(), hot)                       # the hot set, row for row
        assert thr == int(counts[hot].min()) and tied_taken == int((counts[hot] == thr).sum())
        assert np.array_equal(cache.freq.cpu().numpy().view(np.uint32), ref_freq)
        n_kept = int(np.isin(hot, old_hot, assume_unique=True).sum())
        assert cache.moved.cpu().tolist() == [n_kept, K - n_kept]
        sample = np.sort(rng.integers(0, K, size=20_000))
        got = cache.rows[cache.active][torch.from_numpy(sample).to(H.DEV)].cpu().numpy()
        assert np.array_equal(got, oracle.quantize_rows(wl.table_values(w.table_seed(0), hot[sample], w.D), w.quant))
        say("cache policy: refresh ok (threshold count %d, %d rows kept in HBM, %d fetched)" % (thr, n_kept, K - n_kept))
        return hot

    watch([0, 1])
    hot = check_refresh(np.zeros(0, np.int64))
    watch([2])
    hot = check_refresh(hot)

    batch = wl.make_batch(w, 0)
    db = pipeline.DeviceBatch(w, batch, torch.device(H.DEV))
    off_dev = torch.empty(w.B + 1, dtype=torch.int64, device=H.DEV)
    out = torch.empty((1, w.B, w.D), dtype=torch.float32, device=H.DEV)
    emb.emb_lengths_to_offsets(db.lengths, off_dev, cache.status)
    cache.forward_hashed(db.raw, off_dev, w.B, w.pool, out)
    torch.cuda.synchronize()
    assert cache.status.item() == 0
    off, rows = _oracle_index(w, batch)
    touched = np.unique(rows)
    packed = oracle.quantize_rows(wl.table_values(w.table_seed(0), touched, w.D), w.quant)
    hot_compact = np.flatnonzero(np.isin(touched, hot, assume_unique=True)).astype(np.int64)
    ref, absum, (hits, misses), st = oracle.bag_forward_cached(packed, w.quant, hot_compact,
                                                               np.searchsorted(touched, rows).astype(np.int64), off,
                                                               w.B, w.pool, D=w.D)
    assert st == 0 and cache.hit_miss.cpu().tolist() == [hits, misses]
    H.assert_pooled_close(out.cpu().numpy(), ref, absum, what="workload 5q4 through the learnt cache")
    assert hits / max(1, hits + misses) > 0.75             # 1.5e7 watched lookups: what the law allows is ~0.85


def test_workload_5mq4_four_hosted_int4_tables_in_one_launch():
    # The launch bench.py times for workload 5mq4: four hosted INT4 tables with their caches, raw IDs, one
    # cached lookup for all.  The oracle quantises the generator's values of the rows each table's lookups touch.
    w0 = wl.WORKLOADS["5mq4"]
    rb = emb.emb_row_bytes(w0.D, w0.quant)
    w = _full_size_or_skip("5mq4", w0.T * w0.R * rb + (30 << 30))
    assert w.T * w.R == 250_000_000
    _release_pinned_cache()
    K = int(round(w.hot_fraction * w.R))
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    hosts, hots, entries = [], [], []
    for t in range(w.T):
        host = torch.empty((w.R, rb), dtype=torch.uint8, pin_memory=True)
        ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
        src = torch.empty((w.R, w.D), dtype=torch.float32, device=H.DEV)
        emb.emb_table_fill(src, w.R, w.D, "f32", w.table_seed(t))
        emb.emb_quantize_rows(src, w.quant, ptr)
        torch.cuda.synchronize()
        del src
        hot = wl.first_k_distinct_sorted(oracle.hash_ids(wl.hot_raw_ids(w, t, int(K * 1.06) + 1000), w.salt(t), w.R), K)
        assert hot.size == K
        index = torch.empty(emb.emb_cache_index_bytes(w.R), dtype=torch.uint8, device=H.DEV)
        cache = torch.empty((K, rb), dtype=torch.uint8, device=H.DEV)
        emb.emb_cache_build(ptr, w.R, w.D, w.quant, H.dev(hot), cache, index, status)
        hosts.append(host)
        hots.append(hot)
        entries.append((ptr, w.R, cache, index, K, w.salt(t)))
        say("5mq4: table %d quantised into pinned memory, cache built" % t)
    torch.cuda.empty_cache()
    ct = emb.CachedTables(entries, w.D, w.quant, device=torch.device(H.DEV))
    batch = wl.make_batch(w, 0)
    db = pipeline.DeviceBatch(w, batch, torch.device(H.DEV))
    off_dev = torch.empty(w.T * w.B + 1, dtype=torch.int64, device=H.DEV)
    out = torch.full((w.T, w.B, w.D), float("nan"), dtype=torch.float32, device=H.DEV)
    hm = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    emb.emb_lengths_to_offsets(db.lengths, off_dev, status)
    emb.emb_bag_forward_cached_tables_hashed(ct, db.raw, off_dev, w.B, w.pool, out, hm, status)
    torch.cuda.synchronize()
    assert status.item() == 0
    off, rows = _oracle_index(w, batch)
    assert np.array_equal(off_dev.cpu().numpy(), off)
    got = out.cpu().numpy()
    hits = misses = 0
    for t in range(w.T):
        s, e = int(off[t * w.B]), int(off[(t + 1) * w.B])
        r = rows[s:e]
        touched = np.unique(r)
        packed = oracle.quantize_rows(wl.table_values(w.table_seed(t), touched, w.D), w.quant)
        hot_compact = np.flatnonzero(np.isin(touched, hots[t], assume_unique=True)).astype(np.int64)
        ref, absum, (h, m), st = oracle.bag_forward_cached(packed, w.quant, hot_compact,
                                                           np.searchsorted(touched, r).astype(np.int64),
                                                           off[t * w.B:(t + 1) * w.B + 1] - s, w.B, w.pool, D=w.D)
        assert st == 0
        H.assert_pooled_close(got[t], ref[0], absum[0], what="workload 5mq4 table %d" % t)
        hits, misses = hits + h, misses + m
    assert hm.cpu().tolist() == [hits, misses]
    say("5mq4: %d hits, %d misses" % (hits, misses))
    # the call the bench times: the same lookup from the bag lengths (offsets made on the way), bit for bit
    out2 = torch.full_like(out, float("nan"))
    hm2 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    off2 = torch.full_like(off_dev, -1)
    scratch = torch.empty(emb.emb_offsets_scratch_bytes(w.T * w.B), dtype=torch.uint8, device=H.DEV)
    emb.emb_bag_forward_cached_tables_hashed_lengths(ct, db.raw, db.lengths, w.B, w.pool, out2, off2, scratch, hm2, status)
    torch.cuda.synchronize()
    assert status.item() == 0 and np.array_equal(off2.cpu().numpy(), off)
    assert torch.equal(out2, out) and torch.equal(hm2, hm)
    assert 0.8 < hits / max(1, hits + misses) < 0.97


def test_workload_mix_24_tables_of_four_widths_in_one_launch():
    # The launch bench.py times for workload "mix": 24 full-size tables (D = 16/32/64/128, fp32 and bf16),
    # config 2's batch recipe, one mixed-width lookup writing one concatenated vector per sample.
    w = wl.WORKLOADS["mix"]
    spec = wl.MIX_SPEC
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16}
    say("mix: filling %d tables (%.1f GB)" % (len(spec), sum(R * D * (4 if dt == "f32" else 2) for D, dt, R in spec) / 2 ** 30))
    weights = []
    for t, (D, dt, R) in enumerate(spec):
        wt = torch.empty((R, D), dtype=tdt[dt], device=H.DEV)
        emb.emb_table_fill(wt, R, D, dt, w.table_seed(t))
        weights.append(wt)
    mt = emb.MixedTables(weights, w.B, "concat", salts=[w.salt(t) for t in range(w.T)], device=torch.device(H.DEV))
    batch = wl.make_batch(w, 0)
    db = pipeline.DeviceBatch(w, batch, torch.device(H.DEV))
    offsets = torch.empty(w.T * w.B + 1, dtype=torch.int64, device=H.DEV)
    rows_dev = torch.empty(db.nnz, dtype=torch.int64, device=H.DEV)
    out = torch.full((mt.out_floats,), float("nan"), dtype=torch.float32, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_lengths_to_offsets(db.lengths, offsets, status)
    emb.emb_hash_ids_tables(mt.tables, db.raw, offsets, w.B, rows_dev, status)
    emb.emb_bag_forward_mixed(mt, rows_dev, offsets, w.pool, out, status)
    torch.cuda.synchronize()
    assert status.item() == 0
    off, st = oracle.lengths_to_offsets(batch["lengths"])
    assert st == 0 and np.array_equal(offsets.cpu().numpy(), off)
    got = out.cpu().numpy().reshape(w.B, sum(D for D, _, _ in spec))
    rows_got = rows_dev.cpu().numpy()
    col = 0
    for t, (D, dt, R) in enumerate(spec):
        s, e = int(off[t * w.B]), int(off[(t + 1) * w.B])
        rows = oracle.hash_ids(batch["raw"][s:e], w.salt(t), R)
        assert np.array_equal(rows_got[s:e], rows)
        touched = np.unique(rows)
        table = wl.table_rows(w.table_seed(t), touched, D, dt)
        ref, absum, st = oracle.bag_forward([table], dt, np.searchsorted(touched, rows).astype(np.int64),
                                            off[t * w.B:(t + 1) * w.B + 1] - s, w.B, w.pool)
        assert st == 0
        H.assert_pooled_close(got[:, col:col + D], ref[0], absum[0], what="mix table %d (D=%d %s)" % (t, D, dt))
        col += D
    say("mix: %d lookups over %d tables checked" % (db.nnz, w.T))

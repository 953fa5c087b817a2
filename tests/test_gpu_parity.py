"""GPU parity: the HIP library against the CPU oracle, element by element, on
seeded inputs that span several tiles and ragged tails, plus edge cases.
Everything goes through the C ABI (via the ctypes binding)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import emb_oracle as oracle  # noqa: E402
from paper_2508_05700_amd import binding as emb  # noqa: E402
from paper_2508_05700_amd import workloads as wl  # noqa: E402
from tests import harness as H  # noqa: E402

M64 = (1 << 64) - 1


# ---------------------------------------------------------------------------
# hashing: bit-exact
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n", [0, 1, 63, 255, 256, 257, 100_003])
def test_hash_ids_bit_exact(n):
    rng = np.random.default_rng(100 + n)
    raw = rng.integers(0, 1 << 64, size=n, dtype=np.uint64)
    if n >= 8:
        raw[:8] = [0, 1, M64, M64 - 1, 1 << 63, (1 << 63) - 1, 1 << 32, (1 << 32) - 1]
    for R, salt in [(1, 0), (2, 5), (10_000_000, 3), (1_000_000_000, M64), (250_000_000, 1 << 63),
                    ((1 << 31) - 1, 9), (1 << 32, 11), ((1 << 40) + 17, 13), ((1 << 63) - 1, 17)]:
        rows = torch.full((n,), -5, dtype=torch.int64, device=H.DEV)
        emb.emb_hash_ids(H.dev(raw), salt, R, rows)
        torch.cuda.synchronize()
        assert np.array_equal(rows.cpu().numpy(), oracle.hash_ids(raw, salt, R)), (n, R, salt)


def test_hash_ids_tables_bit_exact():
    rng = np.random.default_rng(7)
    T, B = 5, 37
    Rs = [10_000_000, 3, (1 << 33) + 5, 999_983, 1]
    salts = [0, 1, M64, 12345, 1 << 40]
    lengths = rng.integers(0, 50, size=T * B).astype(np.int32)
    lengths[B:2 * B] = 0                                   # a table with no lookups at all
    off, _ = oracle.lengths_to_offsets(lengths)
    nnz = int(off[-1])
    raw = rng.integers(0, 1 << 64, size=nnz, dtype=np.uint64)
    tables = [torch.empty((1, 4), dtype=torch.float32, device=H.DEV) for _ in range(T)]
    ts = emb.TableSet([(int(t.data_ptr()), R) for t, R in zip(tables, Rs)], 4, "f32", salts=salts,
                      device=torch.device(H.DEV))
    rows = torch.full((nnz,), -5, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_hash_ids_tables(ts, H.dev(raw), H.dev(off), B, rows, status)
    torch.cuda.synchronize()
    ref = np.concatenate([oracle.hash_ids(raw[off[t * B]:off[(t + 1) * B]], salts[t], Rs[t]) for t in range(T)])
    assert status.item() == 0 and np.array_equal(rows.cpu().numpy(), ref)


# ---------------------------------------------------------------------------
# offsets: bit-exact
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n", [0, 1, 2, 4095, 4096, 4097, 131_072, 200_003, 262_144, 262_145, 1_000_005, 4096 * 1025 + 3])
def test_offsets_bit_exact(n):
    rng = np.random.default_rng(200 + n % 1000)
    L = rng.integers(0, 101, size=n).astype(np.int32)
    out = torch.full((n + 1,), -9, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_lengths_to_offsets(H.dev(L) if n else torch.empty(0, dtype=torch.int32, device=H.DEV), out, status)
    torch.cuda.synchronize()
    ref, _ = oracle.lengths_to_offsets(L)
    assert status.item() == 0 and np.array_equal(out.cpu().numpy(), ref)


def test_offsets_large_values_and_negative_lengths():
    L = np.full(10_000, 2_000_000_000, dtype=np.int32)      # sums far beyond 32 bits
    L[[5, 4096, 9999]] = [-1, -2_000_000_000, -7]
    out = torch.empty(L.size + 1, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_lengths_to_offsets(H.dev(L), out, status)
    torch.cuda.synchronize()
    ref, st = oracle.lengths_to_offsets(L)
    assert status.item() == st == emb.STATUS_BAD_OFFSETS and np.array_equal(out.cpu().numpy(), ref)


@pytest.mark.parametrize("n", [20_000, 300_000])
def test_offsets_negative_lengths_in_earlier_tiles_and_unaligned_input(n):
    # a negative length counts as 0 wherever it sits, also in tiles before the one that is being summed; the
    # lengths need not start on a 16-byte boundary
    rng = np.random.default_rng(210 + n)
    L = rng.integers(0, 50, size=n + 1).astype(np.int32)
    L[rng.choice(n, size=40, replace=False)] = -rng.integers(1, 1000, size=40).astype(np.int32)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    for skip in (0, 1):
        src = H.dev(L)[skip:skip + n]
        out = torch.full((n + 1,), -9, dtype=torch.int64, device=H.DEV)
        status.zero_()
        emb.emb_lengths_to_offsets(src, out, status)
        torch.cuda.synchronize()
        ref, st = oracle.lengths_to_offsets(L[skip:skip + n])
        assert status.item() == st == emb.STATUS_BAD_OFFSETS and np.array_equal(out.cpu().numpy(), ref)


# ---------------------------------------------------------------------------
# forward
# ---------------------------------------------------------------------------
FWD_SHAPES = [
    # D, dtype  -> lanes per row / chunks per lane exercised
    (4, "f32"), (8, "f32"), (16, "f32"), (32, "f32"), (64, "f32"), (128, "f32"), (256, "f32"),
    (48, "f32"),      # 12 chunks: not a power of two
    (320, "f32"),     # 80 chunks: 64 lanes x 2, ragged
    (1024, "f32"),    # 4 chunks per lane
    (4096, "f32"),    # 16 chunks per lane (16 KB rows)
    (8, "bf16"), (32, "bf16"), (64, "bf16"), (128, "bf16"), (520, "bf16"), (8192, "bf16"),
]


@pytest.mark.parametrize("D,dtype", FWD_SHAPES)
@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_forward_matches_oracle(D, dtype, mode):
    rng = np.random.default_rng(D * 7 + (dtype == "bf16") + 2 * (mode == "mean"))
    T, B = 3, 301 if D <= 256 else 37
    Rs = [1000, 17, 4099] if D <= 256 else [50, 3, 40]
    tables, lengths, off, rows = H.random_case(rng, T, B, D, Rs, 70 if D <= 256 else 20, dtype, scale=0.01)
    ts, _, _ = H.make_tableset(tables, dtype)
    out, st = H.gpu_forward(ts, rows, off, B, mode)
    ref, absum, rst = oracle.bag_forward(tables, dtype, rows, off, B, mode)
    assert st == rst == 0
    H.assert_pooled_close(out, ref, absum, what="forward D=%d %s %s" % (D, dtype, mode))
    assert np.all(out.reshape(T * B, D)[lengths == 0] == 0.0)         # empty bags give exact zeros


def test_forward_integer_valued_tables_are_bit_exact():
    # small integers make every fp32 summation order exact: GPU == oracle bit for bit
    rng = np.random.default_rng(31)
    T, B, D, Rs = 2, 513, 64, [5000, 33]
    tables, lengths, off, rows = H.random_case(rng, T, B, D, Rs, 100)
    tables = [np.rint(t * 300).astype(np.float32) for t in tables]
    ts, _, _ = H.make_tableset(tables, "f32")
    out, st = H.gpu_forward(ts, rows, off, B, "sum")
    ref, _, _ = oracle.bag_forward(tables, "f32", rows, off, B, "sum")
    assert st == 0 and np.array_equal(out, ref)


def test_forward_long_bags_and_single_bag():
    rng = np.random.default_rng(32)
    D, R = 64, 100_000
    table = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
    lengths = np.array([5000, 0, 1, 64, 65, 127, 128, 129, 3000], dtype=np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    rows = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    ts, _, _ = H.make_tableset([table], "f32")
    for mode in ("sum", "mean"):
        out, st = H.gpu_forward(ts, rows, off, lengths.size, mode)
        ref, absum, _ = oracle.bag_forward([table], "f32", rows, off, lengths.size, mode)
        assert st == 0
        H.assert_pooled_close(out, ref, absum, what="long bags " + mode)


def test_forward_bad_indices_and_offsets_are_flagged_and_skipped():
    rng = np.random.default_rng(33)
    T, B, D, Rs = 2, 40, 32, [100, 50]
    tables, lengths, off, rows = H.random_case(rng, T, B, D, Rs, 12)
    rows = rows.copy()
    n0 = int(off[B])
    rows[[0, 7, n0 - 1]] = [100, -1, 1 << 40]           # out of range for table 0
    rows[n0 + 3] = 50                                   # == num_rows of table 1
    ts, _, _ = H.make_tableset(tables, "f32")
    out, st = H.gpu_forward(ts, rows, off, B, "mean")
    ref, absum, rst = oracle.bag_forward(tables, "f32", rows, off, B, "mean")
    assert st == rst == emb.STATUS_BAD_INDEX
    H.assert_pooled_close(out, ref, absum, what="bad index")
    bad_off = off.copy()
    bad_off[5] = bad_off[6] + 3                          # bag 4 too long, bag 5 reversed
    bad_off[-1] = off[-1] + 10                           # last bag runs past nnz
    out, st = H.gpu_forward(ts, rows, bad_off, B, "sum")
    ref, absum, rst = oracle.bag_forward(tables, "f32", rows, bad_off, B, "sum")
    assert st == rst and (st & emb.STATUS_BAD_OFFSETS)
    H.assert_pooled_close(out, ref, absum, what="bad offsets")


@pytest.mark.parametrize("D,dtype", [(64, "f32"), (32, "bf16"), (320, "f32")])
def test_forward_hashed_equals_hash_then_forward(D, dtype):
    rng = np.random.default_rng(1500 + D)
    T, B = 4, 500
    Rs = [100_003, 7, 1 << 20, 5000]
    salts = [0, 11, M64, 1 << 33]
    tables, lengths, off, _ = H.random_case(rng, T, B, D, Rs, 25, dtype)
    nnz = int(off[-1])
    raw = rng.integers(0, 1 << 64, size=nnz, dtype=np.uint64)
    w = [H.dev(t) for t in tables]
    ts = emb.TableSet(w, D, dtype, salts=salts, device=torch.device(H.DEV))
    out = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    rows_out = torch.full((nnz,), -9, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_hashed(ts, H.dev(raw), H.dev(off), B, "mean", out, rows_out, status)
    torch.cuda.synchronize()
    rows = np.concatenate([oracle.hash_ids(raw[off[t * B]:off[(t + 1) * B]], salts[t], Rs[t]) for t in range(T)])
    assert status.item() == 0 and np.array_equal(rows_out.cpu().numpy(), rows)       # bit-exact rows
    ref, absum, _ = oracle.bag_forward(tables, dtype, rows, off, B, "mean")
    H.assert_pooled_close(out.cpu().numpy(), ref, absum, eps=H.EPS32, what="hashed forward")
    two_step, _ = H.gpu_forward(ts, rows, off, B, "mean")
    assert np.array_equal(two_step.reshape(T, B, D), out.cpu().numpy())              # same bits as the two calls
    # without the row output
    out2 = torch.empty_like(out)
    emb.emb_bag_forward_hashed(ts, H.dev(raw), H.dev(off), B, "mean", out2, None, status)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("layout", ["concat", "table_major"])
@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_forward_mixed_widths_and_types_matches_oracle(layout, mode):
    # eight tables, widths 4 .. 256, fp32 and bf16, in one launch; the oracle pools them one by one
    rng = np.random.default_rng(1600 + (layout == "concat") + 2 * (mode == "mean"))
    spec = [(4, "f32", 300), (16, "f32", 5000), (8, "bf16", 77), (64, "f32", 20_000), (256, "f32", 900),
            (32, "bf16", 3000), (512, "bf16", 64), (48, "f32", 1)]
    T, B = len(spec), 333
    tables = []
    for D, dt, R in spec:
        v = rng.standard_normal((R, D)).astype(np.float32)
        tables.append(wl.f32_to_bf16_bits(v).reshape(R, D) if dt == "bf16" else v)
    lengths = rng.integers(0, 30, size=T * B).astype(np.int32)
    lengths[rng.random(T * B) < 0.2] = 0
    off, _ = oracle.lengths_to_offsets(lengths)
    rows = np.concatenate([rng.integers(0, spec[t][2], size=int(off[(t + 1) * B] - off[t * B])) for t in range(T)])
    rows = rows.astype(np.int64)
    rows[[1, 50]] = [-4, 1 << 35]
    mt = emb.MixedTables([H.dev(t) for t in tables], B, layout, device=torch.device(H.DEV))
    out = torch.full((mt.out_floats,), float("nan"), dtype=torch.float32, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_mixed(mt, H.dev(rows), H.dev(off), mode, out, status)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.isfinite(got).all()                              # the layout covers every float
    total = sum(D for D, _, _ in spec)
    col = 0
    st_ref = 0
    for t, (D, dt, R) in enumerate(spec):
        seg = slice(off[t * B], off[(t + 1) * B])
        ref, absum, st = oracle.bag_forward([tables[t]], dt, rows[seg], off[t * B:(t + 1) * B + 1] - off[t * B], B, mode)
        st_ref |= st
        if layout == "concat":
            mine = got.reshape(B, total)[:, col:col + D]
        else:
            mine = got[col * B:(col + D) * B].reshape(B, D)
        H.assert_pooled_close(mine, ref[0], absum[0], eps=H.EPS32, what="mixed table %d" % t)
        col += D
    assert int(status.item()) == st_ref == emb.STATUS_BAD_INDEX


@pytest.mark.parametrize("D,dtype", [(64, "f32"), (16, "bf16"), (1024, "f32")])
def test_forward_streaming_hint_changes_no_bit(D, dtype):
    rng = np.random.default_rng(1700 + D)
    T, B = 2, 300
    Rs = [4000, 90]
    tables, lengths, off, rows = H.random_case(rng, T, B, D, Rs, 20, dtype)
    ts = emb.TableSet([H.dev(t) for t in tables], D, dtype, device=torch.device(H.DEV))
    plain, st = H.gpu_forward(ts, rows, off, B, "mean")
    out = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward(ts, H.dev(rows), H.dev(off), B, "mean", out, status, streaming=True)
    raw = rng.integers(0, 1 << 64, size=rows.size, dtype=np.uint64)
    h1 = torch.empty_like(out)
    h2 = torch.empty_like(out)
    emb.emb_bag_forward_hashed(ts, H.dev(raw), H.dev(off), B, "sum", h1, None, status)
    emb.emb_bag_forward_hashed(ts, H.dev(raw), H.dev(off), B, "sum", h2, None, status, streaming=True)
    torch.cuda.synchronize()
    assert st == 0 and status.item() == 0
    assert np.array_equal(out.cpu().numpy().reshape(plain.shape), plain) and torch.equal(h1, h2)
    ref, absum, _ = oracle.bag_forward(tables, dtype, rows, off, B, "mean")
    H.assert_pooled_close(out.cpu().numpy(), ref, absum, what="streaming forward")


def test_forward_empty_batch_zero_fills():
    table = np.ones((10, 16), dtype=np.float32)
    ts, _, _ = H.make_tableset([table], "f32")
    off = np.zeros(9, dtype=np.int64)
    out, st = H.gpu_forward(ts, np.zeros(0, np.int64), off, 8, "mean")
    assert st == 0 and np.all(out == 0)


# ---------------------------------------------------------------------------
# row-quantised tables: quantiser bit-exact, dequantise-on-gather forward within tolerance
# ---------------------------------------------------------------------------
def _quant_source(rng, R, D):
    x = (rng.standard_normal((R, D)) * rng.uniform(1e-3, 5.0, size=(R, 1))).astype(np.float32)
    x[1] = -0.75                                              # constant row
    x[2, :] = 0.0
    x[2, :8] = [0.0, 15.0, 0.5, 1.5, 2.5, 3.5, 4.5, 14.5]     # exact ties for INT4 (scale 1)
    x[3, :] = 0.0
    x[3, :8] = [0.0, 255.0, 0.5, 1.5, 2.5, 3.5, 254.5, 100.5]  # exact ties for INT8
    x[4] = np.float32(1e-30) * rng.standard_normal(D).astype(np.float32)   # tiny scale
    return x


@pytest.mark.parametrize("D", [16, 32, 48, 64, 128, 208, 1024])
@pytest.mark.parametrize("dtype", ["int8", "int4"])
def test_quantize_rows_bit_exact(D, dtype):
    rng = np.random.default_rng(900 + D)
    R = 1000 + 3
    x = _quant_source(rng, R, D)
    dst = torch.full((R, emb.emb_row_bytes(D, dtype)), 0xAB, dtype=torch.uint8, device=H.DEV)
    emb.emb_quantize_rows(H.dev(x), dtype, dst)
    torch.cuda.synchronize()
    assert emb.emb_row_bytes(D, dtype) == oracle.quant_row_bytes(D, dtype)
    assert np.array_equal(dst.cpu().numpy(), oracle.quantize_rows(x, dtype))


@pytest.mark.parametrize("D", [16, 64, 48, 256, 1024])
@pytest.mark.parametrize("dtype", ["int8", "int4"])
@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_forward_quantized_matches_oracle(D, dtype, mode):
    rng = np.random.default_rng(950 + D + 7 * (dtype == "int4") + (mode == "mean"))
    T, B = 3, (40 if D >= 256 else 600)
    Rs = [5000, 7, 20_000]
    src = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in Rs]
    qt = [oracle.quantize_rows(x, dtype) for x in src]         # the oracle's quantiser makes the inputs
    lengths = rng.integers(0, 40, size=T * B).astype(np.int32)
    lengths[rng.random(T * B) < 0.15] = 0
    lengths[5] = 333                                           # one long bag
    off, _ = oracle.lengths_to_offsets(lengths)
    rows = np.concatenate([rng.integers(0, Rs[t], size=int(off[(t + 1) * B] - off[t * B])) for t in range(T)])
    rows = rows.astype(np.int64)
    rows[[2, 17]] = [-1, 1 << 40]                              # skipped and flagged on both sides
    ts = emb.TableSet([H.dev(q) for q in qt], D, dtype, device=torch.device(H.DEV))
    out, st = H.gpu_forward(ts, rows, off, B, mode)
    ref, absum, rst = oracle.bag_forward(qt, dtype, rows, off, B, mode, D=D)
    assert st == rst == emb.STATUS_BAD_INDEX
    H.assert_pooled_close(out, ref, absum, what="quantised forward %s D=%d" % (dtype, D))


@pytest.mark.parametrize("D", [16, 64, 112, 256])
def test_int4_rows_padded_to_64_bytes_hold_the_int4_row_and_give_the_same_lookups(D):
    # "int4r64" is a layout choice, not another encoding: the first bytes of every row are the oracle's INT4 row, the
    # rest is zero, and every lookup route pools what the oracle pools from the unpadded INT4 table
    rng = np.random.default_rng(990 + D)
    R, B, K = 6007, 500, 700
    x = _quant_source(rng, R, D)
    packed = oracle.quantize_rows(x, "int4")
    rb = (8 + D // 2 + 63) // 64 * 64
    assert emb.emb_row_bytes(D, "int4r64") == rb
    q = torch.full((R, rb), 0xAB, dtype=torch.uint8, device=H.DEV)
    emb.emb_quantize_rows(H.dev(x), "int4r64", q)
    torch.cuda.synchronize()
    got = q.cpu().numpy()
    assert np.array_equal(got[:, :packed.shape[1]], packed) and not got[:, packed.shape[1]:].any()
    lengths = rng.integers(0, 40, size=B).astype(np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    hot = np.sort(rng.choice(R, size=K, replace=False)).astype(np.int64)
    n = int(off[-1])
    rows = np.where(rng.random(n) < 0.6, rng.choice(hot, size=n), rng.integers(0, R, size=n)).astype(np.int64)
    rows[[3, 11]] = [R, -2]
    # plain lookup
    ts = emb.TableSet([q], D, "int4r64", device=torch.device(H.DEV))
    out, st = H.gpu_forward(ts, rows, off, B, "mean")
    ref, absum, rst = oracle.bag_forward([packed], "int4", rows, off, B, "mean", D=D)
    assert st == rst == emb.STATUS_BAD_INDEX
    H.assert_pooled_close(out, ref, absum, what="padded INT4 forward D=%d" % D)
    # cached lookup, and the staged one, over the same table
    ptr = int(q.data_ptr())
    index = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
    cache = torch.full((K, rb), 0xEE, dtype=torch.uint8, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_cache_build(ptr, R, D, "int4r64", H.dev(hot), cache, index, status)
    o1 = torch.full((1, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    hm1 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    emb.emb_bag_forward_cached(ptr, R, D, "int4r64", cache, index, K, H.dev(rows), H.dev(off), B, "sum", o1, hm1, status)
    cap = n
    stage = torch.zeros((cap, rb), dtype=torch.uint8, device=H.DEV)
    loc = torch.full((n,), -5, dtype=torch.int64, device=H.DEV)
    count = torch.zeros(1, dtype=torch.int64, device=H.DEV)
    emb.emb_cache_stage_misses(ptr, R, D, "int4r64", index, K, H.dev(rows), stage, cap, loc, count, status)
    o2 = torch.full((1, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    hm2 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    emb.emb_bag_forward_staged(ptr, R, D, "int4r64", cache, K, stage, cap, loc, H.dev(off), B, "sum", o2, hm2, status)
    torch.cuda.synchronize()
    assert np.array_equal(cache.cpu().numpy(), got[hot])
    ref, absum, (hits, misses), rst = oracle.bag_forward_cached(packed, "int4", hot, rows, off, B, "sum", D=D)
    assert int(status.item()) == rst == emb.STATUS_BAD_INDEX
    assert hm1.cpu().tolist() == hm2.cpu().tolist() == [hits, misses] and int(count.item()) == misses
    H.assert_pooled_close(o1.cpu().numpy(), ref, absum, what="padded INT4 cached lookup")
    H.assert_pooled_close(o2.cpu().numpy(), ref, absum, what="padded INT4 staged lookup")
    # several hosted tables in one launch
    ct = emb.CachedTables([(ptr, R, cache, index, K, 0)] * 2, D, "int4r64", device=torch.device(H.DEV))
    off2 = np.concatenate([off, off[1:] + off[-1]])
    rows2 = np.concatenate([rows, rows])
    o3 = torch.full((2, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    hm3 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    emb.emb_bag_forward_cached_tables(ct, H.dev(rows2), H.dev(off2), B, "sum", o3, hm3, status)
    torch.cuda.synchronize()
    assert hm3.cpu().tolist() == [2 * hits, 2 * misses]
    for t in range(2):
        H.assert_pooled_close(o3[t].cpu().numpy(), ref, absum, what="padded INT4 hosted tables")


@pytest.mark.parametrize("D,dtype", [(64, "int4"), (48, "int8"), (64, "int4r64"), (256, "int4")])
def test_hashed_forward_over_quantized_tables_equals_hashing_first(D, dtype):
    # hashing inside the quantised lookup: bit-identical to emb_hash_ids_tables + emb_bag_forward, row numbers
    # written out, and the pooled values those of the oracle
    rng = np.random.default_rng(970 + D + len(dtype))
    T, B = 3, 500
    Rs = [5000, 7, 20_000]
    salts = [11, 0, M64]
    codes = "int4" if dtype == "int4r64" else dtype
    src = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in Rs]
    qt = [oracle.quantize_rows(x, codes) for x in src]
    rb = emb.emb_row_bytes(D, dtype)
    qdev = []
    for q in qt:
        pad = np.zeros((q.shape[0], rb), np.uint8)
        pad[:, :q.shape[1]] = q
        qdev.append(H.dev(pad))
    lengths = rng.integers(0, 40, size=T * B).astype(np.int32)
    lengths[rng.random(T * B) < 0.15] = 0
    off, _ = oracle.lengths_to_offsets(lengths)
    nnz = int(off[-1])
    raw = rng.integers(0, 1 << 64, size=nnz, dtype=np.uint64)
    rows = np.concatenate([oracle.hash_ids(raw[off[t * B]:off[(t + 1) * B]], salts[t], Rs[t]) for t in range(T)])
    ts = emb.TableSet(qdev, D, dtype, salts=salts, device=torch.device(H.DEV))
    out1 = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    out2 = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    rows_d = torch.full((nnz,), -1, dtype=torch.int64, device=H.DEV)
    st = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_hashed(ts, H.dev(raw), H.dev(off), B, "mean", out1, rows_d, st)
    emb.emb_bag_forward(ts, H.dev(rows), H.dev(off), B, "mean", out2, st)
    torch.cuda.synchronize()
    assert st.item() == 0 and np.array_equal(rows_d.cpu().numpy(), rows) and torch.equal(out1, out2)
    ref, absum, _ = oracle.bag_forward(qt, codes, rows, off, B, "mean", D=D)
    H.assert_pooled_close(out1.cpu().numpy(), ref, absum, what="hashed quantised forward %s D=%d" % (dtype, D))
    # and from bag lengths, the offsets made on the way
    out3 = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    offs = torch.full((T * B + 1,), -9, dtype=torch.int64, device=H.DEV)
    rows_d.fill_(-1)
    scratch = torch.empty(emb.emb_offsets_scratch_bytes(T * B), dtype=torch.uint8, device=H.DEV)
    emb.emb_bag_forward_hashed_lengths(ts, H.dev(raw), H.dev(lengths), B, "mean", out3, offs, scratch, rows_d, st)
    torch.cuda.synchronize()
    assert st.item() == 0 and torch.equal(out3, out1) and np.array_equal(offs.cpu().numpy(), off)
    assert np.array_equal(rows_d.cpu().numpy(), rows)


def test_forward_quantized_grid_tables_are_bit_exact_and_empty_batch():
    # integer codes with scale 1 and integer bias: every partial sum is exact in fp32
    rng = np.random.default_rng(960)
    D, B, R = 64, 50, 300
    x = rng.integers(0, 16, size=(R, D)).astype(np.float32)
    x[:, 0], x[:, 1] = 0, 15
    x += rng.integers(-20, 20, size=(R, 1)).astype(np.float32)
    q = oracle.quantize_rows(x, "int4")
    lengths = rng.integers(0, 30, size=B).astype(np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    rows = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    ts = emb.TableSet([H.dev(q)], D, "int4", device=torch.device(H.DEV))
    out, st = H.gpu_forward(ts, rows, off, B, "sum")
    ref, _, _ = oracle.bag_forward([q], "int4", rows, off, B, "sum", D=D)
    assert st == 0 and np.array_equal(out.reshape(ref.shape), ref)
    out, st = H.gpu_forward(ts, np.zeros(0, np.int64), np.zeros(B + 1, np.int64), B, "mean")
    assert st == 0 and np.all(out == 0)


# ---------------------------------------------------------------------------
# backward + row-wise Adagrad
# ---------------------------------------------------------------------------
def _backward_case(rng, T, B, D, Rs, max_len, dtype, mode, hot=0.0, lr=0.01, eps=1e-8, steps=1):
    """Several training steps; before each one the device state is (re)loaded from the
    oracle's state, so the two sides start every step from identical tables."""
    tables, lengths, off, rows = H.random_case(rng, T, B, D, Rs, max_len, dtype, scale=0.01, hot_row_frac=hot)
    ref_tables = [t.copy() for t in tables]
    ref_acc = [np.zeros(R, dtype=np.float32) for R in Rs]
    bf = dtype == "bf16"
    base = np.concatenate([[0], np.cumsum(Rs)])
    for step in range(steps):
        dout = rng.standard_normal((T, B, D)).astype(np.float32)
        old = [H.as_f32(t).copy() for t in ref_tables]
        old_acc = [a.copy() for a in ref_acc]
        ts, w_dev, acc_dev = H.make_tableset(ref_tables, dtype, accum_np=ref_acc)
        g = H.gpu_backward(ts, rows, off, B, mode, dout, lr, eps, side=(step % 2 == 0))   # both ways
        r = oracle.bag_backward_rowwise_adagrad(ref_tables, ref_acc, dtype, rows, off, B, mode, dout, lr, eps)
        assert g["status"] == r["status"] == 0
        assert np.array_equal(g["unique_keys"], r["unique_keys"])          # bit-exact unique-row set
        assert np.array_equal(g["unique_counts"], r["unique_counts"])
        for t in range(T):
            wg = H.as_f32(H.host_table(w_dev[t]))
            ag = acc_dev[t].cpu().numpy()
            sel = (r["unique_keys"] >= base[t]) & (r["unique_keys"] < base[t + 1])
            touched = r["unique_keys"][sel] - base[t]
            H.assert_rows_close(wg[touched], H.as_f32(ref_tables[t])[touched], old[t][touched], lr,
                                H.EPS_BF16 if bf else H.EPS32, what="rows t=%d step=%d" % (t, step))
            H.assert_accum_close(ag[touched], ref_acc[t][touched], r["Gabs"][sel], what="accum t=%d" % t)
            assert np.all(ag[touched] >= old_acc[t][touched])              # accumulators are monotone
            mask = np.ones(Rs[t], dtype=bool)
            mask[touched] = False
            assert np.array_equal(wg[mask], old[t][mask])                  # untouched rows bit-identical
            assert np.array_equal(ag[mask], old_acc[t][mask])


BWD_SHAPES = [(4, "f32"), (16, "f32"), (32, "f32"), (64, "f32"), (128, "f32"), (48, "f32"), (320, "f32"),
              (2048, "f32"), (4096, "f32"), (32, "bf16"), (64, "bf16"), (8, "bf16"), (1040, "bf16"), (8192, "bf16")]


@pytest.mark.parametrize("D,dtype", BWD_SHAPES)
@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_backward_matches_oracle(D, dtype, mode):
    rng = np.random.default_rng(1000 + D + (dtype == "bf16") + 2 * (mode == "mean"))
    big = D > 256
    T, B = 3, (64 if big else 700)
    Rs = [40, 5, 64] if big else [3000, 11, 20_000]
    _backward_case(rng, T, B, D, Rs, 10 if big else 30, dtype, mode, steps=2)


@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_backward_hot_rows_take_the_workgroup_path(mode):
    # 30 % of all lookups hit row 0 of each table: segments of thousands of lookups
    rng = np.random.default_rng(41)
    _backward_case(rng, 2, 2000, 64, [50_000, 777], 25, "f32", mode, hot=0.3, steps=2)


@pytest.mark.parametrize("seed,D,dtype", [(0, 64, "f32"), (1, 64, "f32"), (2, 32, "bf16"), (3, 320, "f32")])
def test_backward_run_lengths_at_every_boundary(seed, D, dtype):
    # The update works on spans of 256 sorted records, looks 32 records ahead, and hands runs of more than
    # 32 records to another path that cuts them into 256-record chunks.  Here the multiplicities of the rows
    # are chosen around those sizes and shuffled, so that runs of every such length start, end and cross at
    # arbitrary places relative to the spans; lookups are dealt to bags at random, so every record carries a
    # different gradient.
    rng = np.random.default_rng(8000 + seed)
    lengths_pool = [1] * 40 + [2, 3, 5, 30, 31, 32, 33, 34, 35, 63, 64, 65, 96, 223, 224, 225, 255, 256, 257, 258, 288,
                               289, 511, 512, 513, 544, 1000, 2049]
    T, B = 2, 300
    Rs = [4000, 90_000]
    rows_parts, lens = [], []
    for t in range(T):
        runs = rng.choice(lengths_pool, size=260 if t == 0 else 500)
        ids = np.sort(rng.choice(Rs[t], size=runs.size, replace=False))
        recs = np.repeat(ids, runs)
        rng.shuffle(recs)                                             # order in the batch is arbitrary
        cuts = np.sort(rng.integers(0, recs.size + 1, size=B - 1))    # deal them to B bags, some empty
        lens.append(np.diff(np.concatenate([[0], cuts, [recs.size]])))
        rows_parts.append(recs)
    lengths = np.concatenate(lens).astype(np.int32)
    rows = np.concatenate(rows_parts).astype(np.int64)
    off, _ = oracle.lengths_to_offsets(lengths)
    bf = dtype == "bf16"
    tables = []
    for R in Rs:
        v = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
        tables.append(wl.f32_to_bf16_bits(v).reshape(R, D) if bf else v)
    base = np.concatenate([[0], np.cumsum(Rs)])
    for mode, side in (("sum", True), ("mean", False)):
        ref_tables = [t.copy() for t in tables]
        ref_acc = [np.full(R, 0.5, dtype=np.float32) for R in Rs]
        dout = rng.standard_normal((T, B, D)).astype(np.float32)
        ts, w_dev, acc_dev = H.make_tableset(ref_tables, dtype, accum_np=ref_acc)
        g = H.gpu_backward(ts, rows, off, B, mode, dout, 0.01, 1e-8, side=side)
        r = oracle.bag_backward_rowwise_adagrad(ref_tables, ref_acc, dtype, rows, off, B, mode, dout, 0.01, 1e-8)
        assert g["status"] == r["status"] == 0
        assert np.array_equal(g["unique_keys"], r["unique_keys"]) and np.array_equal(g["unique_counts"], r["unique_counts"])
        for t in range(T):
            wg = H.as_f32(H.host_table(w_dev[t]))
            ag = acc_dev[t].cpu().numpy()
            sel = (r["unique_keys"] >= base[t]) & (r["unique_keys"] < base[t + 1])
            touched = r["unique_keys"][sel] - base[t]
            H.assert_rows_close(wg[touched], H.as_f32(ref_tables[t])[touched], H.as_f32(tables[t])[touched], 0.01,
                                H.EPS_BF16 if bf else H.EPS32, what="rows t=%d %s" % (t, mode))
            H.assert_accum_close(ag[touched], ref_acc[t][touched], r["Gabs"][sel], what="accum t=%d %s" % (t, mode))
            mask = np.ones(Rs[t], dtype=bool)
            mask[touched] = False
            assert np.array_equal(wg[mask], H.as_f32(tables[t])[mask]) and (ag[mask] == 0.5).all()


def test_backward_many_tiles_and_64_bit_keys():
    # > 4096 * 8 lookups (several sort tiles, ragged tail); second case: key range past 2^32
    rng = np.random.default_rng(42)
    _backward_case(rng, 4, 3000, 32, [100_000, 9, 65_536, 1_000_003], 20, "f32", "mean")
    # 64-bit keys: a fake huge first table that is never looked up shifts row_base past 2^32
    D, B = 16, 500
    tables, lengths, off, rows = H.random_case(rng, 1, B, D, [5000], 15, scale=0.01)
    w = H.dev(tables[0])
    acc = torch.zeros(5000, dtype=torch.float32, device=H.DEV)
    dummy = torch.zeros((1, D), dtype=torch.float32, device=H.DEV)
    dacc = torch.zeros(1, dtype=torch.float32, device=H.DEV)
    big_rows = (1 << 32) + 12345
    ts = emb.TableSet([(int(dummy.data_ptr()), big_rows), w], D, "f32", accum=None, device=torch.device(H.DEV))
    ts.host["accum"][0] = int(dacc.data_ptr())
    ts.host["accum"][1] = int(acc.data_ptr())
    ts.dev = torch.from_numpy(ts.host.view(np.uint8).reshape(-1).copy()).to(H.DEV)
    off2 = np.concatenate([np.zeros(B, dtype=np.int64), off])          # table 0 has B empty bags
    dout = rng.standard_normal((2, B, D)).astype(np.float32)
    g = H.gpu_backward(ts, rows, off2, B, "sum", dout, 0.01, 1e-8)
    ref_t, ref_a = [tables[0].copy()], [np.zeros(5000, dtype=np.float32)]
    r = oracle.bag_backward_rowwise_adagrad(ref_t, ref_a, "f32", rows, off, B, "sum", dout[1:], 0.01, 1e-8)
    assert g["status"] == 0
    assert np.array_equal(g["unique_keys"], r["unique_keys"] + big_rows)
    assert np.array_equal(g["unique_counts"], r["unique_counts"])
    touched = r["unique_keys"]
    H.assert_rows_close(w.cpu().numpy()[touched], ref_t[0][touched], tables[0][touched], 0.01, what="64-bit keys")


def test_backward_sort_segments_small_empty_and_large_tables():
    # The sort works table by table.  Mix: tables without lookups (first, middle, last), a one-row
    # table, neighbours that touch the same row number, a table with several sort tiles of
    # lookups, and out-of-range rows in several tables (they sort to the end of their table's
    # records, i.e. between the runs of two tables).
    rng = np.random.default_rng(4242)
    D, B = 16, 7
    Rs = [9, 1, 5000, 5000, 3, 70_000, 12, 12, 400, 2, 33, 8]
    T = len(Rs)
    per_bag_max = [0, 4, 1, 1, 0, 4000, 30, 0, 0, 900, 5, 0]
    tables = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in Rs]
    lengths = np.concatenate([rng.integers(0, m + 1, size=B) for m in per_bag_max]).astype(np.int64)
    lengths[2 * B:4 * B] = 1                                   # tables 2 and 3: one lookup per bag, all of row 4999
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    parts = []
    for t in range(T):
        n = int(lengths[t * B:(t + 1) * B].sum())
        r = rng.integers(0, Rs[t], size=n).astype(np.int64)
        if t in (2, 3):
            r[:] = 4999
        if t in (1, 5, 10) and n:
            r[rng.integers(0, n, size=max(1, n // 50))] = Rs[t] + rng.integers(0, 3)
        parts.append(r)
    rows = np.concatenate(parts)
    assert off[6 * B] - off[5 * B] > 2 * 4096                  # table 5 spans several tiles
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    base = np.concatenate([[0], np.cumsum(Rs)])
    ts, w_dev, acc_dev = H.make_tableset(tables, "f32", with_accum=True)
    g = H.gpu_backward(ts, rows, off, B, "mean", dout, 0.01, 1e-8)
    ref_t, ref_a = [t.copy() for t in tables], [np.zeros(R, np.float32) for R in Rs]
    r = oracle.bag_backward_rowwise_adagrad(ref_t, ref_a, "f32", rows, off, B, "mean", dout, 0.01, 1e-8)
    assert g["status"] == r["status"] == emb.STATUS_BAD_INDEX
    assert np.array_equal(g["unique_keys"], r["unique_keys"])
    assert np.array_equal(g["unique_counts"], r["unique_counts"])
    for t in range(T):
        wg, ag = w_dev[t].cpu().numpy(), acc_dev[t].cpu().numpy()
        sel = (r["unique_keys"] >= base[t]) & (r["unique_keys"] < base[t + 1])
        touched = r["unique_keys"][sel] - base[t]
        H.assert_rows_close(wg[touched], ref_t[t][touched], tables[t][touched], 0.01, what="segments t=%d" % t)
        H.assert_accum_close(ag[touched], ref_a[t][touched], r["Gabs"][sel], what="segments accum t=%d" % t)
        mask = np.ones(Rs[t], dtype=bool)
        mask[touched] = False
        assert np.array_equal(wg[mask], tables[t][mask]) and np.all(ag[mask] == 0)
    # the same batch without the list of distinct rows: the update counts them itself
    ts, w_dev2, acc_dev2 = H.make_tableset(tables, "f32", with_accum=True)
    g2 = H.gpu_backward(ts, rows, off, B, "mean", dout, 0.01, 1e-8, want_unique=False)
    assert g2["U"] == len(r["unique_keys"])
    for t in range(T):
        assert np.array_equal(w_dev2[t].cpu().numpy(), w_dev[t].cpu().numpy())


def _check_backward_against_oracle(tables, Rs, rows, off, B, D, mode, dout, what, expect_status=0):
    T = len(Rs)
    base = np.concatenate([[0], np.cumsum(Rs)])
    ts, w_dev, acc_dev = H.make_tableset(tables, "f32", with_accum=True)
    g = H.gpu_backward(ts, rows, off, B, mode, dout, 0.01, 1e-8)
    ref_t, ref_a = [t.copy() for t in tables], [np.zeros(R, np.float32) for R in Rs]
    r = oracle.bag_backward_rowwise_adagrad(ref_t, ref_a, "f32", rows, off, B, mode, dout, 0.01, 1e-8)
    assert g["status"] == r["status"] == expect_status
    assert np.array_equal(g["unique_keys"], r["unique_keys"]), what
    assert np.array_equal(g["unique_counts"], r["unique_counts"]), what
    for t in range(T):
        sel = (r["unique_keys"] >= base[t]) & (r["unique_keys"] < base[t + 1])
        touched = r["unique_keys"][sel] - base[t]
        idx = torch.from_numpy(touched).to(H.DEV)
        H.assert_rows_close(w_dev[t][idx].cpu().numpy(), ref_t[t][touched], tables[t][touched], 0.01,
                            what="%s rows t=%d" % (what, t))
        H.assert_accum_close(acc_dev[t][idx].cpu().numpy(), ref_a[t][touched], r["Gabs"][sel],
                             what="%s accum t=%d" % (what, t))
        assert int((acc_dev[t] != 0).sum().item()) == int((ref_a[t] != 0).sum())      # nothing else was touched


def test_backward_sort_tables_of_very_different_key_widths():
    # Tables whose keys need different numbers of sort passes in one batch (the passes cover the widest):
    # table 0 (22-bit keys): one row with 30 000 lookups and one with 9 000 (runs that leave their span by
    #   dozens of spans; their ends are found from the noted run starts), the rest spread out;
    # table 1 (200 rows, one pass would do): one row with 10 000 lookups, and out-of-range rows (their marker
    #   sorts last inside the table);
    # table 2 (27-bit keys, four passes): rows spread over the whole table, a hot row, and the last row;
    # table 3: no lookups; table 4: a single lookup.
    rng = np.random.default_rng(777)
    D, B = 4, 64
    Rs = [3_000_000, 200, 70_000_000, 50, 1000]
    T = len(Rs)
    parts = []
    r0 = rng.integers(0, Rs[0], size=40_000)
    r0[rng.choice(40_000, size=9_000, replace=False)] = 1_234_567
    parts.append(np.concatenate([r0, np.full(30_000, 2_999_999)]))
    r1 = rng.integers(0, Rs[1], size=3_000)
    r1[:40] = [200, 201, -1, 1 << 33] * 10
    parts.append(np.concatenate([np.full(10_000, 77), r1]))
    r2 = rng.integers(0, Rs[2], size=50_000)
    r2[rng.choice(50_000, size=12_000, replace=False)] = 33_554_431
    r2[:5] = Rs[2] - 1
    parts.append(r2)
    parts.append(np.zeros(0, np.int64))
    parts.append(np.array([999]))
    lens = []
    for p in parts:
        rng.shuffle(p)
        cuts = np.sort(rng.integers(0, p.size + 1, size=B - 1))
        lens.append(np.diff(np.concatenate([[0], cuts, [p.size]])))
    lengths = np.concatenate(lens).astype(np.int64)
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rows = np.concatenate(parts).astype(np.int64)
    tables = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in Rs]
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    _check_backward_against_oracle(tables, Rs, rows, off, B, D, "sum", dout, "buckets", emb.STATUS_BAD_INDEX)


def test_backward_sort_one_table_of_many_tiles():
    # 1.2 M lookups of one table: a sort segment of 293 tiles (the scan over a table's tiles runs over more
    # than one workgroup's worth of them), with a row repeated 20 000 times among them.  A table this large
    # is sorted pass by pass (a counting launch and a scan for every pass).
    rng = np.random.default_rng(778)
    D, B, R = 4, 3000, 1_000_003
    lengths = np.full(B, 400, dtype=np.int64)
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rows = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    rows[rng.choice(rows.size, size=20_000, replace=False)] = 500_000
    tables = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32)]
    dout = rng.standard_normal((1, B, D)).astype(np.float32)
    _check_backward_against_oracle(tables, [R], rows, off, B, D, "mean", dout, "one table")


def test_backward_sort_one_large_table_among_small_ones():
    # Eight tables, 1.2 M of the 1.25 M lookups in one of them: the tables average few tiles, so the later
    # passes exchange their per-tile counts between workgroups, and in the large table (293 tiles) a tile's
    # walk back over the earlier tiles is long and meets tiles in every state.
    rng = np.random.default_rng(779)
    D, B, T = 4, 3000, 8
    Rs = [5000, 300, 1_000_003, 70_000, 9, 2_000_000, 65_536, 1000]
    lengths = np.zeros(T * B, dtype=np.int64)
    lengths[2 * B:3 * B] = 400
    for t in (0, 1, 3, 4, 5, 6, 7):
        lengths[t * B:(t + 1) * B] = rng.integers(0, 5, size=B)
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rows = np.concatenate([rng.integers(0, Rs[t], size=int(off[(t + 1) * B] - off[t * B])) for t in range(T)]).astype(np.int64)
    big = np.arange(int(off[2 * B]), int(off[3 * B]))
    rows[rng.choice(big, size=20_000, replace=False)] = 500_000
    tables = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in Rs]
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    _check_backward_against_oracle(tables, Rs, rows, off, B, D, "sum", dout, "one large table among small ones")


@pytest.mark.parametrize("T", [3, 20])
def test_backward_sort_more_than_a_thousand_tiles(T):
    # 4.5 M lookups are 1 100 sort tiles: the scan over the per-tile digit counts takes more than one round.
    # Three tables (366 tiles each) are sorted pass by pass, twenty tables (55 tiles each) by exchange.
    rng = np.random.default_rng(780 + T)
    D, R = 4, 100_003
    B = 4_500_000 // (T * 250)
    lengths = np.full(T * B, 250, dtype=np.int64)
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    rows = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    rows[rng.choice(rows.size, size=50_000, replace=False)] = 77       # a long run in whichever tables it falls
    tables = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for _ in range(T)]
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    _check_backward_against_oracle(tables, [R] * T, rows, off, B, D, "sum", dout, "more than a thousand tiles")


def test_backward_split_calls_on_two_streams_equal_the_single_call():
    # emb_bag_backward_sort on a second stream (while other work runs on the first), then
    # emb_bag_backward_update: bit-identical tables, accumulators and row lists.
    rng = np.random.default_rng(4343)
    T, B, D, Rs = 3, 1800, 64, [30_000, 500, 70_000]
    tables, lengths, off, rows = H.random_case(rng, T, B, D, Rs, 30, scale=0.01, hot_row_frac=0.1)
    rows = rows.copy()
    rows[[3, 40_000]] = [1 << 40, -1]                        # invalid rows travel through the split too
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    nnz = rows.size
    ts1, w1, a1 = H.make_tableset(tables, "f32", with_accum=True)
    g1 = H.gpu_backward(ts1, rows, off, B, "mean", dout, 0.01, 1e-8, side=False)
    ts2, w2, a2 = H.make_tableset(tables, "f32", with_accum=True)
    ws = torch.empty(emb.emb_bag_backward_workspace_bytes(T, B, nnz, ts2.total_rows, D, "f32"), dtype=torch.uint8,
                     device=H.DEV)
    uk = torch.full((nnz,), -7, dtype=torch.int64, device=H.DEV)
    uc = torch.full((nnz,), -7, dtype=torch.int32, device=H.DEV)
    nu = torch.full((1,), -7, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    rows_d, off_d, dout_d = H.dev(rows), H.dev(off), H.dev(dout)
    out = torch.empty((T, B, D), dtype=torch.float32, device=H.DEV)
    second = torch.cuda.Stream()
    ready, done = torch.cuda.Event(), torch.cuda.Event()
    torch.cuda.synchronize()
    main = torch.cuda.current_stream()
    ready.record(main)
    with torch.cuda.stream(second):
        second.wait_event(ready)
        emb.emb_bag_backward_sort(ts2, rows_d, off_d, B, "mean", ws, uk, uc, nu, status)
        done.record(second)
    emb.emb_bag_forward(ts2, rows_d, off_d, B, "mean", out, status)      # runs beside the sort
    main.wait_event(done)
    emb.emb_bag_backward_update(ts2, B, nnz, dout_d, 0.01, 1e-8, ws, nu, None, H.side_stream())
    torch.cuda.synchronize()
    U = int(nu.item())
    assert int(status.item()) == g1["status"] == emb.STATUS_BAD_INDEX
    assert U == g1["U"]
    assert np.array_equal(uk[:U].cpu().numpy(), g1["unique_keys"])
    assert np.array_equal(uc[:U].cpu().numpy(), g1["unique_counts"])
    for t in range(T):
        assert np.array_equal(w1[t].cpu().numpy(), w2[t].cpu().numpy())
        assert np.array_equal(a1[t].cpu().numpy(), a2[t].cpu().numpy())


@pytest.mark.parametrize("D,dtype", [(64, "f32"), (32, "bf16"), (320, "f32")])
def test_training_forward_equals_hashed_forward_plus_backward(D, dtype):
    # emb_bag_forward_train + sort_prepared + update against emb_bag_forward_hashed + the one-call
    # backward: pooled output, row numbers, tables, accumulators and row lists bit for bit; and
    # against the oracle within tolerance.
    rng = np.random.default_rng(4400 + D)
    T, B = 3, 900
    Rs = [20_000, 13, 70_001]
    salts = [5, 0, M64]
    tables, lengths, off, _ = H.random_case(rng, T, B, D, Rs, 25, dtype, scale=0.01)
    nnz = int(off[-1])
    raw = rng.integers(0, 1 << 64, size=nnz, dtype=np.uint64)
    raw[: nnz // 3] = raw[0]                                   # a hot ID: long runs in table 0
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    rows = np.concatenate([oracle.hash_ids(raw[off[t * B]:off[(t + 1) * B]], salts[t], Rs[t]) for t in range(T)])

    def fresh():
        w = [H.dev(t) for t in tables]
        acc = [torch.zeros(R, dtype=torch.float32, device=H.DEV) for R in Rs]
        return emb.TableSet(w, D, dtype, accum=acc, salts=salts, device=torch.device(H.DEV)), w, acc

    raw_d, off_d, dout_d = H.dev(raw), H.dev(off), H.dev(dout)
    # reference route on the device
    ts1, w1, a1 = fresh()
    out1 = torch.empty((T, B, D), dtype=torch.float32, device=H.DEV)
    rows1 = torch.empty(nnz, dtype=torch.int64, device=H.DEV)
    st1 = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_hashed(ts1, raw_d, off_d, B, "mean", out1, rows1, st1)
    g1 = H.gpu_backward(ts1, rows, off, B, "mean", dout, 0.01, 1e-8, side=False)
    # training route
    ts2, w2, a2 = fresh()
    ws = torch.empty(emb.emb_bag_backward_workspace_bytes(T, B, nnz, ts2.total_rows, D, dtype), dtype=torch.uint8,
                     device=H.DEV)
    out2 = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    rows2 = torch.full((nnz,), -1, dtype=torch.int64, device=H.DEV)
    uk = torch.full((nnz,), -7, dtype=torch.int64, device=H.DEV)
    uc = torch.full((nnz,), -7, dtype=torch.int32, device=H.DEV)
    nu = torch.full((1,), -7, dtype=torch.int64, device=H.DEV)
    st2 = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_train(ts2, raw_d, off_d, B, "mean", out2, ws, rows2, nu, st2)
    emb.emb_bag_backward_sort_prepared(ts2, B, nnz, ws, uk, uc, nu, st2)
    emb.emb_bag_backward_update(ts2, B, nnz, dout_d, 0.01, 1e-8, ws, nu, None, H.side_stream())
    torch.cuda.synchronize()
    assert st1.item() == 0 and st2.item() == 0 and g1["status"] == 0
    assert torch.equal(out1, out2) and torch.equal(rows1, rows2) and np.array_equal(rows2.cpu().numpy(), rows)
    U = int(nu.item())
    assert U == g1["U"] and np.array_equal(uk[:U].cpu().numpy(), g1["unique_keys"])
    assert np.array_equal(uc[:U].cpu().numpy(), g1["unique_counts"])
    for t in range(T):
        assert torch.equal(w1[t], w2[t]) and torch.equal(a1[t], a2[t])
    # and the oracle
    ref, absum, _ = oracle.bag_forward(tables, dtype, rows, off, B, "mean")
    H.assert_pooled_close(out2.cpu().numpy(), ref, absum, what="training forward")
    ref_t, ref_a = [t.copy() for t in tables], [np.zeros(R, np.float32) for R in Rs]
    r = oracle.bag_backward_rowwise_adagrad(ref_t, ref_a, dtype, rows, off, B, "mean", dout, 0.01, 1e-8)
    assert np.array_equal(uk[:U].cpu().numpy(), r["unique_keys"])
    base = np.concatenate([[0], np.cumsum(Rs)])
    for t in range(T):
        sel = (r["unique_keys"] >= base[t]) & (r["unique_keys"] < base[t + 1])
        touched = r["unique_keys"][sel] - base[t]
        H.assert_rows_close(H.as_f32(H.host_table(w2[t]))[touched], H.as_f32(ref_t[t])[touched],
                            H.as_f32(tables[t])[touched], 0.01, H.EPS_BF16 if dtype == "bf16" else H.EPS32,
                            what="training route rows t=%d" % t)
    # malformed offsets: the lookup flags them and the backward does nothing
    bad = off.copy()
    bad[7] = bad[8] + 1
    ts3, w3, a3 = fresh()
    st3 = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_train(ts3, raw_d, H.dev(bad), B, "mean", out2, ws, None, nu, st3)
    emb.emb_bag_backward_sort_prepared(ts3, B, nnz, ws, uk, uc, nu, st3)
    emb.emb_bag_backward_update(ts3, B, nnz, dout_d, 0.01, 1e-8, ws, nu, None, None)
    torch.cuda.synchronize()
    assert st3.item() & emb.STATUS_BAD_OFFSETS and int(nu.item()) == 0
    for t in range(T):
        assert np.array_equal(H.host_table(w3[t]), tables[t]) and float(a3[t].abs().sum()) == 0.0


@pytest.mark.parametrize("T,B,D,dtype", [(3, 5000, 32, "f32"), (2, 4096, 16, "bf16"), (1, 1, 64, "f32"), (5, 1639, 8, "f32")])
def test_training_forward_from_lengths_equals_offsets_then_training_forward(T, B, D, dtype):
    # emb_bag_forward_train_lengths against emb_lengths_to_offsets + emb_bag_forward_train: offsets (also against the
    # oracle), pooled output, row numbers, and after sort + update the tables, accumulators and row lists, bit for bit.
    # The bags span several tiles of 4096 lengths and the tables do not start on tile boundaries.
    rng = np.random.default_rng(4450 + T * B + D)
    Rs = [int(r) for r in rng.integers(50, 30_000, size=T)]
    salts = [int(x) for x in rng.integers(0, 1 << 62, size=T)]
    tables, lengths, off, _ = H.random_case(rng, T, B, D, Rs, 12, dtype, scale=0.01)
    lengths = lengths.copy()
    lengths[0] = 5
    if T * B > 4096:
        lengths[4090:4100] = 0                                 # empty bags across a tile boundary
        lengths[4096] = 77
    off, _ = oracle.lengths_to_offsets(lengths)
    nnz = int(off[-1])
    raw = rng.integers(0, 1 << 64, size=max(nnz, 1), dtype=np.uint64)[:nnz]
    raw[: nnz // 4] = raw[0]                                   # long runs
    dout = rng.standard_normal((T, B, D)).astype(np.float32)

    def fresh():
        w = [H.dev(t) for t in tables]
        acc = [torch.zeros(R, dtype=torch.float32, device=H.DEV) for R in Rs]
        return emb.TableSet(w, D, dtype, accum=acc, salts=salts, device=torch.device(H.DEV)), w, acc

    def route(from_lengths, lengths_np, nnz_arg):
        ts, w, a = fresh()
        ws = torch.full((emb.emb_bag_backward_workspace_bytes(T, B, nnz_arg, ts.total_rows, D, dtype),), 0xA5,
                        dtype=torch.uint8, device=H.DEV)
        out = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
        rows = torch.full((max(nnz_arg, 1),), -1, dtype=torch.int64, device=H.DEV)[:nnz_arg]
        offs = torch.full((T * B + 1,), -9, dtype=torch.int64, device=H.DEV)
        uk = torch.full((max(nnz_arg, 1),), -7, dtype=torch.int64, device=H.DEV)
        uc = torch.full((max(nnz_arg, 1),), -7, dtype=torch.int32, device=H.DEV)
        nu = torch.full((1,), -7, dtype=torch.int64, device=H.DEV)
        st = torch.zeros(1, dtype=torch.int32, device=H.DEV)
        raw_d = H.dev(raw[:nnz_arg]) if nnz_arg else torch.empty(0, dtype=torch.int64, device=H.DEV)
        len_d = H.dev(lengths_np)
        if from_lengths:
            emb.emb_bag_forward_train_lengths(ts, raw_d, len_d, B, "mean", out, offs, ws, rows, nu, st)
        else:
            emb.emb_lengths_to_offsets(len_d, offs, st)
            emb.emb_bag_forward_train(ts, raw_d, offs, B, "mean", out, ws, rows, nu, st)
        emb.emb_bag_backward_sort_prepared(ts, B, nnz_arg, ws, uk, uc, nu, st)
        emb.emb_bag_backward_update(ts, B, nnz_arg, H.dev(dout), 0.01, 1e-8, ws, nu, None, H.side_stream())
        torch.cuda.synchronize()
        return dict(out=out, rows=rows, offs=offs, uk=uk, uc=uc, U=int(nu.item()), st=int(st.item()), w=w, a=a)

    a, b = route(True, lengths, nnz), route(False, lengths, nnz)
    assert a["st"] == b["st"] == 0 and a["U"] == b["U"] > 0
    assert np.array_equal(a["offs"].cpu().numpy(), off) and torch.equal(a["offs"], b["offs"])
    assert torch.equal(a["out"], b["out"]) and torch.equal(a["rows"], b["rows"])
    assert torch.equal(a["uk"][:a["U"]], b["uk"][:b["U"]]) and torch.equal(a["uc"][:a["U"]], b["uc"][:b["U"]])
    for t in range(T):
        assert torch.equal(a["w"][t], b["w"][t]) and torch.equal(a["a"][t], b["a"][t])
    rows_ref = np.concatenate([oracle.hash_ids(raw[off[t * B]:off[(t + 1) * B]], salts[t], Rs[t]) for t in range(T)])
    assert np.array_equal(a["rows"].cpu().numpy(), rows_ref)
    ref, absum, _ = oracle.bag_forward(tables, dtype, rows_ref, off, B, "mean")
    H.assert_pooled_close(a["out"].cpu().numpy(), ref, absum, what="training forward from lengths")
    if T * B < 10:
        return
    # negative lengths count as 0 and are flagged, wherever they stand; both routes agree
    neg = lengths.copy()
    where = rng.choice(T * B, size=5, replace=False)
    neg[where] = -3
    off_n, st_n = oracle.lengths_to_offsets(neg)
    a, b = route(True, neg, int(off_n[-1])), route(False, neg, int(off_n[-1]))
    assert a["st"] == b["st"] == st_n == emb.STATUS_BAD_OFFSETS
    assert np.array_equal(a["offs"].cpu().numpy(), off_n) and torch.equal(a["out"], b["out"]) and a["U"] == b["U"]
    for t in range(T):
        assert torch.equal(a["w"][t], b["w"][t]) and torch.equal(a["a"][t], b["a"][t])
    # an nnz smaller than the sum of the lengths: flagged, the backward does nothing, as with offsets that end past nnz
    a, b = route(True, lengths, nnz - 1), route(False, lengths, nnz - 1)
    assert a["st"] & emb.STATUS_BAD_OFFSETS and b["st"] & emb.STATUS_BAD_OFFSETS and a["U"] == b["U"] == 0
    for t in range(T):
        assert np.array_equal(H.host_table(a["w"][t]), tables[t]) and float(a["a"][t].abs().sum()) == 0.0


@pytest.mark.parametrize("T,B,D,dtype,streaming", [(3, 5000, 32, "f32", False), (2, 4096, 16, "bf16", True),
                                                   (1, 1, 64, "f32", False), (7, 149_796, 4, "f32", False)])
def test_hashed_forward_from_lengths_equals_offsets_then_hashed_forward(T, B, D, dtype, streaming):
    # emb_bag_forward_hashed_lengths against emb_lengths_to_offsets + emb_bag_forward_hashed: offsets (also against
    # the oracle), pooled output and row numbers bit for bit; the last case has 256 tiles of lengths, the most a
    # workgroup scans
    rng = np.random.default_rng(4470 + T * B + D)
    Rs = [int(r) for r in rng.integers(50, 30_000, size=T)]
    salts = [int(x) for x in rng.integers(0, 1 << 62, size=T)]
    big = T * B > 100_000
    tables, lengths, off, _ = H.random_case(rng, T, B, D, Rs, 2 if big else 12, dtype, scale=0.01, empty_frac=0.5 if big else 0.15)
    lengths = lengths.copy()
    lengths[0] = 5
    if T * B > 4096:
        lengths[4090:4100] = 0
        lengths[4096] = 77
    off, _ = oracle.lengths_to_offsets(lengths)
    nnz = int(off[-1])
    raw = rng.integers(0, 1 << 64, size=nnz, dtype=np.uint64)
    ts = emb.TableSet([H.dev(t) for t in tables], D, dtype, salts=salts, device=torch.device(H.DEV))
    scratch = torch.full((emb.emb_offsets_scratch_bytes(T * B),), 0xA5, dtype=torch.uint8, device=H.DEV)

    def route(from_lengths, lengths_np, nnz_arg):
        out = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
        rows = torch.full((nnz_arg,), -1, dtype=torch.int64, device=H.DEV)
        offs = torch.full((T * B + 1,), -9, dtype=torch.int64, device=H.DEV)
        st = torch.zeros(1, dtype=torch.int32, device=H.DEV)
        if from_lengths:
            emb.emb_bag_forward_hashed_lengths(ts, H.dev(raw[:nnz_arg]), H.dev(lengths_np), B, "mean", out, offs, scratch,
                                               rows, st, streaming=streaming)
        else:
            emb.emb_lengths_to_offsets(H.dev(lengths_np), offs, st)
            emb.emb_bag_forward_hashed(ts, H.dev(raw[:nnz_arg]), offs, B, "mean", out, rows, st, streaming=streaming)
        torch.cuda.synchronize()
        return out, rows, offs, int(st.item())

    a, b = route(True, lengths, nnz), route(False, lengths, nnz)
    assert a[3] == b[3] == 0 and np.array_equal(a[2].cpu().numpy(), off) and torch.equal(a[2], b[2])
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    rows_ref = np.concatenate([oracle.hash_ids(raw[off[t * B]:off[(t + 1) * B]], salts[t], Rs[t]) for t in range(T)])
    assert np.array_equal(a[1].cpu().numpy(), rows_ref)
    ref, absum, _ = oracle.bag_forward(tables, dtype, rows_ref, off, B, "mean")
    H.assert_pooled_close(a[0].cpu().numpy(), ref, absum, what="hashed forward from lengths")
    if T * B < 10:
        return
    neg = lengths.copy()
    neg[rng.choice(T * B, size=5, replace=False)] = -3
    off_n, st_n = oracle.lengths_to_offsets(neg)
    a, b = route(True, neg, int(off_n[-1])), route(False, neg, int(off_n[-1]))
    assert a[3] == b[3] == st_n == emb.STATUS_BAD_OFFSETS and np.array_equal(a[2].cpu().numpy(), off_n)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    a, b = route(True, lengths, nnz - 1), route(False, lengths, nnz - 1)      # nnz below the sum of the lengths
    assert a[3] & emb.STATUS_BAD_OFFSETS and b[3] & emb.STATUS_BAD_OFFSETS and torch.equal(a[0], b[0])


def test_hashed_forward_from_lengths_argument_limits():
    ts = emb.TableSet([torch.zeros((5, 16), dtype=torch.float32, device=H.DEV)], 16, "f32", device=torch.device(H.DEV))
    offs = torch.full((1,), -9, dtype=torch.int64, device=H.DEV)
    st = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    empty_i64, empty_i32 = torch.empty(0, dtype=torch.int64, device=H.DEV), torch.empty(0, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_hashed_lengths(ts, empty_i64, empty_i32, 0, "sum", torch.empty((1, 0, 16), dtype=torch.float32,
                                       device=H.DEV), offs, torch.empty(8, dtype=torch.uint8, device=H.DEV), None, st)
    torch.cuda.synchronize()
    assert offs.item() == 0 and st.item() == 0
    B = 256 * 4096 + 1                                                # one bag more than 256 tiles of lengths
    with pytest.raises(emb.EmbError) as e:
        emb.emb_bag_forward_hashed_lengths(ts, empty_i64, torch.zeros(B, dtype=torch.int32, device=H.DEV), B, "sum",
                                           torch.empty((1, B, 16), dtype=torch.float32, device=H.DEV),
                                           torch.empty(B + 1, dtype=torch.int64, device=H.DEV),
                                           torch.empty(emb.emb_offsets_scratch_bytes(B), dtype=torch.uint8, device=H.DEV),
                                           None, st)
    assert e.value.code == -2
    with pytest.raises(emb.EmbError) as e:                           # scratch too small
        emb.emb_bag_forward_hashed_lengths(ts, empty_i64, torch.zeros(100, dtype=torch.int32, device=H.DEV), 100, "sum",
                                           torch.empty((1, 100, 16), dtype=torch.float32, device=H.DEV),
                                           torch.empty(101, dtype=torch.int64, device=H.DEV),
                                           torch.empty(100 * 8, dtype=torch.uint8, device=H.DEV), None, st)
    assert e.value.code == -1


def test_training_forward_from_lengths_with_more_than_a_thousand_tiles_of_bags():
    # 4.2 M bags are more than 1024 tiles of 4096 lengths: the prefix sums over the tile totals take several rounds
    rng = np.random.default_rng(4490)
    T, B, D, R = 1, 4096 * 1030 + 17, 4, 5000
    lengths = (rng.random(T * B) < 0.2).astype(np.int32)
    lengths[[0, 4096 * 1024 - 1, 4096 * 1024, T * B - 1]] = [3, 2, 5, 4]
    off, _ = oracle.lengths_to_offsets(lengths)
    nnz = int(off[-1])
    raw = rng.integers(0, 1 << 64, size=nnz, dtype=np.uint64)
    table = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
    w = H.dev(table)
    acc = torch.zeros(R, dtype=torch.float32, device=H.DEV)
    ts = emb.TableSet([w], D, "f32", accum=[acc], salts=[9], device=torch.device(H.DEV))
    ws = torch.empty(emb.emb_bag_backward_workspace_bytes(T, B, nnz, R, D, "f32"), dtype=torch.uint8, device=H.DEV)
    out = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    offs = torch.full((T * B + 1,), -9, dtype=torch.int64, device=H.DEV)
    nu = torch.zeros(1, dtype=torch.int64, device=H.DEV)
    st = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_train_lengths(ts, H.dev(raw), H.dev(lengths), B, "sum", out, offs, ws, None, nu, st)
    uk = torch.empty(nnz, dtype=torch.int64, device=H.DEV)
    emb.emb_bag_backward_sort_prepared(ts, B, nnz, ws, uk, None, nu, st)
    torch.cuda.synchronize()
    assert st.item() == 0 and np.array_equal(offs.cpu().numpy(), off)
    rows = oracle.hash_ids(raw, 9, R)
    ref, absum, _ = oracle.bag_forward([table], "f32", rows, off, B, "sum")
    H.assert_pooled_close(out.cpu().numpy(), ref, absum, what="lookup over 4.2 M bags")
    assert np.array_equal(uk[:int(nu.item())].cpu().numpy(), np.unique(rows))


def test_training_forward_from_lengths_without_bags():
    ts = emb.TableSet([torch.zeros((5, 16), dtype=torch.float32, device=H.DEV)], 16, "f32",
                      accum=[torch.zeros(5, dtype=torch.float32, device=H.DEV)], device=torch.device(H.DEV))
    ws = torch.empty(emb.emb_bag_backward_workspace_bytes(1, 0, 0, 5, 16, "f32"), dtype=torch.uint8, device=H.DEV)
    offs = torch.full((1,), -9, dtype=torch.int64, device=H.DEV)
    st = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_train_lengths(ts, torch.empty(0, dtype=torch.int64, device=H.DEV),
                                      torch.empty(0, dtype=torch.int32, device=H.DEV), 0, "sum",
                                      torch.empty((1, 0, 16), dtype=torch.float32, device=H.DEV), offs, ws, None, None, st)
    torch.cuda.synchronize()
    assert offs.item() == 0 and st.item() == 0


def test_many_tables_take_the_paths_without_lds_staging():
    # more tables than the kernels stage in LDS (table boundaries in the hashing kernel, the table
    # directory in the update kernels): 1100 small tables, 3 bags each
    rng = np.random.default_rng(4500)
    T, B, D = 1100, 3, 16
    Rs = [int(r) for r in rng.integers(1, 60, size=T)]
    tables = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in Rs]
    lengths = rng.integers(0, 12, size=T * B).astype(np.int32)
    lengths[3 * B:9 * B] = 0                                         # a stretch of tables without lookups
    off, _ = oracle.lengths_to_offsets(lengths)
    nnz = int(off[-1])
    raw = rng.integers(0, 1 << 64, size=nnz, dtype=np.uint64)
    salts = list(range(7, 7 + T))
    w = [H.dev(t) for t in tables]
    acc = [torch.zeros(R, dtype=torch.float32, device=H.DEV) for R in Rs]
    ts = emb.TableSet(w, D, "f32", accum=acc, salts=salts, device=torch.device(H.DEV))
    rows_dev = torch.full((nnz,), -5, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_hash_ids_tables(ts, H.dev(raw), H.dev(off), B, rows_dev, status)
    torch.cuda.synchronize()
    rows = np.concatenate([oracle.hash_ids(raw[off[t * B]:off[(t + 1) * B]], salts[t], Rs[t]) for t in range(T)])
    assert status.item() == 0 and np.array_equal(rows_dev.cpu().numpy(), rows)
    out, st = H.gpu_forward(ts, rows, off, B, "sum")
    ref, absum, _ = oracle.bag_forward(tables, "f32", rows, off, B, "sum")
    assert st == 0
    H.assert_pooled_close(out, ref, absum, what="many tables forward")
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    g = H.gpu_backward(ts, rows, off, B, "sum", dout, 0.01, 1e-8)
    ref_t, ref_a = [t.copy() for t in tables], [np.zeros(R, np.float32) for R in Rs]
    r = oracle.bag_backward_rowwise_adagrad(ref_t, ref_a, "f32", rows, off, B, "sum", dout, 0.01, 1e-8)
    assert g["status"] == 0 and np.array_equal(g["unique_keys"], r["unique_keys"])
    assert np.array_equal(g["unique_counts"], r["unique_counts"])
    for t in range(T):
        H.assert_rows_close(w[t].cpu().numpy(), ref_t[t], tables[t], 0.01, what="many tables rows t=%d" % t)


def test_backward_is_deterministic():
    rng = np.random.default_rng(43)
    T, B, D, Rs = 2, 1500, 64, [20_000, 300]
    tables, lengths, off, rows = H.random_case(rng, T, B, D, Rs, 30, scale=0.01, hot_row_frac=0.2)
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    results = []
    for rep in range(3):                      # the last repetition without the side stream
        ts, w_dev, acc_dev = H.make_tableset(tables, "f32", with_accum=True)
        H.gpu_backward(ts, rows, off, B, "mean", dout, 0.01, 1e-8, side=(rep < 2))
        results.append(([w.cpu().numpy() for w in w_dev], [a.cpu().numpy() for a in acc_dev]))
    for rep in (1, 2):
        for t in range(T):
            assert np.array_equal(results[0][0][t], results[rep][0][t])
            assert np.array_equal(results[0][1][t], results[rep][1][t])


def test_backward_bad_indices_skipped_and_bad_offsets_abort():
    rng = np.random.default_rng(44)
    T, B, D, Rs = 2, 100, 32, [500, 40]
    tables, lengths, off, rows = H.random_case(rng, T, B, D, Rs, 10, scale=0.01)
    rows = rows.copy()
    rows[[1, 5, 9]] = [500, -2, 1 << 50]
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    ts, w_dev, acc_dev = H.make_tableset(tables, "f32", with_accum=True)
    g = H.gpu_backward(ts, rows, off, B, "sum", dout, 0.01, 1e-8)
    ref_t, ref_a = [t.copy() for t in tables], [np.zeros(R, np.float32) for R in Rs]
    r = oracle.bag_backward_rowwise_adagrad(ref_t, ref_a, "f32", rows, off, B, "sum", dout, 0.01, 1e-8)
    assert g["status"] == r["status"] == emb.STATUS_BAD_INDEX
    assert np.array_equal(g["unique_keys"], r["unique_keys"]) and np.array_equal(g["unique_counts"], r["unique_counts"])
    for t in range(T):
        H.assert_rows_close(w_dev[t].cpu().numpy(), ref_t[t], tables[t], 0.01, what="bad idx rows")
    # malformed offsets: nothing may change
    for bad in (lambda o: o.__setitem__(0, 1), lambda o: o.__setitem__(-1, o[-1] - 1),
                lambda o: o.__setitem__(50, o[51] + 2)):
        off_b = off.copy()
        bad(off_b)
        ts, w_dev, acc_dev = H.make_tableset(tables, "f32", with_accum=True)
        g = H.gpu_backward(ts, rows, off_b, B, "sum", dout, 0.01, 1e-8)
        assert g["status"] & emb.STATUS_BAD_OFFSETS and g["U"] == 0
        for t in range(T):
            assert np.array_equal(w_dev[t].cpu().numpy(), tables[t])
            assert np.all(acc_dev[t].cpu().numpy() == 0)


def test_training_steps_with_the_join_deferred_into_the_next_lookup_equal_steps_that_join_at_once():
    # Five training steps over the same tables (hot IDs in every batch, so the long-run path on the side
    # stream has work and its rows are read again by the next step's lookup).  Route A joins the side
    # stream at the end of every backward; route B defers the join into the next step's lookup call and
    # alternates between two workspaces.  Pooled outputs of every step, final tables and accumulators bit
    # for bit; route A's final tables against the oracle run over the same five steps.
    rng = np.random.default_rng(4477)
    T, B, D = 3, 1200, 16
    Rs = [30_000, 17, 50_001]
    salts = [3, 9, 27]
    tables = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in Rs]
    steps = []
    for k in range(5):
        lengths = rng.integers(0, 30, size=T * B).astype(np.int32)
        off, _ = oracle.lengths_to_offsets(lengths)
        raw = rng.integers(0, 1 << 64, size=int(off[-1]), dtype=np.uint64)
        raw[rng.random(raw.size) < 0.3] = 12345                        # a hot ID in every table
        dout = rng.standard_normal((T, B, D)).astype(np.float32)
        steps.append((lengths, off, raw, dout))

    def run(defer):
        w = [H.dev(t) for t in tables]
        acc = [torch.zeros(R, dtype=torch.float32, device=H.DEV) for R in Rs]
        ts = emb.TableSet(w, D, "f32", accum=acc, salts=salts, device=torch.device(H.DEV))
        max_nnz = max(s[2].size for s in steps)
        nbytes = emb.emb_bag_backward_workspace_bytes(T, B, max_nnz, ts.total_rows, D, "f32")
        wss = [torch.empty(nbytes, dtype=torch.uint8, device=H.DEV) for _ in range(2 if defer else 1)]
        nus = [torch.zeros(1, dtype=torch.int64, device=H.DEV) for _ in wss]
        side = emb.SideStream(torch.device(H.DEV))
        side.defer_join = defer
        st = torch.zeros(1, dtype=torch.int32, device=H.DEV)
        outs, offs = [], []
        for k, (lengths, off, raw, dout) in enumerate(steps):
            ws, nu = wss[k % len(wss)], nus[k % len(wss)]
            out = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
            offs_out = torch.full((T * B + 1,), -1, dtype=torch.int64, device=H.DEV)
            emb.emb_bag_forward_train_lengths_after(ts, H.dev(raw), H.dev(lengths), B, "sum", out, offs_out, ws,
                                                    side if defer else None, None, nu, st)
            emb.emb_bag_backward_sort_prepared(ts, B, raw.size, ws, None, None, nu, st)
            emb.emb_bag_backward_update(ts, B, raw.size, H.dev(dout), 0.05, 1e-8, ws, nu, None, side)
            outs.append(out)
            offs.append(offs_out)
        if defer:
            side.join()
        torch.cuda.synchronize()
        assert st.item() == 0
        return outs, offs, w, acc

    outs_a, offs_a, w_a, acc_a = run(False)
    outs_b, offs_b, w_b, acc_b = run(True)
    for k in range(len(steps)):
        assert torch.equal(outs_a[k], outs_b[k]) and torch.equal(offs_a[k], offs_b[k]), k
        assert np.array_equal(offs_a[k].cpu().numpy(), steps[k][1])
    for t in range(T):
        assert torch.equal(w_a[t], w_b[t]) and torch.equal(acc_a[t], acc_b[t]), t
    ref_t, ref_a = [t.copy() for t in tables], [np.zeros(R, np.float32) for R in Rs]
    for lengths, off, raw, dout in steps:
        rows = np.concatenate([oracle.hash_ids(raw[off[t * B]:off[(t + 1) * B]], salts[t], Rs[t]) for t in range(T)])
        oracle.bag_backward_rowwise_adagrad(ref_t, ref_a, "f32", rows, off, B, "sum", dout, 0.05, 1e-8)
    for t in range(T):
        changed = np.flatnonzero((ref_t[t] != tables[t]).any(axis=1))
        assert changed.size > 0
        H.assert_rows_close(w_a[t].cpu().numpy()[changed], ref_t[t][changed], tables[t][changed], 0.05 * len(steps),
                            what="five steps t=%d" % t)
        assert np.array_equal(np.flatnonzero((w_a[t].cpu().numpy() != tables[t]).any(axis=1)), changed)


def test_backward_sort_wait_that_runs_out_abandons_the_backward_and_changes_nothing():
    # From the second pass on, the workgroups of a sort pass wait for each other's digit counts; the waits are
    # bounded.  With the bound at zero every wait fails at once (forced from the host; every kernel still runs
    # to its end): the status word says so, no row and no accumulator changes, and the same call with the
    # default bound afterwards gives the oracle's result.
    rng = np.random.default_rng(4471)
    T, B, D, Rs = 2, 700, 16, [70_000, 300]          # 14 000 lookups per table: several sort tiles, three passes
    tables, lengths, off, rows = H.random_case(rng, T, B, D, Rs, 20, scale=0.01)
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    ts, w_dev, acc_dev = H.make_tableset(tables, "f32", with_accum=True)
    emb.emb_debug_sort_poll_limit(0)
    try:
        g = H.gpu_backward(ts, rows, off, B, "sum", dout, 0.01, 1e-8)
    finally:
        emb.emb_debug_sort_poll_limit(-1)
    assert g["status"] == emb.STATUS_SORT_ABANDONED
    for t in range(T):
        assert np.array_equal(w_dev[t].cpu().numpy(), tables[t]) and np.all(acc_dev[t].cpu().numpy() == 0)
    _check_backward_against_oracle(tables, Rs, rows, off, B, D, "sum", dout, "after an abandoned sort")


def test_backward_empty_batch():
    tables = [np.ones((10, 16), dtype=np.float32)]
    ts, w_dev, acc_dev = H.make_tableset(tables, "f32", with_accum=True)
    g = H.gpu_backward(ts, np.zeros(0, np.int64), np.zeros(5, np.int64), 4, "sum",
                       np.ones((1, 4, 16), np.float32), 0.01, 1e-8)
    assert g["U"] == 0 and g["status"] == 0 and np.all(w_dev[0].cpu().numpy() == 1)


# ---------------------------------------------------------------------------
# cached (hybrid) forward
# ---------------------------------------------------------------------------
def _cached_case(table_np, dtype, hot, rows, off, B, mode, table_ptr=None, keep=None):
    R, D = table_np.shape
    tdev = H.dev(table_np) if table_ptr is None else None
    ptr = int(tdev.data_ptr()) if table_ptr is None else table_ptr
    index = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
    cache = torch.empty((max(hot.size, 1), D), dtype=torch.float32 if dtype == "f32" else torch.bfloat16,
                        device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_cache_build(ptr, R, D, dtype, H.dev(hot) if hot.size else torch.empty(0, dtype=torch.int64, device=H.DEV),
                        cache, index, status)
    out = torch.full((1, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    hm = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    emb.emb_bag_forward_cached(ptr, R, D, dtype, cache, index, hot.size, H.dev(rows), H.dev(off), B, mode, out, hm,
                               status)
    torch.cuda.synchronize()
    ref, absum, (hits, misses), rst = oracle.bag_forward_cached(table_np, dtype, hot, rows, off, B, mode)
    assert int(status.item()) == rst
    assert hm.cpu().tolist() == [hits, misses]                     # bit-exact hit/miss counts
    H.assert_pooled_close(out.cpu().numpy(), ref, absum, what="cached forward")
    if hot.size:                                                   # cached rows are byte copies
        assert np.array_equal(H.host_table(cache[:hot.size]), table_np[hot])
    return out.cpu().numpy()


@pytest.mark.parametrize("D,dtype", [(64, "f32"), (32, "bf16"), (16, "f32"), (320, "f32")])
def test_cached_forward_matches_oracle_and_plain_forward(D, dtype):
    rng = np.random.default_rng(50 + D)
    R, B = 10_007, 400
    tables, lengths, off, rows = H.random_case(rng, 1, B, D, [R], 40, dtype, scale=0.01, hot_row_frac=0.1)
    rows[:3] = [R - 1, 0, 63]
    ts, _, _ = H.make_tableset(tables, dtype)
    plain, _ = H.gpu_forward(ts, rows, off, B, "mean")
    for hot in (np.zeros(0, np.int64), np.arange(R, dtype=np.int64),
                np.sort(rng.permutation(R)[:R // 20]).astype(np.int64),
                np.array([0, 63, 64, 127, 128, R - 1], dtype=np.int64)):
        out = _cached_case(tables[0], dtype, hot, rows, off, B, "mean")
        assert np.array_equal(out, plain)                          # the cache is numerically invisible


def test_cached_forward_bad_hot_set_and_bad_index():
    rng = np.random.default_rng(60)
    R, D, B = 1000, 32, 50
    tables, lengths, off, rows = H.random_case(rng, 1, B, D, [R], 10, scale=0.01)
    rows = rows.copy()
    rows[2] = R + 5
    _cached_case(tables[0], "f32", np.arange(0, R, 3, dtype=np.int64), rows, off, B, "sum")
    index = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
    cache = torch.empty((3, D), dtype=torch.float32, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    for hot in ([5, 5, 9], [9, 5, 20], [1, 2, R]):
        status.zero_()
        emb.emb_cache_build(int(H.dev(tables[0]).data_ptr()), R, D, "f32", H.dev(np.array(hot, np.int64)), cache,
                            index, status)
        torch.cuda.synchronize()
        assert status.item() == emb.STATUS_BAD_HOT_SET


@pytest.mark.parametrize("dtype", ["int4", "int8"])
@pytest.mark.parametrize("D", [64, 48])
def test_cached_forward_over_quantized_table(dtype, D):
    # the table is quantised into pinned host memory by the device; cache and table hold packed rows
    rng = np.random.default_rng(1300 + D)
    R, B, K = 30_000, 900, 2000
    x = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
    packed = oracle.quantize_rows(x, dtype)
    rb = emb.emb_row_bytes(D, dtype)
    host = torch.empty((R, rb), dtype=torch.uint8, pin_memory=True)
    ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
    emb.emb_quantize_rows(H.dev(x), dtype, ptr)
    torch.cuda.synchronize()
    assert np.array_equal(host.numpy(), packed)                       # written over the link, bit-exact
    hot = np.sort(rng.choice(R, size=K, replace=False)).astype(np.int64)
    lengths = rng.integers(0, 40, size=B).astype(np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    rows = np.where(rng.random(int(off[-1])) < 0.8, rng.choice(hot, size=int(off[-1])),
                    rng.integers(0, R, size=int(off[-1]))).astype(np.int64)
    rows[[4, 9]] = [R, -3]
    index = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
    cache = torch.full((K, rb), 0xEE, dtype=torch.uint8, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_cache_build(ptr, R, D, dtype, H.dev(hot), cache, index, status)
    torch.cuda.synchronize()
    assert status.item() == 0 and np.array_equal(cache.cpu().numpy(), packed[hot])
    out = torch.full((1, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    hm = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    emb.emb_bag_forward_cached(ptr, R, D, dtype, cache, index, K, H.dev(rows), H.dev(off), B, "sum", out, hm, status)
    torch.cuda.synchronize()
    ref, absum, (hits, misses), st = oracle.bag_forward_cached(packed, dtype, hot, rows, off, B, "sum", D=D)
    assert int(status.item()) == st == emb.STATUS_BAD_INDEX
    assert hm.cpu().tolist() == [hits, misses] and hits > 0 and misses > 0
    H.assert_pooled_close(out.cpu().numpy(), ref, absum, what="cached quantised forward")
    # hashing inside the cached lookup: same bits and counts as hashing first
    raw = rng.integers(0, 1 << 64, size=rows.size, dtype=np.uint64)
    hrows = oracle.hash_ids(raw, 77, R)
    o1 = torch.empty_like(out)
    o2 = torch.empty_like(out)
    hm1 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    hm2 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    st2 = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_cached(ptr, R, D, dtype, cache, index, K, H.dev(hrows), H.dev(off), B, "mean", o1, hm1, st2)
    emb.emb_bag_forward_cached_hashed(ptr, R, D, dtype, cache, index, K, 77, H.dev(raw), H.dev(off), B, "mean", o2, hm2,
                                      st2)
    torch.cuda.synchronize()
    assert st2.item() == 0 and torch.equal(o1, o2) and torch.equal(hm1, hm2) and int(hm1.sum()) == rows.size
    # the cache is numerically invisible: the plain lookup over the same packed table gives the same bits
    ts = emb.TableSet([H.dev(packed)], D, dtype, device=torch.device(H.DEV))
    plain, _ = H.gpu_forward(ts, rows, off, B, "sum")
    assert np.array_equal(plain.reshape(1, B, D), out.cpu().numpy())


def test_cached_forward_reads_misses_from_pinned_host_memory():
    # the table lives in pinned (device-mapped) host memory; misses are read over PCIe
    rng = np.random.default_rng(61)
    R, D, B = 50_000, 64, 600
    host = torch.empty((R, D), dtype=torch.float32, pin_memory=True)
    ptr = emb.emb_host_device_pointer(int(host.data_ptr()))           # raises unless the memory is device-mapped
    emb.emb_table_fill(ptr, R, D, "f32", 99)                          # the GPU writes the host table
    torch.cuda.synchronize()
    table_np = wl.dense_table(99, R, D, "f32")                         # the oracle's copy comes from the host generator
    assert np.array_equal(host.numpy(), table_np)
    lengths = rng.integers(0, 60, size=B).astype(np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    rows = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    hot = np.sort(rng.permutation(R)[:R // 20]).astype(np.int64)
    _cached_case(table_np, "f32", hot, rows, off, B, "sum", table_ptr=ptr)


def _staged_case(table_np, packed_np, dtype, D, ptr, hot, batches, capacity, mode, salt=None):
    """Several batches staged in one call, then one pooled lookup per batch, against the oracle's cached lookup of
    each batch.  batches: list of (ids, off, B); ids are row numbers, or raw IDs when salt is given."""
    R = packed_np.shape[0]
    rb = emb.emb_row_bytes(D, dtype)
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16}.get(dtype, torch.uint8)
    row_shape = (rb,) if tdt == torch.uint8 else (D,)
    index = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
    cache = torch.empty((max(hot.size, 1),) + row_shape, dtype=tdt, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_cache_build(ptr, R, D, dtype, H.dev(hot), cache, index, status)
    ids_all = np.concatenate([b[0] for b in batches])
    stage = torch.full((max(capacity, 1),) + row_shape, 0, dtype=tdt, device=H.DEV)
    loc = torch.full((max(ids_all.size, 1),), -5, dtype=torch.int64, device=H.DEV)
    count = torch.zeros(1, dtype=torch.int64, device=H.DEV)
    emb.emb_cache_stage_misses(ptr, R, D, dtype, index, hot.size, H.dev(ids_all), stage, capacity, loc, count, status,
                               salt=salt)
    torch.cuda.synchronize()
    want_status = 0
    total_misses = 0
    at = 0
    for ids, off, B in batches:
        rows = ids if salt is None else oracle.hash_ids(ids, salt, R)
        out = torch.full((1, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
        hm = torch.zeros(2, dtype=torch.int64, device=H.DEV)
        emb.emb_bag_forward_staged(ptr, R, D, dtype, cache, hot.size, stage, capacity, loc[at:at + ids.size], H.dev(off), B,
                                   mode, out, hm, status)
        torch.cuda.synchronize()
        kw = {} if dtype in ("f32", "bf16") else {"D": D}
        ref, absum, (hits, misses), rst = oracle.bag_forward_cached(packed_np, dtype, hot, rows, off, B, mode, **kw)
        want_status |= rst
        total_misses += misses
        assert hm.cpu().tolist() == [hits, misses]                 # bit-exact hit / miss counts, batch by batch
        H.assert_pooled_close(out.cpu().numpy(), ref, absum, what="staged lookup")
        at += ids.size
    assert int(status.item()) == want_status
    assert int(count.item()) == total_misses                       # every missed lookup asked for a staging row
    # what the staging buffer holds: a byte copy of a table row for every staged lookup
    loc_np = loc[:ids_all.size].cpu().numpy()
    staged = (loc_np >= 0) & ((loc_np >> 62) & 1).astype(bool)
    slots = loc_np[staged] & ((1 << 61) - 1)
    assert slots.size == min(total_misses, capacity) and np.unique(slots).size == slots.size
    rows_all = ids_all if salt is None else oracle.hash_ids(ids_all, salt, R)
    got = H.host_table(stage)[slots] if slots.size else None
    if slots.size:
        assert np.array_equal(got, packed_np[rows_all[staged]])


@pytest.mark.parametrize("D,dtype", [(64, "f32"), (32, "bf16"), (320, "f32"), (64, "int4"), (48, "int8")])
def test_staged_misses_of_several_batches_match_the_cached_lookup(D, dtype):
    # the table lives in pinned host memory; three batches (one empty, one with out-of-range rows) are staged at once
    rng = np.random.default_rng(2100 + D)
    R = 40_000
    x = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
    if dtype == "f32":
        packed = x
    elif dtype == "bf16":
        packed = wl.f32_to_bf16_bits(x).reshape(R, D)
    else:
        packed = oracle.quantize_rows(x, dtype)
    host = torch.from_numpy(packed.view(np.int16) if dtype == "bf16" else packed).pin_memory()
    ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
    hot = np.sort(rng.choice(R, size=R // 10, replace=False)).astype(np.int64)
    batches = []
    for B, max_len in ((700, 40), (3, 0), (1500, 25)):
        lengths = rng.integers(0, max_len + 1, size=B).astype(np.int32)
        off, _ = oracle.lengths_to_offsets(lengths)
        n = int(off[-1])
        rows = np.where(rng.random(n) < 0.7, rng.choice(hot, size=n), rng.integers(0, R, size=n)).astype(np.int64)
        batches.append((rows, off, B))
    batches[2][0][[5, 77]] = [R + 3, -1]
    n_miss = sum(int((~np.isin(b[0], hot) & (b[0] >= 0) & (b[0] < R)).sum()) for b in batches)
    assert n_miss > 3000
    for capacity in (n_miss + 10, n_miss // 3, 0):                 # room for all; the buffer runs full; no buffer
        _staged_case(x, packed, dtype, D, ptr, hot, batches, capacity, "mean" if capacity else "sum")
    # raw IDs, hashed while they are staged
    raw_batches = [(rng.integers(0, 1 << 63, size=b[0].size, dtype=np.int64).view(np.uint64), b[1], b[2]) for b in batches]
    _staged_case(x, packed, dtype, D, ptr, hot, raw_batches, n_miss * 2, "sum", salt=4242)
    # no cache at all: every lookup is a miss and is staged
    _staged_case(x, packed, dtype, D, ptr, np.zeros(0, np.int64), batches[:1], batches[0][0].size, "sum")


def test_staged_lookup_rejects_locations_it_cannot_hold():
    # a location array that was not written by the staging pass for these buffers: flagged and skipped, never read
    R, D, B = 100, 16, 4
    t = torch.ones((R, D), dtype=torch.float32, device=H.DEV)
    cache = torch.ones((10, D), dtype=torch.float32, device=H.DEV)
    stage = torch.ones((5, D), dtype=torch.float32, device=H.DEV)
    loc = np.array([3, 10, (1 << 62) | 4, (1 << 62) | 5, (1 << 61) | 99, (1 << 61) | 100, -1, 9], dtype=np.int64)
    off = np.array([0, 2, 4, 6, 8], dtype=np.int64)
    out = torch.empty((1, B, D), dtype=torch.float32, device=H.DEV)
    hm = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_bag_forward_staged(int(t.data_ptr()), R, D, "f32", cache, 10, stage, 5, H.dev(loc), H.dev(off), B, "sum", out,
                               hm, status)
    torch.cuda.synchronize()
    assert status.item() == emb.STATUS_BAD_INDEX
    assert out.cpu().numpy()[0, :, 0].tolist() == [1.0, 1.0, 1.0, 1.0]      # one valid location per bag
    assert hm.cpu().tolist() == [2, 2]


# ---------------------------------------------------------------------------
# procedural table fill
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_table_fill_matches_the_host_generator(dtype):
    R, D = 70_001, 64
    w = torch.empty((R, D), dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device=H.DEV)
    emb.emb_table_fill(w, R, D, dtype, 20250805123)
    torch.cuda.synchronize()
    assert np.array_equal(H.host_table(w), wl.dense_table(20250805123, R, D, dtype))


# ---------------------------------------------------------------------------
# frequency-based cache policy: counters, exact top-k selection, refresh
# ---------------------------------------------------------------------------

def _freq_dev(freq_np):
    return torch.from_numpy(freq_np.view(np.int32).copy()).to(H.DEV)


def _freq_host(freq_dev):
    return freq_dev.cpu().numpy().view(np.uint32)


def test_cache_observe_counts_like_the_oracle():
    rng = np.random.default_rng(5000)
    R = 70_001
    freq = rng.integers(0, 9, size=R).astype(np.uint32)
    freq[11] = 0xFFFFFFFE                                             # wraps
    rows = np.minimum(rng.zipf(1.2, size=300_000) - 1, R - 1).astype(np.int64)
    rows[:2000] = 11
    rows[[5, 77]] = [-1, R]
    fd = _freq_dev(freq)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_cache_observe(R, H.dev(rows), fd, status)
    torch.cuda.synchronize()
    ref = freq.copy()
    assert oracle.cache_observe(ref, rows) == 2
    assert status.item() == emb.STATUS_BAD_INDEX and np.array_equal(_freq_host(fd), ref)
    # raw IDs: the row counted is the hashed one
    raw = rng.integers(0, 1 << 64, size=50_000, dtype=np.uint64)
    raw[:5000] = raw[0]
    status.zero_()
    emb.emb_cache_observe_hashed(R, 991, H.dev(raw), fd, status)
    emb.emb_cache_observe(R, H.dev(rows[:0]), fd, status)             # nothing to count
    torch.cuda.synchronize()
    assert oracle.cache_observe(ref, oracle.hash_ids(raw, 991, R)) == 0
    assert status.item() == 0 and np.array_equal(_freq_host(fd), ref)


def _select_case(freq, num_hot, shift):
    R = freq.size
    fd = _freq_dev(freq)
    ws = torch.empty(emb.emb_cache_select_workspace_bytes(R), dtype=torch.uint8, device=H.DEV)
    ws.fill_(0xA5)                                                    # contents must not matter
    hot = torch.full((max(num_hot, 1),), -9, dtype=torch.int64, device=H.DEV)
    info = torch.full((2,), -9, dtype=torch.int64, device=H.DEV)
    emb.emb_cache_select(fd, num_hot, shift, ws, hot, info)
    torch.cuda.synchronize()
    ref_f = freq.copy()
    ref_hot = oracle.cache_select(ref_f, num_hot, shift)
    what = "R=%d num_hot=%d shift=%d" % (R, num_hot, shift)
    assert np.array_equal(hot.cpu().numpy()[:num_hot], ref_hot), what
    assert np.array_equal(_freq_host(fd), ref_f), what
    if num_hot > 0:
        thr = int(freq[ref_hot].min())
        assert info.cpu().tolist() == [thr, int((freq[ref_hot] == thr).sum())], what
    else:
        assert info.cpu().tolist() == [-9, -9] and hot.cpu().tolist() == [-9]


@pytest.mark.parametrize("R", [1, 5, 4095, 4096, 4097, 100_003, 1_300_007])
def test_cache_select_is_the_exact_top_k(R):
    rng = np.random.default_rng(5100 + R % 97)
    dists = {
        "zeros": np.zeros(R, np.uint32),
        "all max": np.full(R, 0xFFFFFFFF, np.uint32),
        "few values": rng.integers(0, 3, size=R).astype(np.uint32),
        "zipf": np.minimum(rng.zipf(1.1, size=R), 0xFFFFFFFF).astype(np.uint32),
        "full range": rng.integers(0, 1 << 32, size=R, dtype=np.uint64).astype(np.uint32),
        "high digits only": (rng.integers(0, 4, size=R).astype(np.uint32) << 24),
    }
    shifts = iter([0, 1, 31, 3, 0, 8, 0, 2])
    for name, freq in dists.items():
        for num_hot in sorted({0, 1, R // 20, R // 2, R - 1 if R > 1 else 0, R}):
            if R > 200_000 and num_hot not in (R // 20, R):
                continue                                              # the oracle sorts every row: keep it short
            try:
                shift = next(shifts)
            except StopIteration:
                shifts = iter([0, 1, 31, 3, 0, 8, 0, 2])
                shift = next(shifts)
            _select_case(freq, num_hot, shift)


def test_cache_select_rejects_bad_arguments():
    R = 1000
    fd = torch.zeros(R, dtype=torch.int32, device=H.DEV)
    ws = torch.empty(emb.emb_cache_select_workspace_bytes(R), dtype=torch.uint8, device=H.DEV)
    hot = torch.empty(R + 1, dtype=torch.int64, device=H.DEV)
    for args in ((R + 1, 0), (-1, 0), (5, 32), (5, -1)):
        with pytest.raises(emb.EmbError) as e:
            emb.emb_cache_select(fd, args[0], args[1], ws, hot)
        assert e.value.code == -1
    with pytest.raises(emb.EmbError) as e:
        emb.emb_cache_select(fd, 5, 0, ws[:ws.numel() - 256], hot)
    assert e.value.code == -3
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", ["f32", "int4"])
def test_cache_rebuild_takes_kept_rows_from_the_old_cache(dtype):
    rng = np.random.default_rng(5200)
    R, D, B = 20_011, 64, 300
    x = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
    table = x if dtype == "f32" else oracle.quantize_rows(x, dtype)
    rb = emb.emb_row_bytes(D, dtype)
    tdev = H.dev(table)
    ptr = int(tdev.data_ptr())
    hot_a = np.sort(rng.choice(R, size=1500, replace=False)).astype(np.int64)
    hot_b = np.sort(np.concatenate([rng.choice(hot_a, size=900, replace=False),
                                    rng.choice(np.setdiff1d(np.arange(R), hot_a), size=800, replace=False)])).astype(np.int64)
    mk = (lambda n: torch.full((n, D), 7.0, dtype=torch.float32, device=H.DEV)) if dtype == "f32" else \
         (lambda n: torch.full((n, rb), 0xEE, dtype=torch.uint8, device=H.DEV))
    cache_a, cache_b = mk(hot_a.size), mk(hot_b.size)
    idx_a = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
    idx_b = torch.empty_like(idx_a)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    moved = torch.zeros(2, dtype=torch.int64, device=H.DEV)
    emb.emb_cache_build(ptr, R, D, dtype, H.dev(hot_a), cache_a, idx_a, status)
    torch.cuda.synchronize()
    # mark the old cache's copies (test only: a real table and its cache agree), so that where a row of the
    # new cache came from shows in its bytes
    marked = cache_a.clone()
    if dtype == "f32":
        marked += 1.0
    else:
        marked ^= 0xFF
    emb.emb_cache_rebuild(ptr, R, D, dtype, marked, idx_a, hot_a.size, H.dev(hot_b), cache_b, idx_b, moved, status)
    torch.cuda.synchronize()
    kept = np.isin(hot_b, hot_a)
    assert status.item() == 0 and moved.cpu().tolist() == [int(kept.sum()), int((~kept).sum())]
    assert np.array_equal(cache_a.cpu().numpy(), table[hot_a])
    got = cache_b.cpu().numpy()
    want = table[hot_b].copy()                                        # expected from the table alone
    want[kept] = (want[kept] + np.float32(1.0)) if dtype == "f32" else (want[kept] ^ np.uint8(0xFF))
    assert np.array_equal(got, want)
    # a refresh without marking gives exactly what a build from the table gives, index included
    emb.emb_cache_rebuild(ptr, R, D, dtype, cache_a, idx_a, hot_a.size, H.dev(hot_b), cache_b, idx_b, None, status)
    cache_c, idx_c = mk(hot_b.size), torch.empty_like(idx_a)
    emb.emb_cache_build(ptr, R, D, dtype, H.dev(hot_b), cache_c, idx_c, status)
    torch.cuda.synchronize()
    assert torch.equal(cache_b, cache_c) and torch.equal(idx_b, idx_c) and status.item() == 0
    # an empty old cache: everything comes from the table; old and new buffers must differ
    moved.zero_()
    emb.emb_cache_build(ptr, R, D, dtype, H.dev(hot_a[:0]), cache_a, idx_a, status)
    emb.emb_cache_rebuild(ptr, R, D, dtype, None, idx_a, 0, H.dev(hot_b), cache_b, idx_b, moved, status)
    torch.cuda.synchronize()
    assert moved.cpu().tolist() == [0, hot_b.size] and torch.equal(cache_b, cache_c)
    with pytest.raises(emb.EmbError):
        emb.emb_cache_rebuild(ptr, R, D, dtype, cache_b, idx_b, hot_b.size, H.dev(hot_b), cache_b, idx_c, None, status)
    with pytest.raises(emb.EmbError):
        emb.emb_cache_rebuild(ptr, R, D, dtype, cache_a, idx_b, hot_b.size, H.dev(hot_b), cache_b, idx_b, None, status)


def test_cache_policy_loop_matches_the_oracle_step_by_step():
    # a drifting Zipf stream of raw IDs: observe each batch, refresh every few batches; the hot set, the
    # counters, hits and misses and the pooled output follow the oracle's at every step
    from paper_2508_05700_amd import pipeline
    rng = np.random.default_rng(5300)
    R, D, B, Hn, salt = 40_009, 32, 200, 2000, 4242
    table = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
    tdev = H.dev(table)
    cache = pipeline.HotRowCache(int(tdev.data_ptr()), R, D, "f32", Hn, salt, torch.device(H.DEV), decay_shift=1)
    freq = np.zeros(R, np.uint32)
    hot = np.zeros(0, np.int64)
    out = torch.empty((1, B, D), dtype=torch.float32, device=H.DEV)
    perm = rng.permutation(1 << 20).astype(np.uint64)
    for step in range(12):
        if step == 6:
            perm = rng.permutation(1 << 20).astype(np.uint64)       # popularity moves to other IDs
        lengths = rng.integers(0, 60, size=B).astype(np.int32)
        off, _ = oracle.lengths_to_offsets(lengths)
        ranks = np.minimum(rng.zipf(1.15, size=int(off[-1])), (1 << 20) - 1)
        raw = perm[ranks] * np.uint64(0x9E3779B97F4A7C15)
        rows = oracle.hash_ids(raw, salt, R)
        cache.hit_miss.zero_()
        cache.forward_hashed(H.dev(raw), H.dev(off), B, "sum", out)
        cache.observe(H.dev(raw))
        ref, absum, (hits, misses), st = oracle.bag_forward_cached(table, "f32", hot, rows, off, B, "sum")
        assert oracle.cache_observe(freq, rows) == 0
        torch.cuda.synchronize()
        assert cache.hit_miss.cpu().tolist() == [hits, misses], step
        H.assert_pooled_close(out.cpu().numpy(), ref, absum, what="policy loop step %d" % step)
        if step % 3 == 2:
            old = hot
            cache.moved.zero_()
            cache.refresh()
            hot = oracle.cache_select(freq, Hn, 1)
            torch.cuda.synchronize()
            assert np.array_equal(cache.hot.cpu().numpy(), hot), step
            assert np.array_equal(_freq_host(cache.freq), freq), step
            kept = int(np.isin(hot, old).sum())
            assert cache.moved.cpu().tolist() == [kept, Hn - kept], step
            assert np.array_equal(cache.rows[cache.active].cpu().numpy(), table[hot])
    assert cache.status.item() == 0 and hits > misses                # the learnt set serves most lookups


# ---------------------------------------------------------------------------
# version-tagged table sets: a lookup returns (E, V), E wholly from version V
# ---------------------------------------------------------------------------

def _version_case(rng, T, B, D, dtype="f32"):
    Rs = {1: [900, 3000, 77], 2: [1200, 500, 4000]}                   # row counts differ between versions
    out = {}
    for v, rs in Rs.items():
        tabs = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in rs[:T]]
        if dtype in ("int8", "int4"):
            tabs = [oracle.quantize_rows(x, dtype) for x in tabs]
        w = [H.dev(t) for t in tabs]
        ts = emb.TableSet(w, D, dtype, salts=[11 * v + t for t in range(T)], device=torch.device(H.DEV))
        rec = torch.empty(emb.emb_version_record_bytes(T), dtype=torch.uint8, device=H.DEV)
        emb.emb_version_record_write(rec, ts, 100 + v)
        out[v] = {"np": tabs, "ts": ts, "rec": rec, "Rs": rs[:T], "salts": [11 * v + t for t in range(T)], "keep": w}
    return out


def _oracle_hashed(ver, D, raw, off, B, T, mode):
    rows = np.concatenate([oracle.hash_ids(raw[off[t * B]:off[(t + 1) * B]], ver["salts"][t], ver["Rs"][t])
                           for t in range(T)])
    return oracle.bag_forward(ver["np"], "f32", rows, off, B, mode)


def test_versioned_lookup_returns_the_latched_version_whatever_is_published_meanwhile():
    rng = np.random.default_rng(6000)
    T, B, D = 3, 120, 32
    vers = _version_case(rng, T, B, D)
    lengths = rng.integers(0, 30, size=T * B).astype(np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    raw = rng.integers(0, 1 << 64, size=int(off[-1]), dtype=np.uint64)
    raw_d, off_d = H.dev(raw), H.dev(off)
    handle = torch.zeros(1, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    latch = torch.empty(emb.emb_version_latch_bytes(T), dtype=torch.uint8, device=H.DEV)
    out = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)

    def lookup():
        emb.emb_version_latch(handle, T, latch, status)
        emb.emb_bag_forward_latched_hashed(latch, T, D, "f32", raw_d, off_d, B, "mean", out, status)
        torch.cuda.synchronize()
        return out.cpu().numpy(), int(emb.latched_version(latch).item())

    # nothing published: version 0, zeros, a status bit, no fault
    E, V = lookup()
    assert V == 0 and status.item() == emb.STATUS_NO_VERSION and not E.any()
    status.zero_()
    for v in (1, 2, 1):                                               # and back: a rollback is a publish too
        emb.emb_version_publish(handle, vers[v]["rec"])
        E, V = lookup()
        ref, absum, st = _oracle_hashed(vers[v], D, raw, off, B, T, "mean")
        assert V == 100 + v and status.item() == 0 == st
        H.assert_pooled_close(E, ref, absum, what="version %d" % v)
    # a latch taken under version 1 keeps serving version 1 after version 2 is published, on another stream,
    # before the lookup's own kernel runs
    other = torch.cuda.Stream(device=H.DEV)
    emb.emb_version_latch(handle, T, latch, status)
    latched = torch.cuda.Event()
    latched.record()
    with torch.cuda.stream(other):
        other.wait_event(latched)
        emb.emb_version_publish(handle, vers[2]["rec"])
        published = torch.cuda.Event()
        published.record()
    torch.cuda.current_stream().wait_event(published)
    emb.emb_bag_forward_latched_hashed(latch, T, D, "f32", raw_d, off_d, B, "mean", out, status)
    torch.cuda.synchronize()
    ref1, absum1, _ = _oracle_hashed(vers[1], D, raw, off, B, T, "mean")
    assert int(emb.latched_version(latch).item()) == 101
    H.assert_pooled_close(out.cpu().numpy(), ref1, absum1, what="latched before the publish")
    E, V = lookup()                                                   # the next lookup sees version 2
    ref2, absum2, _ = _oracle_hashed(vers[2], D, raw, off, B, T, "mean")
    assert V == 102
    H.assert_pooled_close(E, ref2, absum2, what="after the publish")
    # a record for another number of tables is refused by the latch, harmlessly
    rec1 = torch.empty(emb.emb_version_record_bytes(1), dtype=torch.uint8, device=H.DEV)
    ts1 = emb.TableSet([vers[1]["keep"][0]], D, "f32", salts=[5], device=torch.device(H.DEV))
    emb.emb_version_record_write(rec1, ts1, 55)
    emb.emb_version_publish(handle, rec1)
    E, V = lookup()
    assert V == 0 and status.item() == emb.STATUS_NO_VERSION and not E.any()


@pytest.mark.parametrize("dtype", ["f32", "int4"])
def test_versioned_lookup_by_row_number(dtype):
    rng = np.random.default_rng(6100)
    T, B, D = 2, 90, 64
    vers = _version_case(rng, T, B, D, dtype)
    lengths = rng.integers(0, 25, size=T * B).astype(np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    handle = torch.zeros(1, dtype=torch.int64, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    latch = torch.empty(emb.emb_version_latch_bytes(T), dtype=torch.uint8, device=H.DEV)
    out = torch.empty((T, B, D), dtype=torch.float32, device=H.DEV)
    for v in (2, 1):
        Rs = vers[v]["Rs"]
        rows = np.concatenate([rng.integers(0, Rs[t], size=int(off[(t + 1) * B] - off[t * B])) for t in range(T)]).astype(np.int64)
        emb.emb_version_publish(handle, vers[v]["rec"])
        emb.emb_version_latch(handle, T, latch, status)
        emb.emb_bag_forward_latched(latch, T, D, dtype, H.dev(rows), H.dev(off), B, "sum", out, status)
        torch.cuda.synchronize()
        ref, absum, st = oracle.bag_forward(vers[v]["np"], dtype, rows, off, B, "sum", D=D if dtype != "f32" else None)
        assert int(emb.latched_version(latch).item()) == 100 + v and status.item() == 0 == st
        H.assert_pooled_close(out.cpu().numpy(), ref, absum, what="rows, version %d" % v)
        # same bits as the plain lookup over that version's descriptors
        plain, _ = H.gpu_forward(vers[v]["ts"], rows, off, B, "sum")
        assert np.array_equal(out.cpu().numpy(), plain)


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("int4", 64)])
def test_versioned_lookup_over_hosted_tables_and_a_cache_refresh_as_one_switch(dtype, D):
    # Two versions of a hosted table set (tables in pinned host memory, HBM caches), version 2 with other
    # contents and row counts; and a third record that is version 2 again with REFRESHED caches (other hot
    # sets, other cache buffers).  A lookup latches one record and returns (E, V) computed from that record's
    # tables and caches only, whatever is published while it waits.
    rng = np.random.default_rng(6200 + D)
    T, B = 3, 150
    quant = dtype == "int4"
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)

    def make_version(rows_per_table, seed, hot_frac, salt0, tabs=None):
        hosts, packed, hots, entries = [], [], [], []
        for t, R in enumerate(rows_per_table):
            if tabs is None:
                x = (np.random.default_rng(seed + t).standard_normal((R, D)) * 0.01).astype(np.float32)
                tab = oracle.quantize_rows(x, dtype) if quant else x
            else:
                tab = tabs[t]
            host = torch.from_numpy(tab).pin_memory()
            ptr = emb.emb_host_device_pointer(int(host.data_ptr()))
            K = int(R * hot_frac)
            hot = np.sort(np.random.default_rng(seed + 100 + t).choice(R, size=K, replace=False)).astype(np.int64)
            cache = torch.zeros((max(K, 1), tab.shape[1]), dtype=torch.uint8 if quant else torch.float32, device=H.DEV)
            index = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
            emb.emb_cache_build(ptr, R, D, dtype, H.dev(hot), cache, index, status)
            hosts.append(host); packed.append(tab); hots.append(hot)
            entries.append((ptr, R, cache, index, K, salt0 + t))
        ct = emb.CachedTables(entries, D, dtype, device=torch.device(H.DEV))
        return {"ct": ct, "np": packed, "hots": hots, "Rs": list(rows_per_table), "salts": [salt0 + t for t in range(T)],
                "keep": hosts}

    v1 = make_version([5000, 900, 12_000], 1, 0.1, 40)
    v2 = make_version([7000, 2500, 3000], 2, 0.2, 50)
    v2r = make_version(v2["Rs"], 3, 0.5, 50, tabs=v2["np"])             # version 2's tables, refreshed caches
    recs = {}
    for name, ver, number in (("v1", v1, 101), ("v2", v2, 102), ("v2r", v2r, 102)):
        rec = torch.empty(emb.emb_version_hosted_record_bytes(T), dtype=torch.uint8, device=H.DEV)
        emb.emb_version_hosted_record_write(rec, ver["ct"], number)
        recs[name] = rec
    lengths = rng.integers(0, 30, size=T * B).astype(np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    raw = rng.integers(0, 1 << 64, size=int(off[-1]), dtype=np.uint64)
    raw_d, off_d = H.dev(raw), H.dev(off)
    handle = torch.zeros(1, dtype=torch.int64, device=H.DEV)
    latch = torch.empty(emb.emb_version_hosted_latch_bytes(T), dtype=torch.uint8, device=H.DEV)
    out = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
    hm = torch.zeros(2, dtype=torch.int64, device=H.DEV)

    def expect(ver):
        outs, hits, misses = [], 0, 0
        absums = []
        for t in range(T):
            s, e = int(off[t * B]), int(off[(t + 1) * B])
            rows = oracle.hash_ids(raw[s:e], ver["salts"][t], ver["Rs"][t])
            kw = {"D": D} if quant else {}
            ref, absum, (h, m), st = oracle.bag_forward_cached(ver["np"][t], dtype, ver["hots"][t], rows,
                                                               off[t * B:(t + 1) * B + 1] - s, B, "sum", **kw)
            assert st == 0
            outs.append(ref[0]); absums.append(absum[0]); hits += h; misses += m
        return np.stack(outs), np.stack(absums), [hits, misses]

    def lookup():
        hm.zero_()
        emb.emb_version_hosted_latch(handle, T, latch, status)
        emb.emb_bag_forward_cached_latched_hashed(latch, T, D, dtype, raw_d, off_d, B, "sum", out, hm, status)
        torch.cuda.synchronize()
        return out.cpu().numpy(), int(emb.latched_version(latch).item()), hm.cpu().tolist()

    E, V, counts = lookup()                                            # nothing published
    assert V == 0 and status.item() == emb.STATUS_NO_VERSION and not E.any()
    status.zero_()
    for name, ver, number in (("v1", v1, 101), ("v2", v2, 102), ("v2r", v2r, 102), ("v1", v1, 101)):
        emb.emb_version_publish(handle, recs[name])
        E, V, counts = lookup()
        ref, absum, want = expect(ver)
        assert V == number and status.item() == 0 and counts == want, name    # hit / miss counts of THAT record's caches
        H.assert_pooled_close(E, ref, absum, what="hosted " + name)
    # latched under version 1; version 2 with refreshed caches is published, on another stream, before the lookup runs
    other = torch.cuda.Stream(device=H.DEV)
    hm.zero_()
    emb.emb_version_hosted_latch(handle, T, latch, status)
    latched = torch.cuda.Event()
    latched.record()
    with torch.cuda.stream(other):
        other.wait_event(latched)
        emb.emb_version_publish(handle, recs["v2r"])
        published = torch.cuda.Event()
        published.record()
    torch.cuda.current_stream().wait_event(published)
    emb.emb_bag_forward_cached_latched_hashed(latch, T, D, dtype, raw_d, off_d, B, "sum", out, hm, status)
    torch.cuda.synchronize()
    ref1, absum1, want1 = expect(v1)
    assert int(emb.latched_version(latch).item()) == 101 and hm.cpu().tolist() == want1
    H.assert_pooled_close(out.cpu().numpy(), ref1, absum1, what="hosted, latched before the publish")
    E, V, counts = lookup()
    ref2, absum2, want2 = expect(v2r)
    assert V == 102 and counts == want2
    H.assert_pooled_close(E, ref2, absum2, what="hosted, after the publish")
    # a latch for hosted tables refuses a record of HBM tables, and the other way round, harmlessly
    w = [torch.zeros((10, D), dtype=torch.float32, device=H.DEV) for _ in range(T)]
    ts = emb.TableSet(w, D, "f32", device=torch.device(H.DEV))
    plain_rec = torch.empty(emb.emb_version_record_bytes(T), dtype=torch.uint8, device=H.DEV)
    emb.emb_version_record_write(plain_rec, ts, 7)
    emb.emb_version_publish(handle, plain_rec)
    E, V, counts = lookup()
    assert V == 0 and status.item() == emb.STATUS_NO_VERSION and not E.any()
    status.zero_()
    emb.emb_version_publish(handle, recs["v1"])
    platch = torch.empty(emb.emb_version_latch_bytes(T), dtype=torch.uint8, device=H.DEV)
    emb.emb_version_latch(handle, T, platch, status)
    torch.cuda.synchronize()
    assert int(emb.latched_version(platch).item()) == 0 and status.item() == emb.STATUS_NO_VERSION


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 32), ("int4", 64), ("int8", 48)])
def test_cached_forward_over_several_tables_in_one_launch(dtype, D):
    rng = np.random.default_rng(7000 + D)
    T, B = 5, 333
    Rs = [4001, 900, 20_000, 64, 7777]
    quant = dtype in ("int8", "int4")
    tabs, hots, entries, keep = [], [], [], []
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    for t, R in enumerate(Rs):
        x = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
        tab = oracle.quantize_rows(x, dtype) if quant else (wl.f32_to_bf16_bits(x).reshape(R, D) if dtype == "bf16" else x)
        K = [R // 10, 0, R // 3, R, 5][t]                             # an empty and a full cache among them
        hot = np.sort(rng.choice(R, size=K, replace=False)).astype(np.int64)
        tdev = H.dev(tab)
        width = tab.shape[1]
        cache = torch.zeros((max(K, 1), width), dtype=tdev.dtype, device=H.DEV)
        index = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
        emb.emb_cache_build(int(tdev.data_ptr()), R, D, dtype, H.dev(hot), cache, index, status)
        tabs.append(tab)
        hots.append(hot)
        keep.append(tdev)
        entries.append((int(tdev.data_ptr()), R, cache, index, K, 31 + t))
    ct = emb.CachedTables(entries, D, dtype, device=torch.device(H.DEV))
    lengths = rng.integers(0, 40, size=T * B).astype(np.int32)
    lengths[rng.random(T * B) < 0.1] = 0
    off, _ = oracle.lengths_to_offsets(lengths)
    seg = [(int(off[t * B]), int(off[(t + 1) * B])) for t in range(T)]
    rows = np.concatenate([np.where(rng.random(e - s) < 0.6, rng.choice(hots[t], size=e - s) if hots[t].size else 0,
                                    rng.integers(0, Rs[t], size=e - s)) for t, (s, e) in enumerate(seg)]).astype(np.int64)
    rows[[3, 11]] = [-1, Rs[0]]                                       # table 0: two bad rows
    raw = rng.integers(0, 1 << 64, size=rows.size, dtype=np.uint64)
    for hashed in (False, True):
        ids = raw if hashed else rows
        out = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
        hm = torch.zeros(2, dtype=torch.int64, device=H.DEV)
        status.zero_()
        if hashed:
            emb.emb_bag_forward_cached_tables_hashed(ct, H.dev(raw), H.dev(off), B, "mean", out, hm, status)
        else:
            emb.emb_bag_forward_cached_tables(ct, H.dev(rows), H.dev(off), B, "mean", out, hm, status)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        hits = misses = 0
        st_all = 0
        for t, (s, e) in enumerate(seg):
            r = oracle.hash_ids(raw[s:e], 31 + t, Rs[t]) if hashed else rows[s:e]
            o = off[t * B:(t + 1) * B + 1] - off[t * B]
            ref, absum, (h, m), st = oracle.bag_forward_cached(tabs[t], dtype, hots[t], r, o, B, "mean",
                                                               D=D if quant else None)
            H.assert_pooled_close(got[t], ref[0], absum[0], eps=H.EPS32, what="cached tables t=%d hashed=%s" % (t, hashed))
            hits, misses, st_all = hits + h, misses + m, st_all | st
            # and the same bits as the single-table call
            one = torch.empty((1, B, D), dtype=torch.float32, device=H.DEV)
            ptr, R, cache, index, K, salt = entries[t]
            emb.emb_bag_forward_cached(ptr, R, D, dtype, cache, index, K, H.dev(r), H.dev(o), B, "mean", one)
            torch.cuda.synchronize()
            assert np.array_equal(one.cpu().numpy()[0], got[t])
        assert hm.cpu().tolist() == [hits, misses] and int(status.item()) == st_all
        assert st_all == (0 if hashed else emb.STATUS_BAD_INDEX)
        if hashed:
            # the same from the bag lengths: offsets written, same bits, same counts
            o2 = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
            hm2 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
            off2 = torch.full((T * B + 1,), -1, dtype=torch.int64, device=H.DEV)
            scratch = torch.empty(emb.emb_offsets_scratch_bytes(T * B), dtype=torch.uint8, device=H.DEV)
            emb.emb_bag_forward_cached_tables_hashed_lengths(ct, H.dev(raw), H.dev(lengths), B, "mean", o2, off2, scratch,
                                                             hm2, status)
            torch.cuda.synchronize()
            assert np.array_equal(off2.cpu().numpy(), off) and torch.equal(o2, out) and torch.equal(hm2, hm)
            assert int(status.item()) == st_all


@pytest.mark.parametrize("dtype,D,T,B", [("f32", 16, 3, 100_000), ("int4", 64, 1, 270_000), ("bf16", 32, 2, 2500)])
def test_cached_forward_from_lengths_equals_offsets_then_cached_forward(dtype, D, T, B):
    # 1, 66 and 74 tiles of lengths: the wavefront and the workgroup form of the prefix over tile totals;
    # the single-table and the multi-table call; offsets against the oracle, pooled output against the
    # (oracle-checked) calls that take offsets
    rng = np.random.default_rng(7100 + D + T)
    R, K = 5000, 700
    quant = dtype in ("int8", "int4")
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    entries, keep = [], []
    for t in range(T):
        x = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
        tab = oracle.quantize_rows(x, dtype) if quant else (wl.f32_to_bf16_bits(x).reshape(R, D) if dtype == "bf16" else x)
        hot = np.sort(rng.choice(R, size=K, replace=False)).astype(np.int64)
        tdev = H.dev(tab)
        cache = torch.zeros((K, tab.shape[1]), dtype=tdev.dtype, device=H.DEV)
        index = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
        emb.emb_cache_build(int(tdev.data_ptr()), R, D, dtype, H.dev(hot), cache, index, status)
        keep.append(tdev)
        entries.append((int(tdev.data_ptr()), R, cache, index, K, 900 + t))
    n = T * B
    lengths = (rng.random(n) < 0.3).astype(np.int32) * rng.integers(1, 6, size=n).astype(np.int32)
    lengths[[0, n - 1]] = [0, 3]
    off, _ = oracle.lengths_to_offsets(lengths)
    raw = rng.integers(0, 1 << 64, size=int(off[-1]), dtype=np.uint64)
    scratch = torch.empty(emb.emb_offsets_scratch_bytes(n), dtype=torch.uint8, device=H.DEV)
    for mode in ("sum", "mean"):
        want = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
        got = torch.full((T, B, D), float("nan"), dtype=torch.float32, device=H.DEV)
        hm1 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
        hm2 = torch.zeros(2, dtype=torch.int64, device=H.DEV)
        off2 = torch.full((n + 1,), -1, dtype=torch.int64, device=H.DEV)
        if T == 1:
            ptr, _, cache, index, _, salt = entries[0]
            emb.emb_bag_forward_cached_hashed(ptr, R, D, dtype, cache, index, K, salt, H.dev(raw), H.dev(off), B, mode,
                                              want, hm1, status)
            emb.emb_bag_forward_cached_hashed_lengths(ptr, R, D, dtype, cache, index, K, salt, H.dev(raw),
                                                      H.dev(lengths), B, mode, got, off2, scratch, hm2, status)
        else:
            ct = emb.CachedTables(entries, D, dtype, device=torch.device(H.DEV))
            emb.emb_bag_forward_cached_tables_hashed(ct, H.dev(raw), H.dev(off), B, mode, want, hm1, status)
            emb.emb_bag_forward_cached_tables_hashed_lengths(ct, H.dev(raw), H.dev(lengths), B, mode, got, off2, scratch,
                                                             hm2, status)
        torch.cuda.synchronize()
        assert status.item() == 0 and np.array_equal(off2.cpu().numpy(), off)
        assert torch.equal(got, want) and torch.equal(hm1, hm2) and int(hm1.sum()) == raw.size


def test_cached_forward_from_lengths_argument_limits():
    D, R, K = 16, 100, 10
    tab = torch.zeros((R, D), dtype=torch.float32, device=H.DEV)
    cache = torch.zeros((K, D), dtype=torch.float32, device=H.DEV)
    index = torch.empty(emb.emb_cache_index_bytes(R), dtype=torch.uint8, device=H.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    emb.emb_cache_build(int(tab.data_ptr()), R, D, "f32", H.dev(np.arange(K, dtype=np.int64)), cache, index, status)
    ct = emb.CachedTables([(int(tab.data_ptr()), R, cache, index, K, 1)], D, "f32", device=torch.device(H.DEV))
    raw = torch.zeros(0, dtype=torch.int64, device=H.DEV)
    # no bags: the single offset is written, nothing else is touched
    off = torch.full((1,), -1, dtype=torch.int64, device=H.DEV)
    none = torch.zeros(0, dtype=torch.uint8, device=H.DEV)
    emb.emb_bag_forward_cached_hashed_lengths(int(tab.data_ptr()), R, D, "f32", cache, index, K, 1, raw,
                                              torch.zeros(0, dtype=torch.int32, device=H.DEV), 0, "sum",
                                              torch.zeros(0, dtype=torch.float32, device=H.DEV), off, none, None, status)
    torch.cuda.synchronize()
    assert off.item() == 0
    off.fill_(-1)
    emb.emb_bag_forward_cached_tables_hashed_lengths(ct, raw, torch.zeros(0, dtype=torch.int32, device=H.DEV), 0, "sum",
                                                     torch.zeros(0, dtype=torch.float32, device=H.DEV), off, none, None,
                                                     status)
    torch.cuda.synchronize()
    assert off.item() == 0 and status.item() == 0
    # scratch too small; too many bags
    B = 5000
    lengths = torch.zeros(B, dtype=torch.int32, device=H.DEV)
    out = torch.zeros((B, D), dtype=torch.float32, device=H.DEV)
    offs = torch.zeros(B + 1, dtype=torch.int64, device=H.DEV)
    small = torch.empty(emb.emb_offsets_scratch_bytes(B) - 8, dtype=torch.uint8, device=H.DEV)
    with pytest.raises(emb.EmbError) as ei:
        emb.emb_bag_forward_cached_hashed_lengths(int(tab.data_ptr()), R, D, "f32", cache, index, K, 1, raw, lengths, B,
                                                  "sum", out, offs, small, None, status)
    assert ei.value.code == -1
    with pytest.raises(emb.EmbError) as ei:
        emb.emb_bag_forward_cached_tables_hashed_lengths(ct, raw, lengths, B, "sum", out, offs, small, None, status)
    assert ei.value.code == -1
    big = (1 << 20) + 1
    lengths = torch.zeros(big, dtype=torch.int32, device=H.DEV)
    out = torch.zeros((big, D), dtype=torch.float32, device=H.DEV)
    offs = torch.zeros(big + 1, dtype=torch.int64, device=H.DEV)
    scratch = torch.empty(emb.emb_offsets_scratch_bytes(big), dtype=torch.uint8, device=H.DEV)
    with pytest.raises(emb.EmbError) as ei:
        emb.emb_bag_forward_cached_hashed_lengths(int(tab.data_ptr()), R, D, "f32", cache, index, K, 1, raw, lengths, big,
                                                  "sum", out, offs, scratch, None, status)
    assert ei.value.code == -2


def test_hosted_table_set_with_policy_refresh_matches_the_oracle():
    # two hosted tables, caches chosen by the policy, one launch per lookup; after each refresh the
    # descriptor array names the new buffers
    from paper_2508_05700_amd import pipeline
    rng = np.random.default_rng(7100)
    T, B, D = 2, 150, 32
    Rs, Ks, salts = [9001, 30_011], [300, 1500], [5, 6]
    tabs = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in Rs]
    tdev = [H.dev(x) for x in tabs]
    caches = [pipeline.HotRowCache(int(tdev[t].data_ptr()), Rs[t], D, "f32", Ks[t], salts[t], torch.device(H.DEV))
              for t in range(T)]
    hs = pipeline.HostedTableSet(caches, torch.device(H.DEV))
    freq = [np.zeros(R, np.uint32) for R in Rs]
    hots = [np.zeros(0, np.int64) for _ in Rs]
    out = torch.empty((T, B, D), dtype=torch.float32, device=H.DEV)
    out_v = torch.empty((T, B, D), dtype=torch.float32, device=H.DEV)
    version = 1
    hs.publish(version)                                               # the same set behind a version handle
    for step in range(6):
        lengths = rng.integers(0, 50, size=T * B).astype(np.int32)
        off, _ = oracle.lengths_to_offsets(lengths)
        raw = (np.minimum(rng.zipf(1.2, size=int(off[-1])), 1 << 20).astype(np.uint64)) * np.uint64(0x9E3779B97F4A7C15)
        hs.hit_miss.zero_()
        got_version = hs.forward_latched_hashed(H.dev(raw), H.dev(off), B, "sum", out_v)
        torch.cuda.synchronize()
        counts_v = hs.hit_miss.cpu().tolist()
        assert int(got_version.item()) == version
        hs.hit_miss.zero_()
        hs.forward_hashed(H.dev(raw), H.dev(off), B, "sum", out)
        hs.observe(H.dev(raw), off, B)
        torch.cuda.synchronize()
        assert torch.equal(out, out_v) and counts_v == hs.hit_miss.cpu().tolist()   # same caches, same bits
        got = out.cpu().numpy()
        hits = misses = 0
        for t in range(T):
            s, e = int(off[t * B]), int(off[(t + 1) * B])
            rows = oracle.hash_ids(raw[s:e], salts[t], Rs[t])
            ref, absum, (h, m), st = oracle.bag_forward_cached(tabs[t], "f32", hots[t], rows,
                                                               off[t * B:(t + 1) * B + 1] - s, B, "sum")
            H.assert_pooled_close(got[t], ref[0], absum[0], what="hosted set step %d table %d" % (step, t))
            assert oracle.cache_observe(freq[t], rows) == 0 and st == 0
            hits, misses = hits + h, misses + m
        assert hs.hit_miss.cpu().tolist() == [hits, misses], step
        if step % 2 == 1:
            hs.refresh()
            version += 1
            hs.publish(version)                                       # refreshed caches become current in one switch
            torch.cuda.synchronize()
            for t in range(T):
                hots[t] = oracle.cache_select(freq[t], Ks[t], 1)
                assert np.array_equal(caches[t].hot[:Ks[t]].cpu().numpy(), hots[t])
    assert hs.status.item() == 0 and hits > misses


def test_checksum_matches_the_oracle_and_sees_a_single_changed_bit():
    rng = np.random.default_rng(7200)
    out = torch.full((1,), -1, dtype=torch.int64, device=H.DEV)
    for n_words in (0, 4, 1024, 4 * 999_983, 4 * 3_000_001):
        w = rng.integers(0, 1 << 32, size=n_words, dtype=np.uint64).astype(np.uint32)
        d = torch.from_numpy(w.view(np.int32).copy()).to(H.DEV)
        emb.emb_checksum(d, out)
        torch.cuda.synchronize()
        assert int(out.item()) % (1 << 64) == oracle.checksum(w), n_words
    # a table as the backward leaves it: only the touched rows differ, and the checksum of the rest says so
    T, B, D = 1, 64, 32
    tables, lengths, off, rows = H.random_case(rng, T, B, D, [5000], 12, scale=0.01)
    ts, wdev, acc = H.make_tableset(tables, "f32", with_accum=True)
    before = wdev[0].clone()
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    g = H.gpu_backward(ts, rows, off, B, "sum", dout, 0.01, 1e-8)
    assert g["status"] == 0
    untouched = np.setdiff1d(np.arange(5000), np.unique(rows))        # one table: keys are row numbers
    a = torch.zeros(1, dtype=torch.int64, device=H.DEV)
    b = torch.zeros(1, dtype=torch.int64, device=H.DEV)
    idx = torch.from_numpy(untouched).to(H.DEV)
    emb.emb_checksum(before[idx].contiguous(), a)
    emb.emb_checksum(wdev[0][idx].contiguous(), b)
    torch.cuda.synchronize()
    assert a.item() == b.item() and a.item() % (1 << 64) == oracle.checksum(np.ascontiguousarray(tables[0][untouched]))
    flipped = wdev[0][idx].contiguous()
    flipped.view(torch.int32)[1234, 7] ^= 1 << 20
    emb.emb_checksum(flipped, b)
    torch.cuda.synchronize()
    assert a.item() != b.item()


# ---------------------------------------------------------------------------
# the calls only enqueue kernels: a caller can capture them in a HIP graph
# ---------------------------------------------------------------------------

def _graph_inputs(rng, T, B, max_len, Rs):
    lengths = rng.integers(0, max_len + 1, size=T * B).astype(np.int32)
    nnz = int(lengths.sum())
    raw = rng.integers(0, 1 << 64, size=nnz, dtype=np.uint64)
    return lengths, raw


@pytest.mark.parametrize("side,from_lengths", [(False, False), (True, False), (True, True)])
def test_a_captured_training_step_replays_like_eager_calls(side, from_lengths):
    # offsets + training lookup + sort + update captured once into a graph, then replayed on new inputs
    # written into the same buffers (the number of lookups is part of the captured arguments, so every batch
    # here has the same total); each replay is compared with the oracle, with eager work and
    # synchronisations between the replays.
    rng = np.random.default_rng(9000 + side + 2 * from_lengths)
    T, B, D = 3, 400, 64
    Rs = [5000, 300, 20_000]
    tables = [(rng.standard_normal((R, D)) * 0.01).astype(np.float32) for R in Rs]
    ref_tables = [t.copy() for t in tables]
    ref_acc = [np.zeros(R, np.float32) for R in Rs]
    ts, w_dev, acc_dev = H.make_tableset(ref_tables, "f32", accum_np=ref_acc, salts=[3, 4, 5])
    nnz = 9000

    def batch():
        cuts = np.sort(rng.integers(0, nnz + 1, size=T * B - 1))
        lengths = np.diff(np.concatenate([[0], cuts, [nnz]])).astype(np.int32)
        raw = np.minimum(rng.zipf(1.3, size=nnz), 1 << 30).astype(np.uint64) * np.uint64(0x9E3779B97F4A7C15)
        dout = rng.standard_normal((T, B, D)).astype(np.float32)
        return lengths, raw, dout

    dev = torch.device(H.DEV)
    lengths_d = torch.zeros(T * B, dtype=torch.int32, device=dev)
    raw_d = torch.zeros(nnz, dtype=torch.int64, device=dev)
    dout_d = torch.zeros((T, B, D), dtype=torch.float32, device=dev)
    offsets_d = torch.zeros(T * B + 1, dtype=torch.int64, device=dev)
    out_d = torch.zeros((T, B, D), dtype=torch.float32, device=dev)
    ws = torch.empty(emb.emb_bag_backward_workspace_bytes(T, B, nnz, ts.total_rows, D, "f32"), dtype=torch.uint8, device=dev)
    nu = torch.zeros(1, dtype=torch.int64, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    sd = H.side_stream() if side else None

    def step():
        if from_lengths:
            emb.emb_bag_forward_train_lengths(ts, raw_d, lengths_d, B, "mean", out_d, offsets_d, ws, None, nu, status)
        else:
            emb.emb_lengths_to_offsets(lengths_d, offsets_d, status)
            emb.emb_bag_forward_train(ts, raw_d, offsets_d, B, "mean", out_d, ws, None, nu, status)
        emb.emb_bag_backward_sort_prepared(ts, B, nnz, ws, None, None, nu, status, None)
        emb.emb_bag_backward_update(ts, B, nnz, dout_d, 0.01, 1e-8, ws, nu, None, sd)

    def load(b):
        lengths_d.copy_(torch.from_numpy(b[0]))
        raw_d.copy_(torch.from_numpy(b[1].view(np.int64)))
        dout_d.copy_(torch.from_numpy(b[2]))

    def check(b, what):
        off, _ = oracle.lengths_to_offsets(b[0])
        rows = np.concatenate([oracle.hash_ids(b[1][off[t * B]:off[(t + 1) * B]], 3 + t, Rs[t]) for t in range(T)])
        old = [t.copy() for t in ref_tables]
        ref_out, absum, st = oracle.bag_forward(ref_tables, "f32", rows, off, B, "mean")
        r = oracle.bag_backward_rowwise_adagrad(ref_tables, ref_acc, "f32", rows, off, B, "mean", b[2], 0.01, 1e-8)
        assert st == 0 and r["status"] == 0 and status.item() == 0
        assert np.array_equal(offsets_d.cpu().numpy(), off)
        H.assert_pooled_close(out_d.cpu().numpy(), ref_out, absum, what=what + " forward")
        assert int(nu.item()) == r["unique_keys"].size
        for t in range(T):
            H.assert_rows_close(w_dev[t].cpu().numpy(), ref_tables[t], old[t], 0.01, what="%s rows t=%d" % (what, t))
            w_dev[t].copy_(torch.from_numpy(ref_tables[t]))      # both sides go on from identical state
            acc_dev[t].copy_(torch.from_numpy(ref_acc[t]))

    b0 = batch()
    load(b0)
    step()                                                            # eager, also warms everything up
    torch.cuda.synchronize()
    check(b0, "eager")
    cap = torch.cuda.Stream(device=dev)
    graph = torch.cuda.CUDAGraph()
    b1 = batch()
    load(b1)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=cap):
        step()
    # capturing does not run anything: tables and outputs are as the eager step left them
    for i in range(3):
        bi = b1 if i == 0 else batch()
        load(bi)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check(bi, "replay %d" % i)
        junk = torch.randn(1 << 20, device=dev).sum().item()          # eager work between the replays
        assert np.isfinite(junk)

"""The seeded input generators: determinism, distributions, table generator."""
import numpy as np
import pytest
import torch

from paper_2508_05700_amd import workloads as wl


def test_fmix64_is_a_bijection_on_a_sample_and_matches_scalar_definition():
    x = np.arange(1 << 16, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)
    z = wl.fmix64(x)
    assert np.unique(z).size == x.size
    M = (1 << 64) - 1

    def scalar(v):
        v ^= v >> 33
        v = (v * 0xFF51AFD7ED558CCD) & M
        v ^= v >> 33
        v = (v * 0xC4CEB9FE1A85EC53) & M
        v ^= v >> 33
        return v
    for i in (0, 1, 77, 65535):
        assert int(z[i]) == scalar(int(x[i]))


def test_table_values_moments_and_determinism():
    rows = np.arange(20000, dtype=np.int64)
    a = wl.table_values(123, rows, 64)
    b = wl.table_values(123, rows[::-1].copy(), 64)[::-1]
    assert a.dtype == np.float32 and np.array_equal(a, b)
    assert abs(a.mean()) < 5e-5
    assert abs(a.std() - 0.01) < 1e-4
    assert np.abs(a).max() <= 131070 * float(wl.TABLE_SCALE) * (1 + 1e-6)
    c = wl.table_values(124, rows, 64)
    assert abs(np.corrcoef(a.ravel(), c.ravel())[0, 1]) < 0.01
    # a row's values depend on (row, d) only through row*D+d
    d32 = wl.table_values(123, np.array([3], dtype=np.int64), 32)
    d64 = wl.table_values(123, np.array([1], dtype=np.int64), 64)
    assert np.array_equal(d32[0], d64[0, 32:])


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(100000).astype(np.float32) * 0.01
    bits = wl.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(wl.bf16_bits_to_f32(bits), ref.float().numpy())


def test_dense_and_sparse_tables_agree():
    dense = wl.dense_table(5, 1000, 16, "f32")
    touched = np.array([0, 999, 17, 17, 500], dtype=np.int64)
    sp = wl.sparse_host_table(5, 1000, 16, "f32", touched)
    assert sp.shape == dense.shape
    assert np.array_equal(sp[touched], dense[touched])
    assert np.all(sp[1] == 0)
    spb = wl.sparse_host_table(5, 1000, 16, "bf16", touched)
    assert spb.dtype == np.uint16
    assert np.array_equal(spb[touched], wl.f32_to_bf16_bits(dense[touched]).reshape(-1, 16))


# closed-form generalized harmonic numbers H_{N,a} (Euler-Maclaurin), independent
# of the sampler's own tail formula up to the quoted digits
@pytest.mark.parametrize("N,a,H", [(10 ** 9, 1.05, 13.4846), (10 ** 12, 1.2, 5.5717), (10 ** 9, 1.1, 9.3255)])
def test_zipf_normaliser(N, a, H):
    z = wl.BoundedZipf(N, a)
    assert abs(z.H - H) < 2e-4
    # Euler-Maclaurin from the exact head: sum_{k>M} k^-a ~ int_M^N + (N^-a - M^-a)/2
    M = z.M
    em = (M ** (1 - a) - N ** (1 - a)) / (a - 1) + 0.5 * (N ** -a - M ** -a)
    assert abs(z.head_mass + em - z.H) < 1e-9


def test_zipf_sampler_head_frequencies():
    z = wl.BoundedZipf(10 ** 9, 1.05)
    rng = np.random.default_rng(1)
    n = 2_000_000
    r = z.sample(rng, n)
    assert r.min() >= 1 and r.max() <= 10 ** 9
    for k in (1, 2, 10):
        p = z.prob(k)
        assert abs((r == k).mean() - p) < 5 * np.sqrt(p / n)
    for k in (100, 10_000, 1 << 20):
        p = z.head_cdf(k)
        assert abs((r <= k).mean() - p) < 5 * np.sqrt(p * (1 - p) / n)
    # the tail is continuous across the head boundary: mass in (M, 2M]
    M = z.M
    p = ((M + .5) ** -.05 - (2 * M + .5) ** -.05) / .05 / z.H
    assert abs(((r > M) & (r <= 2 * M)).mean() - p) < 5 * np.sqrt(p / n)
    assert abs(z.prob(1) - 0.0742) < 1e-4        # rank-1 key carries ~7.4 % of lookups


def test_make_batch_is_deterministic_and_shaped():
    w = wl.WORKLOADS["3"].scaled(rows=100_000, bags=256, tables=3)
    a = wl.make_batch(w, 0)
    b = wl.make_batch(w, 0)
    c = wl.make_batch(w, 1)
    assert np.array_equal(a["raw"], b["raw"]) and np.array_equal(a["lengths"], b["lengths"])
    assert np.array_equal(a["dout"], b["dout"])
    assert not np.array_equal(a["lengths"], c["lengths"])
    assert a["lengths"].size == 3 * 256 and a["lengths"].max() <= 100 and a["lengths"].min() >= 0
    assert a["raw"].dtype == np.uint64 and a["raw"].size == a["nnz"] == sum(a["nnz_per_table"])
    assert a["dout"].shape == (3, 256, 64) and a["dout"].dtype == np.float32
    assert abs(a["lengths"].mean() - 20) < 1.0
    # tables draw from different raw-ID streams
    n0 = a["nnz_per_table"][0]
    assert np.intersect1d(a["raw"][:n0], a["raw"][n0:]).size == 0
    w1 = wl.WORKLOADS["1"]
    b1 = wl.make_batch(w1, 0)
    assert b1["raw"] is None and b1["rows"].size == 512 * 8 and b1["rows"].max() < 100_000
    assert np.all(b1["lengths"] == 8)


def test_first_k_distinct_sorted():
    v = np.array([5, 3, 5, 9, 3, 1, 7])
    assert wl.first_k_distinct_sorted(v, 3).tolist() == [3, 5, 9]
    assert wl.first_k_distinct_sorted(v, 10).tolist() == [1, 3, 5, 7, 9]

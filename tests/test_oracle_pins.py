"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle is checked against things other than itself: published test
vectors, a hand-worked example, brute force on tiny inputs, library routines
that the definitions reduce to (torch's CPU embedding_bag, autograd and
Adagrad), closed forms and invariants.
"""
import os

import numpy as np
import pytest
import torch

from tests import harness as H

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
GAMMA = 0x9E3779B97F4A7C15
M64 = (1 << 64) - 1


# ---------------------------------------------------------------------------
# hashing
# ---------------------------------------------------------------------------
def _vectors():
    out = []
    with open(os.path.join(GOLDEN, "splitmix64_vectors.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            s, k, v = line.split()
            out.append((int(s), int(k), int(v, 0)))
    return out


def test_splitmix64_published_vectors(oracle):
    for state, k, value in _vectors():
        assert oracle.splitmix64((state + k * GAMMA) & M64) == value


def test_hash_ids_vector_form_and_mod(oracle):
    vec = _vectors()
    raw = np.array([(s + k * GAMMA) & M64 for s, k, _ in vec], dtype=np.uint64)
    for R in (1, 2, 7, 10_000_000, 1_000_000_000, (1 << 40) + 17, (1 << 63) - 1):
        rows = oracle.hash_ids(raw, 0, R)
        assert rows.tolist() == [v % R for _, _, v in vec]
        assert rows.min() >= 0 and rows.max() < R


def test_hash_salt_is_xor_before_mixing(oracle):
    # hash(raw, salt) must equal hash(raw ^ salt, 0): pins where the salt enters
    raw = np.array([0, 1, 12345, M64, 0xDEADBEEFCAFEF00D], dtype=np.uint64)
    salt = 0x0123456789ABCDEF
    a = oracle.hash_ids(raw, salt, 10_000_019)
    b = oracle.hash_ids(raw ^ np.uint64(salt), 0, 10_000_019)
    assert np.array_equal(a, b)
    # and the salt value s hashes x == s to the hash of zero
    assert oracle.hash_ids(np.array([salt], dtype=np.uint64), salt, 1 << 62)[0] == \
        0xE220A8397B1DCDAF % (1 << 62)


def test_hash_is_injective_before_mod_and_uniform_after(oracle):
    n = 1 << 20
    raw = np.arange(n, dtype=np.uint64)
    full = oracle.hash_ids(raw, 7, (1 << 63) - 1)   # mod a huge prime-ish value: collisions only if mix collides
    assert np.unique(full).size == n
    R = 1000
    rows = oracle.hash_ids(raw, 7, R)
    counts = np.bincount(rows, minlength=R)
    chi2 = ((counts - n / R) ** 2 / (n / R)).sum()
    # chi-square with 999 dof: mean 999, sd ~44.7; 6 sigma band
    assert 999 - 270 < chi2 < 999 + 270


# ---------------------------------------------------------------------------
# offsets
# ---------------------------------------------------------------------------
def test_offsets_match_cumsum(oracle):
    rng = np.random.default_rng(1)
    for n in (0, 1, 2, 63, 64, 65, 1000, 4097):
        L = rng.integers(0, 101, size=n).astype(np.int32)
        off, st = oracle.lengths_to_offsets(L)
        assert st == 0
        assert off[0] == 0 and off.size == n + 1
        assert np.array_equal(off[1:], np.cumsum(L.astype(np.int64)))


def test_offsets_do_not_wrap_at_32_bits(oracle):
    L = np.full(3, 2_000_000_000, dtype=np.int32)
    off, st = oracle.lengths_to_offsets(L)
    assert off.tolist() == [0, 2_000_000_000, 4_000_000_000, 6_000_000_000] and st == 0


def test_offsets_negative_length_flagged_and_clamped(oracle):
    off, st = oracle.lengths_to_offsets(np.array([3, -2, 4], dtype=np.int32))
    assert off.tolist() == [0, 3, 3, 7]
    assert st == oracle.STATUS_BAD_OFFSETS


# ---------------------------------------------------------------------------
# forward
# ---------------------------------------------------------------------------
def _worked():
    d = {}
    with open(os.path.join(GOLDEN, "worked_example_bag.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d[k] = np.array([float(x) for x in v])
    return d


def test_forward_worked_example(oracle):
    w = _worked()
    W = w["W"].reshape(3, 2).astype(np.float32)
    rows = w["rows"].astype(np.int64)
    off = w["offsets"].astype(np.int64)
    out, absum, st = oracle.bag_forward([W], "f32", rows, off, 3, "sum")
    assert st == 0 and np.array_equal(out.reshape(-1), w["fwd_sum"].astype(np.float32))
    assert np.array_equal(absum.reshape(-1), w["fwd_sum"])      # all terms positive
    out, absum, st = oracle.bag_forward([W], "f32", rows, off, 3, "mean")
    assert np.array_equal(out.reshape(-1), w["fwd_mean"].astype(np.float32))


def _random_case(rng, T, B, D, Rs, max_len, empty_frac=0.2):
    tables = [rng.standard_normal((R, D)).astype(np.float32) for R in Rs]
    lengths = rng.integers(0, max_len + 1, size=T * B).astype(np.int32)
    lengths[rng.random(T * B) < empty_frac] = 0
    off = np.concatenate([[0], np.cumsum(lengths.astype(np.int64))])
    rows = np.concatenate([rng.integers(0, Rs[t], size=int(lengths[t * B:(t + 1) * B].sum()))
                           for t in range(T)]).astype(np.int64) if T else np.zeros(0, np.int64)
    return tables, lengths, off, rows


def test_forward_brute_force_multiplicity_matrix(oracle):
    # out = A @ W with A[b, r] = number of times row r occurs in bag b
    rng = np.random.default_rng(2)
    T, B, D, Rs = 3, 17, 5, [11, 4, 29]
    tables, lengths, off, rows = _random_case(rng, T, B, D, Rs, 9)
    out_s, _, st = oracle.bag_forward(tables, "f32", rows, off, B, "sum")
    out_m, _, _ = oracle.bag_forward(tables, "f32", rows, off, B, "mean")
    assert st == 0
    for t in range(T):
        A = np.zeros((B, Rs[t]))
        for b in range(B):
            for j in range(off[t * B + b], off[t * B + b + 1]):
                A[b, rows[j]] += 1
        ref = A @ tables[t].astype(np.float64)
        np.testing.assert_allclose(out_s[t], ref, rtol=1e-6, atol=1e-6)
        L = lengths[t * B:(t + 1) * B].astype(np.float64)
        refm = np.where(L[:, None] > 0, ref / np.maximum(L, 1)[:, None], 0.0)
        np.testing.assert_allclose(out_m[t], refm, rtol=1e-6, atol=1e-6)
        assert np.all(out_m[t][L == 0] == 0.0)


@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_forward_matches_torch_embedding_bag(oracle, mode):
    rng = np.random.default_rng(3)
    T, B, D, Rs = 2, 64, 16, [1000, 37]
    tables, lengths, off, rows = _random_case(rng, T, B, D, Rs, 30)
    out, absum, st = oracle.bag_forward(tables, "f32", rows, off, B, mode)
    assert st == 0
    for t in range(T):
        lo, hi = off[t * B], off[(t + 1) * B]
        ref = torch.nn.functional.embedding_bag(
            torch.from_numpy(rows[lo:hi]), torch.from_numpy(tables[t]).double(),
            torch.from_numpy(off[t * B:(t + 1) * B + 1] - lo), mode=mode,
            include_last_offset=True).numpy()
        assert np.all(np.abs(out[t] - ref) <= 1e-6 * np.maximum(absum[t], 1e-30) + 1e-30)


def test_forward_invariants(oracle):
    rng = np.random.default_rng(4)
    T, B, D, Rs = 1, 50, 8, [200]
    tables, lengths, off, rows = _random_case(rng, T, B, D, Rs, 12)
    out_s, ab_s, _ = oracle.bag_forward(tables, "f32", rows, off, B, "sum")
    out_m, _, _ = oracle.bag_forward(tables, "f32", rows, off, B, "mean")
    # total mass: sum over bags of pooled sums == sum of all gathered rows
    np.testing.assert_allclose(out_s[0].astype(np.float64).sum(0),
                               tables[0][rows].astype(np.float64).sum(0), rtol=1e-5, atol=1e-5)
    # mean * L == sum
    L = lengths.astype(np.float64)[:, None]
    np.testing.assert_allclose(out_m[0] * L, out_s[0], rtol=1e-6, atol=1e-6)
    # scaling the table by 2 scales the output by exactly 2
    out2, _, _ = oracle.bag_forward([tables[0] * 2], "f32", rows, off, B, "sum")
    assert np.array_equal(out2, out_s * 2)
    # permuting lookups inside every bag changes nothing beyond rounding
    rows_p = rows.copy()
    for b in range(B):
        rows_p[off[b]:off[b + 1]] = rng.permutation(rows[off[b]:off[b + 1]])
    outp, _, _ = oracle.bag_forward(tables, "f32", rows_p, off, B, "sum")
    assert np.all(np.abs(outp - out_s) <= 1e-6 * ab_s)
    # absum dominates |out| and equals the pooled sum of |W|
    outa, _, _ = oracle.bag_forward([np.abs(tables[0])], "f32", rows, off, B, "sum")
    np.testing.assert_allclose(ab_s, outa, rtol=1e-6)
    assert np.all(np.abs(out_s) <= ab_s * (1 + 1e-6) + 1e-30)


def test_forward_integer_valued_is_exact(oracle):
    rng = np.random.default_rng(5)
    W = rng.integers(-1000, 1000, size=(300, 4)).astype(np.float32)
    lengths = rng.integers(0, 100, size=40).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(lengths.astype(np.int64))])
    rows = rng.integers(0, 300, size=int(off[-1])).astype(np.int64)
    out, _, _ = oracle.bag_forward([W], "f32", rows, off, 40, "sum")
    ref = np.stack([W[rows[off[b]:off[b + 1]]].astype(np.int64).sum(0) for b in range(40)])
    assert np.array_equal(out[0].astype(np.int64), ref)


def test_forward_bf16_widening_is_exact(oracle):
    rng = np.random.default_rng(6)
    Wt = torch.from_numpy(rng.standard_normal((50, 8)).astype(np.float32)).to(torch.bfloat16)
    bits = Wt.view(torch.int16).numpy().view(np.uint16).copy()
    rows = np.arange(50, dtype=np.int64)
    off = np.arange(51, dtype=np.int64)     # one lookup per bag -> out == widened row
    out, _, _ = oracle.bag_forward([bits], "bf16", rows, off, 50, "sum")
    assert np.array_equal(out[0], Wt.float().numpy())


def test_forward_bad_inputs_are_flagged_not_read(oracle):
    W = np.arange(12, dtype=np.float32).reshape(6, 2)
    rows = np.array([0, 6, 1, -1, 2], dtype=np.int64)
    off = np.array([0, 2, 5], dtype=np.int64)
    out, _, st = oracle.bag_forward([W], "f32", rows, off, 2, "sum")
    assert st == oracle.STATUS_BAD_INDEX
    assert out[0].tolist() == [[0, 1], [2 + 4, 3 + 5]]
    # mean still divides by the declared bag length
    out, _, st = oracle.bag_forward([W], "f32", rows, off, 2, "mean")
    assert out[0].tolist() == [[0, 0.5], [2.0, 8 / 3]] or np.allclose(out[0], [[0, .5], [2, 8 / 3]])
    # bag with reversed / overflowing offsets -> zeros + flag
    out, _, st = oracle.bag_forward([W], "f32", rows, np.array([0, 7, 5], dtype=np.int64), 2, "sum")
    assert st & oracle.STATUS_BAD_OFFSETS
    assert out[0].tolist() == [[0, 0], [0, 0]]


# ---------------------------------------------------------------------------
# backward + row-wise Adagrad
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_backward_worked_example(oracle, mode):
    w = _worked()
    W = w["W"].reshape(3, 2).astype(np.float32)
    S = np.zeros(3, dtype=np.float32)
    res = oracle.bag_backward_rowwise_adagrad(
        [W], [S], "f32", w["rows"].astype(np.int64), w["offsets"].astype(np.int64), 3, mode,
        w["dout"].reshape(3, 2).astype(np.float32), 0.01, 1e-8)
    assert res["status"] == 0
    assert res["unique_keys"].tolist() == [0, 1, 2]
    assert res["unique_counts"].tolist() == w["counts"].astype(int).tolist()
    np.testing.assert_allclose(res["G"].reshape(-1), w["G_" + mode], rtol=1e-15)
    np.testing.assert_allclose(S, w["S_" + mode], rtol=1e-7)
    np.testing.assert_allclose(W.reshape(-1), w["W_new"], atol=1e-6)


def _torch_dense_grad(table, rows, off, B, mode, dout):
    Wt = torch.from_numpy(table).double().requires_grad_(True)
    out = torch.nn.functional.embedding_bag(torch.from_numpy(rows), Wt, torch.from_numpy(off),
                                            mode=mode, include_last_offset=True)
    out.backward(torch.from_numpy(dout).double())
    return Wt.grad.numpy()


@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_backward_summed_gradient_matches_autograd(oracle, mode):
    rng = np.random.default_rng(7)
    T, B, D, Rs = 3, 40, 6, [50, 7, 300]
    tables, lengths, off, rows = _random_case(rng, T, B, D, Rs, 10)
    dout = rng.standard_normal((T, B, D)).astype(np.float32)
    W0 = [t.copy() for t in tables]
    S = [np.zeros(R, dtype=np.float32) for R in Rs]
    res = oracle.bag_backward_rowwise_adagrad(tables, S, "f32", rows, off, B, mode, dout, 0.01, 1e-8)
    assert res["status"] == 0
    base = np.concatenate([[0], np.cumsum(Rs)])
    # unique keys == numpy.unique of (table base + row), counts too
    keys = np.concatenate([base[t] + rows[off[t * B]:off[(t + 1) * B]] for t in range(T)])
    uk, uc = np.unique(keys, return_counts=True)
    assert np.array_equal(res["unique_keys"], uk) and np.array_equal(res["unique_counts"], uc)
    assert res["unique_counts"].sum() == rows.size
    for t in range(T):
        lo = off[t * B]
        g = _torch_dense_grad(W0[t], rows[lo:off[(t + 1) * B]], off[t * B:(t + 1) * B + 1] - lo,
                              B, mode, dout[t])
        sel = (res["unique_keys"] >= base[t]) & (res["unique_keys"] < base[t + 1])
        r = res["unique_keys"][sel] - base[t]
        np.testing.assert_allclose(res["G"][sel], g[r], rtol=1e-12, atol=1e-12)
        untouched = np.setdiff1d(np.arange(Rs[t]), r)
        assert np.all(g[untouched] == 0)
        # rows outside the batch are bit-identical, accumulators too
        assert np.array_equal(tables[t][untouched], W0[t][untouched])
        assert np.all(S[t][untouched] == 0)
        # gradient mass: sum_r G == sum_b L_b c_b dOut
        L = lengths[t * B:(t + 1) * B].astype(np.float64)
        c = L if mode == "sum" else (L > 0).astype(np.float64)
        np.testing.assert_allclose(res["G"][sel].sum(0), (c[:, None] * dout[t]).sum(0),
                                   rtol=1e-9, atol=1e-9)
        # first step from S = 0: ||dW||^2 == lr^2 * D for every touched row with G != 0
        dW = (tables[t][r].astype(np.float64) - W0[t][r]) ** 2
        nz = np.abs(res["G"][sel]).sum(1) > 0
        np.testing.assert_allclose(dW.sum(1)[nz], 0.01 ** 2 * D, rtol=1e-3)
        # the step goes against the gradient
        assert np.all((tables[t][r] - W0[t][r]) * res["G"][sel] <= 0)


def test_backward_d1_is_elementwise_adagrad_over_several_steps(oracle):
    rng = np.random.default_rng(8)
    R, B, D = 60, 25, 1
    W = rng.standard_normal((R, D)).astype(np.float32)
    S = np.zeros(R, dtype=np.float32)
    Wt = torch.from_numpy(W.copy()).double().requires_grad_(True)
    opt = torch.optim.Adagrad([Wt], lr=0.05, eps=1e-8, initial_accumulator_value=0.0)
    for step in range(4):
        lengths = rng.integers(0, 8, size=B).astype(np.int32)
        off = np.concatenate([[0], np.cumsum(lengths.astype(np.int64))])
        rows = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
        dout = rng.standard_normal((1, B, D)).astype(np.float32)
        S_prev = S.copy()
        oracle.bag_backward_rowwise_adagrad([W], [S], "f32", rows, off, B, "sum", dout, 0.05, 1e-8)
        assert np.all(S >= S_prev)                       # accumulators are monotone
        opt.zero_grad()
        out = torch.nn.functional.embedding_bag(torch.from_numpy(rows), Wt, torch.from_numpy(off),
                                                mode="sum", include_last_offset=True)
        out.backward(torch.from_numpy(dout[0]).double())
        opt.step()
        np.testing.assert_allclose(W, Wt.detach().numpy(), rtol=2e-6, atol=2e-7)
        np.testing.assert_allclose(S, opt.state[Wt]["sum"].numpy()[:, 0], rtol=2e-6, atol=1e-12)


def test_backward_equal_magnitude_rows_match_elementwise_adagrad_any_d(oracle):
    # if |G_d| is the same for all d, mean_d G_d^2 == G_d^2 and the row-wise rule
    # coincides with element-wise Adagrad: pins the 1/D, the order accumulate-then-
    # use, and eps outside the square root, for D > 1 and S_old != 0.
    rng = np.random.default_rng(9)
    R, B, D = 40, 40, 8
    W = rng.standard_normal((R, D)).astype(np.float32)
    S = np.zeros(R, dtype=np.float32)
    Wt = torch.from_numpy(W.copy()).double().requires_grad_(True)
    opt = torch.optim.Adagrad([Wt], lr=0.01, eps=1e-3, initial_accumulator_value=0.0)
    for step in range(3):
        rows = rng.permutation(R)[:B].astype(np.int64)         # each row in exactly one bag
        off = np.arange(B + 1, dtype=np.int64)
        mag = rng.uniform(0.5, 2.0, size=(B, 1))
        dout = (mag * rng.choice([-1.0, 1.0], size=(B, D))).astype(np.float32)[None]
        oracle.bag_backward_rowwise_adagrad([W], [S], "f32", rows, off, B, "sum", dout, 0.01, 1e-3)
        opt.zero_grad()
        out = torch.nn.functional.embedding_bag(torch.from_numpy(rows), Wt, torch.from_numpy(off),
                                                mode="sum", include_last_offset=True)
        out.backward(torch.from_numpy(dout[0]).double())
        opt.step()
        np.testing.assert_allclose(W, Wt.detach().numpy(), rtol=2e-6, atol=2e-7)
        np.testing.assert_allclose(S, opt.state[Wt]["sum"].numpy()[:, 0], rtol=2e-6)


def test_backward_duplicates_are_summed_before_the_nonlinear_update(oracle):
    # one row looked up 4 times with the same gradient: exact semantics gives one
    # update with G = 4g (step length lr), not four updates.
    W = np.zeros((2, 2), dtype=np.float32)
    S = np.zeros(2, dtype=np.float32)
    rows = np.array([1, 1, 1, 1], dtype=np.int64)
    off = np.array([0, 1, 2, 3, 4], dtype=np.int64)
    dout = np.tile(np.array([[3.0, -4.0]], dtype=np.float32), (4, 1))[None]
    res = oracle.bag_backward_rowwise_adagrad([W], [S], "f32", rows, off, 4, "sum", dout, 0.1, 0.0)
    assert res["unique_keys"].tolist() == [1] and res["unique_counts"].tolist() == [4]
    # G = (12,-16), S = (144+256)/2 = 200, W = -0.1*G/sqrt(200)
    np.testing.assert_allclose(S, [0, 200.0])
    np.testing.assert_allclose(W[1], [-0.1 * 12 / np.sqrt(200), 0.1 * 16 / np.sqrt(200)], rtol=1e-6)
    assert np.all(W[0] == 0)


def test_backward_zero_gradient_row_is_listed_and_unchanged(oracle):
    W = np.ones((3, 2), dtype=np.float32)
    S = np.zeros(3, dtype=np.float32)
    rows = np.array([2, 2], dtype=np.int64)
    off = np.array([0, 1, 2], dtype=np.int64)
    dout = np.array([[[1.0, 2.0], [-1.0, -2.0]]], dtype=np.float32)
    res = oracle.bag_backward_rowwise_adagrad([W], [S], "f32", rows, off, 2, "sum", dout, 0.01, 1e-8)
    assert res["unique_keys"].tolist() == [2]
    assert np.all(W == 1) and np.all(S == 0) and np.all(np.isfinite(W))


def test_backward_bf16_rows_round_to_nearest_even(oracle):
    rng = np.random.default_rng(10)
    R, B, D = 30, 30, 4
    Wt = torch.from_numpy(rng.standard_normal((R, D)).astype(np.float32)).to(torch.bfloat16)
    bits = Wt.view(torch.int16).numpy().view(np.uint16).copy()
    Wf = Wt.float().numpy().copy()
    S = np.zeros(R, dtype=np.float32)
    Sf = np.zeros(R, dtype=np.float32)
    rows = rng.permutation(R).astype(np.int64)
    off = np.arange(B + 1, dtype=np.int64)
    dout = rng.standard_normal((1, B, D)).astype(np.float32)
    oracle.bag_backward_rowwise_adagrad([bits], [S], "bf16", rows, off, B, "sum", dout, 0.05, 1e-8)
    oracle.bag_backward_rowwise_adagrad([Wf], [Sf], "f32", rows, off, B, "sum", dout, 0.05, 1e-8)
    expect = torch.from_numpy(Wf).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, expect)
    assert np.array_equal(S, Sf)


def test_backward_bad_inputs(oracle):
    W = np.ones((4, 2), dtype=np.float32)
    S = np.zeros(4, dtype=np.float32)
    dout = np.ones((1, 2, 2), dtype=np.float32)
    # out-of-range rows are skipped, the rest is processed
    res = oracle.bag_backward_rowwise_adagrad(
        [W], [S], "f32", np.array([0, 9, -3, 1], dtype=np.int64), np.array([0, 2, 4], dtype=np.int64),
        2, "sum", dout, 0.01, 1e-8)
    assert res["status"] == oracle.STATUS_BAD_INDEX
    assert res["unique_keys"].tolist() == [0, 1] and res["unique_counts"].tolist() == [1, 1]
    # broken offsets: nothing is touched
    W2, S2 = np.ones((4, 2), dtype=np.float32), np.zeros(4, dtype=np.float32)
    for off in ([0, 3, 2], [1, 2, 4], [0, 2, 3]):
        res = oracle.bag_backward_rowwise_adagrad(
            [W2], [S2], "f32", np.array([0, 1, 2, 3], dtype=np.int64), np.array(off, dtype=np.int64),
            2, "sum", dout, 0.01, 1e-8)
        assert res["status"] == oracle.STATUS_BAD_OFFSETS and res["unique_keys"].size == 0
        assert np.all(W2 == 1) and np.all(S2 == 0)


# ---------------------------------------------------------------------------
# cached (hybrid) forward
# ---------------------------------------------------------------------------
def test_cached_forward_equals_plain_forward_and_counts_hits(oracle):
    rng = np.random.default_rng(11)
    T, B, D, Rs = 1, 30, 4, [100]
    tables, lengths, off, rows = _random_case(rng, T, B, D, Rs, 9)
    ref, _, _ = oracle.bag_forward(tables, "f32", rows, off, B, "mean")
    for hot in (np.zeros(0, np.int64), np.arange(100, dtype=np.int64),
                np.sort(rng.permutation(100)[:17]).astype(np.int64)):
        out, _, (hits, misses), st = oracle.bag_forward_cached(tables[0], "f32", hot, rows, off, B, "mean")
        assert st == 0 and np.array_equal(out, ref)
        assert hits == int(np.isin(rows, hot).sum()) and hits + misses == rows.size


def test_backward_bf16_tie_rounds_to_even(oracle):
    # W_old = 1.0, equal-magnitude gradient, eps = 0, S_old = 0  =>  step = -lr*sign(G)
    # exactly.  With lr = 2^-8 the new value 1 + 2^-8 lies exactly half-way between
    # the bf16 neighbours 1.0 (even mantissa) and 1 + 2^-7: ties-to-even keeps 1.0.
    # With G > 0 the new value 1 - 2^-8 is representable and must be hit exactly.
    D = 8
    one = np.uint16(0x3F80)
    bits = np.full((2, D), one, dtype=np.uint16)
    S = np.zeros(2, dtype=np.float32)
    rows = np.array([0, 1], dtype=np.int64)
    off = np.array([0, 1, 2], dtype=np.int64)
    dout = np.stack([np.full(D, -3.0), np.full(D, 3.0)]).astype(np.float32)[None]
    oracle.bag_backward_rowwise_adagrad([bits], [S], "bf16", rows, off, 2, "sum", dout, 2.0 ** -8, 0.0)
    assert np.all(bits[0] == 0x3F80)
    assert np.all(bits[1] == 0x3F7F)
    np.testing.assert_array_equal(S, [9.0, 9.0])


# ---------------------------------------------------------------------------
# row-quantised tables (INT8 / INT4 storage, Section 4.1.2)
# ---------------------------------------------------------------------------
def _unpack(q, D, dtype):
    """scale, bias, codes of packed rows, taken apart by hand from the stated layout."""
    scale = q[:, 0:4].copy().view(np.float32)[:, 0]
    bias = q[:, 4:8].copy().view(np.float32)[:, 0]
    if dtype == "int8":
        codes = q[:, 8:8 + D].astype(np.int64)
    else:
        b = q[:, 8:8 + D // 2].astype(np.int64)
        codes = np.empty((q.shape[0], D), dtype=np.int64)
        codes[:, 0::2] = b & 15
        codes[:, 1::2] = b >> 4
    return scale, bias, codes


def test_quantized_row_size_matches_the_papers_ratio(oracle):
    # Section 4.1.2: the INT4 tables take about 40 % of their fp16 size.  An fp16 row of D = 64 is 128 bytes.
    assert oracle.quant_row_bytes(64, "int4") == 48            # 37.5 %
    assert oracle.quant_row_bytes(32, "int4") == 32 and oracle.quant_row_bytes(128, "int4") == 80
    assert oracle.quant_row_bytes(64, "int8") == 80 and oracle.quant_row_bytes(8, "int8") == 16
    assert oracle.quant_row_bytes(63, "int4") == 0 and oracle.quant_row_bytes(0, "int8") == 0
    assert oracle.quant_row_bytes(64, "f32") == 0


@pytest.mark.parametrize("dtype,qmax", [("int8", 255), ("int4", 15)])
def test_quantizer_invariants(oracle, dtype, qmax):
    rng = np.random.default_rng(77)
    D = 64
    x = (rng.standard_normal((300, D)) * rng.uniform(1e-3, 10, size=(300, 1))).astype(np.float32)
    x[7] = 0.25                                                   # a constant row
    q = oracle.quantize_rows(x, dtype)
    assert q.shape == (300, oracle.quant_row_bytes(D, dtype))
    scale, bias, codes = _unpack(q, D, dtype)
    assert np.array_equal(bias, x.min(axis=1))                    # bias is the row minimum, exactly
    lo, hi = x.min(axis=1).astype(np.float64), x.max(axis=1).astype(np.float64)
    var = hi > lo
    assert np.allclose(scale[var], (hi[var] - lo[var]) / qmax, rtol=2e-7, atol=0)
    assert scale[7] == 1.0 and np.all(codes[7] == 0)
    assert codes.min() >= 0 and codes.max() <= qmax
    rows = np.arange(300)
    assert np.all(codes[rows, x.argmin(axis=1)] == 0)             # the extremes get the end codes
    assert np.all(codes[rows[var], x[var].argmax(axis=1)] == qmax)
    deq = scale[:, None].astype(np.float64) * codes + bias[:, None].astype(np.float64)
    err = np.abs(deq - x.astype(np.float64))
    assert np.all(err <= 0.5 * scale[:, None] * (1 + 1e-5) + 1e-12)   # nearest code
    order = np.argsort(x, axis=1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(codes, order, axis=1), axis=1) >= 0)   # monotone in x
    pad = q[:, 8 + (D if dtype == "int8" else D // 2):]
    assert pad.size > 0 and not pad.any()                         # padding is zero


@pytest.mark.parametrize("dtype,qmax", [("int8", 255), ("int4", 15)])
def test_quantizer_is_exact_on_grid_rows(oracle, dtype, qmax):
    # rows whose elements are bias + k * 2^-e with both end codes present come back unchanged
    rng = np.random.default_rng(78)
    D = 32
    k = rng.integers(0, qmax + 1, size=(50, D))
    k[:, 3], k[:, 17] = 0, qmax
    step = 2.0 ** -rng.integers(2, 9, size=(50, 1))
    base = rng.integers(-40, 40, size=(50, 1)) * step
    x = (base + k * step).astype(np.float32)
    scale, bias, codes = _unpack(oracle.quantize_rows(x, dtype), D, dtype)
    assert np.array_equal(codes, k)
    assert np.array_equal(scale, step[:, 0].astype(np.float32)) and np.array_equal(bias, base[:, 0].astype(np.float32))


@pytest.mark.parametrize("dtype,qmax", [("int8", 255), ("int4", 15)])
def test_quantizer_rounds_ties_to_even(oracle, dtype, qmax):
    # a row spanning [0, qmax] has scale exactly 1: x = k + 0.5 is an exact tie
    D = 16
    x = np.zeros((1, D), dtype=np.float32)
    x[0, :8] = [0.0, qmax, 0.5, 1.5, 2.5, 3.5, 4.5, qmax - 0.5]
    scale, bias, codes = _unpack(oracle.quantize_rows(x, dtype), D, dtype)
    assert scale[0] == 1.0 and bias[0] == 0.0
    assert list(codes[0, :8]) == [0, qmax, 0, 2, 2, 4, 4, qmax - 1]


@pytest.mark.parametrize("dtype,tdtype,qmax", [("int8", torch.quint8, 255), ("int4", torch.quint4x2, 15)])
def test_quantizer_agrees_with_torch_per_channel_float_qparams(oracle, dtype, tdtype, qmax):
    # torch's row-wise quantiser with float scale / zero point (its embedding-table scheme) rounds
    # x / scale + zero_point instead of (x - bias) / scale: codes may differ by one at near-ties only
    rng = np.random.default_rng(79)
    D = 64
    x = torch.from_numpy((rng.standard_normal((400, D)) * 0.01).astype(np.float32))
    lo, hi = x.min(1).values, x.max(1).values
    tscale = (hi - lo) / qmax
    tq = torch.quantize_per_channel(x, tscale, -lo / tscale, 0, tdtype)
    tdeq = tq.dequantize().numpy().astype(np.float64)
    tcodes = np.rint((tdeq - lo.numpy()[:, None].astype(np.float64)) / tscale.numpy()[:, None].astype(np.float64))
    scale, bias, codes = _unpack(oracle.quantize_rows(x.numpy(), dtype), D, dtype)
    diff = np.abs(codes - tcodes)
    assert diff.max() <= 1 and (diff != 0).mean() < 2e-3
    assert np.array_equal(scale, tscale.numpy())
    if dtype == "int4":   # same nibble order as torch's packed storage
        packed = tq.int_repr().numpy().reshape(400, D // 2)
        mine = oracle.quantize_rows(x.numpy(), dtype)[:, 8:8 + D // 2]
        assert (packed != mine).mean() < 4e-3


@pytest.mark.parametrize("dtype,qmax", [("int8", 255), ("int4", 15)])
@pytest.mark.parametrize("mode", ["sum", "mean"])
def test_quantized_forward_equals_fp32_forward_of_the_dequantized_table(oracle, dtype, qmax, mode):
    rng = np.random.default_rng(80)
    T, B, D, R = 2, 9, 16, 40
    # grid-valued tables: quantisation is lossless (pinned above), so both paths sum identical numbers
    tabs = []
    for t in range(T):
        k = rng.integers(0, qmax + 1, size=(R, D))
        k[:, 0], k[:, 5] = 0, qmax
        step = 2.0 ** -rng.integers(2, 7, size=(R, 1))
        tabs.append((rng.integers(-9, 9, size=(R, 1)) * step + k * step).astype(np.float32))
    lengths = rng.integers(0, 6, size=T * B).astype(np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    rows = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    qt = [oracle.quantize_rows(x, dtype) for x in tabs]
    out_q, absum_q, st = oracle.bag_forward(qt, dtype, rows, off, B, mode, D=D)
    out_f, absum_f, _ = oracle.bag_forward(tabs, "f32", rows, off, B, mode)
    assert st == 0 and np.array_equal(out_q, out_f) and np.array_equal(absum_q, absum_f)
    # and torch's embedding_bag over its own dequantised copy of a generic (lossy) table
    x = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
    scale, bias, codes = _unpack(oracle.quantize_rows(x, dtype), D, dtype)
    deq = torch.from_numpy(scale[:, None].astype(np.float64) * codes + bias[:, None].astype(np.float64))
    o1, _, _ = oracle.bag_forward([oracle.quantize_rows(x, dtype)], dtype, rows[:off[B]], off[:B + 1], B, mode, D=D)
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(rows[:off[B]]), deq, torch.from_numpy(off[:B]),
                                            mode=mode, include_last_offset=False)
    assert np.allclose(o1[0], ref.numpy(), rtol=1e-6, atol=1e-9)


# ---------------------------------------------------------------------------
# frequency-based cache policy (which rows the hot-row cache of Section 3.3 holds; "caching strategies", Section 6)
# ---------------------------------------------------------------------------

def test_cache_observe_is_a_histogram_of_the_in_range_rows(oracle):
    rng = np.random.default_rng(90)
    R = 257
    freq = rng.integers(0, 50, size=R).astype(np.uint32)
    before = freq.copy()
    rows = rng.integers(-40, R + 40, size=20000).astype(np.int64)
    rows[:3000] = 7                                                  # one very hot row
    bad = oracle.cache_observe(freq, rows)
    ok = rows[(rows >= 0) & (rows < R)]
    assert bad == rows.size - ok.size
    assert np.array_equal(freq.astype(np.int64), before.astype(np.int64) + np.bincount(ok, minlength=R))
    # counters are u32 and wrap
    freq = np.array([0xFFFFFFFE, 5], dtype=np.uint32)
    assert oracle.cache_observe(freq, np.array([0, 0, 0, 1], dtype=np.int64)) == 0
    assert freq.tolist() == [1, 6]
    # nothing observed, nothing changes
    assert oracle.cache_observe(freq, np.zeros(0, np.int64)) == 0 and freq.tolist() == [1, 6]


@pytest.mark.parametrize("seed", range(6))
def test_cache_select_equals_brute_force_on_small_inputs_with_many_ties(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    R = int(rng.integers(1, 40))
    freq = rng.integers(0, 4, size=R).astype(np.uint32)              # few distinct values: ties everywhere
    if seed == 0:
        freq[:] = 0xFFFFFFFF                                         # the largest counter value, all equal
    for num_hot in sorted({0, 1, R // 3, R - 1 if R > 1 else 0, R}):
        f = freq.copy()
        hot = oracle.cache_select(f, num_hot, 0)
        # plain statement of the rule: walk the rows by (larger counter, then smaller row) and keep num_hot
        pref = sorted(range(R), key=lambda r: (-int(freq[r]), r))
        assert hot.tolist() == sorted(pref[:num_hot])
        assert np.array_equal(f, freq)                               # shift 0 leaves the counters alone


def test_cache_select_invariants_and_aging(oracle):
    rng = np.random.default_rng(110)
    R, H = 5000, 600
    freq = np.minimum(rng.zipf(1.3, size=R), 1 << 20).astype(np.uint32)
    f = freq.copy()
    hot = oracle.cache_select(f, H, 3)
    assert hot.size == H and (np.diff(hot) > 0).all() and hot[0] >= 0 and hot[-1] < R
    assert np.array_equal(f, freq >> 3)                              # every counter aged, selected or not
    sel = np.zeros(R, bool)
    sel[hot] = True
    thr = freq[sel].min()
    assert freq[~sel].max() <= thr                                   # nothing left out beats anything kept
    tied = np.flatnonzero(freq == thr)                               # the tie at the threshold goes to small rows
    kept = sel[tied]
    assert not (~kept[:-1] & kept[1:]).any()
    # distinct counters: the rule is a plain top-k (torch.topk as the library routine)
    distinct = rng.permutation(R).astype(np.uint32) + 5
    hot = oracle.cache_select(distinct.copy(), H, 0)
    top = torch.topk(torch.from_numpy(distinct.astype(np.int64)), H).indices.numpy()
    assert np.array_equal(hot, np.sort(top))
    # all counters equal: the first rows
    assert oracle.cache_select(np.full(R, 9, np.uint32), H, 0).tolist() == list(range(H))


def test_cache_policy_keeps_the_set_with_the_most_hits_on_the_observed_stream(oracle):
    # Observing a stream and selecting H rows must give the H-row set with the most hits on that same
    # stream (no other set of that size can have more: its hits are a sum of H counters), as counted by
    # the cached lookup's own hit accounting.
    rng = np.random.default_rng(120)
    R, D, B, H = 300, 4, 50, 25
    table = rng.standard_normal((R, D)).astype(np.float32)
    lengths = rng.integers(0, 30, size=B).astype(np.int32)
    off, _ = oracle.lengths_to_offsets(lengths)
    rows = np.minimum(rng.zipf(1.2, size=int(off[-1])) - 1, R - 1).astype(np.int64)
    freq = np.zeros(R, np.uint32)
    assert oracle.cache_observe(freq, rows) == 0
    counts = freq.copy()
    hot = oracle.cache_select(freq, H, 0)
    _, _, (hits, misses), st = oracle.bag_forward_cached(table, "f32", hot, rows, off, B, "sum")
    assert st == 0 and hits + misses == rows.size
    assert hits == int(np.sort(counts.astype(np.int64))[-H:].sum())
    other = np.sort(rng.permutation(R)[:H]).astype(np.int64)
    _, _, (hits2, _), _ = oracle.bag_forward_cached(table, "f32", other, rows, off, B, "sum")
    assert hits2 <= hits


# ---------------------------------------------------------------------------
# checksum of table memory
# ---------------------------------------------------------------------------

def test_checksum_closed_forms_and_brute_force(oracle):
    n = 1000
    assert oracle.checksum(np.ones(n, np.uint32)) == n * (n + 1) // 2                    # sum of the weights
    i = np.arange(n, dtype=np.uint32)
    assert oracle.checksum(i) == sum(k * (k + 1) for k in range(n))                      # = (n-1) n (n+1) / 3
    assert oracle.checksum(i) == (n - 1) * n * (n + 1) // 3
    assert oracle.checksum(np.zeros(0, np.uint32)) == 0
    # little-endian words, whatever the element type of the array
    assert oracle.checksum(np.array([1, 0, 0, 0, 0, 1, 0, 0], np.uint8)) == 1 * 1 + 256 * 2
    rng = np.random.default_rng(130)
    w = rng.integers(0, 1 << 32, size=3001, dtype=np.uint64).astype(np.uint32)
    want = sum(int(x) * (k + 1) for k, x in enumerate(w)) % (1 << 64)                    # big integers, then modulo
    assert oracle.checksum(w) == want and want != sum(int(x) for x in w)
    assert oracle.checksum(w.view(np.float32)) == want                                   # the bits, not the values
    big = np.full(70_000, 0xFFFFFFFF, np.uint32)                                         # wraps past 2^64
    assert oracle.checksum(big) == (0xFFFFFFFF * (70_000 * 70_001 // 2)) % (1 << 64)
    sw = w.copy()
    sw[[5, 900]] = sw[[900, 5]]
    assert oracle.checksum(sw) != want                                                   # position matters


def test_cache_select_by_partition_agrees_with_the_sorting_definition(oracle):
    rng = np.random.default_rng(140)
    for R in (1, 2, 37, 1000, 50_001):
        for freq in (rng.integers(0, 3, size=R).astype(np.uint32),
                     np.minimum(rng.zipf(1.2, size=R), 1 << 31).astype(np.uint32),
                     np.full(R, 0xFFFFFFFF, np.uint32), np.zeros(R, np.uint32)):
            for num_hot in sorted({0, 1, R // 20, R // 2, R}):
                a, b = freq.copy(), freq.copy()
                ha = oracle.cache_select(a, num_hot, 2)
                hb = H.cache_select_large(b, num_hot, 2)
                assert np.array_equal(ha, hb) and np.array_equal(a, b)

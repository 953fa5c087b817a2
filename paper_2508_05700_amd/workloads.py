"""Seeded synthetic inputs for the hashed-embedding-table lookup path.

This module only *makes data*: raw 64-bit IDs, bag lengths, upstream gradients
and the contents of the embedding tables.  It holds none of the method's own
arithmetic (no ID hashing, no offsets, no pooling, no optimizer) so that the
HIP library and the CPU oracle can both be fed from it without sharing any
code of the method.

The paper (Section 2.2, "Large Embedding Tables"; Section 3.1) only fixes the
shape of the traffic: several high-cardinality ID features (Pin, user, image
signature, item, advertiser IDs), each mapped through a hashed lookup table of
1e7..1e9 rows, with heavy popularity skew.  Its production logs are private,
so the five workloads below stand in for them.

Table contents are *procedural*: element ``i = row * D + d`` of a table with
seed ``s`` is a pure function of ``(s, i)`` (a counter-based generator, defined
in ``table_element_u64``/``table_values``).  A 40-64 GB table can therefore be
filled on the device by a small kernel, while the CPU side evaluates only the
rows a batch touches, and both hold bit-identical values.
"""
from __future__ import annotations

import dataclasses
import mmap
from typing import Dict, List, Optional

import numpy as np

DEFAULT_SEED = 20250805

# ---------------------------------------------------------------------------
# counter-based generator for table contents
# ---------------------------------------------------------------------------
_FMIX_C1 = np.uint64(0xFF51AFD7ED558CCD)
_FMIX_C2 = np.uint64(0xC4CEB9FE1A85EC53)
_SEED_MUL = np.uint64(0xD1B54A32D192ED03)
_U33 = np.uint64(33)

# The sum of four independent uniform 16-bit integers has mean 2*65535 = 131070
# and standard deviation 2*sqrt((65536^2 - 1)/12) = 37837.2275...; scaling by
# 0.01/37837.2275 gives an Irwin-Hall(4) stand-in for N(0, 0.01^2).
TABLE_CENTER = 131070
TABLE_SCALE = np.float32(0.01 / 37837.227524)


def fmix64(z: np.ndarray) -> np.ndarray:
    """The 64-bit finalizer of MurmurHash3 (a published bijection on u64)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = z ^ (z >> _U33)
        z = z * _FMIX_C1
        z = z ^ (z >> _U33)
        z = z * _FMIX_C2
        z = z ^ (z >> _U33)
    return z


def table_element_u64(seed: int, elem: np.ndarray) -> np.ndarray:
    """64 random bits for element counter ``elem`` of the table with ``seed``."""
    with np.errstate(over="ignore"):
        base = np.uint64((int(seed) + 1) % (1 << 64)) * _SEED_MUL
        return fmix64(np.asarray(elem, dtype=np.uint64) + base)


def table_values(seed: int, rows: np.ndarray, D: int) -> np.ndarray:
    """fp32 contents ``[len(rows), D]`` of the given rows of a procedural table.

    value = TABLE_SCALE * float(s - 131070), s = sum of the four 16-bit fields
    of ``table_element_u64(seed, row * D + d)``; the integer is exact in fp32
    and the product is one correctly rounded fp32 multiply.
    """
    rows = np.asarray(rows, dtype=np.int64).astype(np.uint64)
    with np.errstate(over="ignore"):
        elem = rows[:, None] * np.uint64(D) + np.arange(D, dtype=np.uint64)[None, :]
    z = table_element_u64(seed, elem)
    m = np.uint64(0xFFFF)
    s = (z & m) + ((z >> np.uint64(16)) & m) + ((z >> np.uint64(32)) & m) + (z >> np.uint64(48))
    return (s.astype(np.int64) - TABLE_CENTER).astype(np.float32) * TABLE_SCALE


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); finite inputs only."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def table_rows(seed: int, rows: np.ndarray, D: int, dtype: str) -> np.ndarray:
    """Stored representation (fp32 array, or bf16 bit patterns as uint16)."""
    v = table_values(seed, rows, D)
    if dtype == "f32":
        return v
    if dtype == "bf16":
        return f32_to_bf16_bits(v)
    raise ValueError(dtype)


def dense_table(seed: int, R: int, D: int, dtype: str = "f32", chunk: int = 1 << 18) -> np.ndarray:
    """Materialise a whole (small) table on the host."""
    out = np.empty((R, D), dtype=np.float32 if dtype == "f32" else np.uint16)
    for lo in range(0, R, chunk):
        hi = min(R, lo + chunk)
        out[lo:hi] = table_rows(seed, np.arange(lo, hi, dtype=np.int64), D, dtype)
    return out


def sparse_host_table(seed: int, R: int, D: int, dtype: str, touched_rows: np.ndarray) -> np.ndarray:
    """A full-size ``[R, D]`` host array in which only ``touched_rows`` are filled.

    The array is an anonymous no-reserve mapping, so a 2.5-64 GB table costs
    only the pages that are written.  Rows that were not listed read as zero;
    a caller must list every row it is going to look at.
    """
    np_dtype = np.float32 if dtype == "f32" else np.uint16
    nbytes = int(R) * int(D) * np.dtype(np_dtype).itemsize
    flags = mmap.MAP_PRIVATE | mmap.MAP_ANONYMOUS | getattr(mmap, "MAP_NORESERVE", 0)
    buf = mmap.mmap(-1, max(nbytes, 1), flags=flags)
    arr = np.frombuffer(buf, dtype=np_dtype, count=int(R) * int(D)).reshape(int(R), int(D))
    touched = np.unique(np.asarray(touched_rows, dtype=np.int64))
    step = 1 << 18
    for lo in range(0, touched.size, step):
        sel = touched[lo:lo + step]
        arr[sel] = table_rows(seed, sel, D, dtype)
    return arr


# ---------------------------------------------------------------------------
# bounded Zipf sampler
# ---------------------------------------------------------------------------
class BoundedZipf:
    """Ranks k in 1..N with P(k) proportional to k**-a (a > 1).

    The first ``head`` ranks use the exact cumulative table; the tail uses the
    continuous inverse of the midpoint-rule mass  int_{M+1/2}^{x} t**-a dt.
    """

    def __init__(self, n_keys: int, alpha: float, head: int = 1 << 20):
        self.N = int(n_keys)
        self.a = float(alpha)
        self.M = int(min(head, self.N))
        k = np.arange(1, self.M + 1, dtype=np.float64)
        self.cum = np.cumsum(k ** (-self.a))
        self.head_mass = float(self.cum[-1])
        a1 = self.a - 1.0
        if self.N > self.M:
            self.lo_pow = (self.M + 0.5) ** (-a1)
            self.tail_mass = (self.lo_pow - (self.N + 0.5) ** (-a1)) / a1
        else:
            self.lo_pow = 0.0
            self.tail_mass = 0.0
        self.H = self.head_mass + self.tail_mass

    def prob(self, k: int) -> float:
        return float(k) ** (-self.a) / self.H

    def head_cdf(self, k: int) -> float:
        """P(rank <= k) for k <= head size."""
        return float(self.cum[k - 1]) / self.H

    def sample(self, rng: np.random.Generator, size: int) -> np.ndarray:
        u = rng.random(size) * self.H
        ranks = np.empty(size, dtype=np.int64)
        in_head = u < self.head_mass
        ranks[in_head] = np.searchsorted(self.cum, u[in_head], side="right") + 1
        if self.tail_mass > 0.0:
            t = u[~in_head] - self.head_mass
            a1 = self.a - 1.0
            x = (self.lo_pow - a1 * t) ** (-1.0 / a1)
            ranks[~in_head] = np.clip(np.rint(x), self.M + 1, self.N).astype(np.int64)
        np.clip(ranks, 1, self.N, out=ranks)
        return ranks


def ranks_to_raw_ids(ranks: np.ndarray, stream_key: int) -> np.ndarray:
    """Distinct ranks -> distinct, well-spread raw 64-bit IDs (a bijection)."""
    with np.errstate(over="ignore"):
        return fmix64(np.asarray(ranks, dtype=np.int64).astype(np.uint64) + np.uint64(stream_key % (1 << 64)))


# ---------------------------------------------------------------------------
# workloads
# ---------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    T: int                    # number of tables
    R: int                    # rows per table
    D: int                    # embedding dimension
    dtype: str                # "f32" | "bf16" table storage
    B: int                    # bags per table
    length: str               # "fixed" | "poisson"
    mean_len: float
    max_len: Optional[int]    # clip for poisson lengths (None = no clip)
    ids: str                  # "rows_uniform" | "raw_uniform" | "zipf"
    alpha: float = 0.0
    n_keys: int = 0
    pool: str = "sum"         # "sum" | "mean"
    backward: bool = False
    hybrid: bool = False
    hot_fraction: float = 0.0
    lr: float = 0.01
    eps: float = 1e-8
    # "int8" | "int4" | "int4r64" (INT4 rows padded to 64 bytes): the fp32 tables are stored row-quantised
    # (forward only)
    quant: Optional[str] = None
    streaming: bool = False       # the lookups pass the "rows are not reused" hint (IDs without popular heads)

    def scaled(self, rows: Optional[int] = None, bags: Optional[int] = None,
               tables: Optional[int] = None, n_keys: Optional[int] = None) -> "Workload":
        """Same recipe at a smaller size (for CPU-side and quick GPU tests)."""
        return dataclasses.replace(
            self,
            name=self.name + "-scaled",
            R=self.R if rows is None else int(rows),
            B=self.B if bags is None else int(bags),
            T=self.T if tables is None else int(tables),
            n_keys=self.n_keys if n_keys is None else int(n_keys),
        )

    @property
    def esz(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def storage(self) -> str:
        """Storage type of the table rows the lookups read."""
        return self.quant or self.dtype

    @property
    def codes(self) -> Optional[str]:
        """The quantised encoding without its row padding ("int4r64" holds the rows of "int4")."""
        return "int4" if self.quant == "int4r64" else self.quant

    def table_seed(self, t: int, seed: int = DEFAULT_SEED) -> int:
        return int(seed) * 1000 + int(t)

    def salt(self, t: int) -> int:
        return int(t)


WORKLOADS: Dict[str, Workload] = {
    # 1: single small table, fixed-length bags, row IDs drawn directly (no hashing)
    "1": Workload("1", T=1, R=100_000, D=32, dtype="f32", B=512, length="fixed", mean_len=8,
                  max_len=None, ids="rows_uniform", pool="sum"),
    # 2: 16 tables, Zipf(1.05) over 1e9 keys, mean pooling, forward
    "2": Workload("2", T=16, R=10_000_000, D=64, dtype="f32", B=8192, length="poisson", mean_len=20,
                  max_len=100, ids="zipf", alpha=1.05, n_keys=10 ** 9, pool="mean"),
    # 2u: config 2's shapes with uniformly distributed raw IDs (no reuse: every row read is an HBM read)
    "2u": Workload("2u", T=16, R=10_000_000, D=64, dtype="f32", B=8192, length="poisson", mean_len=20,
                   max_len=100, ids="raw_uniform", pool="mean", streaming=True),
    # 2un: the same without the hint (rows read with ordinary cached loads)
    "2un": Workload("2un", T=16, R=10_000_000, D=64, dtype="f32", B=8192, length="poisson", mean_len=20,
                    max_len=100, ids="raw_uniform", pool="mean"),
    # 3: config 2 plus the sparse row-wise Adagrad backward
    "3": Workload("3", T=16, R=10_000_000, D=64, dtype="f32", B=8192, length="poisson", mean_len=20,
                  max_len=100, ids="zipf", alpha=1.05, n_keys=10 ** 9, pool="mean", backward=True),
    # 3b: workload 3 with the tables stored as bf16 (rows halve; accumulators, gradients and outputs stay fp32)
    "3b": Workload("3b", T=16, R=10_000_000, D=64, dtype="bf16", B=8192, length="poisson", mean_len=20,
                   max_len=100, ids="zipf", alpha=1.05, n_keys=10 ** 9, pool="mean", backward=True),
    # 4: one 1e9-row bf16 table, Zipf(1.2) over 1e12 keys, sum pooling
    "4": Workload("4", T=1, R=1_000_000_000, D=32, dtype="bf16", B=65536, length="poisson", mean_len=50,
                  max_len=None, ids="zipf", alpha=1.2, n_keys=10 ** 12, pool="sum"),
    # 2q4 / 2q8 / 2uq4: config 2 (and its uniform-ID variant) over post-training-quantised tables
    "2q4": Workload("2q4", T=16, R=10_000_000, D=64, dtype="f32", B=8192, length="poisson", mean_len=20,
                    max_len=100, ids="zipf", alpha=1.05, n_keys=10 ** 9, pool="mean", quant="int4"),
    "2q8": Workload("2q8", T=16, R=10_000_000, D=64, dtype="f32", B=8192, length="poisson", mean_len=20,
                    max_len=100, ids="zipf", alpha=1.05, n_keys=10 ** 9, pool="mean", quant="int8"),
    "2uq4": Workload("2uq4", T=16, R=10_000_000, D=64, dtype="f32", B=8192, length="poisson", mean_len=20,
                     max_len=100, ids="raw_uniform", pool="mean", quant="int4"),
    # 2uq4r: 2uq4 with every INT4 row padded from 48 to 64 bytes (no row straddles a 64-byte sector)
    "2uq4r": Workload("2uq4r", T=16, R=10_000_000, D=64, dtype="f32", B=8192, length="poisson", mean_len=20,
                      max_len=100, ids="raw_uniform", pool="mean", quant="int4r64"),
    # 5: host-resident table plus an HBM cache of the hottest 5 % of rows
    "5": Workload("5", T=1, R=250_000_000, D=64, dtype="f32", B=16384, length="poisson", mean_len=30,
                  max_len=None, ids="zipf", alpha=1.1, n_keys=10 ** 9, pool="sum", hybrid=True,
                  hot_fraction=0.05),
    # 5q4: the same with the host table (and the cache) stored as INT4 rows
    "5q4": Workload("5q4", T=1, R=250_000_000, D=64, dtype="f32", B=16384, length="poisson", mean_len=30,
                    max_len=None, ids="zipf", alpha=1.1, n_keys=10 ** 9, pool="sum", hybrid=True,
                    hot_fraction=0.05, quant="int4"),
    # 5m / 5mq4: workload 5's rows and lookups split over four hosted tables (a hosted model has several)
    "5m": Workload("5m", T=4, R=62_500_000, D=64, dtype="f32", B=4096, length="poisson", mean_len=30,
                   max_len=None, ids="zipf", alpha=1.1, n_keys=10 ** 9, pool="sum", hybrid=True,
                   hot_fraction=0.05),
    "5mq4": Workload("5mq4", T=4, R=62_500_000, D=64, dtype="f32", B=4096, length="poisson", mean_len=30,
                     max_len=None, ids="zipf", alpha=1.1, n_keys=10 ** 9, pool="sum", hybrid=True,
                     hot_fraction=0.05, quant="int4"),
}


# "mix": config 2's batch recipe over 24 tables of different width and storage type (D, dtype, rows):
# the kind of table set a ranking model with several ID features has.
MIX_SPEC = ([(16, "f32", 2_000_000)] * 6 + [(32, "bf16", 5_000_000)] * 6 + [(64, "f32", 10_000_000)] * 8 +
            [(128, "f32", 2_000_000)] * 4)
WORKLOADS["mix"] = dataclasses.replace(WORKLOADS["2"], name="mix", T=len(MIX_SPEC), D=0, R=0)


def _rng(seed: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), *[int(k) for k in key]])))


def _stream_key(seed: int, t: int) -> int:
    return (int(seed) * 0x9E3779B1 + 0x51ED27 * (t + 1)) % (1 << 64)


_zipf_cache: Dict[tuple, BoundedZipf] = {}


def zipf_for(w: Workload) -> BoundedZipf:
    key = (w.n_keys, w.alpha)
    if key not in _zipf_cache:
        _zipf_cache[key] = BoundedZipf(w.n_keys, w.alpha)
    return _zipf_cache[key]


def make_lengths(w: Workload, rng: np.random.Generator, n: int) -> np.ndarray:
    if w.length == "fixed":
        return np.full(n, int(w.mean_len), dtype=np.int32)
    L = rng.poisson(w.mean_len, size=n)
    if w.max_len is not None:
        L = np.minimum(L, w.max_len)
    return L.astype(np.int32)


def make_batch(w: Workload, batch_index: int = 0, seed: int = DEFAULT_SEED) -> Dict[str, object]:
    """One batch of inputs for workload ``w`` (numpy arrays on the host).

    Keys: ``lengths`` int32 [T*B] (table-major), ``nnz_per_table`` list,
    ``raw`` uint64 [nnz] (None for workload 1), ``rows`` int64 [nnz] (only for
    workload 1, whose IDs are row numbers already), ``salts`` list of per-table
    salts, ``dout`` fp32 [T, B, D] when the workload has a backward.
    """
    lengths = np.empty(w.T * w.B, dtype=np.int32)
    raws: List[np.ndarray] = []
    rows: List[np.ndarray] = []
    per_table: List[int] = []
    for t in range(w.T):
        rng = _rng(seed, 1, t, batch_index)
        L = make_lengths(w, rng, w.B)
        lengths[t * w.B:(t + 1) * w.B] = L
        n = int(L.sum(dtype=np.int64))
        per_table.append(n)
        if w.ids == "rows_uniform":
            rows.append(rng.integers(0, w.R, size=n, dtype=np.int64))
        elif w.ids == "raw_uniform":
            raws.append(rng.integers(0, 1 << 64, size=n, dtype=np.uint64))
        elif w.ids == "zipf":
            ranks = zipf_for(w).sample(rng, n)
            raws.append(ranks_to_raw_ids(ranks, _stream_key(seed, t)))
        else:
            raise ValueError(w.ids)
    batch: Dict[str, object] = {
        "lengths": lengths,
        "nnz_per_table": per_table,
        "nnz": int(sum(per_table)),
        "salts": [w.salt(t) for t in range(w.T)],
        "raw": np.concatenate(raws) if raws else None,
        "rows": np.concatenate(rows) if rows else None,
    }
    if w.backward:
        batch["dout"] = _rng(seed, 2, batch_index).standard_normal((w.T, w.B, w.D), dtype=np.float32)
    return batch


def traffic_raw_ids(w: Workload, t: int, n: int, chunk_index: int, seed: int = DEFAULT_SEED) -> np.ndarray:
    """``n`` raw IDs of table ``t`` drawn like the lookups of a batch (same Zipf law, same rank -> ID map), as
    one flat stream: the traffic a cache policy watches between refreshes."""
    assert w.ids == "zipf"
    ranks = zipf_for(w).sample(_rng(seed, 3, t, chunk_index), n)
    return ranks_to_raw_ids(ranks, _stream_key(seed, t))


def hot_raw_ids(w: Workload, t: int, n_ranks: int, seed: int = DEFAULT_SEED) -> np.ndarray:
    """Raw IDs of Zipf ranks 1..n_ranks of table ``t`` (most popular first)."""
    ranks = np.arange(1, n_ranks + 1, dtype=np.int64)
    return ranks_to_raw_ids(ranks, _stream_key(seed, t))


def first_k_distinct_sorted(values: np.ndarray, k: int) -> np.ndarray:
    """The first ``k`` distinct entries of ``values`` (in order of first
    appearance), returned sorted ascending.  Used to turn "rows of the most
    popular IDs" into a static hot-row set for the cached table."""
    uniq, first = np.unique(np.asarray(values), return_index=True)
    keep = uniq[np.argsort(first, kind="stable")[:k]]
    return np.sort(keep)

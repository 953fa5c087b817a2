"""ctypes wrapper around the CPU oracle (``emb_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the test suite, the smoke check and the
benchmark's CPU-baseline leg; never by the product path.  It marshals numpy
arrays to the plain-C functions and adds no arithmetic of its own.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "emb_oracle.c")
_LIB = os.path.join(_HERE, "libemb_oracle.so")

POOL = {"sum": 0, "mean": 1}
DTYPE = {"f32": 0, "bf16": 1, "int8": 2, "int4": 3}
STATUS_BAD_INDEX = 1
STATUS_BAD_OFFSETS = 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no optimisation beyond -O2, no OpenMP)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "emb_oracle.h")))
    if force or stale:
        subprocess.check_call(["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, i64, i32, u64, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_float
        L.oracle_splitmix64.restype = u64
        L.oracle_splitmix64.argtypes = [u64]
        L.oracle_hash_ids.restype = None
        L.oracle_hash_ids.argtypes = [vp, i64, u64, i64, vp]
        L.oracle_lengths_to_offsets.restype = None
        L.oracle_lengths_to_offsets.argtypes = [vp, i64, vp, vp]
        L.oracle_quant_row_bytes.restype = i64
        L.oracle_quant_row_bytes.argtypes = [i32, i32]
        L.oracle_quantize_rows.restype = None
        L.oracle_quantize_rows.argtypes = [vp, i64, i32, i32, vp]
        L.oracle_bag_forward.restype = None
        L.oracle_bag_forward.argtypes = [vp, i32, vp, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp]
        L.oracle_bag_backward_rowwise_adagrad.restype = C.c_int
        L.oracle_bag_backward_rowwise_adagrad.argtypes = [
            vp, vp, i32, vp, i32, i32, vp, vp, i64, i64, i32, vp, f32, f32, vp, vp, vp, vp, vp, vp]
        L.oracle_cache_observe.restype = i64
        L.oracle_cache_observe.argtypes = [vp, i64, vp, i64]
        L.oracle_cache_select.restype = C.c_int
        L.oracle_cache_select.argtypes = [vp, i64, i64, i32, vp]
        L.oracle_checksum.restype = u64
        L.oracle_checksum.argtypes = [vp, u64]
        L.oracle_bag_forward_cached.restype = None
        L.oracle_bag_forward_cached.argtypes = [vp, i64, i32, i32, vp, i64, vp, vp, i64, i64, i32,
                                                vp, vp, vp, vp]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a: np.ndarray, dtype) -> np.ndarray:
    assert a.dtype == np.dtype(dtype), (a.dtype, dtype)
    assert a.flags["C_CONTIGUOUS"]
    return a


def _ptr_array(arrs: Sequence[np.ndarray]):
    return (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def _table_np_dtype(dtype: str):
    return {"f32": np.float32, "bf16": np.uint16, "int8": np.uint8, "int4": np.uint8}[dtype]


def quant_row_bytes(D: int, dtype: str) -> int:
    return int(lib().oracle_quant_row_bytes(int(D), DTYPE[dtype]))


def quantize_rows(table: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 [R, D] -> row-quantised storage, uint8 [R, quant_row_bytes(D, dtype)]."""
    table = _chk(np.ascontiguousarray(table), np.float32)
    R, D = table.shape
    rb = quant_row_bytes(D, dtype)
    assert rb > 0
    out = np.empty((R, rb), dtype=np.uint8)
    lib().oracle_quantize_rows(_p(table), R, D, DTYPE[dtype], _p(out))
    return out


def splitmix64(x: int) -> int:
    return int(lib().oracle_splitmix64(C.c_uint64(x % (1 << 64))))


def hash_ids(raw: np.ndarray, salt: int, num_rows: int) -> np.ndarray:
    raw = _chk(np.ascontiguousarray(raw), np.uint64)
    rows = np.empty(raw.size, dtype=np.int64)
    lib().oracle_hash_ids(_p(raw), raw.size, C.c_uint64(salt % (1 << 64)), int(num_rows), _p(rows))
    return rows


def lengths_to_offsets(lengths: np.ndarray) -> Tuple[np.ndarray, int]:
    lengths = _chk(np.ascontiguousarray(lengths), np.int32)
    offsets = np.empty(lengths.size + 1, dtype=np.int64)
    status = np.zeros(1, dtype=np.uint32)
    lib().oracle_lengths_to_offsets(_p(lengths), lengths.size, _p(offsets), _p(status))
    return offsets, int(status[0])


def bag_forward(tables: Sequence[np.ndarray], dtype: str, rows: np.ndarray, offsets: np.ndarray,
                B: int, mode: str, want_absum: bool = True, D: Optional[int] = None):
    """Returns (out fp32 [T,B,D], absum fp64 [T,B,D] or None, status).  Row-quantised tables
    (``int8`` / ``int4``) are uint8 [R, quant_row_bytes] and need ``D``."""
    T = len(tables)
    quant = dtype in ("int8", "int4")
    assert quant == (D is not None)
    width = quant_row_bytes(D, dtype) if quant else int(tables[0].shape[1])
    D = int(D) if quant else width
    for t in tables:
        _chk(t, _table_np_dtype(dtype))
        assert t.shape[1] == width
    rows = _chk(np.ascontiguousarray(rows), np.int64)
    offsets = _chk(np.ascontiguousarray(offsets), np.int64)
    assert offsets.size == T * B + 1
    num_rows = np.array([t.shape[0] for t in tables], dtype=np.int64)
    out = np.empty((T, B, D), dtype=np.float32)
    absum = np.empty((T, B, D), dtype=np.float64) if want_absum else None
    status = np.zeros(1, dtype=np.uint32)
    lib().oracle_bag_forward(_ptr_array(tables), T, _p(num_rows), D, DTYPE[dtype], _p(rows),
                             _p(offsets), B, rows.size, POOL[mode], _p(out), _p(absum), _p(status))
    return out, absum, int(status[0])


def bag_backward_rowwise_adagrad(tables: Sequence[np.ndarray], accum: Sequence[np.ndarray],
                                 dtype: str, rows: np.ndarray, offsets: np.ndarray, B: int,
                                 mode: str, dout: np.ndarray, lr: float, eps: float,
                                 want_G: bool = True):
    """Updates ``tables`` and ``accum`` IN PLACE.

    Returns dict(unique_keys, unique_counts, G, Gabs, status)."""
    T = len(tables)
    D = int(tables[0].shape[1])
    for t, s in zip(tables, accum):
        _chk(t, _table_np_dtype(dtype))
        _chk(s, np.float32)
        assert s.shape == (t.shape[0],)
    rows = _chk(np.ascontiguousarray(rows), np.int64)
    offsets = _chk(np.ascontiguousarray(offsets), np.int64)
    dout = _chk(np.ascontiguousarray(dout), np.float32)
    assert offsets.size == T * B + 1 and dout.size == T * B * D
    nnz = rows.size
    num_rows = np.array([t.shape[0] for t in tables], dtype=np.int64)
    uk = np.empty(max(nnz, 1), dtype=np.int64)
    uc = np.empty(max(nnz, 1), dtype=np.int32)
    nu = np.zeros(1, dtype=np.int64)
    G = np.empty((max(nnz, 1), D), dtype=np.float64) if want_G else None
    Gabs = np.empty((max(nnz, 1), D), dtype=np.float64) if want_G else None
    status = np.zeros(1, dtype=np.uint32)
    rc = lib().oracle_bag_backward_rowwise_adagrad(
        _ptr_array(tables), _ptr_array(accum), T, _p(num_rows), D, DTYPE[dtype], _p(rows),
        _p(offsets), B, nnz, POOL[mode], _p(dout), C.c_float(lr), C.c_float(eps), _p(uk), _p(uc),
        _p(nu), _p(G), _p(Gabs), _p(status))
    if rc != 0:
        raise MemoryError("oracle backward could not allocate")
    U = int(nu[0])
    return {
        "unique_keys": uk[:U].copy(),
        "unique_counts": uc[:U].copy(),
        "G": None if G is None else G[:U].copy(),
        "Gabs": None if Gabs is None else Gabs[:U].copy(),
        "status": int(status[0]),
    }


def bag_forward_cached(table: np.ndarray, dtype: str, hot_rows: np.ndarray, rows: np.ndarray,
                       offsets: np.ndarray, B: int, mode: str, D: Optional[int] = None):
    """Returns (out fp32 [1,B,D], absum, (hits, misses), status).  A row-quantised table
    (``int8`` / ``int4``: uint8 [R, quant_row_bytes]) needs ``D``."""
    _chk(table, _table_np_dtype(dtype))
    quant = dtype in ("int8", "int4")
    assert quant == (D is not None)
    if quant:
        assert table.shape[1] == quant_row_bytes(D, dtype)
    D = int(D) if quant else int(table.shape[1])
    hot_rows = _chk(np.ascontiguousarray(hot_rows), np.int64)
    rows = _chk(np.ascontiguousarray(rows), np.int64)
    offsets = _chk(np.ascontiguousarray(offsets), np.int64)
    assert offsets.size == B + 1
    out = np.empty((1, B, D), dtype=np.float32)
    absum = np.empty((1, B, D), dtype=np.float64)
    hm = np.zeros(2, dtype=np.uint64)
    status = np.zeros(1, dtype=np.uint32)
    lib().oracle_bag_forward_cached(_p(table), table.shape[0], D, DTYPE[dtype], _p(hot_rows),
                                    hot_rows.size, _p(rows), _p(offsets), B, rows.size, POOL[mode],
                                    _p(out), _p(absum), _p(hm), _p(status))
    return out, absum, (int(hm[0]), int(hm[1])), int(status[0])


def cache_observe(freq: np.ndarray, rows: np.ndarray) -> int:
    """freq (uint32 [R], updated in place) += 1 per in-range entry of rows; returns the number out of range."""
    _chk(freq, np.uint32)
    rows = _chk(np.ascontiguousarray(rows), np.int64)
    return int(lib().oracle_cache_observe(_p(freq), freq.size, _p(rows), rows.size))


def cache_select(freq: np.ndarray, num_hot: int, decay_shift: int = 0) -> np.ndarray:
    """The num_hot rows with the largest counters (ties to the smaller row), ascending; freq is aged in place."""
    _chk(freq, np.uint32)
    assert 0 <= num_hot <= freq.size and 0 <= decay_shift <= 31
    hot = np.empty(num_hot, dtype=np.int64)
    rc = lib().oracle_cache_select(_p(freq), freq.size, num_hot, decay_shift, _p(hot))
    assert rc == 0
    return hot


def checksum(a: np.ndarray) -> int:
    """Position-weighted checksum of the array's memory (C-contiguous, a multiple of 4 bytes)."""
    assert a.flags["C_CONTIGUOUS"] and a.nbytes % 4 == 0
    return int(lib().oracle_checksum(_p(a), a.nbytes))

"""ctypes binding of the C ABI in ``include/emb.h``.

Argument marshalling only: every function here has the name of the C entry
point it calls, checks dtype / device / contiguity of the torch tensors it is
given, passes their ``data_ptr()`` and the current HIP stream, and raises
``EmbError`` on a negative status.  No step of the path is computed in Python.
PyTorch is used for device memory and streams.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import build as _build

POOL = {"sum": 0, "mean": 1}
DTYPE = {"f32": 0, "bf16": 1, "int8": 2, "int4": 3, "int4r64": 4}
QUANT_DTYPES = ("int8", "int4", "int4r64")   # row-quantised storage; "int4r64": INT4 rows padded to 64 bytes
ROWS_STREAMING = 0x100   # hint bit for the forward lookups (EMB_ROWS_STREAMING)
STATUS_BAD_INDEX = 1
STATUS_BAD_OFFSETS = 2
STATUS_BAD_HOT_SET = 4
STATUS_NO_VERSION = 8
STATUS_SORT_ABANDONED = 16
BWD_STAGE_EVENTS = 6

# numpy mirror of ``struct emb_table``
TABLE_DESC = np.dtype([("weights", "<u8"), ("accum", "<u8"), ("num_rows", "<i8"), ("row_base", "<i8"),
                       ("salt", "<u8"), ("mod_magic", "<u8")])
assert TABLE_DESC.itemsize == 48

# numpy mirror of ``struct emb_cached_table``
CACHED_DESC = np.dtype([("table", "<u8"), ("cache_rows", "<u8"), ("cache_index", "<u8"), ("num_rows", "<i8"),
                        ("num_hot", "<i8"), ("salt", "<u8"), ("mod_magic", "<u8"), ("reserved", "<u8")])
assert CACHED_DESC.itemsize == 64

# numpy mirror of ``struct emb_table_shape``
SHAPE_DESC = np.dtype([("D", "<i4"), ("dtype", "<i4"), ("out_offset", "<i8"), ("out_stride", "<i8"),
                       ("first_block", "<u4"), ("lanes", "<i4")])
assert SHAPE_DESC.itemsize == 32

EXPORTS = [
    "emb_status_string", "emb_tables_init", "emb_hash_ids", "emb_hash_ids_tables", "emb_lengths_to_offsets",
    "emb_bag_forward", "emb_bag_forward_hashed", "emb_table_shapes_init", "emb_bag_forward_mixed", "emb_bag_backward_workspace_bytes", "emb_bag_backward_rowwise_adagrad",
    "emb_bag_backward_sort", "emb_debug_sort_poll_limit", "emb_bag_backward_update", "emb_bag_forward_train", "emb_bag_forward_train_lengths", "emb_offsets_scratch_bytes", "emb_bag_forward_hashed_lengths", "emb_bag_backward_sort_prepared", "emb_row_bytes", "emb_quantize_rows",
    "emb_side_stream_create", "emb_side_stream_destroy", "emb_side_stream_join", "emb_bag_forward_train_lengths_after", "emb_event_create", "emb_event_destroy", "emb_event_record",
    "emb_event_elapsed_ms",
    "emb_cache_index_bytes", "emb_cache_build", "emb_bag_forward_cached", "emb_bag_forward_cached_hashed", "emb_bag_forward_cached_hashed_lengths", "emb_host_device_pointer",
    "emb_cache_stage_misses", "emb_cache_stage_misses_hashed", "emb_bag_forward_staged",
    "emb_version_record_bytes", "emb_version_latch_bytes", "emb_version_record_write", "emb_version_publish",
    "emb_version_latch", "emb_bag_forward_latched", "emb_bag_forward_latched_hashed",
    "emb_version_hosted_record_bytes", "emb_version_hosted_latch_bytes", "emb_version_hosted_record_write",
    "emb_version_hosted_latch", "emb_bag_forward_cached_latched", "emb_bag_forward_cached_latched_hashed",
    "emb_cached_tables_init", "emb_bag_forward_cached_tables", "emb_bag_forward_cached_tables_hashed", "emb_bag_forward_cached_tables_hashed_lengths",
    "emb_cache_observe", "emb_cache_observe_hashed", "emb_cache_select_workspace_bytes", "emb_cache_select", "emb_cache_select_static",
    "emb_cache_rebuild",
    "emb_table_fill", "emb_checksum",
]


class EmbError(RuntimeError):
    def __init__(self, fn: str, code: int):
        self.code = code
        name = lib().emb_status_string(code).decode()
        super().__init__(f"{fn} failed: {name} ({code})")


_lib = None


def lib_path() -> str:
    return _build.LIB


def lib() -> C.CDLL:
    """Load ``libemb_hip.so``; build it first if no built library exists or if a
    kernel source or header is newer than the built one (where the sources are
    present and a compiler is at hand: a stale library is never loaded silently).
    There is no fallback: without the HIP library nothing in this package works."""
    global _lib
    if _lib is not None:
        return _lib
    if _build.is_stale():
        if os.path.exists(_build.LIB) and not os.path.exists(_build.HIPCC):
            raise RuntimeError("libemb_hip.so is older than its sources and no hipcc is here to rebuild it")
        _build.build(verbose=False)
    L = C.CDLL(_build.LIB)
    vp, i64, i32, u64, f32, sz = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_float, C.c_size_t
    L.emb_status_string.restype = C.c_char_p
    L.emb_status_string.argtypes = [C.c_int]
    L.emb_tables_init.restype = C.c_int
    L.emb_tables_init.argtypes = [vp, i32]
    L.emb_hash_ids.restype = C.c_int
    L.emb_hash_ids.argtypes = [vp, i64, u64, i64, vp, vp]
    L.emb_hash_ids_tables.restype = C.c_int
    L.emb_hash_ids_tables.argtypes = [vp, vp, i32, vp, vp, i64, i64, vp, vp, vp]
    L.emb_lengths_to_offsets.restype = C.c_int
    L.emb_lengths_to_offsets.argtypes = [vp, i64, vp, vp, vp]
    L.emb_bag_forward.restype = C.c_int
    L.emb_bag_forward.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp]
    L.emb_bag_forward_hashed.restype = C.c_int
    L.emb_bag_forward_hashed.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    L.emb_table_shapes_init.restype = C.c_int
    L.emb_table_shapes_init.argtypes = [vp, i32, i64]
    L.emb_bag_forward_mixed.restype = C.c_int
    L.emb_bag_forward_mixed.argtypes = [vp, vp, vp, vp, i32, vp, vp, i64, i64, i32, vp, i64, vp, vp]
    L.emb_bag_backward_workspace_bytes.restype = sz
    L.emb_bag_backward_workspace_bytes.argtypes = [i32, i64, i64, i64, i32, i32]
    L.emb_bag_backward_rowwise_adagrad.restype = C.c_int
    L.emb_bag_backward_rowwise_adagrad.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, f32, f32,
                                                   vp, sz, vp, vp, vp, vp, vp, vp, vp]
    L.emb_bag_backward_sort.restype = C.c_int
    L.emb_bag_backward_sort.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, sz, vp, vp, vp, vp, vp, vp]
    L.emb_bag_forward_train.restype = C.c_int
    L.emb_bag_forward_train.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp, sz, vp, vp, vp]
    L.emb_debug_sort_poll_limit.restype = None
    L.emb_debug_sort_poll_limit.argtypes = [i64]
    L.emb_offsets_scratch_bytes.restype = sz
    L.emb_offsets_scratch_bytes.argtypes = [i64]
    L.emb_bag_forward_hashed_lengths.restype = C.c_int
    L.emb_bag_forward_hashed_lengths.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp, vp, sz, vp, vp]
    L.emb_bag_forward_train_lengths.restype = C.c_int
    L.emb_bag_forward_train_lengths.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp, vp, sz, vp, vp, vp]
    L.emb_bag_backward_sort_prepared.restype = C.c_int
    L.emb_bag_backward_sort_prepared.argtypes = [vp, vp, i32, i32, i32, i64, i64, vp, sz, vp, vp, vp, vp, vp, vp]
    L.emb_bag_backward_update.restype = C.c_int
    L.emb_bag_backward_update.argtypes = [vp, vp, i32, i32, i32, i64, i64, vp, f32, f32, vp, sz, vp, vp, vp, vp]
    L.emb_side_stream_create.restype = C.c_int
    L.emb_side_stream_create.argtypes = [vp]
    L.emb_side_stream_join.restype = C.c_int
    L.emb_side_stream_join.argtypes = [vp, vp]
    L.emb_bag_forward_train_lengths_after.restype = C.c_int
    L.emb_bag_forward_train_lengths_after.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp, vp, sz, vp,
                                                      vp, vp, vp]
    L.emb_side_stream_destroy.restype = C.c_int
    L.emb_side_stream_destroy.argtypes = [vp]
    L.emb_event_create.restype = C.c_int
    L.emb_event_create.argtypes = [C.POINTER(vp), i32]
    L.emb_event_destroy.restype = C.c_int
    L.emb_event_destroy.argtypes = [vp]
    L.emb_event_record.restype = C.c_int
    L.emb_event_record.argtypes = [vp, vp]
    L.emb_event_elapsed_ms.restype = C.c_int
    L.emb_event_elapsed_ms.argtypes = [vp, vp, C.POINTER(f32)]
    L.emb_row_bytes.restype = i64
    L.emb_row_bytes.argtypes = [i32, i32]
    L.emb_quantize_rows.restype = C.c_int
    L.emb_quantize_rows.argtypes = [vp, i64, i32, i32, vp, vp]
    L.emb_cache_index_bytes.restype = C.c_int
    L.emb_cache_index_bytes.argtypes = [i64, C.POINTER(sz)]
    L.emb_cache_build.restype = C.c_int
    L.emb_cache_build.argtypes = [vp, i64, i32, i32, vp, i64, vp, vp, vp, vp]
    L.emb_bag_forward_cached.restype = C.c_int
    L.emb_bag_forward_cached.argtypes = [vp, i64, i32, i32, vp, vp, i64, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    L.emb_bag_forward_cached_hashed.restype = C.c_int
    L.emb_bag_forward_cached_hashed.argtypes = [vp, i64, i32, i32, vp, vp, i64, u64, vp, vp, i64, i64, i32, vp, vp, vp,
                                                vp]
    L.emb_cache_observe.restype = C.c_int
    L.emb_cache_observe.argtypes = [i64, vp, i64, vp, vp, vp]
    L.emb_cache_observe_hashed.restype = C.c_int
    L.emb_cache_observe_hashed.argtypes = [i64, u64, vp, i64, vp, vp, vp]
    L.emb_cache_select_workspace_bytes.restype = C.c_int
    L.emb_cache_select_workspace_bytes.argtypes = [i64, C.POINTER(sz)]
    L.emb_cache_select.restype = C.c_int
    L.emb_cache_select.argtypes = [vp, i64, i64, i32, vp, sz, vp, vp, vp]
    for fn in ("emb_version_hosted_record_bytes", "emb_version_hosted_latch_bytes"):
        getattr(L, fn).restype = C.c_int
        getattr(L, fn).argtypes = [i32, C.POINTER(sz)]
    L.emb_version_hosted_record_write.restype = C.c_int
    L.emb_version_hosted_record_write.argtypes = [vp, vp, vp, i32, u64, vp]
    L.emb_version_hosted_latch.restype = C.c_int
    L.emb_version_hosted_latch.argtypes = [vp, i32, vp, vp, vp]
    for fn in ("emb_bag_forward_cached_latched", "emb_bag_forward_cached_latched_hashed"):
        getattr(L, fn).restype = C.c_int
        getattr(L, fn).argtypes = [vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    L.emb_cache_stage_misses.restype = C.c_int
    L.emb_cache_stage_misses.argtypes = [vp, i64, i32, i32, vp, i64, vp, i64, vp, i64, vp, vp, vp, vp]
    L.emb_cache_stage_misses_hashed.restype = C.c_int
    L.emb_cache_stage_misses_hashed.argtypes = [vp, i64, i32, i32, vp, i64, u64, vp, i64, vp, i64, vp, vp, vp, vp]
    L.emb_bag_forward_staged.restype = C.c_int
    L.emb_bag_forward_staged.argtypes = [vp, i64, i32, i32, vp, i64, vp, i64, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    L.emb_cache_select_static.restype = C.c_int
    L.emb_cache_select_static.argtypes = [vp, i64, i64, i32, vp, vp, vp]
    L.emb_cache_rebuild.restype = C.c_int
    L.emb_cache_rebuild.argtypes = [vp, i64, i32, i32, vp, vp, i64, vp, i64, vp, vp, vp, vp, vp]
    L.emb_version_record_bytes.restype = C.c_int
    L.emb_version_record_bytes.argtypes = [i32, C.POINTER(sz)]
    L.emb_version_latch_bytes.restype = C.c_int
    L.emb_version_latch_bytes.argtypes = [i32, C.POINTER(sz)]
    L.emb_version_record_write.restype = C.c_int
    L.emb_version_record_write.argtypes = [vp, vp, vp, i32, u64, vp]
    L.emb_version_publish.restype = C.c_int
    L.emb_version_publish.argtypes = [vp, vp, vp]
    L.emb_version_latch.restype = C.c_int
    L.emb_version_latch.argtypes = [vp, i32, vp, vp, vp]
    L.emb_bag_forward_latched.restype = C.c_int
    L.emb_bag_forward_latched.argtypes = [vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp]
    L.emb_bag_forward_latched_hashed.restype = C.c_int
    L.emb_bag_forward_latched_hashed.argtypes = [vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp]
    L.emb_cached_tables_init.restype = C.c_int
    L.emb_cached_tables_init.argtypes = [vp, i32]
    L.emb_bag_forward_cached_tables.restype = C.c_int
    L.emb_bag_forward_cached_tables.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    L.emb_bag_forward_cached_tables_hashed_lengths.restype = C.c_int
    L.emb_bag_forward_cached_tables_hashed_lengths.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp,
                                                               sz, vp, vp, vp, vp]
    L.emb_bag_forward_cached_hashed_lengths.restype = C.c_int
    L.emb_bag_forward_cached_hashed_lengths.argtypes = [vp, i64, i32, i32, vp, vp, i64, u64, vp, vp, i64, i64, i32, vp,
                                                        vp, vp, sz, vp, vp, vp, vp]
    L.emb_bag_forward_cached_tables_hashed.restype = C.c_int
    L.emb_bag_forward_cached_tables_hashed.argtypes = [vp, vp, i32, i32, i32, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    L.emb_checksum.restype = C.c_int
    L.emb_checksum.argtypes = [vp, u64, vp, vp]
    L.emb_host_device_pointer.restype = C.c_int
    L.emb_host_device_pointer.argtypes = [vp, C.POINTER(vp)]
    L.emb_table_fill.restype = C.c_int
    L.emb_table_fill.argtypes = [vp, i64, i32, i32, u64, vp]
    _lib = L
    return L


# ---------------------------------------------------------------------------
# marshalling helpers
# ---------------------------------------------------------------------------
def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor], dtype=None, name: str = "tensor") -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise TypeError(f"{name} must be contiguous")
    if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return int(t.data_ptr())


def _check(fn: str, rc: int) -> None:
    if rc != 0:
        raise EmbError(fn, rc)


_U64 = (torch.int64, torch.uint64)
_TABLE_TORCH = {"f32": torch.float32, "bf16": torch.bfloat16, "int8": torch.uint8, "int4": torch.uint8,
                "int4r64": torch.uint8}


class TableSet:
    """The ``emb_table`` descriptor array of T tables, on the host and on the device.

    ``weights[t]`` is a device tensor ``[R_t, D]`` (fp32 or bf16; uint8
    ``[R_t, emb_row_bytes]`` for the quantised types) or, for memory that torch
    does not own (mapped host memory), a tuple ``(ptr, num_rows)``.
    ``accum[t]`` is a device fp32 tensor ``[R_t]`` or None.
    """

    def __init__(self, weights: Sequence, D: int, dtype: str, accum: Optional[Sequence] = None,
                 salts: Optional[Sequence[int]] = None, device: Optional[torch.device] = None):
        self.T = len(weights)
        self.D = int(D)
        self.dtype = dtype
        self.weights = list(weights)
        self.accum = list(accum) if accum is not None else [None] * self.T
        self.host = np.zeros(self.T, dtype=TABLE_DESC)
        for t, w in enumerate(self.weights):
            if isinstance(w, tuple):
                ptr, rows = int(w[0]), int(w[1])
            else:
                width = emb_row_bytes(self.D, dtype) if dtype in QUANT_DTYPES else self.D
                if w.dim() != 2 or w.shape[1] != width:
                    raise TypeError("weights[%d] must be [num_rows, %d]" % (t, width))
                ptr, rows = _ptr(w, _TABLE_TORCH[dtype], "weights[%d]" % t), int(w.shape[0])
            self.host["weights"][t] = ptr
            self.host["num_rows"][t] = rows
            a = self.accum[t]
            if a is not None:
                if a.numel() != rows:
                    raise TypeError("accum[%d] must have num_rows elements" % t)
                self.host["accum"][t] = _ptr(a, torch.float32, "accum[%d]" % t)
            self.host["salt"][t] = (int(salts[t]) if salts is not None else t) % (1 << 64)
        _check("emb_tables_init", lib().emb_tables_init(self.host.ctypes.data, self.T))
        self.total_rows = int(self.host["num_rows"].sum()) if self.T else 0
        if device is None:
            device = torch.device("cuda", torch.cuda.current_device())
        raw = torch.from_numpy(self.host.view(np.uint8).reshape(-1).copy())
        self.dev = raw.to(device) if self.T else torch.empty(0, dtype=torch.uint8, device=device)

    @property
    def host_ptr(self) -> int:
        return int(self.host.ctypes.data)

    @property
    def dev_ptr(self) -> int:
        return int(self.dev.data_ptr())


# ---------------------------------------------------------------------------
# the entry points
# ---------------------------------------------------------------------------
def emb_hash_ids(raw: torch.Tensor, salt: int, num_rows: int, rows: torch.Tensor) -> None:
    n = raw.numel()
    if rows.numel() != n:
        raise TypeError("rows must have as many elements as raw")
    _check("emb_hash_ids", lib().emb_hash_ids(_ptr(raw, _U64, "raw"), n, C.c_uint64(int(salt) % (1 << 64)),
                                              int(num_rows), _ptr(rows, torch.int64, "rows"), _stream()))


def emb_hash_ids_tables(tables: TableSet, raw: torch.Tensor, offsets: torch.Tensor, B: int, rows: torch.Tensor,
                        status: Optional[torch.Tensor] = None) -> None:
    nnz = raw.numel()
    if rows.numel() != nnz or offsets.numel() != tables.T * B + 1:
        raise TypeError("shape mismatch")
    _check("emb_hash_ids_tables", lib().emb_hash_ids_tables(
        tables.host_ptr, tables.dev_ptr, tables.T, _ptr(raw, _U64, "raw"), _ptr(offsets, torch.int64, "offsets"),
        int(B), nnz, _ptr(rows, torch.int64, "rows"), _ptr(status, torch.int32, "status"), _stream()))


def emb_lengths_to_offsets(lengths: torch.Tensor, offsets: torch.Tensor, status: Optional[torch.Tensor] = None) -> None:
    n = lengths.numel()
    if offsets.numel() != n + 1:
        raise TypeError("offsets must have lengths.numel() + 1 elements")
    _check("emb_lengths_to_offsets", lib().emb_lengths_to_offsets(
        _ptr(lengths, torch.int32, "lengths") if n else None, n, _ptr(offsets, torch.int64, "offsets"),
        _ptr(status, torch.int32, "status"), _stream()))


def emb_bag_forward(tables: TableSet, rows: torch.Tensor, offsets: torch.Tensor, B: int, mode: str,
                    out: torch.Tensor, status: Optional[torch.Tensor] = None, streaming: bool = False) -> None:
    """``streaming``: the EMB_ROWS_STREAMING hint (rows of this batch are unlikely to be reused)."""
    if offsets.numel() != tables.T * B + 1 or out.numel() != tables.T * B * tables.D:
        raise TypeError("shape mismatch")
    _check("emb_bag_forward", lib().emb_bag_forward(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype],
        _ptr(rows, torch.int64, "rows"), _ptr(offsets, torch.int64, "offsets"), int(B), rows.numel(),
        POOL[mode] | (ROWS_STREAMING if streaming else 0),
        _ptr(out, torch.float32, "out"), _ptr(status, torch.int32, "status"), _stream()))


def emb_bag_forward_hashed(tables: TableSet, raw: torch.Tensor, offsets: torch.Tensor, B: int, mode: str,
                           out: torch.Tensor, rows_out: Optional[torch.Tensor] = None,
                           status: Optional[torch.Tensor] = None, streaming: bool = False) -> None:
    """Hashing and pooled lookup in one pass; ``rows_out`` (int64 [nnz]) receives the row numbers."""
    nnz = raw.numel()
    if offsets.numel() != tables.T * B + 1 or out.numel() != tables.T * B * tables.D:
        raise TypeError("shape mismatch")
    if rows_out is not None and rows_out.numel() != nnz:
        raise TypeError("rows_out must have as many elements as raw")
    _check("emb_bag_forward_hashed", lib().emb_bag_forward_hashed(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype], _ptr(raw, _U64, "raw"),
        _ptr(offsets, torch.int64, "offsets"), int(B), nnz, POOL[mode] | (ROWS_STREAMING if streaming else 0),
        _ptr(out, torch.float32, "out"), _ptr(rows_out, torch.int64, "rows_out"), _ptr(status, torch.int32, "status"),
        _stream()))


def emb_debug_sort_poll_limit(polls: int) -> None:
    """Test hook: how often a pass of the backward's sort polls another workgroup's word before it abandons the
    sort (0: every wait fails at once; negative: the default)."""
    lib().emb_debug_sort_poll_limit(int(polls))


def emb_offsets_scratch_bytes(num_bags_total: int) -> int:
    return int(lib().emb_offsets_scratch_bytes(int(num_bags_total)))


def emb_bag_forward_hashed_lengths(tables: TableSet, raw: torch.Tensor, lengths: torch.Tensor, B: int, mode: str,
                                   out: torch.Tensor, offsets_out: torch.Tensor, scratch: torch.Tensor,
                                   rows_out: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None,
                                   streaming: bool = False) -> None:
    """``emb_lengths_to_offsets`` + ``emb_bag_forward_hashed`` in one call: takes the bag lengths, writes the
    offsets; ``scratch`` holds ``emb_offsets_scratch_bytes(T * B)`` bytes."""
    nnz = raw.numel()
    n = tables.T * B
    if lengths.numel() != n or offsets_out.numel() != n + 1 or out.numel() != n * tables.D:
        raise TypeError("shape mismatch")
    if rows_out is not None and rows_out.numel() != nnz:
        raise TypeError("rows_out must have as many elements as raw")
    _check("emb_bag_forward_hashed_lengths", lib().emb_bag_forward_hashed_lengths(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype], _ptr(raw, _U64, "raw"),
        _ptr(lengths, torch.int32, "lengths") if n else None, int(B), nnz,
        POOL[mode] | (ROWS_STREAMING if streaming else 0), _ptr(out, torch.float32, "out"),
        _ptr(offsets_out, torch.int64, "offsets_out"), _ptr(rows_out, torch.int64, "rows_out"),
        _ptr(scratch, torch.uint8, "scratch"), scratch.numel(), _ptr(status, torch.int32, "status"), _stream()))


class MixedTables:
    """Tables of different width / storage type for ``emb_bag_forward_mixed``.

    ``weights[t]`` is a device tensor ``[R_t, D_t]`` (fp32 or bf16).  ``layout``: "table_major" puts
    table t's pooled rows in a ``[B, D_t]`` block of their own, one block after the other;
    "concat" gives one row of ``sum(D_t)`` floats per sample with the tables side by side.
    """

    def __init__(self, weights: Sequence[torch.Tensor], B: int, layout: str = "concat",
                 salts: Optional[Sequence[int]] = None, device: Optional[torch.device] = None):
        self.T = len(weights)
        self.B = int(B)
        self.weights = list(weights)
        names = {torch.float32: "f32", torch.bfloat16: "bf16"}
        self.Ds = [int(w.shape[1]) for w in weights]
        self.dtypes = [names[w.dtype] for w in weights]
        self.tables = TableSet([(_ptr(w, None, "weights"), int(w.shape[0])) for w in weights], 0, "f32", salts=salts,
                               device=device)
        self.host = np.zeros(self.T, dtype=SHAPE_DESC)
        total = sum(self.Ds)
        col = 0
        for t in range(self.T):
            self.host["D"][t] = self.Ds[t]
            self.host["dtype"][t] = DTYPE[self.dtypes[t]]
            if layout == "concat":
                self.host["out_offset"][t], self.host["out_stride"][t] = col, total
            elif layout == "table_major":
                self.host["out_offset"][t], self.host["out_stride"][t] = col * self.B, self.Ds[t]
            else:
                raise ValueError(layout)
            col += self.Ds[t]
        self.layout = layout
        self.out_floats = total * self.B
        _check("emb_table_shapes_init", lib().emb_table_shapes_init(self.host.ctypes.data, self.T, self.B))
        dev = self.tables.dev.device
        self.dev = torch.from_numpy(self.host.view(np.uint8).reshape(-1).copy()).to(dev)


def emb_bag_forward_mixed(mt: MixedTables, rows: torch.Tensor, offsets: torch.Tensor, mode: str, out: torch.Tensor,
                          status: Optional[torch.Tensor] = None) -> None:
    if offsets.numel() != mt.T * mt.B + 1 or out.numel() < mt.out_floats:
        raise TypeError("shape mismatch")
    _check("emb_bag_forward_mixed", lib().emb_bag_forward_mixed(
        mt.tables.host_ptr, mt.tables.dev_ptr, int(mt.host.ctypes.data), int(mt.dev.data_ptr()), mt.T,
        _ptr(rows, torch.int64, "rows"), _ptr(offsets, torch.int64, "offsets"), mt.B, rows.numel(), POOL[mode],
        _ptr(out, torch.float32, "out"), out.numel(), _ptr(status, torch.int32, "status"), _stream()))


def emb_row_bytes(D: int, dtype: str) -> int:
    return int(lib().emb_row_bytes(int(D), DTYPE[dtype]))


def emb_quantize_rows(src: torch.Tensor, dtype: str, dst) -> None:
    """fp32 ``src`` [R, D] -> row-quantised ``dst``: a device tensor uint8 [R, emb_row_bytes(D, dtype)],
    or a raw device-visible pointer (int) to that many bytes, e.g. mapped host memory."""
    R, D = int(src.shape[0]), int(src.shape[1])
    if isinstance(dst, int):
        dptr = dst
    else:
        if dst.numel() != R * emb_row_bytes(D, dtype):
            raise TypeError("dst must hold R * emb_row_bytes bytes")
        dptr = _ptr(dst, torch.uint8, "dst")
    _check("emb_quantize_rows", lib().emb_quantize_rows(_ptr(src, torch.float32, "src"), R, D, DTYPE[dtype], dptr,
                                                        _stream()))


def emb_bag_backward_workspace_bytes(T: int, B: int, nnz: int, total_rows: int, D: int, dtype: str) -> int:
    return int(lib().emb_bag_backward_workspace_bytes(int(T), int(B), int(nnz), int(total_rows), int(D),
                                                      DTYPE[dtype]))


class _SideStreamC(C.Structure):
    _fields_ = [("stream", C.c_void_p), ("fork_event", C.c_void_p), ("join_event", C.c_void_p),
                ("defer_join", C.c_int32), ("reserved", C.c_int32)]


class SideStream:
    """The ``emb_side_stream`` argument, made by ``emb_side_stream_create`` (a stream of default
    priority and two events that release to device scope) on the current device and destroyed with
    this object."""

    def __init__(self, device: Optional[torch.device] = None):
        self.c = _SideStreamC()
        with torch.cuda.device(device if device is not None else torch.cuda.current_device()):
            _check("emb_side_stream_create", lib().emb_side_stream_create(C.addressof(self.c)))

    @property
    def defer_join(self) -> bool:
        """True: a backward leaves its long-run work pending on this stream; the caller joins later
        (``join``, or ``emb_bag_forward_train_lengths_after``) and alternates workspaces."""
        return bool(self.c.defer_join)

    @defer_join.setter
    def defer_join(self, on: bool) -> None:
        self.c.defer_join = 1 if on else 0

    def join(self) -> None:
        """Make the current stream wait for what the last backward left on this stream."""
        _check("emb_side_stream_join", lib().emb_side_stream_join(C.addressof(self.c), _stream()))

    def __del__(self):
        try:
            lib().emb_side_stream_destroy(C.addressof(self.c))
        except Exception:
            pass


class Event:
    """A HIP event with device-scope release (``emb_event_create``); ``cuda_event`` is its handle,
    so it can be passed where a torch event is accepted by this module."""

    def __init__(self, timing: bool = True):
        h = C.c_void_p()
        _check("emb_event_create", lib().emb_event_create(C.byref(h), 1 if timing else 0))
        self.cuda_event = int(h.value)

    def record(self, stream: Optional[torch.cuda.Stream] = None) -> None:
        s = _stream() if stream is None else int(stream.cuda_stream)
        _check("emb_event_record", lib().emb_event_record(self.cuda_event, s))

    def elapsed_time(self, end: "Event") -> float:
        ms = C.c_float()
        _check("emb_event_elapsed_ms", lib().emb_event_elapsed_ms(self.cuda_event, end.cuda_event, C.byref(ms)))
        return float(ms.value)

    def __del__(self):
        try:
            lib().emb_event_destroy(self.cuda_event)
        except Exception:
            pass


def _lookup_events(events):
    """Two events (each may be None) recorded around the lookup kernel of a call that launches two."""
    if events is None:
        return None
    if len(events) != 2:
        raise TypeError("lookup_events must hold 2 events")
    return (C.c_void_p * 2)(*[None if e is None else int(e.cuda_event) for e in events])


def _stage_events(stage_events):
    if stage_events is None:
        return None
    if len(stage_events) != BWD_STAGE_EVENTS:
        raise TypeError("stage_events must hold %d events" % BWD_STAGE_EVENTS)
    return (C.c_void_p * BWD_STAGE_EVENTS)(*[None if e is None else int(e.cuda_event) for e in stage_events])


def emb_bag_backward_sort(tables: TableSet, rows: torch.Tensor, offsets: torch.Tensor, B: int, mode: str,
                          workspace: torch.Tensor, unique_keys: Optional[torch.Tensor] = None,
                          unique_counts: Optional[torch.Tensor] = None, num_unique: Optional[torch.Tensor] = None,
                          status: Optional[torch.Tensor] = None,
                          stage_events: Optional[Sequence[torch.cuda.Event]] = None) -> None:
    """First half of the backward (indices only); see emb_bag_backward_rowwise_adagrad."""
    nnz = rows.numel()
    if offsets.numel() != tables.T * B + 1:
        raise TypeError("shape mismatch")
    for t, name in ((unique_keys, "unique_keys"), (unique_counts, "unique_counts")):
        if t is not None and t.numel() < nnz:
            raise TypeError(name + " must hold at least nnz elements")
    _check("emb_bag_backward_sort", lib().emb_bag_backward_sort(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype],
        _ptr(rows, torch.int64, "rows"), _ptr(offsets, torch.int64, "offsets"), int(B), nnz, POOL[mode],
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _ptr(unique_keys, torch.int64, "unique_keys"), _ptr(unique_counts, torch.int32, "unique_counts"),
        _ptr(num_unique, torch.int64, "num_unique"), _ptr(status, torch.int32, "status"),
        _stage_events(stage_events), _stream()))


def emb_bag_forward_train(tables: TableSet, raw: torch.Tensor, offsets: torch.Tensor, B: int, mode: str,
                          out: torch.Tensor, workspace: torch.Tensor, rows_out: Optional[torch.Tensor] = None,
                          num_unique: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None) -> None:
    """The lookup of a training step: hashing, pooling, and the backward's records into ``workspace``."""
    nnz = raw.numel()
    if offsets.numel() != tables.T * B + 1 or out.numel() != tables.T * B * tables.D:
        raise TypeError("shape mismatch")
    if rows_out is not None and rows_out.numel() != nnz:
        raise TypeError("rows_out must have as many elements as raw")
    _check("emb_bag_forward_train", lib().emb_bag_forward_train(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype], _ptr(raw, _U64, "raw"),
        _ptr(offsets, torch.int64, "offsets"), int(B), nnz, POOL[mode], _ptr(out, torch.float32, "out"),
        _ptr(rows_out, torch.int64, "rows_out"), _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _ptr(num_unique, torch.int64, "num_unique"), _ptr(status, torch.int32, "status"), _stream()))


def emb_bag_forward_train_lengths(tables: TableSet, raw: torch.Tensor, lengths: torch.Tensor, B: int, mode: str,
                                  out: torch.Tensor, offsets_out: torch.Tensor, workspace: torch.Tensor,
                                  rows_out: Optional[torch.Tensor] = None, num_unique: Optional[torch.Tensor] = None,
                                  status: Optional[torch.Tensor] = None) -> None:
    """``emb_lengths_to_offsets`` + ``emb_bag_forward_train`` in one call: takes the bag lengths, writes the offsets."""
    nnz = raw.numel()
    n = tables.T * B
    if lengths.numel() != n or offsets_out.numel() != n + 1 or out.numel() != n * tables.D:
        raise TypeError("shape mismatch")
    if rows_out is not None and rows_out.numel() != nnz:
        raise TypeError("rows_out must have as many elements as raw")
    _check("emb_bag_forward_train_lengths", lib().emb_bag_forward_train_lengths(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype], _ptr(raw, _U64, "raw"),
        _ptr(lengths, torch.int32, "lengths") if n else None, int(B), nnz, POOL[mode], _ptr(out, torch.float32, "out"),
        _ptr(offsets_out, torch.int64, "offsets_out"), _ptr(rows_out, torch.int64, "rows_out"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _ptr(num_unique, torch.int64, "num_unique"),
        _ptr(status, torch.int32, "status"), _stream()))


def emb_bag_forward_train_lengths_after(tables: TableSet, raw: torch.Tensor, lengths: torch.Tensor, B: int, mode: str,
                                        out: torch.Tensor, offsets_out: torch.Tensor, workspace: torch.Tensor,
                                        after: Optional["SideStream"], rows_out: Optional[torch.Tensor] = None,
                                        num_unique: Optional[torch.Tensor] = None,
                                        status: Optional[torch.Tensor] = None) -> None:
    """``emb_bag_forward_train_lengths`` that waits, just before its lookup, for the work a backward with a
    deferred join left on ``after``; ``workspace`` and ``num_unique`` are not that backward's."""
    nnz = raw.numel()
    n = tables.T * B
    if lengths.numel() != n or offsets_out.numel() != n + 1 or out.numel() != n * tables.D:
        raise TypeError("shape mismatch")
    if rows_out is not None and rows_out.numel() != nnz:
        raise TypeError("rows_out must have as many elements as raw")
    _check("emb_bag_forward_train_lengths_after", lib().emb_bag_forward_train_lengths_after(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype], _ptr(raw, _U64, "raw"),
        _ptr(lengths, torch.int32, "lengths") if n else None, int(B), nnz, POOL[mode], _ptr(out, torch.float32, "out"),
        _ptr(offsets_out, torch.int64, "offsets_out"), _ptr(rows_out, torch.int64, "rows_out"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _ptr(num_unique, torch.int64, "num_unique"),
        _ptr(status, torch.int32, "status"), C.addressof(after.c) if after is not None else None, _stream()))


def emb_bag_backward_sort_prepared(tables: TableSet, B: int, nnz: int, workspace: torch.Tensor,
                                   unique_keys: Optional[torch.Tensor] = None,
                                   unique_counts: Optional[torch.Tensor] = None,
                                   num_unique: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None,
                                   stage_events: Optional[Sequence[torch.cuda.Event]] = None) -> None:
    """The sort of a backward whose records ``emb_bag_forward_train`` has already written."""
    for t, name in ((unique_keys, "unique_keys"), (unique_counts, "unique_counts")):
        if t is not None and t.numel() < nnz:
            raise TypeError(name + " must hold at least nnz elements")
    _check("emb_bag_backward_sort_prepared", lib().emb_bag_backward_sort_prepared(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype], int(B), int(nnz),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _ptr(unique_keys, torch.int64, "unique_keys"), _ptr(unique_counts, torch.int32, "unique_counts"),
        _ptr(num_unique, torch.int64, "num_unique"), _ptr(status, torch.int32, "status"),
        _stage_events(stage_events), _stream()))


def emb_bag_backward_update(tables: TableSet, B: int, nnz: int, dout: torch.Tensor, lr: float, eps: float,
                            workspace: torch.Tensor, num_unique: Optional[torch.Tensor] = None,
                            stage_events: Optional[Sequence[torch.cuda.Event]] = None,
                            side: Optional["SideStream"] = None) -> None:
    """Second half of the backward, from the records emb_bag_backward_sort left in ``workspace``."""
    if dout.numel() != tables.T * B * tables.D:
        raise TypeError("shape mismatch")
    _check("emb_bag_backward_update", lib().emb_bag_backward_update(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype], int(B), int(nnz),
        _ptr(dout, torch.float32, "dout"), C.c_float(lr), C.c_float(eps),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _ptr(num_unique, torch.int64, "num_unique"),
        _stage_events(stage_events), None if side is None else C.addressof(side.c), _stream()))


def emb_bag_backward_rowwise_adagrad(tables: TableSet, rows: torch.Tensor, offsets: torch.Tensor, B: int, mode: str,
                                     dout: torch.Tensor, lr: float, eps: float, workspace: torch.Tensor,
                                     unique_keys: Optional[torch.Tensor] = None,
                                     unique_counts: Optional[torch.Tensor] = None,
                                     num_unique: Optional[torch.Tensor] = None,
                                     status: Optional[torch.Tensor] = None,
                                     stage_events: Optional[Sequence[torch.cuda.Event]] = None,
                                     side: Optional["SideStream"] = None) -> None:
    """``stage_events``: BWD_STAGE_EVENTS entries, each None or a torch event that has been
    recorded at least once (so that its HIP handle exists); the library records the given ones
    between its stages.  ``side``: a SideStream on which the long-run path runs beside the
    short-run update."""
    nnz = rows.numel()
    if offsets.numel() != tables.T * B + 1 or dout.numel() != tables.T * B * tables.D:
        raise TypeError("shape mismatch")
    for t, name in ((unique_keys, "unique_keys"), (unique_counts, "unique_counts")):
        if t is not None and t.numel() < nnz:
            raise TypeError(name + " must hold at least nnz elements")
    _check("emb_bag_backward_rowwise_adagrad", lib().emb_bag_backward_rowwise_adagrad(
        tables.host_ptr, tables.dev_ptr, tables.T, tables.D, DTYPE[tables.dtype],
        _ptr(rows, torch.int64, "rows"), _ptr(offsets, torch.int64, "offsets"), int(B), nnz, POOL[mode],
        _ptr(dout, torch.float32, "dout"), C.c_float(lr), C.c_float(eps),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _ptr(unique_keys, torch.int64, "unique_keys"), _ptr(unique_counts, torch.int32, "unique_counts"),
        _ptr(num_unique, torch.int64, "num_unique"), _ptr(status, torch.int32, "status"),
        _stage_events(stage_events), None if side is None else C.addressof(side.c), _stream()))


def emb_cache_index_bytes(num_rows: int) -> int:
    out = C.c_size_t(0)
    _check("emb_cache_index_bytes", lib().emb_cache_index_bytes(int(num_rows), C.byref(out)))
    return int(out.value)


def emb_cache_build(table_ptr: int, num_rows: int, D: int, dtype: str, hot_rows: torch.Tensor,
                    cache_rows: torch.Tensor, cache_index: torch.Tensor,
                    status: Optional[torch.Tensor] = None) -> None:
    _check("emb_cache_build", lib().emb_cache_build(
        int(table_ptr), int(num_rows), int(D), DTYPE[dtype], _ptr(hot_rows, torch.int64, "hot_rows"),
        hot_rows.numel(), _ptr(cache_rows, _TABLE_TORCH[dtype], "cache_rows"),
        _ptr(cache_index, torch.uint8, "cache_index"), _ptr(status, torch.int32, "status"), _stream()))


def emb_bag_forward_cached(table_ptr: int, num_rows: int, D: int, dtype: str, cache_rows: torch.Tensor,
                           cache_index: torch.Tensor, num_hot: int, rows: torch.Tensor, offsets: torch.Tensor,
                           B: int, mode: str, out: torch.Tensor, hit_miss: Optional[torch.Tensor] = None,
                           status: Optional[torch.Tensor] = None) -> None:
    if offsets.numel() != B + 1 or out.numel() != B * D:
        raise TypeError("shape mismatch")
    _check("emb_bag_forward_cached", lib().emb_bag_forward_cached(
        int(table_ptr), int(num_rows), int(D), DTYPE[dtype], _ptr(cache_rows, _TABLE_TORCH[dtype], "cache_rows"),
        _ptr(cache_index, torch.uint8, "cache_index"), int(num_hot), _ptr(rows, torch.int64, "rows"),
        _ptr(offsets, torch.int64, "offsets"), int(B), rows.numel(), POOL[mode], _ptr(out, torch.float32, "out"),
        _ptr(hit_miss, _U64, "hit_miss"), _ptr(status, torch.int32, "status"), _stream()))


def emb_bag_forward_cached_hashed(table_ptr: int, num_rows: int, D: int, dtype: str, cache_rows: torch.Tensor,
                                  cache_index: torch.Tensor, num_hot: int, salt: int, raw: torch.Tensor,
                                  offsets: torch.Tensor, B: int, mode: str, out: torch.Tensor,
                                  hit_miss: Optional[torch.Tensor] = None,
                                  status: Optional[torch.Tensor] = None) -> None:
    if offsets.numel() != B + 1 or out.numel() != B * D:
        raise TypeError("shape mismatch")
    _check("emb_bag_forward_cached_hashed", lib().emb_bag_forward_cached_hashed(
        int(table_ptr), int(num_rows), int(D), DTYPE[dtype], _ptr(cache_rows, _TABLE_TORCH[dtype], "cache_rows"),
        _ptr(cache_index, torch.uint8, "cache_index"), int(num_hot), C.c_uint64(int(salt) % (1 << 64)),
        _ptr(raw, _U64, "raw"), _ptr(offsets, torch.int64, "offsets"), int(B), raw.numel(), POOL[mode],
        _ptr(out, torch.float32, "out"), _ptr(hit_miss, _U64, "hit_miss"), _ptr(status, torch.int32, "status"),
        _stream()))


def emb_bag_forward_cached_hashed_lengths(table_ptr: int, num_rows: int, D: int, dtype: str, cache_rows: torch.Tensor,
                                          cache_index: torch.Tensor, num_hot: int, salt: int, raw: torch.Tensor,
                                          lengths: torch.Tensor, B: int, mode: str, out: torch.Tensor,
                                          offsets_out: torch.Tensor, scratch: torch.Tensor,
                                          hit_miss: Optional[torch.Tensor] = None,
                                          status: Optional[torch.Tensor] = None, lookup_events=None) -> None:
    """``emb_bag_forward_cached_hashed`` from the ``B`` bag lengths; writes the offsets to ``offsets_out``;
    ``scratch`` holds ``emb_offsets_scratch_bytes(B)`` bytes."""
    if lengths.numel() != B or offsets_out.numel() != B + 1 or out.numel() != B * D:
        raise TypeError("shape mismatch")
    _check("emb_bag_forward_cached_hashed_lengths", lib().emb_bag_forward_cached_hashed_lengths(
        int(table_ptr), int(num_rows), int(D), DTYPE[dtype], _ptr(cache_rows, _TABLE_TORCH[dtype], "cache_rows"),
        _ptr(cache_index, torch.uint8, "cache_index"), int(num_hot), C.c_uint64(int(salt) % (1 << 64)),
        _ptr(raw, _U64, "raw"), _ptr(lengths, torch.int32, "lengths") if B else None, int(B), raw.numel(), POOL[mode],
        _ptr(out, torch.float32, "out"), _ptr(offsets_out, torch.int64, "offsets_out"),
        _ptr(scratch, torch.uint8, "scratch"), scratch.numel(), _ptr(hit_miss, _U64, "hit_miss"),
        _ptr(status, torch.int32, "status"), _lookup_events(lookup_events), _stream()))


def emb_cache_stage_misses(table_ptr: int, num_rows: int, D: int, dtype: str, cache_index: torch.Tensor, num_hot: int,
                           ids: torch.Tensor, stage_rows: Optional[torch.Tensor], stage_capacity: int, loc: torch.Tensor,
                           stage_count: torch.Tensor, status: Optional[torch.Tensor] = None,
                           salt: Optional[int] = None) -> None:
    """Resolve the lookups ``ids`` (row numbers, or raw IDs when ``salt`` is given) of one or several batches and
    copy the rows they miss in the cache into ``stage_rows``; ``loc`` receives one location per lookup."""
    if loc.numel() < ids.numel() or stage_count.numel() < 1:
        raise TypeError("shape mismatch")
    if stage_rows is not None and stage_rows.numel() * stage_rows.element_size() < stage_capacity * emb_row_bytes(D, dtype):
        raise TypeError("stage_rows smaller than stage_capacity rows")
    common = (int(table_ptr), int(num_rows), int(D), DTYPE[dtype], _ptr(cache_index, torch.uint8, "cache_index"), int(num_hot))
    tail = (ids.numel(), _ptr(stage_rows, _TABLE_TORCH[dtype], "stage_rows"), int(stage_capacity),
            _ptr(loc, torch.int64, "loc"), _ptr(stage_count, _U64, "stage_count"), _ptr(status, torch.int32, "status"),
            _stream())
    if salt is None:
        _check("emb_cache_stage_misses", lib().emb_cache_stage_misses(*common, _ptr(ids, torch.int64, "rows"), *tail))
    else:
        _check("emb_cache_stage_misses_hashed", lib().emb_cache_stage_misses_hashed(
            *common, C.c_uint64(int(salt) % (1 << 64)), _ptr(ids, _U64, "raw"), *tail))


def emb_bag_forward_staged(table_ptr: int, num_rows: int, D: int, dtype: str, cache_rows: Optional[torch.Tensor],
                           num_hot: int, stage_rows: Optional[torch.Tensor], stage_capacity: int, loc: torch.Tensor,
                           offsets: torch.Tensor, B: int, mode: str, out: torch.Tensor,
                           hit_miss: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None) -> None:
    """The pooled lookup of one batch over the locations ``loc`` that ``emb_cache_stage_misses`` left."""
    if offsets.numel() != B + 1 or out.numel() != B * D:
        raise TypeError("shape mismatch")
    _check("emb_bag_forward_staged", lib().emb_bag_forward_staged(
        int(table_ptr), int(num_rows), int(D), DTYPE[dtype], _ptr(cache_rows, _TABLE_TORCH[dtype], "cache_rows"),
        int(num_hot), _ptr(stage_rows, _TABLE_TORCH[dtype], "stage_rows"), int(stage_capacity),
        _ptr(loc, torch.int64, "loc"), _ptr(offsets, torch.int64, "offsets"), int(B), loc.numel(), POOL[mode],
        _ptr(out, torch.float32, "out"), _ptr(hit_miss, _U64, "hit_miss"), _ptr(status, torch.int32, "status"),
        _stream()))


_U32 = (torch.int32, torch.uint32)


def emb_cache_observe(num_rows: int, rows: torch.Tensor, freq: torch.Tensor,
                      status: Optional[torch.Tensor] = None) -> None:
    if freq.numel() != num_rows:
        raise TypeError("freq must hold one counter per table row")
    _check("emb_cache_observe", lib().emb_cache_observe(
        int(num_rows), _ptr(rows, torch.int64, "rows"), rows.numel(), _ptr(freq, _U32, "freq"),
        _ptr(status, torch.int32, "status"), _stream()))


def emb_cache_observe_hashed(num_rows: int, salt: int, raw: torch.Tensor, freq: torch.Tensor,
                             status: Optional[torch.Tensor] = None) -> None:
    if freq.numel() != num_rows:
        raise TypeError("freq must hold one counter per table row")
    _check("emb_cache_observe_hashed", lib().emb_cache_observe_hashed(
        int(num_rows), C.c_uint64(int(salt) % (1 << 64)), _ptr(raw, _U64, "raw"), raw.numel(),
        _ptr(freq, _U32, "freq"), _ptr(status, torch.int32, "status"), _stream()))


def emb_cache_select_workspace_bytes(num_rows: int) -> int:
    out = C.c_size_t(0)
    _check("emb_cache_select_workspace_bytes", lib().emb_cache_select_workspace_bytes(int(num_rows), C.byref(out)))
    return int(out.value)


def emb_cache_select(freq: torch.Tensor, num_hot: int, decay_shift: int, workspace: torch.Tensor,
                     hot_rows_out: torch.Tensor, info_out: Optional[torch.Tensor] = None) -> None:
    if hot_rows_out.numel() < num_hot:
        raise TypeError("hot_rows_out too small")
    _check("emb_cache_select", lib().emb_cache_select(
        _ptr(freq, _U32, "freq"), freq.numel(), int(num_hot), int(decay_shift), _ptr(workspace, torch.uint8, "workspace"),
        workspace.numel(), _ptr(hot_rows_out, torch.int64, "hot_rows_out"), _ptr(info_out, _U64, "info_out"), _stream()))


CACHE_SELECT_STATIC_MAX_ROWS = 700_000_000   # EMB_CACHE_SELECT_STATIC_MAX_ROWS


def emb_cache_select_static(freq: torch.Tensor, num_hot: int, decay_shift: int, hot_rows_out: torch.Tensor,
                            info_out: Optional[torch.Tensor] = None) -> None:
    """``emb_cache_select`` with the library's own static scratch array instead of a workspace."""
    if hot_rows_out.numel() < num_hot:
        raise TypeError("hot_rows_out too small")
    _check("emb_cache_select_static", lib().emb_cache_select_static(
        _ptr(freq, _U32, "freq"), freq.numel(), int(num_hot), int(decay_shift),
        _ptr(hot_rows_out, torch.int64, "hot_rows_out"), _ptr(info_out, _U64, "info_out"), _stream()))


def emb_cache_rebuild(table_ptr: int, num_rows: int, D: int, dtype: str, old_cache_rows: Optional[torch.Tensor],
                      old_cache_index: torch.Tensor, old_num_hot: int, hot_rows: torch.Tensor,
                      cache_rows: torch.Tensor, cache_index: torch.Tensor, moved: Optional[torch.Tensor] = None,
                      status: Optional[torch.Tensor] = None) -> None:
    _check("emb_cache_rebuild", lib().emb_cache_rebuild(
        int(table_ptr), int(num_rows), int(D), DTYPE[dtype], _ptr(old_cache_rows, _TABLE_TORCH[dtype], "old_cache_rows"),
        _ptr(old_cache_index, torch.uint8, "old_cache_index"), int(old_num_hot),
        _ptr(hot_rows, torch.int64, "hot_rows"), hot_rows.numel(), _ptr(cache_rows, _TABLE_TORCH[dtype], "cache_rows"),
        _ptr(cache_index, torch.uint8, "cache_index"), _ptr(moved, _U64, "moved"), _ptr(status, torch.int32, "status"),
        _stream()))


def emb_version_record_bytes(T: int) -> int:
    out = C.c_size_t(0)
    _check("emb_version_record_bytes", lib().emb_version_record_bytes(int(T), C.byref(out)))
    return int(out.value)


def emb_version_latch_bytes(T: int) -> int:
    out = C.c_size_t(0)
    _check("emb_version_latch_bytes", lib().emb_version_latch_bytes(int(T), C.byref(out)))
    return int(out.value)


def emb_version_record_write(record: torch.Tensor, tables: "TableSet", version: int) -> None:
    if record.numel() < emb_version_record_bytes(tables.T):
        raise TypeError("record too small")
    _check("emb_version_record_write", lib().emb_version_record_write(
        _ptr(record, torch.uint8, "record"), tables.host_ptr, tables.dev_ptr, tables.T,
        C.c_uint64(int(version)), _stream()))


def emb_version_publish(handle: torch.Tensor, record: torch.Tensor) -> None:
    _check("emb_version_publish", lib().emb_version_publish(
        _ptr(handle, _U64, "handle"), _ptr(record, torch.uint8, "record"), _stream()))


def emb_version_latch(handle: torch.Tensor, T: int, latch: torch.Tensor,
                      status: Optional[torch.Tensor] = None) -> None:
    if latch.numel() < emb_version_latch_bytes(T):
        raise TypeError("latch too small")
    _check("emb_version_latch", lib().emb_version_latch(
        _ptr(handle, _U64, "handle"), int(T), _ptr(latch, torch.uint8, "latch"), _ptr(status, torch.int32, "status"),
        _stream()))


def latched_version(latch: torch.Tensor) -> torch.Tensor:
    """The u64 version number at the start of a latch, as a one-element int64 view (device tensor)."""
    return latch[:8].view(torch.int64)


def _forward_latched(fn: str, latch, T, D, dtype, ids, id_dtype, offsets, B, mode, out, status, streaming):
    if latch.numel() < emb_version_latch_bytes(T):
        raise TypeError("latch too small")
    if offsets.numel() != T * B + 1 or out.numel() != T * B * D:
        raise TypeError("shape mismatch")
    _check(fn, getattr(lib(), fn)(
        _ptr(latch, torch.uint8, "latch"), int(T), int(D), DTYPE[dtype], _ptr(ids, id_dtype, "ids"),
        _ptr(offsets, torch.int64, "offsets"), int(B), ids.numel(), POOL[mode] | (ROWS_STREAMING if streaming else 0),
        _ptr(out, torch.float32, "out"), _ptr(status, torch.int32, "status"), _stream()))


def emb_bag_forward_latched(latch: torch.Tensor, T: int, D: int, dtype: str, rows: torch.Tensor, offsets: torch.Tensor,
                            B: int, mode: str, out: torch.Tensor, status: Optional[torch.Tensor] = None,
                            streaming: bool = False) -> None:
    _forward_latched("emb_bag_forward_latched", latch, T, D, dtype, rows, torch.int64, offsets, B, mode, out, status,
                     streaming)


def emb_bag_forward_latched_hashed(latch: torch.Tensor, T: int, D: int, dtype: str, raw: torch.Tensor,
                                   offsets: torch.Tensor, B: int, mode: str, out: torch.Tensor,
                                   status: Optional[torch.Tensor] = None, streaming: bool = False) -> None:
    _forward_latched("emb_bag_forward_latched_hashed", latch, T, D, dtype, raw, _U64, offsets, B, mode, out, status,
                     streaming)


class CachedTables:
    """The ``emb_cached_table`` descriptor array of T hosted tables with their caches, on the host and on the
    device.  ``entries[t]`` = (table_ptr, num_rows, cache_rows tensor, cache_index tensor, num_hot, salt)."""

    def __init__(self, entries: Sequence, D: int, dtype: str, device: Optional[torch.device] = None):
        self.T, self.D, self.dtype = len(entries), int(D), dtype
        self.keep = list(entries)                       # the cache tensors stay referenced
        self.host = np.zeros(self.T, dtype=CACHED_DESC)
        for t, (ptr, rows, cache_rows, cache_index, num_hot, salt) in enumerate(entries):
            self.host["table"][t] = int(ptr)
            self.host["num_rows"][t] = int(rows)
            self.host["cache_rows"][t] = _ptr(cache_rows, _TABLE_TORCH[dtype], "cache_rows[%d]" % t) or 0
            self.host["cache_index"][t] = _ptr(cache_index, torch.uint8, "cache_index[%d]" % t)
            self.host["num_hot"][t] = int(num_hot)
            self.host["salt"][t] = int(salt) % (1 << 64)
        _check("emb_cached_tables_init", lib().emb_cached_tables_init(self.host.ctypes.data, self.T))
        if device is None:
            device = torch.device("cuda", torch.cuda.current_device())
        self.dev = torch.from_numpy(self.host.view(np.uint8).reshape(-1).copy()).to(device)


def _forward_cached_tables(fn: str, ct: CachedTables, ids, id_dtype, offsets, B, mode, out, hit_miss, status):
    if offsets.numel() != ct.T * B + 1 or out.numel() != ct.T * B * ct.D:
        raise TypeError("shape mismatch")
    _check(fn, getattr(lib(), fn)(
        int(ct.host.ctypes.data), int(ct.dev.data_ptr()), ct.T, ct.D, DTYPE[ct.dtype], _ptr(ids, id_dtype, "ids"),
        _ptr(offsets, torch.int64, "offsets"), int(B), ids.numel(), POOL[mode], _ptr(out, torch.float32, "out"),
        _ptr(hit_miss, _U64, "hit_miss"), _ptr(status, torch.int32, "status"), _stream()))


def emb_bag_forward_cached_tables(ct: CachedTables, rows: torch.Tensor, offsets: torch.Tensor, B: int, mode: str,
                                  out: torch.Tensor, hit_miss: Optional[torch.Tensor] = None,
                                  status: Optional[torch.Tensor] = None) -> None:
    _forward_cached_tables("emb_bag_forward_cached_tables", ct, rows, torch.int64, offsets, B, mode, out, hit_miss,
                           status)


def emb_bag_forward_cached_tables_hashed(ct: CachedTables, raw: torch.Tensor, offsets: torch.Tensor, B: int, mode: str,
                                         out: torch.Tensor, hit_miss: Optional[torch.Tensor] = None,
                                         status: Optional[torch.Tensor] = None) -> None:
    _forward_cached_tables("emb_bag_forward_cached_tables_hashed", ct, raw, _U64, offsets, B, mode, out, hit_miss,
                           status)


def emb_bag_forward_cached_tables_hashed_lengths(ct: CachedTables, raw: torch.Tensor, lengths: torch.Tensor, B: int,
                                                 mode: str, out: torch.Tensor, offsets_out: torch.Tensor,
                                                 scratch: torch.Tensor, hit_miss: Optional[torch.Tensor] = None,
                                                 status: Optional[torch.Tensor] = None, lookup_events=None) -> None:
    """``emb_bag_forward_cached_tables_hashed`` from the ``T * B`` bag lengths; writes the offsets to
    ``offsets_out``; ``scratch`` holds ``emb_offsets_scratch_bytes(T * B)`` bytes."""
    n = ct.T * B
    if lengths.numel() != n or offsets_out.numel() != n + 1 or out.numel() != n * ct.D:
        raise TypeError("shape mismatch")
    _check("emb_bag_forward_cached_tables_hashed_lengths", lib().emb_bag_forward_cached_tables_hashed_lengths(
        int(ct.host.ctypes.data), int(ct.dev.data_ptr()), ct.T, ct.D, DTYPE[ct.dtype], _ptr(raw, _U64, "raw"),
        _ptr(lengths, torch.int32, "lengths") if n else None, int(B), raw.numel(), POOL[mode],
        _ptr(out, torch.float32, "out"), _ptr(offsets_out, torch.int64, "offsets_out"),
        _ptr(scratch, torch.uint8, "scratch"), scratch.numel(), _ptr(hit_miss, _U64, "hit_miss"),
        _ptr(status, torch.int32, "status"), _lookup_events(lookup_events), _stream()))


def emb_checksum(data, sum_out: torch.Tensor, nbytes: Optional[int] = None) -> None:
    """``data``: a contiguous device tensor, or a raw device-visible pointer (int) with ``nbytes``."""
    if isinstance(data, int):
        ptr, n = data, int(nbytes)
    else:
        ptr, n = _ptr(data, None, "data"), data.numel() * data.element_size()
    _check("emb_checksum", lib().emb_checksum(ptr, C.c_uint64(n), _ptr(sum_out, _U64, "sum_out"), _stream()))


def emb_host_device_pointer(host_ptr: int) -> int:
    out = C.c_void_p(0)
    _check("emb_host_device_pointer", lib().emb_host_device_pointer(int(host_ptr), C.byref(out)))
    return int(out.value)


def emb_table_fill(weights, num_rows: int, D: int, dtype: str, seed: int) -> None:
    """``weights``: a device tensor, or a raw device-visible pointer (int)."""
    ptr = weights if isinstance(weights, int) else _ptr(weights, _TABLE_TORCH[dtype], "weights")
    _check("emb_table_fill", lib().emb_table_fill(ptr, int(num_rows), int(D), DTYPE[dtype],
                                                  C.c_uint64(int(seed) % (1 << 64)), _stream()))


# ---- version records of hosted tables ----------------------------------------------------------------
def emb_version_hosted_record_bytes(T: int) -> int:
    out = C.c_size_t(0)
    _check("emb_version_hosted_record_bytes", lib().emb_version_hosted_record_bytes(int(T), C.byref(out)))
    return int(out.value)


def emb_version_hosted_latch_bytes(T: int) -> int:
    out = C.c_size_t(0)
    _check("emb_version_hosted_latch_bytes", lib().emb_version_hosted_latch_bytes(int(T), C.byref(out)))
    return int(out.value)


def emb_version_hosted_record_write(record: torch.Tensor, ct: CachedTables, version: int) -> None:
    if record.numel() < emb_version_hosted_record_bytes(ct.T):
        raise TypeError("record too small")
    _check("emb_version_hosted_record_write", lib().emb_version_hosted_record_write(
        _ptr(record, torch.uint8, "record"), int(ct.host.ctypes.data), int(ct.dev.data_ptr()), ct.T,
        C.c_uint64(int(version)), _stream()))


def emb_version_hosted_latch(handle: torch.Tensor, T: int, latch: torch.Tensor,
                             status: Optional[torch.Tensor] = None) -> None:
    if latch.numel() < emb_version_hosted_latch_bytes(T):
        raise TypeError("latch too small")
    _check("emb_version_hosted_latch", lib().emb_version_hosted_latch(
        _ptr(handle, _U64, "handle"), int(T), _ptr(latch, torch.uint8, "latch"), _ptr(status, torch.int32, "status"),
        _stream()))


def _forward_cached_latched(fn: str, latch, T, D, dtype, ids, id_dtype, offsets, B, mode, out, hit_miss, status):
    if latch.numel() < emb_version_hosted_latch_bytes(T):
        raise TypeError("latch too small")
    if offsets.numel() != T * B + 1 or out.numel() != T * B * D:
        raise TypeError("shape mismatch")
    _check(fn, getattr(lib(), fn)(
        _ptr(latch, torch.uint8, "latch"), int(T), int(D), DTYPE[dtype], _ptr(ids, id_dtype, "ids"),
        _ptr(offsets, torch.int64, "offsets"), int(B), ids.numel(), POOL[mode], _ptr(out, torch.float32, "out"),
        _ptr(hit_miss, _U64, "hit_miss"), _ptr(status, torch.int32, "status"), _stream()))


def emb_bag_forward_cached_latched(latch: torch.Tensor, T: int, D: int, dtype: str, rows: torch.Tensor,
                                   offsets: torch.Tensor, B: int, mode: str, out: torch.Tensor,
                                   hit_miss: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None) -> None:
    _forward_cached_latched("emb_bag_forward_cached_latched", latch, T, D, dtype, rows, torch.int64, offsets, B, mode, out,
                            hit_miss, status)


def emb_bag_forward_cached_latched_hashed(latch: torch.Tensor, T: int, D: int, dtype: str, raw: torch.Tensor,
                                          offsets: torch.Tensor, B: int, mode: str, out: torch.Tensor,
                                          hit_miss: Optional[torch.Tensor] = None,
                                          status: Optional[torch.Tensor] = None) -> None:
    _forward_cached_latched("emb_bag_forward_cached_latched_hashed", latch, T, D, dtype, raw, _U64, offsets, B, mode, out,
                            hit_miss, status)

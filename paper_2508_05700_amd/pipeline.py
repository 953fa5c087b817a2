"""Device-side plumbing for running a workload through the library: allocates
the tables and per-batch buffers with torch, fills the tables procedurally and
enqueues the entry points in path order (offsets -> hash -> forward ->
backward).  It only sequences calls of ``binding``; nothing is computed here.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as emb
from .workloads import DEFAULT_SEED, Workload

_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


class DeviceTables:
    """The T tables of a workload in HBM, filled by ``emb_table_fill``; for a workload with
    ``quant`` set, each filled fp32 table is quantised by ``emb_quantize_rows`` and dropped."""

    def __init__(self, w: Workload, seed: int = DEFAULT_SEED, device: str = "cuda:0"):
        self.w = w
        self.device = torch.device(device)
        self.weights: List[torch.Tensor] = []
        self.accum: Optional[List[torch.Tensor]] = [] if w.backward else None
        for t in range(w.T):
            wt = torch.empty((w.R, w.D), dtype=_TORCH_DT[w.dtype], device=self.device)
            emb.emb_table_fill(wt, w.R, w.D, w.dtype, w.table_seed(t, seed))
            if w.quant:
                self.weights.append(quantize_table(wt, w.quant))
                del wt
            else:
                self.weights.append(wt)
            if w.backward:
                self.accum.append(torch.zeros(w.R, dtype=torch.float32, device=self.device))
        self.set = emb.TableSet(self.weights, w.D, w.storage, accum=self.accum,
                                salts=[w.salt(t) for t in range(w.T)], device=self.device)


def quantize_table(table: torch.Tensor, quant: str) -> torch.Tensor:
    """fp32 device table -> its row-quantised storage (a new uint8 tensor)."""
    R, D = table.shape
    q = torch.empty((R, emb.emb_row_bytes(D, quant)), dtype=torch.uint8, device=table.device)
    emb.emb_quantize_rows(table, quant, q)
    return q


def quantized_tableset(tabs: DeviceTables, quant: str):
    """Row-quantised copies of fp32 DeviceTables: (list of uint8 tensors, TableSet)."""
    w = tabs.w
    qs = [quantize_table(t, quant) for t in tabs.weights]
    return qs, emb.TableSet(qs, w.D, quant, salts=[w.salt(t) for t in range(w.T)], device=tabs.device)


class DeviceBatch:
    """One batch's inputs, resident on the device."""

    def __init__(self, w: Workload, batch: Dict[str, object], device: torch.device):
        self.nnz = int(batch["nnz"])
        self.lengths = torch.from_numpy(batch["lengths"]).to(device)
        raw = batch["raw"]
        self.raw = None if raw is None else torch.from_numpy(raw.view(np.int64)).to(device)
        rows = batch["rows"]
        self.rows_given = None if rows is None else torch.from_numpy(rows).to(device)
        dout = batch.get("dout")
        self.dout = None if dout is None else torch.from_numpy(dout).to(device)


class StepBuffers:
    """Outputs and scratch of one step, sized for at most ``max_nnz`` lookups."""

    def __init__(self, w: Workload, max_nnz: int, total_rows: int, device: torch.device, want_unique: bool = False,
                 side_stream: bool = True):
        n = max(int(max_nnz), 1)
        self.offsets = torch.empty(w.T * w.B + 1, dtype=torch.int64, device=device)
        # scratch of the lookups that take bag lengths (sums within tiles)
        self.offsets_scratch = torch.empty(emb.emb_offsets_scratch_bytes(w.T * w.B), dtype=torch.uint8, device=device)
        self.rows = torch.empty(n, dtype=torch.int64, device=device)
        self.out = torch.empty((w.T, w.B, w.D), dtype=torch.float32, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.workspace = None
        self.side = None
        self.unique_keys = self.unique_counts = self.num_unique = None
        if w.backward:
            nbytes = emb.emb_bag_backward_workspace_bytes(w.T, w.B, n, total_rows, w.D, w.dtype)
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
            self.num_unique = torch.zeros(1, dtype=torch.int64, device=device)
            if side_stream:   # the backward's two update paths run side by side
                self.side = emb.SideStream(device)
            # for run_step_overlapped: the backward's sort runs beside the forward
            self.sort_stream = torch.cuda.Stream(device=device)
            self.sort_events = [torch.cuda.Event(), torch.cuda.Event()]
            if want_unique:   # the ordered list of distinct rows is optional output
                self.unique_keys = torch.empty(n, dtype=torch.int64, device=device)
                self.unique_counts = torch.empty(n, dtype=torch.int32, device=device)


def run_index_stage(w: Workload, tables: emb.TableSet, db: DeviceBatch, buf: StepBuffers) -> torch.Tensor:
    """Bag offsets, then hashed row numbers.  Returns the view of the row buffer in use."""
    emb.emb_lengths_to_offsets(db.lengths, buf.offsets, buf.status)
    if db.raw is None:
        return db.rows_given
    rows = buf.rows[:db.nnz]
    emb.emb_hash_ids_tables(tables, db.raw, buf.offsets, w.B, rows, buf.status)
    return rows


LENGTHS_ROUTE_MAX_BAGS = 1 << 20    # what emb_bag_forward_hashed_lengths accepts (256 tiles of 4096 lengths)


def run_index_and_forward_fused(w: Workload, tables: emb.TableSet, db: DeviceBatch, buf: StepBuffers) -> torch.Tensor:
    """Bag offsets, hashing and pooled lookup (one call where the number of bags allows).  Returns the view of the row
    buffer the kernel filled (for the backward).  Workloads whose IDs are row numbers already take the two-kernel route."""
    if db.raw is None:
        rows = run_index_stage(w, tables, db, buf)
        run_forward(w, tables, rows, buf)
        return rows
    rows = buf.rows[:db.nnz]
    if w.T * w.B <= LENGTHS_ROUTE_MAX_BAGS:      # offsets made inside the lookup's call
        emb.emb_bag_forward_hashed_lengths(tables, db.raw, db.lengths, w.B, w.pool, buf.out, buf.offsets,
                                           buf.offsets_scratch, rows if w.backward else None, buf.status,
                                           streaming=w.streaming)
        return rows
    emb.emb_lengths_to_offsets(db.lengths, buf.offsets, buf.status)
    emb.emb_bag_forward_hashed(tables, db.raw, buf.offsets, w.B, w.pool, buf.out, rows if w.backward else None,
                               buf.status, streaming=w.streaming)
    return rows


def run_forward(w: Workload, tables: emb.TableSet, rows: torch.Tensor, buf: StepBuffers) -> None:
    emb.emb_bag_forward(tables, rows, buf.offsets, w.B, w.pool, buf.out, buf.status, streaming=w.streaming)


def run_backward(w: Workload, tables: emb.TableSet, rows: torch.Tensor, db: DeviceBatch, buf: StepBuffers,
                 stage_events=None) -> None:
    emb.emb_bag_backward_rowwise_adagrad(tables, rows, buf.offsets, w.B, w.pool, db.dout, w.lr, w.eps, buf.workspace,
                                         buf.unique_keys, buf.unique_counts, buf.num_unique, buf.status,
                                         stage_events, buf.side)


def run_step_overlapped(w: Workload, tables: emb.TableSet, db: DeviceBatch, buf: StepBuffers,
                        stage_events=None) -> torch.Tensor:
    """One pass of the whole path with the backward's sort enqueued on a second stream as soon as
    the indices exist, beside the forward (it needs neither the tables nor the gradient); the
    update follows on the calling stream once both are done.  ``stage_events`` go to the update only
    (entries 3 to 5)."""
    rows = run_index_stage(w, tables, db, buf)
    if not w.backward:
        run_forward(w, tables, rows, buf)
        return rows
    main = torch.cuda.current_stream()
    buf.sort_events[0].record(main)
    with torch.cuda.stream(buf.sort_stream):
        buf.sort_stream.wait_event(buf.sort_events[0])
        emb.emb_bag_backward_sort(tables, rows, buf.offsets, w.B, w.pool, buf.workspace, buf.unique_keys,
                                  buf.unique_counts, buf.num_unique, buf.status)
        buf.sort_events[1].record(buf.sort_stream)
    run_forward(w, tables, rows, buf)
    main.wait_event(buf.sort_events[1])
    emb.emb_bag_backward_update(tables, w.B, rows.numel(), db.dout, w.lr, w.eps, buf.workspace, buf.num_unique,
                                stage_events, buf.side)
    return rows


def run_train_step(w: Workload, tables: emb.TableSet, db: DeviceBatch, buf: StepBuffers, stage_events=None,
                   after: Optional[emb.SideStream] = None) -> None:
    """One pass of the whole path for a workload with a backward and raw IDs: the training lookup from
    bag lengths and raw IDs (offsets, hashing, pooling and the backward's records), sort, update.
    ``after``: the side stream of the previous step when its join was deferred (``defer_join``); the lookup
    then waits for it, and ``buf`` must not be the previous step's."""
    emb.emb_bag_forward_train_lengths_after(tables, db.raw, db.lengths, w.B, w.pool, buf.out, buf.offsets,
                                            buf.workspace, after, None, buf.num_unique, buf.status)
    emb.emb_bag_backward_sort_prepared(tables, w.B, db.nnz, buf.workspace, buf.unique_keys, buf.unique_counts,
                                       buf.num_unique, buf.status, stage_events)
    emb.emb_bag_backward_update(tables, w.B, db.nnz, db.dout, w.lr, w.eps, buf.workspace, buf.num_unique,
                                stage_events, buf.side)


def run_step(w: Workload, tables: emb.TableSet, db: DeviceBatch, buf: StepBuffers) -> Optional[torch.Tensor]:
    """One pass of the whole path over one batch, by the shortest route the workload allows: the
    training lookup when there is a backward and the IDs are raw, hashing inside the lookup when
    the IDs are raw, separate kernels otherwise.  Returns the row view where one was produced."""
    if w.backward and db.raw is not None and not w.quant:
        run_train_step(w, tables, db, buf)
        return None
    rows = run_index_and_forward_fused(w, tables, db, buf)
    if w.backward:
        run_backward(w, tables, rows, db, buf)
    return rows


class HotRowCache:
    """The HBM hot-row cache of one host-resident table together with the frequency-based policy that
    decides what it holds: two cache buffers (the lookups read one while a refresh fills the other),
    one access counter per table row, and the selection workspace.  Call sequencing only."""

    def __init__(self, table_ptr: int, num_rows: int, D: int, dtype: str, num_hot: int, salt: int,
                 device: torch.device, decay_shift: int = 1):
        self.table_ptr, self.R, self.D, self.dtype, self.salt = int(table_ptr), int(num_rows), int(D), dtype, int(salt)
        self.capacity, self.decay_shift = int(num_hot), int(decay_shift)
        rowb = emb.emb_row_bytes(D, dtype)
        shape = (self.capacity, rowb) if dtype in emb.QUANT_DTYPES else (self.capacity, D)
        tdt = torch.uint8 if dtype in emb.QUANT_DTYPES else (torch.float32 if dtype == "f32" else torch.bfloat16)
        self.rows = [torch.empty(shape, dtype=tdt, device=device) for _ in range(2)]
        self.index = [torch.empty(emb.emb_cache_index_bytes(num_rows), dtype=torch.uint8, device=device)
                      for _ in range(2)]
        self.hot = torch.empty(max(self.capacity, 1), dtype=torch.int64, device=device)
        self.freq = torch.zeros(num_rows, dtype=torch.int32, device=device)
        self.workspace = torch.empty(emb.emb_cache_select_workspace_bytes(num_rows), dtype=torch.uint8, device=device)
        self.info = torch.zeros(2, dtype=torch.int64, device=device)
        self.moved = torch.zeros(2, dtype=torch.int64, device=device)
        self.hit_miss = torch.zeros(2, dtype=torch.int64, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.active = 0
        self.num_hot = 0                                             # starts empty: every lookup is a miss
        emb.emb_cache_build(self.table_ptr, self.R, D, dtype, self.hot[:0], self.rows[0], self.index[0], self.status)

    def set_static(self, hot_rows: torch.Tensor) -> None:
        """Load a given hot set (ascending rows) into the active buffers."""
        self.num_hot = hot_rows.numel()
        emb.emb_cache_build(self.table_ptr, self.R, self.D, self.dtype, hot_rows, self.rows[self.active],
                            self.index[self.active], self.status)

    def observe(self, raw: torch.Tensor) -> None:
        emb.emb_cache_observe_hashed(self.R, self.salt, raw, self.freq, self.status)

    def refresh(self) -> None:
        """Select the most frequently looked-up rows and fill the idle buffers with them, taking the rows the
        active cache already holds from HBM; then swap.  In stream order with the lookups."""
        emb.emb_cache_select(self.freq, self.capacity, self.decay_shift, self.workspace, self.hot, self.info)
        new = 1 - self.active
        emb.emb_cache_rebuild(self.table_ptr, self.R, self.D, self.dtype, self.rows[self.active],
                              self.index[self.active], self.num_hot, self.hot[:self.capacity], self.rows[new],
                              self.index[new], self.moved, self.status)
        self.active, self.num_hot = new, self.capacity

    def forward_hashed(self, raw: torch.Tensor, offsets: torch.Tensor, B: int, mode: str, out: torch.Tensor) -> None:
        emb.emb_bag_forward_cached_hashed(self.table_ptr, self.R, self.D, self.dtype, self.rows[self.active],
                                          self.index[self.active], self.num_hot, self.salt, raw, offsets, B, mode, out,
                                          self.hit_miss, self.status)


class HostedTableSet:
    """Several host-resident tables, each with a ``HotRowCache``, looked up with one launch.  The descriptor
    array names each table's active cache buffers, so it is rebuilt (a copy of T x 64 bytes) after a refresh."""

    def __init__(self, caches: List[HotRowCache], device: torch.device):
        assert len({(c.D, c.dtype) for c in caches}) == 1, "the tables of one launch share D and storage type"
        self.caches, self.device = list(caches), device
        self.D, self.dtype = caches[0].D, caches[0].dtype
        self.hit_miss = torch.zeros(2, dtype=torch.int64, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self._describe()

    def _describe(self) -> None:
        self.tables = emb.CachedTables([(c.table_ptr, c.R, c.rows[c.active], c.index[c.active], c.num_hot, c.salt)
                                        for c in self.caches], self.D, self.dtype, device=self.device)

    def observe(self, raw: torch.Tensor, offsets_host: Sequence[int], B: int) -> None:
        """Count the lookups of a batch: ``offsets_host[t * B]`` bounds table t's slice of ``raw``."""
        for t, c in enumerate(self.caches):
            c.observe(raw[int(offsets_host[t * B]):int(offsets_host[(t + 1) * B])])

    def refresh(self) -> None:
        for c in self.caches:
            c.refresh()
        self._describe()

    def forward_hashed(self, raw: torch.Tensor, offsets: torch.Tensor, B: int, mode: str, out: torch.Tensor) -> None:
        emb.emb_bag_forward_cached_tables_hashed(self.tables, raw, offsets, B, mode, out, self.hit_miss, self.status)

    # ---- the same set behind a version handle: a refresh becomes visible to lookups by one publish ----
    def publish(self, version: int) -> None:
        """Write a record of the descriptors as they are now (the active caches) and make it current.  Records
        alternate between two buffers; the caller retires the older one's caches after the lookups that latched
        it have finished (here: the next refresh but one overwrites them, in stream order)."""
        T = len(self.caches)
        if not hasattr(self, "handle"):
            self.handle = torch.zeros(1, dtype=torch.int64, device=self.device)
            self.records = [torch.empty(emb.emb_version_hosted_record_bytes(T), dtype=torch.uint8, device=self.device)
                            for _ in range(2)]
            self.latch = torch.empty(emb.emb_version_hosted_latch_bytes(T), dtype=torch.uint8, device=self.device)
            self._rec = 0
        self._rec = 1 - self._rec
        emb.emb_version_hosted_record_write(self.records[self._rec], self.tables, version)
        emb.emb_version_publish(self.handle, self.records[self._rec])

    def forward_latched_hashed(self, raw: torch.Tensor, offsets: torch.Tensor, B: int, mode: str,
                               out: torch.Tensor) -> torch.Tensor:
        """Latch the current record, look up over it; returns the one-element view of the latched version."""
        T = len(self.caches)
        emb.emb_version_hosted_latch(self.handle, T, self.latch, self.status)
        emb.emb_bag_forward_cached_latched_hashed(self.latch, T, self.D, self.dtype, raw, offsets, B, mode, out,
                                                  self.hit_miss, self.status)
        return emb.latched_version(self.latch)

"""The C ABI without a GPU: the library loads, exports what the header
declares, and every host-checkable error is reported without a launch."""
import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest

from paper_2508_05700_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, INVALID, UNSUPPORTED, WORKSPACE = 0, -1, -2, -3
FAKE = 0x1000  # a non-null, 256-byte aligned address; every call below that uses it has one invalid
               # argument, so the library returns before any launch and never dereferences it


@pytest.fixture(scope="module")
def L():
    return b.lib()


def _tables(rows=(1000, 7), with_accum=True):
    d = np.zeros(len(rows), dtype=b.TABLE_DESC)
    d["num_rows"] = rows
    d["weights"] = FAKE
    if with_accum:
        d["accum"] = FAKE
    assert b.lib().emb_tables_init(d.ctypes.data, len(rows)) == OK
    return d


def test_library_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "emb.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(emb_[a-z_0-9]+)\s*\(", header))
    assert declared == set(b.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_descriptor_layout_matches_header():
    header = open(os.path.join(ROOT, "include", "emb.h")).read()
    body = re.search(r"typedef struct emb_table \{(.*?)\} emb_table;", header, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(\w+);", body)
    assert fields == list(b.TABLE_DESC.names)
    assert b.TABLE_DESC.itemsize == 48


def test_status_strings(L):
    assert L.emb_status_string(0) == b"EMB_OK"
    assert L.emb_status_string(-3) == b"EMB_ERR_WORKSPACE"
    assert L.emb_status_string(-99) == b"EMB_ERR_UNKNOWN"


def test_tables_init(L):
    d = _tables((10_000_000, 7, 1))
    assert d["row_base"].tolist() == [0, 10_000_000, 10_000_007]
    assert d["mod_magic"].tolist() == [((1 << 64) - 1) // r for r in (10_000_000, 7, 1)]
    bad = np.zeros(1, dtype=b.TABLE_DESC)
    assert L.emb_tables_init(bad.ctypes.data, 1) == INVALID         # num_rows == 0
    assert L.emb_tables_init(None, 1) == INVALID
    assert L.emb_tables_init(None, 0) == OK


def test_hash_ids_argument_errors(L):
    assert L.emb_hash_ids(None, 5, 0, 10, None, None) == INVALID
    assert L.emb_hash_ids(FAKE, -1, 0, 10, FAKE, None) == INVALID
    assert L.emb_hash_ids(FAKE, 5, 0, 0, FAKE, None) == INVALID
    assert L.emb_hash_ids(None, 0, 0, 10, None, None) == OK            # empty input: nothing to do


def test_offsets_argument_errors(L):
    assert L.emb_lengths_to_offsets(None, 4, FAKE, None, None) == INVALID
    assert L.emb_lengths_to_offsets(FAKE, -1, FAKE, None, None) == INVALID
    assert L.emb_lengths_to_offsets(FAKE, 4, None, None, None) == INVALID


def test_forward_argument_errors(L):
    d = _tables()
    f = L.emb_bag_forward
    args = lambda **k: [k.get("th", d.ctypes.data), k.get("td", FAKE), k.get("T", 2), k.get("D", 64),
                        k.get("dt", 0), k.get("rows", FAKE), k.get("off", FAKE), k.get("B", 4), k.get("nnz", 8),
                        k.get("mode", 0), k.get("out", FAKE), None, None]
    assert f(*args(D=0)) == INVALID
    assert f(*args(D=3)) == UNSUPPORTED            # 12-byte rows cannot be read with 128-bit loads
    assert f(*args(D=4, dt=1)) == UNSUPPORTED      # 8-byte bf16 rows
    assert f(*args(D=8192)) == UNSUPPORTED         # 32 KB rows
    assert f(*args(dt=5)) == INVALID
    assert f(*args(mode=2)) == INVALID
    assert f(*args(B=-1)) == INVALID
    assert f(*args(nnz=-1)) == INVALID
    assert f(*args(out=None)) == INVALID
    assert f(*args(off=None)) == INVALID
    assert f(*args(rows=None)) == INVALID
    assert f(*args(td=None)) == INVALID
    assert f(*args(out=FAKE + 4)) == INVALID       # misaligned output
    assert f(*args(B=0)) == OK                     # no bags: nothing to do
    d2 = d.copy()
    d2["row_base"][1] += 1
    assert f(*args(th=d2.ctypes.data)) == INVALID  # descriptors not initialised consistently
    d3 = d.copy()
    d3["weights"][0] = 0
    assert f(*args(th=d3.ctypes.data)) == INVALID


def test_backward_argument_errors(L):
    d = _tables()
    need = L.emb_bag_backward_workspace_bytes(2, 4, 8, 1007, 64, 0)
    assert need > 0 and need % 256 == 0
    f = L.emb_bag_backward_rowwise_adagrad

    def args(**k):
        return [k.get("th", d.ctypes.data), FAKE, 2, k.get("D", 64), 0, FAKE, FAKE, 4, k.get("nnz", 8),
                k.get("mode", 1), k.get("dout", FAKE), C.c_float(0.01), C.c_float(1e-8), k.get("ws", FAKE),
                k.get("wsb", need), None, None, None, None, None, k.get("side", None), None]
    assert f(*args(ws=None)) == WORKSPACE
    assert f(*args(wsb=need - 1)) == WORKSPACE
    assert f(*args(ws=FAKE + 16)) == WORKSPACE          # workspace must be 256-byte aligned
    assert f(*args(D=3)) == UNSUPPORTED
    assert f(*args(mode=7)) == INVALID
    assert f(*args(dout=None)) == INVALID
    assert f(*args(nnz=1 << 31)) == UNSUPPORTED
    noacc = _tables(with_accum=False)
    assert f(*args(th=noacc.ctypes.data)) == UNSUPPORTED
    # a side stream needs a stream of its own and both events
    side = (C.c_void_p * 4)(FAKE, FAKE, None, None)
    assert f(*args(side=C.addressof(side))) == INVALID
    side = (C.c_void_p * 4)(None, FAKE, FAKE, None)           # NULL is the call's own (default) stream here
    assert f(*args(side=C.addressof(side))) == INVALID


def fhq(L):
    # padded INT4 rows, like the other quantised types, are not read by the backward; the hashing lookup
    # applies the quantised shape rules to them (D a multiple of 16)
    d0 = _tables()
    assert L.emb_bag_backward_workspace_bytes(2, 4, 8, 1007, 64, 4) == 0
    return L.emb_bag_forward_hashed(d0.ctypes.data, FAKE, 2, 24, 4, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None)


def test_quantized_row_size_and_argument_errors(L):
    L.emb_row_bytes.restype = C.c_int64
    rb = L.emb_row_bytes
    assert rb(64, 0) == 256 and rb(64, 1) == 128 and rb(64, 2) == 80 and rb(64, 3) == 48
    assert rb(32, 3) == 32 and rb(16, 3) == 16 and rb(0, 3) == 0 and rb(63, 3) == 0 and rb(64, 9) == 0
    # INT4 rows padded to whole 64-byte sectors
    assert rb(64, 4) == 64 and rb(16, 4) == 64 and rb(112, 4) == 64 and rb(128, 4) == 128 and rb(63, 4) == 0
    q = L.emb_quantize_rows
    assert q(FAKE, 10, 24, 3, FAKE, None) == UNSUPPORTED        # D must be a multiple of 16
    assert q(FAKE, 10, 2048, 2, FAKE, None) == UNSUPPORTED
    assert q(FAKE, 10, 64, 0, FAKE, None) == INVALID            # not a quantised type
    assert q(None, 10, 64, 3, FAKE, None) == INVALID
    assert q(FAKE, 10, 64, 3, FAKE + 8, None) == INVALID        # 16-byte alignment
    assert q(FAKE, -1, 64, 3, FAKE, None) == INVALID
    assert q(FAKE, 0, 64, 3, FAKE, None) == OK                  # nothing to do
    assert q(FAKE, 0, 64, 4, FAKE, None) == OK and q(FAKE, 10, 24, 4, FAKE, None) == UNSUPPORTED
    assert fhq(L) == UNSUPPORTED
    # the streaming hint is the only extra bit a mode may carry
    dm = _tables()
    assert L.emb_bag_forward(dm.ctypes.data, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0x200, FAKE, None, None) == INVALID
    assert L.emb_bag_forward(dm.ctypes.data, FAKE, 2, 64, 0, FAKE, FAKE, 0, 8, 0x100 | 1, FAKE, None, None) == OK
    # (no bags: the mode with the hint bit passes validation and nothing is launched)
    # hashing fused into the forward (quantised tables included; their shape rules apply)
    d0 = _tables()
    fh = L.emb_bag_forward_hashed
    assert fh(d0.ctypes.data, FAKE, 2, 24, 3, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == UNSUPPORTED
    assert fh(d0.ctypes.data, FAKE, 2, 64, 3, FAKE, FAKE, 4, 8, 0, None, None, None, None) == INVALID
    assert fh(d0.ctypes.data, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0, None, None, None, None) == INVALID
    assert fh(d0.ctypes.data, FAKE, 2, 64, 0, None, FAKE, 4, 8, 0, FAKE, None, None, None) == INVALID
    # quantised tables are read by the forward only
    assert L.emb_bag_backward_workspace_bytes(2, 4, 8, 1007, 64, 3) == 0
    d = _tables()
    f = L.emb_bag_forward
    assert f(d.ctypes.data, FAKE, 2, 24, 3, FAKE, FAKE, 4, 8, 0, FAKE, None, None) == UNSUPPORTED
    assert f(d.ctypes.data, FAKE, 2, 64, 3, FAKE, FAKE, 4, 8, 0, None, None, None) == INVALID


def test_split_backward_and_helper_argument_errors(L):
    d = _tables()
    need = L.emb_bag_backward_workspace_bytes(2, 4, 8, 1007, 64, 0)
    srt, upd = L.emb_bag_backward_sort, L.emb_bag_backward_update

    def sort_args(**k):
        return [k.get("th", d.ctypes.data), FAKE, 2, k.get("D", 64), 0, k.get("rows", FAKE), FAKE, 4, k.get("nnz", 8),
                k.get("mode", 1), k.get("ws", FAKE), k.get("wsb", need), None, None, None, None, None, None]

    def upd_args(**k):
        return [d.ctypes.data, FAKE, 2, k.get("D", 64), 0, 4, k.get("nnz", 8), k.get("dout", FAKE), C.c_float(0.01),
                C.c_float(1e-8), k.get("ws", FAKE), k.get("wsb", need), None, None, k.get("side", None), None]
    assert srt(*sort_args(mode=5)) == INVALID
    assert srt(*sort_args(rows=None)) == INVALID
    assert srt(*sort_args(wsb=need - 1)) == WORKSPACE
    assert srt(*sort_args(D=3)) == UNSUPPORTED
    assert srt(*sort_args(nnz=-1)) == INVALID
    assert upd(*upd_args(dout=None)) == INVALID
    assert upd(*upd_args(dout=FAKE + 4)) == INVALID           # gradient rows are read 16 bytes at a time
    assert upd(*upd_args(ws=None)) == WORKSPACE
    assert upd(*upd_args(nnz=1 << 31)) == UNSUPPORTED
    side = (C.c_void_p * 4)(FAKE, None, FAKE, None)
    assert upd(*upd_args(side=C.addressof(side))) == INVALID
    # the training lookup and the sort that follows it
    tr, sp = L.emb_bag_forward_train, L.emb_bag_backward_sort_prepared

    def tr_args(**k):
        return [k.get("th", d.ctypes.data), FAKE, 2, k.get("D", 64), k.get("dtype", 0), k.get("raw", FAKE), FAKE, 4, 8,
                k.get("mode", 1), k.get("out", FAKE), None, k.get("ws", FAKE), k.get("wsb", need), None, None, None]
    assert tr(*tr_args(mode=9)) == INVALID
    assert tr(*tr_args(out=None)) == INVALID
    assert tr(*tr_args(raw=None)) == INVALID
    assert tr(*tr_args(wsb=need - 256)) == WORKSPACE
    assert tr(*tr_args(dtype=3)) == UNSUPPORTED                       # quantised tables are not trained
    noacc = _tables(with_accum=False)
    assert tr(*tr_args(th=noacc.ctypes.data)) == UNSUPPORTED          # training needs accumulators
    # the same lookup taking bag lengths: an array for the offsets it makes is required
    trl = L.emb_bag_forward_train_lengths

    def trl_args(**k):
        return [d.ctypes.data, FAKE, 2, 64, 0, k.get("raw", FAKE), k.get("lengths", FAKE), 4, 8, k.get("mode", 1),
                k.get("out", FAKE), k.get("offs", FAKE), None, k.get("ws", FAKE), k.get("wsb", need), None, None, None]
    assert trl(*trl_args(offs=None)) == INVALID
    assert trl(*trl_args(lengths=None)) == INVALID
    assert trl(*trl_args(out=None)) == INVALID and trl(*trl_args(raw=None)) == INVALID
    assert trl(*trl_args(mode=2)) == INVALID
    assert trl(*trl_args(wsb=need - 256)) == WORKSPACE and trl(*trl_args(ws=None)) == WORKSPACE
    # ... and the form that waits for an earlier backward's side stream: the same refusals, and the side
    # stream needs its join event and must not be the call's own stream (NULL here)
    tra = L.emb_bag_forward_train_lengths_after
    for kw in (dict(offs=None), dict(lengths=None), dict(out=None), dict(raw=None), dict(mode=2)):
        assert tra(*(trl_args(**kw)[:-1] + [None, None])) == INVALID, kw
    assert tra(*(trl_args(wsb=need - 256)[:-1] + [None, None])) == WORKSPACE
    side = (C.c_void_p * 4)(FAKE, FAKE, None, None)
    assert tra(*(trl_args()[:-1] + [C.addressof(side), None])) == INVALID
    side = (C.c_void_p * 4)(None, FAKE, FAKE, None)
    assert tra(*(trl_args()[:-1] + [C.addressof(side), None])) == INVALID
    # the forward-only lookup taking bag lengths
    L.emb_offsets_scratch_bytes.restype = C.c_size_t
    assert L.emb_offsets_scratch_bytes(C.c_int64(8)) == 72 and L.emb_offsets_scratch_bytes(C.c_int64(-1)) == 0
    fhl = L.emb_bag_forward_hashed_lengths

    def fhl_args(**k):
        return [d.ctypes.data, FAKE, 2, 64, k.get("dtype", 0), k.get("raw", FAKE), k.get("lengths", FAKE), k.get("B", 4), 8,
                k.get("mode", 1), k.get("out", FAKE), k.get("offs", FAKE), None, k.get("scratch", FAKE), k.get("sb", 72),
                None, None]
    assert fhl(*fhl_args(offs=None)) == INVALID and fhl(*fhl_args(lengths=None)) == INVALID
    assert fhl(*fhl_args(scratch=None)) == INVALID and fhl(*fhl_args(sb=64)) == INVALID
    assert fhl(*fhl_args(out=None)) == INVALID and fhl(*fhl_args(raw=None)) == INVALID
    assert fhl(*fhl_args(mode=7)) == INVALID and fhl(*fhl_args(dtype=9)) == INVALID
    assert fhl(*fhl_args(B=600_000, sb=1 << 30)) == UNSUPPORTED       # 1.2 M bags: more than 256 tiles
    assert sp(d.ctypes.data, FAKE, 2, 64, 0, 4, 8, None, need, None, None, None, None, None, None) == WORKSPACE
    assert sp(d.ctypes.data, FAKE, 2, 3, 0, 4, 8, FAKE, need, None, None, None, None, None, None) == UNSUPPORTED
    # helpers: null arguments are refused before the runtime is touched
    assert L.emb_event_create(None, 1) == INVALID
    assert L.emb_event_record(None, None) == INVALID
    assert L.emb_event_elapsed_ms(None, None, None) == INVALID
    assert L.emb_event_destroy(None) == OK
    assert L.emb_side_stream_create(None) == INVALID and L.emb_side_stream_destroy(None) == INVALID
    # the struct as the header declares it and as the binding mirrors it
    header = open(os.path.join(ROOT, "include", "emb.h")).read()
    body = re.search(r"typedef struct emb_side_stream \{(.*?)\} emb_side_stream;", header, flags=re.S).group(1)
    fields = re.findall(r"\b(\w+);", re.sub(r"/\*.*?\*/", "", body, flags=re.S))
    assert fields == [f[0] for f in b._SideStreamC._fields_] and C.sizeof(b._SideStreamC) == 32
    # joining: a side stream with its event, and not the stream that is to wait
    assert L.emb_side_stream_join(None, None) == INVALID
    side = (C.c_void_p * 4)(FAKE, FAKE, None, None)
    assert L.emb_side_stream_join(C.addressof(side), None) == INVALID           # no join event
    side = (C.c_void_p * 4)(None, FAKE, FAKE, None)
    assert L.emb_side_stream_join(C.addressof(side), None) == INVALID           # its stream is the waiting one


def test_mixed_forward_shapes_and_argument_errors(L):
    import numpy as np
    SH = np.dtype([("D", "<i4"), ("dtype", "<i4"), ("out_offset", "<i8"), ("out_stride", "<i8"),
                   ("first_block", "<u4"), ("lanes", "<i4")])
    sh = np.zeros(2, dtype=SH)
    sh["D"], sh["dtype"] = [64, 8], [0, 1]
    sh["out_offset"], sh["out_stride"] = [0, 64], [72, 72]
    init = L.emb_table_shapes_init
    assert init(sh.ctypes.data, 2, 100) == OK
    assert list(sh["lanes"]) == [16, 1] and list(sh["first_block"]) == [0, 7]     # 100 bags / 16 groups = 7 blocks
    bad = sh.copy(); bad["D"][1] = 6
    assert init(bad.ctypes.data, 2, 100) == UNSUPPORTED                              # 12-byte rows
    bad = sh.copy(); bad["dtype"][0] = 3
    assert init(bad.ctypes.data, 2, 100) == INVALID                                  # quantised tables: not here
    bad = sh.copy(); bad["out_stride"][0] = 60
    assert init(bad.ctypes.data, 2, 100) == INVALID
    bad = sh.copy(); bad["out_offset"][1] = 66
    assert init(bad.ctypes.data, 2, 100) == INVALID
    d = _tables()
    f = L.emb_bag_forward_mixed

    def args(**k):
        return [d.ctypes.data, FAKE, k.get("sh", sh.ctypes.data), FAKE, 2, FAKE, FAKE, k.get("B", 100), 8,
                k.get("mode", 0), k.get("out", FAKE), k.get("floats", 7200), None, None]
    assert f(*args(floats=7199)) == INVALID                # the last output row would not fit
    assert f(*args(B=101)) == INVALID                      # shapes were derived for another B
    assert f(*args(mode=2)) == INVALID
    assert f(*args(out=None)) == INVALID
    assert f(*args(B=0)) == OK


def test_workspace_bytes(L):
    w = L.emb_bag_backward_workspace_bytes
    assert w(-1, 1, 1, 1, 64, 0) == 0 and w(1, -1, 1, 1, 64, 0) == 0 and w(1, 1, -1, 1, 64, 0) == 0
    assert w(1, 1, 1, 1, 0, 0) == 0 and w(1, 1, 1, 1, 3, 0) == 0 and w(1, 1, 1, 1, 64, 9) == 0
    a, c = w(16, 8192, 1_000_000, 160_000_000, 64, 0), w(16, 8192, 2_000_000, 160_000_000, 64, 0)
    assert 0 < a < c
    # keys widen to 64 bits once the key range passes 2^32
    assert w(1, 8, 1_000_000, 1 << 33, 64, 0) > w(1, 8, 1_000_000, 1 << 30, 64, 0) + 7_000_000


def test_cache_argument_errors(L):
    n = C.c_size_t(0)
    assert L.emb_cache_index_bytes(250_000_000, C.byref(n)) == OK
    assert n.value == ((250_000_000 + 63) // 64) * 16
    assert L.emb_cache_index_bytes(0, C.byref(n)) == INVALID
    assert L.emb_cache_build(FAKE, 100, 64, 0, FAKE, 101, FAKE, FAKE, None, None) == INVALID   # more hot rows than rows
    assert L.emb_cache_build(FAKE, 100, 3, 0, FAKE, 10, FAKE, FAKE, None, None) == UNSUPPORTED
    assert L.emb_cache_build(None, 100, 64, 0, FAKE, 10, FAKE, FAKE, None, None) == INVALID
    assert L.emb_bag_forward_cached(FAKE, 100, 64, 0, FAKE, None, 10, FAKE, FAKE, 4, 8, 0, FAKE, None, None,
                                    None) == INVALID
    assert L.emb_bag_forward_cached(FAKE, 100, 64, 0, FAKE, FAKE, 10, FAKE, FAKE, 4, 8, 3, FAKE, None, None,
                                    None) == INVALID
    assert L.emb_table_fill(None, 10, 64, 0, 1, None) == INVALID
    assert L.emb_table_fill(FAKE, 10, 6, 0, 1, None) == UNSUPPORTED


def test_staging_argument_errors(L):
    # emb_cache_stage_misses(table, R, D, dtype, index, num_hot, ids, nnz, stage_rows, capacity, loc, count, status, stream)
    assert L.emb_cache_stage_misses(FAKE, 100, 64, 0, FAKE, 10, None, 0, None, 0, None, None, None, None) == OK   # no lookups
    assert L.emb_cache_stage_misses(FAKE, 0, 64, 0, FAKE, 0, FAKE, 5, FAKE, 8, FAKE, FAKE, None, None) == INVALID
    assert L.emb_cache_stage_misses(FAKE, 100, 64, 0, FAKE, 101, FAKE, 5, FAKE, 8, FAKE, FAKE, None, None) == INVALID
    assert L.emb_cache_stage_misses(FAKE, 100, 6, 0, FAKE, 10, FAKE, 5, FAKE, 8, FAKE, FAKE, None, None) == UNSUPPORTED
    assert L.emb_cache_stage_misses(FAKE, 100, 64, 0, FAKE, 10, FAKE, 5, None, 8, FAKE, FAKE, None, None) == INVALID
    assert L.emb_cache_stage_misses(FAKE, 100, 64, 0, FAKE, 10, FAKE, 5, FAKE, 8, None, FAKE, None, None) == INVALID
    assert L.emb_cache_stage_misses(FAKE, 100, 64, 0, FAKE, 10, FAKE, 5, FAKE, 8, FAKE, None, None, None) == INVALID
    assert L.emb_cache_stage_misses(FAKE, 100, 64, 0, FAKE, 10, FAKE, 5, FAKE, -1, FAKE, FAKE, None, None) == INVALID
    assert L.emb_cache_stage_misses(FAKE, 1 << 61, 64, 0, FAKE, 10, FAKE, 5, FAKE, 8, FAKE, FAKE, None, None) == UNSUPPORTED
    assert L.emb_cache_stage_misses_hashed(FAKE, 100, 64, 0, None, 10, 7, FAKE, 5, FAKE, 8, FAKE, FAKE, None, None) == INVALID
    # emb_bag_forward_staged(table, R, D, dtype, cache_rows, num_hot, stage_rows, capacity, loc, offsets, B, nnz, mode, out, ...)
    assert L.emb_bag_forward_staged(FAKE, 100, 64, 0, FAKE, 10, FAKE, 8, FAKE, FAKE, 0, 0, 0, FAKE, None, None, None) == OK
    assert L.emb_bag_forward_staged(FAKE, 100, 64, 0, FAKE, 10, FAKE, 8, FAKE, FAKE, 4, 8, 2, FAKE, None, None, None) == INVALID
    assert L.emb_bag_forward_staged(FAKE, 100, 64, 0, None, 10, FAKE, 8, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == INVALID
    assert L.emb_bag_forward_staged(FAKE, 100, 64, 0, FAKE, 10, None, 8, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == INVALID
    assert L.emb_bag_forward_staged(FAKE, 100, 64, 0, FAKE, 10, FAKE, 8, None, FAKE, 4, 8, 0, FAKE, None, None, None) == INVALID
    assert L.emb_bag_forward_staged(FAKE, 100, 64, 0, FAKE, 10, FAKE, 8, FAKE, FAKE, 4, 8, 0, FAKE + 4, None, None, None) == INVALID
    assert L.emb_bag_forward_staged(FAKE, 100, 24, 2, FAKE, 10, FAKE, 8, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == UNSUPPORTED


def test_hosted_version_argument_errors(L):
    n = C.c_size_t(0)
    assert L.emb_version_hosted_record_bytes(4, C.byref(n)) == OK and n.value == 16 + 4 * 64
    m = C.c_size_t(0)
    assert L.emb_version_hosted_latch_bytes(4, C.byref(m)) == OK and m.value == n.value + 16384
    assert L.emb_version_hosted_record_bytes(0, C.byref(n)) == INVALID
    assert L.emb_version_hosted_latch_bytes(3, None) == INVALID
    d = np.zeros(2, dtype=b.CACHED_DESC)
    d["table"] = FAKE; d["cache_rows"] = FAKE; d["cache_index"] = FAKE
    d["num_rows"] = [100, 7]; d["num_hot"] = [10, 7]
    assert L.emb_cached_tables_init(d.ctypes.data, 2) == OK
    assert L.emb_version_hosted_record_write(FAKE, d.ctypes.data, FAKE, 2, 0, None) == INVALID      # version 0 means none
    assert L.emb_version_hosted_record_write(None, d.ctypes.data, FAKE, 2, 5, None) == INVALID
    assert L.emb_version_hosted_record_write(FAKE, d.ctypes.data, None, 2, 5, None) == INVALID
    bad = d.copy(); bad["num_hot"][1] = 8                                                            # more hot rows than rows
    assert L.emb_version_hosted_record_write(FAKE, bad.ctypes.data, FAKE, 2, 5, None) == INVALID
    bad = d.copy(); bad["mod_magic"][0] += 1                                                         # not initialised
    assert L.emb_version_hosted_record_write(FAKE, bad.ctypes.data, FAKE, 2, 5, None) == INVALID
    assert L.emb_version_hosted_latch(None, 2, FAKE, None, None) == INVALID
    assert L.emb_version_hosted_latch(FAKE, 2, FAKE + 8, None, None) == INVALID
    assert L.emb_bag_forward_cached_latched(None, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == INVALID
    assert L.emb_bag_forward_cached_latched(FAKE, 2, 6, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == UNSUPPORTED
    assert L.emb_bag_forward_cached_latched_hashed(FAKE, 2, 64, 0, FAKE, None, 4, 8, 0, FAKE, None, None, None) == INVALID
    assert L.emb_bag_forward_cached_latched(FAKE, 2, 64, 0, FAKE, FAKE, 0, 0, 0, FAKE, None, None, None) == OK   # no bags


def test_cache_policy_argument_errors(L):
    n = C.c_size_t(0)
    assert L.emb_cache_select_workspace_bytes(250_000_000, C.byref(n)) == OK
    assert 1 << 20 < n.value < 2 << 20 and n.value % 256 == 0       # a few bytes per thousand rows
    small = C.c_size_t(0)
    assert L.emb_cache_select_workspace_bytes(1, C.byref(small)) == OK and 0 < small.value < n.value
    assert L.emb_cache_select_workspace_bytes(0, C.byref(n)) == INVALID
    assert L.emb_cache_select_workspace_bytes(10, None) == INVALID
    # nothing to count is not an error and launches nothing; bad sizes and null pointers are
    assert L.emb_cache_observe(100, None, 0, None, None, None) == OK
    assert L.emb_cache_observe(0, FAKE, 5, FAKE, None, None) == INVALID
    assert L.emb_cache_observe(100, FAKE, -1, FAKE, None, None) == INVALID
    assert L.emb_cache_observe(100, None, 5, FAKE, None, None) == INVALID
    assert L.emb_cache_observe_hashed(100, 7, FAKE, 5, None, None, None) == INVALID
    ws = small.value
    assert L.emb_cache_select(FAKE, 100, 101, 0, FAKE, ws, FAKE, None, None) == INVALID     # more hot rows than rows
    assert L.emb_cache_select(FAKE, 100, 10, 32, FAKE, ws, FAKE, None, None) == INVALID     # shift out of range
    assert L.emb_cache_select(FAKE + 4, 100, 10, 0, FAKE, ws, FAKE, None, None) == INVALID  # counters misaligned
    assert L.emb_cache_select(FAKE, 100, 10, 0, FAKE, ws, None, None, None) == INVALID
    assert L.emb_cache_select(FAKE, 100, 10, 0, None, ws, FAKE, None, None) == WORKSPACE
    assert L.emb_cache_select(FAKE, 100, 10, 0, FAKE, ws - 1, FAKE, None, None) == WORKSPACE
    assert L.emb_cache_select(FAKE, 100, 10, 0, FAKE + 16, ws, FAKE, None, None) == WORKSPACE
    # the variant with the library's own scratch array: same checks, and a stated maximum size, all before
    # anything is launched or the array is looked up
    assert L.emb_cache_select_static(FAKE, 100, 101, 0, FAKE, None, None) == INVALID
    assert L.emb_cache_select_static(FAKE, 100, 10, 32, FAKE, None, None) == INVALID
    assert L.emb_cache_select_static(FAKE + 4, 100, 10, 0, FAKE, None, None) == INVALID
    assert L.emb_cache_select_static(FAKE, 100, 10, 0, None, None, None) == INVALID
    assert L.emb_cache_select_static(None, 100, 10, 0, FAKE, None, None) == INVALID
    assert L.emb_cache_select_static(FAKE, b.CACHE_SELECT_STATIC_MAX_ROWS + 1, 10, 0, FAKE, None, None) == UNSUPPORTED
    header = open(os.path.join(ROOT, "include", "emb.h")).read()
    assert int(re.search(r"#define EMB_CACHE_SELECT_STATIC_MAX_ROWS (\d+)", header).group(1)) == b.CACHE_SELECT_STATIC_MAX_ROWS
    assert L.emb_cache_select_workspace_bytes(b.CACHE_SELECT_STATIC_MAX_ROWS, C.byref(n)) == OK and n.value <= 4 << 20
    # a refresh needs an older cache, in buffers other than the new ones
    OLD = FAKE + 4096
    assert L.emb_cache_rebuild(FAKE, 100, 64, 0, OLD, None, 5, FAKE, 10, FAKE, FAKE, None, None, None) == INVALID
    assert L.emb_cache_rebuild(FAKE, 100, 64, 0, OLD, FAKE, 5, FAKE, 10, FAKE, FAKE, None, None, None) == INVALID
    assert L.emb_cache_rebuild(FAKE, 100, 64, 0, FAKE, OLD, 5, FAKE, 10, FAKE, FAKE, None, None, None) == INVALID
    assert L.emb_cache_rebuild(FAKE, 100, 64, 0, None, OLD, 5, FAKE, 10, FAKE, FAKE, None, None, None) == INVALID
    assert L.emb_cache_rebuild(FAKE, 100, 64, 0, OLD, OLD, 101, FAKE, 10, FAKE, FAKE, None, None, None) == INVALID
    assert L.emb_cache_rebuild(FAKE, 100, 6, 0, OLD, OLD, 5, FAKE, 10, FAKE, FAKE, None, None, None) == UNSUPPORTED


def test_versioned_tables_argument_errors(L):
    n, m = C.c_size_t(0), C.c_size_t(0)
    assert L.emb_version_record_bytes(16, C.byref(n)) == OK and n.value == 16 + 16 * b.TABLE_DESC.itemsize
    assert L.emb_version_latch_bytes(16, C.byref(m)) == OK and m.value == n.value + 16384
    assert L.emb_version_record_bytes(0, C.byref(n)) == INVALID and L.emb_version_latch_bytes(3, None) == INVALID
    tabs = _tables()
    th = tabs.ctypes.data
    assert L.emb_version_record_write(None, th, FAKE, 2, 7, None) == INVALID
    assert L.emb_version_record_write(FAKE, th, FAKE, 2, 0, None) == INVALID          # version 0 means "none"
    assert L.emb_version_record_write(FAKE + 8, th, FAKE, 2, 7, None) == INVALID      # misaligned record
    assert L.emb_version_record_write(FAKE, None, FAKE, 2, 7, None) == INVALID        # descriptors are validated here
    bad = tabs.copy()
    bad["mod_magic"][1] += 1
    assert L.emb_version_record_write(FAKE, bad.ctypes.data, FAKE, 2, 7, None) == INVALID
    assert L.emb_version_publish(None, FAKE, None) == INVALID and L.emb_version_publish(FAKE, None, None) == INVALID
    assert L.emb_version_publish(FAKE + 4, FAKE, None) == INVALID
    assert L.emb_version_latch(None, 2, FAKE, None, None) == INVALID
    assert L.emb_version_latch(FAKE, 0, FAKE, None, None) == INVALID
    assert L.emb_version_latch(FAKE, 2, None, None, None) == INVALID
    for fn in (L.emb_bag_forward_latched, L.emb_bag_forward_latched_hashed):
        assert fn(None, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, None) == INVALID
        assert fn(FAKE, 0, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, None) == INVALID
        assert fn(FAKE, 2, 6, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, None) == UNSUPPORTED
        assert fn(FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 7, FAKE, None, None) == INVALID   # pooling mode
        assert fn(FAKE, 2, 64, 0, FAKE, None, 4, 8, 0, FAKE, None, None) == INVALID
        assert fn(FAKE, 2, 64, 0, FAKE, FAKE, 0, 0, 0, FAKE, None, None) == OK        # no bags: nothing launched
    assert L.emb_bag_forward_latched_hashed(FAKE, 2, 24, 3, FAKE, FAKE, 4, 8, 0, FAKE, None, None) == UNSUPPORTED


def test_cached_tables_descriptor_and_argument_errors(L):
    header = open(os.path.join(ROOT, "include", "emb.h")).read()
    body = re.search(r"typedef struct emb_cached_table \{(.*?)\} emb_cached_table;", header, flags=re.S).group(1)
    fields = re.findall(r"\b(\w+);", re.sub(r"/\*.*?\*/", "", body, flags=re.S))
    assert fields == list(b.CACHED_DESC.names)
    d = np.zeros(2, dtype=b.CACHED_DESC)
    d["table"], d["cache_rows"], d["cache_index"] = FAKE, FAKE, FAKE
    d["num_rows"], d["num_hot"] = [1000, 7], [10, 7]
    assert L.emb_cached_tables_init(d.ctypes.data, 2) == OK
    assert d["mod_magic"].tolist() == [(2 ** 64 - 1) // 1000, (2 ** 64 - 1) // 7]
    assert L.emb_cached_tables_init(None, 2) == INVALID
    bad = d.copy()
    bad["num_rows"][1] = 0
    assert L.emb_cached_tables_init(bad.ctypes.data, 2) == INVALID
    for fn in (L.emb_bag_forward_cached_tables, L.emb_bag_forward_cached_tables_hashed):
        th = d.ctypes.data
        assert fn(th, FAKE, 2, 64, 0, FAKE, FAKE, 0, 0, 0, FAKE, None, None, None) == OK          # no bags
        assert fn(None, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == INVALID
        assert fn(th, None, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == INVALID
        assert fn(th, FAKE, 2, 6, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == UNSUPPORTED
        assert fn(th, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 5, FAKE, None, None, None) == INVALID     # pooling mode
        assert fn(th, FAKE, 2, 64, 0, FAKE, None, 4, 8, 0, FAKE, None, None, None) == INVALID
        for field, value in (("num_hot", 8), ("cache_index", 0), ("mod_magic", 1), ("table", FAKE + 8)):
            bad = d.copy()
            bad[field][1] = value
            assert fn(bad.ctypes.data, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, None, None) == INVALID, field


def test_cached_lookups_from_lengths_argument_errors(L):
    # every refusal comes before the first launch
    d = np.zeros(2, dtype=b.CACHED_DESC)
    d["table"], d["cache_rows"], d["cache_index"] = FAKE, FAKE, FAKE
    d["num_rows"], d["num_hot"] = [1000, 7], [10, 7]
    assert L.emb_cached_tables_init(d.ctypes.data, 2) == OK
    th = d.ctypes.data
    fn = L.emb_bag_forward_cached_tables_hashed_lengths
    #  th, td, T, D, dtype, raw, lengths, B, nnz, mode, out, offsets_out, scratch, scratch_bytes, hit_miss, status,
    #  lookup_events, stream
    assert fn(th, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, None, FAKE, 72, None, None, None, None) == INVALID   # no offsets_out
    assert fn(th, FAKE, 2, 64, 0, FAKE, None, 4, 8, 0, FAKE, FAKE, FAKE, 72, None, None, None, None) == INVALID   # no lengths
    assert fn(th, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, None, 72, None, None, None, None) == INVALID   # no scratch
    assert fn(th, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, FAKE, 64, None, None, None, None) == INVALID   # 9 sums need 72 bytes
    assert fn(th, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, FAKE + 8, 72, None, None, None, None) == INVALID
    assert fn(None, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, FAKE, 72, None, None, None, None) == INVALID
    assert fn(th, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 7, FAKE, FAKE, FAKE, 72, None, None, None, None) == INVALID   # pooling mode
    assert fn(th, FAKE, 2, 6, 0, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, FAKE, 72, None, None, None, None) == UNSUPPORTED
    assert fn(th, FAKE, 2, 64, 0, FAKE, FAKE, (1 << 19) + 1, 8, 0, FAKE, FAKE, FAKE, 1 << 24, None, None, None, None) == UNSUPPORTED
    bad = d.copy()
    bad["mod_magic"][1] = 1
    assert fn(bad.ctypes.data, FAKE, 2, 64, 0, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, FAKE, 72, None, None, None, None) == INVALID
    one = L.emb_bag_forward_cached_hashed_lengths
    #  table, num_rows, D, dtype, cache_rows, cache_index, num_hot, salt, raw, lengths, B, nnz, mode, out, offsets_out,
    #  scratch, scratch_bytes, hit_miss, status, lookup_events, stream
    assert one(FAKE, 100, 64, 0, FAKE, FAKE, 10, 1, FAKE, FAKE, 4, 8, 0, FAKE, None, FAKE, 40, None, None, None, None) == INVALID
    assert one(FAKE, 100, 64, 0, FAKE, FAKE, 10, 1, FAKE, None, 4, 8, 0, FAKE, FAKE, FAKE, 40, None, None, None, None) == INVALID
    assert one(FAKE, 100, 64, 0, FAKE, FAKE, 10, 1, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, FAKE, 32, None, None, None, None) == INVALID
    assert one(None, 100, 64, 0, FAKE, FAKE, 10, 1, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, FAKE, 40, None, None, None, None) == INVALID
    assert one(FAKE, 0, 64, 0, FAKE, FAKE, 10, 1, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, FAKE, 40, None, None, None, None) == INVALID
    assert one(FAKE, 100, 64, 0, FAKE, FAKE, 10, 1, None, FAKE, 4, 8, 0, FAKE, FAKE, FAKE, 40, None, None, None, None) == INVALID
    assert one(FAKE, 100, 6, 0, FAKE, FAKE, 10, 1, FAKE, FAKE, 4, 8, 0, FAKE, FAKE, FAKE, 40, None, None, None, None) == UNSUPPORTED
    assert one(FAKE, 100, 64, 0, FAKE, FAKE, 10, 1, FAKE, FAKE, (1 << 20) + 1, 8, 0, FAKE, FAKE, FAKE, 1 << 24, None, None,
               None, None) == UNSUPPORTED


def test_checksum_argument_errors(L):
    assert L.emb_checksum(FAKE, 64, None, None) == INVALID
    assert L.emb_checksum(None, 64, FAKE, None) == INVALID
    assert L.emb_checksum(FAKE, 60, FAKE, None) == INVALID            # not whole 16-byte chunks
    assert L.emb_checksum(FAKE + 8, 64, FAKE, None) == INVALID        # misaligned data
    assert L.emb_checksum(FAKE, 64, FAKE + 4, None) == INVALID        # misaligned result


def test_header_is_plain_c_and_links_against_the_library(L, tmp_path):
    # The boundary is a C ABI: the header must compile as C11 (and as C++) on its own, and a C program that
    # takes the address of every declared entry point must link against the built library.
    header = open(os.path.join(ROOT, "include", "emb.h")).read()
    names = sorted(set(re.findall(r"\b(emb_[a-z_0-9]+)\s*\(", re.sub(r"/\*.*?\*/", "", header, flags=re.S))))
    src = tmp_path / "use.c"
    src.write_text('#include "emb.h"\n#include <stdio.h>\ntypedef void (*fn)(void);\nint main(void) {\n    fn f[] = {%s};\n'
                   '    printf("%%d %%s\\n", (int)(sizeof f / sizeof f[0]), emb_status_string(EMB_ERR_WORKSPACE));\n'
                   '    return f[0] == 0;\n}\n' % ", ".join("(fn)%s" % n for n in names))
    inc = os.path.join(ROOT, "include")
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)])
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)])
    exe = tmp_path / "use"
    libdir = os.path.dirname(b.lib_path())
    subprocess.check_call(["gcc", "-std=c11", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-lemb_hip",
                           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"])
    out = subprocess.check_output([str(exe)], env=dict(os.environ, LD_LIBRARY_PATH="/opt/rocm/lib")).decode().split(None, 1)
    assert int(out[0]) == len(names) == len(b.EXPORTS) and "workspace" in out[1].lower()


def test_exact_remainder_on_the_host(tmp_path):
    exe = str(tmp_path / "u64mod_check")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "paper_2508_05700_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host", "u64mod_check.cpp"), "-o", exe])
    out = subprocess.run([exe], stdout=subprocess.PIPE, text=True)
    assert out.returncode == 0 and out.stdout.startswith("OK"), out.stdout

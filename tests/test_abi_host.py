"""Host side of the C ABI, no GPU needed: the library loads, exports what include/turborag.h declares, computes
the gather plan bit-exactly, and turns every invalid call into an error code before anything is enqueued.

Device pointers handed to the library here are made-up non-null addresses: every call below either fails
validation or is a documented no-op, so none of them is ever dereferenced or passed to a kernel.
"""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2410_07590_amd import binding as B
from paper_2410_07590_amd import build as trbuild
from paper_2410_07590_amd import synth

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "turborag.h")
FAKE = C.c_void_p(0x7000_0000_1000)   # 256-byte aligned, never touched
FAKE2 = C.c_void_p(0x7000_0100_0000)


@pytest.fixture(scope="module")
def L():
    if trbuild.needs_build():
        trbuild.build()
    return B.lib()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tr_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_and_library_exports_the_same_symbols(L):
    declared = _declared_functions()
    assert len(declared) >= 14
    for name in declared:
        assert hasattr(L, name), "library does not export %s" % name
    assert sorted(B.EXPORTS) == declared


def test_status_codes_match_header():
    text = open(HEADER).read()
    for name in ["TR_OK", "TR_ERR_INVALID_ARG", "TR_ERR_BAD_CHUNK_ID", "TR_ERR_BAD_PLAN", "TR_ERR_SHAPE",
                 "TR_ERR_UNSUPPORTED", "TR_ERR_HIP", "TR_ERR_WORKSPACE", "TR_ERR_NO_MEMORY", "TR_POS_COMPOSITE", "TR_POS_REORDERED",
                 "TR_F32", "TR_BF16", "TR_ROPE_INTERLEAVED", "TR_ROPE_HALF"]:
        m = re.search(r"\b%s\s*=\s*(-?\d+)" % name, text)
        assert m, name
        assert getattr(B, name) == int(m.group(1)), name


def _shape(hq=28, hkv=4, d=128, dtype=B.TR_BF16, base=1e6, layout=B.TR_ROPE_INTERLEAVED):
    return B.tr_shape(hq, hkv, d, dtype, float(base), layout, 0)


def _store(L, shape, row_start):
    rs = np.ascontiguousarray(row_start, dtype=np.int64)
    h = C.c_void_p(0)
    rc = L.tr_store_create(C.byref(shape), FAKE, FAKE2, rs.ctypes.data_as(C.c_void_p), C.c_int32(rs.size - 1), C.byref(h))
    return rc, h


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.c_void_p)


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(C.c_void_p)


def test_shape_validation(L):
    bad = [(_shape(hq=28, hkv=5), B.TR_ERR_SHAPE), (_shape(d=96), B.TR_ERR_SHAPE), (_shape(hq=0), B.TR_ERR_SHAPE),
           (_shape(dtype=7), B.TR_ERR_SHAPE), (_shape(layout=7), B.TR_ERR_INVALID_ARG),
           (_shape(base=0.0), B.TR_ERR_SHAPE)]
    for sh, want in bad:
        rc, h = _store(L, sh, [0, 4])
        assert rc == want, (rc, want, L.tr_last_error())
        assert L.tr_last_error() != b""
    rc, h = _store(L, _shape(), [0, 4])
    assert rc == B.TR_OK
    assert L.tr_store_destroy(h) == B.TR_OK


def test_store_create_validation(L):
    sh = _shape()
    assert _store(L, sh, [0, 8, 4])[0] == B.TR_ERR_INVALID_ARG          # row starts must not decrease
    assert _store(L, sh, [1, 8])[0] in (B.TR_OK, B.TR_ERR_INVALID_ARG)    # a base offset is the caller's business
    h = C.c_void_p(0)
    rs, rs_p = _i64([0, 4])
    assert L.tr_store_create(C.byref(sh), None, FAKE2, rs_p, C.c_int32(1), C.byref(h)) == B.TR_ERR_INVALID_ARG
    assert L.tr_store_create(C.byref(sh), FAKE, FAKE2, None, C.c_int32(1), C.byref(h)) == B.TR_ERR_INVALID_ARG
    assert L.tr_store_create(C.byref(sh), FAKE, FAKE2, rs_p, C.c_int32(-1), C.byref(h)) == B.TR_ERR_INVALID_ARG
    assert L.tr_store_create(C.byref(sh), FAKE, FAKE2, rs_p, C.c_int32(1), None) == B.TR_ERR_INVALID_ARG


@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4])
@pytest.mark.parametrize("pos_mode", [B.TR_POS_COMPOSITE, B.TR_POS_REORDERED])
def test_plan_is_bit_exact_against_the_oracle(L, cfg_id, pos_mode):
    """Sec. 3.2: offsets, and position ids under both schemes, for the chunk-length mix of each configuration."""
    cfg = synth.CONFIGS[cfg_id]
    lens = synth.chunk_lengths(cfg)
    row_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rc, h = _store(L, _shape(cfg.shape.n_q_heads, cfg.shape.n_kv_heads, cfg.shape.head_dim), row_start)
    assert rc == B.TR_OK
    rng = np.random.default_rng(cfg_id)
    ids = rng.integers(0, lens.size, size=min(10, lens.size) + 3).astype(np.int32)   # duplicates allowed
    ids_a, ids_p = _i32(ids)
    off = np.full(ids.size + 1, -1, np.int64)
    assert L.tr_plan(h, ids_p, C.c_int32(ids.size), C.c_int32(pos_mode), off.ctypes.data_as(C.c_void_p), None, C.c_int64(0)) == B.TR_OK
    pos = np.full(int(off[-1]), -1, np.int32)
    assert L.tr_plan(h, ids_p, C.c_int32(ids.size), C.c_int32(pos_mode), off.ctypes.data_as(C.c_void_p),
                     pos.ctypes.data_as(C.c_void_p), C.c_int64(pos.size)) == B.TR_OK
    want_off, want_delta, want_pos = oracle.plan(row_start, ids, pos_mode)
    assert off.dtype == want_off.dtype and np.array_equal(off, want_off)
    assert np.array_equal(pos, want_pos)
    # capacity one short: error, not a partial write
    if pos.size:
        assert L.tr_plan(h, ids_p, C.c_int32(ids.size), C.c_int32(pos_mode), off.ctypes.data_as(C.c_void_p),
                         pos.ctypes.data_as(C.c_void_p), C.c_int64(pos.size - 1)) == B.TR_ERR_BAD_PLAN
    L.tr_store_destroy(h)


def test_plan_errors(L):
    rc, h = _store(L, _shape(), [0, 4, 9, 9, 20])
    assert rc == B.TR_OK
    off = np.zeros(8, np.int64)
    off_p = off.ctypes.data_as(C.c_void_p)
    for bad in ([0, 4], [-1, 0], [1, 2, 3, 99]):
        a, p = _i32(bad)
        assert L.tr_plan(h, p, C.c_int32(a.size), C.c_int32(B.TR_POS_REORDERED), off_p, None, C.c_int64(0)) == B.TR_ERR_BAD_CHUNK_ID
        assert b"chunk" in L.tr_last_error()
    a, p = _i32([0, 1])
    assert L.tr_plan(None, p, C.c_int32(2), C.c_int32(0), off_p, None, C.c_int64(0)) == B.TR_ERR_INVALID_ARG
    assert L.tr_plan(h, None, C.c_int32(2), C.c_int32(0), off_p, None, C.c_int64(0)) == B.TR_ERR_INVALID_ARG
    assert L.tr_plan(h, p, C.c_int32(2), C.c_int32(0), None, None, C.c_int64(0)) == B.TR_ERR_INVALID_ARG
    assert L.tr_plan(h, p, C.c_int32(-2), C.c_int32(0), off_p, None, C.c_int64(0)) == B.TR_ERR_INVALID_ARG
    assert L.tr_plan(h, p, C.c_int32(2), C.c_int32(5), off_p, None, C.c_int64(0)) == B.TR_ERR_INVALID_ARG
    # empty request and empty chunk are legal
    assert L.tr_plan(h, p, C.c_int32(0), C.c_int32(0), off_p, None, C.c_int64(0)) == B.TR_OK and off[0] == 0
    a, p = _i32([2, 2])
    assert L.tr_plan(h, p, C.c_int32(2), C.c_int32(1), off_p, None, C.c_int64(0)) == B.TR_OK
    assert list(off[:3]) == [0, 0, 0]
    L.tr_store_destroy(h)


@pytest.mark.parametrize("entry", ["tr_kv_assemble", "tr_kv_assemble_raw"])
def test_assemble_validation_happens_before_any_enqueue(L, entry):
    rc, h = _store(L, _shape(), [0, 4, 9, 9, 20])
    assert rc == B.TR_OK
    ids, ids_p = _i32([1, 3, 0])
    good, good_p = _i64([0, 5, 16, 20])

    def call(ids_p=ids_p, off_p=good_p, n=3, mode=B.TR_POS_REORDERED, k=FAKE, v=FAKE2, cap=64, store=h):
        return getattr(L, entry)(store, ids_p, off_p, C.c_int32(n), C.c_int32(mode), k, v, C.c_int64(cap), None)

    assert call(cap=19) == B.TR_ERR_BAD_PLAN                       # does not fit
    bad, bad_p = _i64([0, 5, 15, 20])
    assert call(off_p=bad_p) == B.TR_ERR_BAD_PLAN                  # not the prefix sum of the lengths
    bad2, bad2_p = _i64([1, 6, 17, 21])
    assert call(off_p=bad2_p) == B.TR_ERR_BAD_PLAN                 # must start at 0
    ids_bad, ids_bad_p = _i32([1, 4, 0])
    assert call(ids_p=ids_bad_p) == B.TR_ERR_BAD_CHUNK_ID
    assert call(k=None) == B.TR_ERR_INVALID_ARG
    assert call(v=None) == B.TR_ERR_INVALID_ARG
    assert call(store=None) == B.TR_ERR_INVALID_ARG
    assert call(n=-1) == B.TR_ERR_INVALID_ARG
    assert call(mode=2) == B.TR_ERR_INVALID_ARG
    assert call(n=0) == B.TR_OK                                     # no chunks: nothing to do, nothing enqueued
    e_ids, e_ids_p = _i32([2])
    e_off, e_off_p = _i64([0, 0])
    assert call(ids_p=e_ids_p, off_p=e_off_p, n=1) == B.TR_OK       # one empty chunk: nothing to move
    L.tr_store_destroy(h)


def test_assemble_batched_validation(L):
    rc, h = _store(L, _shape(), [0, 4, 9, 9, 20])
    ids, ids_p = _i32([1, 3, 0, 0])
    cu, cu_p = _i32([0, 3, 4])
    pm, pm_p = _i32([1, 0])
    rows, rows_p = _i64([0, 24, 30])       # request 0: 20 doc rows + 4 query rows; request 1: 4 + 2

    def call(ids_p=ids_p, cu_p=cu_p, pm_p=pm_p, rows_p=rows_p, n=2, cap=30):
        return L.tr_kv_assemble_batched(h, ids_p, cu_p, pm_p, rows_p, C.c_int32(n), FAKE, FAKE2, C.c_int64(cap), None)

    assert call(cap=29) == B.TR_ERR_BAD_PLAN
    small, small_p = _i64([0, 19, 30])
    assert call(rows_p=small_p) == B.TR_ERR_BAD_PLAN               # request 0's documents do not fit its rows
    badcu, badcu_p = _i32([0, 3, 2])
    assert call(cu_p=badcu_p) == B.TR_ERR_INVALID_ARG
    badpm, badpm_p = _i32([1, 3])
    assert call(pm_p=badpm_p) == B.TR_ERR_INVALID_ARG
    badid, badid_p = _i32([1, 3, 0, 7])
    assert call(ids_p=badid_p) == B.TR_ERR_BAD_CHUNK_ID
    assert call(n=0) == B.TR_OK
    L.tr_store_destroy(h)


def test_append_validation(L):
    sh = _shape()

    def call(n_q=4, dst=16, cap=20, k=FAKE, qpos=FAKE, ck=FAKE2, shape=sh):
        return L.tr_kv_append(C.byref(shape), k, FAKE, qpos, C.c_int32(n_q), ck, FAKE2, C.c_int64(dst), C.c_int64(cap), None)

    assert call(cap=19) == B.TR_ERR_BAD_PLAN
    assert call(dst=-1) == B.TR_ERR_INVALID_ARG
    assert call(n_q=-1) == B.TR_ERR_INVALID_ARG
    assert call(k=None) == B.TR_ERR_INVALID_ARG
    assert call(qpos=None) == B.TR_ERR_INVALID_ARG
    assert call(shape=_shape(d=100)) == B.TR_ERR_SHAPE
    assert call(n_q=0) == B.TR_OK


def test_prefill_attn_validation_and_workspace(L):
    sh = _shape()
    size = L.tr_prefill_attn_workspace_size(C.byref(sh), C.c_int32(64), C.c_int64(4160))
    assert size > 0 and size % 256 == 0
    # a long query over few keys fills the chip without splitting: no workspace needed
    assert L.tr_prefill_attn_workspace_size(C.byref(sh), C.c_int32(4096), C.c_int64(4096)) == 0
    # fp32 path never splits
    assert L.tr_prefill_attn_workspace_size(C.byref(_shape(4, 4, 64, B.TR_F32, 1e4)), C.c_int32(16), C.c_int64(144)) == 0

    def call(n_q=64, kv_len=4160, ws=FAKE2, ws_bytes=size, q=FAKE, out=FAKE, shape=sh):
        return L.tr_prefill_attn(C.byref(shape), q, FAKE, FAKE, FAKE, C.c_int32(n_q), C.c_int64(kv_len), out, ws,
                                 C.c_size_t(ws_bytes), None)

    assert call(kv_len=63) == B.TR_ERR_INVALID_ARG                 # fewer cache rows than query tokens
    assert call(q=None) == B.TR_ERR_INVALID_ARG
    assert call(out=None) == B.TR_ERR_INVALID_ARG
    assert call(n_q=-1) == B.TR_ERR_INVALID_ARG
    assert call(ws=None, ws_bytes=0) == B.TR_ERR_WORKSPACE
    assert call(ws_bytes=size - 1) == B.TR_ERR_WORKSPACE
    assert call(ws=C.c_void_p(FAKE2.value + 16)) == B.TR_ERR_WORKSPACE
    assert b"aligned" in L.tr_last_error()
    assert call(shape=_shape(hq=30)) == B.TR_ERR_SHAPE
    assert call(n_q=0, kv_len=100) == B.TR_OK


def test_static_scratch_prefill_validation_and_size_limit(L):
    """tr_prefill_attn_static: the same validation as tr_prefill_attn, and a refusal, before any GPU call, of shapes
    whose split-KV partials exceed the library's static array."""
    sh = _shape(32, 8, 128, base=5e5)
    L.tr_prefill_attn_static_scratch_bytes.restype = C.c_size_t
    cap = L.tr_prefill_attn_static_scratch_bytes()
    assert cap == 32 << 20

    def call(n_q=1024, kv_len=70000, q=FAKE, out=FAKE, shape=sh):
        return L.tr_prefill_attn_static(C.byref(shape), q, FAKE, FAKE, FAKE, C.c_int32(n_q), C.c_int64(kv_len), out, None)

    assert call(kv_len=63) == B.TR_ERR_INVALID_ARG
    assert call(q=None) == B.TR_ERR_INVALID_ARG
    assert call(out=None) == B.TR_ERR_INVALID_ARG
    assert call(n_q=-1) == B.TR_ERR_INVALID_ARG
    assert call(shape=_shape(hq=30)) == B.TR_ERR_SHAPE
    assert call(n_q=0, kv_len=100) == B.TR_OK
    # under the default policy a single request at this shape stays below the array's size; four workgroups per CU as
    # the target cuts it into 8 pieces, 66 MiB of partial results
    assert L.tr_prefill_attn_workspace_size(C.byref(sh), C.c_int32(1024), C.c_int64(70000)) <= cap
    assert L.tr_set_tuning(b"target_items", C.c_int32(1024)) == B.TR_OK
    try:
        assert L.tr_prefill_attn_workspace_size(C.byref(sh), C.c_int32(1024), C.c_int64(70000)) > cap
        assert call() == B.TR_ERR_WORKSPACE
        assert b"static" in L.tr_last_error()
    finally:
        assert L.tr_set_tuning(b"target_items", C.c_int32(0)) == B.TR_OK


def test_set_tuning_validation_and_effect(L):
    sh = _shape()
    assert L.tr_set_tuning(None, C.c_int32(1)) == B.TR_ERR_INVALID_ARG
    assert L.tr_set_tuning(b"no_such_knob", C.c_int32(1)) == B.TR_ERR_INVALID_ARG
    assert b"no_such_knob" in L.tr_last_error()
    assert L.tr_set_tuning(b"wg_rows", C.c_int32(-1)) == B.TR_ERR_INVALID_ARG
    base = L.tr_prefill_attn_workspace_size(C.byref(sh), C.c_int32(64), C.c_int64(4160))
    assert L.tr_set_tuning(b"target_items", C.c_int32(32)) == B.TR_OK
    try:
        assert L.tr_prefill_attn_workspace_size(C.byref(sh), C.c_int32(64), C.c_int64(4160)) < base   # fewer key splits
    finally:
        assert L.tr_set_tuning(b"target_items", C.c_int32(0)) == B.TR_OK
    assert L.tr_prefill_attn_workspace_size(C.byref(sh), C.c_int32(64), C.c_int64(4160)) == base


def test_prefill_attn_batched_validation(L):
    sh = _shape()
    cu, cu_p = _i32([0, 40, 100])
    rows, rows_p = _i64([0, 3000, 7000])
    size = L.tr_prefill_attn_batched_workspace_size(C.byref(sh), cu_p, rows_p, C.c_int32(2))
    assert size > 0

    def call(cu_p=cu_p, rows_p=rows_p, n=2, ws=FAKE2, ws_bytes=size):
        return L.tr_prefill_attn_batched(C.byref(sh), FAKE, FAKE, FAKE, FAKE, cu_p, rows_p, C.c_int32(n), FAKE, ws,
                                         C.c_size_t(ws_bytes), None)

    short, short_p = _i64([0, 30, 7000])        # request 0 has 40 query tokens but 30 cache rows
    assert call(rows_p=short_p) == B.TR_ERR_INVALID_ARG
    badcu, badcu_p = _i32([0, 50, 40])
    assert call(cu_p=badcu_p) == B.TR_ERR_INVALID_ARG
    assert call(ws_bytes=size // 2) == B.TR_ERR_WORKSPACE
    assert call(n=-1) == B.TR_ERR_INVALID_ARG
    assert call(n=0) == B.TR_OK


def test_chunk_prefill_validation(L):
    sh = _shape(32, 8, 128, B.TR_BF16, 5e5)
    size = L.tr_chunk_prefill_attn_workspace_size(C.byref(sh), C.c_int64(32768), C.c_int32(512))
    assert size > 0 and size % 256 == 0

    def call(n_chunks=64, total=32768, max_len=512, ws=FAKE2, ws_bytes=size, krot=FAKE, cu=FAKE, shape=sh):
        return L.tr_chunk_prefill_attn(C.byref(shape), FAKE, FAKE, FAKE, cu, C.c_int32(n_chunks), C.c_int64(total),
                                       C.c_int32(max_len), FAKE, krot, ws, C.c_size_t(ws_bytes), None)

    assert call(krot=None) == B.TR_ERR_INVALID_ARG                  # the rotated keys are the attention kernel's input
    assert call(cu=None) == B.TR_ERR_INVALID_ARG
    assert call(ws=None, ws_bytes=0) == B.TR_ERR_WORKSPACE
    assert call(ws_bytes=size - 256) == B.TR_ERR_WORKSPACE
    assert call(max_len=0) == B.TR_ERR_INVALID_ARG
    assert call(n_chunks=-1) == B.TR_ERR_INVALID_ARG
    assert call(shape=_shape(32, 8, 128, B.TR_BF16, 5e5, 9)) == B.TR_ERR_INVALID_ARG                  # unknown rope layout
    assert call(shape=_shape(32, 8, 128, B.TR_BF16, 5e5, B.TR_ROPE_HALF), total=0, n_chunks=0) == B.TR_OK
    assert call(total=0, n_chunks=0) == B.TR_OK


def test_binding_raises_with_the_library_message(L):
    sh = B.make_shape(28, 4, 96, "bf16", 1e6)
    with pytest.raises(B.TurboRagError) as e:
        B.Store(sh, None, None, np.array([0, 4]))
    assert e.value.code in (B.TR_ERR_SHAPE, B.TR_ERR_INVALID_ARG)


@pytest.mark.parametrize("mode", [B.TR_POS_COMPOSITE, B.TR_POS_REORDERED])
def test_sequence_plan_is_bit_exact_against_the_oracle(L, mode):
    for lens, n_tail, tail_start in [((3, 2), 2, -1), ((512,) * 8, 64, -1), ((), 5, -1), ((7, 0, 9), 0, -1), ((4, 4), 3, 100)]:
        seg, pos = B.tr_sequence_plan(lens, n_tail, mode, tail_start)
        want_seg, want_pos = oracle.sequence_plan(lens, n_tail, mode, None if tail_start < 0 else tail_start)
        assert np.array_equal(seg, want_seg) and np.array_equal(pos, want_pos)
    lens, lens_p = _i32([3, 2])
    buf = np.zeros(8, np.int32)
    bp = buf.ctypes.data_as(C.c_void_p)
    assert L.tr_sequence_plan(lens_p, C.c_int32(2), C.c_int32(2), C.c_int32(mode), C.c_int32(-1), bp, bp, C.c_int64(6)) == B.TR_ERR_BAD_PLAN
    assert L.tr_sequence_plan(lens_p, C.c_int32(2), C.c_int32(2), C.c_int32(7), C.c_int32(-1), bp, bp, C.c_int64(8)) == B.TR_ERR_INVALID_ARG
    assert L.tr_sequence_plan(None, C.c_int32(2), C.c_int32(2), C.c_int32(mode), C.c_int32(-1), bp, bp, C.c_int64(8)) == B.TR_ERR_INVALID_ARG
    bad, bad_p = _i32([3, -2])
    assert L.tr_sequence_plan(bad_p, C.c_int32(2), C.c_int32(2), C.c_int32(mode), C.c_int32(-1), bp, bp, C.c_int64(8)) == B.TR_ERR_INVALID_ARG


def test_sequence_prefill_validation(L):
    sh = _shape()
    call = lambda **kw: L.tr_sequence_prefill_attn(C.byref(kw.get("shape", sh)), kw.get("q", FAKE), FAKE, FAKE, kw.get("seg", FAKE),
                                                   kw.get("pos", FAKE), kw.get("seg_host", None), C.c_int64(kw.get("T", 100)), FAKE,
                                                   kw.get("krot", FAKE2), kw.get("ws", None), C.c_size_t(kw.get("ws_bytes", 0)), None)
    assert call(q=None) == B.TR_ERR_INVALID_ARG
    assert call(seg=None) == B.TR_ERR_INVALID_ARG
    assert call(pos=None) == B.TR_ERR_INVALID_ARG
    assert call(krot=None) == B.TR_ERR_INVALID_ARG
    assert call(T=-1) == B.TR_ERR_INVALID_ARG
    assert call(shape=_shape(d=96)) == B.TR_ERR_SHAPE
    assert call(T=0) == B.TR_OK
    # with the host copy of the starts, 256 tokens that each attend 40000 rows are cut into pieces: a workspace is needed
    T = 40000 + 256
    seg, seg_p = _i32(np.concatenate([np.arange(40000) // 1000 * 1000, np.zeros(256)]))
    L.tr_sequence_prefill_attn_workspace_size.restype = C.c_size_t
    size = L.tr_sequence_prefill_attn_workspace_size(C.byref(sh), seg_p, C.c_int64(T))
    n_split = size // (256 * sh.n_q_heads * (sh.head_dim * 2 + 8))
    assert 2 <= n_split <= 32 and size % 256 == 0, size
    assert L.tr_sequence_prefill_attn_workspace_size(C.byref(sh), None, C.c_int64(T)) == 0
    assert L.tr_sequence_prefill_attn_workspace_size(C.byref(sh), seg_p, C.c_int64(40000)) == 0    # chunks only: nothing is cut
    assert call(T=T, seg_host=seg_p) == B.TR_ERR_WORKSPACE
    assert call(T=T, seg_host=seg_p, ws=FAKE, ws_bytes=size - 256) == B.TR_ERR_WORKSPACE
    assert call(T=T, seg_host=seg_p, ws=C.c_void_p(0x1010), ws_bytes=size) == B.TR_ERR_WORKSPACE   # not 256-byte aligned


def test_gather_attention_validation(L):
    rc, h = _store(L, _shape(), [0, 4, 9, 9, 20])
    assert rc == B.TR_OK
    ids, ids_p = _i32([1, 3, 0])
    good, good_p = _i64([0, 5, 16, 20])
    size = L.tr_prefill_attn_gather_workspace_size(h, ids_p, good_p, C.c_int32(3), C.c_int32(1), C.c_int32(8))
    assert size == 0          # 20 document rows: nothing to split

    def call(ids_p=ids_p, off_p=good_p, n=3, mode=B.TR_POS_REORDERED, q=FAKE, ck=FAKE, n_q=8, cap=28, store=h):
        return L.tr_prefill_attn_gather(store, ids_p, off_p, C.c_int32(n), C.c_int32(mode), q, ck, FAKE2, FAKE, C.c_int32(n_q),
                                        C.c_int64(cap), FAKE2, None, C.c_size_t(0), None)

    bad, bad_p = _i64([0, 5, 15, 20])
    assert call(off_p=bad_p) == B.TR_ERR_BAD_PLAN
    badid, badid_p = _i32([1, 9, 0])
    assert call(ids_p=badid_p) == B.TR_ERR_BAD_CHUNK_ID
    assert call(cap=27) == B.TR_ERR_BAD_PLAN                  # the query rows do not fit the cache
    assert call(q=None) == B.TR_ERR_INVALID_ARG
    assert call(ck=None) == B.TR_ERR_INVALID_ARG
    assert call(store=None) == B.TR_ERR_INVALID_ARG
    assert call(mode=3) == B.TR_ERR_INVALID_ARG
    assert call(n_q=-1) == B.TR_ERR_INVALID_ARG
    assert call(n_q=0) == B.TR_OK
    L.tr_store_destroy(h)
    rc, h32 = _store(L, _shape(4, 4, 64, B.TR_F32, 1e4), [0, 4])
    one, one_p = _i32([0])
    off, off_p = _i64([0, 4])
    assert call(store=h32, ids_p=one_p, off_p=off_p, n=1) == B.TR_ERR_UNSUPPORTED     # bf16 only
    L.tr_store_destroy(h32)


def test_assemble_append_and_decode_validation(L):
    rc, h = _store(L, _shape(), [0, 4, 9, 9, 20])
    ids, ids_p = _i32([1, 3, 0])
    good, good_p = _i64([0, 5, 16, 20])

    def fused(n_q=4, cap=24, k=FAKE, off_p=good_p):
        return L.tr_kv_assemble_append(h, ids_p, off_p, C.c_int32(3), C.c_int32(1), k, FAKE, FAKE, C.c_int32(n_q), FAKE2, FAKE2,
                                       C.c_int64(cap), None)

    assert fused(cap=23) == B.TR_ERR_BAD_PLAN                 # documents fit, the query rows do not
    assert fused(k=None) == B.TR_ERR_INVALID_ARG
    assert fused(n_q=-1) == B.TR_ERR_INVALID_ARG
    bad, bad_p = _i64([0, 5, 15, 20])
    assert fused(off_p=bad_p) == B.TR_ERR_BAD_PLAN
    L.tr_store_destroy(h)

    sh = _shape()
    rows, rows_p = _i64([0, 100, 100, 250])                    # the second request has no cache row at all
    assert L.tr_decode_attn(C.byref(sh), FAKE, FAKE, FAKE, FAKE, rows_p, C.c_int32(3), FAKE, None, C.c_size_t(0), None) == B.TR_ERR_INVALID_ARG
    ok, ok_p = _i64([0, 100, 180, 250])
    assert L.tr_decode_attn_workspace_size(C.byref(sh), ok_p, C.c_int32(3)) == 0      # short caches: no key split
    assert L.tr_decode_attn(C.byref(sh), None, FAKE, FAKE, FAKE, ok_p, C.c_int32(3), FAKE, None, C.c_size_t(0), None) == B.TR_ERR_INVALID_ARG
    assert L.tr_decode_attn(C.byref(sh), FAKE, FAKE, FAKE, FAKE, ok_p, C.c_int32(-1), FAKE, None, C.c_size_t(0), None) == B.TR_ERR_INVALID_ARG
    assert L.tr_decode_attn(C.byref(sh), FAKE, FAKE, FAKE, FAKE, ok_p, C.c_int32(0), FAKE, None, C.c_size_t(0), None) == B.TR_OK


def test_linear_validation(L):
    L.tr_linear_workspace_size.restype = C.c_size_t
    ptrs = lambda *vals: (C.c_void_p * len(vals))(*vals)

    def call(x=FAKE, M=64, K=3584, feats=(3584,), w=None, y=None, ws=FAKE, ws_bytes=1 << 30, n_out=None):
        f, f_p = _i32(list(feats))
        n = len(feats) if n_out is None else n_out
        w = ptrs(*([0x10000] * len(feats))) if w is None else w
        y = ptrs(*([0x20000] * len(feats))) if y is None else y
        return L.tr_linear(x, C.c_int32(M), C.c_int32(K), C.c_int32(n), w, y, f_p, ws, C.c_size_t(ws_bytes), None)

    assert call(M=0) == B.TR_OK                                      # nothing to do, nothing enqueued
    assert call(x=None) == B.TR_ERR_INVALID_ARG
    assert call(w=ptrs(0)) == B.TR_ERR_INVALID_ARG
    assert call(y=ptrs(0)) == B.TR_ERR_INVALID_ARG
    assert call(M=-1) == B.TR_ERR_INVALID_ARG
    assert call(feats=(0,)) == B.TR_ERR_INVALID_ARG
    assert call(n_out=0) == B.TR_ERR_INVALID_ARG
    assert call(feats=(32,) * 5) == B.TR_ERR_INVALID_ARG             # at most four weights share x
    assert call(feats=(3600,)) == B.TR_ERR_SHAPE                     # not a multiple of 32
    assert call(feats=(3584, 500, 512)) == B.TR_ERR_SHAPE
    assert call(K=3590) == B.TR_ERR_SHAPE                            # not a multiple of 16
    assert call(M=129) == B.TR_ERR_UNSUPPORTED                       # more rows than the weight-streaming kernel takes
    assert call(x=C.c_void_p(0x1008)) == B.TR_ERR_INVALID_ARG        # misaligned operand
    assert call(w=ptrs(0x10008)) == B.TR_ERR_INVALID_ARG
    one, one_p = _i32([3584])
    size = L.tr_linear_workspace_size(C.c_int32(64), C.c_int32(1), one_p, C.c_int32(3584))
    assert size > 0 and size % 256 == 0 and size % (64 * 3584 * 4) == 0          # whole fp32 slices of y
    assert call(ws=None) == B.TR_ERR_WORKSPACE
    assert call(ws_bytes=size - 256) == B.TR_ERR_WORKSPACE
    assert call(ws=C.c_void_p(0x1010)) == B.TR_ERR_WORKSPACE
    qkv, qkv_p = _i32([3584, 512, 512])
    fused = L.tr_linear_workspace_size(C.c_int32(64), C.c_int32(3), qkv_p, C.c_int32(3584))
    assert fused % (64 * 4608 * 4) == 0 and fused > 0                # slices of all three outputs side by side
    big, big_p = _i32([131072])
    assert L.tr_linear_workspace_size(C.c_int32(64), C.c_int32(1), big_p, C.c_int32(3584)) == 0   # enough row tiles: no slicing
    bad, bad_p = _i32([3600])
    assert L.tr_linear_workspace_size(C.c_int32(64), C.c_int32(1), bad_p, C.c_int32(3584)) == 0   # invalid shape: 0


def test_batched_plan_is_the_same_with_and_without_its_memo(L):
    """The launch search of a mixed batch keeps its result for the last few batch shapes.  Twelve shapes (more than it
    keeps) queried forwards, backwards and forwards again, and once more after a policy override and its removal, give
    the same workspace sizes every time; two batches that differ in one cache length only are told apart."""
    rng = np.random.Generator(np.random.PCG64(99))
    sh = B.make_shape(28, 4, 128, "bf16", 1.0e6)
    batches = []
    for _ in range(12):
        n_req = int(rng.integers(2, 20))
        n_q = rng.integers(1, 129, n_req)
        n_doc = rng.integers(2000, 12000, n_req)
        batches.append((np.concatenate([[0], np.cumsum(n_q)]).astype(np.int32), np.concatenate([[0], np.cumsum(n_doc + n_q)]).astype(np.int64)))
    size = lambda b: B.tr_prefill_attn_batched_workspace_size(sh, b[0], b[1])
    first = [size(b) for b in batches]
    assert [size(b) for b in reversed(batches)] == first[::-1]
    assert [size(b) for b in batches] == first
    B.tr_set_tuning("min_split_keys", 1024)
    [size(b) for b in batches]   # whatever the override chooses must not stick once it is removed
    B.tr_set_tuning("min_split_keys", 0)
    assert [size(b) for b in batches] == first
    cu_q, crs = batches[0]
    longer = crs.copy()
    longer[-1] += 4096
    assert size((cu_q, longer)) >= first[0] and size(batches[0]) == first[0]


def test_launch_planners_on_random_request_mixes(L):
    """The host-side launch planners (key splits per request, chosen by playing the launch through) on 300 seeded
    random request mixes, through the workspace-size entry points: they return, the same input gives the same size,
    and the size stays within what the largest allowed number of key splits could need (64 partial rows of head_dim
    fp16 values plus two fp32 statistics per query row and head)."""
    rng = np.random.Generator(np.random.PCG64(4242))
    for case in range(300):
        hkv = int(rng.choice([1, 2, 4, 8]))
        g = int(rng.choice([1, 2, 4, 7, 8]))
        d = int(rng.choice([64, 128]))
        sh = B.make_shape(hkv * g, hkv, d, "bf16", 1.0e6)
        n_req = int(rng.integers(1, 24))
        n_q = rng.integers(0, 200, n_req) if case % 3 else rng.integers(0, 20, n_req)
        n_doc = rng.integers(0, 40000, n_req) if case % 2 else rng.integers(0, 3000, n_req)
        cu_q = np.concatenate([[0], np.cumsum(n_q)]).astype(np.int32)
        crs = np.concatenate([[0], np.cumsum(n_doc + n_q)]).astype(np.int64)
        size = B.tr_prefill_attn_batched_workspace_size(sh, cu_q, crs)
        assert size == B.tr_prefill_attn_batched_workspace_size(sh, cu_q, crs)
        bound = 64 * int(n_q.sum()) * hkv * g * (2 * d + 8) + 256
        assert 0 <= size <= bound, (case, size, bound)
        one = B.tr_prefill_attn_workspace_size(sh, int(n_q[0]), int(n_doc[0] + n_q[0]))
        assert 0 <= one <= 64 * int(n_q[0]) * hkv * g * (2 * d + 8) + 256
        dec = B.tr_decode_attn_workspace_size(sh, np.concatenate([[0], np.cumsum(n_doc + 1)]).astype(np.int64))
        assert 0 <= dec <= 64 * n_req * hkv * g * (2 * d + 8) + 256
        # a packed sequence: the documents of the first request as chunks, its query tokens as the tail
        lens = [int(x) for x in rng.integers(0, 1500, int(rng.integers(0, 12)))]
        seg, pos = B.tr_sequence_plan(lens, int(n_q[0]), int(case % 2))
        if seg.size:
            ws = B.tr_sequence_prefill_attn_workspace_size(sh, seg, seg.size)
            assert 0 <= ws <= 64 * seg.size * hkv * g * (2 * d + 8) + 256

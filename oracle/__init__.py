"""CPU fp64 oracle for the TurboRAG online-prefill hot path (arXiv 2410.07590).

TEST INFRASTRUCTURE ONLY: slow, plain and independent of the HIP library.  It
may be imported by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg, and by nothing else.  It imports nothing from the GPU package.

The arithmetic lives in turborag_oracle.c (one loop nest per definition); this
module only marshals numpy arrays into it and chains the steps of the pipeline
(Sec. 3.4 steps 2, 5, 6) in the paper's order.

Storage-typed arrays are passed as numpy float32, or numpy uint16 holding
bfloat16 bit patterns; everything the oracle returns is float64 unless the
function says it rounds to storage.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
ROPE_INTERLEAVED, ROPE_HALF = 0, 1
POS_COMPOSITE, POS_REORDERED = 0, 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        # TR_ORACLE_LIB: another build of turborag_oracle.c; the test that plants mistakes in copies of the source
        # and expects the pins to fail runs the pin tests against such a copy
        _lib = C.CDLL(os.environ.get("TR_ORACLE_LIB") or _build.build())
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _dtype_of(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("storage arrays are float32 or uint16 (bf16 bits), got %s" % a.dtype)


def _c(a, dtype=None):
    return np.ascontiguousarray(a, dtype=dtype)


def num_threads():
    return int(lib().orc_num_threads())


def theta(base, d):
    """theta_m = base^(-2m/d) (text after Eq. 3)."""
    out = np.empty(d // 2, np.float64)
    lib().orc_theta(C.c_double(base), C.c_int(d), _p(out))
    return out


def widen(x):
    """Exact storage -> float64."""
    x = _c(x)
    out = np.empty(x.shape, np.float64)
    lib().orc_widen(_p(x), C.c_int64(x.size), C.c_int(_dtype_of(x)), _p(out))
    return out


def round_to(x, dtype):
    """float64 -> storage dtype, round to nearest even.  Returns float32 or uint16 (bf16 bits)."""
    x = _c(x, np.float64)
    out = np.empty(x.shape, np.float32 if dtype == F32 else np.uint16)
    lib().orc_round(_p(x), C.c_int64(x.size), C.c_int(dtype), _p(out))
    return out


def rope(x, pos, base, layout=ROPE_INTERLEAVED):
    """R(pos[row]) x for x [rows, heads, d] (storage-typed or float64), Eq. 3."""
    x = _c(x)
    rows, heads, d = x.shape
    pos = _c(pos, np.int64)
    assert pos.shape == (rows,)
    out = np.empty(x.shape, np.float64)
    if x.dtype == np.float64:
        lib().orc_rope_f64(_p(x), C.c_int64(rows), C.c_int(heads), C.c_int(d), _p(pos),
                           C.c_double(base), C.c_int(layout), _p(out))
    else:
        lib().orc_rope(_p(x), C.c_int(_dtype_of(x)), C.c_int64(rows), C.c_int(heads), C.c_int(d),
                       _p(pos), C.c_double(base), C.c_int(layout), _p(out))
    return out


def plan(row_start, chunk_ids, pos_mode):
    """Gather plan and position ids (Sec. 3.2): returns (offsets[k+1], delta[k], pos[n_doc])."""
    row_start = _c(row_start, np.int64)
    chunk_ids = _c(chunk_ids, np.int32)
    k = chunk_ids.size
    n_store = row_start.size - 1
    offsets = np.zeros(k + 1, np.int64)
    delta = np.zeros(k, np.int64)
    # first pass without ids to learn n_doc (and validate), second pass fills ids
    rc = lib().orc_plan(_p(row_start), C.c_int(n_store), _p(chunk_ids), C.c_int(k), C.c_int(pos_mode),
                        _p(offsets), _p(delta), None)
    if rc != 0:
        raise ValueError("chunk id outside the store")
    pos = np.zeros(int(offsets[k]), np.int32)
    lib().orc_plan(_p(row_start), C.c_int(n_store), _p(chunk_ids), C.c_int(k), C.c_int(pos_mode),
                   _p(offsets), _p(delta), _p(pos))
    return offsets, delta, pos


def assemble(k_store, v_store, row_start, chunk_ids, offsets, delta, base, layout=ROPE_INTERLEAVED):
    """Contextual KV-cache formation (Sec. 3.4 step 5): float64 (K_asm, V_asm), each [n_doc, n_kv, d]."""
    k_store, v_store = _c(k_store), _c(v_store)
    _, n_kv, d = k_store.shape
    row_start = _c(row_start, np.int64)
    chunk_ids = _c(chunk_ids, np.int32)
    offsets = _c(offsets, np.int64)
    delta = _c(delta, np.int64)
    k = chunk_ids.size
    n_doc = int(offsets[k])
    out_k = np.empty((n_doc, n_kv, d), np.float64)
    out_v = np.empty((n_doc, n_kv, d), np.float64)
    lib().orc_assemble(_p(k_store), _p(v_store), C.c_int(_dtype_of(k_store)), _p(row_start), _p(chunk_ids),
                       C.c_int(k), _p(offsets), _p(delta), C.c_int(n_kv), C.c_int(d), C.c_double(base),
                       C.c_int(layout), _p(out_k), _p(out_v))
    return out_k, out_v


def attn_prefix(q_rot, k, v, rows=None):
    """Query prefill attention over an assembled cache (Eq. 2, Eq. 4, Sec. 3.4 step 6).

    q_rot [n_q, n_qh, d], k, v [kv_len, n_kv, d], all float64; the last n_q cache
    rows are the query tokens.  rows: query-token indices to compute (default all).
    """
    q_rot, k, v = _c(q_rot, np.float64), _c(k, np.float64), _c(v, np.float64)
    n_q, n_qh, d = q_rot.shape
    kv_len, n_kv, _ = k.shape
    assert v.shape == k.shape and kv_len >= n_q and n_qh % n_kv == 0
    rows = np.arange(n_q, dtype=np.int32) if rows is None else _c(rows, np.int32)
    out = np.empty((rows.size, n_qh, d), np.float64)
    lib().orc_attn_prefix(_p(q_rot), _p(k), _p(v), C.c_int(n_q), C.c_int64(kv_len), C.c_int(n_qh),
                          C.c_int(n_kv), C.c_int(d), _p(rows), C.c_int(rows.size), _p(out))
    return out


def attn_blockdiag(q_rot, k_rot, v, cu, rows=None):
    """Offline chunk prefill attention under the block-diagonal causal mask (Sec. 3.2, Sec. 3.4 step 2)."""
    q_rot, k_rot, v = _c(q_rot, np.float64), _c(k_rot, np.float64), _c(v, np.float64)
    T, n_qh, d = q_rot.shape
    _, n_kv, _ = k_rot.shape
    cu = _c(cu, np.int32)
    assert cu[0] == 0 and cu[-1] == T
    rows = np.arange(T, dtype=np.int32) if rows is None else _c(rows, np.int32)
    out = np.empty((rows.size, n_qh, d), np.float64)
    lib().orc_attn_blockdiag(_p(q_rot), _p(k_rot), _p(v), _p(cu), C.c_int(cu.size - 1), C.c_int(n_qh),
                             C.c_int(n_kv), C.c_int(d), _p(rows), C.c_int(rows.size), _p(out))
    return out


def attn_rows(q_rot, k_rot, v, lo, rows=None):
    """Attention over a packed sequence where token t sees rows lo[t] .. t (documents: their own chunk; query and
    answer tokens: everything before them), Sec. 3.2 / Sec. 3.3."""
    q_rot, k_rot, v = _c(q_rot, np.float64), _c(k_rot, np.float64), _c(v, np.float64)
    T, n_qh, d = q_rot.shape
    _, n_kv, _ = k_rot.shape
    lo = _c(lo, np.int32)
    assert lo.shape == (T,) and (lo >= 0).all() and (lo <= np.arange(T)).all()
    rows = np.arange(T, dtype=np.int32) if rows is None else _c(rows, np.int32)
    out = np.empty((rows.size, n_qh, d), np.float64)
    lib().orc_attn_rows(_p(q_rot), _p(k_rot), _p(v), _p(lo), C.c_int64(T), C.c_int(n_qh), C.c_int(n_kv), C.c_int(d),
                        _p(rows), C.c_int(rows.size), _p(out))
    return out


def sequence_plan(chunk_lens, n_tail, pos_mode, tail_start=None):
    """Visible-range starts and position ids of a packed training/prefill sequence [chunk_1 .. chunk_k, tail]
    (Sec. 3.2, Sec. 3.3): a document token sees its own chunk up to itself, a tail (query/answer) token sees
    everything before it; ids are chunk-local (composite) or run on (reordered); the tail's ids start at
    tail_start (default: longest chunk under composite positions, n_doc under reordered positions)."""
    chunk_lens = [int(l) for l in chunk_lens]
    n_doc = sum(chunk_lens)
    lo = np.zeros(n_doc + n_tail, np.int32)
    pos = np.zeros(n_doc + n_tail, np.int32)
    off = 0
    for l in chunk_lens:
        lo[off:off + l] = off
        pos[off:off + l] = np.arange(l) + (off if pos_mode == POS_REORDERED else 0)
        off += l
    if tail_start is None:
        tail_start = n_doc if pos_mode == POS_REORDERED else (max(chunk_lens) if chunk_lens else 0)
    pos[n_doc:] = tail_start + np.arange(n_tail)
    return lo, pos


# ---- the pipeline, steps chained in the paper's order ---------------------------------------------

def local_positions(cu):
    """Chunk-local position t - cu[c] of every packed token."""
    cu = np.asarray(cu, np.int64)
    pos = np.empty(int(cu[-1]), np.int64)
    for c in range(cu.size - 1):
        pos[cu[c]:cu[c + 1]] = np.arange(cu[c + 1] - cu[c])
    return pos


def online_prefill(k_store, v_store, row_start, chunk_ids, pos_mode, q, k_q, v_q, q_pos, base,
                   layout=ROPE_INTERLEAVED, rows=None, storage_rounding=True):
    """Sec. 3.4 steps 5 and 6 for one request, end to end.

    Store keys are already rotated at chunk-local positions.  Steps: plan -> assemble
    (re-rotate by the chunk offset under reordered positions) -> append the query tokens'
    own K (rotated at q_pos) and V -> attention of the rotated queries over the cache.
    With storage_rounding the assembled cache is rounded once to the storage dtype, as a
    cache held in that dtype is; the rounded cache is returned too (uint16/float32).
    Returns dict(out, offsets, delta, pos, k_cache, v_cache[, k_cache_st, v_cache_st]).
    """
    dt = _dtype_of(np.asarray(k_store))
    offsets, delta, pos = plan(row_start, chunk_ids, pos_mode)
    k_asm, v_asm = assemble(k_store, v_store, row_start, chunk_ids, offsets, delta, base, layout)
    kq_rot = rope(k_q, q_pos, base, layout)
    k_cache = np.concatenate([k_asm, kq_rot], axis=0)
    v_cache = np.concatenate([v_asm, widen(v_q)], axis=0)
    res = dict(offsets=offsets, delta=delta, pos=pos)
    if storage_rounding:
        res["k_cache_st"] = round_to(k_cache, dt)
        res["v_cache_st"] = round_to(v_cache, dt)
        k_cache, v_cache = widen(res["k_cache_st"]), widen(res["v_cache_st"])
    q_rot = rope(q, q_pos, base, layout)
    res["out"] = attn_prefix(q_rot, k_cache, v_cache, rows)
    res["k_cache"], res["v_cache"] = k_cache, v_cache
    return res


def offline_chunk_prefill(q, k, v, cu, base, layout=ROPE_INTERLEAVED, rows=None, storage_rounding=True):
    """Sec. 3.4 step 2 (attention part): rotate q, k at chunk-local positions, block-diagonal causal attention.

    Returns dict(out, k_rot[, k_rot_st]); k_rot_st is what the store keeps (rounded to storage).
    """
    dt = _dtype_of(np.asarray(k))
    lp = local_positions(cu)
    k_rot = rope(k, lp, base, layout)
    res = {}
    if storage_rounding:
        res["k_rot_st"] = round_to(k_rot, dt)
        k_rot = widen(res["k_rot_st"])
    q_rot = rope(q, lp, base, layout)
    res["out"] = attn_blockdiag(q_rot, k_rot, widen(v), cu, rows)
    res["k_rot"] = k_rot
    return res


def masked_prefill(q, k, v, lo, pos, base, layout=ROPE_INTERLEAVED, rows=None, storage_rounding=True):
    """One pass over a packed sequence: rotate q, k at pos (Eq. 3), token t attends rows lo[t] .. t.

    Returns dict(out, k_rot[, k_rot_st])."""
    dt = _dtype_of(np.asarray(k))
    k_rot = rope(k, pos, base, layout)
    res = {}
    if storage_rounding:
        res["k_rot_st"] = round_to(k_rot, dt)
        k_rot = widen(res["k_rot_st"])
    q_rot = rope(q, pos, base, layout)
    res["out"] = attn_rows(q_rot, k_rot, widen(v), lo, rows)
    res["k_rot"] = k_rot
    return res


def linear(x, w):
    """Projection of Eq. 1 (X W for the query, key and value weights; the output projection is the same product):
    y[m, n] = sum_k x[m, k] w[n, k], with w stored [out_features, in_features].  x, w: storage-typed arrays; returns
    float64 [M, N].  The contraction is numpy's matmul on the widened operands."""
    return np.matmul(widen(x), widen(w).T)

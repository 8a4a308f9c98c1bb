"""ctypes binding of libturborag_hip.so - same names as include/turborag.h, argument marshalling only.

Every step of the hot path runs in the library's HIP kernels.  torch is used for device
memory and for the current stream handle; nothing here computes.  If the library is missing
the import fails loudly: there is no fallback path.
"""
import ctypes as C
import os

import numpy as np
import torch

from . import build as _build

TR_OK = 0
TR_ERR_INVALID_ARG, TR_ERR_BAD_CHUNK_ID, TR_ERR_BAD_PLAN, TR_ERR_SHAPE = -1, -2, -3, -4
TR_ERR_UNSUPPORTED, TR_ERR_HIP, TR_ERR_WORKSPACE, TR_ERR_NO_MEMORY = -5, -6, -7, -8
TR_POS_COMPOSITE, TR_POS_REORDERED = 0, 1
TR_F32, TR_BF16 = 0, 1
TR_ROPE_INTERLEAVED, TR_ROPE_HALF = 0, 1

EXPORTS = [
    "tr_last_error", "tr_store_create", "tr_store_destroy", "tr_plan",
    "tr_kv_assemble", "tr_kv_assemble_raw", "tr_kv_assemble_batched", "tr_kv_append", "tr_kv_append_batched", "tr_kv_assemble_append",
    "tr_prefill_attn_workspace_size", "tr_prefill_attn", "tr_prefill_attn_static_scratch_bytes", "tr_prefill_attn_static",
    "tr_prefill_attn_batched_workspace_size", "tr_prefill_attn_batched",
    "tr_prefill_attn_gather_workspace_size", "tr_prefill_attn_gather",
    "tr_decode_attn_workspace_size", "tr_decode_attn",
    "tr_chunk_prefill_attn_workspace_size", "tr_chunk_prefill_attn",
    "tr_sequence_plan", "tr_sequence_prefill_attn_workspace_size", "tr_sequence_prefill_attn",
    "tr_linear_workspace_size", "tr_linear", "tr_set_tuning",
    "tr_probe_mfma_loop_sink_bytes", "tr_probe_mfma_loop",
]


class tr_shape(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("rope_base", C.c_double), ("rope_layout", C.c_int32),
                ("reserved", C.c_int32)]


class TurboRagError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("tr error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib_path():
    return _build.LIB


def lib():
    """Load the in-tree library (it must have been built: __graft_entry__.build() or `python -m ...build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            raise RuntimeError("libturborag_hip.so is not built; run `python -m paper_2410_07590_amd.build`")
        L = C.CDLL(_build.LIB)
        L.tr_last_error.restype = C.c_char_p
        for name in ("tr_prefill_attn_workspace_size", "tr_prefill_attn_batched_workspace_size",
                     "tr_prefill_attn_gather_workspace_size", "tr_decode_attn_workspace_size",
                     "tr_chunk_prefill_attn_workspace_size", "tr_sequence_prefill_attn_workspace_size",
                     "tr_linear_workspace_size", "tr_prefill_attn_static_scratch_bytes",
                     "tr_probe_mfma_loop_sink_bytes"):
            getattr(L, name).restype = C.c_size_t
        _lib = L
    return _lib


def _check(rc):
    if rc != TR_OK:
        raise TurboRagError(rc, lib().tr_last_error().decode())


def make_shape(n_q_heads, n_kv_heads, head_dim, dtype, rope_base, rope_layout=TR_ROPE_INTERLEAVED):
    if isinstance(dtype, str):
        dtype = {"f32": TR_F32, "bf16": TR_BF16}[dtype]
    elif isinstance(dtype, torch.dtype):
        dtype = {torch.float32: TR_F32, torch.bfloat16: TR_BF16}[dtype]
    return tr_shape(n_q_heads, n_kv_heads, head_dim, dtype, float(rope_base), rope_layout, 0)


def _dev(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous"
    return C.c_void_p(t.data_ptr())


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(C.c_void_p)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev_or_pinned(t):
    """Device tensor, or a pinned host tensor (its address is valid on the device: a host-resident store)."""
    if t is None:
        return None
    if not t.is_cuda:
        assert t.is_pinned() and t.is_contiguous(), "a host-resident store must be pinned, contiguous memory"
        return C.c_void_p(t.data_ptr())
    return _dev(t)


class Store:
    """Owns a tr_store handle; keeps the store tensors alive."""

    def __init__(self, shape, k_store, v_store, chunk_row_start):
        self.shape, self.k, self.v = shape, k_store, v_store
        rs, rs_p = _host(chunk_row_start, np.int64)
        self.row_start = rs
        self.handle = C.c_void_p(0)
        _check(lib().tr_store_create(C.byref(shape), _dev_or_pinned(k_store), _dev_or_pinned(v_store), rs_p,
                                     C.c_int32(rs.size - 1), C.byref(self.handle)))

    def close(self):
        if self.handle:
            lib().tr_store_destroy(self.handle)
            self.handle = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def tr_store_create(shape, k_store, v_store, chunk_row_start):
    return Store(shape, k_store, v_store, chunk_row_start)


def tr_plan(store, chunk_ids, pos_mode, want_pos_ids=True):
    """Returns (offsets int64[n+1], pos_ids int32[n_doc] or None)."""
    ids, ids_p = _host(chunk_ids, np.int32)
    offsets = np.zeros(ids.size + 1, np.int64)
    _check(lib().tr_plan(store.handle, ids_p, C.c_int32(ids.size), C.c_int32(pos_mode),
                         offsets.ctypes.data_as(C.c_void_p), None, C.c_int64(0)))
    if not want_pos_ids:
        return offsets, None
    pos = np.zeros(int(offsets[-1]), np.int32)
    _check(lib().tr_plan(store.handle, ids_p, C.c_int32(ids.size), C.c_int32(pos_mode),
                         offsets.ctypes.data_as(C.c_void_p), pos.ctypes.data_as(C.c_void_p), C.c_int64(pos.size)))
    return offsets, pos


def tr_kv_assemble(store, chunk_ids, offsets, pos_mode, out_k, out_v, stream=None):
    ids, ids_p = _host(chunk_ids, np.int32)
    off, off_p = _host(offsets, np.int64)
    _check(lib().tr_kv_assemble(store.handle, ids_p, off_p, C.c_int32(ids.size), C.c_int32(pos_mode),
                                _dev(out_k), _dev(out_v), C.c_int64(out_k.shape[0]), _stream(stream)))


def tr_kv_assemble_raw(store, chunk_ids, offsets, pos_mode, out_k, out_v, stream=None):
    """`store` holds un-rotated keys; every key is turned once, at its position id."""
    ids, ids_p = _host(chunk_ids, np.int32)
    off, off_p = _host(offsets, np.int64)
    _check(lib().tr_kv_assemble_raw(store.handle, ids_p, off_p, C.c_int32(ids.size), C.c_int32(pos_mode),
                                    _dev(out_k), _dev(out_v), C.c_int64(out_k.shape[0]), _stream(stream)))


def tr_kv_assemble_batched(store, chunk_ids, cu_chunks, pos_modes, cache_row_start, out_k, out_v, stream=None):
    ids, ids_p = _host(chunk_ids, np.int32)
    cu, cu_p = _host(cu_chunks, np.int32)
    pm, pm_p = _host(pos_modes, np.int32)
    rs, rs_p = _host(cache_row_start, np.int64)
    _check(lib().tr_kv_assemble_batched(store.handle, ids_p, cu_p, pm_p, rs_p, C.c_int32(pm.size),
                                        _dev(out_k), _dev(out_v), C.c_int64(out_k.shape[0]), _stream(stream)))


def tr_kv_append(shape, k_new, v_new, q_pos, cache_k, cache_v, dst_row, stream=None):
    _check(lib().tr_kv_append(C.byref(shape), _dev(k_new), _dev(v_new), _dev(q_pos), C.c_int32(k_new.shape[0]),
                              _dev(cache_k), _dev(cache_v), C.c_int64(dst_row), C.c_int64(cache_k.shape[0]),
                              _stream(stream)))


def tr_kv_assemble_append(store, chunk_ids, offsets, pos_mode, k_new, v_new, q_pos, out_k, out_v, stream=None):
    ids, ids_p = _host(chunk_ids, np.int32)
    off, off_p = _host(offsets, np.int64)
    _check(lib().tr_kv_assemble_append(store.handle, ids_p, off_p, C.c_int32(ids.size), C.c_int32(pos_mode), _dev(k_new), _dev(v_new),
                                       _dev(q_pos), C.c_int32(k_new.shape[0]), _dev(out_k), _dev(out_v), C.c_int64(out_k.shape[0]),
                                       _stream(stream)))


def tr_kv_append_batched(shape, k_new, v_new, q_pos, cu_q, cache_row_start, cache_k, cache_v, stream=None):
    cu, cu_p = _host(cu_q, np.int32)
    rs, rs_p = _host(cache_row_start, np.int64)
    _check(lib().tr_kv_append_batched(C.byref(shape), _dev(k_new), _dev(v_new), _dev(q_pos), cu_p, rs_p,
                                      C.c_int32(cu.size - 1), _dev(cache_k), _dev(cache_v),
                                      C.c_int64(cache_k.shape[0]), _stream(stream)))


def tr_prefill_attn_workspace_size(shape, n_q, kv_len):
    return int(lib().tr_prefill_attn_workspace_size(C.byref(shape), C.c_int32(n_q), C.c_int64(kv_len)))


def tr_prefill_attn(shape, q, k, v, q_pos, kv_len, out, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tr_prefill_attn(C.byref(shape), _dev(q), _dev(k), _dev(v), _dev(q_pos), C.c_int32(q.shape[0]),
                                 C.c_int64(kv_len), _dev(out), _dev(workspace), C.c_size_t(ws_bytes), _stream(stream)))


def tr_prefill_attn_static_scratch_bytes():
    return int(lib().tr_prefill_attn_static_scratch_bytes())


def tr_prefill_attn_static(shape, q, k, v, q_pos, kv_len, out, stream=None):
    """tr_prefill_attn with the library's own static scratch array instead of a workspace (no device allocation)."""
    _check(lib().tr_prefill_attn_static(C.byref(shape), _dev(q), _dev(k), _dev(v), _dev(q_pos), C.c_int32(q.shape[0]),
                                        C.c_int64(kv_len), _dev(out), _stream(stream)))


def tr_set_tuning(name, value):
    _check(lib().tr_set_tuning(name.encode(), C.c_int32(int(value))))


def tr_probe_mfma_loop_sink_bytes():
    return int(lib().tr_probe_mfma_loop_sink_bytes())


def tr_probe_mfma_loop(iters, random_operands, sink, stream=None):
    """Launch the matrix-instruction loop; returns the flops of the launch (the caller times it)."""
    flops = C.c_double(0.0)
    _check(lib().tr_probe_mfma_loop(C.c_int32(int(iters)), C.c_int32(1 if random_operands else 0), _dev(sink),
                                    C.c_size_t(sink.numel() * sink.element_size()), C.byref(flops), _stream(stream)))
    return flops.value


def tr_prefill_attn_batched_workspace_size(shape, cu_q, cache_row_start):
    cu, cu_p = _host(cu_q, np.int32)
    rs, rs_p = _host(cache_row_start, np.int64)
    return int(lib().tr_prefill_attn_batched_workspace_size(C.byref(shape), cu_p, rs_p, C.c_int32(cu.size - 1)))


def tr_prefill_attn_batched(shape, q, k, v, q_pos, cu_q, cache_row_start, out, workspace=None, stream=None):
    cu, cu_p = _host(cu_q, np.int32)
    rs, rs_p = _host(cache_row_start, np.int64)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tr_prefill_attn_batched(C.byref(shape), _dev(q), _dev(k), _dev(v), _dev(q_pos), cu_p, rs_p,
                                         C.c_int32(cu.size - 1), _dev(out), _dev(workspace), C.c_size_t(ws_bytes),
                                         _stream(stream)))


def tr_prefill_attn_gather_workspace_size(store, chunk_ids, offsets, pos_mode, n_q):
    ids, ids_p = _host(chunk_ids, np.int32)
    off, off_p = _host(offsets, np.int64)
    return int(lib().tr_prefill_attn_gather_workspace_size(store.handle, ids_p, off_p, C.c_int32(ids.size), C.c_int32(pos_mode),
                                                           C.c_int32(n_q)))


def tr_prefill_attn_gather(store, chunk_ids, offsets, pos_mode, q, cache_k, cache_v, q_pos, out, workspace=None, stream=None):
    ids, ids_p = _host(chunk_ids, np.int32)
    off, off_p = _host(offsets, np.int64)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tr_prefill_attn_gather(store.handle, ids_p, off_p, C.c_int32(ids.size), C.c_int32(pos_mode), _dev(q), _dev(cache_k),
                                        _dev(cache_v), _dev(q_pos), C.c_int32(q.shape[0]), C.c_int64(cache_k.shape[0]), _dev(out),
                                        _dev(workspace), C.c_size_t(ws_bytes), _stream(stream)))


def tr_decode_attn_workspace_size(shape, cache_row_start):
    rs, rs_p = _host(cache_row_start, np.int64)
    return int(lib().tr_decode_attn_workspace_size(C.byref(shape), rs_p, C.c_int32(rs.size - 1)))


def tr_decode_attn(shape, q, k, v, q_pos, cache_row_start, out, workspace=None, stream=None):
    rs, rs_p = _host(cache_row_start, np.int64)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tr_decode_attn(C.byref(shape), _dev(q), _dev(k), _dev(v), _dev(q_pos), rs_p, C.c_int32(rs.size - 1),
                                _dev(out), _dev(workspace), C.c_size_t(ws_bytes), _stream(stream)))


def tr_chunk_prefill_attn_workspace_size(shape, total_tokens, max_chunk_len):
    return int(lib().tr_chunk_prefill_attn_workspace_size(C.byref(shape), C.c_int64(total_tokens), C.c_int32(max_chunk_len)))


def tr_chunk_prefill_attn(shape, q, k, v, cu_chunk_lens, n_chunks, max_chunk_len, out, k_rot_out, workspace, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tr_chunk_prefill_attn(C.byref(shape), _dev(q), _dev(k), _dev(v), _dev(cu_chunk_lens),
                                       C.c_int32(n_chunks), C.c_int64(q.shape[0]), C.c_int32(max_chunk_len),
                                       _dev(out), _dev(k_rot_out), _dev(workspace), C.c_size_t(ws_bytes),
                                       _stream(stream)))


def tr_sequence_plan(chunk_lens, n_tail, pos_mode, tail_start=-1):
    """Returns (seg_start int32[T], pos int32[T]) for the packed sequence [chunks, tail]."""
    lens, lens_p = _host(chunk_lens, np.int32)
    total = int(lens.sum()) + int(n_tail)
    seg = np.zeros(max(total, 1), np.int32)
    pos = np.zeros(max(total, 1), np.int32)
    _check(lib().tr_sequence_plan(lens_p, C.c_int32(lens.size), C.c_int32(n_tail), C.c_int32(pos_mode), C.c_int32(tail_start),
                                  seg.ctypes.data_as(C.c_void_p), pos.ctypes.data_as(C.c_void_p), C.c_int64(total)))
    return seg[:total], pos[:total]


def tr_sequence_prefill_attn_workspace_size(shape, seg_start_host, total_tokens):
    if seg_start_host is None:
        return 0
    h = np.ascontiguousarray(seg_start_host, dtype=np.int32)
    return int(lib().tr_sequence_prefill_attn_workspace_size(C.byref(shape), h.ctypes.data_as(C.c_void_p), C.c_int64(total_tokens)))


def tr_sequence_prefill_attn(shape, q, k, v, seg_start, pos, out, k_rot_out, seg_start_host=None, workspace=None, stream=None):
    """seg_start_host: the host array tr_sequence_plan returned (lets the library cut long key ranges into pieces)."""
    h = None if seg_start_host is None else np.ascontiguousarray(seg_start_host, dtype=np.int32)
    hp = C.c_void_p(0) if h is None else h.ctypes.data_as(C.c_void_p)
    _check(lib().tr_sequence_prefill_attn(C.byref(shape), _dev(q), _dev(k), _dev(v), _dev(seg_start), _dev(pos), hp,
                                          C.c_int64(q.shape[0]), _dev(out), _dev(k_rot_out), _dev(workspace),
                                          C.c_size_t(0 if workspace is None else workspace.numel()), _stream(stream)))


def _features(n_features):
    f = np.atleast_1d(np.asarray(n_features, dtype=np.int32))
    return f, f.ctypes.data_as(C.c_void_p)


def tr_linear_workspace_size(M, n_features, K):
    f, fp = _features(n_features)
    return int(lib().tr_linear_workspace_size(C.c_int32(M), C.c_int32(f.size), fp, C.c_int32(K)))


def tr_linear(x, w, y, workspace=None, stream=None):
    """y[j][M, N_j] = x[M, K] @ w[j][N_j, K]^T, bf16, at most 128 rows of x.  w, y: one tensor each, or lists of up to four
    that share x."""
    ws_, ys_ = (list(w), list(y)) if isinstance(w, (list, tuple)) else ([w], [y])
    M, K = x.shape
    for wj, yj in zip(ws_, ys_):
        assert wj.shape[1] == K and yj.numel() == M * wj.shape[0]
    f, fp = _features([wj.shape[0] for wj in ws_])
    wp = (C.c_void_p * len(ws_))(*[_dev(t) for t in ws_])
    yp = (C.c_void_p * len(ys_))(*[_dev(t) for t in ys_])
    _check(lib().tr_linear(_dev(x), C.c_int32(M), C.c_int32(K), C.c_int32(len(ws_)), wp, yp, fp, _dev(workspace),
                           C.c_size_t(0 if workspace is None else workspace.numel()), _stream(stream)))


def workspace(nbytes, device="cuda"):
    """A 256-byte aligned device scratch tensor (torch's allocator aligns to at least 512 bytes)."""
    t = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    assert t.data_ptr() % 256 == 0
    return t

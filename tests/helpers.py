"""Shared plumbing of the GPU parity tests: run one workload through the C ABI (via the binding)
and through the CPU oracle on the same bits."""
import numpy as np
import torch

import oracle
from paper_2410_07590_amd import synth

BF16_TOL = 2e-2   # max abs error, bf16 storage with fp32 accumulation
F32_TOL = 1e-4    # max abs error, fp32 configurations


def tol_for(shape):
    return F32_TOL if shape.dtype == "f32" else BF16_TOL


def to_f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def bits(t):
    return synth.as_oracle_array(t)


def bits_t(t):
    """The tensor's storage as integers, for bit-for-bit comparisons that treat equal NaNs as equal."""
    t = t.detach().cpu().contiguous()
    return t.view(torch.int16 if t.element_size() == 2 else torch.int32)


def assert_same_bits(got, want, what, max_mismatch_frac=0.0):
    """Bit-for-bit equality of two storage-typed arrays.  For rotated keys a tiny fraction of one-ulp
    differences is tolerated: device and host sin/cos are each within ~1 ulp of fp64, so an fp64
    result that lands within ~1e-16 relative of a rounding boundary may round the other way."""
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape and got.dtype == want.dtype, what
    neq = got != want
    n_bad = int(neq.sum())
    if n_bad == 0:
        return 0
    assert n_bad <= max_mismatch_frac * got.size, "%s: %d of %d elements differ" % (what, n_bad, got.size)
    if got.dtype == np.uint16:
        d = np.abs(got[neq].astype(np.int32) - want[neq].astype(np.int32))
    else:
        d = np.abs(got[neq].view(np.int32).astype(np.int64) - want[neq].view(np.int32).astype(np.int64))
    assert d.max() <= 1, "%s: a mismatch larger than one ulp" % what
    return n_bad


def gpu_shape(B, sh):
    return B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base, sh.rope_layout)


def run_request_gpu(B, sh, store_dev, req, slack_rows=0):
    """assemble + append + prefill attention for one request through the C ABI.  Returns dict of CPU tensors."""
    gs = store_dev.shape
    offsets, pos = B.tr_plan(store_dev, req.chunk_ids, req.pos_mode)
    n_doc = int(offsets[-1])
    kv_len = n_doc + req.n_q
    dt = sh.torch_dtype
    cache_k = torch.full((kv_len + slack_rows, sh.n_kv_heads, sh.head_dim), float("nan"), dtype=dt, device="cuda")
    cache_v = torch.full_like(cache_k, float("nan"))
    B.tr_kv_assemble(store_dev, req.chunk_ids, offsets, req.pos_mode, cache_k, cache_v)
    q_pos = torch.from_numpy(req.q_pos).cuda()
    if req.n_q > 0:
        B.tr_kv_append(gs, req.k_q.cuda(), req.v_q.cuda(), q_pos, cache_k, cache_v, n_doc)
    out = torch.full((req.n_q, sh.n_q_heads, sh.head_dim), float("nan"), dtype=dt, device="cuda")
    ws = B.workspace(B.tr_prefill_attn_workspace_size(gs, req.n_q, kv_len))
    if req.n_q > 0:
        B.tr_prefill_attn(gs, req.q.cuda(), cache_k, cache_v, q_pos, kv_len, out, ws)
    torch.cuda.synchronize()
    return dict(offsets=offsets, pos=pos, cache_k=cache_k.cpu(), cache_v=cache_v.cpu(), out=out.cpu(), kv_len=kv_len)


def run_request_oracle(sh, store, req, rows=None):
    return oracle.online_prefill(bits(store.k), bits(store.v), store.row_start, req.chunk_ids, req.pos_mode,
                                 bits(req.q), bits(req.k_q), bits(req.v_q), req.q_pos, sh.rope_base, layout=sh.rope_layout, rows=rows)


def check_request(B, sh, store, store_dev, req, rows=None, k_mismatch_frac=1e-5):
    """Full parity of one request: plan and ids bit-exact, cache bytes bit-exact, output within tolerance."""
    g = run_request_gpu(B, sh, store_dev, req)
    o = run_request_oracle(sh, store, req, rows)
    assert np.array_equal(g["offsets"], o["offsets"])
    assert np.array_equal(g["pos"], o["pos"])
    kv_len = g["kv_len"]
    assert_same_bits(bits(g["cache_v"])[:kv_len], o["v_cache_st"], "assembled V")
    frac = k_mismatch_frac if (req.pos_mode == synth.POS_REORDERED or req.n_q > 0) else 0.0
    n_bad = assert_same_bits(bits(g["cache_k"])[:kv_len], o["k_cache_st"], "assembled K", frac)
    got = to_f64(g["out"])
    if rows is not None:
        got = got[np.asarray(rows)]
    err = float(np.abs(got - o["out"]).max()) if got.size else 0.0
    assert np.isfinite(got).all()
    assert err <= tol_for(sh), "attention max abs err %.3e" % err
    return err, n_bad


def run_request_gather_gpu(B, sh, store_dev, req):
    """The same request through tr_prefill_attn_gather: only the query tokens' rows of the cache are written (append); the
    document rows stay NaN, which shows that the attention reads the documents from the store."""
    gs = store_dev.shape
    offsets, _ = B.tr_plan(store_dev, req.chunk_ids, req.pos_mode, want_pos_ids=False)
    n_doc = int(offsets[-1])
    kv_len = n_doc + req.n_q
    dt = sh.torch_dtype
    cache_k = torch.full((kv_len, sh.n_kv_heads, sh.head_dim), float("nan"), dtype=dt, device="cuda")
    cache_v = torch.full_like(cache_k, float("nan"))
    q_pos = torch.from_numpy(req.q_pos).cuda()
    B.tr_kv_append(gs, req.k_q.cuda(), req.v_q.cuda(), q_pos, cache_k, cache_v, n_doc)
    out = torch.full((req.n_q, sh.n_q_heads, sh.head_dim), float("nan"), dtype=dt, device="cuda")
    ws = B.workspace(B.tr_prefill_attn_gather_workspace_size(store_dev, req.chunk_ids, offsets, req.pos_mode, req.n_q))
    B.tr_prefill_attn_gather(store_dev, req.chunk_ids, offsets, req.pos_mode, req.q.cuda(), cache_k, cache_v, q_pos, out, ws)
    torch.cuda.synchronize()
    return out.cpu()


def check_request_gather(B, sh, store, store_dev, req, rows=None):
    got = to_f64(run_request_gather_gpu(B, sh, store_dev, req))
    o = run_request_oracle(sh, store, req, rows)
    if rows is not None:
        got = got[np.asarray(rows)]
    assert np.isfinite(got).all()
    err = float(np.abs(got - o["out"]).max()) if got.size else 0.0
    assert err <= tol_for(sh), "gather attention max abs err %.3e" % err
    return err

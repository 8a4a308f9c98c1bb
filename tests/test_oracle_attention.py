"""Pins for the oracle's masked softmax attention (Eq. 2, Eq. 4, Sec. 3.2) and for the
chained pipeline.  The paper prints no worked numeric example of attention, so these are
the independent routes to the same numbers: brute force with an explicit mask matrix in
extended precision, a library attention routine on the special cases it covers, and
exact closed-form cases that show which keys are visible."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2410_07590_amd import accounting, synth

RNG = np.random.default_rng(23)


def brute_force(q, k, v, mask):
    """Triple loop with a materialised mask matrix, long double.  q [nq,H,d], k,v [nk,Hkv,d], mask [nq,nk] bool."""
    nq, H, d = q.shape
    nk, Hkv, _ = k.shape
    g = H // Hkv
    out = np.zeros((nq, H, d), np.longdouble)
    for i in range(nq):
        for h in range(H):
            s = np.full(nk, -np.inf, np.longdouble)
            for j in range(nk):
                if mask[i, j]:
                    acc = np.longdouble(0)
                    for e in range(d):
                        acc += np.longdouble(q[i, h, e]) * np.longdouble(k[j, h // g, e])
                    s[j] = acc / np.sqrt(np.longdouble(d))
            w = np.exp(s - s.max())
            w = w / w.sum()
            for j in range(nk):
                out[i, h] += w[j] * v[j, h // g].astype(np.longdouble)
    return out.astype(np.float64)


def prefix_mask(n_q, kv_len):
    n_doc = kv_len - n_q
    return np.array([[j <= n_doc + i for j in range(kv_len)] for i in range(n_q)])


def blockdiag_mask(cu):
    T = cu[-1]
    owner = np.zeros(T, int)
    for c in range(len(cu) - 1):
        owner[cu[c]:cu[c + 1]] = c
    return np.array([[owner[i] == owner[j] and j <= i for j in range(T)] for i in range(T)])


@pytest.mark.parametrize("n_q,kv_len,H,Hkv,d", [(3, 8, 2, 1, 4), (4, 4, 4, 2, 8), (1, 6, 3, 3, 6), (5, 7, 6, 2, 4)])
def test_prefix_attention_brute_force(n_q, kv_len, H, Hkv, d):
    q = RNG.standard_normal((n_q, H, d)); k = RNG.standard_normal((kv_len, Hkv, d)); v = RNG.standard_normal((kv_len, Hkv, d))
    want = brute_force(q, k, v, prefix_mask(n_q, kv_len))
    assert np.allclose(oracle.attn_prefix(q, k, v), want, atol=1e-13)
    rows = np.array([n_q - 1, 0], np.int32)
    assert np.allclose(oracle.attn_prefix(q, k, v, rows), want[rows], atol=1e-13)


@pytest.mark.parametrize("lens,H,Hkv,d", [((3, 1, 4), 2, 1, 4), ((2, 5), 4, 2, 6), ((6,), 2, 2, 4)])
def test_blockdiag_attention_brute_force(lens, H, Hkv, d):
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    q = RNG.standard_normal((T, H, d)); k = RNG.standard_normal((T, Hkv, d)); v = RNG.standard_normal((T, Hkv, d))
    want = brute_force(q, k, v, blockdiag_mask(cu))
    assert np.allclose(oracle.attn_blockdiag(q, k, v, cu), want, atol=1e-13)


def sdpa(q, k, v, mask=None, causal=False):
    """Library routine: torch's scaled_dot_product_attention in float64, heads repeated for GQA."""
    g = q.shape[1] // k.shape[1]
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).repeat_interleave(g, dim=1).permute(1, 0, 2)[None]
    tv = torch.from_numpy(v).repeat_interleave(g, dim=1).permute(1, 0, 2)[None]
    m = None if mask is None else torch.from_numpy(mask)[None, None]
    o = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=m, is_causal=causal)
    return o[0].permute(1, 0, 2).numpy()


def test_prefix_attention_against_library_routine():
    n_q, kv_len, H, Hkv, d = 16, 144, 8, 2, 64
    q = RNG.standard_normal((n_q, H, d)); k = RNG.standard_normal((kv_len, Hkv, d)); v = RNG.standard_normal((kv_len, Hkv, d))
    got = oracle.attn_prefix(q, k, v)
    assert np.allclose(got, sdpa(q, k, v, mask=prefix_mask(n_q, kv_len)), atol=1e-12)
    # special cases the library covers without a mask argument:
    # kv_len == n_q is ordinary causal self-attention; n_q == 1 sees every key (no mask at all)
    assert np.allclose(oracle.attn_prefix(q, k[:n_q], v[:n_q]), sdpa(q, k[:n_q], v[:n_q], causal=True), atol=1e-12)
    assert np.allclose(oracle.attn_prefix(q[:1], k, v), sdpa(q[:1], k, v), atol=1e-12)
    # GQA == MHA after repeating each KV head g times (consecutive grouping)
    g = H // Hkv
    assert np.allclose(got, oracle.attn_prefix(q, np.repeat(k, g, axis=1), np.repeat(v, g, axis=1)), atol=1e-14)


def test_blockdiag_equals_independent_causal_attention_per_chunk():
    # Sec. 3.2: independent attention == computing each chunk on its own
    lens = (33, 1, 64, 20)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, H, Hkv, d = int(cu[-1]), 4, 2, 32
    q = RNG.standard_normal((T, H, d)); k = RNG.standard_normal((T, Hkv, d)); v = RNG.standard_normal((T, Hkv, d))
    got = oracle.attn_blockdiag(q, k, v, cu)
    for c in range(len(lens)):
        s, e = cu[c], cu[c + 1]
        assert np.allclose(got[s:e], sdpa(q[s:e], k[s:e], v[s:e], causal=True), atol=1e-12)
        assert np.allclose(got[s:e], oracle.attn_prefix(q[s:e], k[s:e], v[s:e]), atol=1e-14)
        assert np.allclose(got[s], np.repeat(v[s], H // Hkv, axis=0), atol=1e-15)   # first token of a chunk: o = v
    rows = np.array([0, 33, 34, 97, T - 1], np.int32)
    assert np.allclose(oracle.attn_blockdiag(q, k, v, cu, rows), got[rows], atol=0)


def test_zero_queries_expose_the_mask_geometry():
    # Q = 0 -> uniform weights over the visible keys -> output = mean of the visible values, exactly
    n_q, kv_len, H, Hkv, d = 5, 12, 4, 2, 8
    k = RNG.standard_normal((kv_len, Hkv, d)); v = RNG.standard_normal((kv_len, Hkv, d))
    got = oracle.attn_prefix(np.zeros((n_q, H, d)), k, v)
    n_doc = kv_len - n_q
    for i in range(n_q):
        want = v[: n_doc + i + 1].mean(axis=0)
        assert np.allclose(got[i], np.repeat(want, H // Hkv, axis=0), atol=1e-15)
    cu = np.array([0, 4, 5, 12], np.int32)
    got = oracle.attn_blockdiag(np.zeros((12, H, d)), k, v, cu)
    for c in range(3):
        for t in range(cu[c], cu[c + 1]):
            want = v[cu[c]: t + 1].mean(axis=0)
            assert np.allclose(got[t], np.repeat(want, H // Hkv, axis=0), atol=1e-15)


def test_softmax_properties():
    n_q, kv_len, H, d = 3, 9, 2, 8
    q = RNG.standard_normal((n_q, H, d)); k = RNG.standard_normal((kv_len, H, d)); v = RNG.standard_normal((kv_len, H, d))
    base = oracle.attn_prefix(q, k, v)
    # weights sum to one: constant values come back unchanged
    assert np.allclose(oracle.attn_prefix(q, k, np.full_like(v, 2.5)), 2.5, atol=1e-14)
    # adding the same vector to every key shifts every score of a row by a constant: output unchanged
    assert np.allclose(oracle.attn_prefix(q, k + RNG.standard_normal((1, H, d)), v), base, atol=1e-12)
    # identical keys -> mean of visible values; a single key -> its value
    same = np.repeat(k[:1], kv_len, axis=0)
    got = oracle.attn_prefix(q, same, v)
    for i in range(n_q):
        assert np.allclose(got[i], v[: kv_len - n_q + i + 1].mean(axis=0), atol=1e-14)
    assert np.allclose(oracle.attn_prefix(q[:1], k[:1], v[:1]), v[:1], atol=1e-15)
    # the scale is 1/sqrt(d): with one-hot q and keys e_0 * s_j the weights are softmax(s_j / sqrt(d))
    qq = np.zeros((1, 1, d)); qq[0, 0, 0] = 1.0
    s = np.array([0.3, -1.2, 2.0, 0.0])
    kk = np.zeros((4, 1, d)); kk[:, 0, 0] = s
    vv = np.eye(4)[:, None, :]
    vv = np.concatenate([vv, np.zeros((4, 1, d - 4))], axis=-1)
    w = np.exp(s / np.sqrt(d)); w /= w.sum()
    assert np.allclose(oracle.attn_prefix(qq, kk, vv)[0, 0, :4], w, atol=1e-15)


def test_softmax_is_exact_for_scores_of_any_size():
    """Scores hundreds of nats above and below zero, where exp of the score itself overflows or vanishes in fp64: the
    weights are those of the shifted scores (closed form in extended precision), in any key order."""
    d = 16
    qq = np.zeros((1, 1, d)); qq[0, 0, 0] = 1.0
    for s in ([-3000.0, -2990.5, -2992.0, -3400.0], [800.0, 805.0, -20.0, 803.5, 0.0], [-5.0, 900.0, 899.0], [750.0, 10.0, 751.0]):
        s = np.array(s)
        kk = np.zeros((s.size, 1, d)); kk[:, 0, 0] = s * np.sqrt(d)
        vv = np.zeros((s.size, 1, d)); vv[np.arange(s.size), 0, np.arange(s.size)] = 1.0
        w = np.exp(s.astype(np.longdouble) - np.longdouble(s.max()))
        w = (w / w.sum()).astype(np.float64)
        got = oracle.attn_prefix(qq, kk, vv)[0, 0, :s.size]
        assert np.isfinite(got).all() and np.allclose(got, w, atol=1e-14)
        lo = np.zeros(s.size, np.int32)
        got = oracle.attn_rows(np.repeat(qq, s.size, axis=0), kk, vv, lo, rows=np.array([s.size - 1], np.int32))[0, 0, :s.size]
        assert np.allclose(got, w, atol=1e-14)
        cu = np.array([0, s.size], np.int32)
        got = oracle.attn_blockdiag(np.repeat(qq, s.size, axis=0), kk, vv, cu, rows=np.array([s.size - 1], np.int32))[0, 0, :s.size]
        assert np.allclose(got, w, atol=1e-14)


def test_pipeline_reordered_equals_standard_rope_attention_with_independent_chunks():
    """End to end (Sec. 3.2 + Sec. 3.4): a store built offline from raw keys at chunk-local positions,
    assembled with re-rotation by the chunk offsets, gives the same query output as rotating the raw keys
    once at their global ids and running ordinary attention; composite mode likewise with composite ids."""
    n_kv, g, d, base = 2, 2, 16, 1e4
    H = n_kv * g
    lens = (6, 9, 4)
    row_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rows = int(row_start[-1])
    k_raw = RNG.standard_normal((rows, n_kv, d)).astype(np.float32)
    v = RNG.standard_normal((rows, n_kv, d)).astype(np.float32)
    k_store = oracle.round_to(oracle.rope(k_raw, oracle.local_positions(row_start), base), oracle.F32)
    ids = np.array([1, 2, 0], np.int32)
    n_q = 5
    q = RNG.standard_normal((n_q, H, d)).astype(np.float32)
    k_q = RNG.standard_normal((n_q, n_kv, d)).astype(np.float32)
    v_q = RNG.standard_normal((n_q, n_kv, d)).astype(np.float32)
    for mode in (oracle.POS_REORDERED, oracle.POS_COMPOSITE):
        _, _, pos = oracle.plan(row_start, ids, mode)
        lens_sel = [lens[c] for c in ids]
        q_pos = synth.query_start(mode, lens_sel) + np.arange(n_q)
        res = oracle.online_prefill(k_store, v, row_start, ids, mode, q, k_q, v_q, q_pos, base, storage_rounding=False)
        # the textbook route: gather raw, rotate once at the final ids, attend
        gathered_k = np.concatenate([k_raw[row_start[c]:row_start[c + 1]] for c in ids] + [k_q])
        gathered_v = np.concatenate([v[row_start[c]:row_start[c + 1]] for c in ids] + [v_q])
        all_pos = np.concatenate([pos, q_pos])
        k_direct = oracle.rope(gathered_k, all_pos, base)
        want = sdpa(oracle.rope(q, q_pos, base), k_direct, gathered_v.astype(np.float64),
                    mask=prefix_mask(n_q, len(all_pos)))
        assert np.allclose(res["out"], want, atol=2e-6)     # the float32 rounding of the store: ~1e-7 relative
        assert np.array_equal(res["pos"], pos)


def test_offline_pipeline_store_feeds_online_pipeline():
    """The keys the offline step saves are R(local position) k (Sec. 3.4 step 2): chunk-by-chunk
    attention of the offline oracle equals prefix attention over that chunk alone."""
    lens = (5, 8)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, H, Hkv, d, base = int(cu[-1]), 4, 2, 8, 1e4
    q = RNG.standard_normal((T, H, d)).astype(np.float32)
    k = RNG.standard_normal((T, Hkv, d)).astype(np.float32)
    v = RNG.standard_normal((T, Hkv, d)).astype(np.float32)
    res = oracle.offline_chunk_prefill(q, k, v, cu, base, storage_rounding=False)
    for c in range(2):
        s, e = cu[c], cu[c + 1]
        pos = np.arange(e - s)
        want = sdpa(oracle.rope(q[s:e], pos, base), oracle.rope(k[s:e], pos, base), v[s:e].astype(np.float64), causal=True)
        assert np.allclose(res["out"][s:e], want, atol=1e-12)
        assert np.allclose(res["k_rot"][s:e], oracle.rope(k[s:e], pos, base), atol=0)


def test_flop_accounting_reproduces_table4():
    # Appendix C with Qwen2-7B's shape; Table 4's TFLOPs column is the pin (tests/golden/table4_tflops.txt)
    rows = {}
    for line in open(__file__.rsplit("/", 1)[0] + "/golden/table4_tflops.txt"):
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        rows[parts[0]] = [float(x) for x in parts[1:]]
    shape = dict(layer_num=28, head_num=28, kv_head_num=4, head_size=128, hidden_size=3584, intermediate_size=18944)
    n_ctx, n_query = 8192, 128
    n_total = n_ctx + n_query
    per_tok = accounting.model_flops_per_token(n_total, **shape)
    for b in (1, 2, 4, 6, 8):
        naive = b * n_total * per_tok / 1e12
        turbo = b * n_query * per_tok / 1e12
        assert round(naive, 2) == pytest.approx(rows[str(b)][0], abs=0.011)
        assert round(turbo, 2) == pytest.approx(rows[str(b)][1], abs=0.011)
    assert round(100 * (1 - n_query / n_total), 2) == rows["reduction_percent"][0]
    # the attention term alone is what this repository counts per visible pair
    assert accounting.attn_flops(28, 128, accounting.visible_pairs_prefix(1, n_total)) == 4 * 28 * 128 * n_total
    assert accounting.visible_pairs_prefix(16, 144) == 16 * 128 + 16 * 17 // 2
    assert accounting.visible_pairs_blockdiag([512] * 64) == 64 * 512 * 513 // 2

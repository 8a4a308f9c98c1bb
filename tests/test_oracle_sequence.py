"""Pins for the oracle's one-pass attention over a packed sequence with a per-token visible range, and for the plan
that builds the ranges and position ids of [chunk_1 .. chunk_k, query/answer] (Sec. 3.2, Sec. 3.3: fine-tuning
runs with the masks and position ids of inference).  Routes to the same numbers: brute force with an explicit
mask matrix, the two special cases the other oracle functions cover, the literal id vectors of Sec. 3.2, and the
statement that the one pass equals the offline pass over the documents plus the online pass of the query."""
import numpy as np
import pytest

import oracle
from tests.test_oracle_attention import brute_force

RNG = np.random.default_rng(41)


def range_mask(lo):
    T = len(lo)
    return np.array([[lo[i] <= j <= i for j in range(T)] for i in range(T)])


@pytest.mark.parametrize("lens,tail,H,Hkv,d", [((3, 1, 4), 2, 2, 1, 4), ((2, 5), 3, 4, 2, 6), ((), 5, 2, 2, 4), ((4,), 0, 3, 1, 8)])
def test_one_pass_attention_brute_force(lens, tail, H, Hkv, d):
    lo, _ = oracle.sequence_plan(lens, tail, oracle.POS_COMPOSITE)
    T = lo.size
    q = RNG.standard_normal((T, H, d)); k = RNG.standard_normal((T, Hkv, d)); v = RNG.standard_normal((T, Hkv, d))
    want = brute_force(q, k, v, range_mask(lo))
    assert np.allclose(oracle.attn_rows(q, k, v, lo), want, atol=1e-13)
    rows = np.array([T - 1, 0], np.int32)
    assert np.allclose(oracle.attn_rows(q, k, v, lo, rows), want[rows], atol=1e-13)


def test_special_cases_reduce_to_the_other_oracle_functions():
    H, Hkv, d = 6, 2, 8
    lens = (5, 9, 1, 7)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    q = RNG.standard_normal((T, H, d)); k = RNG.standard_normal((T, Hkv, d)); v = RNG.standard_normal((T, Hkv, d))
    # every token sees everything before it: plain causal attention = the prefix form with n_q = kv_len
    assert np.array_equal(oracle.attn_rows(q, k, v, np.zeros(T, np.int32)), oracle.attn_prefix(q, k, v))
    # every token sees its own chunk: the block-diagonal form
    lo, _ = oracle.sequence_plan(lens, 0, oracle.POS_COMPOSITE)
    assert np.array_equal(oracle.attn_rows(q, k, v, lo), oracle.attn_blockdiag(q, k, v, cu))


def test_sequence_plan_literal_vectors():
    """Sec. 3.2 with the off-by-one of the printed ranges fixed: composite ids restart in every chunk, reordered ids
    run on; the tail follows the longest chunk (composite) or the documents (reordered)."""
    lo, pos = oracle.sequence_plan((3, 2), 2, oracle.POS_COMPOSITE)
    assert lo.tolist() == [0, 0, 0, 3, 3, 0, 0]
    assert pos.tolist() == [0, 1, 2, 0, 1, 3, 4]
    lo, pos = oracle.sequence_plan((3, 2), 2, oracle.POS_REORDERED)
    assert lo.tolist() == [0, 0, 0, 3, 3, 0, 0]
    assert pos.tolist() == [0, 1, 2, 3, 4, 5, 6]
    lo, pos = oracle.sequence_plan((2, 2), 1, oracle.POS_COMPOSITE, tail_start=10)
    assert pos.tolist() == [0, 1, 0, 1, 10]
    # the document part agrees with the gather plan's position ids
    row_start = np.array([0, 3, 5], np.int64)
    for mode in (oracle.POS_COMPOSITE, oracle.POS_REORDERED):
        _, _, want = oracle.plan(row_start, np.array([0, 1], np.int32), mode)
        assert np.array_equal(oracle.sequence_plan((3, 2), 4, mode)[1][:5], want)


@pytest.mark.parametrize("mode", [oracle.POS_COMPOSITE, oracle.POS_REORDERED])
def test_one_pass_equals_offline_documents_plus_online_query(mode):
    """The training-time pass over [documents, query] gives, on the document tokens, what the offline chunk prefill
    gives (composite ids; under reordered ids the chunk-local result again, by the relative-position property), and on
    the query tokens what the online prefill over the assembled cache gives."""
    H, Hkv, d, base = 4, 2, 16, 1e4
    lens, n_q = (6, 3, 8), 5
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n_doc = int(cu[-1])
    T = n_doc + n_q
    q = RNG.standard_normal((T, H, d)).astype(np.float32)
    k = RNG.standard_normal((T, Hkv, d)).astype(np.float32)
    v = RNG.standard_normal((T, Hkv, d)).astype(np.float32)
    lo, pos = oracle.sequence_plan(lens, n_q, mode)
    one = oracle.masked_prefill(q, k, v, lo, pos, base, storage_rounding=False)["out"]
    off = oracle.offline_chunk_prefill(q[:n_doc], k[:n_doc], v[:n_doc], cu, base, storage_rounding=False)
    assert np.allclose(one[:n_doc], off["out"], atol=1e-12)
    # online: the store holds the offline keys (chunk-local rotation, here rounded to float32), the request takes all
    # chunks in order
    k_store = oracle.round_to(off["k_rot"], oracle.F32)
    on = oracle.online_prefill(k_store, v[:n_doc], cu.astype(np.int64), np.arange(len(lens), dtype=np.int32), mode,
                               q[n_doc:], k[n_doc:], v[n_doc:], pos[n_doc:], base, storage_rounding=False)
    assert np.allclose(one[n_doc:], on["out"], atol=2e-6)     # the float32 rounding of the store: ~1e-7 relative


def test_zero_queries_average_the_visible_values():
    lens, tail = (4, 2), 3
    lo, _ = oracle.sequence_plan(lens, tail, oracle.POS_REORDERED)
    T = lo.size
    v = RNG.standard_normal((T, 1, 4)); k = RNG.standard_normal((T, 1, 4))
    out = oracle.attn_rows(np.zeros((T, 2, 4)), k, v, lo)
    for t in range(T):
        assert np.allclose(out[t, 0], v[lo[t]:t + 1, 0].mean(0), atol=1e-14)

"""GPU parity where the softmax has to work for its result: logits that climb, fall and jump by tens of log2 units.

With N(0,1) inputs every scaled score stays within about six log2 units of zero, so a kernel that keeps its running
softmax relative to a lazily moved reference never moves it, a merge of key splits never sees statistics that differ,
and none of that arithmetic is compared with the oracle.  Eq. 2 / Eq. 4 with the softmax of Sec. 3.1 are exact for
any logits, so here the logits are put where they hurt:

* queries and keys carry a bias in the LAST RoPE pair (the slowest frequency: it turns by less than 0.01 rad over
  these contexts), query bias A, key bias b_j, so that key j sits at level_j = A b_j log2(e)/sqrt(d) log2 units for
  every query; the other channels stay N(0,1) (about +-6 log2 units of noise), and V stays N(0,1), so outputs are
  O(1) and the 2e-2 bound binds;
* the level patterns are chosen so that, whatever 64-key tiling and whatever cut into pieces of >= 256 keys a kernel
  uses, a tile maximum exceeds everything seen before by more than 16 log2 units several times (a rescale of the
  accumulators), a walk starts more than 40 below zero (the reference has to come down before anything underflows),
  pieces end with maxima more than 32 apart (the merge), and - for the kernels whose key range may start in the
  middle of a 64-key step - a row's first visible keys fall into one half of the step only and everything after
  them lies more than 40 lower.

Each test first checks on the fp64 logits (a few rows, one head) that its input really does this, then compares every
output element with the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_07590_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

A_BIAS = 16.0
LOG2E = 1.4426950408889634


@pytest.fixture(scope="module")
def B():
    from paper_2410_07590_amd import binding
    binding.lib()
    return binding


# ---- level patterns over the key index j of a request (or of a chunk) ------------------------------------------
def staircase_up(j):      # starts 60 below zero and climbs 24 every 96 keys
    return -60.0 + 24.0 * (j // 96)


def staircase_down(j):    # the first keys dominate everything that follows
    return 100.0 - 24.0 * (j // 96)


def deep_flat(j):         # everything 200 below the initial reference: exp2 of it is zero in fp32
    return -200.0 + 0.0 * j


BLOCKS = np.array([0.0, -45.0, 40.0, -90.0, 85.0, -20.0])


def blocks(j):            # jumps up and down by 45 .. 175 every 160 keys
    return BLOCKS[(j // 160) % BLOCKS.size]


WAVE_LEVEL = np.array([-80.0, 0.0, -40.0, 45.0])


def wave_slabs(j):        # 32-key slabs of a 128-key step at different levels, climbing 24 per step
    return WAVE_LEVEL[(j % 128) // 32] + 24.0 * (j // 128)


PATTERNS = {"staircase_up": staircase_up, "staircase_down": staircase_down, "deep_flat": deep_flat, "blocks": blocks}


def _bias_of(levels, d):
    return np.asarray(levels, np.float64) * np.sqrt(d) / (A_BIAS * LOG2E)


def _biased(rng, rows, heads, d, bias, dtype=torch.bfloat16):
    """N(0,1) rows whose last interleaved RoPE pair (channels d-2, d-1) holds (bias[row], 0); one rounding to storage."""
    t = torch.from_numpy(rng.standard_normal((rows, heads, d), dtype=np.float32))
    b = torch.as_tensor(np.broadcast_to(np.asarray(bias, np.float32), (rows,)).copy())
    t[:, :, d - 2] = b[:, None]
    t[:, :, d - 1] = 0.0
    return t.to(dtype)


def _logits2(q_rot, k_rot, h, g, rows):
    """log2-domain scores of query head h for the listed rows against every key: [len(rows), n_keys]."""
    d = q_rot.shape[-1]
    return (q_rot[rows, h] @ k_rot[:, h // g].T) * (LOG2E / np.sqrt(d))


def _walk(s_row, start, stop, tile=64):
    """The lazy reference over the keys [start, stop) in tiles of `tile` from `start`, with margins twice the kernel's
    own: returns (rescales, came_down, m) - tiles whose maximum exceeds zero and every earlier tile by more than 16,
    whether the first tile lies more than 40 below zero, and the maximum of the walk."""
    seen, grow, down = None, 0, False
    for t0 in range(start, stop, tile):
        mx = float(s_row[t0:min(t0 + tile, stop)].max())
        if seen is None:
            down = mx < -40.0
            grow += mx > 16.0
            seen = mx
        else:
            bound = seen if down else max(seen, 0.0)
            grow += mx > bound + 16.0
            seen = max(seen, mx)
    return grow, down, seen


def _every_cut_moves_the_reference(s_row, n_vis, want_grow, want_down, tile=64, piece=256, first=0):
    """Whatever aligned piece of `piece` keys from key `first` on a kernel walks, it meets the events asked for."""
    for start in range(first, max(n_vis - piece, 0) + 1, tile):
        grow, down, _ = _walk(s_row, start, min(start + piece, n_vis), tile)
        assert grow >= want_grow, "keys %d..%d: %d rescales" % (start, start + piece, grow)
        assert down or not want_down, "keys %d..: the walk does not start below the reference" % start


def _request(rng, sh, lens, n_q, level_fn, mode):
    """A store whose chunks are the request's chunks in order, so that store row == cache row."""
    d = sh.head_dim
    row_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    n_doc = int(row_start[-1])
    j = np.arange(n_doc + n_q)
    b = _bias_of(level_fn(j), d)
    store = synth.Store(_biased(rng, n_doc, sh.n_kv_heads, d, b[:n_doc]), synth.normal_tensor(rng, (n_doc, sh.n_kv_heads, d), sh.torch_dtype), row_start)
    ids = np.arange(len(lens), dtype=np.int32)
    q_pos = (synth.query_start(mode, list(lens)) + np.arange(n_q)).astype(np.int32)
    req = synth.Request(ids, mode, n_q, _biased(rng, n_q, sh.n_q_heads, d, A_BIAS), _biased(rng, n_q, sh.n_kv_heads, d, b[n_doc:]),
                        synth.normal_tensor(rng, (n_q, sh.n_kv_heads, d), sh.torch_dtype), q_pos, n_doc, list(lens))
    return store, req


def _request_logits(sh, store, req, rows, h=1):
    o = H.run_request_oracle(sh, store, req, rows=np.zeros(1, np.int32))
    q_rot = oracle.rope(H.bits(req.q), req.q_pos, sh.rope_base, sh.rope_layout)
    return _logits2(q_rot, o["k_cache"], h, sh.group, rows)


def _rel_check(got, want, what):
    err = float(np.abs(got - want).max())
    scale = float(np.abs(want).max())
    assert scale > 0.05, "%s: outputs of magnitude %.3f do not make the tolerance bind" % (what, scale)
    assert err <= H.BF16_TOL and err <= H.BF16_TOL * scale, "%s: max abs err %.3e (outputs up to %.3f)" % (what, err, scale)
    return err


# ---- prefill over the assembled cache (split keys + merge) and the gathering attention -------------------------------
@pytest.mark.parametrize("pattern", sorted(PATTERNS))
@pytest.mark.parametrize("shape_no", [0, 1])
def test_prefill_and_gather_with_moving_logits(B, pattern, shape_no):
    sh = (synth.LLAMA3_8B, synth.QWEN2_7B)[shape_no]
    rng = np.random.Generator(np.random.PCG64([4242, shape_no, sorted(PATTERNS).index(pattern)]))
    lens, n_q = (300, 290, 310, 300, 280, 320), 70
    mode = synth.POS_REORDERED if shape_no == 0 else synth.POS_COMPOSITE
    store, req = _request(rng, sh, lens, n_q, PATTERNS[pattern], mode)
    # what the input does, on the fp64 logits of three query tokens
    rows = np.array([0, 33, n_q - 1])
    s = _request_logits(sh, store, req, rows)
    n_doc = req.n_doc
    for r, i in enumerate(rows):
        n_vis = n_doc + int(i) + 1
        if pattern == "staircase_up":
            # pieces that begin behind the climb through zero (keys 0 .. 383 lie within 40 of the initial reference)
            _every_cut_moves_the_reference(s[r], n_vis, want_grow=1, want_down=False, first=384)
            assert _walk(s[r], 0, n_vis)[0] >= 10 and _walk(s[r], 0, n_vis)[1]      # one long walk: comes down once, then climbs
        elif pattern == "deep_flat":
            _every_cut_moves_the_reference(s[r], n_vis, want_grow=0, want_down=True)
        elif pattern == "blocks":
            ms = [_walk(s[r], a, min(a + 256, n_vis))[2] for a in range(0, n_vis - 255, 64)]
            assert max(ms) - min(ms) > 32.0                                           # pieces to merge lie far apart
            assert _walk(s[r], 0, n_vis)[0] >= 2
        else:
            assert _walk(s[r], 0, n_vis)[0] == 1 and s[r, :96].max() > s[r, 96:n_vis].max() + 10.0
    sd = B.Store(H.gpu_shape(B, sh), store.k.cuda(), store.v.cuda(), store.row_start)
    kv_len = n_doc + n_q
    assert B.tr_prefill_attn_workspace_size(sd.shape, n_q, kv_len) > 0        # the keys are split: the merge runs
    g = H.run_request_gpu(B, sh, sd, req)
    o = H.run_request_oracle(sh, store, req)
    H.assert_same_bits(H.bits(g["cache_k"])[:kv_len], o["k_cache_st"], "assembled K", 1e-5)
    err = _rel_check(H.to_f64(g["out"]), o["out"], "prefill attention, " + pattern)
    err_g = _rel_check(H.to_f64(H.run_request_gather_gpu(B, sh, sd, req)), o["out"], "gather attention, " + pattern)
    print("%s %s: prefill %.3e, gather %.3e" % (pattern, sh, err, err_g))


def test_logits_beyond_the_exponent_range(B):
    """The first chunk 1100 log2 units below zero and every other key 1100 above (exp of such a score, or of its distance
    from the first score, overflows even in fp64): only a softmax taken relative to the row maximum, as Sec. 3.1's
    definition allows, gives a finite result.  Prefill with split keys, gather, decode."""
    sh = synth.LLAMA3_8B
    rng = np.random.Generator(np.random.PCG64(4248))
    store, req = _request(rng, sh, (200, 330, 150), 37, lambda j: np.where(j < 200, -1100.0, 1100.0), synth.POS_REORDERED)
    s = _request_logits(sh, store, req, np.array([0, 36]))
    assert s[:, :200].max() < -1050.0 and s[:, 200:req.n_doc + 1].min() > 1050.0
    sd = B.Store(H.gpu_shape(B, sh), store.k.cuda(), store.v.cuda(), store.row_start)
    o = H.run_request_oracle(sh, store, req)
    g = H.run_request_gpu(B, sh, sd, req)
    err = _rel_check(H.to_f64(g["out"]), o["out"], "prefill, logits near 1100")
    err_g = _rel_check(H.to_f64(H.run_request_gather_gpu(B, sh, sd, req)), o["out"], "gather, logits near 1100")
    gs = H.gpu_shape(B, sh)
    kv = np.array([0, g["kv_len"]], np.int64)
    dec = torch.full((1, sh.n_q_heads, sh.head_dim), float("nan"), dtype=sh.torch_dtype, device="cuda")
    B.tr_decode_attn(gs, req.q[-1:].cuda(), g["cache_k"].cuda(), g["cache_v"].cuda(), torch.from_numpy(req.q_pos[-1:]).cuda(), kv, dec,
                     B.workspace(B.tr_decode_attn_workspace_size(gs, kv)))
    torch.cuda.synchronize()
    err_d = _rel_check(H.to_f64(dec), o["out"][-1:], "decode, logits near 1100")
    print("logits near 1100: prefill %.3e, gather %.3e, decode %.3e" % (err, err_g, err_d))


def test_batched_prefill_with_moving_logits(B):
    """Four requests of different lengths and patterns in one launch (the planner cuts each into its own pieces)."""
    sh = synth.QWEN2_7B
    rng = np.random.Generator(np.random.PCG64(4243))
    names = sorted(PATTERNS)
    cases = [_request(rng, sh, lens, n_q, PATTERNS[names[i]], i % 2)
             for i, (lens, n_q) in enumerate([((500, 400), 40), ((300,) * 5, 100), ((700, 200, 350), 33), ((260, 250), 128)])]
    k = torch.cat([c[0].k for c in cases])
    v = torch.cat([c[0].v for c in cases])
    row_start = np.concatenate([[0], np.cumsum(np.concatenate([np.diff(c[0].row_start) for c in cases]))]).astype(np.int64)
    store = synth.Store(k, v, row_start)
    reqs, c0 = [], 0
    for st, r in cases:
        reqs.append(synth.Request(r.chunk_ids + c0, r.pos_mode, r.n_q, r.q, r.k_q, r.v_q, r.q_pos, r.n_doc, r.chunk_lens))
        c0 += st.n_chunks
    sd = B.Store(H.gpu_shape(B, sh), store.k.cuda(), store.v.cuda(), store.row_start)
    from tests.test_gpu_parity import _run_batched
    cfg = synth.scaled(synth.CONFIGS[3], shape=sh)
    ck, cv, out, crs, cu_q = _run_batched(B, cfg, store, sd, reqs)
    for r, req in enumerate(reqs):
        o = H.run_request_oracle(sh, store, req)
        H.assert_same_bits(H.bits(ck[int(crs[r]):int(crs[r + 1])]), o["k_cache_st"], "request %d K" % r, 1e-5)
        print("batched request %d (%s): %.3e" % (r, names[r], _rel_check(H.to_f64(out[cu_q[r]:cu_q[r + 1]]), o["out"], "batched request %d" % r)))


# ---- decode: four waves share the rows and own 32-key slabs of every 128-key step ---------------------------------
@pytest.mark.parametrize("shape_no", [0, 1])
def test_decode_slabs_at_different_levels(B, shape_no):
    """Slab w of every 128-key step sits at its own level (-80, 0, -40, +45) and all climb 24 per step: every wave
    rescales at every step, wave 0 starts below the reference, and the four partial results the workgroup merges have
    maxima 35 .. 125 apart; long caches are also cut into pieces whose maxima differ by the climb."""
    sh = (synth.QWEN2_7B, synth.LLAMA3_8B)[shape_no]
    rng = np.random.Generator(np.random.PCG64([4244, shape_no]))
    cases = [_request(rng, sh, lens, 1, wave_slabs, synth.POS_REORDERED) for lens in [(640, 640, 700), (128,), (200, 300), (1500, 1100)]]
    for st, r in cases:
        s = _request_logits(sh, st, r, np.array([0]))[0]
        n_vis = r.n_doc + 1
        ms = []
        for w in range(4):
            slab = np.concatenate([s[a + 32 * w:a + 32 * w + 32] for a in range(0, n_vis, 128)])
            ms.append(float(slab.max()))
        assert max(ms) - min(ms) > 32.0 or n_vis <= 129
        if n_vis > 300:
            steps = [float(s[a:a + 32].max()) for a in range(0, n_vis - 31, 128)]
            assert all(b > a + 16.0 for a, b in zip(steps, steps[1:])) and steps[0] < -40.0
    k = torch.cat([c[0].k for c in cases])
    v = torch.cat([c[0].v for c in cases])
    row_start = np.concatenate([[0], np.cumsum(np.concatenate([np.diff(c[0].row_start) for c in cases]))]).astype(np.int64)
    store = synth.Store(k, v, row_start)
    reqs, c0 = [], 0
    for st, r in cases:
        reqs.append(synth.Request(r.chunk_ids + c0, r.pos_mode, 1, r.q, r.k_q, r.v_q, r.q_pos, r.n_doc, r.chunk_lens))
        c0 += st.n_chunks
    sd = B.Store(H.gpu_shape(B, sh), store.k.cuda(), store.v.cuda(), store.row_start)
    from tests.test_gpu_parity import _run_batched
    cfg = synth.scaled(synth.CONFIGS[3], shape=sh)
    crs = np.concatenate([[0], np.cumsum([r.n_doc + 1 for r in reqs])]).astype(np.int64)
    assert B.tr_decode_attn_workspace_size(sd.shape, crs) > 0            # some cache is cut into pieces
    ck, cv, out, crs, cu_q = _run_batched(B, cfg, store, sd, reqs, decode=True)
    for r, req in enumerate(reqs):
        o = H.run_request_oracle(sh, store, req)
        print("decode request %d: %.3e" % (r, _rel_check(H.to_f64(out[r:r + 1]), o["out"], "decode request %d" % r)))


# ---- offline chunk prefill and the one-pass sequence: key ranges that start in the middle of a 64-key step -----------
def _packed(rng, sh, lens, level_of_local):
    """Packed chunks whose key at chunk-local index t sits at level_of_local(chunk, t)."""
    d = sh.head_dim
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    lev = np.concatenate([level_of_local(c, np.arange(l)) for c, l in enumerate(lens)]) if T else np.zeros(0)
    return synth.PackedChunks(_biased(rng, T, sh.n_q_heads, d, A_BIAS), _biased(rng, T, sh.n_kv_heads, d, _bias_of(lev, d)),
                              synth.normal_tensor(rng, (T, sh.n_kv_heads, d), sh.torch_dtype), cu)


def _offline_both_ways(B, sh, pc, what):
    from tests.test_gpu_parity import _run_offline, _run_sequence
    o = oracle.offline_chunk_prefill(H.bits(pc.q), H.bits(pc.k), H.bits(pc.v), pc.cu, sh.rope_base, layout=sh.rope_layout)
    out, k_rot = _run_offline(B, sh, pc)
    H.assert_same_bits(H.bits(k_rot), o["k_rot_st"], "rotated keys K'", 1e-5)
    err = _rel_check(H.to_f64(out), o["out"], what + ", offline entry point")
    seg, pos = B.tr_sequence_plan(np.diff(pc.cu), 0, synth.POS_COMPOSITE)
    out_s, _ = _run_sequence(B, sh, pc.q, pc.k, pc.v, seg, pos)
    err_s = _rel_check(H.to_f64(out_s), o["out"], what + ", one-pass entry point")
    return err, err_s, o


def test_first_visible_keys_in_one_half_of_a_key_step(B):
    """Chunks of 10, 60 and 40 tokens at a GQA group of 4 (32 tokens per 128-row tile): the row tile of tokens 64..95
    walks its keys in 64-key steps from row 10 (the start of the second chunk), so tokens 74..95 of the third chunk
    (rows 70..109) meet in the first step only keys 70..73 - offsets 60..63 of the step, the four keys one half of the
    wave holds - and their other keys, 74 and up, lie 60 log2 units lower.  The same with chunks of 7, 61 and 60."""
    sh = synth.LLAMA3_8B
    worst = 0.0
    for case, (lens, third_start, step_start) in enumerate([((10, 60, 40), 70, 10), ((7, 61, 60, 30), 68, 7)]):
        rng = np.random.Generator(np.random.PCG64([4245, case]))
        first = step_start + 64 - third_start          # keys of the third chunk inside the first 64-key step
        assert 1 <= first <= 4 and (third_start - step_start) % 64 >= 60
        pc = _packed(rng, sh, lens, lambda c, t: np.where(t < first, 0.0, -60.0) if c == 2 else 0.0 * t)
        lp = oracle.local_positions(pc.cu)
        q_rot = oracle.rope(H.bits(pc.q), lp, sh.rope_base)
        k_rot = oracle.rope(H.bits(pc.k), lp, sh.rope_base)
        rows = np.arange(third_start + first, min(96, int(pc.cu[3])))
        s = _logits2(q_rot, k_rot, 2, sh.group, rows)
        for r, t in enumerate(rows):     # the few first keys dominate everything else the token sees by far
            assert s[r, third_start:third_start + first].max() > s[r, third_start + first:t + 1].max() + 40.0
        err, err_s, _ = _offline_both_ways(B, sh, pc, "chunks %s" % (lens,))
        worst = max(worst, err, err_s)
    print("first keys in one half of a step: max abs err %.3e" % worst)


def test_gather_attention_after_a_first_chunk_of_a_few_rows(B):
    """The gathering attention walks chunk by chunk: after a first chunk of 1 .. 4 rows (one half of the wave holds
    them) the next chunks lie 60 log2 units lower."""
    sh = synth.LLAMA3_8B
    worst = 0.0
    for first in (1, 3, 4):
        rng = np.random.Generator(np.random.PCG64([4246, first]))
        store, req = _request(rng, sh, (first, 150, 90), 40, lambda j: np.where(j < first, 0.0, -60.0), synth.POS_REORDERED)
        s = _request_logits(sh, store, req, np.array([0, 39]))
        assert (s[:, :first].max(axis=1) > s[:, first:req.n_doc + 1].max(axis=1) + 40.0).all()
        sd = B.Store(H.gpu_shape(B, sh), store.k.cuda(), store.v.cuda(), store.row_start)
        o = H.run_request_oracle(sh, store, req)
        worst = max(worst, _rel_check(H.to_f64(H.run_request_gather_gpu(B, sh, sd, req)), o["out"], "gather, first chunk of %d rows" % first))
        worst = max(worst, _rel_check(H.to_f64(H.run_request_gpu(B, sh, sd, req)["out"]), o["out"], "prefill, first chunk of %d rows" % first))
    print("short first chunk: max abs err %.3e" % worst)


@pytest.mark.parametrize("pattern", sorted(PATTERNS))
def test_offline_and_one_pass_with_moving_logits(B, pattern):
    """Ragged chunks whose keys follow the level patterns chunk-locally, through tr_chunk_prefill_attn and through
    tr_sequence_prefill_attn; then the one-pass form with query tokens behind the documents, its long key ranges cut
    into pieces and merged."""
    sh = synth.LLAMA3_8B
    rng = np.random.Generator(np.random.PCG64([4247, sorted(PATTERNS).index(pattern)]))
    fn = PATTERNS[pattern]
    lens = (300, 10, 60, 40, 520, 5)
    pc = _packed(rng, sh, lens, lambda c, t: fn(t))
    err, err_s, _ = _offline_both_ways(B, sh, pc, pattern)
    # [chunks, tail]: the tail's keys and the documents' follow the pattern over the packed index
    from tests.test_gpu_parity import _run_sequence
    lens2, n_tail = (900, 850, 800), 90
    seg, pos = B.tr_sequence_plan(lens2, n_tail, synth.POS_REORDERED)
    T, d = seg.size, sh.head_dim
    q = _biased(rng, T, sh.n_q_heads, d, A_BIAS)
    k = _biased(rng, T, sh.n_kv_heads, d, _bias_of(fn(np.arange(T)), d))
    v = synth.normal_tensor(rng, (T, sh.n_kv_heads, d), sh.torch_dtype)
    assert B.tr_sequence_prefill_attn_workspace_size(H.gpu_shape(B, sh), seg, T) > 0      # the tail's key range is cut
    out, k_rot = _run_sequence(B, sh, q, k, v, seg, pos)
    rows = np.unique(np.concatenate([np.arange(0, T, 41), np.arange(T - n_tail, T)])).astype(np.int32)
    o = oracle.masked_prefill(H.bits(q), H.bits(k), H.bits(v), seg, pos, sh.rope_base, rows=rows)
    H.assert_same_bits(H.bits(k_rot), o["k_rot_st"], "keys rotated at their position ids", 1e-5)
    err_t = _rel_check(H.to_f64(out)[rows], o["out"], pattern + ", one pass with a tail")
    print("%s: offline %.3e, one pass %.3e, one pass with a tail %.3e" % (pattern, err, err_s, err_t))

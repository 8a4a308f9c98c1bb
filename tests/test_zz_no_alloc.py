"""The prefill entry point for callers that cannot allocate device memory (tr_prefill_attn_static: the split-KV partial
results live in a static device array inside the library) against tr_prefill_attn with a caller's workspace: same bits,
on two calls in a row, the second with a smaller input; sizes beyond the array are refused before anything is enqueued."""
import numpy as np
import pytest
import torch

from paper_2410_07590_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2410_07590_amd import binding
    binding.lib()
    return binding


def _inputs(sh, kv_len, n_q, seed):
    rng = np.random.Generator(np.random.PCG64([808, seed]))
    k = synth.normal_tensor(rng, (kv_len, sh.n_kv_heads, sh.head_dim), sh.torch_dtype).cuda()
    v = synth.normal_tensor(rng, (kv_len, sh.n_kv_heads, sh.head_dim), sh.torch_dtype).cuda()
    q = synth.normal_tensor(rng, (n_q, sh.n_q_heads, sh.head_dim), sh.torch_dtype).cuda()
    q_pos = torch.arange(kv_len - n_q, kv_len, dtype=torch.int32, device="cuda")
    return q, k, v, q_pos


def test_static_scratch_entry_point_matches_the_workspace_one(B):
    sh = synth.QWEN2_7B
    gs = H.gpu_shape(B, sh)
    assert B.tr_prefill_attn_static_scratch_bytes() == 32 << 20
    # the first call fills a large part of the array, the second, smaller one must not be disturbed by what it left
    for seed, (kv_len, n_q) in enumerate([(4160, 64), (900, 19), (4160, 64), (300, 1)]):
        q, k, v, q_pos = _inputs(sh, kv_len, n_q, seed)
        need = B.tr_prefill_attn_workspace_size(gs, n_q, kv_len)
        assert 0 < need <= B.tr_prefill_attn_static_scratch_bytes()      # these shapes do split their keys
        want = torch.full((n_q, sh.n_q_heads, sh.head_dim), float("nan"), dtype=sh.torch_dtype, device="cuda")
        got = torch.full_like(want, float("nan"))
        B.tr_prefill_attn(gs, q, k, v, q_pos, kv_len, want, B.workspace(need))
        B.tr_prefill_attn_static(gs, q, k, v, q_pos, kv_len, got)
        torch.cuda.synchronize()
        assert not torch.isnan(got.float()).any()
        assert np.array_equal(H.bits(got.cpu()), H.bits(want.cpu())), "kv_len %d, n_q %d" % (kv_len, n_q)


def test_static_scratch_entry_point_refuses_what_does_not_fit(B):
    sh = synth.LLAMA3_8B
    gs = H.gpu_shape(B, sh)
    # the default policy aims at one workgroup per CU, which keeps any single request at these head counts below the
    # array's size; aiming at four per CU cuts 1024 query tokens over 70000 rows into 8 pieces: 66 MiB of partials
    kv_len, n_q = 70000, 1024
    B.tr_set_tuning("target_items", 1024)
    try:
        _refused(B, gs, sh, kv_len, n_q)
    finally:
        B.tr_set_tuning("target_items", 0)


def _refused(B, gs, sh, kv_len, n_q):
    need = B.tr_prefill_attn_workspace_size(gs, n_q, kv_len)
    assert need > B.tr_prefill_attn_static_scratch_bytes()
    q = torch.zeros((n_q, sh.n_q_heads, sh.head_dim), dtype=sh.torch_dtype, device="cuda")
    k = torch.zeros((kv_len, sh.n_kv_heads, sh.head_dim), dtype=sh.torch_dtype, device="cuda")
    out = torch.full_like(q, float("nan"))
    with pytest.raises(B.TurboRagError) as e:
        B.tr_prefill_attn_static(gs, q, k, k, torch.zeros(n_q, dtype=torch.int32, device="cuda"), kv_len, out)
    assert e.value.code == B.TR_ERR_WORKSPACE and "static" in str(e.value)
    torch.cuda.synchronize()
    assert torch.isnan(out.float()).all()        # nothing was enqueued

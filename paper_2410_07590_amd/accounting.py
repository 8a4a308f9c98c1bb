"""Algorithmic work of the hot path: flops and bytes per unit, for roofline figures.

Host-side bookkeeping only.  Attention is counted as 4 * n_q_heads * head_dim flops
per (query, key) pair that is visible under the mask (QK^T and PV, a multiply and an
add each).  That is the count the paper's Table 4 uses: its TFLOPs column is
reproduced digit for digit by Appendix C's per-token formula only when the attention
term is 4 * head_num * head_size * n_context (the printed term has a 2).
"""


def visible_pairs_prefix(n_q: int, kv_len: int) -> int:
    """Query token i sees kv_len - n_q + i + 1 keys."""
    n_doc = kv_len - n_q
    return n_q * n_doc + n_q * (n_q + 1) // 2


def visible_pairs_blockdiag(chunk_lens) -> int:
    return sum(int(l) * (int(l) + 1) // 2 for l in chunk_lens)


def attn_flops(n_q_heads: int, head_dim: int, pairs: int) -> int:
    return 4 * n_q_heads * head_dim * pairs


def assemble_bytes(n_doc: int, n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    """K and V, each read once from the store and written once to the cache."""
    return 4 * n_doc * n_kv_heads * head_dim * elem_bytes


def append_bytes(n_q: int, n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    return 4 * n_q * n_kv_heads * head_dim * elem_bytes


def prefill_attn_bytes(n_q: int, kv_len: int, n_q_heads: int, n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    """Cache K and V streamed once, Q read once, O written once."""
    return (2 * kv_len * n_kv_heads + 2 * n_q * n_q_heads) * head_dim * elem_bytes


def chunk_prefill_bytes(total_tokens: int, n_q_heads: int, n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    """Q, K, V read once; O and the rotated keys K' written once."""
    return total_tokens * (2 * n_q_heads + 3 * n_kv_heads) * head_dim * elem_bytes


def model_flops_per_token(n_context: int, layer_num: int, head_num: int, kv_head_num: int, head_size: int,
                          hidden_size: int, intermediate_size: int) -> int:
    """Appendix C's per-token cost with the attention term as Table 4 counts it."""
    c_qkv = 2 * hidden_size * (head_num + 2 * kv_head_num) * head_size
    c_attn = 4 * head_num * head_size * n_context
    c_o = 2 * hidden_size * hidden_size
    c_mlp = 2 * 3 * hidden_size * intermediate_size
    return layer_num * (c_qkv + c_attn + c_o + c_mlp)

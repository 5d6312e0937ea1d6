"""Work and traffic accounting for the attention path (host arithmetic only)."""


def kv_cache_bytes_per_token(batch, len_in, len_out, layers, n_head, s_head, s_dtype):
    """KV-cache bytes read to generate one token: the paper's Eq. (1), section 2.2.
    2 * b * (L_i + L_o) * l * n_head * s_head * s_d, the 2 being K and V."""
    return 2 * batch * (len_in + len_out) * layers * n_head * s_head * s_dtype


def prefill_flops(batch, q_heads, seq_len, head_dim, causal):
    """Multiply-add flops of QK^T and PV over the visible (query, key) pairs only:
    4 * B * Hq * D * pairs, pairs = S(S+1)/2 under the causal mask, S^2 otherwise."""
    pairs = seq_len * (seq_len + 1) // 2 if causal else seq_len * seq_len
    return 4 * batch * q_heads * head_dim * pairs


def prefill_bytes(batch, q_heads, kv_heads, seq_len, head_dim, kv_int8, out_f32):
    """Each operand once: Q (bf16), K and V (bf16, or int8 + one fp32 scale per token and
    head), O (bf16 or fp32)."""
    q = batch * q_heads * seq_len * head_dim * 2
    kv = 2 * batch * kv_heads * seq_len * (head_dim * (1 if kv_int8 else 2) + (4 if kv_int8 else 0))
    o = batch * q_heads * seq_len * head_dim * (4 if out_f32 else 2)
    return q + kv + o


def decode_bytes(batch, q_heads, kv_heads, kv_len, head_dim):
    """One decode step over the INT8 cache: Eq. (1) for one layer at s_d = 1, plus both
    fp32 scale tensors, plus the bf16 query and output rows."""
    codes = kv_cache_bytes_per_token(batch, kv_len, 0, 1, kv_heads, head_dim, 1)
    scales = 2 * batch * kv_heads * kv_len * 4
    q_and_o = 2 * batch * q_heads * head_dim * 2
    return codes + scales + q_and_o


def decode_flops(batch, q_heads, kv_len, head_dim):
    return 4 * batch * q_heads * kv_len * head_dim


def kv_quant_bytes(rows, head_dim):
    """bf16 in, int8 out, one fp32 scale per row."""
    return rows * (2 * head_dim + head_dim + 4)

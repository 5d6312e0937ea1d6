"""Pins for the attention oracle (CPU only).

The oracle (oracle/slim_oracle.c and the numpy forms in oracle/reference.py) is checked
against things that are not the oracle: a pure-Python brute force of
softmax(Q K^T * scale + mask) V, closed forms, and invariants that a dropped term, a
wrong sign or index, or a transposed operand would break.  Paper section 2.1 fixes the
computation (score row, softmax over the row, row times V) and states it is exact.
"""
import math

import numpy as np
import pytest

from paper_2407_07304_amd.inputs import f32_to_bf16_bits, bf16_bits_to_f32, normal_bf16


def _rand_bits(rng, shape):
    return normal_bf16(rng, shape)


def _f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def brute_force(q, k, v, scale, causal):
    """Pure-Python full-matrix attention on nested lists (floats are fp64)."""
    B, Hq, Sq, D = q.shape
    Hkv, Skv = k.shape[1], k.shape[2]
    G = Hq // Hkv
    out = np.zeros((B, Hq, Sq, D))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            S = [[scale * math.fsum(float(q[b, h, i, d]) * float(k[b, g, j, d]) for d in range(D))
                  for j in range(Skv)] for i in range(Sq)]
            for i in range(Sq):
                lim = i + (Skv - Sq) if causal else Skv - 1
                row = S[i][:lim + 1]
                mx = max(row)
                e = [math.exp(x - mx) for x in row]
                tot = math.fsum(e)
                for d in range(D):
                    out[b, h, i, d] = math.fsum(e[j] * float(v[b, g, j, d]) for j in range(lim + 1)) / tot
    return out


@pytest.mark.parametrize("B,Hq,Hkv,S,D", [(2, 4, 2, 1, 4), (2, 4, 2, 2, 4), (1, 4, 2, 7, 64), (1, 2, 1, 33, 8),
                                          (1, 3, 3, 19, 16)])
@pytest.mark.parametrize("causal", [True, False])
def test_c_oracle_matches_pure_python_brute_force(oracle, B, Hq, Hkv, S, D, causal):
    rng = np.random.default_rng(100 + S + D)
    q, k, v = (_rand_bits(rng, (B, Hq, S, D)), _rand_bits(rng, (B, Hkv, S, D)), _rand_bits(rng, (B, Hkv, S, D)))
    scale = 1.0 / math.sqrt(D)
    ref = brute_force(_f64(q), _f64(k), _f64(v), scale, causal)
    got = oracle.attn(q, k, v, scale, causal)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    got_np = oracle.attn_full_matrix_np(_f64(q), _f64(k), _f64(v), scale, causal)
    np.testing.assert_allclose(got_np, ref, rtol=0, atol=1e-12)


def test_closed_form_two_keys_is_a_sigmoid(oracle):
    # q=[1], k=[[0],[1]], v=[[0],[1]], scale 1: p = (1, e)/(1+e) so o = e/(1+e) = sigmoid(1).
    q = f32_to_bf16_bits(np.array([[[[1.0]]]], dtype=np.float32))
    k = f32_to_bf16_bits(np.array([[[[0.0], [1.0]]]], dtype=np.float32))
    v = k.copy()
    o = oracle.attn(q, k, v, 1.0, False)
    assert abs(o[0, 0, 0, 0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    # the scale multiplies the score: scale 3 -> sigmoid(3); a sign slip would give sigmoid(-3)
    o3 = oracle.attn(q, k, v, 3.0, False)
    assert abs(o3[0, 0, 0, 0] - 1.0 / (1.0 + math.exp(-3.0))) < 1e-15


def test_rows_of_p_sum_to_one_and_masked_keys_get_zero(oracle):
    rng = np.random.default_rng(7)
    B, Hq, Hkv, S, D = 1, 4, 2, 37, 16
    q, k, v = _rand_bits(rng, (B, Hq, S, D)), _rand_bits(rng, (B, Hkv, S, D)), _rand_bits(rng, (B, Hkv, S, D))
    for causal in (True, False):
        for i in (0, 1, 17, S - 1):
            p, o = oracle.attn_row_probs(q, k, v, 0.25, causal, 0, 3, i)
            assert abs(p.sum() - 1.0) < 1e-14
            assert (p >= 0).all()
            if causal:
                assert (p[i + 1:] == 0).all() and (p[:i + 1] > 0).all()
            # the output is the p-weighted mean of V
            np.testing.assert_allclose(o, p @ _f64(v)[0, 1], atol=1e-14)


def test_uniform_keys_return_mean_of_visible_values(oracle):
    rng = np.random.default_rng(8)
    B, Hq, Hkv, S, D = 2, 2, 2, 21, 8
    q, v = _rand_bits(rng, (B, Hq, S, D)), _rand_bits(rng, (B, Hkv, S, D))
    k = np.broadcast_to(_rand_bits(rng, (B, Hkv, 1, D)), (B, Hkv, S, D)).copy()
    vf = _f64(v)
    o = oracle.attn(q, k, v, 0.5, True)
    csum = np.cumsum(vf, axis=2) / np.arange(1, S + 1)[None, None, :, None]
    np.testing.assert_allclose(o, csum, atol=1e-13)
    o = oracle.attn(q, k, v, 0.5, False)
    np.testing.assert_allclose(o, np.broadcast_to(vf.mean(axis=2, keepdims=True), o.shape), atol=1e-13)


def test_causal_row_zero_returns_v0_exactly(oracle):
    rng = np.random.default_rng(9)
    q, k, v = _rand_bits(rng, (2, 4, 9, 16)), _rand_bits(rng, (2, 2, 9, 16)), _rand_bits(rng, (2, 2, 9, 16))
    o = oracle.attn(q, k, v, 0.25, True)
    vf = _f64(v)
    for h in range(4):
        assert np.array_equal(o[:, h, 0, :], vf[:, h // 2, 0, :])


def test_one_dominant_key_selects_its_value_row(oracle):
    rng = np.random.default_rng(10)
    S, D = 12, 8
    q = f32_to_bf16_bits(np.ones((1, 1, 1, D), dtype=np.float32))
    kf = rng.standard_normal((1, 1, S, D)).astype(np.float32)
    kf[0, 0, 5] = 1000.0  # q.k_5 = 8000 against |q.k_j| of a few units
    k, v = f32_to_bf16_bits(kf), _rand_bits(rng, (1, 1, S, D))
    o = oracle.attn(q, k, v, 1.0, False)
    np.testing.assert_allclose(o[0, 0, 0], _f64(v)[0, 0, 5], atol=1e-300)


def test_row_decomposition_equals_full_matrix_for_any_block(oracle):
    # Section 2.1: one horizontal score block at a time gives the full result exactly.
    rng = np.random.default_rng(11)
    B, Hq, Hkv, S, D = 1, 4, 2, 29, 16
    q, k, v = (_f64(_rand_bits(rng, (B, Hq, S, D))), _f64(_rand_bits(rng, (B, Hkv, S, D))),
               _f64(_rand_bits(rng, (B, Hkv, S, D))))
    for causal in (True, False):
        full = oracle.attn_full_matrix_np(q, k, v, 0.25, causal)
        for block in (1, 2, 5, 16, S, S + 3):
            slim = oracle.slim_attn_rowblocks_np(q, k, v, 0.25, causal, block)
            np.testing.assert_allclose(slim, full, rtol=0, atol=1e-13)


def test_c_oracle_equals_numpy_forms_at_a_mid_size(oracle):
    rng = np.random.default_rng(12)
    B, Hq, Hkv, S, D = 2, 4, 2, 130, 64
    qb, kb, vb = _rand_bits(rng, (B, Hq, S, D)), _rand_bits(rng, (B, Hkv, S, D)), _rand_bits(rng, (B, Hkv, S, D))
    for causal in (True, False):
        full = oracle.attn_full_matrix_np(_f64(qb), _f64(kb), _f64(vb), 0.125, causal)
        np.testing.assert_allclose(oracle.attn(qb, kb, vb, 0.125, causal), full, rtol=0, atol=1e-12)
    rows = np.array([0, 1, 63, 64, 129], dtype=np.int32)
    sub = oracle.attn(qb, kb, vb, 0.125, True, rows=rows)
    full = oracle.attn(qb, kb, vb, 0.125, True)
    assert np.array_equal(sub, full[:, :, rows, :])


def test_gqa_equals_mha_on_repeated_kv_heads(oracle):
    rng = np.random.default_rng(13)
    B, Hq, Hkv, S, D = 1, 8, 2, 17, 16
    q, k, v = _rand_bits(rng, (B, Hq, S, D)), _rand_bits(rng, (B, Hkv, S, D)), _rand_bits(rng, (B, Hkv, S, D))
    G = Hq // Hkv
    k_rep, v_rep = np.repeat(k, G, axis=1), np.repeat(v, G, axis=1)  # heads g,g,g,g,...: h -> h // G
    assert np.array_equal(oracle.attn(q, k, v, 0.25, True), oracle.attn(q, k_rep, v_rep, 0.25, True))
    # the mapping is blocked (consecutive query heads share a kv head), not interleaved
    k_tile = np.tile(k, (1, G, 1, 1))
    assert not np.array_equal(oracle.attn(q, k, v, 0.25, True), oracle.attn(q, k_tile, np.tile(v, (1, G, 1, 1)), 0.25, True))


def test_decode_equals_last_row_of_causal_prefill(oracle):
    rng = np.random.default_rng(14)
    B, Hq, Hkv, T, D = 2, 4, 2, 23, 16
    q, k, v = _rand_bits(rng, (B, Hq, T, D)), _rand_bits(rng, (B, Hkv, T, D)), _rand_bits(rng, (B, Hkv, T, D))
    pre = oracle.attn(q, k, v, 0.25, True)
    q_last = np.ascontiguousarray(q[:, :, T - 1:T, :])
    for causal in (True, False):  # one query at the last position: the flag changes nothing
        dec = oracle.attn(q_last, k, v, 0.25, causal)
        assert np.array_equal(dec[:, :, 0], pre[:, :, T - 1])


def test_shift_of_all_keys_leaves_output_unchanged(oracle):
    # k_j -> k_j + c moves every score of a row by q.c, which the softmax removes.
    rng = np.random.default_rng(15)
    B, H, S, D = 1, 2, 13, 8
    # small integers: k + c stays exactly representable in bf16
    q = f32_to_bf16_bits(rng.integers(-3, 4, (B, H, S, D)).astype(np.float32))
    kf = rng.integers(-3, 4, (B, H, S, D)).astype(np.float32)
    c = rng.integers(-2, 3, (1, 1, 1, D)).astype(np.float32)
    v = _rand_bits(rng, (B, H, S, D))
    a = oracle.attn(q, f32_to_bf16_bits(kf), v, 0.25, True)
    b = oracle.attn(q, f32_to_bf16_bits(kf + c), v, 0.25, True)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_permuting_keys_with_values_leaves_noncausal_output_unchanged(oracle):
    rng = np.random.default_rng(16)
    q, k, v = _rand_bits(rng, (1, 2, 5, 8)), _rand_bits(rng, (1, 2, 11, 8)), _rand_bits(rng, (1, 2, 11, 8))
    # Sq < Skv, non causal: every key visible to every row
    perm = rng.permutation(11)
    a = oracle.attn(q, k, v, 0.3, False)
    b = oracle.attn(q, np.ascontiguousarray(k[:, :, perm]), np.ascontiguousarray(v[:, :, perm]), 0.3, False)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)


def test_int8_kv_is_attention_on_dequantised_operands(oracle):
    # Section 2.2: the cached INT8 value is widened and multiplied by its token's scale.
    rng = np.random.default_rng(17)
    B, Hq, Hkv, S, D = 1, 4, 2, 9, 8
    q = _rand_bits(rng, (B, Hq, S, D))
    kc = rng.integers(-127, 128, (B, Hkv, S, D)).astype(np.int8)
    vc = rng.integers(-127, 128, (B, Hkv, S, D)).astype(np.int8)
    ks = rng.uniform(0.01, 0.05, (B, Hkv, S)).astype(np.float32)
    vs = rng.uniform(0.01, 0.05, (B, Hkv, S)).astype(np.float32)
    khat = kc.astype(np.float64) * ks.astype(np.float64)[..., None]
    vhat = vc.astype(np.float64) * vs.astype(np.float64)[..., None]
    assert np.array_equal(khat, oracle.dequant_np(kc, ks))
    for causal in (True, False):
        ref = brute_force(_f64(q), khat, vhat, 0.35, causal)
        got = oracle.attn(q, kc, vc, 0.35, causal, k_scale=ks, v_scale=vs)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    # scales are per token: moving a factor 2 from one key's scale into its codes changes nothing
    kc2, ks2 = kc.copy(), ks.copy()
    kc2[0, 0, 3] = np.clip(kc[0, 0, 3] // 2 * 2, -126, 126)
    kc_half = (kc2[0, 0, 3] // 2).astype(np.int8)
    a = oracle.attn(q, kc2, vc, 0.35, True, k_scale=ks2, v_scale=vs)
    kc3, ks3 = kc2.copy(), ks2.copy()
    kc3[0, 0, 3], ks3[0, 0, 3] = kc_half, np.float32(2.0) * ks2[0, 0, 3]
    b = oracle.attn(q, kc3, vc, 0.35, True, k_scale=ks3, v_scale=vs)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_int8_codes_with_unit_scale_equal_bf16_attention_on_the_integers(oracle):
    rng = np.random.default_rng(18)
    B, H, S, D = 1, 2, 10, 8
    q = _rand_bits(rng, (B, H, S, D))
    kc = rng.integers(-5, 6, (B, H, S, D)).astype(np.int8)
    vc = rng.integers(-5, 6, (B, H, S, D)).astype(np.int8)
    one = np.ones((B, H, S), dtype=np.float32)
    a = oracle.attn(q, kc, vc, 0.2, True, k_scale=one, v_scale=one)
    b = oracle.attn(q, f32_to_bf16_bits(kc.astype(np.float32)), f32_to_bf16_bits(vc.astype(np.float32)), 0.2, True)
    assert np.array_equal(a, b)


def test_eq1_kv_bytes_golden():
    # Paper Eq. (1), section 2.2; fixture rows are integer evaluations of the printed formula.
    import os
    from paper_2407_07304_amd.accounting import kv_cache_bytes_per_token
    path = os.path.join(os.path.dirname(__file__), "golden", "eq1_kv_bytes.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for b, li, lo, layers, nh, sh, sd, want in rows:
        assert kv_cache_bytes_per_token(int(b), int(li), int(lo), int(layers), int(nh), int(sh), int(sd)) == int(want)
    # the example's "approximately 128GB" is half of what the formula gives at 16 bit
    assert int(rows[0][-1]) == 2 * 128 * 2 ** 30

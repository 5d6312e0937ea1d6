"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element.

INT8 codes and scales must match bit for bit; attention outputs must stay within
max-abs 2e-2 and mean-abs 2e-3 of the fp64 oracle.
"""
import math

import numpy as np
import pytest
import torch

from paper_2407_07304_amd import inputs
from paper_2407_07304_amd.inputs import WORKLOADS, normal_bf16, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sa():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2407_07304_amd import slimattn
    slimattn.load()
    return slimattn


from _gpu_util import dev, dev_bf16, host_f64, check_close  # noqa: E402


# ---------------------------------------------------------------- quantiser

def _quant_both(sa, oracle, bits):
    codes, scales = sa.kv_quant_int8(dev_bf16(bits))
    torch.cuda.synchronize()
    want_c, want_s = oracle.kv_quant_int8(bits)
    got_c, got_s = codes.cpu().numpy(), scales.cpu().numpy()
    assert np.array_equal(got_s.view(np.uint32), want_s.view(np.uint32)), "scales differ"
    assert np.array_equal(got_c, want_c), "codes differ"


@pytest.mark.parametrize("shape", [(2, 3, 301, 128), (1, 2, 77, 64), (1, 1, 1, 128), (3, 5, 1000, 64)])
def test_kv_quant_bit_exact_normal(sa, oracle, shape):
    print("kv_quant", shape, flush=True)
    _quant_both(sa, oracle, normal_bf16(np.random.default_rng(31), shape))


def test_kv_quant_bit_exact_special_rows(sa, oracle):
    rng = np.random.default_rng(32)
    bits = normal_bf16(rng, (1, 4, 64, 128))
    bits[0, 0, 0] = 0                                                     # all-zero row
    bits[0, 0, 1] = rng.integers(0, 0x0080, 128).astype(np.uint16)        # bf16 subnormals
    bits[0, 0, 2] = rng.integers(0, 0x7f80, 128).astype(np.uint16)        # any magnitude
    halves = np.array([0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 126.5, -126.5, 127.0], dtype=np.float32)
    row = np.zeros(128, dtype=np.float32)
    row[:10] = halves
    bits[0, 0, 3] = f32_to_bf16_bits(row)                                 # exact ties at scale 1
    bits[0, 0, 4] = f32_to_bf16_bits(row / 1024)
    bits[0, 1] = f32_to_bf16_bits((rng.standard_normal((64, 128)) * 1e-30).astype(np.float32))
    bits[0, 2] = f32_to_bf16_bits((rng.standard_normal((64, 128)) * 1e30).astype(np.float32))
    print("kv_quant special rows", flush=True)
    _quant_both(sa, oracle, bits)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("shape", [(2, 3, 301, 128), (1, 2, 77, 64), (1, 1, 1, 128), (1, 32, 2048, 128), (4, 32, 3000, 128)])
def test_kv_quant_pair_gives_the_single_calls_bits(sa, oracle, shape):
    # K and V in one launch: each tensor's codes and scales are the oracle's (the last shape is past the size at
    # which the pair takes the streaming loads, the one before is C2's)
    print("kv_quant pair", shape, flush=True)
    rng = np.random.default_rng(34)
    kb, vb = normal_bf16(rng, shape), normal_bf16(rng, shape)
    vb[0, 0, 0] = 0                                                       # an all-zero row in the second tensor only
    kb[-1, -1, -1] = rng.integers(0, 0x0080, shape[-1]).astype(np.uint16) # subnormals in the first tensor's last row
    kc, ks, vc, vs = sa.kv_quant_int8_pair(dev_bf16(kb), dev_bf16(vb))
    torch.cuda.synchronize()
    for name, bits, codes, scales in (("K", kb, kc, ks), ("V", vb, vc, vs)):
        want_c, want_s = oracle.kv_quant_int8(bits)
        assert np.array_equal(scales.cpu().numpy().view(np.uint32), want_s.view(np.uint32)), name + " scales differ"
        assert np.array_equal(codes.cpu().numpy(), want_c), name + " codes differ"


@pytest.mark.timeout(600)
def test_kv_quant_bit_exact_c3_shape(sa, oracle):
    w = WORKLOADS["C3"]
    print("kv_quant C3 K tensor", flush=True)
    _quant_both(sa, oracle, normal_bf16(np.random.default_rng(w.seed), (w.batch, w.kv_heads, w.seq_len, w.head_dim)))


@pytest.mark.timeout(600)
@pytest.mark.parametrize("D", [128, 64])
def test_kv_quant_bit_exact_beyond_the_last_level_cache(sa, oracle, D):
    # an input of more than 256 MB takes the quantiser's streaming loads: same bits
    shape = (6, 32, 6000 * 128 // D, D)
    print("kv_quant", shape, flush=True)
    base = normal_bf16(np.random.default_rng(33), shape[1:])
    bits = np.stack([base ^ np.uint16(b * 0x8003 & 0xffff) for b in range(shape[0])])   # other signs and last mantissa bits
    assert bits.nbytes > (256 << 20)
    bits[1, 2, 100] = 0
    _quant_both(sa, oracle, bits)


# ---------------------------------------------------------------- prefill

def _prefill_case(sa, oracle, B, Hq, Hkv, S, D, causal, kv_int8, out_f32, seed, rows=None, two_sweep=False, strip=False):
    rng = np.random.default_rng(seed)
    q = normal_bf16(rng, (B, Hq, S, D))
    k = normal_bf16(rng, (B, Hkv, S, D))
    v = normal_bf16(rng, (B, Hkv, S, D))
    scale = 1.0 / math.sqrt(D)
    od = torch.float32 if out_f32 else torch.bfloat16
    if kv_int8:
        kc, ks = oracle.kv_quant_int8(k)
        vc, vs = oracle.kv_quant_int8(v)
        out = sa.slim_attn_prefill(dev_bf16(q), dev(kc), dev(vc), scale, causal, k_scale=dev(ks), v_scale=dev(vs),
                                   out_dtype=od)
        torch.cuda.synchronize()
        want = oracle.attn(q, kc, vc, scale, causal, k_scale=ks, v_scale=vs, rows=rows)
    else:
        fn = sa.slim_attn_prefill_two_sweep if two_sweep else (sa.slim_attn_prefill_strip if strip else sa.slim_attn_prefill)
        out = fn(dev_bf16(q), dev_bf16(k), dev_bf16(v), scale, causal, out_dtype=od)
        torch.cuda.synchronize()
        want = oracle.attn(q, k, v, scale, causal, rows=rows)
    got = host_f64(out)
    if rows is not None:
        got = got[:, :, rows, :]
    return check_close(got, want, "prefill B%d Hq%d Hkv%d S%d D%d causal%d int8%d" % (B, Hq, Hkv, S, D, causal, kv_int8))


SMALL = [
    # B, Hq, Hkv, S, D
    (1, 2, 2, 1, 128), (1, 2, 1, 5, 64), (2, 4, 2, 127, 128), (1, 2, 2, 128, 64), (1, 4, 1, 129, 128),
    (1, 2, 2, 200, 128), (2, 3, 3, 333, 64), (1, 8, 2, 640, 128), (1, 2, 2, 1000, 64),
    # two, three and nine row blocks: row-block pairs, a lone middle block, K/V tiles of the second block of a
    # pair requested while the first one finishes; 96 keys: fewer tiles than ring slots
    (1, 2, 2, 256, 128), (1, 2, 1, 384, 64), (1, 1, 1, 1152, 128), (1, 2, 2, 96, 128), (1, 1, 1, 1120, 64),
]


@pytest.mark.parametrize("B,Hq,Hkv,S,D", SMALL)
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("kv_int8", [False, True])
def test_prefill_small_shapes(sa, oracle, B, Hq, Hkv, S, D, causal, kv_int8):
    print("prefill", B, Hq, Hkv, S, D, causal, kv_int8, flush=True)
    _prefill_case(sa, oracle, B, Hq, Hkv, S, D, causal, kv_int8, out_f32=(S % 2 == 1), seed=40 + S)


def test_prefill_c1_full(sa, oracle):
    w = WORKLOADS["C1"]
    print("prefill C1 full tensor", flush=True)
    _prefill_case(sa, oracle, w.batch, w.q_heads, w.kv_heads, w.seq_len, w.head_dim, True, False, True, w.seed)


def test_prefill_causal_row0_is_v0(sa):
    rng = np.random.default_rng(45)
    q, k, v = normal_bf16(rng, (1, 4, 300, 128)), normal_bf16(rng, (1, 4, 300, 128)), normal_bf16(rng, (1, 4, 300, 128))
    out = sa.slim_attn_prefill(dev_bf16(q), dev_bf16(k), dev_bf16(v), 0.1, True)
    torch.cuda.synchronize()
    assert torch.equal(out[:, :, 0, :].cpu(), dev_bf16(v)[:, :, 0, :].cpu())


@pytest.mark.timeout(600)
def test_prefill_c2_full_size(sa, oracle):
    w = WORKLOADS["C2"]
    print("prefill C2, every row of every head", flush=True)
    _prefill_case(sa, oracle, w.batch, w.q_heads, w.kv_heads, w.seq_len, w.head_dim, True, False, False, w.seed)


@pytest.mark.timeout(900)
def test_prefill_c3_full_size(sa, oracle):
    w = WORKLOADS["C3"]
    print("prefill C3, every row of every head", flush=True)
    _prefill_case(sa, oracle, w.batch, w.q_heads, w.kv_heads, w.seq_len, w.head_dim, True, True, False, w.seed)


def _c5_rows_of_head(S, h, seed):
    """One row in every 128-row block, at a position inside the block that changes with the block and the head,
    plus the first and last rows and the rows around the first block boundaries."""
    rng = np.random.default_rng(seed * 1000 + h)
    n_rb = S // 128
    rows = 128 * np.arange(n_rb) + rng.integers(0, 128, n_rb)
    fixed = [0, 1, 31, 32, 127, 128, S - 129, S - 128, S - 1]
    return np.array(sorted(set(rows.tolist() + fixed)), dtype=np.int32)


@pytest.mark.timeout(1200)
def test_prefill_c5_full_size(sa, oracle):
    # The whole tensor is 17.6 TFLOP of oracle work, so the oracle takes a row sample, which the row decomposition
    # makes exact: for every query head one row out of each of the 256 row blocks (a different position inside the
    # block per block and per head) and the edge rows, about 140 GFLOP in all.  Everything else is checked for
    # being finite.
    w = WORKLOADS["C5"]
    S, D = w.seq_len, w.head_dim
    print("prefill C5 (one row per row block and head, every head)", flush=True)
    q, k, v = inputs.make_qkv(w)
    kc, ks = oracle.kv_quant_int8(k)
    vc, vs = oracle.kv_quant_int8(v)
    del k, v
    out = sa.slim_attn_prefill(dev_bf16(q), dev(kc), dev(vc), w.softmax_scale, True, k_scale=dev(ks), v_scale=dev(vs))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all()), "non-finite values in the C5 output"
    G = w.q_heads // w.kv_heads
    worst, total, count, blocks = 0.0, 0.0, 0, set()
    for h in range(w.q_heads):
        g = h // G
        rows = _c5_rows_of_head(S, h, w.seed)
        want = oracle.attn(q[:, h:h + 1], kc[:, g:g + 1], vc[:, g:g + 1], w.softmax_scale, True,
                           k_scale=ks[:, g:g + 1], v_scale=vs[:, g:g + 1], rows=rows)
        got = host_f64(out[:, h:h + 1, torch.from_numpy(rows).long().cuda()])
        err = np.abs(got - want)
        worst, total, count = max(worst, float(err.max())), total + float(err.sum()), count + err.size
        blocks |= set((rows // 128).tolist())
        if h % 8 == 7:
            print("  heads 0..%d: max-abs %.3e" % (h, worst), flush=True)
    assert len(blocks) == S // 128
    assert worst <= 2e-2 and total / count <= 2e-3, (worst, total / count)


# ---------------------------------------------------------------- decode

def _decode_case(sa, oracle, B, Hq, Hkv, T, D, seed):
    rng = np.random.default_rng(seed)
    q = normal_bf16(rng, (B, Hq, 1, D))
    k = normal_bf16(rng, (B, Hkv, T, D))
    v = normal_bf16(rng, (B, Hkv, T, D))
    kc, ks = oracle.kv_quant_int8(k)
    vc, vs = oracle.kv_quant_int8(v)
    del k, v
    scale = 1.0 / math.sqrt(D)
    dq, dkc, dks, dvc, dvs = dev_bf16(q), dev(kc), dev(ks), dev(vc), dev(vs)
    out = sa.slim_attn_decode_int8(dq, dkc, dks, dvc, dvs, scale)
    out2 = sa.slim_attn_decode_int8(dq, dkc, dks, dvc, dvs, scale, causal=True)
    torch.cuda.synchronize()
    assert torch.equal(out, out2), "decode must be deterministic and ignore the causal flag"
    want = oracle.attn(q, kc, vc, scale, False, k_scale=ks, v_scale=vs)
    return check_close(host_f64(out), want, "decode B%d Hq%d Hkv%d T%d D%d" % (B, Hq, Hkv, T, D))


@pytest.mark.parametrize("T", [1, 7, 255, 256, 257, 1000, 1024, 1025, 3000, 5121])
@pytest.mark.parametrize("D,Hq,Hkv", [(128, 4, 4), (64, 4, 2), (128, 8, 1)])
def test_decode_small_shapes(sa, oracle, T, D, Hq, Hkv):
    print("decode", T, D, Hq, Hkv, flush=True)
    _decode_case(sa, oracle, 2, Hq, Hkv, T, D, 50 + T)


@pytest.mark.timeout(600)
def test_decode_c4_full_size(sa, oracle):
    w = WORKLOADS["C4"]
    print("decode C4 full tensor", flush=True)
    _decode_case(sa, oracle, w.batch, w.q_heads, w.kv_heads, w.seq_len, w.head_dim, w.seed)


def test_decode_equals_last_prefill_row(sa, oracle):
    rng = np.random.default_rng(60)
    B, H, T, D = 1, 4, 777, 128
    q, k, v = normal_bf16(rng, (B, H, T, D)), normal_bf16(rng, (B, H, T, D)), normal_bf16(rng, (B, H, T, D))
    kc, ks = oracle.kv_quant_int8(k)
    vc, vs = oracle.kv_quant_int8(v)
    scale = 1.0 / math.sqrt(D)
    pre = sa.slim_attn_prefill(dev_bf16(q), dev(kc), dev(vc), scale, True, k_scale=dev(ks), v_scale=dev(vs))
    dec = sa.slim_attn_decode_int8(dev_bf16(np.ascontiguousarray(q[:, :, T - 1:T])), dev(kc), dev(ks), dev(vc), dev(vs), scale)
    torch.cuda.synchronize()
    diff = (pre[:, :, T - 1].float() - dec[:, :, 0].float()).abs().max().item()
    assert diff <= 2e-2, diff


# ---------------------------------------------------------------- quantise -> attend, all on the GPU

def test_gpu_quantiser_feeds_gpu_attention(sa, oracle):
    rng = np.random.default_rng(61)
    B, Hq, Hkv, S, D = 1, 4, 2, 500, 128
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    kc, ks = sa.kv_quant_int8(dev_bf16(k))
    vc, vs = sa.kv_quant_int8(dev_bf16(v))
    scale = 1.0 / math.sqrt(D)
    out = sa.slim_attn_prefill(dev_bf16(q), kc, vc, scale, True, k_scale=ks, v_scale=vs)
    torch.cuda.synchronize()
    okc, oks = oracle.kv_quant_int8(k)
    ovc, ovs = oracle.kv_quant_int8(v)
    want = oracle.attn(q, okc, ovc, scale, True, k_scale=oks, v_scale=ovs)
    check_close(host_f64(out), want, "quantise -> prefill")


def test_kv_quant_bit_exact_every_bf16_value_against_many_scales(sa, oracle):
    # Rows [amax, x_1 .. x_127]: for 1024 amax values (every exponent a normal bf16 amax can take, random
    # mantissas, plus subnormal and huge ones) the rows together enumerate every bf16 x with |x| <= amax,
    # both signs.  This walks the quantiser through every quotient x/scale it can meet, near-ties included.
    rng = np.random.default_rng(33)
    amax_bits = np.unique(np.concatenate([
        rng.integers(0x0080, 0x7f00, 900), rng.integers(0x0001, 0x0080, 60), np.array([0x7f7f, 0x0001, 0x3f80, 0x42fe])
    ]).astype(np.uint16))[:1024]
    rows = []
    for ab in amax_bits.tolist():
        xs = np.arange(0, ab + 1, dtype=np.uint32)          # every non-negative bf16 up to amax
        if xs.size > 8128:                                   # subsample large ranges, keep the top of the range dense
            xs = np.unique(np.concatenate([rng.choice(xs, 6000, replace=False), xs[-2128:]]))
        signs = rng.integers(0, 2, xs.size).astype(np.uint32) << 15
        vals = (xs | signs).astype(np.uint16)
        pad = (-vals.size) % 127
        vals = np.concatenate([vals, np.zeros(pad, dtype=np.uint16)]).reshape(-1, 127)
        rows.append(np.concatenate([np.full((vals.shape[0], 1), ab, dtype=np.uint16), vals], axis=1))
    bits = np.concatenate(rows, axis=0)
    bits = bits[: (bits.shape[0] // 4) * 4].reshape(1, 4, -1, 128)
    print("kv_quant exhaustive-style rows", bits.shape, flush=True)
    _quant_both(sa, oracle, np.ascontiguousarray(bits))


@pytest.mark.timeout(1200)
def test_kv_quant_bit_exact_every_bf16_pair(sa, oracle):
    # EVERY finite positive bf16 amax (32 639 of them, subnormal and huge ones included) with EVERY bf16 0 <= x <= amax
    # (random signs): 5.3e8 quotients, the whole domain of the quantiser's per-value arithmetic, on the hardware's own
    # reciprocal.  Rows are [amax, x_1 .. x_127]; processed in slices of the amax range to bound the host memory.
    rng = np.random.default_rng(34)
    edges = [1, 0x2000, 0x4000, 0x5000, 0x6000, 0x6800, 0x7000, 0x7800, 0x7f80]
    total = 0
    for lo, hi in zip(edges[:-1], edges[1:]):
        n_rows = sum((ab + 1 + 126) // 127 for ab in range(lo, hi))
        n_rows_pad = (n_rows + 3) // 4 * 4
        bits = np.zeros((n_rows_pad, 128), dtype=np.uint16)
        r = 0
        for ab in range(lo, hi):
            xs = np.arange(0, ab + 1, dtype=np.uint16)
            k = (xs.size + 126) // 127
            blk = np.zeros(k * 127, dtype=np.uint16)
            blk[:xs.size] = xs
            bits[r:r + k, 0] = ab
            bits[r:r + k, 1:] = blk.reshape(k, 127)
            r += k
        assert r == n_rows
        bits[:, 1:] |= (rng.integers(0, 2, (n_rows_pad, 127)).astype(np.uint16) << 15)
        total += int(n_rows) * 127
        print("kv_quant every pair: amax bits [0x%04x, 0x%04x), %d rows" % (lo, hi, n_rows), flush=True)
        _quant_both(sa, oracle, np.ascontiguousarray(bits.reshape(1, 4, n_rows_pad // 4, 128)))
        del bits
    assert total >= 532_000_000


def test_prefill_int8_with_all_zero_tokens(sa, oracle):
    # a token whose K (or V) row is all zeros quantises to scale 0 and codes 0: it must act as a zero vector
    rng = np.random.default_rng(62)
    B, Hq, Hkv, S, D = 1, 2, 2, 200, 128
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    k[0, 0, 5] = 0
    k[0, 1, 0] = 0
    v[0, 0, 7] = 0
    v[0, 1, 199] = 0
    kc, ks = oracle.kv_quant_int8(k)
    vc, vs = oracle.kv_quant_int8(v)
    assert ks[0, 0, 5] == 0 and vs[0, 1, 199] == 0
    scale = 1.0 / math.sqrt(D)
    out = sa.slim_attn_prefill(dev_bf16(q), dev(kc), dev(vc), scale, True, k_scale=dev(ks), v_scale=dev(vs))
    dec = sa.slim_attn_decode_int8(dev_bf16(np.ascontiguousarray(q[:, :, S - 1:S])), dev(kc), dev(ks), dev(vc), dev(vs), scale)
    torch.cuda.synchronize()
    want = oracle.attn(q, kc, vc, scale, True, k_scale=ks, v_scale=vs)
    check_close(host_f64(out), want, "prefill with zero tokens")
    check_close(host_f64(dec)[:, :, 0], want[:, :, S - 1], "decode with zero tokens")


def test_prefill_large_scores_and_repeat_runs_are_bit_identical(sa, oracle):
    # scores far from zero (softmax scale 1.0 on N(0,1) data with D=64 gives |s| up to ~40): the lazy
    # running max must still track them; two launches must agree bit for bit
    rng = np.random.default_rng(63)
    B, Hq, Hkv, S, D = 1, 4, 2, 700, 64
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    o1 = sa.slim_attn_prefill(dev_bf16(q), dev_bf16(k), dev_bf16(v), 1.0, True, out_dtype=torch.float32)
    o2 = sa.slim_attn_prefill(dev_bf16(q), dev_bf16(k), dev_bf16(v), 1.0, True, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)
    check_close(host_f64(o1), oracle.attn(q, k, v, 1.0, True), "prefill, softmax scale 1.0")
    on = sa.slim_attn_prefill(dev_bf16(q), dev_bf16(k), dev_bf16(v), 1.0, False, out_dtype=torch.float32)
    torch.cuda.synchronize()
    check_close(host_f64(on), oracle.attn(q, k, v, 1.0, False), "non-causal prefill, softmax scale 1.0")


def test_prefill_batched_gqa_full_tensor(sa, oracle):
    rng = np.random.default_rng(64)
    B, Hq, Hkv, S, D = 3, 8, 2, 385, 128
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    scale = 1.0 / math.sqrt(D)
    out = sa.slim_attn_prefill(dev_bf16(q), dev_bf16(k), dev_bf16(v), scale, True)
    torch.cuda.synchronize()
    check_close(host_f64(out), oracle.attn(q, k, v, scale, True), "batched GQA prefill")


@pytest.mark.parametrize("kv_int8", [False, True])
def test_prefill_many_launches_are_bit_identical(sa, oracle, kv_int8):
    # the ring slots are reused from the first phase on: a missing wait between a read and the next request
    # for the same slot shows as a rare difference between launches, so every launch is compared
    rng = np.random.default_rng(65)
    B, Hq, Hkv, S, D = 1, 8, 2, 640, 128
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    scale = 1.0 / math.sqrt(D)
    dq = dev_bf16(q)
    if kv_int8:
        kc, ks = oracle.kv_quant_int8(k)
        vc, vs = oracle.kv_quant_int8(v)
        args = (dq, dev(kc), dev(vc), scale, True)
        kw = dict(k_scale=dev(ks), v_scale=dev(vs))
        want = oracle.attn(q, kc, vc, scale, True, k_scale=ks, v_scale=vs)
    else:
        args = (dq, dev_bf16(k), dev_bf16(v), scale, True)
        kw = {}
        want = oracle.attn(q, k, v, scale, True)
    first = sa.slim_attn_prefill(*args, **kw)
    torch.cuda.synchronize()
    check_close(host_f64(first), want, "first launch")
    differing = 0
    for _ in range(200):
        out = sa.slim_attn_prefill(*args, **kw)
        differing += int(not torch.equal(out, first))
    torch.cuda.synchronize()
    assert differing == 0


def _random_shape(i):
    rng = np.random.default_rng(1000 + i)
    hkv = int(rng.integers(1, 4))
    return dict(B=int(rng.integers(1, 4)), Hkv=hkv, Hq=hkv * int(rng.choice([1, 2, 4])),
                n=int(rng.choice([rng.integers(1, 40), rng.integers(40, 300), rng.integers(300, 900)])),
                D=int(rng.choice([64, 128])), causal=bool(rng.integers(0, 2)), kv_int8=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("i", range(16))
def test_prefill_seeded_random_shapes(sa, oracle, i):
    # lengths that are no multiple of a tile, a row block or a ring depth, batches and head groupings mixed
    c = _random_shape(i)
    print("prefill random shape", i, c, flush=True)
    _prefill_case(sa, oracle, c["B"], c["Hq"], c["Hkv"], c["n"], c["D"], c["causal"], c["kv_int8"], out_f32=bool(i & 1),
                  seed=2000 + i)


@pytest.mark.parametrize("i", range(12))
def test_decode_seeded_random_shapes(sa, oracle, i):
    c = _random_shape(100 + i)
    T = c["n"] * 7 + 1   # up to ~6300 cached tokens: several splits and a ragged last chunk
    print("decode random shape", i, c, "T", T, flush=True)
    _decode_case(sa, oracle, c["B"], c["Hq"], c["Hkv"], T, c["D"], seed=3000 + i)


@pytest.mark.parametrize("D,Hq,Hkv,T", [(128, 64, 2, 333), (128, 32, 1, 1500), (64, 32, 1, 97), (128, 33, 1, 200),
                                        (64, 48, 3, 2049), (128, 6, 2, 4100), (128, 16, 1, 31), (128, 24, 8, 129)])
def test_decode_grouped_query_heads(sa, oracle, D, Hq, Hkv, T):
    # 2 to 32 query heads per KV head take the kernel that reads the cache once per KV head (one tile, ragged
    # tails, several tiles per wave, runs that end inside a tile); 33 heads per KV head take the per-head kernel
    print("decode grouped", D, Hq, Hkv, T, flush=True)
    _decode_case(sa, oracle, 2, Hq, Hkv, T, D, 70 + T)


@pytest.mark.timeout(600)
def test_decode_llama70b_shape_full_size(sa, oracle):
    # the grouped-query shape of the paper's larger model: 64 query heads on 8 KV heads, 8192 cached tokens
    print("decode 64/8 heads, full tensor", flush=True)
    _decode_case(sa, oracle, 16, 64, 8, 8192, 128, 77)


def test_decode_grouped_all_zero_tokens_and_huge_scores(sa, oracle):
    # tokens whose row is all zero (scale 0) and a softmax scale that makes the scores large
    rng = np.random.default_rng(78)
    B, Hq, Hkv, T, D = 1, 8, 2, 700, 128
    q, k, v = normal_bf16(rng, (B, Hq, 1, D)), normal_bf16(rng, (B, Hkv, T, D)), normal_bf16(rng, (B, Hkv, T, D))
    k[:, :, 5::7, :] = 0
    v[:, :, 3::11, :] = 0
    kc, ks = oracle.kv_quant_int8(k)
    vc, vs = oracle.kv_quant_int8(v)
    for scale in (1.0 / math.sqrt(D), 1.0):
        out = sa.slim_attn_decode_int8(dev_bf16(q), dev(kc), dev(ks), dev(vc), dev(vs), scale)
        torch.cuda.synchronize()
        check_close(host_f64(out), oracle.attn(q, kc, vc, scale, False, k_scale=ks, v_scale=vs), "grouped decode, scale %g" % scale)


@pytest.mark.parametrize("D,Hq,Hkv", [(128, 4, 4), (128, 16, 2), (64, 8, 8), (64, 6, 3)])
def test_decode_per_sequence_lengths(sa, oracle, D, Hq, Hkv):
    # every sequence attends to its own number of cached tokens (one tile, ragged tails, the whole allocation);
    # what lies past a sequence's length in the cache must not reach the result: it is filled with huge codes
    rng = np.random.default_rng(81 + D + Hq)
    B, T = 6, 1500
    lens = np.array([1, 31, 32, 700, 1499, 1500], dtype=np.int32)
    q = normal_bf16(rng, (B, Hq, 1, D))
    k, v = normal_bf16(rng, (B, Hkv, T, D)), normal_bf16(rng, (B, Hkv, T, D))
    kc, ks = oracle.kv_quant_int8(k)
    vc, vs = oracle.kv_quant_int8(v)
    kc2, ks2, vc2, vs2 = kc.copy(), ks.copy(), vc.copy(), vs.copy()
    for b in range(B):
        kc2[b, :, lens[b]:] = 127
        vc2[b, :, lens[b]:] = -127
        ks2[b, :, lens[b]:] = 1.0e6
        vs2[b, :, lens[b]:] = 1.0e6
    scale = 1.0 / math.sqrt(D)
    out = sa.slim_attn_decode_int8_varlen(dev_bf16(q), dev(kc2), dev(ks2), dev(vc2), dev(vs2),
                                          torch.from_numpy(lens).cuda(), scale)
    torch.cuda.synchronize()
    # (the tolerance is that of an output tensor: max-abs over everything, mean-abs over the batch.  A sequence of
    # one token returns v_0 times its v_scale rounded to bf16 in the grouped-query kernel, a relative error of up
    # to 2^-8 on every element of that row, so a single short row sits near the mean-abs limit by itself.)
    def expect(lengths):
        return np.concatenate([oracle.attn(q[b:b + 1], kc[b:b + 1, :, :n], vc[b:b + 1, :, :n], scale, False,
                                           k_scale=ks[b:b + 1, :, :n], v_scale=vs[b:b + 1, :, :n])
                               for b, n in enumerate(lengths)], axis=0)
    check_close(host_f64(out), expect([int(n) for n in lens]), "decode with per-sequence lengths")
    # lengths outside [1, T] are taken as the nearest bound
    lens2 = np.array([0, -5, 1, 1501, 99999, 1500], dtype=np.int32)
    out2 = sa.slim_attn_decode_int8_varlen(dev_bf16(q), dev(kc), dev(ks), dev(vc), dev(vs), torch.from_numpy(lens2).cuda(), scale)
    torch.cuda.synchronize()
    check_close(host_f64(out2), expect([1, 1, 1, 1500, 1500, 1500]), "decode with clamped lengths")


@pytest.mark.parametrize("D,Hq,Hkv", [(128, 8, 2), (64, 4, 4)])
def test_append_then_decode_serving_step(sa, oracle, D, Hq, Hkv):
    # one step of a serving loop: the new token's K and V rows are quantised into each sequence's cache at its
    # own position, then every sequence attends to its cache including the new token
    rng = np.random.default_rng(90 + D)
    B, T = 5, 600
    lens = np.array([0, 1, 31, 300, 599], dtype=np.int32)          # tokens cached so far = position of the new one
    pos = np.array([0, 1, 31, 300, 599], dtype=np.int32)
    q = normal_bf16(rng, (B, Hq, 1, D))
    k, v = normal_bf16(rng, (B, Hkv, T, D)), normal_bf16(rng, (B, Hkv, T, D))
    k_new, v_new = normal_bf16(rng, (B, Hkv, 1, D)), normal_bf16(rng, (B, Hkv, 1, D))
    k_new[2, 0] = 0                                                  # an all-zero row: scale 0, codes 0
    kc, ks = oracle.kv_quant_int8(k)
    vc, vs = oracle.kv_quant_int8(v)
    dkc, dks, dvc, dvs = dev(kc), dev(ks), dev(vc), dev(vs)
    dpos = torch.from_numpy(pos).cuda()
    sa.kv_quant_int8_append(dev_bf16(k_new), dkc, dks, dpos)
    sa.kv_quant_int8_append(dev_bf16(v_new), dvc, dvs, dpos)
    torch.cuda.synchronize()
    # the cache afterwards: the oracle's codes and scale of the new row at its position, nothing else touched
    knc, kns = oracle.kv_quant_int8(k_new)
    vnc, vns = oracle.kv_quant_int8(v_new)
    for b in range(B):
        kc[b, :, pos[b]] = knc[b, :, 0]
        ks[b, :, pos[b]] = kns[b, :, 0]
        vc[b, :, pos[b]] = vnc[b, :, 0]
        vs[b, :, pos[b]] = vns[b, :, 0]
    assert np.array_equal(dkc.cpu().numpy(), kc) and np.array_equal(dvc.cpu().numpy(), vc)
    assert np.array_equal(dks.cpu().numpy().view(np.uint32), ks.view(np.uint32))
    assert np.array_equal(dvs.cpu().numpy().view(np.uint32), vs.view(np.uint32))
    # a position outside the cache writes nothing
    bad = torch.from_numpy(np.array([-1, T, T + 5, -7, 1 << 30], dtype=np.int32)).cuda()
    sa.kv_quant_int8_append(dev_bf16(k_new), dkc, dks, bad)
    torch.cuda.synchronize()
    assert np.array_equal(dkc.cpu().numpy(), kc)
    scale = 1.0 / math.sqrt(D)
    out = sa.slim_attn_decode_int8_varlen(dev_bf16(q), dkc, dks, dvc, dvs, torch.from_numpy(lens + 1).cuda(), scale)
    torch.cuda.synchronize()
    want = np.concatenate([oracle.attn(q[b:b + 1], kc[b:b + 1, :, :n + 1], vc[b:b + 1, :, :n + 1], scale, False,
                                       k_scale=ks[b:b + 1, :, :n + 1], v_scale=vs[b:b + 1, :, :n + 1])
                           for b, n in enumerate(lens)], axis=0)
    check_close(host_f64(out), want, "append + decode")


def test_calls_follow_the_current_stream(sa, oracle):
    # every entry point enqueues on the stream it is given: a chain of calls on a side stream, with no
    # synchronisation in between, gives bit for bit what the default stream gives
    rng = np.random.default_rng(95)
    B, Hq, Hkv, S, D = 1, 8, 2, 520, 128
    q, k, v = (dev_bf16(normal_bf16(rng, shp)) for shp in ((B, Hq, S, D), (B, Hkv, S, D), (B, Hkv, S, D)))
    scale = 1.0 / math.sqrt(D)

    def chain():
        kc, ks = sa.kv_quant_int8(k)
        vc, vs = sa.kv_quant_int8(v)
        pre = sa.slim_attn_prefill(q, kc, vc, scale, True, k_scale=ks, v_scale=vs)
        dec = sa.slim_attn_decode_int8(q[:, :, S - 1:S].contiguous(), kc, ks, vc, vs, scale)
        return kc, ks, pre, dec

    ref = chain()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        got = chain()
    side.synchronize()
    for a, b in zip(ref, got):
        assert torch.equal(a, b)


def test_calls_on_two_streams_at_once_do_not_disturb_each_other(sa, oracle):
    # the library keeps no state between calls (the static-scratch decode aside): two different chains of calls,
    # each with buffers of its own, enqueued alternately on two streams with nothing to order them, give bit for bit
    # what each gives alone
    rng = np.random.default_rng(96)
    scale = 1.0 / math.sqrt(128)
    shapes = [(1, 8, 2, 700, 128), (2, 4, 4, 333, 128)]
    data = []
    for B, Hq, Hkv, S, D in shapes:
        q, k, v = (dev_bf16(normal_bf16(rng, shp)) for shp in ((B, Hq, S, D), (B, Hkv, S, D), (B, Hkv, S, D)))
        ws = torch.empty((sa.slim_attn_decode_int8_workspace_bytes(B, Hq, Hkv, S, D),), dtype=torch.uint8, device="cuda")
        data.append((q, k, v, q[:, :, S - 1:S].contiguous(), ws))

    def links(q, k, v, q1, ws):
        # one chain, cut into its calls, so that the two chains can be dealt out alternately
        box = {}
        yield lambda: box.update(zip(("kc", "ks", "vc", "vs"), sa.kv_quant_int8_pair(k, v)))
        yield lambda: box.update(pre=sa.slim_attn_prefill(q, k, v, scale, True))
        yield lambda: box.update(pre8=sa.slim_attn_prefill(q, box["kc"], box["vc"], scale, True, k_scale=box["ks"], v_scale=box["vs"]))
        yield lambda: box.update(dec=sa.slim_attn_decode_int8(q1, box["kc"], box["ks"], box["vc"], box["vs"], scale, workspace=ws))
        yield lambda: box.update(strip=sa.slim_attn_prefill_strip(q, k, v, scale, True))
        yield box

    def run_alone(d):
        *calls, box = list(links(*d))
        for c in calls:
            c()
        torch.cuda.synchronize()
        return box

    refs = [run_alone(d) for d in data]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    chains = [list(links(*d)) for d in data]
    for step_i in range(len(chains[0]) - 1):
        for st, ch in zip(streams, chains):
            with torch.cuda.stream(st):
                ch[step_i]()
    for st in streams:
        st.synchronize()
    for ref, ch in zip(refs, chains):
        got = ch[-1]
        for name in ref:
            assert torch.equal(got[name].view(torch.uint8), ref[name].view(torch.uint8)), name + " differs when two streams run at once"


def test_every_entry_point_replays_from_a_hip_graph(sa, oracle):
    # no entry point allocates, synchronises or clears memory with a memset node: a whole serving step (build the
    # cache, prefill over it, the comparison variants, append a token, decode) recorded into one HIP graph gives, on
    # every replay, with eager work and synchronisations in between, the bits of the eager calls
    rng = np.random.default_rng(97)
    B, Hq, Hkv, S, D = 1, 8, 2, 520, 128
    q, k, v = (dev_bf16(normal_bf16(rng, shp)) for shp in ((B, Hq, S, D), (B, Hkv, S, D), (B, Hkv, S, D)))
    k_new, v_new = (dev_bf16(normal_bf16(rng, (B, Hkv, 1, D))) for _ in range(2))
    q1 = q[:, :, S - 1:S].contiguous()
    scale = 1.0 / math.sqrt(D)
    pos = torch.full((B,), S - 1, dtype=torch.int32, device="cuda")
    lens = torch.full((B,), S, dtype=torch.int32, device="cuda")
    ws = torch.empty((sa.slim_attn_decode_int8_workspace_bytes(B, Hq, Hkv, S, D),), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty((B * Hq * S * 2,), dtype=torch.float32, device="cuda")

    def buffers():
        return {"kc": torch.empty((B, Hkv, S, D), dtype=torch.int8, device="cuda"),
                "ks": torch.empty((B, Hkv, S), dtype=torch.float32, device="cuda"),
                "vc": torch.empty((B, Hkv, S, D), dtype=torch.int8, device="cuda"),
                "vs": torch.empty((B, Hkv, S), dtype=torch.float32, device="cuda"),
                "kc2": torch.empty((B, Hkv, S, D), dtype=torch.int8, device="cuda"),
                "ks2": torch.empty((B, Hkv, S), dtype=torch.float32, device="cuda"),
                "vc2": torch.empty((B, Hkv, S, D), dtype=torch.int8, device="cuda"),
                "vs2": torch.empty((B, Hkv, S), dtype=torch.float32, device="cuda"),
                "pre": torch.empty_like(q), "pre8": torch.empty_like(q), "two": torch.empty_like(q),
                "strip": torch.empty_like(q), "dec": torch.empty_like(q1), "var": torch.empty_like(q1),
                "stat": torch.empty_like(q1)}

    def step(o):
        sa.kv_quant_int8(k, o["kc"], o["ks"])
        sa.kv_quant_int8(v, o["vc"], o["vs"])
        sa.kv_quant_int8_pair(k, v, o["kc2"], o["ks2"], o["vc2"], o["vs2"])
        sa.slim_attn_prefill(q, k, v, scale, True, out=o["pre"])
        sa.slim_attn_prefill(q, o["kc"], o["vc"], scale, True, k_scale=o["ks"], v_scale=o["vs"], out=o["pre8"])
        sa.slim_attn_prefill_two_sweep(q, k, v, scale, True, out=o["two"], workspace=ws2)
        sa.slim_attn_prefill_strip(q, k, v, scale, True, out=o["strip"])
        sa.kv_quant_int8_append(k_new, o["kc"], o["ks"], pos)
        sa.kv_quant_int8_append(v_new, o["vc"], o["vs"], pos)
        sa.slim_attn_decode_int8(q1, o["kc"], o["ks"], o["vc"], o["vs"], scale, out=o["dec"], workspace=ws)
        sa.slim_attn_decode_int8_varlen(q1, o["kc"], o["ks"], o["vc"], o["vs"], lens, scale, out=o["var"], workspace=ws)
        sa.slim_attn_decode_int8_static(q1, o["kc"], o["ks"], o["vc"], o["vs"], scale, o["stat"])

    ref = buffers()
    step(ref)
    torch.cuda.synchronize()
    assert torch.equal(ref["dec"], ref["var"]) and torch.equal(ref["dec"], ref["stat"])
    got = buffers()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(got)
    for rep in range(3):
        for name, t in got.items():                       # eager work between the replays: every output is spoiled
            t.fill_(1) if t.dtype == torch.int8 else t.fill_(float("nan"))
        sa.slim_attn_decode_int8(q1, ref["kc"], ref["ks"], ref["vc"], ref["vs"], scale, workspace=ws)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in ref:
            assert torch.equal(got[name].view(torch.uint8), ref[name].view(torch.uint8)), "replay %d: %s differs" % (rep, name)


def _loaded_hip_runtime():
    """The HIP runtime this process already has mapped (the one the library and torch call into)."""
    import ctypes
    for ln in open("/proc/self/maps"):
        path = ln.split()[-1]
        if "libamdhip64" in path:
            return ctypes.CDLL(path)
    raise AssertionError("no HIP runtime is mapped")


def test_a_stale_hip_error_is_not_reported_as_a_failed_launch(sa, oracle):
    # An error that one of the caller's own HIP calls left behind on the thread must not come back as
    # SLIM_ERR_LAUNCH (and must not stop a call after its first of two launches): every entry point drops it.
    rng = np.random.default_rng(96)
    B, Hq, Hkv, T, D = 2, 4, 4, 3000, 128
    q = dev_bf16(normal_bf16(rng, (B, Hq, 1, D)))
    k, v = dev_bf16(normal_bf16(rng, (B, Hkv, T, D))), dev_bf16(normal_bf16(rng, (B, Hkv, T, D)))
    scale = 1.0 / math.sqrt(D)
    kc, ks = sa.kv_quant_int8(k)
    vc, vs = sa.kv_quant_int8(v)
    ref = sa.slim_attn_decode_int8(q, kc, ks, vc, vs, scale)
    torch.cuda.synchronize()
    hip = _loaded_hip_runtime()
    # everything torch has to launch or allocate comes first: torch checks for left-over errors itself
    kc2, ks2, out = torch.zeros_like(kc), torch.zeros_like(ks), torch.zeros_like(ref)
    qp, kp, vp = (t[:, :, :300].contiguous() for t in (k, k, v))
    pre = torch.zeros_like(qp)
    ws = torch.zeros((sa.slim_attn_decode_int8_workspace_bytes(B, Hq, Hkv, T, D),), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()

    def plant():
        assert hip.hipSetDevice(12345) != 0   # an invalid device: fails, changes nothing, leaves its error behind

    plant()
    sa.kv_quant_int8(k, kc2, ks2)
    plant()
    sa.slim_attn_decode_int8(q, kc, ks, vc, vs, scale, out=out, workspace=ws)   # split kernel + combine kernel
    plant()
    sa.slim_attn_prefill(qp, kp, vp, scale, True, out=pre)
    torch.cuda.synchronize()
    assert torch.equal(kc2, kc) and torch.equal(ks2, ks) and torch.equal(out, ref)
    assert bool(torch.isfinite(pre).all()) and bool((pre != 0).any())
    hip.hipGetLastError()


def test_closed_forms_on_the_gpu(sa, oracle):
    # checks that need no oracle: equal keys give the running mean of V (causal) or its mean (decode); one key that
    # dominates every score returns its V row.  bf16 K/V for prefill, the INT8 cache for decode (both kernels).
    rng = np.random.default_rng(97)
    B, H, S, D = 1, 4, 300, 128
    q = normal_bf16(rng, (B, H, S, D))
    v = normal_bf16(rng, (B, H, S, D))
    k_same = np.broadcast_to(normal_bf16(rng, (B, H, 1, D)), (B, H, S, D)).copy()
    scale = 1.0 / math.sqrt(D)
    vf = (v.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    run_mean = np.cumsum(vf, axis=2) / np.arange(1, S + 1)[None, None, :, None]
    out = sa.slim_attn_prefill(dev_bf16(q), dev_bf16(k_same), dev_bf16(v), scale, True, out_dtype=torch.float32)
    torch.cuda.synchronize()
    check_close(host_f64(out), run_mean, "equal keys: running mean of V")
    for Hq, Hkv in ((4, 4), (8, 2)):
        qd = normal_bf16(rng, (B, Hq, 1, D))
        kd = np.broadcast_to(normal_bf16(rng, (B, Hkv, 1, D)), (B, Hkv, S, D)).copy()
        vd = normal_bf16(rng, (B, Hkv, S, D))
        kc, ks = oracle.kv_quant_int8(kd)
        vc, vs = oracle.kv_quant_int8(vd)
        dec = sa.slim_attn_decode_int8(dev_bf16(qd), dev(kc), dev(ks), dev(vc), dev(vs), scale)
        torch.cuda.synchronize()
        v_hat = vc.astype(np.float64) * vs.astype(np.float64)[..., None]
        mean_v = np.repeat(v_hat.mean(axis=2, keepdims=True), Hq // Hkv, axis=1)
        check_close(host_f64(dec), mean_v, "equal keys: mean of the dequantised V (decode %d/%d)" % (Hq, Hkv))
    # one dominant key: key j0 is 8 q_i / |q_i| for no i in particular, so use a key aligned with every query: all
    # queries equal; the key at j0 equals the query scaled up, the others are orthogonal noise scaled down
    q1 = np.broadcast_to(normal_bf16(rng, (B, H, 1, D)), (B, H, S, D)).copy()
    q1f = (q1.astype(np.uint32) << 16).view(np.float32)
    k_small = (0.01 * rng.standard_normal((B, H, S, D))).astype(np.float32)
    j0 = 3
    k_small[:, :, j0] = 4.0 * q1f[:, :, 0]
    from paper_2407_07304_amd.inputs import f32_to_bf16_bits
    kb = f32_to_bf16_bits(k_small)
    out = sa.slim_attn_prefill(dev_bf16(q1), dev_bf16(kb), dev_bf16(v), 1.0, False, out_dtype=torch.float32)
    torch.cuda.synchronize()
    want = np.broadcast_to(vf[:, :, j0:j0 + 1], (B, H, S, D))
    check_close(host_f64(out), want, "one dominant key returns its V row")


@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal", [(1, 4, 4, 300, 128, True), (2, 8, 2, 517, 128, True), (1, 4, 2, 130, 64, False),
                                                (1, 2, 2, 1, 128, True), (1, 6, 3, 1000, 64, True)])
def test_prefill_that_emits_the_int8_cache(sa, oracle, B, Hq, Hkv, S, D, causal):
    # one launch: the attention of the plain bf16 prefill, bit for bit, and the oracle quantiser's codes and scales
    rng = np.random.default_rng(99 + S)
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    if S > 40:   # rows the quantiser treats specially: all zero, one non-zero, subnormal and huge values
        k[0, 0, 7] = 0
        v[0, 0, 9] = 0
        v[0, 0, 9, 5] = 0x3f80
        k[0, 0, 11] = 0x0001
        v[0, 0, 12] = 0x7f7f
    scale = 1.0 / math.sqrt(D)
    dq, dk, dv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    ref = sa.slim_attn_prefill(dq, dk, dv, scale, causal)
    out, kc, ks, vc, vs = sa.slim_attn_prefill_emit_int8(dq, dk, dv, scale, causal)
    torch.cuda.synchronize()
    fin = torch.isfinite(ref.float())
    assert torch.equal(out[fin], ref[fin]) and torch.equal(torch.isfinite(out.float()), fin)
    okc, oks = oracle.kv_quant_int8(k)
    ovc, ovs = oracle.kv_quant_int8(v)
    assert np.array_equal(kc.cpu().numpy(), okc) and np.array_equal(vc.cpu().numpy(), ovc)
    assert np.array_equal(ks.cpu().numpy().view(np.uint32), oks.view(np.uint32))
    assert np.array_equal(vs.cpu().numpy().view(np.uint32), ovs.view(np.uint32))


# ---------------------------------------------------------------- the two-sweep comparison variant

@pytest.mark.parametrize("B,Hq,Hkv,S,D", SMALL)
@pytest.mark.parametrize("causal", [True, False])
def test_prefill_two_sweep_small_shapes(sa, oracle, B, Hq, Hkv, S, D, causal):
    print("two-sweep prefill", B, Hq, Hkv, S, D, causal, flush=True)
    _prefill_case(sa, oracle, B, Hq, Hkv, S, D, causal, False, out_f32=(S % 2 == 1), seed=40 + S, two_sweep=True)


@pytest.mark.timeout(600)
def test_prefill_two_sweep_c2_full_size(sa, oracle):
    w = WORKLOADS["C2"]
    print("two-sweep prefill C2, every row of every head", flush=True)
    _prefill_case(sa, oracle, w.batch, w.q_heads, w.kv_heads, w.seq_len, w.head_dim, True, False, False, w.seed,
                  two_sweep=True)


def test_prefill_two_sweep_large_scores_and_repeats(sa, oracle):
    # scores far from zero (the first sweep's maxima carry the whole range), run twice into a workspace that
    # starts dirty: the same bits both times, and the one-sweep kernel's result up to rounding order
    B, Hq, Hkv, S, D = 1, 4, 2, 700, 128
    rng = np.random.default_rng(77)
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    dq, dk, dv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    ws = torch.full((B * Hq * S * 2,), float("nan"), dtype=torch.float32, device="cuda")
    a = sa.slim_attn_prefill_two_sweep(dq, dk, dv, 2.0, True, out_dtype=torch.float32, workspace=ws)
    b = sa.slim_attn_prefill_two_sweep(dq, dk, dv, 2.0, True, out_dtype=torch.float32, workspace=ws)
    one = sa.slim_attn_prefill(dq, dk, dv, 2.0, True, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    check_close(host_f64(a), oracle.attn(q, k, v, 2.0, True), "two-sweep, scale 2")
    assert (a - one).abs().max().item() <= 2e-2


# ---------------------------------------------------------------- the on-chip score strip comparison variant

@pytest.mark.parametrize("B,Hq,Hkv,S,D", SMALL + [(1, 2, 1, 31, 128), (1, 1, 1, 1057, 64), (2, 2, 2, 2048, 128), (1, 2, 1, 2047, 64)])
@pytest.mark.parametrize("causal", [True, False])
def test_prefill_strip_small_shapes(sa, oracle, B, Hq, Hkv, S, D, causal):
    # every strip size class (512, 1024 and 2048 columns), ragged last tiles, chunks and row blocks, both head sizes
    print("strip prefill", B, Hq, Hkv, S, D, causal, flush=True)
    _prefill_case(sa, oracle, B, Hq, Hkv, S, D, causal, False, out_f32=(S % 2 == 1), seed=40 + S, strip=True)


@pytest.mark.timeout(600)
def test_prefill_strip_c2_full_size(sa, oracle):
    w = WORKLOADS["C2"]
    print("strip prefill C2, every row of every head", flush=True)
    _prefill_case(sa, oracle, w.batch, w.q_heads, w.kv_heads, w.seq_len, w.head_dim, True, False, False, w.seed, strip=True)


def test_prefill_strip_large_scores_repeats_and_long_sequences(sa, oracle):
    # scores far from zero (the strip holds them as fp16: scale 2 on N(0,1) data with D = 128 reaches |u| of a few
    # hundred in log2 units), the same bits on a second run, and a sequence whose strip does not fit on chip,
    # which takes the streamed kernel and must give its bits
    B, Hq, Hkv, S, D = 1, 4, 2, 700, 128
    rng = np.random.default_rng(79)
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    dq, dk, dv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    a = sa.slim_attn_prefill_strip(dq, dk, dv, 2.0, True, out_dtype=torch.float32)
    b = sa.slim_attn_prefill_strip(dq, dk, dv, 2.0, True, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    check_close(host_f64(a), oracle.attn(q, k, v, 2.0, True), "strip, scale 2")
    S2 = sa.slim_attn_prefill_strip_max_seq_len() + 1
    assert S2 == 2049
    q, k, v = normal_bf16(rng, (1, 2, S2, 64)), normal_bf16(rng, (1, 1, S2, 64)), normal_bf16(rng, (1, 1, S2, 64))
    dq, dk, dv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    long_strip = sa.slim_attn_prefill_strip(dq, dk, dv, 0.125, True)
    long_plain = sa.slim_attn_prefill(dq, dk, dv, 0.125, True)
    torch.cuda.synchronize()
    assert torch.equal(long_strip, long_plain)
    check_close(host_f64(long_strip), oracle.attn(q, k, v, 0.125, True), "strip entry point beyond its length")


@pytest.mark.parametrize("i", range(12))
def test_prefill_strip_seeded_random_shapes_and_scales(sa, oracle, i):
    # lengths that are no multiple of a tile, a chunk or a row block, batches, head groupings and softmax scales mixed
    c = _random_shape(200 + i)
    rng = np.random.default_rng(5000 + i)
    S = int(rng.choice([c["n"], c["n"] * 2 + 1, 1024 + c["n"]]))
    scale = float(rng.choice([1.0 / math.sqrt(c["D"]), 0.02, 0.3, 1.0]))
    print("strip prefill random shape", i, c, "S", S, "scale", scale, flush=True)
    q = normal_bf16(rng, (c["B"], c["Hq"], S, c["D"]))
    k, v = normal_bf16(rng, (c["B"], c["Hkv"], S, c["D"])), normal_bf16(rng, (c["B"], c["Hkv"], S, c["D"]))
    od = torch.float32 if i & 1 else torch.bfloat16
    out = sa.slim_attn_prefill_strip(dev_bf16(q), dev_bf16(k), dev_bf16(v), scale, c["causal"], out_dtype=od)
    one = sa.slim_attn_prefill(dev_bf16(q), dev_bf16(k), dev_bf16(v), scale, c["causal"], out_dtype=od)
    torch.cuda.synchronize()
    want = oracle.attn(q, k, v, scale, c["causal"])
    if scale <= 0.3:
        check_close(host_f64(out), want, "strip prefill, random shape %d" % i)
    else:
        # sharp rows: held to the streamed kernel's own distance from the oracle plus the tolerance's slack
        # (what the rounding of P to bf16 costs there is the same in both orders)
        err, err_one = np.abs(host_f64(out) - want), np.abs(host_f64(one) - want)
        assert np.isfinite(host_f64(out)).all() and err.max() <= max(2e-2, 1.5 * err_one.max()) and err.mean() <= 2e-3


def test_non_finite_values_stay_inside_their_kv_head(sa, oracle):
    # the documented contract: a non-finite value in a (batch, KV head)'s K, V or scales may spoil every output row of
    # the query heads that read that KV head (masked keys take part in the matrix products with probability zero),
    # and nothing else
    rng = np.random.default_rng(98)
    B, Hq, Hkv, S, D = 2, 4, 2, 300, 128
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    v_bad = v.copy()
    v_bad[0, 0, 250, 7] = 0x7f80                                     # +inf in V of (batch 0, KV head 0), at a late key
    scale = 1.0 / math.sqrt(D)
    out = sa.slim_attn_prefill(dev_bf16(q), dev_bf16(k), dev_bf16(v_bad), scale, True)
    torch.cuda.synchronize()
    want = oracle.attn(q, k, v, scale, True)
    got = host_f64(out)
    clean = np.ones((B, Hq), dtype=bool)
    clean[0, :2] = False                                             # query heads 0 and 1 of batch 0 read KV head 0
    check_close(got[clean], want[clean], "heads that do not read the spoiled KV head")
    kc, ks = oracle.kv_quant_int8(k)
    vc, vs = oracle.kv_quant_int8(v)
    vs_bad = vs.copy()
    vs_bad[1, 1, 5] = np.inf
    dec = sa.slim_attn_decode_int8(dev_bf16(np.ascontiguousarray(q[:, :, S - 1:S])), dev(kc), dev(ks), dev(vc), dev(vs_bad), scale)
    torch.cuda.synchronize()
    want_d = oracle.attn(np.ascontiguousarray(q[:, :, S - 1:S]), kc, vc, scale, False, k_scale=ks, v_scale=vs)
    clean = np.ones((B, Hq), dtype=bool)
    clean[1, 2:] = False
    check_close(host_f64(dec)[clean], want_d[clean], "decode heads that do not read the spoiled KV head")


# ---------------------------------------------------------------- sharp softmax: the arithmetic's own bound

@pytest.mark.parametrize("kv_int8", [False, True])
@pytest.mark.parametrize("out_f32", [False, True])
def test_sharp_softmax_stays_within_the_rounding_bound(sa, oracle, kv_int8, out_f32):
    # scale 0.5 on N(0,1) inputs: most rows are carried by one key, so the rounding of P (INT8: of P * v_scale) to
    # bf16 is not averaged over the keys.  One rounding to nearest is off by at most 2^-8 relative, hence per element
    #   |o - o_exact| <= 2^-8 * sum_j p_j |v_j|  (+ 2^-8 |o| for a bf16 output)  + fp32 noise,
    # the first sum being the oracle's attention over |V|.
    B, Hq, Hkv, S, D, scale = 2, 8, 2, 700, 128, 0.5
    rng = np.random.default_rng(321)
    q, k, v = normal_bf16(rng, (B, Hq, S, D)), normal_bf16(rng, (B, Hkv, S, D)), normal_bf16(rng, (B, Hkv, S, D))
    od = torch.float32 if out_f32 else torch.bfloat16
    causal = not out_f32
    if kv_int8:
        kc, ks = oracle.kv_quant_int8(k)
        vc, vs = oracle.kv_quant_int8(v)
        out = sa.slim_attn_prefill(dev_bf16(q), dev(kc), dev(vc), scale, causal, k_scale=dev(ks), v_scale=dev(vs), out_dtype=od)
        torch.cuda.synchronize()
        want = oracle.attn(q, kc, vc, scale, causal, k_scale=ks, v_scale=vs)
        mass = oracle.attn(q, kc, np.abs(vc), scale, causal, k_scale=ks, v_scale=vs)
    else:
        out = sa.slim_attn_prefill(dev_bf16(q), dev_bf16(k), dev_bf16(v), scale, causal, out_dtype=od)
        torch.cuda.synchronize()
        want = oracle.attn(q, k, v, scale, causal)
        mass = oracle.attn(q, k, v & np.uint16(0x7fff), scale, causal)
    got = host_f64(out)
    bound = 2.0 ** -8 * mass + (0.0 if out_f32 else 2.0 ** -8 * np.abs(want)) + 1e-5 * (1.0 + mass)
    err = np.abs(got - want)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), "element %s: error %.3e above its bound %.3e" % (worst, err[worst], bound[worst])
    assert float(err.mean()) <= 2e-3
    # the regime is the intended one: most rows are carried by a single key
    rows = range(S - 40, S)
    if kv_int8:
        tops = [oracle.attn_row_probs(q, kc, vc, scale, causal, 0, 0, i, k_scale=ks, v_scale=vs)[0].max() for i in rows]
    else:
        tops = [oracle.attn_row_probs(q, k, v, scale, causal, 0, 0, i)[0].max() for i in rows]
    assert np.median(tops) > 0.5


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2)])
def test_sharp_softmax_decode_stays_within_the_rounding_bound(sa, oracle, Hq, Hkv):
    # the same bound for the decode kernels (per-head: P * v_scale stays in fp32, only the bf16 output rounds;
    # grouped query heads: P * v_scale is rounded to bf16 as in the prefill)
    B, T, D, scale = 3, 1500, 128, 0.5
    rng = np.random.default_rng(654)
    q, k, v = normal_bf16(rng, (B, Hq, 1, D)), normal_bf16(rng, (B, Hkv, T, D)), normal_bf16(rng, (B, Hkv, T, D))
    kc, ks = oracle.kv_quant_int8(k)
    vc, vs = oracle.kv_quant_int8(v)
    out = sa.slim_attn_decode_int8(dev_bf16(q), dev(kc), dev(ks), dev(vc), dev(vs), scale)
    torch.cuda.synchronize()
    want = oracle.attn(q, kc, vc, scale, False, k_scale=ks, v_scale=vs)
    mass = oracle.attn(q, kc, np.abs(vc), scale, False, k_scale=ks, v_scale=vs)
    p_round = 2.0 ** -8 * mass if Hq != Hkv else 0.0
    bound = p_round + 2.0 ** -8 * np.abs(want) + 1e-5 * (1.0 + mass)
    err = np.abs(host_f64(out) - want)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), "element %s: error %.3e above its bound %.3e" % (worst, err[worst], bound[worst])

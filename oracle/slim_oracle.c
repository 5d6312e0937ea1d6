/*
 * CPU oracle for the SlimAttention hot path — TEST INFRASTRUCTURE, not product code.
 *
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may load this
 * library.  It shares no code, header, table or helper with the HIP kernels.
 *
 * Everything is the plain definition, evaluated in fp64 with scalar loops:
 *
 *   attention (paper section 2.1: a horizontal score row Q_i.K^T, a softmax over that
 *   row, then the row times V; repeated for the next row):
 *       s_j = softmax_scale * sum_d q[i,d] * k^[j,d]        for every visible key j
 *       m   = max_j s_j ;  p_j = exp(s_j - m) ;  l = sum_j p_j
 *       o_d = ( sum_j p_j * v^[j,d] ) / l
 *   The paper states that this ordering has no redundant computation and that the
 *   tiled alternative only needs corrections to reach the same final result, so the
 *   result is exactly softmax(Q K^T * scale + mask) V; the row-by-row form above IS
 *   that definition with a block of one row.
 *
 *   INT8 KV cache (paper section 2.2: K and V held as INT8 with one scale for each
 *   token and each head; the INT8 value is widened to FP32 and then used in an FMA):
 *       k^[j,d] = (double)code[j,d] * (double)scale[j]      (exact in fp64)
 *   Quantiser (symmetric, per (batch, kv head, token) row of D values):
 *       amax  = max_d |x_d|
 *       scale = fl32(amax / 127)                  one IEEE fp32 division, RNE
 *       code  = clamp(RNE(fl32(x_d / scale)), -127, 127)    ties to even
 *       amax == 0  ->  scale = 0 and every code = 0
 *
 * Pins (tests/test_oracle_*.py): pure-Python brute force, closed forms (uniform keys ->
 * mean of V, causal row 0 -> V_0, one dominant key), shift invariance, GQA == MHA on
 * repeated heads, decode == last causal row, exact rational arithmetic for the
 * quantiser, exhaustive bf16 sweeps of the two fp32 divisions.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC (never -ffast-math: the fp32 divisions above
 * must stay correctly rounded and nearbyintf must honour ties-to-even).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline float bf16_bits_to_float(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* ---------------------------------------------------------------- quantiser */

/* Quantise n_rows rows of D bf16 values each. x: [n_rows, D] bf16 bit patterns.
 * codes: [n_rows, D] int8, scales: [n_rows] fp32.  Returns 0. */
int oracle_kv_quant_int8(const uint16_t *x, int8_t *codes, float *scales,
                         long n_rows, int D) {
#pragma omp parallel for schedule(static)
    for (long r = 0; r < n_rows; ++r) {
        const uint16_t *row = x + r * (long)D;
        float amax = 0.0f;
        for (int d = 0; d < D; ++d) {
            float a = fabsf(bf16_bits_to_float(row[d]));
            if (a > amax) amax = a;
        }
        if (amax == 0.0f) {
            scales[r] = 0.0f;
            for (int d = 0; d < D; ++d) codes[r * (long)D + d] = 0;
            continue;
        }
        volatile float scale = amax / 127.0f; /* volatile: one rounding to fp32, no excess precision */
        scales[r] = scale;
        for (int d = 0; d < D; ++d) {
            volatile float quo = bf16_bits_to_float(row[d]) / scale;
            float rn = nearbyintf(quo); /* default rounding mode: ties to even */
            if (rn > 127.0f) rn = 127.0f;
            if (rn < -127.0f) rn = -127.0f;
            codes[r * (long)D + d] = (int8_t)rn;
        }
    }
    return 0;
}

/* Exhaustive check of the two fp32 divisions over bf16 inputs: for every positive
 * finite bf16 amax (bit patterns 0x0001..0x7f7f) the fp32 route amax/127 is compared
 * with the fp64 quotient narrowed to fp32; for every pair (|x| <= amax) the fp32
 * quotient x/scale is compared the same way.  Returns the number of disagreements in
 * out[0] (scale) and out[1] (quotient), pairs visited in out[2].  amax_step > 1
 * visits every amax_step-th amax (for a quick run). */
int oracle_quant_division_sweep(long long *out, int amax_step) {
    long long bad_scale = 0, bad_quo = 0, pairs = 0;
    if (amax_step < 1) amax_step = 1;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : bad_scale, bad_quo, pairs)
    for (int ab = 1; ab <= 0x7f7f; ab += amax_step) {
        float amax = bf16_bits_to_float((uint16_t)ab);
        volatile float s32 = amax / 127.0f;
        float s64 = (float)((double)amax / 127.0);
        if (memcmp((const void *)&s32, &s64, 4) != 0) bad_scale++;
        float scale = s32;
        if (scale == 0.0f) continue; /* not reached: the smallest bf16, 2^-133, over 127 is still an fp32 subnormal */
        for (int xb = 0; xb <= ab; ++xb) {
            float x = bf16_bits_to_float((uint16_t)xb);
            volatile float q32 = x / scale;
            float q64 = (float)((double)x / (double)scale);
            if (memcmp((const void *)&q32, &q64, 4) != 0) bad_quo++;
            pairs++;
        }
    }
    out[0] = bad_scale;
    out[1] = bad_quo;
    out[2] = pairs;
    return 0;
}

/* ---------------------------------------------------------------- attention */

/* One query row.  q: D bf16.  k, v: the kv head's [Skv, D] block (bf16 bits or int8
 * codes), ks/vs: its [Skv] scales (int8 only).  n_vis keys 0..n_vis-1 are visible.
 * o: D doubles.  probs (optional): n_vis doubles p_j / l.  scratch: n_vis doubles. */
static void attn_row(const uint16_t *q, const void *k, const void *v,
                     const float *ks, const float *vs, int kv_is_int8,
                     int n_vis, int D, double softmax_scale,
                     double *o, double *probs, double *scratch) {
    double *s = scratch;
    double m = -INFINITY;
    for (int j = 0; j < n_vis; ++j) {
        double dot = 0.0;
        if (kv_is_int8) {
            const int8_t *kr = (const int8_t *)k + (long)j * D;
            double sc = (double)ks[j];
            for (int d = 0; d < D; ++d)
                dot += (double)bf16_bits_to_float(q[d]) * ((double)kr[d] * sc);
        } else {
            const uint16_t *kr = (const uint16_t *)k + (long)j * D;
            for (int d = 0; d < D; ++d)
                dot += (double)bf16_bits_to_float(q[d]) * (double)bf16_bits_to_float(kr[d]);
        }
        s[j] = softmax_scale * dot;
        if (s[j] > m) m = s[j];
    }
    double l = 0.0;
    for (int j = 0; j < n_vis; ++j) {
        s[j] = exp(s[j] - m);
        l += s[j];
    }
    for (int d = 0; d < D; ++d) o[d] = 0.0;
    for (int j = 0; j < n_vis; ++j) {
        double p = s[j];
        if (kv_is_int8) {
            const int8_t *vr = (const int8_t *)v + (long)j * D;
            double sc = (double)vs[j];
            for (int d = 0; d < D; ++d) o[d] += p * ((double)vr[d] * sc);
        } else {
            const uint16_t *vr = (const uint16_t *)v + (long)j * D;
            for (int d = 0; d < D; ++d) o[d] += p * (double)bf16_bits_to_float(vr[d]);
        }
    }
    for (int d = 0; d < D; ++d) o[d] /= l;
    if (probs)
        for (int j = 0; j < n_vis; ++j) probs[j] = s[j] / l;
}

/* Attention over q [B,Hq,Sq,D] bf16 and k, v [B,Hkv,Skv,D] (bf16 bits, or int8 codes
 * with k_scale, v_scale [B,Hkv,Skv] fp32 when kv_is_int8).  Query head h reads kv head
 * h / (Hq/Hkv).  Query row i sits at absolute position i + (Skv - Sq); with causal != 0
 * it sees keys j <= that position (prefill: Sq == Skv -> j <= i; decode: Sq == 1 -> all
 * keys), otherwise every key.
 * rows == NULL: out is [B,Hq,Sq,D] doubles.  rows != NULL: only the n_rows listed query
 * rows are evaluated and out is [B,Hq,n_rows,D].
 * Returns 0, or 1 on a bad argument, 2 if memory ran out. */
int oracle_attn(const uint16_t *q, const void *k, const void *v,
                const float *k_scale, const float *v_scale, double *out,
                int B, int Hq, int Hkv, int Sq, int Skv, int D, int causal,
                double softmax_scale, int kv_is_int8, const int *rows, int n_rows) {
    if (!q || !k || !v || !out) return 1;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Sq <= 0 || Skv <= 0 || D <= 0) return 1;
    if (Hq % Hkv != 0 || Sq > Skv) return 1;
    if (kv_is_int8 && (!k_scale || !v_scale)) return 1;
    const int G = Hq / Hkv;
    const int R = rows ? n_rows : Sq;
    const long units = (long)B * Hq * R;
    const size_t esz = kv_is_int8 ? 1 : 2;
    int failed = 0;
#pragma omp parallel
    {
        double *scratch = (double *)malloc(sizeof(double) * (size_t)Skv);
        if (!scratch) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 4)
            for (long u = 0; u < units; ++u) {
                int r = (int)(u % R);
                int h = (int)((u / R) % Hq);
                int b = (int)(u / ((long)R * Hq));
                int i = rows ? rows[r] : r;
                int g = h / G;
                int n_vis = causal ? (i + (Skv - Sq) + 1) : Skv;
                long kvoff = ((long)b * Hkv + g) * (long)Skv;
                attn_row(q + (((long)b * Hq + h) * Sq + i) * (long)D,
                         (const char *)k + kvoff * D * esz,
                         (const char *)v + kvoff * D * esz,
                         kv_is_int8 ? k_scale + kvoff : NULL,
                         kv_is_int8 ? v_scale + kvoff : NULL,
                         kv_is_int8, n_vis, D, softmax_scale,
                         out + u * (long)D, NULL, scratch);
            }
        }
        free(scratch);
    }
    return failed ? 2 : 0;
}

/* Softmax probabilities p_j / l of ONE query row (b, h, i) of the same problem:
 * probs receives Skv doubles (0 for masked keys), o receives the D outputs. */
int oracle_attn_row_probs(const uint16_t *q, const void *k, const void *v,
                          const float *k_scale, const float *v_scale,
                          double *probs, double *o,
                          int B, int Hq, int Hkv, int Sq, int Skv, int D, int causal,
                          double softmax_scale, int kv_is_int8, int b, int h, int i) {
    if (!q || !k || !v || !probs || !o) return 1;
    if (b < 0 || b >= B || h < 0 || h >= Hq || i < 0 || i >= Sq || Hq % Hkv != 0 || Sq > Skv) return 1;
    const int G = Hq / Hkv;
    const size_t esz = kv_is_int8 ? 1 : 2;
    double *scratch = (double *)malloc(sizeof(double) * (size_t)Skv);
    if (!scratch) return 2;
    int g = h / G;
    int n_vis = causal ? (i + (Skv - Sq) + 1) : Skv;
    long kvoff = ((long)b * Hkv + g) * (long)Skv;
    for (int j = 0; j < Skv; ++j) probs[j] = 0.0;
    attn_row(q + (((long)b * Hq + h) * Sq + i) * (long)D,
             (const char *)k + kvoff * D * esz, (const char *)v + kvoff * D * esz,
             kv_is_int8 ? k_scale + kvoff : NULL, kv_is_int8 ? v_scale + kvoff : NULL,
             kv_is_int8, n_vis, D, softmax_scale, o, probs, scratch);
    free(scratch);
    return 0;
}

/* Threads an OpenMP region of this library actually runs with. */
int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}

/* Driver for a sanitizer build of the CPU oracle: it is compiled together with oracle/slim_oracle.c under
 * -fsanitize=address,undefined into one executable and walks every exported routine over small shapes that
 * reach its edges (one row, ragged lengths, grouped heads, row subsets, INT8 operands, all-zero, subnormal and
 * huge quantiser rows).  It checks nothing but a few invariants: the sanitizers are the test.  Exit code 0 = clean. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_kv_quant_int8(const uint16_t *x, int8_t *codes, float *scales, long n_rows, int D);
int oracle_quant_division_sweep(long long *out, int amax_step);
int oracle_attn(const uint16_t *q, const void *k, const void *v, const float *k_scale, const float *v_scale, double *out,
                int B, int Hq, int Hkv, int Sq, int Skv, int D, int causal, double softmax_scale, int kv_is_int8,
                const int *rows, int n_rows);
int oracle_attn_row_probs(const uint16_t *q, const void *k, const void *v, const float *k_scale, const float *v_scale,
                          double *probs, double *o, int B, int Hq, int Hkv, int Sq, int Skv, int D, int causal,
                          double softmax_scale, int kv_is_int8, int b, int h, int i);
int oracle_num_threads(void);

static uint32_t rng_state = 12345u;
static uint32_t next_u32(void) {
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state;
}
static uint16_t random_bf16(void) {   /* magnitudes around 1, both signs */
    uint32_t r = next_u32();
    return (uint16_t)(((r >> 16) & 0x8000u) | (0x3f00u + ((r >> 8) & 0xffu)));
}

static int check(int cond, const char *what) {
    if (!cond) fprintf(stderr, "oracle_sanitize_driver: %s\n", what);
    return cond ? 0 : 1;
}

int main(void) {
    int bad = 0;
    const int shapes[][6] = {   /* B, Hq, Hkv, S, D, causal */
        {1, 1, 1, 1, 4, 1}, {2, 4, 2, 7, 8, 1}, {1, 6, 3, 33, 64, 0}, {1, 2, 1, 40, 128, 1}, {3, 3, 3, 5, 16, 0}};
    for (unsigned c = 0; c < sizeof(shapes) / sizeof(shapes[0]); ++c) {
        const int B = shapes[c][0], Hq = shapes[c][1], Hkv = shapes[c][2], S = shapes[c][3], D = shapes[c][4], causal = shapes[c][5];
        const long nq = (long)B * Hq * S * D, nk = (long)B * Hkv * S * D, nr = (long)B * Hkv * S;
        uint16_t *q = malloc(sizeof(uint16_t) * nq), *k = malloc(sizeof(uint16_t) * nk), *v = malloc(sizeof(uint16_t) * nk);
        int8_t *kc = malloc(nk), *vc = malloc(nk);
        float *ks = malloc(sizeof(float) * nr), *vs = malloc(sizeof(float) * nr);
        double *out = malloc(sizeof(double) * nq), *out8 = malloc(sizeof(double) * nq);
        for (long i = 0; i < nq; ++i) q[i] = random_bf16();
        for (long i = 0; i < nk; ++i) { k[i] = random_bf16(); v[i] = random_bf16(); }
        if (S > 2) {   /* quantiser edge rows: all zero, subnormal, huge */
            memset(k, 0, sizeof(uint16_t) * D);
            for (int d = 0; d < D; ++d) { k[D + d] = (uint16_t)(1 + d % 100); v[D + d] = 0x7f7f; }
        }
        bad += check(oracle_kv_quant_int8(k, kc, ks, nr, D) == 0, "quantiser status (K)");
        bad += check(oracle_kv_quant_int8(v, vc, vs, nr, D) == 0, "quantiser status (V)");
        for (long i = 0; i < nk; ++i) bad += check(kc[i] >= -127 && vc[i] >= -127, "code below -127");
        bad += check(oracle_attn(q, k, v, NULL, NULL, out, B, Hq, Hkv, S, S, D, causal, 0.25, 0, NULL, 0) == 0, "attention status");
        bad += check(oracle_attn(q, kc, vc, ks, vs, out8, B, Hq, Hkv, S, S, D, causal, 0.25, 1, NULL, 0) == 0, "INT8 attention status");
        for (long i = 0; i < nq; ++i) bad += check(isfinite(out[i]) && isfinite(out8[i]), "non-finite output");
        /* a row subset, last and first rows, written to a buffer of exactly its size */
        const int rows[2] = {S - 1, 0};
        double *sub = malloc(sizeof(double) * (long)B * Hq * 2 * D);
        bad += check(oracle_attn(q, k, v, NULL, NULL, sub, B, Hq, Hkv, S, S, D, causal, 0.25, 0, rows, 2) == 0, "row subset status");
        for (int d = 0; d < D; ++d) bad += check(sub[d] == out[(long)(S - 1) * D + d], "row subset differs from the full result");
        /* decode form: one query row against S keys */
        double *dec = malloc(sizeof(double) * (long)B * Hq * D);
        uint16_t *q1 = malloc(sizeof(uint16_t) * (long)B * Hq * D);
        for (long i = 0; i < (long)B * Hq * D; ++i) q1[i] = random_bf16();
        bad += check(oracle_attn(q1, kc, vc, ks, vs, dec, B, Hq, Hkv, 1, S, D, 1, 0.25, 1, NULL, 0) == 0, "decode status");
        /* probabilities of the last row of the last head: sum to one, masked keys zero */
        double *probs = malloc(sizeof(double) * S), *o = malloc(sizeof(double) * D);
        bad += check(oracle_attn_row_probs(q, k, v, NULL, NULL, probs, o, B, Hq, Hkv, S, S, D, causal, 0.25, 0, B - 1, Hq - 1, S / 2) == 0, "row probs status");
        double total = 0.0;
        for (int j = 0; j < S; ++j) total += probs[j];
        bad += check(fabs(total - 1.0) < 1e-12, "probabilities do not sum to one");
        if (causal) for (int j = S / 2 + 1; j < S; ++j) bad += check(probs[j] == 0.0, "masked key with a probability");
        /* bad arguments are refused, not dereferenced */
        bad += check(oracle_attn(NULL, k, v, NULL, NULL, out, B, Hq, Hkv, S, S, D, causal, 0.25, 0, NULL, 0) != 0, "null q accepted");
        bad += check(oracle_attn(q, kc, vc, NULL, NULL, out, B, Hq, Hkv, S, S, D, causal, 0.25, 1, NULL, 0) != 0, "INT8 without scales accepted");
        free(q); free(k); free(v); free(kc); free(vc); free(ks); free(vs); free(out); free(out8); free(sub); free(dec); free(q1); free(probs); free(o);
    }
    long long sweep[3] = {0, 0, 0};
    bad += check(oracle_quant_division_sweep(sweep, 97) == 0 && sweep[2] > 0 && sweep[0] == 0 && sweep[1] == 0, "division sweep");
    bad += check(oracle_num_threads() >= 1, "thread count");
    if (bad == 0) printf("oracle_sanitize_driver: clean\n");
    return bad ? 1 : 0;
}

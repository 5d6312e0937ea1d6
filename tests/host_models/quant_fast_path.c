/* Host model of the quantiser's short route (the row routine in the HIP sources), swept over every input it
 * can meet, against the definition it must reproduce: scale = fl32(amax / 127), code = rint(fl32(x / scale)),
 * IEEE fp32 divisions, ties to even.  Plain C, no GPU: a proof by exhaustion that the GPU tests then confirm on
 * the hardware's own reciprocal.
 *
 * The one thing the host cannot run is v_rcp_f32, documented as accurate to 1 ulp.  The exact reciprocal lies
 * within half an ulp of R = fl32(1 / scale), so every value the instruction may return is one of R - 1 ulp, R,
 * R + 1 ulp; y = x * r is monotone in r, so a decision that holds at the two ends holds in between.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static float bf16_bits_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}
static uint32_t bits_of(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

/* scale by multiply + fma correction against the IEEE quotient, for every bf16 amax in [lo, hi].
 * out[0] = values checked, out[1] = mismatches. */
int model_scale_sweep(float lo, float hi, long *out) {
    long n = 0, bad = 0;
    const float c = 1.0f / 127.0f;
    for (int ab = 1; ab < 0x7f80; ++ab) {
        const float amax = bf16_bits_to_float((uint16_t)ab);
        if (!(amax >= lo && amax <= hi)) continue;
        volatile float want = amax / 127.0f;
        const float q = amax * c;
        const float got = fmaf(fmaf(-q, 127.0f, amax), c, q);
        n++;
        if (bits_of(got) != bits_of(want)) bad++;
    }
    out[0] = n;
    out[1] = bad;
    return 0;
}

/* codes by reciprocal multiply, magic-number rounding and the tie guard, for every bf16 amax in [lo, hi]
 * (every amax_step-th one) and every bf16 0 <= x <= amax, both signs, and the three candidate reciprocals.
 * out[0] = (pair, reciprocal) cases, out[1] = cases the short route accepts, out[2] = accepted cases whose byte
 * differs from the definition's code, out[3] = largest |y - exact quotient| seen, in units of 2^-24. */
int model_code_sweep(float lo, float hi, float guard, int amax_step, long *out) {
    long cases = 0, accepted = 0, bad = 0;
    double worst = 0.0;
    const float magic = 12582912.0f;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : cases, accepted, bad) reduction(max : worst)
    for (int ab = 1; ab < 0x7f80; ab += amax_step) {
        const float amax = bf16_bits_to_float((uint16_t)ab);
        if (!(amax >= lo && amax <= hi)) continue;
        volatile float scale_v = amax / 127.0f;
        const float scale = scale_v;
        volatile float R_v = 1.0f / scale;
        const float R = R_v;
        const float rs[3] = {nextafterf(R, 0.0f), R, nextafterf(R, INFINITY)};
        for (int xb = 0; xb <= ab; ++xb) {
            for (int sign = 0; sign < 2; ++sign) {
                const float x = bf16_bits_to_float((uint16_t)(xb | (sign << 15)));
                volatile float quo_v = x / scale;
                float want = nearbyintf(quo_v);
                if (want > 127.0f) want = 127.0f;
                if (want < -127.0f) want = -127.0f;
                const uint8_t want_byte = (uint8_t)(int8_t)(int)want;
                const double exact = (double)x / (double)scale;
                for (int k = 0; k < 3; ++k) {
                    volatile float y_v = x * rs[k];
                    const float y = y_v;
                    volatile float f_v = y + magic;
                    const float f = f_v;
                    volatile float n_v = f - magic;
                    const float off = fabsf(y - n_v);
                    const double d = fabs((double)y - exact) * 16777216.0;
                    if (d > worst) worst = d;
                    cases++;
                    if (off < 0.5f - guard) {
                        accepted++;
                        if ((uint8_t)(bits_of(f) & 0xffu) != want_byte) bad++;
                    }
                }
            }
        }
    }
    out[0] = cases;
    out[1] = accepted;
    out[2] = bad;
    out[3] = (long)ceil(worst);
    return 0;
}

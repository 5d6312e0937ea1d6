// Shared device helpers for the gfx950 kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slim {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMasked = -1.0e30f;  // finite stand-in for -inf: exp2(kMasked - m) == 0 for any finite m

__device__ __forceinline__ float bf16_bits_to_f32(unsigned int bits16) { return __uint_as_float(bits16 << 16); }

// fp32 -> bf16, round to nearest even (the hardware conversion on gfx950)
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi) {
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(unsigned int, v);
}

// signed byte n of a dword, widened exactly to fp32 (INT8 -> INT32 -> FP32, section 2.2)
template <int N>
__device__ __forceinline__ float i8_to_f32(unsigned int w) {
    return (float)(int)(signed char)(w >> (8 * N));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ s16x4 lds_read_tr16(const uint16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
}

// value of the other 32-lane half of the wave, combined with op: every lane ends with op(lo, hi)
__device__ __forceinline__ float half_max(float x) {
    const unsigned b = __float_as_uint(x);
    const auto sw = __builtin_amdgcn_permlane32_swap(b, b, false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}
__device__ __forceinline__ float half_sum(float x) {
    const unsigned b = __float_as_uint(x);
    const auto sw = __builtin_amdgcn_permlane32_swap(b, b, false, false);
    return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

// max over the LPR (4, 8 or 16) adjacent lanes that hold one row, in every one of them: DPP exchanges inside a
// row of 16 lanes (the two quad permutations, then the mirror of 8 and the mirror of 16 lanes), no LDS traffic
template <int CTRL>
__device__ __forceinline__ float dpp_mov_f32(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
template <int LPR>
__device__ __forceinline__ float row_group_max(float v) {
    static_assert(LPR == 4 || LPR == 8 || LPR == 16, "a row is held by 4, 8 or 16 adjacent lanes");
    v = fmaxf(v, dpp_mov_f32<0xB1>(v));                  // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_mov_f32<0x4E>(v));                  // quad_perm [2,3,0,1]
    if (LPR >= 8) v = fmaxf(v, dpp_mov_f32<0x141>(v));   // row_half_mirror: lane i <-> 7 - i of its 8
    if (LPR >= 16) v = fmaxf(v, dpp_mov_f32<0x140>(v));  // row_mirror: lane i <-> 15 - i of its 16
    return v;
}

// The INT8 quantiser of one K or V row (paper section 2.2), shared by the quantiser kernels and the prefill
// kernel that emits the cache.  The definition is scale = fl32(amax / 127) and code = rint(fl32(x / scale)), both
// IEEE fp32 divisions (one rounding each, denormals kept), ties to even.  An IEEE division is about a dozen vector
// instructions, and a row needs one per value, so the common case takes a shorter route that provably lands on
// the same bits, and everything else takes the divisions themselves:
//   scale: q = amax * fl32(1/127), r = fma(-q, 127, amax), scale = fma(r, fl32(1/127), q).  Equal to the IEEE
//          quotient for every bf16 amax in [kQuantFastLo, kQuantFastHi] (all 2^15 values are checked on the host).
//   code:  with y = x * rcp(scale) (v_rcp_f32: within 1 ulp; the product adds half an ulp; |y| < 128), y lies
//          within 2^-15 of the exact quotient and the IEEE quotient within 2^-17 of it, so unless y is within
//          kQuantTieGuard = 2^-14 of a half-integer both round to the same integer (swept on the host over every
//          bf16 pair and every reciprocal within 1.5 ulp).  That integer is read off
//          y + 1.5 * 2^23, whose low mantissa byte is the code in two's complement (the addition itself rounds to
//          nearest even).  A value closer to a tie, or a row whose scale lies outside the checked range, sends
//          its wave through the divisions.  (|x| <= amax keeps |code| <= 127: the fast path needs no clamp.)
constexpr float kQuantFastLo = 0x1p-60f, kQuantFastHi = 0x1p60f;   // rows with amax in this range take the fast scale and codes
constexpr float kQuantTieGuard = 0x1p-14f;
constexpr float kQuantMagic = 12582912.0f;   // 1.5 * 2^23

// One row: this lane's 8 values (of the LPR lanes that hold the row) -> its 8 codes and the row's scale.
template <int LPR>
__device__ __forceinline__ void quant_row_piece(const u32x4 raw, u32x2& out2, float& scale) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = bf16_bits_to_f32(raw[i] & 0xffffu);
        v[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
    }
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[i]));
    amax = row_group_max<LPR>(amax);
    const bool in_range = amax >= kQuantFastLo && amax <= kQuantFastHi;
    constexpr float kInv127 = 1.0f / 127.0f;
    const float q127 = amax * kInv127;
    scale = fmaf(fmaf(-q127, 127.0f, amax), kInv127, q127);
    const float inv = __builtin_amdgcn_rcpf(scale);
    unsigned int bits[8];
    float off_int = 0.0f;   // largest distance of a y from its nearest integer
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float y = v[i] * inv;
        const float f = y + kQuantMagic;
        off_int = fmaxf(off_int, fabsf(y - (f - kQuantMagic)));
        bits[i] = __float_as_uint(f);
    }
    // byte 0 of four words -> one word
    out2[0] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(bits[3], bits[2], 0x0c0c0400u),
                                    __builtin_amdgcn_perm(bits[1], bits[0], 0x0c0c0400u), 0x05040100u);
    out2[1] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(bits[7], bits[6], 0x0c0c0400u),
                                    __builtin_amdgcn_perm(bits[5], bits[4], 0x0c0c0400u), 0x05040100u);
    const bool fast_ok = in_range && off_int < 0.5f - kQuantTieGuard;   // (false as well when anything is NaN)
    if (__builtin_amdgcn_ballot_w64(!fast_ok) != 0) {
        // the definition itself, for every lane of the wave (lanes that were fine get the same bits again)
        scale = amax / 127.0f;   // IEEE division, one rounding
        unsigned int packed[2] = {0u, 0u};
        if (amax != 0.0f) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float r = rintf(v[i] / scale);   // IEEE division, then ties-to-even
                r = fminf(fmaxf(r, -127.0f), 127.0f);
                packed[i / 4] |= ((unsigned int)(int)r & 0xffu) << (8 * (i % 4));
            }
        }
        out2[0] = packed[0];
        out2[1] = packed[1];
    }
}

}  // namespace slim

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

// The INT8 quantiser of one K or V row (paper section 2.2), shared by the quantiser kernels and the prefill
// kernel that emits the cache: scale = amax / 127 and code = rint(x / scale) with IEEE fp32 divisions.
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
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
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

}  // namespace slim

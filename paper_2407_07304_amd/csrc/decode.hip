// Decode attention over the INT8 KV cache (paper section 2.2: next-token attention is a
// matrix-vector product bound by memory bandwidth; cached INT8 values are widened to FP32
// in registers and fed to FMAs, with one scale per token per head).
//
// HBM-bound streaming kernel.  A workgroup of 4 waves covers kTokensPerSplit consecutive
// tokens of one (batch, query head); every wave streams 256 of them:
//   - a token row of D codes is read by D/16 adjacent lanes with one 128-bit load each,
//     so one load instruction of a wave fetches 64/(D/16) whole rows;
//   - each such group of lanes ("slot") owns a run of consecutive tokens, which keeps its
//     per-token scales contiguous (staged once per wave through LDS);
//   - pass 1 computes the wave's scores, pass 2 takes one max for the wave and the
//     probabilities, pass 3 streams V with the probability (times the V scale) as the
//     only multiplier, so nothing is rescaled inside a wave;
//   - the 4 waves are merged in LDS, and a second kernel merges the splits in a fixed
//     order (no atomics: the result does not depend on workgroup arrival order).
#include "slim_common.h"
#include "slim_kernels.h"

namespace slim {

constexpr int kDecodeWaves = 4;
constexpr int kTokensPerWave = 256;
constexpr int kTokensPerSplit = kDecodeWaves * kTokensPerWave;

template <int D>
__global__ __launch_bounds__(256) void slim_decode_int8_split_kernel(
    const uint16_t* __restrict__ q, const int8_t* __restrict__ kc, const float* __restrict__ ks,
    const int8_t* __restrict__ vc, const float* __restrict__ vs, uint16_t* __restrict__ out,
    float* __restrict__ ws_acc, float* __restrict__ ws_ml, int Hq, int Hkv, int T, int n_split, float scale_log2e) {
    constexpr int LPR = D / 16;             // lanes per token row
    constexpr int SLOTS = 64 / LPR;         // token rows per load instruction of a wave
    constexpr int NI = kTokensPerWave / SLOTS;  // consecutive tokens per slot

    __shared__ float scaleS[kDecodeWaves][2][kTokensPerWave];
    __shared__ float accS[kDecodeWaves][SLOTS][D];
    __shared__ float lS[kDecodeWaves][SLOTS];
    __shared__ float mS[kDecodeWaves];

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int c = lane % LPR, s = lane / LPR;
    const int sp = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int g = h / (Hq / Hkv);
    const long kvbase = ((long)b * Hkv + g) * (long)T;
    const int8_t* kp = kc + kvbase * D + c * 16;
    const int8_t* vp = vc + kvbase * D + c * 16;
    const int t_wave0 = sp * kTokensPerSplit + w * kTokensPerWave;

    // this lane's 16 query values, fp32
    float qf[16];
    {
        const uint16_t* qp = q + ((long)b * Hq + h) * D + c * 16;
        const u32x4 q0 = *reinterpret_cast<const u32x4*>(qp);
        const u32x4 q1 = *reinterpret_cast<const u32x4*>(qp + 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            qf[2 * i] = bf16_bits_to_f32(q0[i] & 0xffffu);
            qf[2 * i + 1] = __uint_as_float(q0[i] & 0xffff0000u);
            qf[8 + 2 * i] = bf16_bits_to_f32(q1[i] & 0xffffu);
            qf[8 + 2 * i + 1] = __uint_as_float(q1[i] & 0xffff0000u);
        }
    }

    // the wave's 256 K scales and V scales, coalesced, through LDS
#pragma unroll
    for (int j = 0; j < kTokensPerWave / 64; ++j) {
        const int t = min(t_wave0 + lane + 64 * j, T - 1);
        scaleS[w][0][lane + 64 * j] = ks[kvbase + t];
        scaleS[w][1][lane + 64 * j] = vs[kvbase + t];
    }
    __syncthreads();

    const int t_slot0 = t_wave0 + s * NI;

    // pass 1: scores (in log2 units)
    float sc[NI];
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int t = t_slot0 + it;
        const u32x4 kw = *reinterpret_cast<const u32x4*>(kp + (long)min(t, T - 1) * D);
        float dot = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dot = fmaf(qf[4 * i + 0], i8_to_f32<0>(kw[i]), dot);
            dot = fmaf(qf[4 * i + 1], i8_to_f32<1>(kw[i]), dot);
            dot = fmaf(qf[4 * i + 2], i8_to_f32<2>(kw[i]), dot);
            dot = fmaf(qf[4 * i + 3], i8_to_f32<3>(kw[i]), dot);
        }
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) dot += __shfl_xor(dot, off);
        sc[it] = (t < T) ? dot * (scaleS[w][0][s * NI + it] * scale_log2e) : kMasked;
    }

    // pass 2: one max for the wave, probabilities, the slot's sum
    float m = sc[0];
#pragma unroll
    for (int it = 1; it < NI; ++it) m = fmaxf(m, sc[it]);
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) m = fmaxf(m, __shfl_xor(m, off));
    float l = 0.0f;
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        float p = fast_exp2(sc[it] - m);
        p = (t_slot0 + it < T) ? p : 0.0f;
        l += p;
        sc[it] = p * scaleS[w][1][s * NI + it];   // probability times the token's V scale
    }

    // pass 3: acc[d] += p * v_scale * code
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int t = t_slot0 + it;
        const u32x4 vw = *reinterpret_cast<const u32x4*>(vp + (long)min(t, T - 1) * D);
        const float pv = sc[it];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[4 * i + 0] = fmaf(pv, i8_to_f32<0>(vw[i]), acc[4 * i + 0]);
            acc[4 * i + 1] = fmaf(pv, i8_to_f32<1>(vw[i]), acc[4 * i + 1]);
            acc[4 * i + 2] = fmaf(pv, i8_to_f32<2>(vw[i]), acc[4 * i + 2]);
            acc[4 * i + 3] = fmaf(pv, i8_to_f32<3>(vw[i]), acc[4 * i + 3]);
        }
    }

    // merge slots and waves in LDS
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f32x4 a4 = {acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]};
        *reinterpret_cast<f32x4*>(&accS[w][s][c * 16 + 4 * i]) = a4;
    }
    if (c == 0) lS[w][s] = l;
    if (lane == 0) mS[w] = m;
    __syncthreads();
    if (threadIdx.x < D) {
        const int d = threadIdx.x;
        float M = mS[0];
#pragma unroll
        for (int ww = 1; ww < kDecodeWaves; ++ww) M = fmaxf(M, mS[ww]);
        float L = 0.0f, o = 0.0f;
#pragma unroll
        for (int ww = 0; ww < kDecodeWaves; ++ww) {
            const float f = fast_exp2(mS[ww] - M);   // a wave past the end has m = kMasked -> f = 0
            float lw = 0.0f, ow = 0.0f;
#pragma unroll
            for (int ss = 0; ss < SLOTS; ++ss) {
                lw += lS[ww][ss];
                ow += accS[ww][ss][d];
            }
            L = fmaf(f, lw, L);
            o = fmaf(f, ow, o);
        }
        const long bh = (long)b * Hq + h;
        if (n_split == 1) {
            out[bh * D + d] = (uint16_t)(pack_bf16x2(o / L, 0.0f) & 0xffffu);
        } else {
            const long idx = bh * n_split + sp;
            ws_acc[idx * D + d] = o;
            if (d == 0) {
                ws_ml[idx * 2] = M;
                ws_ml[idx * 2 + 1] = L;
            }
        }
    }
}

// Merges the n_split partial (max, sum, accumulator) triples of one (batch, head) in
// split order and writes the bf16 output row.
template <int D>
__global__ __launch_bounds__(D) void slim_decode_combine_kernel(const float* __restrict__ ws_acc,
                                                                const float* __restrict__ ws_ml,
                                                                uint16_t* __restrict__ out, int n_split) {
    const long bh = blockIdx.x;
    const int d = threadIdx.x;
    float M = kMasked;
    for (int sp = 0; sp < n_split; ++sp) M = fmaxf(M, ws_ml[(bh * n_split + sp) * 2]);
    float L = 0.0f, o = 0.0f;
    for (int sp = 0; sp < n_split; ++sp) {
        const long idx = bh * n_split + sp;
        const float f = fast_exp2(ws_ml[idx * 2] - M);
        L = fmaf(f, ws_ml[idx * 2 + 1], L);
        o = fmaf(f, ws_acc[idx * D + d], o);
    }
    out[bh * D + d] = (uint16_t)(pack_bf16x2(o / L, 0.0f) & 0xffffu);
}

int decode_tokens_per_split(int) { return kTokensPerSplit; }

int decode_num_splits(int kv_len, int) { return (kv_len + kTokensPerSplit - 1) / kTokensPerSplit; }

size_t decode_workspace_bytes(int batch, int q_heads, int kv_len, int head_dim) {
    const size_t n = (size_t)batch * q_heads * decode_num_splits(kv_len, head_dim);
    return n * ((size_t)head_dim + 2) * sizeof(float);
}

hipError_t launch_decode(const DecodeArgs& a, hipStream_t stream) {
    const int n_split = decode_num_splits(a.kv_len, a.head_dim);
    const size_t n_part = (size_t)a.batch * a.q_heads * n_split;
    float* ws_acc = a.workspace;
    float* ws_ml = a.workspace + n_part * a.head_dim;
    const float scale_log2e = a.softmax_scale * kLog2e;
    dim3 grid((unsigned)n_split, (unsigned)a.q_heads, (unsigned)a.batch);
    if (a.head_dim == 128)
        hipLaunchKernelGGL(slim_decode_int8_split_kernel<128>, grid, dim3(256), 0, stream, (const uint16_t*)a.q,
                           a.k_codes, a.k_scale, a.v_codes, a.v_scale, (uint16_t*)a.out, ws_acc, ws_ml, a.q_heads,
                           a.kv_heads, a.kv_len, n_split, scale_log2e);
    else
        hipLaunchKernelGGL(slim_decode_int8_split_kernel<64>, grid, dim3(256), 0, stream, (const uint16_t*)a.q,
                           a.k_codes, a.k_scale, a.v_codes, a.v_scale, (uint16_t*)a.out, ws_acc, ws_ml, a.q_heads,
                           a.kv_heads, a.kv_len, n_split, scale_log2e);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_split == 1) return e;
    const unsigned nbh = (unsigned)(a.batch * a.q_heads);
    if (a.head_dim == 128)
        hipLaunchKernelGGL(slim_decode_combine_kernel<128>, dim3(nbh), dim3(128), 0, stream, ws_acc, ws_ml,
                           (uint16_t*)a.out, n_split);
    else
        hipLaunchKernelGGL(slim_decode_combine_kernel<64>, dim3(nbh), dim3(64), 0, stream, ws_acc, ws_ml,
                           (uint16_t*)a.out, n_split);
    return hipGetLastError();
}

}  // namespace slim

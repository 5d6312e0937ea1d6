// Decode attention over the INT8 KV cache (paper section 2.2: next-token attention is a
// matrix-vector product bound by memory bandwidth; cached INT8 values are widened to FP32
// in registers and fed to FMAs, with one scale per token per head).
//
// HBM-bound streaming kernel.  A workgroup of 4 waves serves one (batch, query head) and
// one split of the key axis; every wave streams a contiguous run of tokens in chunks of
// 64 tokens:
//   - a token row of D codes is read by D/16 adjacent lanes ("slot") with one 128-bit
//     load each, so one load instruction of a wave fetches 64/(D/16) whole rows, and the
//     wave's loads of a chunk cover one contiguous piece of K and one of V;
//   - the K and V loads of chunk c+1 are issued before chunk c is consumed, so a wave
//     always has a chunk of 128-bit loads in flight;
//   - lane i of the wave owns token i of the chunk: it loads that token's two scales
//     (coalesced), keeps its score, and computes ONE exponential per chunk;
//   - each slot carries its own running max / sum (online softmax, fp32), so the only
//     cross-lane traffic in the loop is DPP adds inside a slot and a 256-byte LDS
//     exchange of the chunk's probabilities;
//   - slots and waves are merged in LDS at the end, and a second kernel merges the splits
//     in a fixed order (no atomics: the result does not depend on arrival order).
#include <mutex>
#include <type_traits>

#include "slim_common.h"
#include "slim_kernels.h"

namespace slim {

constexpr int kDecodeWaves = 4;
constexpr int kChunk = 64;   // tokens per wave per chunk
typedef float f32x2 __attribute__((ext_vector_type(2)));

// lane exchange inside a slot via DPP (no LDS traffic); every lane of the slot ends with the slot total
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
template <int LPR>
__device__ __forceinline__ float slot_sum(float v) {
    v += dpp_f32<0xB1>(v);                 // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E>(v);                 // quad_perm [2,3,0,1]
    if (LPR == 8) v += dpp_f32<0x141>(v);  // row_half_mirror: the other quad of the 8 lanes
    return v;
}
template <int LPR>
__device__ __forceinline__ float slot_max(float v) {
    v = fmaxf(v, dpp_f32<0xB1>(v));
    v = fmaxf(v, dpp_f32<0x4E>(v));
    if (LPR == 8) v = fmaxf(v, dpp_f32<0x141>(v));
    return v;
}

template <int D>
__global__ __launch_bounds__(256) void slim_decode_int8_split_kernel(
    const uint16_t* __restrict__ q, const int8_t* __restrict__ kc, const float* __restrict__ ks,
    const int8_t* __restrict__ vc, const float* __restrict__ vs, uint16_t* __restrict__ out,
    float* __restrict__ ws_acc, float* __restrict__ ws_ml, const int* __restrict__ kv_lens, int Hq, int Hkv, int T_alloc,
    int n_split, int tokens_per_wave, float scale_log2e) {
    constexpr int LPR = D / 16;        // lanes per token row
    constexpr int SLOTS = 64 / LPR;    // token rows per load instruction of a wave
    constexpr int CH = LPR;            // rows per slot per chunk: SLOTS * CH == kChunk, one token per lane

    __shared__ __attribute__((aligned(16))) float pvS[kDecodeWaves][kChunk];
    __shared__ __attribute__((aligned(16))) float accS[kDecodeWaves][SLOTS][D];
    __shared__ float lS[kDecodeWaves][SLOTS];
    __shared__ float mS[kDecodeWaves][SLOTS];

    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // (the wave index as a scalar: everything derived from it stays uniform)
    const int c = lane % LPR, s = lane / LPR;
    const int sp = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int g = h / (Hq / Hkv);
    // T_alloc is the cache's allocated length (the row stride); this sequence's first T tokens count
    const int T = kv_lens ? min(max(kv_lens[b], 1), T_alloc) : T_alloc;
    const long kvbase = ((long)b * Hkv + g) * (long)T_alloc;
    // Buffer descriptors over exactly this (batch, KV head)'s first T tokens: a row past the end reads as zeros (and
    // is masked below), an address is one 32-bit offset per lane plus a constant per row, and the descriptors live in
    // scalar registers (with pointers and clamped row indices the addresses of a chunk's loads took some eighty
    // vector instructions and a dozen more vector registers).
    const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc((void*)(kc + kvbase * D), 0, (int)((unsigned)T * D), 0x00020000);
    const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc((void*)(vc + kvbase * D), 0, (int)((unsigned)T * D), 0x00020000);
    const __amdgpu_buffer_rsrc_t ksr = __builtin_amdgcn_make_buffer_rsrc((void*)(ks + kvbase), 0, (int)((unsigned)T * 4u), 0x00020000);
    const __amdgpu_buffer_rsrc_t vsr = __builtin_amdgcn_make_buffer_rsrc((void*)(vs + kvbase), 0, (int)((unsigned)T * 4u), 0x00020000);
    const int lane_off = (s * CH) * D + c * 16;   // this lane's piece of its slot's first row, relative to the chunk
    const int t_wave0 = (sp * kDecodeWaves + w) * tokens_per_wave;
    const int t_wave_end = min(T, t_wave0 + tokens_per_wave);
    const int n_chunks = t_wave0 < T ? (t_wave_end - t_wave0 + kChunk - 1) / kChunk : 0;

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

    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
    float m = kMasked, l = 0.0f;   // slot max (identical in the slot's lanes), this lane's part of the slot sum

    u32x4 kbuf[CH], vbuf[CH];
    float ksc = 0.0f, vsc = 0.0f;
    // the codes are read once per step, so their loads are non-temporal (measured: 5.6 -> 6.3 TB/s on the B=16,
    // T=8192 cache)
    auto issue_k = [&](int t_chunk0) {
        const int off = t_chunk0 * D + lane_off;
#pragma unroll
        for (int it = 0; it < CH; ++it) kbuf[it] = __builtin_amdgcn_raw_buffer_load_b128(krs, off + it * D, 0, 2 /* nt */);
        ksc = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ksr, (t_chunk0 + lane) * 4, 0, 0));
    };
    auto issue_v = [&](int t_chunk0) {
        const int off = t_chunk0 * D + lane_off;
        // (the scale first: it is wanted before the codes, and loads complete in order, so a wait for a scale
        // issued after the codes would be a wait for the codes)
        vsc = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(vsr, (t_chunk0 + lane) * 4, 0, 0));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int it = 0; it < CH; ++it) vbuf[it] = __builtin_amdgcn_raw_buffer_load_b128(vrs, off + it * D, 0, 2 /* nt */);
    };

    // unconditional (a wave past the end gets zeros and reads nothing): keeps the prologue free of branches
    issue_k(t_wave0);
    issue_v(t_wave0);
    // one chunk; PREFETCH is a compile-time flag so the loop body has no branch around its loads
    auto chunk = [&](int ch, auto prefetch) {
        constexpr bool more = decltype(prefetch)::value;
        const int t_chunk0 = t_wave0 + ch * kChunk;

        // scores: the slot's CH rows; lane c of the slot keeps row c (token t_chunk0 + lane)
        float my_dot = 0.0f;
#pragma unroll
        for (int it = 0; it < CH; ++it) {
            const u32x4 kw = kbuf[it];
            float dot = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                dot = fmaf(qf[4 * i + 0], i8_to_f32<0>(kw[i]), dot);
                dot = fmaf(qf[4 * i + 1], i8_to_f32<1>(kw[i]), dot);
                dot = fmaf(qf[4 * i + 2], i8_to_f32<2>(kw[i]), dot);
                dot = fmaf(qf[4 * i + 3], i8_to_f32<3>(kw[i]), dot);
            }
            dot = slot_sum<LPR>(dot);
            my_dot = (c == it) ? dot : my_dot;
        }
        const bool valid = t_chunk0 + lane < T;
        const float my_s = valid ? my_dot * (ksc * scale_log2e) : kMasked;
        if constexpr (more) issue_k(t_chunk0 + kChunk);

        const float m_new = fmaxf(m, slot_max<LPR>(my_s));
        const float alpha = fast_exp2(m - m_new);
        float p = fast_exp2(my_s - m_new);
        p = valid ? p : 0.0f;
        l = fmaf(l, alpha, p);
        pvS[w][lane] = p * vsc;   // probability times the token's V scale
        if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] *= alpha;
        }
        m = m_new;

        float pv[CH];
#pragma unroll
        for (int i = 0; i < CH / 4; ++i) {
            const f32x4 t4 = *reinterpret_cast<const f32x4*>(&pvS[w][s * CH + 4 * i]);
            pv[4 * i] = t4[0];
            pv[4 * i + 1] = t4[1];
            pv[4 * i + 2] = t4[2];
            pv[4 * i + 3] = t4[3];
        }
#pragma unroll
        for (int it = 0; it < CH; ++it) {
            const u32x4 vw = vbuf[it];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[4 * i + 0] = fmaf(pv[it], i8_to_f32<0>(vw[i]), acc[4 * i + 0]);
                acc[4 * i + 1] = fmaf(pv[it], i8_to_f32<1>(vw[i]), acc[4 * i + 1]);
                acc[4 * i + 2] = fmaf(pv[it], i8_to_f32<2>(vw[i]), acc[4 * i + 2]);
                acc[4 * i + 3] = fmaf(pv[it], i8_to_f32<3>(vw[i]), acc[4 * i + 3]);
            }
        }
        if constexpr (more) issue_v(t_chunk0 + kChunk);
    };
    for (int ch = 0; ch + 1 < n_chunks; ++ch) chunk(ch, std::true_type{});
    if (n_chunks > 0) chunk(n_chunks - 1, std::false_type{});

    // merge slots and waves in LDS
    l = slot_sum<LPR>(l);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f32x4 a4 = {acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]};
        *reinterpret_cast<f32x4*>(&accS[w][s][c * 16 + 4 * i]) = a4;
    }
    if (c == 0) {
        lS[w][s] = l;
        mS[w][s] = m;
    }
    __syncthreads();
    if (threadIdx.x < D) {
        const int d = threadIdx.x;
        float M = kMasked;
#pragma unroll
        for (int ww = 0; ww < kDecodeWaves; ++ww)
#pragma unroll
            for (int ss = 0; ss < SLOTS; ++ss) M = fmaxf(M, mS[ww][ss]);
        float L = 0.0f, o = 0.0f;
#pragma unroll
        for (int ww = 0; ww < kDecodeWaves; ++ww)
#pragma unroll
            for (int ss = 0; ss < SLOTS; ++ss) {
                const float f = fast_exp2(mS[ww][ss] - M);   // an empty slot has l = 0 and acc = 0
                L = fmaf(f, lS[ww][ss], L);
                o = fmaf(f, accS[ww][ss][d], o);
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

// Merges the n_split partial (max, sum, accumulator) triples of one (batch, head) in split order and writes the
// bf16 output row.  The launch is latency-bound (a few kilobytes per workgroup, just written by the split kernel),
// so all loads of up to kCombineChunk splits are issued before anything is computed: one round trip to memory
// instead of one for the maxima and another for the sums and accumulators.  More splits than that (short batches of
// long caches) are merged a chunk at a time with a running (max, sum, accumulator), still in split order.  Slots
// past the last split re-read the last one and count as empty (max = kMasked, sum = 0).
constexpr int kCombineChunk = 16;

template <int D>
__global__ __launch_bounds__(D) void slim_decode_combine_kernel(const float* __restrict__ ws_acc,
                                                                const float* __restrict__ ws_ml,
                                                                uint16_t* __restrict__ out, int n_split) {
    constexpr int CH = kCombineChunk;
    const long bh = blockIdx.x;
    const int d = threadIdx.x;
    const float* const ml = ws_ml + bh * n_split * 2;
    const float* const acc = ws_acc + bh * n_split * D + d;
    float M = kMasked, L = 0.0f, o = 0.0f;
    for (int s0 = 0; s0 < n_split; s0 += CH) {
        float m[CH], l[CH], a[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int sp = min(s0 + i, n_split - 1);
            const bool there = s0 + i < n_split;
            const f32x2 t = *reinterpret_cast<const f32x2*>(ml + 2 * sp);
            const float av = acc[(long)sp * D];
            m[i] = there ? t[0] : kMasked;
            l[i] = there ? t[1] : 0.0f;
            a[i] = there ? av : 0.0f;
        }
        float m_new = M;
#pragma unroll
        for (int i = 0; i < CH; ++i) m_new = fmaxf(m_new, m[i]);
        const float keep = fast_exp2(M - m_new);   // first chunk: L = o = 0, whatever this is
        L *= keep;
        o *= keep;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const float f = fast_exp2(m[i] - m_new);   // an empty split has sum = 0 and accumulator = 0
            L = fmaf(f, l[i], L);
            o = fmaf(f, a[i], o);
        }
        M = m_new;
    }
    out[bh * D + d] = (uint16_t)(pack_bf16x2(o / L, 0.0f) & 0xffffu);
}

constexpr int kTokensPerWave = 512;   // 8 chunks: measured flat from 512 to 2048 on a B=16, T=8192 cache

// Tokens of the key axis one wave streams: a multiple of the 64-token chunk.  Long
// enough to amortise the merge; shortened when (batch x heads) alone cannot fill the
// chip (aim: at least ~4 workgroups per compute unit) or when the cache is short.
int decode_tokens_per_wave(int kv_len, long n_bh) {
    long tpw = kTokensPerWave;
    const long want_blocks = 256L * 4;
    const long fill = (long)kv_len * n_bh / (want_blocks * kDecodeWaves);   // tokens per wave that give want_blocks
    if (tpw > fill) tpw = fill;
    tpw = tpw / kChunk * kChunk;
    if (tpw < kChunk) tpw = kChunk;
    return (int)tpw;
}

int decode_num_splits(int kv_len, long n_bh) {
    const int per_block = decode_tokens_per_wave(kv_len, n_bh) * kDecodeWaves;
    return (kv_len + per_block - 1) / per_block;
}

bool decode_uses_gqa_kernel(int q_heads, int kv_heads) {
    const int G = q_heads / kv_heads;
    return G >= 2 && G <= 32;
}

size_t decode_workspace_bytes(int batch, int q_heads, int kv_heads, int kv_len, int head_dim) {
    const int n_split = decode_uses_gqa_kernel(q_heads, kv_heads) ? decode_gqa_num_splits(kv_len, (long)batch * kv_heads)
                                                                  : decode_num_splits(kv_len, (long)batch * q_heads);
    const size_t n = (size_t)batch * q_heads * n_split;
    return n * ((size_t)head_dim + 2) * sizeof(float);
}

// Scratch of the decode entry point that may not allocate: the same (max, sum, accumulator) partials as the
// caller-owned workspace, in one array per GPU that lives as long as the process.  In host code the array's
// name only stands for the symbol: its device address is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[kDecodeStaticScratchBytes];

hipError_t decode_static_scratch(float** ptr) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* per_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (per_device[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // this device's copy of the array
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = static_cast<float*>(per_device[dev]);
    return hipSuccess;
}

hipError_t launch_decode(const DecodeArgs& a, hipStream_t stream) {
    if (decode_uses_gqa_kernel(a.q_heads, a.kv_heads)) {
        // the query heads of a KV head share one pass over its cache; every wave's token run is a split
        const int n_split = decode_gqa_num_splits(a.kv_len, (long)a.batch * a.kv_heads);
        const size_t n_part = (size_t)a.batch * a.q_heads * n_split;
        float* ws_acc = a.workspace;
        float* ws_ml = a.workspace + n_part * a.head_dim;
        hipError_t e = launch_decode_gqa_split(a, ws_acc, ws_ml, n_split, stream);
        if (e != hipSuccess) return e;
        const unsigned nbh = (unsigned)(a.batch * a.q_heads);
        if (a.head_dim == 128)
            hipLaunchKernelGGL(slim_decode_combine_kernel<128>, dim3(nbh), dim3(128), 0, stream, ws_acc, ws_ml,
                               (uint16_t*)a.out, n_split);
        else
            hipLaunchKernelGGL(slim_decode_combine_kernel<64>, dim3(nbh), dim3(64), 0, stream, ws_acc, ws_ml,
                               (uint16_t*)a.out, n_split);
        return hipGetLastError();
    }
    const long n_bh = (long)a.batch * a.q_heads;
    const int tpw = decode_tokens_per_wave(a.kv_len, n_bh);
    const int n_split = decode_num_splits(a.kv_len, n_bh);
    const size_t n_part = (size_t)a.batch * a.q_heads * n_split;
    float* ws_acc = a.workspace;
    float* ws_ml = a.workspace + n_part * a.head_dim;
    const float scale_log2e = a.softmax_scale * kLog2e;
    dim3 grid((unsigned)n_split, (unsigned)a.q_heads, (unsigned)a.batch);
    if (a.head_dim == 128)
        hipLaunchKernelGGL(slim_decode_int8_split_kernel<128>, grid, dim3(256), 0, stream, (const uint16_t*)a.q,
                           a.k_codes, a.k_scale, a.v_codes, a.v_scale, (uint16_t*)a.out, ws_acc, ws_ml, a.kv_lens,
                           a.q_heads, a.kv_heads, a.kv_len, n_split, tpw, scale_log2e);
    else
        hipLaunchKernelGGL(slim_decode_int8_split_kernel<64>, grid, dim3(256), 0, stream, (const uint16_t*)a.q,
                           a.k_codes, a.k_scale, a.v_codes, a.v_scale, (uint16_t*)a.out, ws_acc, ws_ml, a.kv_lens,
                           a.q_heads, a.kv_heads, a.kv_len, n_split, tpw, scale_log2e);
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

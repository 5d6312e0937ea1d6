// Prefill attention (paper section 2.1): one workgroup owns a block of query rows and the
// whole softmax direction; K/V stream through it in tiles while an fp32 running max and
// sum keep the softmax exact.  INT8 K/V (section 2.2) are widened exactly to bf16 while
// being staged; their per-token scales multiply the fp32 score column (K) and the
// probability before it is rounded to bf16 (V), so dequantisation adds no rounding.
//
// Mapping on gfx950 (wave64, v_mfma_f32_32x32x16_bf16):
//   - 4 waves per workgroup, 32 query rows per wave, 128 rows per workgroup.
//   - The score tile is computed transposed, S^T = K Q^T: the K tile is the A operand
//     (from LDS), Q^T the B operand (held in registers for the whole kernel).  In the
//     result every lane holds ONE query column and 16 of the 32 keys, so the row max and
//     row sum are in-lane reductions plus one exchange between lanes l and l+32.
//   - The same registers, rounded to bf16, are directly the B operand of
//     O^T += V^T P^T; V^T comes from the row-major V tile in LDS through the LDS
//     transpose read (ds_read_b64_tr_b16), so V is never transposed in memory.
//   - O^T accumulators: lane = query column, so the online-softmax rescale is a per-lane
//     scalar multiply.
#include "slim_common.h"
#include "slim_kernels.h"

namespace slim {

constexpr int kBR = 128;   // query rows per workgroup
constexpr int kBC = 64;    // keys per staged tile
constexpr int kPrefillThreads = 256;

struct PrefillParams {
    const uint16_t* q;
    const void* k;
    const void* v;
    const float* ks;
    const float* vs;
    void* out;
    int Hq, Hkv, S, causal, n_rb, total, chunk;
    float scale_log2e;
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ s16x4 lds_read_tr16(const uint16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
}

template <int D, bool KV_I8, bool OUT_F32>
__global__ __launch_bounds__(kPrefillThreads) void slim_prefill_kernel(const PrefillParams p) {
    constexpr int KS = D / 16;      // k-steps of the score MFMA
    constexpr int DT = D / 32;      // 32-row tiles of O^T
    constexpr int LDK = D + 8;      // LDS row stride in bf16 elements (16 B of padding)
    constexpr int NCH = KV_I8 ? (kBC * D / 16 / kPrefillThreads) : (kBC * D / 8 / kPrefillThreads);  // 16-byte chunks per thread per tile
    constexpr int CPR = KV_I8 ? (D / 16) : (D / 8);   // chunks per row

    __shared__ __attribute__((aligned(16))) uint16_t Ks[kBC * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[kBC * LDK];
    __shared__ __attribute__((aligned(16))) float ksS[kBC];
    __shared__ __attribute__((aligned(16))) float vsS[kBC];

    // workgroup -> (batch*head, row block): consecutive virtual ids share K/V and are sent
    // to the same XCD (hardware deals workgroup ids round-robin over the 8 XCDs); within a
    // head the long (late) row blocks go first.
    const int n = blockIdx.x;
    const int vid = (n % 8) * p.chunk + n / 8;
    if (vid >= p.total) return;
    const int bh = vid / p.n_rb;
    const int rb = p.n_rb - 1 - (vid % p.n_rb);
    const int b = bh / p.Hq, h = bh % p.Hq;
    const int g = h / (p.Hq / p.Hkv);
    const int S = p.S;
    const int i0 = rb * kBR;

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
    const int my_q = i0 + 32 * w + l32;          // this lane's query row (may be >= S in the last block)
    const int wave_q_lo = i0 + 32 * w, wave_q_hi = wave_q_lo + 31;

    // Q^T B-operands: lane holds row my_q, d = 16 s + 8 hh + [0,8)
    bf16x8 qreg[KS];
    {
        const uint16_t* qp = p.q + (((long)b * p.Hq + h) * S + min(my_q, S - 1)) * (long)D + 8 * hh;
#pragma unroll
        for (int s = 0; s < KS; ++s) qreg[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
    }

    const long kvrow0 = ((long)b * p.Hkv + g) * (long)S;
    const int kend = p.causal ? min(S, i0 + kBR) : S;
    const int n_tiles = (kend + kBC - 1) / kBC;

    u32x4 kst[NCH], vst[NCH];
    float sst = 0.0f;
    auto load_tile = [&](int j0) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int cidx = tid + kPrefillThreads * i;
            const int row = cidx / CPR, col = cidx % CPR;
            const long grow = kvrow0 + min(j0 + row, S - 1);
            if (KV_I8) {
                kst[i] = *reinterpret_cast<const u32x4*>((const int8_t*)p.k + grow * D + col * 16);
                vst[i] = *reinterpret_cast<const u32x4*>((const int8_t*)p.v + grow * D + col * 16);
            } else {
                kst[i] = *reinterpret_cast<const u32x4*>((const uint16_t*)p.k + grow * D + col * 8);
                vst[i] = *reinterpret_cast<const u32x4*>((const uint16_t*)p.v + grow * D + col * 8);
            }
        }
        if (KV_I8) {
            if (tid < kBC) sst = p.ks[kvrow0 + min(j0 + tid, S - 1)];
            else if (tid < 2 * kBC) sst = p.vs[kvrow0 + min(j0 + tid - kBC, S - 1)];
        }
    };
    auto widen16 = [&](const u32x4 cw, uint16_t* dst) {   // 16 INT8 codes -> 16 bf16 (exact)
        u32x4 lo, hi;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            lo[2 * i] = pack_bf16x2(i8_to_f32<0>(cw[i]), i8_to_f32<1>(cw[i]));
            lo[2 * i + 1] = pack_bf16x2(i8_to_f32<2>(cw[i]), i8_to_f32<3>(cw[i]));
            hi[2 * i] = pack_bf16x2(i8_to_f32<0>(cw[2 + i]), i8_to_f32<1>(cw[2 + i]));
            hi[2 * i + 1] = pack_bf16x2(i8_to_f32<2>(cw[2 + i]), i8_to_f32<3>(cw[2 + i]));
        }
        *reinterpret_cast<u32x4*>(dst) = lo;
        *reinterpret_cast<u32x4*>(dst + 8) = hi;
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int cidx = tid + kPrefillThreads * i;
            const int row = cidx / CPR, col = cidx % CPR;
            if (KV_I8) {
                widen16(kst[i], &Ks[row * LDK + col * 16]);
                widen16(vst[i], &Vs[row * LDK + col * 16]);
            } else {
                *reinterpret_cast<u32x4*>(&Ks[row * LDK + col * 8]) = kst[i];
                *reinterpret_cast<u32x4*>(&Vs[row * LDK + col * 8]) = vst[i];
            }
        }
        if (KV_I8) {
            if (tid < kBC) ksS[tid] = sst * p.scale_log2e;
            else if (tid < 2 * kBC) vsS[tid - kBC] = sst;
        }
    };

    f32x16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;
    float m = kMasked, lsum = 0.0f;

    load_tile(0);
    for (int j = 0; j < n_tiles; ++j) {
        const int j0 = j * kBC;
        __syncthreads();   // every wave has finished reading the previous tile
        store_tile();
        __syncthreads();
        if (j + 1 < n_tiles) load_tile(j0 + kBC);   // in flight while this tile is computed

#pragma unroll
        for (int kt = 0; kt < kBC / 32; ++kt) {
            const int key0 = j0 + 32 * kt;
            if (key0 >= S) continue;                          // wave-uniform
            if (p.causal && key0 > wave_q_hi) continue;       // whole sub-tile above the diagonal for this wave

            // S^T[key][query] = sum_d K[key][d] Q[query][d]
            f32x16 st;
#pragma unroll
            for (int r = 0; r < 16; ++r) st[r] = 0.0f;
            const uint16_t* ka = &Ks[(32 * kt + l32) * LDK + 8 * hh];
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(ka + 16 * s);
                st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[s], st, 0, 0, 0);
            }

            // register r of this lane is key  key0 + 8 (r/4) + 4 hh + r%4
            float t[16];
            if (KV_I8) {
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 kf = *reinterpret_cast<const f32x4*>(&ksS[32 * kt + 8 * r4 + 4 * hh]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[4 * r4 + e] = st[4 * r4 + e] * kf[e];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) t[r] = st[r] * p.scale_log2e;
            }
            const bool need_mask = (p.causal && key0 + 31 > wave_q_lo) || (key0 + 32 > S);
            if (need_mask) {
                const int lim = p.causal ? min(my_q, S - 1) : S - 1;   // last visible key
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key0 + 8 * (r / 4) + 4 * hh + (r % 4);
                    t[r] = (key <= lim) ? t[r] : kMasked;
                }
            }
            float mloc = t[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mloc = fmaxf(mloc, t[r]);
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
            const float m_new = fmaxf(m, mloc);
            const float alpha = fast_exp2(m - m_new);
            float psum = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                t[r] = fast_exp2(t[r] - m_new);
                psum += t[r];
            }
            lsum = fmaf(lsum, alpha, psum);
            if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {   // rescale only when some row's max moved
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
            }
            m = m_new;
            if (KV_I8) {
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 vf = *reinterpret_cast<const f32x4*>(&vsS[32 * kt + 8 * r4 + 4 * hh]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[4 * r4 + e] *= vf[e];
                }
            }

            // O^T[d][query] += sum_key V[key][d] P[query][key]; k-step u covers registers 8u..8u+7,
            // i.e. keys key0 + 16u + {4hh..4hh+3} and key0 + 16u + 8 + {4hh..4hh+3}
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                u32x4 pw;
#pragma unroll
                for (int i = 0; i < 4; ++i) pw[i] = pack_bf16x2(t[8 * u + 2 * i], t[8 * u + 2 * i + 1]);
                const bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
                // transpose read: the 16 lanes of a group fetch rows k..k+3 (4 lanes per row, 4 columns
                // each) and lane i of the group receives column i of those 4 rows
                const uint16_t* va = &Vs[(32 * kt + 16 * u + 4 * hh + (l & 15) / 4) * LDK + 16 * ((l >> 4) & 1) + 4 * (l & 3)];
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const s16x4 lo = lds_read_tr16(va + 32 * dt);
                    const s16x4 hi = lds_read_tr16(va + 8 * LDK + 32 * dt);
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb, o[dt], 0, 0, 0);
                }
            }
        }
    }

    // epilogue: O = O^T / l ; register r of tile dt is d = 32 dt + 8 (r/4) + 4 hh + r%4
    const float ltot = lsum + __shfl_xor(lsum, 32);
    const float inv = 1.0f / ltot;
    if (my_q < S) {
        const long orow = (((long)b * p.Hq + h) * S + my_q) * (long)D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d = 32 * dt + 8 * r4 + 4 * hh;
                const float x0 = o[dt][4 * r4] * inv, x1 = o[dt][4 * r4 + 1] * inv;
                const float x2 = o[dt][4 * r4 + 2] * inv, x3 = o[dt][4 * r4 + 3] * inv;
                if (OUT_F32) {
                    f32x4 ov = {x0, x1, x2, x3};
                    *reinterpret_cast<f32x4*>((float*)p.out + orow + d) = ov;
                } else {
                    u32x2 ov;
                    ov[0] = pack_bf16x2(x0, x1);
                    ov[1] = pack_bf16x2(x2, x3);
                    *reinterpret_cast<u32x2*>((uint16_t*)p.out + orow + d) = ov;
                }
            }
    }
}

template <int D, bool KV_I8, bool OUT_F32>
static hipError_t launch_one(const PrefillParams& p, hipStream_t stream) {
    hipLaunchKernelGGL((slim_prefill_kernel<D, KV_I8, OUT_F32>), dim3((unsigned)(8 * p.chunk)), dim3(kPrefillThreads), 0,
                       stream, p);
    return hipGetLastError();
}

hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream) {
    PrefillParams p;
    p.q = (const uint16_t*)a.q;
    p.k = a.k;
    p.v = a.v;
    p.ks = a.k_scale;
    p.vs = a.v_scale;
    p.out = a.out;
    p.Hq = a.q_heads;
    p.Hkv = a.kv_heads;
    p.S = a.seq_len;
    p.causal = a.causal ? 1 : 0;
    p.n_rb = (a.seq_len + kBR - 1) / kBR;
    p.total = a.batch * a.q_heads * p.n_rb;
    p.chunk = (p.total + 7) / 8;
    p.scale_log2e = a.softmax_scale * kLog2e;
    const int sel = (a.head_dim == 128 ? 4 : 0) | (a.kv_int8 ? 2 : 0) | (a.out_f32 ? 1 : 0);
    switch (sel) {
        case 0: return launch_one<64, false, false>(p, stream);
        case 1: return launch_one<64, false, true>(p, stream);
        case 2: return launch_one<64, true, false>(p, stream);
        case 3: return launch_one<64, true, true>(p, stream);
        case 4: return launch_one<128, false, false>(p, stream);
        case 5: return launch_one<128, false, true>(p, stream);
        case 6: return launch_one<128, true, false>(p, stream);
        default: return launch_one<128, true, true>(p, stream);
    }
}

}  // namespace slim

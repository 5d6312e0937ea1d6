// Prefill attention (paper section 2.1): one work item owns a block of query rows and the
// whole softmax direction; K/V stream through it in 32-key steps while an fp32 running max
// and sum keep the softmax exact.  INT8 K/V (section 2.2) are widened exactly to bf16 while
// being staged; their per-token scales multiply the fp32 score column (K) and the
// probability before it is rounded to bf16 (V), so dequantisation adds no rounding.
//
// Mapping on gfx950 (wave64, v_mfma_f32_32x32x16_bf16):
//   - 4 waves per workgroup, 32 query rows per wave, 128 rows per row block.  Under the
//     causal mask a workgroup takes the row-block pair (n-1-x, x) one after the other, so
//     every workgroup does the same amount of work.
//   - The score tile is computed transposed, S^T = K Q^T: the K tile is the A operand
//     (from LDS), Q^T the B operand (held in registers for the whole pass).  In the
//     result every lane holds ONE query column and 16 of the 32 keys, so the row max and
//     row sum are in-lane reductions plus one exchange between lanes l and l+32.
//   - The same registers, rounded to bf16, are directly the B operand of
//     O^T += V^T P^T; V^T comes from the row-major V tile in LDS through the LDS
//     transpose read (ds_read_b64_tr_b16), so V is never transposed in memory.
//   - O^T accumulators: lane = query column, so the online-softmax rescale is a per-lane
//     scalar multiply, skipped while no row's max moves.
//   - Software pipeline: the score MFMAs of step k+1 are issued before the softmax of
//     step k, so the matrix pipe works while the vector ALU does the exponentials; a
//     three-deep LDS ring is filled through registers one step ahead, one barrier per step.
#include <type_traits>

#include "slim_common.h"
#include "slim_kernels.h"

namespace slim {

constexpr int kBR = 128;   // query rows per row block (4 waves x 32)
constexpr int kBC = 32;    // keys per step
constexpr int kNS = 3;     // LDS ring depth
constexpr int kPrefillThreads = 256;

struct PrefillParams {
    const uint16_t* q;
    const void* k;
    const void* v;
    const float* ks;
    const float* vs;
    void* out;
    int Hq, Hkv, S, causal, n_rb, n_pair, total, chunk;
    int single, local_heads, per_xcd;   // single != 0: one row block per workgroup (small grids)
    float scale_log2e;
};

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

template <int D, bool KV_I8, bool OUT_F32>
__global__ __launch_bounds__(kPrefillThreads, 1) void slim_prefill_kernel(const PrefillParams p) {
    constexpr int KS = D / 16;       // k-steps of the score MFMA
    constexpr int DT = D / 32;       // 32-row tiles of O^T
    constexpr int LDKK = D + 8;      // K rows: 16 B of padding, conflict-free 128-bit row reads
    constexpr int LDKV = D + 32;     // V rows: 64 B of padding, conflict-free transpose reads
    constexpr int CPR = KV_I8 ? D / 16 : D / 8;                  // 16-byte chunks per row
    constexpr int NCHUNK = kBC * CPR;                            // chunks per step and tensor
    constexpr int NCH = (NCHUNK + kPrefillThreads - 1) / kPrefillThreads;

    __shared__ __attribute__((aligned(16))) uint16_t Ks[kNS][kBC * LDKK];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[kNS][kBC * LDKV];
    __shared__ __attribute__((aligned(16))) float scS[kNS][2 * kBC];   // INT8: [0,32) k_scale*c, [32,64) v_scale

    // workgroup -> (batch*head, row-block pair).  Hardware deals workgroup ids round-robin over the 8
    // XCDs, so consecutive virtual ids (which share K/V) are steered to one XCD.
    // Small grids (fewer pairs than two workgroups per compute unit) run one row block per workgroup
    // instead: inside an XCD the hardware fills its 32 compute units once before any gets a second
    // workgroup, so the local index j is laid out as a snake over rows of 32 through the heavy-first
    // list, and the two workgroups that share a compute unit carry a long and a short row block.
    int bh, x, rb_single = 0;
    {
        const int n = blockIdx.x;
        if (p.single) {
            const int xcd = n % 8, j = n / 8;
            if (j >= p.per_xcd) return;
            const int r = j / 32, cpos = j % 32;
            const int row_len = min(32, p.per_xcd - r * 32);
            const int rank = r * 32 + ((r & 1) ? row_len - 1 - cpos : cpos);
            rb_single = p.n_rb - 1 - rank / p.local_heads;
            bh = xcd * p.local_heads + rank % p.local_heads;
            x = 0;
        } else {
            const int vid = (n % 8) * p.chunk + n / 8;
            if (vid >= p.total) return;
            bh = vid / p.n_pair;
            x = vid % p.n_pair;
        }
    }
    const int b = bh / p.Hq, h = bh % p.Hq;
    const int g = h / (p.Hq / p.Hkv);
    const int S = p.S;
    const float c = p.scale_log2e;

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l32 = l & 31, hh = l >> 5;
    const long kvrow0 = ((long)b * p.Hkv + g) * (long)S;

    // ---- staging: global -> registers (one step ahead) -> LDS ring
    // Addresses: a uniform base (this head's K / V slab) plus a 32-bit per-thread offset, so the loads
    // take the scalar-base form; the LDS destinations are a per-thread constant plus the ring slot.
    constexpr int ROWB = KV_I8 ? D : 2 * D;   // bytes per K/V row in memory
    const char* kslab = (const char*)p.k + kvrow0 * ROWB;
    const char* vslab = (const char*)p.v + kvrow0 * ROWB;
    const float* ksslab = KV_I8 ? p.ks + kvrow0 : nullptr;
    const float* vsslab = KV_I8 ? p.vs + kvrow0 : nullptr;
    int st_row[NCH], st_colb[NCH], st_kdst[NCH], st_vdst[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int cidx = tid + kPrefillThreads * i;
        st_row[i] = cidx / CPR;
        st_colb[i] = (cidx % CPR) * 16;
        st_kdst[i] = st_row[i] * LDKK + (cidx % CPR) * (KV_I8 ? 16 : 8);
        st_vdst[i] = st_row[i] * LDKV + (cidx % CPR) * (KV_I8 ? 16 : 8);
    }
    u32x4 kst[NCH], vst[NCH];
    float sst = 0.0f;
    auto load_step = [&](int s) {
        const int j0 = s * kBC;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            if (NCHUNK % kPrefillThreads == 0 || tid + kPrefillThreads * i < NCHUNK) {
                // rows past the end of the sequence: clamped here, masked in the softmax
                const unsigned off = (unsigned)min(j0 + st_row[i], S - 1) * (unsigned)ROWB + (unsigned)st_colb[i];
                kst[i] = *reinterpret_cast<const u32x4*>(kslab + off);
                vst[i] = *reinterpret_cast<const u32x4*>(vslab + off);
            }
        }
        if (KV_I8) {
            if (tid < kBC) sst = ksslab[min(j0 + tid, S - 1)];
            else if (tid < 2 * kBC) sst = vsslab[min(j0 + tid - kBC, S - 1)];
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
    auto store_step = [&](int buf) {
        uint16_t* kdst = &Ks[0][0] + buf * (kBC * LDKK);
        uint16_t* vdst = &Vs[0][0] + buf * (kBC * LDKV);
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            if (NCHUNK % kPrefillThreads == 0 || tid + kPrefillThreads * i < NCHUNK) {
                if (KV_I8) {
                    widen16(kst[i], kdst + st_kdst[i]);
                    widen16(vst[i], vdst + st_vdst[i]);
                } else {
                    *reinterpret_cast<u32x4*>(kdst + st_kdst[i]) = kst[i];
                    *reinterpret_cast<u32x4*>(vdst + st_vdst[i]) = vst[i];
                }
            }
        }
        if (KV_I8) {
            if (tid < kBC) scS[buf][tid] = sst * c;
            else if (tid < 2 * kBC) scS[buf][tid] = sst;
        }
    };

    bf16x8 qreg[KS];
    f32x16 o[DT];
    const int ka_off = l32 * LDKK + 8 * hh;                                              // K fragment (row l32)
    const int va_off = (4 * hh + (l & 15) / 4) * LDKV + 16 * ((l >> 4) & 1) + 4 * (l & 3);   // V transpose read

    // S^T[key][query] = sum_d K[key][d] Q[query][d] for the 32 keys of a step
    auto score = [&](int buf) {
        f32x16 st;
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = 0.0f;
        const uint16_t* ka = &Ks[0][0] + buf * (kBC * LDKK) + ka_off;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(ka + 16 * s);
            st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[s], st, 0, 0, 0);
        }
        return st;
    };

    for (int pass = 0; pass < (p.single ? 1 : 2); ++pass) {
        const int rb = p.single ? rb_single : (pass == 0 ? p.n_rb - 1 - x : x);
        if (pass == 1 && rb == p.n_rb - 1 - x) break;   // the middle row block of an odd count
        const int i0 = rb * kBR;
        const int my_q = i0 + 32 * w + l32;             // this lane's query row (may be >= S in the last block)
        const int wave_q_lo = i0 + 32 * w;
        const int kend = p.causal ? min(S, i0 + kBR) : S;
        const int n_steps = (kend + kBC - 1) / kBC;
        // last step this wave computes: its diagonal step under the causal mask; none if it has no row
        const int wave_last = wave_q_lo >= S ? -1 : (p.causal ? min(n_steps - 1, wave_q_lo / kBC) : n_steps - 1);
        const int lim = p.causal ? min(my_q, S - 1) : S - 1;   // last key this lane's row may see

        // Q^T B-operands: lane holds row my_q, d = 16 s + 8 hh + [0,8)
        {
            const uint16_t* qp = p.q + (((long)b * p.Hq + h) * S + min(my_q, S - 1)) * (long)D + 8 * hh;
#pragma unroll
            for (int s = 0; s < KS; ++s) qreg[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;
        float m = kMasked, lsum = 0.0f;   // bf16 K/V: m in raw score units; INT8: in scaled (log2) units

        // prologue: steps 0 and 1 into the ring, step 2 into registers
        __syncthreads();   // the previous pass has finished reading the ring
        // (the three loads are issued together, so the pass pays one memory latency, not three)
        {
            u32x4 k0[NCH], v0[NCH], k1[NCH], v1[NCH];
            float s0 = 0.0f, s1 = 0.0f;
            load_step(0);
#pragma unroll
            for (int i = 0; i < NCH; ++i) { k0[i] = kst[i]; v0[i] = vst[i]; }
            s0 = sst;
            load_step(min(1, n_steps - 1));
#pragma unroll
            for (int i = 0; i < NCH; ++i) { k1[i] = kst[i]; v1[i] = vst[i]; }
            s1 = sst;
            load_step(min(2, n_steps - 1));
            u32x4 k2[NCH], v2[NCH];
            const float s2 = sst;
#pragma unroll
            for (int i = 0; i < NCH; ++i) { k2[i] = kst[i]; v2[i] = vst[i]; }
#pragma unroll
            for (int i = 0; i < NCH; ++i) { kst[i] = k0[i]; vst[i] = v0[i]; }
            sst = s0;
            store_step(0);
#pragma unroll
            for (int i = 0; i < NCH; ++i) { kst[i] = k1[i]; vst[i] = v1[i]; }
            sst = s1;
            store_step(1);
#pragma unroll
            for (int i = 0; i < NCH; ++i) { kst[i] = k2[i]; vst[i] = v2[i]; }
            sst = s2;
        }
        __syncthreads();
        // Steady-state step k of this wave (k is below its diagonal, no mask).  The instruction order is
        // fixed by hand (sched_barrier) for a wave that runs alone on its SIMD:
        //   K fragments of step k+1  ->  row max / alpha of step k  ->  score MFMAs of step k+1, each
        //   followed by a slice of step k's exponentials  ->  ring traffic  ->  P V MFMAs of step k with
        //   the V fragment reads between them.
        auto steady_step = [&](int k, int buf, f32x16& st_cur, f32x16& st_nxt) {
            constexpr int EPM = 16 / KS;   // exponentials issued after each score MFMA
            const int nbuf = buf == kNS - 1 ? 0 : buf + 1;
            const int wbuf = nbuf == kNS - 1 ? 0 : nbuf + 1;
            bf16x8 kfr[KS];
            {
                const uint16_t* ka = &Ks[0][0] + nbuf * (kBC * LDKK) + ka_off;
#pragma unroll
                for (int s = 0; s < KS; ++s) kfr[s] = *reinterpret_cast<const bf16x8*>(ka + 16 * s);
            }
            float t[16];
            if (KV_I8) {
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 kf = *reinterpret_cast<const f32x4*>(&scS[buf][8 * r4 + 4 * hh]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[4 * r4 + e] = st_cur[4 * r4 + e] * kf[e];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) t[r] = st_cur[r];
            }
            float mloc = fmaxf(t[0], t[1]);
#pragma unroll
            for (int r = 2; r < 16; r += 2) mloc = fmaxf(mloc, fmaxf(t[r], t[r + 1]));
            // lazy running max: it only moves when some row's max grew by more than 2^8, so the
            // probabilities stay below 256 and the accumulator is rescaled a few times per row block
            const float cand = fmaxf(m, half_max(mloc));
            const float jump = KV_I8 ? cand - m : (cand - m) * c;
            if (__builtin_amdgcn_ballot_w64(jump > 8.0f) != 0) {
                const float alpha = fast_exp2(KV_I8 ? m - cand : (m - cand) * c);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
                lsum *= alpha;
                m = cand;
            }
            const float mc = KV_I8 ? m : m * c;
            __builtin_amdgcn_sched_barrier(0);

            const uint16_t* va = &Vs[0][0] + buf * (kBC * LDKV) + va_off;
            s16x4 vlo[DT], vhi[DT];
            float ps = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) st_nxt[r] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                st_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[s], qreg[s], st_nxt, 0, 0, 0);
#pragma unroll
                for (int e = s * EPM; e < (s + 1) * EPM; ++e) {
                    t[e] = KV_I8 ? fast_exp2(t[e] - mc) : fast_exp2(fmaf(t[e], c, -mc));
                    ps += t[e];
                }
                if (s == KS / 2) {   // V fragments of the first 16 keys, in flight under the remaining exponentials
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        vlo[dt] = lds_read_tr16(va + 32 * dt);
                        vhi[dt] = lds_read_tr16(va + 8 * LDKV + 32 * dt);
                    }
                }
            }
            lsum += ps;
            if (KV_I8) {
                // the probabilities take their token's v_scale before they are rounded to bf16
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 vf = *reinterpret_cast<const f32x4*>(&scS[buf][kBC + 8 * r4 + 4 * hh]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[4 * r4 + e] *= vf[e];
                }
            }
            u32x4 pw[2];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) pw[u][i] = pack_bf16x2(t[8 * u + 2 * i], t[8 * u + 2 * i + 1]);
            // ring: registers (step k+2) -> LDS, then fetch step k+3 into registers
            store_step(wbuf);
            load_step(min(k + 3, n_steps - 1));

            // O^T[d][query] += sum_key V[key][d] P[query][key]; k-step u covers registers 8u..8u+7,
            // i.e. keys 16u + {4hh..4hh+3} and 16u + 8 + {4hh..4hh+3} of the step
            s16x4 wlo[DT], whi[DT];
            const bf16x8 pb0 = __builtin_bit_cast(bf16x8, pw[0]);
            const bf16x8 pb1 = __builtin_bit_cast(bf16x8, pw[1]);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                wlo[dt] = lds_read_tr16(va + 16 * LDKV + 32 * dt);
                whi[dt] = lds_read_tr16(va + 24 * LDKV + 32 * dt);
                const s16x8 av = {vlo[dt][0], vlo[dt][1], vlo[dt][2], vlo[dt][3], vhi[dt][0], vhi[dt][1], vhi[dt][2], vhi[dt][3]};
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb0, o[dt], 0, 0, 0);
            }
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const s16x8 av = {wlo[dt][0], wlo[dt][1], wlo[dt][2], wlo[dt][3], whi[dt][0], whi[dt][1], whi[dt][2], whi[dt][3]};
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb1, o[dt], 0, 0, 0);
            }
            // instruction pipeline of the region above (one scheduling region): every score MFMA is followed
            // by a slice of the exponentials, the ring traffic sits between the two MFMA runs, and the
            // second half of the V fragments is read under the first P V MFMAs
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, (KV_I8 ? 4 : 3) * EPM + 1, 0);   // its share of the softmax VALU work
                if (s == KS / 2) __builtin_amdgcn_sched_group_barrier(0x100, 2 * DT, 0);   // V fragments, first 16 keys
            }
            __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);    // row sum, packing
            __builtin_amdgcn_sched_group_barrier(0x200, 2 * NCH * (KV_I8 ? 2 : 1), 0);   // ring: LDS writes
            __builtin_amdgcn_sched_group_barrier(0x020, 2 * NCH, 0);                       // ring: global loads
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, DT, 0);
            __syncthreads();
        };
        // The wave's last step (its diagonal under the causal mask, or the tail of the key axis): masked,
        // nothing to issue ahead.
        auto last_step = [&](int k, int buf, f32x16& st_cur) {
            const int wbuf = buf == 0 ? kNS - 1 : buf - 1;   // (buf + 2) mod 3
            const int key0 = k * kBC;
            // register r of this lane is key  key0 + 8 (r/4) + 4 hh + r%4
            float t[16];
            if (KV_I8) {
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 kf = *reinterpret_cast<const f32x4*>(&scS[buf][8 * r4 + 4 * hh]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[4 * r4 + e] = st_cur[4 * r4 + e] * kf[e];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) t[r] = st_cur[r];
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + 8 * (r / 4) + 4 * hh + (r % 4);
                t[r] = (key <= lim) ? t[r] : kMasked;
            }
            float mloc = fmaxf(t[0], t[1]);
#pragma unroll
            for (int r = 2; r < 16; r += 2) mloc = fmaxf(mloc, fmaxf(t[r], t[r + 1]));
            const float m_new = fmaxf(m, half_max(mloc));
            const float alpha = KV_I8 ? fast_exp2(m - m_new) : fast_exp2((m - m_new) * c);
            const float mc = KV_I8 ? m_new : m_new * c;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
            m = m_new;
            float ps = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                t[r] = KV_I8 ? fast_exp2(t[r] - mc) : fast_exp2(fmaf(t[r], c, -mc));
                ps += t[r];
            }
            lsum = fmaf(lsum, alpha, ps);
            if (KV_I8) {
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 vf = *reinterpret_cast<const f32x4*>(&scS[buf][kBC + 8 * r4 + 4 * hh]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[4 * r4 + e] *= vf[e];
                }
            }
            u32x4 pw[2];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) pw[u][i] = pack_bf16x2(t[8 * u + 2 * i], t[8 * u + 2 * i + 1]);
            store_step(wbuf);
            load_step(min(k + 3, n_steps - 1));
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const bf16x8 pb = __builtin_bit_cast(bf16x8, pw[u]);
                // transpose read: the 16 lanes of a group fetch rows k..k+3 (4 lanes per row, 4 columns
                // each) and lane i of the group receives column i of those 4 rows
                const uint16_t* va = &Vs[0][0] + buf * (kBC * LDKV) + va_off + 16 * u * LDKV;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const s16x4 lo = lds_read_tr16(va + 32 * dt);
                    const s16x4 hi = lds_read_tr16(va + 8 * LDKV + 32 * dt);
                    const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb, o[dt], 0, 0, 0);
                }
            }
            __syncthreads();
        };
        // one step for this wave, whatever its role in it
        auto do_step = [&](int k, int buf, f32x16& st_cur, f32x16& st_nxt) {
            if (k < wave_last) {
                steady_step(k, buf, st_cur, st_nxt);
            } else if (k == wave_last) {
                last_step(k, buf, st_cur);
            } else {   // past this wave's diagonal: keep the ring and the barriers going
                store_step(buf == 0 ? kNS - 1 : buf - 1);
                load_step(min(k + 3, n_steps - 1));
                __syncthreads();
            }
        };

        f32x16 st_a, st_b;
#pragma unroll
        for (int r = 0; r < 16; ++r) st_a[r] = st_b[r] = 0.0f;
        if (wave_last >= 0) st_a = score(0);
        int buf = 0;
        for (int k = 0; k < n_steps; k += 2) {
            do_step(k, buf, st_a, st_b);
            buf = buf == kNS - 1 ? 0 : buf + 1;
            if (k + 1 < n_steps) do_step(k + 1, buf, st_b, st_a);
            buf = buf == kNS - 1 ? 0 : buf + 1;
        }

        // epilogue: O = O^T / l ; register r of tile dt is d = 32 dt + 8 (r/4) + 4 hh + r%4
        const float inv = 1.0f / half_sum(lsum);
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
}

template <int D, bool KV_I8, bool OUT_F32>
static hipError_t launch_one(const PrefillParams& p, hipStream_t stream) {
    const unsigned grid = (unsigned)(8 * (p.single ? p.per_xcd : p.chunk));
    hipLaunchKernelGGL((slim_prefill_kernel<D, KV_I8, OUT_F32>), dim3(grid), dim3(kPrefillThreads), 0,
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
    p.n_pair = (p.n_rb + 1) / 2;
    p.total = a.batch * a.q_heads * p.n_pair;
    p.chunk = (p.total + 7) / 8;
    // fewer pairs than two workgroups per compute unit (256 CUs): one row block per workgroup
    const int n_bh = a.batch * a.q_heads;
    p.single = (p.causal && n_bh % 8 == 0 && p.n_rb > 1 && p.total < 512) ? 1 : 0;
    p.local_heads = n_bh / 8;
    p.per_xcd = p.local_heads * p.n_rb;
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

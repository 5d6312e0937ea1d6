// Decode attention over the INT8 KV cache when several query heads share a KV head (paper
// section 2.2 for the cache; section 2.1 names MHA and GQA side by side).  The cache is
// the bandwidth: every byte of it is read once per KV head here, not once per query head.
//
// With G query heads per KV head the step is a (G x D) by (D x T) product followed by a
// (G x T) by (T x D) one: dense enough for the matrix cores.  One wave streams a run of
// tokens of one (batch, KV head) in 32-token tiles and serves all G heads at once:
//   - K and V tiles are read with coalesced 128-bit loads (a load instruction of a wave
//     covers whole rows), widened exactly to bf16 and written to a wave-private LDS tile
//     each.  No other wave touches them: no barriers, LDS runs a wave's accesses in order.
//   - scores, transposed: S^T = K Q^T with v_mfma_f32_32x32x16_bf16, the K tile as A operand
//     (lane = token, 128-bit LDS reads), Q^T as B operand (held in registers, columns = the
//     G heads, the rest zero).
//   - every lane then holds one head's column and 16 of the 32 tokens: the token's
//     k_scale multiplies the fp32 score, max and sum are in-lane plus one exchange between
//     the wave's halves, the probability takes the token's v_scale before it is rounded
//     to bf16 and is the B operand of O^T += V^T P^T as it stands; V^T comes from the
//     row-major V tile through the LDS transpose read.
//   - two tiles of loads are in flight per wave: the registers of a tile are refilled with
//     the tile after the next as soon as they are consumed.
// Each wave writes its (max, sum, accumulator) per head as one split of the workspace; the
// combine kernel of decode.hip merges the splits in fixed order.
#include <type_traits>

#include "slim_common.h"
#include "slim_kernels.h"

namespace slim {

constexpr int kGqaWaves = 2;    // waves per workgroup, each with a token run of its own (the waves share nothing: on B=16, 64/8 heads,
                                // T=8192 two-wave workgroups run 8 % faster than four-wave ones with the same runs, one-wave ones the same)
constexpr int kGqaTile = 32;    // tokens per tile

// 16 INT8 codes -> 16 bf16, exact: the first and the second eight
__device__ __forceinline__ void widen16(const u32x4 cw, u32x4& lo, u32x4& hi) {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        lo[2 * e] = pack_bf16x2(i8_to_f32<0>(cw[e]), i8_to_f32<1>(cw[e]));
        lo[2 * e + 1] = pack_bf16x2(i8_to_f32<2>(cw[e]), i8_to_f32<3>(cw[e]));
        hi[2 * e] = pack_bf16x2(i8_to_f32<0>(cw[2 + e]), i8_to_f32<1>(cw[2 + e]));
        hi[2 * e + 1] = pack_bf16x2(i8_to_f32<2>(cw[2 + e]), i8_to_f32<3>(cw[2 + e]));
    }
}

// TRAFFIC_ONLY: the measurement form of the kernel (include/slimprobe.h): the same workgroups, waves, token runs and
// loads, issued at the same points, but a tile's registers are only XORed together before they are refilled.  What it
// takes is what the memory system charges for this access pattern on this shape, arithmetic aside.
template <int D, bool TRAFFIC_ONLY = false>
__global__ __launch_bounds__(64 * kGqaWaves) void slim_decode_int8_gqa_kernel(
    const uint16_t* __restrict__ q, const int8_t* __restrict__ kc, const float* __restrict__ ks,
    const int8_t* __restrict__ vc, const float* __restrict__ vs, float* __restrict__ ws_acc,
    float* __restrict__ ws_ml, const int* __restrict__ kv_lens, int Hq, int Hkv, int T_alloc, int n_split,
    int tokens_per_wave, float scale_log2e) {
    constexpr int KS = D / 16;            // k-steps of the score MFMA
    constexpr int DT = D / 32;            // 32-row tiles of O^T
    constexpr int CPR = D / 16;           // 16-byte pieces per row
    constexpr int NP = kGqaTile * CPR / 64;   // 128-bit loads per lane, tile and tensor
    // LDS row pitches of the bf16 tiles: the padding spreads the 128-bit K row reads and the V transpose reads over the banks
    constexpr int ROWLK = 2 * D + 16, ROWLV = 2 * D + 64;
    constexpr int TILEK = kGqaTile * ROWLK, TILEV = kGqaTile * ROWLV;
    // one tile buffer per wave: the K tile, and once its fragments are read (LDS runs a wave's accesses in order)
    // the V tile; then the tile's 32 + 32 scales
    constexpr int WAVE_LDS = (TILEK > TILEV ? TILEK : TILEV) + 256;

    __shared__ __attribute__((aligned(16))) char smem[kGqaWaves * WAVE_LDS];

    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // (the wave index as a scalar: everything derived from it stays uniform)
    const int l32 = lane & 31, hh = lane >> 5;
    const int G = Hq / Hkv;
    const int sp = blockIdx.x * kGqaWaves + w, g = blockIdx.y, b = blockIdx.z;
    char* const kS = smem + w * WAVE_LDS;
    char* const vS = kS;
    float* const scS = reinterpret_cast<float*>(kS + WAVE_LDS - 256);   // [0,32) k_scale * c, [32,64) v_scale

    // T_alloc is the cache's allocated length (the row stride); this sequence's first T tokens count
    const int T = kv_lens ? min(max(kv_lens[b], 1), T_alloc) : T_alloc;
    const long kvrow0 = ((long)b * Hkv + g) * (long)T_alloc;
    const int t_begin = sp * tokens_per_wave;
    const int t_end = min(T, t_begin + tokens_per_wave);
    const int n_tiles = t_begin < T ? (t_end - t_begin + kGqaTile - 1) / kGqaTile : 0;

    // Q^T B operands: lane holds head l32 (of the group), d = 16 s + 8 hh + [0,8)
    bf16x8 qB[KS];
    {
        const uint16_t* qp = q + ((long)b * Hq + (long)g * G + min(l32, G - 1)) * D + 8 * hh;
#pragma unroll
        for (int s2 = 0; s2 < KS; ++s2) {
            u32x4 a = *reinterpret_cast<const u32x4*>(qp + 16 * s2);
            if (l32 >= G) a = u32x4{0u, 0u, 0u, 0u};
            qB[s2] = __builtin_bit_cast(bf16x8, a);
        }
    }

    // Piece lane + 64 n of a tile (row-major, 16 codes each), through buffer descriptors that cover exactly this
    // (batch, KV head)'s slab: rows past the end of the cache read as zero (and are masked) and a load costs one
    // vector add.  The codes are used once: non-temporal.  Two tiles of
    // loads are in flight per wave (the registers of tile i are refilled with tile i+2 as soon as they are
    // consumed): with 8 waves per compute unit that is what it takes to cover the memory latency.
    const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc((void*)(kc + kvrow0 * D), 0, (int)((unsigned)T * D), 0x00020000);
    const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc((void*)(vc + kvrow0 * D), 0, (int)((unsigned)T * D), 0x00020000);
    // (the scales through descriptors as well: lanes 0-31 want the K scale of token l32, lanes 32-63 the V scale; each
    // load asks the other half's lanes for an offset past the end, which reads nothing, so a tile's loads are the
    // same instructions whether the tile is wanted or not)
    const __amdgpu_buffer_rsrc_t ksr = __builtin_amdgcn_make_buffer_rsrc((void*)(ks + kvrow0), 0, (int)((unsigned)T * 4u), 0x00020000);
    const __amdgpu_buffer_rsrc_t vsr = __builtin_amdgcn_make_buffer_rsrc((void*)(vs + kvrow0), 0, (int)((unsigned)T * 4u), 0x00020000);
    const int s_off_k = hh == 0 ? l32 * 4 : (int)0x7ffffff0, s_off_v = hh == 1 ? l32 * 4 : (int)0x7ffffff0;
    int p_off[NP];
#pragma unroll
    for (int n = 0; n < NP; ++n) p_off[n] = ((lane + 64 * n) / CPR) * D + ((lane + 64 * n) % CPR) * 16;
    u32x4 kbuf[2][NP], vbuf[2][NP];
    float sc[2] = {0.0f, 0.0f};
    auto issue = [&](auto par, const __amdgpu_buffer_rsrc_t rs, u32x4 (&buf)[2][NP], int t0) {
        constexpr int P = decltype(par)::value;
#pragma unroll
        for (int n = 0; n < NP; ++n) buf[P][n] = __builtin_amdgcn_raw_buffer_load_b128(rs, p_off[n] + t0 * D, 0, 2 /* nt */);
    };
    auto issue_k = [&](auto par, int t0) {
        issue(par, krs, kbuf, t0);
        const uint32_t a = __builtin_amdgcn_raw_buffer_load_b32(ksr, s_off_k + t0 * 4, 0, 0);
        const uint32_t c = __builtin_amdgcn_raw_buffer_load_b32(vsr, s_off_v + t0 * 4, 0, 0);
        sc[decltype(par)::value] = __builtin_bit_cast(float, a | c);   // (the lanes a load left out received zero)
    };
    auto issue_v = [&](auto par, int t0) { issue(par, vrs, vbuf, t0); };
    auto stage = [&](auto par, const u32x4 (&buf)[2][NP], char* tile, int pitch) {   // widen a tile into LDS
        constexpr int P = decltype(par)::value;
#pragma unroll
        for (int n = 0; n < NP; ++n) {
            const int pid = lane + 64 * n;
            u32x4 lo, hi;
            widen16(buf[P][n], lo, hi);
            char* dst = tile + (pid / CPR) * pitch + (pid % CPR) * 32;
            *reinterpret_cast<u32x4*>(dst) = lo;
            *reinterpret_cast<u32x4*>(dst + 16) = hi;
        }
    };
    const int k_addr = l32 * ROWLK + 16 * hh;   // K fragment of k-step s: row l32, bytes 32 s + 16 hh + [0,16)
    // LDS addresses of the V transpose reads: the 16 lanes of a group fetch rows k..k+3 (4 lanes per row, 4
    // columns each) and lane i of the group receives column i of those 4 rows
    int v_addr[DT];
    {
        const int rv = 4 * hh + ((lane & 15) >> 2);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            v_addr[dt] = rv * ROWLV + (4 * dt + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) * 16 + 8 * (lane & 1);
    }

    f32x16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;
    float M = kMasked, lsum = 0.0f;   // running max of this lane's head (log2 units), this lane's part of the row sum

    // Every load of the kernel is issued unconditionally: a tile that is not wanted (past the end of this wave's
    // run) is asked for at token T, past the end of the descriptor, so zeros arrive and no memory is read.  The
    // compiler places a wait by counting the loads issued after the one it needs, along the worst path that leads
    // there; loads under a branch are not outstanding on the path that skips them, and at the loop's head the
    // worst path may be the one from the prologue.  So the prologue's four groups keep the order the loop issues
    // them in (K, V of a tile, then the next tile's): with the sixteen loads interleaved by the scheduler, the first
    // tile's K came last, and the loop began every pair of tiles by waiting for everything in flight, which
    // drained the two tiles of loads that are meant to stay in flight.
    __builtin_amdgcn_sched_barrier(0);
    issue_k(std::integral_constant<int, 0>{}, n_tiles > 0 ? t_begin : T);
    __builtin_amdgcn_sched_barrier(0);
    issue_v(std::integral_constant<int, 0>{}, n_tiles > 0 ? t_begin : T);
    __builtin_amdgcn_sched_barrier(0);
    issue_k(std::integral_constant<int, 1>{}, n_tiles > 1 ? t_begin + kGqaTile : T);
    __builtin_amdgcn_sched_barrier(0);
    issue_v(std::integral_constant<int, 1>{}, n_tiles > 1 ? t_begin + kGqaTile : T);
    __builtin_amdgcn_sched_barrier(0);
    auto tile = [&](auto par, int i) {
        constexpr int P = decltype(par)::value;
        const int t0 = t_begin + i * kGqaTile;
        const int t_next = i + 2 < n_tiles ? t0 + 2 * kGqaTile : T;   // (T: nothing is read, zeros arrive)
        if constexpr (TRAFFIC_ONLY) {
            u32x4 x = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int n = 0; n < NP; ++n) x ^= kbuf[P][n] ^ vbuf[P][n];
            lsum += __uint_as_float((x[0] ^ x[1] ^ x[2] ^ x[3]) & 0x3fffffffu) + sc[P];
            issue_k(par, t_next);
            issue_v(par, t_next);
            // (each tile is consumed and refilled on its own, as in the full kernel: without this the compiler
            // folds the two tiles of a pair into one sum and waits for both at once)
            asm volatile("" : "+v"(lsum));
            __builtin_amdgcn_sched_barrier(0);
            return;
        }

        stage(par, kbuf, kS, ROWLK);
        scS[lane] = hh == 0 ? sc[P] * scale_log2e : sc[P];
        issue_k(par, t_next);

        // scores of the tile, register r of a lane = token 8 (r/4) + 4 hh + r%4, column = head l32.  The V tile
        // is widened behind the MFMAs, which need nothing from the vector ALU while they run.
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        bf16x8 kf[KS];
#pragma unroll
        for (int s2 = 0; s2 < KS; ++s2) kf[s2] = *reinterpret_cast<const bf16x8*>(kS + k_addr + 32 * s2);
#pragma unroll
        for (int s2 = 0; s2 < KS; ++s2) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s2], qB[s2], acc, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        stage(par, vbuf, vS, ROWLV);
        issue_v(par, t_next);
        __builtin_amdgcn_sched_barrier(0);

        // softmax over the tile's tokens (the K scale multiplies the fp32 score; tokens past the end are masked)
        float u[16];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const f32x4 kf4 = *reinterpret_cast<const f32x4*>(&scS[8 * r4 + 4 * hh]);
#pragma unroll
            for (int e = 0; e < 4; ++e) u[4 * r4 + e] = acc[4 * r4 + e] * kf4[e];
        }
        if (t0 + kGqaTile > t_end) {   // the run ends inside this tile
#pragma unroll
            for (int r = 0; r < 16; ++r) u[r] = (t0 + 8 * (r / 4) + 4 * hh + r % 4 < t_end) ? u[r] : kMasked;
        }
        float umax = fmaxf(u[0], u[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) umax = fmaxf(umax, fmaxf(u[r], u[r + 1]));
        const float m_new = fmaxf(M, half_max(umax));
        if (__builtin_amdgcn_ballot_w64(m_new > M) != 0) {
            const float alpha = fast_exp2(M - m_new);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
            lsum *= alpha;
            M = m_new;
        }
        float ps0 = 0.0f, ps1 = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            u[r] = fast_exp2(u[r] - M);
            u[r + 1] = fast_exp2(u[r + 1] - M);
            ps0 += u[r];
            ps1 += u[r + 1];
        }
        lsum += ps0 + ps1;
        // the probabilities take their token's v_scale before they are rounded to bf16
        u32x4 pw[2];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const f32x4 vf = *reinterpret_cast<const f32x4*>(&scS[32 + 8 * r4 + 4 * hh]);
            pw[r4 >> 1][2 * (r4 & 1)] = pack_bf16x2(u[4 * r4] * vf[0], u[4 * r4 + 1] * vf[1]);
            pw[r4 >> 1][2 * (r4 & 1) + 1] = pack_bf16x2(u[4 * r4 + 2] * vf[2], u[4 * r4 + 3] * vf[3]);
        }

        // O^T += V^T P^T: k-step u2 covers registers 8 u2 .. 8 u2 + 7 of the probabilities, i.e. tokens
        // 16 u2 + {4 hh .. 4 hh + 3} and 16 u2 + 8 + {4 hh .. 4 hh + 3} of the tile
#pragma unroll
        for (int u2 = 0; u2 < 2; ++u2)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const char* va = vS + v_addr[dt] + 16 * u2 * ROWLV;
                const s16x4 lo = lds_read_tr16(reinterpret_cast<const uint16_t*>(va));
                const s16x4 hi = lds_read_tr16(reinterpret_cast<const uint16_t*>(va + 8 * ROWLV));
                const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                                __builtin_bit_cast(bf16x8, pw[u2]), o[dt], 0, 0, 0);
            }
    };
    // (tiles come in pairs without a branch between them, for the same reason: a run of an odd number of tiles ends
    // on a tile that lies past its end, whose loads asked for nothing and whose tokens are all masked)
    for (int i = 0; i < n_tiles; i += 2) {
        tile(std::integral_constant<int, 0>{}, i);
        tile(std::integral_constant<int, 1>{}, i + 1);
    }

    // this wave's split: register r of tile dt is d = 32 dt + 8 (r/4) + 4 hh + r%4 of head l32
    if (l32 < G) {
        const long idx = ((long)b * Hq + (long)g * G + l32) * n_split + sp;
        float* dst = ws_acc + idx * D + 4 * hh;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const f32x4 ov = {o[dt][4 * r4], o[dt][4 * r4 + 1], o[dt][4 * r4 + 2], o[dt][4 * r4 + 3]};
                *reinterpret_cast<f32x4*>(dst + 32 * dt + 8 * r4) = ov;
            }
        const float L = half_sum(lsum);
        if (hh == 0) {
            ws_ml[idx * 2] = M;
            ws_ml[idx * 2 + 1] = L;
        }
    }
}

// One wave streams tokens_per_wave tokens (a multiple of the tile), a workgroup kGqaWaves such runs, and k
// workgroups share one (batch, KV head).  A compute unit holds eight waves (230 VGPRs: two per SIMD), the chip 2048:
// k is chosen so that (rounds of resident workgroups) x (tiles per wave + a wave's set-up, about two tiles' worth) is
// smallest, which avoids a last round that is nearly empty and runs that differ in length.
int decode_gqa_tokens_per_wave(int kv_len, long n_bg) {
    const long tiles = ((long)kv_len + kGqaTile - 1) / kGqaTile;
    long best_k = 1, best_cost = -1;
    const long resident = 2048 / kGqaWaves;   // workgroups the chip holds at a time
    for (long k = 1; k <= 64 / kGqaWaves; ++k) {
        const long per_wave = (tiles + kGqaWaves * k - 1) / (kGqaWaves * k);
        const long rounds = (n_bg * k + resident - 1) / resident;
        const long cost = rounds * (per_wave + 2);
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost;
            best_k = k;
        }
        if (per_wave == 1) break;
    }
    const long per_wave = (tiles + kGqaWaves * best_k - 1) / (kGqaWaves * best_k);
    return (int)(per_wave * kGqaTile);
}

int decode_gqa_num_splits(int kv_len, long n_bg) {
    const int tpw = decode_gqa_tokens_per_wave(kv_len, n_bg);
    const int waves = (kv_len + tpw - 1) / tpw;
    return (waves + kGqaWaves - 1) / kGqaWaves * kGqaWaves;   // whole workgroups; a wave past the end writes an empty split
}

hipError_t launch_decode_gqa_split(const DecodeArgs& a, float* ws_acc, float* ws_ml, int n_split, hipStream_t stream,
                                   bool traffic_only) {
    const long n_bg = (long)a.batch * a.kv_heads;
    const int tpw = decode_gqa_tokens_per_wave(a.kv_len, n_bg);
    const float scale_log2e = a.softmax_scale * kLog2e;
    dim3 grid((unsigned)(n_split / kGqaWaves), (unsigned)a.kv_heads, (unsigned)a.batch);
    if (traffic_only) {
        if (a.head_dim == 128)
            hipLaunchKernelGGL((slim_decode_int8_gqa_kernel<128, true>), grid, dim3(64 * kGqaWaves), 0, stream,
                               (const uint16_t*)a.q, a.k_codes, a.k_scale, a.v_codes, a.v_scale, ws_acc, ws_ml, a.kv_lens,
                               a.q_heads, a.kv_heads, a.kv_len, n_split, tpw, scale_log2e);
        else
            hipLaunchKernelGGL((slim_decode_int8_gqa_kernel<64, true>), grid, dim3(64 * kGqaWaves), 0, stream,
                               (const uint16_t*)a.q, a.k_codes, a.k_scale, a.v_codes, a.v_scale, ws_acc, ws_ml, a.kv_lens,
                               a.q_heads, a.kv_heads, a.kv_len, n_split, tpw, scale_log2e);
        return hipGetLastError();
    }
    if (a.head_dim == 128)
        hipLaunchKernelGGL(slim_decode_int8_gqa_kernel<128>, grid, dim3(64 * kGqaWaves), 0, stream,
                           (const uint16_t*)a.q, a.k_codes, a.k_scale, a.v_codes, a.v_scale, ws_acc, ws_ml, a.kv_lens,
                           a.q_heads, a.kv_heads, a.kv_len, n_split, tpw, scale_log2e);
    else
        hipLaunchKernelGGL(slim_decode_int8_gqa_kernel<64>, grid, dim3(64 * kGqaWaves), 0, stream,
                           (const uint16_t*)a.q, a.k_codes, a.k_scale, a.v_codes, a.v_scale, ws_acc, ws_ml, a.kv_lens,
                           a.q_heads, a.kv_heads, a.kv_len, n_split, tpw, scale_log2e);
    return hipGetLastError();
}

}  // namespace slim

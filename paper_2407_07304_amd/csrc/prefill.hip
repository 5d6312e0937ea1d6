// Prefill attention (paper section 2.1): one work item owns a block of query rows and the
// whole softmax direction; K/V stream through it in 32-key tiles while an fp32 running max
// and sum keep the softmax exact.  INT8 K/V (section 2.2) are widened exactly to bf16 while
// being staged; their per-token scales multiply the fp32 score column (K) and the
// probability before it is rounded to bf16 (V), so dequantisation adds no rounding.
//
// Mapping on gfx950 (wave64, v_mfma_f32_32x32x16_bf16):
//   - A workgroup is 8 waves and owns 128 query rows.  Waves w and w+4 sit on the same SIMD
//     and own the same 32 rows; the first four waves (group 0) take the even key tiles, the
//     other four (group 1) the odd ones, each with its own running max, sum and accumulator,
//     merged once at the end of the row block.
//   - The two groups run in opposite phases, one barrier per phase: while one group does the
//     softmax of its tile on the vector ALU, the other feeds the matrix pipe (P V of its last
//     tile, then the score tile two tiles ahead).  A SIMD therefore always holds one wave that
//     wants the vector ALU and one that wants the MFMA unit.
//   - The score tile is computed transposed, S^T = K Q^T: the K tile is the A operand
//     (from LDS), Q^T the B operand (held in registers for the whole row block).  In the
//     result every lane holds ONE query column and 16 of the 32 keys, so the row max and
//     row sum are in-lane reductions plus one exchange between lanes l and l+32.
//   - The same registers, rounded to bf16, are directly the B operand of
//     O^T += V^T P^T; V^T comes from the row-major V tile in LDS through the LDS
//     transpose read (ds_read_b64_tr_b16), so V is never transposed in memory.
//   - O^T accumulators: lane = query column, so the online-softmax rescale is a per-lane
//     scalar multiply; the running max is lazy (it moves only when a row's max grew by more
//     than 2^8), so the rescale runs a few times per row block.
//   - K/V tiles live in an LDS ring (eight K slots, four V slots).  bf16 tiles are written by the
//     memory pipe itself (buffer loads with an LDS destination, issued by the group in its
//     matrix phase, six (K) and four (V) tiles ahead, one load between two MFMAs, the same
//     loads and the same wait in every phase: past the last tile they ask for zeros) as unpadded
//     rows whose 16-byte chunks are
//     XOR-swizzled by the row, so both the 128-bit K row reads and the V transpose reads are
//     free of bank conflicts; INT8 tiles pass through registers, where they are widened, into
//     padded rows.
//   - A wave reads its MFMA operands from LDS one matrix phase ahead, each fragment right after
//     the MFMA that consumed its predecessor: the reads issue in the shadow of the MFMAs and
//     the softmax phase is pure vector work.
//   - Under the causal mask a workgroup takes the row-block pair (x, n-1-x) one after the
//     other, so every workgroup does the same amount of work.  The short block goes first: the
//     key tiles it read are still in the L2 when the long block starts over at tile 0 (the other
//     order re-fetched them: 81.5 MB of HBM traffic on B=1, H=32, S=2048 against 68.8 MB now,
//     which is Q, K, V and O once each).
#include <type_traits>

#include "slim_common.h"
#include "slim_kernels.h"

namespace slim {

constexpr int kBR = 128;   // query rows per row block (4 row groups x 32)
constexpr int kBC = 32;    // keys per tile
constexpr int kRingK = 8;  // LDS ring depth, K tiles
constexpr int kRingV = 4;  // LDS ring depth, V tiles
constexpr int kPrefillThreads = 512;

struct PrefillParams {
    const uint16_t* q;
    const void* k;
    const void* v;
    const float* ks;
    const float* vs;
    void* out;
    float* row_max;   // the two-sweep variant's row maxima [batch, q_heads, seq_len, 2], else null
    int8_t* kq;    // INT8 cache to write next to the attention (bf16 K/V only), or null
    float* kqs;
    int8_t* vq;
    float* vqs;
    int Hq, Hkv, S, causal, n_rb, n_pair, total, chunk;
    float scale_log2e;
};

template <int N>
using int_c = std::integral_constant<int, N>;

// MODE 1 and 2: the paper's own order of operations (section 2.1: the whole score row is there before the softmax
// is applied), for comparison.  A row block's scores do not fit on chip, so K is swept twice, by two launches
// of this kernel: MODE 1 computes the scores and keeps only the row maxima (one per row and wave group, written
// to p.row_max), MODE 2 computes them again, exponentiates against those final maxima and multiplies by V:
// no running maximum, no rescaling of the accumulator, 1.5 times the MFMAs.  MODE 0 is the kernel proper.
template <int D, bool KV_I8, bool OUT_F32, int MODE = 0>
__global__ __launch_bounds__(kPrefillThreads) void slim_prefill_kernel(const PrefillParams p) {
    static_assert(!(MODE != 0 && KV_I8), "the two-sweep variant exists for bf16 K/V only");
    constexpr bool stats_only = MODE == 1;
    constexpr int KS = D / 16;       // k-steps of the score MFMA
    constexpr int DT = D / 32;       // 32-row tiles of O^T
    constexpr int ROWB = KV_I8 ? D : 2 * D;   // bytes per K/V row in memory
    // LDS tile layouts.  bf16 K/V: unpadded rows (that is how the memory pipe writes them), the 16-byte
    // chunk c of row r at chunk position c ^ swz(r).  K: the 16 rows a 128-bit read touches in one pass
    // land on 16 different bank groups.  V: the 4 rows x 4 chunks a transpose read touches in one pass do.
    // INT8 K/V (written from registers): no swizzle, rows padded by 16 bytes (K) and 64 bytes (V) instead,
    // which keeps every address a base register plus a constant.
    constexpr int ROWL = 2 * D;               // bytes of data per LDS row
    constexpr int ROWLK = KV_I8 ? ROWL + 16 : ROWL, ROWLV = KV_I8 ? ROWL + 64 : ROWL;   // row pitch
    constexpr int TILEBK = kBC * ROWLK, TILEBV = kBC * ROWLV;   // bytes per tile in LDS
    constexpr int TILEB = TILEBK;             // (bf16: both tensors)
    constexpr int CPL = ROWL / 16;            // 16-byte chunks per LDS row: 16 or 8
    constexpr int RPL = 256 / ROWL;           // rows per 256-byte line of banks: 1 or 2
    constexpr int K_BYTES = kRingK * TILEBK, V_BYTES = kRingV * TILEBV;
    constexpr int NV = DT / 2 * 4 + 1;        // f32x4 vectors a wave hands to its partner at the merge
    constexpr int MERGE_BYTES = 8 * NV * 64 * 16;
    // (the merge buffer takes the place of the ring, which is quiet by then)
    constexpr int RING_BYTES = K_BYTES + V_BYTES > MERGE_BYTES ? K_BYTES + V_BYTES : MERGE_BYTES;
    auto swz_k = [](int r) { return KV_I8 ? 0 : (r / RPL) & (CPL - 1); };
    auto swz_v = [](int r) { return KV_I8 ? 0 : ((r / RPL) & (CPL / 4 - 1)) << 2; };

    // The row block's Q: 128 unpadded rows, the 16-byte chunk c of row r at chunk position c ^ qswz(r) (the bf16 K tile's layout)
    constexpr int ROWQ = 2 * D;                // bytes per Q row, in memory and in LDS
    constexpr int CPQ = ROWQ / 16;             // 16-byte chunks per row: 16 or 8
    constexpr int RPQ = 64 / CPQ;              // rows per wave-wide load: 4 or 8
    constexpr int NQ = kBR / 8 / RPQ;          // loads per wave and row block (a wave brings in 16 rows): 4 or 2
    constexpr int Q_OFF = RING_BYTES + kRingK * 2 * kBC * 4;
    auto qswz = [](int r) { return (r / (256 / ROWQ)) & (CPQ - 1); };

    constexpr bool Q_LDS = !KV_I8;             // (the INT8 kernel keeps plain loads into the registers: measured faster there)
    __shared__ __attribute__((aligned(16))) char smem[Q_OFF + (Q_LDS ? kBR * ROWQ : 0)];
    float* const scS = reinterpret_cast<float*>(smem + RING_BYTES);   // INT8: per slot [0,32) k_scale*c, [32,64) v_scale

    // workgroup -> (batch*head, row-block pair).  Hardware deals workgroup ids round-robin over the 8
    // XCDs, so consecutive virtual ids (which share K/V) are steered to one XCD.
    int bh, x;
    {
        const int n = (int)__builtin_amdgcn_workgroup_id_x();   // the builtin, not a library call: stays a scalar
        const int vid = (n % 8) * p.chunk + n / 8;
        if (vid >= p.total) return;
        bh = vid / p.n_pair;
        x = vid % p.n_pair;
    }
    const int b = bh / p.Hq, h = bh % p.Hq;
    const int g = h / (p.Hq / p.Hkv);
    const int S = p.S;
    const float c = p.scale_log2e;

    // wave index as a scalar: everything derived from it (group, row group, last tile) stays uniform
    const int tid = (int)__builtin_amdgcn_workitem_id_x(), w8 = __builtin_amdgcn_readfirstlane(tid >> 6), grp = w8 >> 2, w = w8 & 3;
    const int l = tid & 63, l32 = l & 31, hh = l >> 5;
    const long kvrow0 = ((long)b * p.Hkv + g) * (long)S;

    // Q^T B-operands of a row block: lane holds row my_q, d = 16 s + 8 hh + [0,8).  With bf16 K/V the 128 rows come
    // in through LDS, by buffer loads with an LDS destination that move 64 consecutive 16-byte pieces each: loads
    // that give every lane a row of its own are taken lane by lane by the memory pipe (about 4 k cycles per row block
    // for the eight waves' fragments, with the first K and V tiles waiting behind them, against about 0.7 k this
    // way); rows past the end of the sequence arrive as zeros.  The INT8 kernel loads its fragments straight into
    // the registers.  The first row block's are requested here, ahead of the address tables below: they come from
    // cold memory.
    bf16x8 qreg[KS];
    const unsigned smem_base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
    u32x4 qrs_raw;
    {
        const unsigned long long a64 = (unsigned long long)(p.q + ((long)b * p.Hq + h) * (long)S * D);
        qrs_raw[0] = __builtin_amdgcn_readfirstlane((unsigned)a64);
        qrs_raw[1] = __builtin_amdgcn_readfirstlane((unsigned)(a64 >> 32) & 0xffffu);
        qrs_raw[2] = __builtin_amdgcn_readfirstlane((unsigned)S * ROWQ);
        qrs_raw[3] = 0x00020000u;
    }
    auto request_q = [&](int rb_q) {
        if constexpr (!Q_LDS) {
            const int q_row = min(rb_q * kBR + 32 * w + l32, S - 1);
            const uint16_t* qp = p.q + (((long)b * p.Hq + h) * S + q_row) * (long)D + 8 * hh;
#pragma unroll
            for (int s = 0; s < KS; ++s) qreg[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
            return;
        }
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            const int r = 16 * w8 + RPQ * j + l / CPQ, pos = l % CPQ;   // row of the block, chunk position in LDS
            const unsigned voff = (unsigned)(rb_q * kBR + r) * ROWQ + (unsigned)((pos ^ qswz(r)) * 16);
            const unsigned dst = __builtin_amdgcn_readfirstlane(smem_base + (unsigned)(Q_OFF + (16 * w8 + RPQ * j) * ROWQ));
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                         :
                         : "s"(dst), "v"(voff), "s"(qrs_raw)
                         : "memory", "m0");
        }
    };
    // this wave's fragments of the Q in LDS (once the requests have landed and a barrier has passed)
    auto read_q = [&]() {
        if constexpr (!Q_LDS) return;
#pragma unroll
        for (int s = 0; s < KS; ++s)
            qreg[s] = *reinterpret_cast<const bf16x8*>(smem + Q_OFF + (32 * w + l32) * ROWQ + (((2 * s + hh) ^ qswz(l32)) * 16));
    };
    request_q(x);
    __builtin_amdgcn_sched_barrier(0);

    // ---- staging.  The buffer descriptors cover exactly this head's K (V) slab: pieces past the end of
    // the sequence read as zero (those keys are masked in the softmax).  A tile is staged by the four
    // waves of ONE group.
    const char* const kslab = (const char*)p.k + kvrow0 * ROWB;
    const char* const vslab = (const char*)p.v + kvrow0 * ROWB;
    const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc((void*)kslab, 0, (int)((unsigned)S * ROWB), 0x00020000);
    const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc((void*)vslab, 0, (int)((unsigned)S * ROWB), 0x00020000);

    // bf16: one buffer load with an LDS destination moves 64 consecutive 16-byte chunk positions (RPW whole
    // rows); lane i fills position i, so it asks for the chunk the swizzle puts there.  The load is
    // written as inline assembly on purpose: the compiler then keeps no book on it, and neither its
    // barriers nor its LDS reads wait for requests that are meant to stay in flight for two phases.
    // Completion is tracked by hand (vmcnt) where a tile becomes readable.
    constexpr int RPW = 64 / CPL;              // rows per wave-wide load: 4 or 8
    constexpr int NLD = kBC / (4 * RPW);       // loads per wave, tile and tensor: 2 or 1
    auto raw_rsrc = [&](const char* base) {    // the same descriptor as four plain dwords
        const unsigned long long a64 = (unsigned long long)base;
        u32x4 d;
        d[0] = __builtin_amdgcn_readfirstlane((unsigned)a64);
        d[1] = __builtin_amdgcn_readfirstlane((unsigned)(a64 >> 32) & 0xffffu);
        d[2] = __builtin_amdgcn_readfirstlane((unsigned)S * ROWB);
        d[3] = 0x00020000u;
        return d;
    };
    const u32x4 krs_raw = raw_rsrc(kslab), vrs_raw = raw_rsrc(vslab);
    unsigned d_koff[NLD], d_voff[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int r = (kBC / NLD) * j + RPW * w + l / CPL, pos = l % CPL;
        d_koff[j] = (unsigned)r * ROWB + (unsigned)((pos ^ swz_k(r)) * 16);
        d_voff[j] = (unsigned)r * ROWB + (unsigned)((pos ^ swz_v(r)) * 16);
    }
    auto dma_tile = [&](const u32x4 rs, const unsigned (&off)[NLD], int t, int lds_off, bool wanted = true) {
        // (a tile that is not wanted is requested past the end of the slab: zeros arrive, no memory is read)
        const unsigned tbase = wanted ? (unsigned)t * (kBC * ROWB) : (unsigned)S * ROWB;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const unsigned dst = __builtin_amdgcn_readfirstlane(smem_base + (unsigned)(lds_off + ((kBC / NLD) * j + RPW * w) * ROWL));
            const unsigned voff = tbase + off[j];
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                         :
                         : "s"(dst), "v"(voff), "s"(rs)
                         : "memory", "m0");
        }
    };

    // The same, one load at a time: the address work first, the request later, so that a matrix phase can tuck
    // them between its MFMAs without ever keeping the matrix pipe waiting for the next one.
    auto dma_prep = [&](const unsigned (&off)[NLD], int j, int t, int lds_off, bool wanted, unsigned& dst, unsigned& voff) {
        const unsigned tbase = wanted ? (unsigned)t * (kBC * ROWB) : (unsigned)S * ROWB;
        dst = __builtin_amdgcn_readfirstlane(smem_base + (unsigned)(lds_off + ((kBC / NLD) * j + RPW * w) * ROWL));
        voff = tbase + off[j];
    };
    auto dma_fire = [&](const u32x4 rs, unsigned dst, unsigned voff) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     :
                     : "s"(dst), "v"(voff), "s"(rs)
                     : "memory", "m0");
    };

    // INT8: piece gl + 256 i of thread gl (16 codes) goes through registers and leaves as two bf16 chunks.
    // The last wave of a group also carries the tile's 32 + 32 scales.
    constexpr int CPR = ROWB / 16;            // 16-byte pieces per row in memory
    constexpr int CH = kBC * CPR;             // pieces per tile and tensor
    constexpr int NP = CH >= 256 ? CH / 256 : 1;
    const int gl = tid & 255;
    const bool has_p = CH >= 256 || w < CH / 64;
    // The tile's scales: the last wave of a group carries the 32 k_scales, the one before it the 32 v_scales (every
    // choice here is uniform over the wave: a value that depends on the lane would have to live, as a register or as
    // a spill, through the whole kernel).  Both halves of the wave load and store the same 32 values.
    const bool has_s = KV_I8 && w >= 2;
    const bool s_is_k = w == 3;
    const float* const sbase = KV_I8 ? ((s_is_k ? p.ks : p.vs) + kvrow0) : nullptr;
    const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc((void*)sbase, 0, KV_I8 ? (int)((unsigned)S * 4u) : 0, 0x00020000);
    unsigned p_off[NP];
    int p_kdst[NP][2], p_vdst[NP][2];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const int pid = gl + 256 * i, row = pid / CPR, col = pid % CPR;
        p_off[i] = (unsigned)row * ROWB + (unsigned)col * 16u;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            p_kdst[i][e] = row * ROWLK + (((2 * col + e) ^ swz_k(row)) * 16);
            p_vdst[i][e] = K_BYTES + row * ROWLV + (((2 * col + e) ^ swz_v(row)) * 16);
        }
    }
    auto load_tile_at = [&](const __amdgpu_buffer_rsrc_t rs, int t, u32x4 (&dst)[NP], const unsigned (&off)[NP]) {
        if (has_p) {
#pragma unroll
            for (int i = 0; i < NP; ++i)
                dst[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)((unsigned)t * (kBC * ROWB) + off[i]), 0, 0);
        }
    };
    auto load_tile = [&](const __amdgpu_buffer_rsrc_t rs, int t, u32x4 (&dst)[NP]) { load_tile_at(rs, t, dst, p_off); };
    auto load_s_at = [&](int t, float& dst, int lane32, bool wanted) {   // (a key past the end of the sequence gets scale 0: it is masked anyway)
        if (wanted) dst = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(srs, (t * kBC + lane32) * 4, 0, 0));
    };
    auto load_s = [&](int t, float& dst) { load_s_at(t, dst, l32, has_s); };
    auto store_tile = [&](int slot_off, const int (&dsts)[NP][2], const u32x4 (&src)[NP]) {   // 16 INT8 codes -> 16 bf16 (exact)
        if (has_p) {
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const u32x4 cw = src[i];
                u32x4 lo, hi;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    lo[2 * e] = pack_bf16x2(i8_to_f32<0>(cw[e]), i8_to_f32<1>(cw[e]));
                    lo[2 * e + 1] = pack_bf16x2(i8_to_f32<2>(cw[e]), i8_to_f32<3>(cw[e]));
                    hi[2 * e] = pack_bf16x2(i8_to_f32<0>(cw[2 + e]), i8_to_f32<1>(cw[2 + e]));
                    hi[2 * e + 1] = pack_bf16x2(i8_to_f32<2>(cw[2 + e]), i8_to_f32<3>(cw[2 + e]));
                }
                *reinterpret_cast<u32x4*>(smem + slot_off + dsts[i][0]) = lo;
                *reinterpret_cast<u32x4*>(smem + slot_off + dsts[i][1]) = hi;
            }
        }
    };
    auto store_s = [&](int slot, float s) {
        if (has_s) scS[slot * (2 * kBC) + (s_is_k ? 0 : kBC) + l32] = s_is_k ? s * c : s;
    };
    struct Stage {
        u32x4 k[NP], v[NP];
        float s;
    };

    f32x16 o[DT];
    // LDS read addresses (bytes).  K fragment of k-step s: row l32, chunk 2 s + hh.  V transpose read: the
    // 16 lanes of a group fetch rows k..k+3 (4 lanes per row, 8 bytes each) and lane i of the group
    // receives column i of those 4 rows; per 32-column tile dt the lane reads chunk 4 dt + 2 b4 + (l&3)/2.
    int k_addr[KS], v_addr[DT];
#pragma unroll
    for (int s2 = 0; s2 < KS; ++s2) k_addr[s2] = l32 * ROWLK + (((2 * s2 + hh) ^ swz_k(l32)) * 16);
    {
        const int rv = 4 * hh + ((l & 15) >> 2);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            v_addr[dt] = K_BYTES + rv * ROWLV + (((4 * dt + 2 * ((l >> 4) & 1) + ((l & 3) >> 1)) ^ swz_v(rv)) * 16) + 8 * (l & 1);
    }

    for (int pass = 0; pass < 2; ++pass) {
        const int rb = pass == 0 ? x : p.n_rb - 1 - x;
        if (pass == 1 && rb == x) break;   // the middle row block of an odd count
        const bool has_next = pass == 0 && x != p.n_rb - 1 - x;
        const int i0 = rb * kBR;
        const int my_q = i0 + 32 * w + l32;             // this lane's query row (may be >= S in the last block)
        const int wave_q_lo = i0 + 32 * w;
        const int kend = p.causal ? min(S, i0 + kBR) : S;
        const int n_tiles = (kend + kBC - 1) / kBC;
        const int last_phase = 2 * ((n_tiles + 1) / 2);   // phases 0..last_phase, one barrier each
        // last tile of this row group: its diagonal under the causal mask, else the tail of the key axis
        // (always taken through the masked path); -1 if the row group lies past the sequence
        const int t_last = wave_q_lo >= S ? -1 : (p.causal ? min(n_tiles - 1, wave_q_lo / kBC) : n_tiles - 1);
        const int lim = p.causal ? min(my_q, S - 1) : S - 1;   // last key this lane's row may see

        // (the first pass's Q was requested at the top of the kernel, the second pass's is before the first one's merge)
        float M = kMasked, lsum = 0.0f;   // running max in scaled (log2) units; per-lane partial row sum

        // ---- prologue.  In the steady state a group stages in its matrix phase phi: bf16 requests K tile
        // phi+6 and V tile phi+4 (in LDS by the end of its next matrix phase); INT8 stores K tile phi+5
        // and V tile phi+3 from registers and loads K tile phi+7, V tile phi+5 into them.  Everything
        // earlier is staged here, all requests issued together.  Every V slot gets a tile (zeros past the
        // end of the sequence): whatever a skipped tile later leaves in place is finite data of this row
        // block, never the previous pass's merge buffer.
        if constexpr (MODE == 2) {   // the final maximum of this lane's row over this group's tiles
            M = p.row_max[((((long)b * p.Hq + h) * S + min(my_q, S - 1)) * 2) + grp];
        }
        Stage sg;
        __syncthreads();   // the previous pass (or sweep) has finished with the ring and the merge buffer that lies over it
        if constexpr (!KV_I8) {
            if (grp == 0) {
                dma_tile(krs_raw, d_koff, 0, 0);
                dma_tile(krs_raw, d_koff, 2, 2 * TILEB);
                dma_tile(krs_raw, d_koff, 4, 4 * TILEB);
                if (!stats_only) {
                    dma_tile(vrs_raw, d_voff, 0, K_BYTES);
                    dma_tile(vrs_raw, d_voff, 2, K_BYTES + 2 * TILEB);
                }
            } else {
                dma_tile(krs_raw, d_koff, 1, TILEB);
                dma_tile(krs_raw, d_koff, 3, 3 * TILEB);
                dma_tile(krs_raw, d_koff, 5, 5 * TILEB);
                if (!stats_only) {
                    dma_tile(vrs_raw, d_voff, 1, K_BYTES + TILEB);
                    dma_tile(vrs_raw, d_voff, 3, K_BYTES + 3 * TILEB);
                }
            }
            __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wave's requests have landed in LDS
        } else {
            // LDS: K tiles 0..4, V tiles 0..2 (group 0: K 0, 2, 4, V 0, 2; group 1: K 1, 3, V 1); registers: what
            // each group stores in its first matrix phase (group 1 in phase 0: K 5, V 3; group 0 in phase 1: K 6, V 4)
            u32x4 ta[NP], tb[NP], tc[NP], td[NP], te[NP];
            float sa = 0.0f, sb = 0.0f, sc3 = 0.0f;
            // The addresses of these loads are put together here, from copies the compiler cannot see through: left
            // to itself it computes all of them ahead of the pass loop, spills them, and reloads them one by one
            // between the loads, and a reload is a memory access that waits, in order, for the tile loads before it
            // (eight trips to cold memory one after the other instead of one).
            unsigned off_now[NP];
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                off_now[i] = p_off[i];
                asm volatile("" : "+v"(off_now[i]));
            }
            int l32_now = l32, w_now = w;
            asm volatile("" : "+v"(l32_now));
            asm volatile("" : "+s"(w_now));
            const bool has_s_now = w_now >= 2;   // (likewise: a flag kept from the top of the kernel comes back as a reload between the loads)
            load_tile_at(krs, grp, ta, off_now);
            load_tile_at(krs, 2 + grp, tb, off_now);
            load_tile_at(vrs, grp, td, off_now);
            load_s_at(grp, sa, l32_now, has_s_now);
            load_s_at(2 + grp, sb, l32_now, has_s_now);
            // (K tile 4 and V tile 2 belong to group 0's share; group 1 brings them in as well and writes the same
            // bytes to the same place: a branch around these loads makes the compiler spill a tile that has just
            // been asked for, and waiting for that store lets the loads after it start a memory latency late)
            load_tile_at(krs, 4, tc, off_now);
            load_tile_at(vrs, 2, te, off_now);
            load_s_at(4, sc3, l32_now, has_s_now);
            load_tile_at(krs, 6 - grp, sg.k, off_now);
            load_tile_at(vrs, 4 - grp, sg.v, off_now);
            load_s_at(6 - grp, sg.s, l32_now, has_s_now);
            store_tile(grp * TILEBK, p_kdst, ta);
            store_tile((2 + grp) * TILEBK, p_kdst, tb);
            store_tile(grp * TILEBV, p_vdst, td);
            store_s(grp, sa);
            store_s(2 + grp, sb);
            store_tile(4 * TILEBK, p_kdst, tc);
            store_tile(2 * TILEBV, p_vdst, te);
            store_s(4, sc3);
        }
        __syncthreads();
        read_q();
        // (the accumulators start here, not above: 64 registers the prologue's loads in flight can use)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;

        // Operand fragments, read from LDS one matrix phase ahead:
        //   kfr: K tile as A operand, lane = key l32, d = 16 s + 8 hh + [0,8)
        //   vfr[u]: V^T tile as A operand for keys 16u..16u+15.  Transpose read: the 16 lanes of a group
        //   fetch rows k..k+3 (4 lanes per row, 4 columns each) and lane i receives column i of those rows.
        bf16x8 kfr[KS];
        s16x4 vfr[2][2 * DT];
        auto fetch_k1 = [&](int s, int slot_off) {   // slot_off: byte offset of the K ring slot
            kfr[s] = *reinterpret_cast<const bf16x8*>(smem + k_addr[s] + slot_off);
        };
        auto fetch_v1 = [&](int u, int dt, int slot_off) {   // slot_off: byte offset of the V ring slot
            const char* va = smem + v_addr[dt] + slot_off + 16 * u * ROWLV;
            vfr[u][2 * dt] = lds_read_tr16(reinterpret_cast<const uint16_t*>(va));
            vfr[u][2 * dt + 1] = lds_read_tr16(reinterpret_cast<const uint16_t*>(va + 8 * ROWLV));
        };
        // One score MFMA, S^T[key][query] += sum over d in [16 s, 16 s + 16) of K[key][d] Q[query][d], and one
        // P V MFMA, O^T[d][query] += sum_key V[key][d] P[query][key] for d in [32 dt, 32 dt + 32); k-step u of
        // the latter covers registers 8u..8u+7 of the probabilities, i.e. keys 16u + {4hh..4hh+3} and
        // 16u + 8 + {4hh..4hh+3} of the tile.
        auto score_mfma = [&](int s, f32x16& acc) {
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[s], qreg[s], acc, 0, 0, 0);
        };
        auto pv_mfma = [&](int u, int dt, const u32x4 (&pw)[2]) {
            const bf16x8 pb = __builtin_bit_cast(bf16x8, pw[u]);
            const s16x4 lo = vfr[u][2 * dt], hi = vfr[u][2 * dt + 1];
            const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb, o[dt], 0, 0, 0);
        };
        // softmax of tile t (scores in st, register r of this lane is key 32 t + 8 (r/4) + 4 hh + r%4):
        // probabilities, rounded to bf16, into pw.  Pure vector work.
        auto softmax = [&](int sc_slot, int t, const f32x16& st, u32x4 (&pw)[2]) {
            if (t > t_last) {   // tile skipped by this row group: its P V MFMAs run on zeros
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int i = 0; i < 4; ++i) pw[u][i] = 0u;
                return;
            }
            float cf[16];
            if (KV_I8) {
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 kf = *reinterpret_cast<const f32x4*>(&scS[sc_slot * (2 * kBC) + 8 * r4 + 4 * hh]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) cf[4 * r4 + e] = kf[e];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) cf[r] = c;
            }
            // Fast path: exponentials against the running max as it stands; the lane's partial sum doubles
            // as the overflow check (lazy running max: it only moves when the sum of a lane's 16
            // probabilities exceeds 2^8, so the accumulator is rescaled a few times per row block).
            const bool full = t == t_last;   // masked tile: recompute the max exactly
            float a[16], ps = 0.0f;
            bool redo = full;
            if (!full) {
                float ps0 = 0.0f, ps1 = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    a[r] = fast_exp2(fmaf(st[r], cf[r], -M));
                    a[r + 1] = fast_exp2(fmaf(st[r + 1], cf[r + 1], -M));
                    ps0 += a[r];
                    ps1 += a[r + 1];
                }
                ps = ps0 + ps1;
                redo = __builtin_amdgcn_ballot_w64(ps > 256.0f) != 0;
            }
            if (redo) {
                const int rel = full ? lim - (t * kBC + 4 * hh) : kBC;   // keys of this lane up to offset rel are visible
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float u = st[r] * cf[r];
                    a[r] = (8 * (r / 4) + (r % 4) <= rel) ? u : kMasked;
                }
                float umax = fmaxf(a[0], a[1]);
#pragma unroll
                for (int r = 2; r < 16; r += 2) umax = fmaxf(umax, fmaxf(a[r], a[r + 1]));
                const float m_new = fmaxf(M, half_max(umax));
                const float alpha = fast_exp2(M - m_new);
                // (the accumulator is still zero on a group's first tile, and on the diagonal tile the maximum has
                // usually been met already: the 16 DT multiplications are skipped when they would change nothing)
                if (KV_I8 || (t >= 2 && __builtin_amdgcn_ballot_w64(m_new > M) != 0)) {   // (INT8: the branch costs registers the kernel does not have)
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
                }
                lsum *= alpha;
                M = m_new;
                float ps0 = 0.0f, ps1 = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    a[r] = fast_exp2(a[r] - m_new);
                    a[r + 1] = fast_exp2(a[r + 1] - m_new);
                    ps0 += a[r];
                    ps1 += a[r + 1];
                }
                ps = ps0 + ps1;
            }
            lsum += ps;
            if (KV_I8) {
                // the probabilities take their token's v_scale before they are rounded to bf16
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 vf = *reinterpret_cast<const f32x4*>(&scS[sc_slot * (2 * kBC) + kBC + 8 * r4 + 4 * hh]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) a[4 * r4 + e] *= vf[e];
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) pw[u][i] = pack_bf16x2(a[8 * u + 2 * i], a[8 * u + 2 * i + 1]);
        };

        // MODE 1: the tile's scores only raise the row maximum
        auto row_max_only = [&](int t, const f32x16& st) {
            if (t > t_last) return;
            const int rel = t == t_last ? lim - (t * kBC + 4 * hh) : kBC;   // keys of this lane up to offset rel are visible
            float umax = kMasked;
#pragma unroll
            for (int r = 0; r < 16; ++r) umax = fmaxf(umax, (8 * (r / 4) + (r % 4) <= rel) ? st[r] * c : kMasked);
            M = fmaxf(M, half_max(umax));
        };
        f32x16 st;
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = 0.0f;
        u32x4 pw[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};

        // One phase.  The group whose parity matches the phase does the softmax of tile phi; the other one
        // does the matrix work of tile phi-1 (P V, and the scores of tile phi+1), reads the operands of its
        // next matrix phase and moves the ring on.
        auto phase = [&](auto p4_c, auto grp_c, int phi) {
            constexpr int P4 = decltype(p4_c)::value, G = decltype(grp_c)::value;
            if constexpr ((P4 & 1) == G) {
                if constexpr (MODE == 1) {
                    row_max_only(phi, st);
                } else {
                    // (MODE 2: the running maximum starts at the final one, so the overflow watch never
                    // fires and the masked tile's rescale is by one)
                    softmax(phi & (kRingK - 1), phi, st, pw);
                }
            } else {
                // Matrix phase of tile t = phi - 1: its P V MFMAs and the score MFMAs of tile t + 2, always all
                // sixteen (a skipped tile has P = 0, unused scores are dropped), alternating so that the score
                // chain never issues two dependent MFMAs back to back.  Every operand fragment is refilled
                // right after the MFMA that consumed it, with the fragment the next matrix phase of this wave
                // needs (K tile phi+3, V tile phi+1): the LDS reads, and the ring traffic, are issued in the
                // shadow of the MFMAs.  (The fences keep the issue order as written.)
                const int k_rd = ((phi + 3) & (kRingK - 1)) * TILEBK;
                constexpr int v_rd = ((P4 + 1) & 3) * TILEBV;
                // the wave that feeds the matrix pipe goes first: without this the older wave of the SIMD wins
                // the issue port whatever it is doing, and the matrix phases of group 1 run 30 % longer
                __builtin_amdgcn_s_setprio(3);
                f32x16 acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
                __builtin_amdgcn_sched_barrier(0);
                // bf16: K tile phi+6 and V tile phi+4 go straight into their ring slots, one load per step of
                // this loop (DT = 2 NLD steps: first the K tile's loads, then the V tile's), the address work
                // behind the score MFMA and the request behind the P V MFMA.  Always the same number of
                // requests, so that the wait at the end of the phase is the same instruction every time: past
                // the last tile this row block needs, zeros are requested from beyond the slab.
                // Invariant the hand-written wait below rests on: a matrix phase issues exactly REQ ring requests
                // (steps i < NLD of the loop: the K tile's, the remaining DT - NLD steps: the V tile's, none of
                // those in the maxima-only sweep), buffer loads complete in the order they were issued, and the
                // requests of the wave's PREVIOUS matrix phase are the ones that must have landed.  So the wait
                // at the end of the phase is vmcnt(REQ): everything but this phase's own requests.
                constexpr int REQ = KV_I8 ? 0 : NLD + (stats_only ? 0 : DT - NLD);
                static_assert(KV_I8 || DT == 2 * NLD, "one ring load per step of the first MFMA loop");
                static_assert(KV_I8 || REQ == (stats_only ? NLD : 2 * NLD), "requests per matrix phase");
                static_assert(REQ < 16, "vmcnt is written into the low four bits of the wait's immediate");
#pragma unroll
                for (int i = 0; i < DT; ++i) {
                    unsigned dma_dst = 0, dma_voff = 0;
                    score_mfma(i, acc);
                    __builtin_amdgcn_sched_barrier(0);
                    fetch_k1(i, k_rd);
                    if constexpr (!KV_I8) {
                        if (i < NLD) dma_prep(d_koff, i, phi + 6, ((phi + 6) & (kRingK - 1)) * TILEB, phi + 6 < n_tiles, dma_dst, dma_voff);
                        else if (!stats_only) dma_prep(d_voff, i - NLD, phi + 4, K_BYTES + P4 * TILEB, phi + 4 < n_tiles, dma_dst, dma_voff);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (!stats_only) {
                        pv_mfma(0, i, pw);
                        __builtin_amdgcn_sched_barrier(0);
                        fetch_v1(0, i, v_rd);
                    }
                    if constexpr (!KV_I8) {
                        if (i < NLD) dma_fire(krs_raw, dma_dst, dma_voff);
                        else if (!stats_only) dma_fire(vrs_raw, dma_dst, dma_voff);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (KV_I8) {
                    // the pieces loaded two phases ago go to K tile phi+5 and V tile phi+3
                    store_tile(((phi + 5) & (kRingK - 1)) * TILEBK, p_kdst, sg.k);
                    store_tile(((P4 + 3) & 3) * TILEBV, p_vdst, sg.v);
                    store_s((phi + 5) & (kRingK - 1), sg.s);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < DT; ++i) {
                    score_mfma(DT + i, acc);
                    __builtin_amdgcn_sched_barrier(0);
                    fetch_k1(DT + i, k_rd);
                    __builtin_amdgcn_sched_barrier(0);
                    if (!stats_only) {
                        pv_mfma(1, i, pw);
                        __builtin_amdgcn_sched_barrier(0);
                        fetch_v1(1, i, v_rd);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                st = acc;
                __builtin_amdgcn_s_setprio(0);
                if constexpr (!KV_I8) {
                    // what this wave requested in its previous matrix phase is read from the next phase on
                    __builtin_amdgcn_s_waitcnt(0x0f70 | REQ);   // vmcnt(REQ), see the invariant above
                } else {
                    load_tile(krs, phi + 7, sg.k);
                    load_tile(vrs, phi + 5, sg.v);
                    load_s(phi + 7, sg.s);
                }
            }
            // End of phase: this wave's LDS reads and writes are done, then the workgroup barrier.  (Not
            // __syncthreads(): its fence would also wait for the buffer loads just sent towards LDS.  The
            // empty statements keep the compiler from moving memory accesses across.)
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
        };
        auto run = [&](auto grp_c) {
            constexpr int G = decltype(grp_c)::value;
            // Group 0 starts with the scores of tile 0 and then reads the operands of its matrix phase 1 (K
            // tile 2, V tile 0); group 1 reads those of its matrix phase 0 (K tile 1; there is no tile -1,
            // and nothing but zeros may meet its zero probabilities).
            if (G == 0) {
#pragma unroll
                for (int s = 0; s < KS; ++s) fetch_k1(s, 0);
#pragma unroll
                for (int r = 0; r < 16; ++r) st[r] = 0.0f;
#pragma unroll
                for (int s = 0; s < KS; ++s) score_mfma(s, st);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < KS; ++s) fetch_k1(s, 2 * TILEBK);
                if (!stats_only) {
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        fetch_v1(0, dt, 0);
                        fetch_v1(1, dt, 0);
                    }
                }
            } else {
#pragma unroll
                for (int s = 0; s < KS; ++s) fetch_k1(s, TILEBK);
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int i = 0; i < 2 * DT; ++i) vfr[u][i] = s16x4{0, 0, 0, 0};
            }
            // these reads are done before phase 0 begins: its matrix phase already sends V tile 4 to the slot
            // of V tile 0
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            for (int phi = 0; phi <= last_phase; phi += 4) {
                phase(int_c<0>{}, grp_c, phi);
                if (phi + 1 > last_phase) break;
                phase(int_c<1>{}, grp_c, phi + 1);
                phase(int_c<2>{}, grp_c, phi + 2);   // last_phase is even: phases come in pairs after the first
                if (phi + 3 > last_phase) break;
                phase(int_c<3>{}, grp_c, phi + 3);
            }
        };
        if (grp == 0) run(int_c<0>{});
        else run(int_c<1>{});
        if constexpr (!KV_I8) {
            // the last phases' requests (zeros) have landed before the ring is used for anything else
            __builtin_amdgcn_s_waitcnt(0x0f70);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        if constexpr (MODE == 1) {   // this sweep's result: the row maxima; nothing to merge, nothing to store
            if (hh == 0 && my_q < S) p.row_max[((((long)b * p.Hq + h) * S + my_q) * 2) + grp] = M;
            if (has_next) request_q(p.n_rb - 1 - x);
            continue;
        }
        if (has_next) request_q(p.n_rb - 1 - x);   // in flight during the merge (every wave read its fragments of this block's Q long ago)

        // ---- merge the two groups' partial results.  A wave keeps half of its O^T tiles and hands the
        // other half, with its max and row sum, to its partner (same rows, other group) through LDS.
        // The row block's output then goes out through LDS as well: a lane holds a few values of a row of its own,
        // and stores of that shape (64 lanes, 32 rows, 8 or 16 bytes each) are taken lane by lane by the memory
        // pipe and land as partial lines.  The tile is put together in the merge records' place (once every wave
        // has read its partner's) and leaves as whole rows, 64 consecutive 16-byte pieces per instruction.
        auto finish = [&](auto grp_c) {
            constexpr int G = decltype(grp_c)::value;
            constexpr int HALF = DT / 2;
            constexpr int keep0 = G == 0 ? 0 : HALF, send0 = G == 0 ? HALF : 0;
            f32x4* mg = reinterpret_cast<f32x4*>(smem);   // [wave][NV][lane]; the ring is dead and quiet after the last barrier
            const float L = half_sum(lsum);
#pragma unroll
            for (int dt = 0; dt < HALF; ++dt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 vsend = {o[send0 + dt][4 * r4], o[send0 + dt][4 * r4 + 1], o[send0 + dt][4 * r4 + 2], o[send0 + dt][4 * r4 + 3]};
                    mg[(w8 * NV + dt * 4 + r4) * 64 + l] = vsend;
                }
            {
                const f32x4 ml = {M, L, 0.0f, 0.0f};
                mg[(w8 * NV + NV - 1) * 64 + l] = ml;
            }
            __syncthreads();
            const int pw8 = w8 ^ 4;
            const f32x4 oml = mg[(pw8 * NV + NV - 1) * 64 + l];
            const float m_all = fmaxf(M, oml[0]);
            const float a_me = fast_exp2(M - m_all), a_ot = fast_exp2(oml[0] - m_all);
            const float inv = 1.0f / (L * a_me + oml[1] * a_ot);
            const float s_me = a_me * inv, s_ot = a_ot * inv;
#pragma unroll
            for (int dt = 0; dt < HALF; ++dt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 ot = mg[(pw8 * NV + dt * 4 + r4) * 64 + l];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[keep0 + dt][4 * r4 + e] = fmaf(o[keep0 + dt][4 * r4 + e], s_me, ot[e] * s_ot);
                }
            constexpr int OB = OUT_F32 ? 4 * D : 2 * D;   // bytes per output row
            constexpr int OPITCH = OB + 16;               // tile row pitch: spreads the column-wise writes over the banks
            static_assert(kBR * OPITCH <= RING_BYTES, "the output tile fits where the ring was");
            __syncthreads();
#pragma unroll
            for (int dt = 0; dt < HALF; ++dt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    // register r of tile dt is d = 32 dt + 8 (r/4) + 4 hh + r%4
                    const int d = 32 * (keep0 + dt) + 8 * r4 + 4 * hh;
                    char* at = smem + (32 * w + l32) * OPITCH;
                    const f32x16& ok = o[keep0 + dt];
                    if (OUT_F32) {
                        const f32x4 ov = {ok[4 * r4], ok[4 * r4 + 1], ok[4 * r4 + 2], ok[4 * r4 + 3]};
                        *reinterpret_cast<f32x4*>(at + 4 * d) = ov;
                    } else {
                        u32x2 ov;
                        ov[0] = pack_bf16x2(ok[4 * r4], ok[4 * r4 + 1]);
                        ov[1] = pack_bf16x2(ok[4 * r4 + 2], ok[4 * r4 + 3]);
                        *reinterpret_cast<u32x2*>(at + 2 * d) = ov;
                    }
                }
            __syncthreads();
            constexpr int PPR = OB / 16;                           // 16-byte pieces per row
            constexpr int NST = kBR * PPR / kPrefillThreads;       // pieces per thread
            char* const obase = (char*)p.out + (((long)b * p.Hq + h) * S + i0) * (long)OB;
#pragma unroll
            for (int i = 0; i < NST; ++i) {
                // (the thread id, counted afresh: keeping it alive through the phase loops costs spills)
                const int lane_now = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
                const int pid = (w8 * 64 + lane_now) + kPrefillThreads * i, row = pid / PPR, col = pid % PPR;
                const u32x4 piece = *reinterpret_cast<const u32x4*>(smem + row * OPITCH + col * 16);
                if (i0 + row < S) *reinterpret_cast<u32x4*>(obase + (long)row * OB + col * 16) = piece;
            }
        };
        if (grp == 0) finish(int_c<0>{});
        else finish(int_c<1>{});

        // ---- the INT8 cache of this row block's own K and V rows, if asked for (section 2.2): the workgroup of
        // a KV head's first query head quantises them, 16 rows per wave, with the quantiser's row routine.
        // The rows were this row block's last tiles, so they come from the L2.
        if constexpr (!KV_I8) {
            if (p.kq != nullptr && h % (p.Hq / p.Hkv) == 0) {
                constexpr int LPR = D / 8;          // lanes per row
                constexpr int RPI = 64 / LPR;       // rows per wave-wide access
                constexpr int NJ = 16 / RPI;        // accesses per wave and tensor
                u32x4 raw[2][NJ];
#pragma unroll
                for (int ten = 0; ten < 2; ++ten) {   // all the loads first: their latencies overlap
                    const uint16_t* src = (const uint16_t*)(ten == 0 ? p.k : p.v) + kvrow0 * D;
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        const int row = i0 + 16 * w8 + RPI * j + l / LPR;
                        raw[ten][j] = *reinterpret_cast<const u32x4*>(src + (long)min(row, S - 1) * D + (l % LPR) * 8);
                    }
                }
#pragma unroll
                for (int ten = 0; ten < 2; ++ten) {
                    int8_t* codes = (ten == 0 ? p.kq : p.vq) + kvrow0 * D;
                    float* scales = (ten == 0 ? p.kqs : p.vqs) + kvrow0;
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        const int row = i0 + 16 * w8 + RPI * j + l / LPR;
                        const int piece = l % LPR;
                        u32x2 cw;
                        float scale;
                        quant_row_piece<LPR>(raw[ten][j], cw, scale);
                        if (row < S) {
                            *reinterpret_cast<u32x2*>(codes + (long)row * D + piece * 8) = cw;
                            if (piece == 0) scales[row] = scale;
                        }
                    }
                }
            }
        }
    }
}

template <int D, bool KV_I8, bool OUT_F32, int MODE = 0>
static hipError_t launch_one(const PrefillParams& p, hipStream_t stream) {
    const unsigned grid = (unsigned)(8 * p.chunk);
    hipLaunchKernelGGL((slim_prefill_kernel<D, KV_I8, OUT_F32, MODE>), dim3(grid), dim3(kPrefillThreads), 0,
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
    p.kq = a.k_codes_out;
    p.kqs = a.k_scale_out;
    p.vq = a.v_codes_out;
    p.vqs = a.v_scale_out;
    p.Hq = a.q_heads;
    p.Hkv = a.kv_heads;
    p.S = a.seq_len;
    p.causal = a.causal ? 1 : 0;
    p.n_rb = (a.seq_len + kBR - 1) / kBR;
    p.n_pair = (p.n_rb + 1) / 2;
    p.total = a.batch * a.q_heads * p.n_pair;
    p.chunk = (p.total + 7) / 8;
    p.scale_log2e = a.softmax_scale * kLog2e;
    p.row_max = a.row_max;
    if (a.row_max) {   // the comparison variant: bf16 K/V only (checked by the caller); two launches
        hipError_t e = a.head_dim == 128 ? launch_one<128, false, false, 1>(p, stream) : launch_one<64, false, false, 1>(p, stream);
        if (e != hipSuccess) return e;
        if (a.head_dim == 128) return a.out_f32 ? launch_one<128, false, true, 2>(p, stream) : launch_one<128, false, false, 2>(p, stream);
        return a.out_f32 ? launch_one<64, false, true, 2>(p, stream) : launch_one<64, false, false, 2>(p, stream);
    }
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

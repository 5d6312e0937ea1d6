// Prefill attention in the order of operations the paper gives (section 2.1), with the whole score strip of a
// row block on chip: a block of query rows times ALL its keys goes into one buffer, the softmax is applied to
// that buffer (one maximum, one pass of exponentials, one sum: no running maximum, nothing is ever rescaled),
// and the buffer times V is the block's slice of the output; the next block reuses the buffer.  A comparison
// variant of slim_prefill_kernel, which never holds more than a 32-key tile of a row block's scores.
//
// The buffer is LDS: 32 query rows x up to 2048 keys x 2 bytes = 128 KB of the compute unit's 160 KB, which is
// what fixes the block at 32 rows.  One workgroup (8 waves, two per SIMD) owns a row block:
//   pass 1  scores.  Wave w takes the 32-key tiles t = w, w + 8, ...: S^T = K Q^T on v_mfma_f32_32x32x16_bf16,
//           the K tile as A operand straight from global memory (lane = key, 16-byte pieces of its row), Q^T as B
//           operand in registers.  Scaled to log2 units, masked, and written to the strip as fp16, each tile
//           relative to a reference of its own (kept per tile and row in a small table); the row maxima are kept
//           on the way (in-lane, then across the wave's halves, then across the waves).
//   pass 2  softmax over the strip, in place: p = exp2(u - max) in fp32, summed in fp32, rounded to bf16 over
//           the fp16 score it came from.  Pure vector work, all 512 threads.
//   pass 3  strip times V.  A wave takes one 32-column slice of the head dimension and one tile position of every
//           chunk (D = 128: 4 slices x 2 tiles of a 64-key chunk; D = 64: 2 slices x 4 tiles of a 128-key chunk),
//           and brings in just that piece of V itself (128-bit loads, three chunks ahead in registers, an LDS
//           region of its own, so no barriers): O^T += V^T P^T with P^T read from the strip as it stands (B
//           operand: lane = query, 8 consecutive keys) and V^T through the LDS transpose read.  The tile
//           positions of a slice are added at the end, divided by the row sum and stored.
// A score waits in the strip as the fp16 of u - ref, ref being the wave's row maximum up to and including the
// score's own tile: never positive, small exactly where the probability is not, so the 11 significant bits cost
// less than 2^-11 of log2(1/p) in the exponent (at most 0.4 % of a probability near 2^-8, less above and nothing
// that matters below), whatever the magnitude of the scores.  Differences below -65000 (probability 0 in any
// arithmetic) and masked keys are written as -65000.
#include "slim_common.h"
#include "slim_kernels.h"

namespace slim {

constexpr int kStripRows = 32;     // query rows per row block
constexpr int kStripTile = 32;     // keys per score tile
constexpr int kStripWaves = 8;     // waves per workgroup
constexpr float kStripClamp = 65000.0f;

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

struct StripParams {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    void* out;
    int Hq, Hkv, S, causal, n_rb, total, chunk;
    float scale_log2e;
};

template <int CTRL>
__device__ __forceinline__ float strip_dpp(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// NC: key columns the strip has room for (the sequence length rounded up, one of a few size classes)
template <int D, int NC, bool OUT_F32>
__global__ __launch_bounds__(64 * kStripWaves) void slim_prefill_strip_kernel(const StripParams p) {
    constexpr int NW = kStripWaves;
    constexpr int KS = D / 16;          // k-steps of a score tile
    constexpr int DT = D / 32;          // 32-column slices of the head dimension (32-row tiles of O^T): a wave takes one
    constexpr int NTP = NW / DT;        // tile positions of a V chunk: the waves that share a slice
    constexpr int CHUNK = kStripTile * NTP;   // keys per V chunk
    static_assert(NW % DT == 0, "slices times tile positions = waves");
    constexpr int ROWB = 2 * D;         // bytes per K/V row in memory
    constexpr int SROW = 2 * NC + 16;   // strip row pitch: the padding shifts every row by 16 bytes, so the 128-bit reads of 16 rows meet 16 different bank groups
    constexpr int STRIP_BYTES = kStripRows * SROW;
    constexpr int PITCH = 64 + 16;      // staged V row pitch: a 32-column slice of a row, padded
    constexpr int STAGE_BYTES = NW * kStripTile * PITCH;   // V staging: a region of 32 row slices per wave
    constexpr int REF_BYTES = (NC / kStripTile) * 32 * 4;   // one reference per tile and row
    static_assert(NC % CHUNK == 0, "the strip holds whole chunks");
    static_assert(STRIP_BYTES >= NW * 4 * 64 * 16, "the partial outputs are merged in the strip's place");

    __shared__ __attribute__((aligned(16))) char smem[STRIP_BYTES + STAGE_BYTES + REF_BYTES + (NW * 32 + 32 + 32) * 4];
    char* const strip = smem;
    char* const stage = smem + STRIP_BYTES;
    float* const refS = reinterpret_cast<float*>(stage + STAGE_BYTES);   // [tile][32 rows] what a tile's scores are relative to
    float* const mS = refS + (NC / kStripTile) * 32;                      // [waves][32 rows] maxima of pass 1
    float* const mrow = mS + NW * 32;                                     // [32] the rows' maxima
    float* const lrow = mrow + 32;                                        // [32] the rows' sums

    // workgroup -> (batch*head, row block); consecutive virtual ids (the row blocks of a head, which share K/V)
    // are steered to one XCD (hardware deals workgroup ids round-robin over the 8 XCDs).  Under the causal mask
    // a head's long row blocks come first.
    int bh, rb;
    {
        const int n = (int)blockIdx.x;
        const int vid = (n % 8) * p.chunk + n / 8;
        if (vid >= p.total) return;
        bh = vid / p.n_rb;
        rb = vid % p.n_rb;
        if (p.causal) rb = p.n_rb - 1 - rb;
    }
    const int b = bh / p.Hq, h = bh % p.Hq;
    const int g = h / (p.Hq / p.Hkv);
    const int S = p.S;
    const float c = p.scale_log2e;
    const int tid = (int)threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l = tid & 63, l32 = l & 31, hh = l >> 5;
    const int i0 = rb * kStripRows;
    const int my_q = i0 + l32;                                // this lane's query row (may be >= S in the last block)
    const int lim = p.causal ? min(my_q, S - 1) : S - 1;      // last key this lane's row may see
    const int kend = p.causal ? min(S, i0 + kStripRows) : S;  // keys this row block attends to
    const int n_tiles = (kend + kStripTile - 1) / kStripTile;
    const int n_keys = n_tiles * kStripTile;                  // strip columns in use (whole tiles)
    const long kvrow0 = ((long)b * p.Hkv + g) * (long)S;

    // buffer descriptors over exactly this head's K and V slabs: rows past the end read as zero
    const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc((void*)(p.k + kvrow0 * D), 0, (int)((unsigned)S * ROWB), 0x00020000);
    const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc((void*)(p.v + kvrow0 * D), 0, (int)((unsigned)S * ROWB), 0x00020000);

    // ---- pass 1: the score strip.  Q^T B operands: lane holds row my_q, d = 16 s + 8 hh + [0,8); the same for every
    // wave.  The block's 32 rows are loaded once, 64 consecutive 16-byte pieces per instruction, into the V staging
    // buffer (idle until pass 3) and every wave reads its fragments from there: eight waves each loading a row per
    // lane would keep the memory pipe busy lane by lane for some four thousand cycles per workgroup.
    bf16x8 qreg[KS];
    {
        constexpr int CPQ = ROWB / 16;              // 16-byte pieces per Q row
        constexpr int QPITCH = ROWB + 16;           // staged row pitch: 16 rows' 128-bit reads meet 16 different bank groups
        static_assert(kStripRows * QPITCH <= STAGE_BYTES, "the Q rows fit the staging buffer");
        const __amdgpu_buffer_rsrc_t qrs = __builtin_amdgcn_make_buffer_rsrc((void*)(p.q + ((long)b * p.Hq + h) * (long)S * D), 0, (int)((unsigned)S * ROWB), 0x00020000);
        for (int pid = tid; pid < kStripRows * CPQ; pid += 64 * NW) {
            const int row = pid / CPQ, col = pid % CPQ;   // (rows past the end of the sequence read as zero)
            const u32x4 piece = __builtin_amdgcn_raw_buffer_load_b128(qrs, (i0 + row) * ROWB + col * 16, 0, 0);
            *reinterpret_cast<u32x4*>(stage + row * QPITCH + col * 16) = piece;
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < KS; ++s) qreg[s] = *reinterpret_cast<const bf16x8*>(stage + l32 * QPITCH + 32 * s + 16 * hh);
    }
    // K fragment of k-step s of tile t: lane = key 32 t + l32, bytes 32 s + 16 hh + [0,16) of its row
    auto load_k = [&](int t, u32x4 (&dst)[KS]) {
        const int off = (t * kStripTile + l32) * ROWB + 16 * hh;
#pragma unroll
        for (int s = 0; s < KS; ++s) dst[s] = __builtin_amdgcn_raw_buffer_load_b128(krs, off + 32 * s, 0, 0);
    };
    float m = kMasked;   // this wave's running row maximum (log2 units), the same in both halves of the wave
    // (three tiles' fragments are in flight per wave)
    constexpr int KDEPTH = 3;
    u32x4 kf[KDEPTH][KS];
#pragma unroll
    for (int j = 0; j < KDEPTH; ++j)
        if (w + NW * j < n_tiles) load_k(w + NW * j, kf[j]);
    auto score_tile = [&](int t, u32x4 (&kfr)[KS]) {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kfr[s]), qreg[s], acc, 0, 0, 0);
        if (t + NW * KDEPTH < n_tiles) load_k(t + NW * KDEPTH, kfr);   // the registers are free again: the tile three turns ahead
        // register r of this lane is key 32 t + 8 (r/4) + 4 hh + r%4 of query row my_q
        const int rel = lim - (t * kStripTile + 4 * hh);   // keys of this lane up to offset rel are visible
        float u[16];
        float tm = kMasked;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            u[r] = (8 * (r / 4) + (r % 4) <= rel) ? acc[r] * c : kMasked;
            tm = fmaxf(tm, u[r]);
        }
        m = fmaxf(m, half_max(tm));   // (every tile a wave meets holds a visible key of every row)
        if (hh == 0) refS[t * 32 + l32] = m;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            f16x4 hv;
#pragma unroll
            for (int e = 0; e < 4; ++e) hv[e] = (_Float16)fmaxf(u[4 * r4 + e] - m, -kStripClamp);
            *reinterpret_cast<f16x4*>(strip + l32 * SROW + (t * kStripTile + 8 * r4 + 4 * hh) * 2) = hv;
        }
    };
    for (int t = w; t < n_tiles; t += NW * KDEPTH) {
#pragma unroll
        for (int j = 0; j < KDEPTH; ++j)
            if (t + NW * j < n_tiles) score_tile(t + NW * j, kf[j]);
    }
    if (hh == 0) mS[w * 32 + l32] = m;   // (a wave without tiles leaves the stand-in for minus infinity)
    __syncthreads();
    if (tid < 32) {
        float mx = mS[tid];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) mx = fmaxf(mx, mS[ww * 32 + tid]);
        mrow[tid] = mx;
    }
    __syncthreads();

    // ---- pass 2: softmax over the strip, in place.  Thread = (row tid / 16, 8-key groups tid % 16, +16, ...).
    {
        const int row = tid >> 4;
        const float mr = mrow[row];
        float sum = 0.0f;
        for (int j = (tid & 15) * 8; j < n_keys; j += 128) {
            char* at = strip + row * SROW + j * 2;
            const f16x8 u8 = *reinterpret_cast<const f16x8*>(at);
            const float shift = refS[(j / kStripTile) * 32 + row] - mr;   // the tile's reference against the row's maximum
            float pr[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pr[e] = fast_exp2((float)u8[e] + shift);
                sum += pr[e];
            }
            u32x4 pk;
#pragma unroll
            for (int e = 0; e < 4; ++e) pk[e] = pack_bf16x2(pr[2 * e], pr[2 * e + 1]);
            *reinterpret_cast<u32x4*>(at) = pk;
        }
        sum += strip_dpp<0xB1>(sum);    // quad_perm [1,0,3,2]
        sum += strip_dpp<0x4E>(sum);    // quad_perm [2,3,0,1]
        sum += strip_dpp<0x141>(sum);   // row_half_mirror: the other quad of the eight
        sum += strip_dpp<0x140>(sum);   // row_mirror: the other eight of the row's 16 threads
        if ((tid & 15) == 0) lrow[row] = sum;
    }
    __syncthreads();

    // ---- pass 3: strip times V.  Wave (tpos, dq) needs, of every chunk, the 32 keys at its tile position and its
    // 32-column slice of the head dimension: it loads exactly that piece (4 lanes per row, 64 bytes of it), stages it
    // in an LDS region of its own and reads it back through the transpose read.  No other wave touches the region
    // and LDS runs a wave's accesses in order, so the pass needs no barrier at all.
    const int tpos = w % NTP, dq = w / NTP;
    constexpr int NPV = 2;                               // 128-bit loads per lane and chunk: 16 rows each
    char* const mine = stage + w * (kStripTile * PITCH);
    auto load_v = [&](int ch, u32x4 (&dst)[NPV]) {
#pragma unroll
        for (int i = 0; i < NPV; ++i) {
            const int row = 16 * i + l / 4, col = l % 4;
            dst[i] = __builtin_amdgcn_raw_buffer_load_b128(vrs, (ch * CHUNK + kStripTile * tpos + row) * ROWB + 64 * dq + col * 16, 0, 0);
        }
    };
    auto store_v = [&](const u32x4 (&src)[NPV]) {
#pragma unroll
        for (int i = 0; i < NPV; ++i) {
            const int row = 16 * i + l / 4, col = l % 4;
            *reinterpret_cast<u32x4*>(mine + row * PITCH + col * 16) = src[i];
        }
    };
    f32x16 o;
#pragma unroll
    for (int r = 0; r < 16; ++r) o[r] = 0.0f;
    // V^T A operand of 16 keys x 32 columns: the 16 lanes of a group fetch 4 rows (4 lanes per row, 8 bytes each)
    // and lane i of the group receives column i of those rows; this lane's rows are 8 hh + [0,4) and + 4.
    const int v_addr = (8 * hh + ((l & 15) >> 2)) * PITCH + (2 * ((l >> 4) & 1) + ((l & 3) >> 1)) * 16 + 8 * (l & 1);
    const int n_chunks = (n_keys + CHUNK - 1) / CHUNK;
    constexpr int VDEPTH = 3;   // chunks in registers ahead of the one in LDS
    u32x4 vst[VDEPTH][NPV];
#pragma unroll
    for (int j = 0; j < VDEPTH; ++j)
        if (j < n_chunks) load_v(j, vst[j]);
    auto chunk = [&](int ch, u32x4 (&vreg)[NPV]) {
        store_v(vreg);
        if (ch + VDEPTH < n_chunks) load_v(ch + VDEPTH, vreg);
        const int kb = ch * CHUNK + kStripTile * tpos;   // first key of this wave's tile
        if (kb < n_keys) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                // P^T B operand: lane = query row l32, keys kb + 16 ks + 8 hh + [0,8)
                const bf16x8 pb = *reinterpret_cast<const bf16x8*>(strip + l32 * SROW + (kb + 16 * ks + 8 * hh) * 2);
                const char* va = mine + v_addr + 16 * ks * PITCH;
                const s16x4 lo = lds_read_tr16(reinterpret_cast<const uint16_t*>(va));
                const s16x4 hi = lds_read_tr16(reinterpret_cast<const uint16_t*>(va + 4 * PITCH));
                const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb, o, 0, 0, 0);
            }
        }
    };
    for (int ch = 0; ch < n_chunks; ch += VDEPTH) {
#pragma unroll
        for (int j = 0; j < VDEPTH; ++j)
            if (ch + j < n_chunks) chunk(ch + j, vst[j]);
    }
    __syncthreads();   // every wave is done with the strip, whose place the merge below takes

    // ---- the tile positions of each slice are added (through the strip's place: the strip is dead), divided by
    // the row sum and stored.  Register r is d = 32 dq + 8 (r/4) + 4 hh + r%4 of row my_q.
    f32x4* const mg = reinterpret_cast<f32x4*>(smem);   // [wave][r4][lane]
    if (tpos != 0) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const f32x4 vsend = {o[4 * r4], o[4 * r4 + 1], o[4 * r4 + 2], o[4 * r4 + 3]};
            mg[(w * 4 + r4) * 64 + l] = vsend;
        }
    }
    __syncthreads();
    // The finished rows go out through the staging buffer (idle again) as whole rows, 64 consecutive 16-byte pieces
    // per instruction: stores of a few values per lane and row are taken lane by lane by the memory pipe.
    constexpr int OB = OUT_F32 ? 4 * D : 2 * D;   // bytes per output row
    constexpr int OPITCH = OB + 16;
    static_assert(kStripRows * OPITCH <= STAGE_BYTES, "the output tile fits the staging buffer");
    if (tpos == 0) {
        const float inv = 1.0f / lrow[l32];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            float xo[4] = {o[4 * r4], o[4 * r4 + 1], o[4 * r4 + 2], o[4 * r4 + 3]};
#pragma unroll
            for (int t2 = 1; t2 < NTP; ++t2) {   // in the order of the tile positions
                const f32x4 ot = mg[((w + t2) * 4 + r4) * 64 + l];
#pragma unroll
                for (int e = 0; e < 4; ++e) xo[e] += ot[e];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) xo[e] *= inv;
            const int d = 32 * dq + 8 * r4 + 4 * hh;
            char* at = stage + l32 * OPITCH;
            if (OUT_F32) {
                const f32x4 ov = {xo[0], xo[1], xo[2], xo[3]};
                *reinterpret_cast<f32x4*>(at + 4 * d) = ov;
            } else {
                u32x2 ov;
                ov[0] = pack_bf16x2(xo[0], xo[1]);
                ov[1] = pack_bf16x2(xo[2], xo[3]);
                *reinterpret_cast<u32x2*>(at + 2 * d) = ov;
            }
        }
    }
    __syncthreads();
    {
        constexpr int PPR = OB / 16;   // 16-byte pieces per row
        char* const obase = (char*)p.out + (((long)b * p.Hq + h) * S + i0) * (long)OB;
        for (int pid = tid; pid < kStripRows * PPR; pid += 64 * NW) {
            const int row = pid / PPR, col = pid % PPR;
            const u32x4 piece = *reinterpret_cast<const u32x4*>(stage + row * OPITCH + col * 16);
            if (i0 + row < S) *reinterpret_cast<u32x4*>(obase + (long)row * OB + col * 16) = piece;
        }
    }
}

template <int D, int NC>
static hipError_t launch_strip_nc(const StripParams& p, bool out_f32, hipStream_t stream) {
    const unsigned grid = (unsigned)(8 * p.chunk);
    if (out_f32) hipLaunchKernelGGL((slim_prefill_strip_kernel<D, NC, true>), dim3(grid), dim3(64 * kStripWaves), 0, stream, p);
    else hipLaunchKernelGGL((slim_prefill_strip_kernel<D, NC, false>), dim3(grid), dim3(64 * kStripWaves), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_prefill_strip(const PrefillArgs& a, hipStream_t stream) {
    StripParams p;
    p.q = (const uint16_t*)a.q;
    p.k = (const uint16_t*)a.k;
    p.v = (const uint16_t*)a.v;
    p.out = a.out;
    p.Hq = a.q_heads;
    p.Hkv = a.kv_heads;
    p.S = a.seq_len;
    p.causal = a.causal ? 1 : 0;
    p.n_rb = (a.seq_len + kStripRows - 1) / kStripRows;
    p.total = a.batch * a.q_heads * p.n_rb;
    p.chunk = (p.total + 7) / 8;
    p.scale_log2e = a.softmax_scale * kLog2e;
    // the strip's size class: short sequences leave room for two or three workgroups per compute unit
    static_assert(kPrefillStripMaxSeqLen == 2048, "the largest size class below");
    const int S = a.seq_len;
    if (a.head_dim == 128) {
        if (S <= 512) return launch_strip_nc<128, 512>(p, a.out_f32, stream);
        if (S <= 1024) return launch_strip_nc<128, 1024>(p, a.out_f32, stream);
        return launch_strip_nc<128, 2048>(p, a.out_f32, stream);
    }
    if (S <= 512) return launch_strip_nc<64, 512>(p, a.out_f32, stream);
    if (S <= 1024) return launch_strip_nc<64, 1024>(p, a.out_f32, stream);
    return launch_strip_nc<64, 2048>(p, a.out_f32, stream);
}

}  // namespace slim

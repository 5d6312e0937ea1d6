// INT8 KV-cache quantiser (paper section 2.2: INT8 K/V, one scale per token per head).
//
// One row of D bf16 values (one token of one head) is held by D/8 adjacent lanes, 16
// bytes each.  amax is reduced across those lanes; scale = amax / 127 and
// code = rint(x / scale) are defined by IEEE fp32 division (correctly rounded, denormals
// kept), so that codes and scales are reproducible bit for bit on any IEEE machine; the row
// routine reaches those bits by a shorter route wherever that is proved to be safe and by the
// divisions themselves elsewhere (slim_common.h).
// Streaming kernel: 2 B read + 1 B written per element, plus 4 B per row.
#include "slim_common.h"
#include "slim_kernels.h"

namespace slim {

// STREAM: input and output together are larger than the last-level cache, so the input is read with
// non-temporal loads and every thread keeps U = 4 rows in flight (all loads issued before any is used): 5.6 TB/s on
// a 1.6 GB stream, where the same loads and stores with no arithmetic in between reach 5.9.  A smaller input may
// be what the next kernel reads again (the K/V of a prefill): it is left to the caches, one row per thread, which
// finishes a launch-bound call soonest.
template <int D, bool STREAM, int U>
__device__ __forceinline__ void kv_quant_rows(const uint16_t* __restrict__ x, int8_t* __restrict__ codes,
                                              float* __restrict__ scales, long n_rows) {
    constexpr int LPR = D / 8;           // lanes per row
    constexpr int ROWS = 256 / LPR;      // rows per workgroup and load
    const int lane_in_row = threadIdx.x % LPR;
    const long stride = (long)gridDim.x * (ROWS * U);
    // (rows past the end re-read the last row and store nothing: every lane stays in the loop as long as its
    // wave does, so the row routine's shuffles and its wave-wide vote see whole waves)
    const long first = (long)blockIdx.x * (ROWS * U);
    for (long base = first; base < n_rows; base += stride) {
        const long row0 = base + threadIdx.x / LPR;
        u32x4 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long row = min(row0 + (long)u * ROWS, n_rows - 1);
            const u32x4* src = reinterpret_cast<const u32x4*>(x + row * D + lane_in_row * 8);
            raw[u] = STREAM ? __builtin_nontemporal_load(src) : *src;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long row = row0 + (long)u * ROWS;
            u32x2 out2;
            float scale;
            quant_row_piece<LPR>(raw[u], out2, scale);
            if (row < n_rows) {
                *reinterpret_cast<u32x2*>(codes + row * D + lane_in_row * 8) = out2;
                if (lane_in_row == 0) scales[row] = scale;
            }
        }
    }
}

template <int D, bool STREAM, int U>
__global__ __launch_bounds__(256) void kv_quant_int8_kernel(const uint16_t* __restrict__ x, int8_t* __restrict__ codes,
                                                            float* __restrict__ scales, long n_rows) {
    kv_quant_rows<D, STREAM, U>(x, codes, scales, n_rows);
}

// Two tensors of the same shape in one launch (the K and the V of a cache): blockIdx.y picks the tensor.  On
// inputs of a few megabytes a call is launch-bound, and one launch does the work of two in little more than the
// time of one.
struct QuantPair {
    const uint16_t* x[2];
    int8_t* codes[2];
    float* scales[2];
};
template <int D, bool STREAM, int U>
__global__ __launch_bounds__(256) void kv_quant_int8_pair_kernel(const QuantPair p, long n_rows) {
    const int t = (int)blockIdx.y;   // uniform
    kv_quant_rows<D, STREAM, U>(t == 0 ? p.x[0] : p.x[1], t == 0 ? p.codes[0] : p.codes[1], t == 0 ? p.scales[0] : p.scales[1], n_rows);
}

// One new token per (batch, KV head): row r = b * Hkv + g of x goes to token positions[b] of that head's cache.
template <int D>
__global__ __launch_bounds__(256) void kv_quant_int8_append_kernel(const uint16_t* __restrict__ x, int8_t* __restrict__ codes,
                                                                   float* __restrict__ scales,
                                                                   const int* __restrict__ positions, int n_rows, int Hkv,
                                                                   int T) {
    constexpr int LPR = D / 8;
    constexpr int ROWS = 256 / LPR;
    const int lane_in_row = threadIdx.x % LPR;
    const int row = blockIdx.x * ROWS + threadIdx.x / LPR;
    if (row >= n_rows) return;   // (whole row groups leave together: the shuffles below stay inside a row)
    const u32x4 raw = *reinterpret_cast<const u32x4*>(x + (long)row * D + lane_in_row * 8);
    u32x2 out2;
    float scale;
    quant_row_piece<LPR>(raw, out2, scale);
    const int pos = positions[row / Hkv];
    if (pos < 0 || pos >= T) return;   // no room in this sequence's cache: nothing is written
    const long out_row = (long)row * T + pos;
    *reinterpret_cast<u32x2*>(codes + out_row * D + lane_in_row * 8) = out2;
    if (lane_in_row == 0) scales[out_row] = scale;
}

hipError_t launch_kv_quant_int8(const void* x, int8_t* codes, float* scales, long n_rows, int head_dim,
                                hipStream_t stream) {
    const bool stream_in = n_rows * head_dim * 3 > (256L << 20);   // input + codes beyond the 256 MB last-level cache
    const int rows_per_block = 256 / (head_dim / 8) * (stream_in ? 4 : 1);
    long blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    // one pass per workgroup (measured faster than fewer workgroups that loop); the loop is for grids beyond this
    const long max_blocks = 1L << 20;
    if (blocks > max_blocks) blocks = max_blocks;
    const dim3 grid((unsigned)blocks), block(256);
    if (head_dim == 128) {
        if (stream_in) hipLaunchKernelGGL((kv_quant_int8_kernel<128, true, 4>), grid, block, 0, stream, (const uint16_t*)x, codes, scales, n_rows);
        else hipLaunchKernelGGL((kv_quant_int8_kernel<128, false, 1>), grid, block, 0, stream, (const uint16_t*)x, codes, scales, n_rows);
    } else {
        if (stream_in) hipLaunchKernelGGL((kv_quant_int8_kernel<64, true, 4>), grid, block, 0, stream, (const uint16_t*)x, codes, scales, n_rows);
        else hipLaunchKernelGGL((kv_quant_int8_kernel<64, false, 1>), grid, block, 0, stream, (const uint16_t*)x, codes, scales, n_rows);
    }
    return hipGetLastError();
}

hipError_t launch_kv_quant_int8_pair(const void* k, const void* v, int8_t* k_codes, float* k_scale, int8_t* v_codes,
                                     float* v_scale, long n_rows, int head_dim, hipStream_t stream) {
    const bool stream_in = 2 * n_rows * head_dim * 3 > (256L << 20);   // both inputs + both code tensors beyond the last-level cache
    const int rows_per_block = 256 / (head_dim / 8) * (stream_in ? 4 : 1);
    long blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    const long max_blocks = 1L << 20;
    if (blocks > max_blocks) blocks = max_blocks;
    const dim3 grid((unsigned)blocks, 2u), block(256);
    QuantPair p;
    p.x[0] = (const uint16_t*)k;
    p.x[1] = (const uint16_t*)v;
    p.codes[0] = k_codes;
    p.codes[1] = v_codes;
    p.scales[0] = k_scale;
    p.scales[1] = v_scale;
    if (head_dim == 128) {
        if (stream_in) hipLaunchKernelGGL((kv_quant_int8_pair_kernel<128, true, 4>), grid, block, 0, stream, p, n_rows);
        else hipLaunchKernelGGL((kv_quant_int8_pair_kernel<128, false, 1>), grid, block, 0, stream, p, n_rows);
    } else {
        if (stream_in) hipLaunchKernelGGL((kv_quant_int8_pair_kernel<64, true, 4>), grid, block, 0, stream, p, n_rows);
        else hipLaunchKernelGGL((kv_quant_int8_pair_kernel<64, false, 1>), grid, block, 0, stream, p, n_rows);
    }
    return hipGetLastError();
}

hipError_t launch_kv_quant_int8_append(const void* x, int8_t* codes, float* scales, const int* positions, int batch,
                                       int kv_heads, int kv_len, int head_dim, hipStream_t stream) {
    const int n_rows = batch * kv_heads;
    const int rows_per_block = 256 / (head_dim / 8);
    const unsigned blocks = (unsigned)((n_rows + rows_per_block - 1) / rows_per_block);
    if (head_dim == 128)
        hipLaunchKernelGGL(kv_quant_int8_append_kernel<128>, dim3(blocks), dim3(256), 0, stream, (const uint16_t*)x, codes,
                           scales, positions, n_rows, kv_heads, kv_len);
    else
        hipLaunchKernelGGL(kv_quant_int8_append_kernel<64>, dim3(blocks), dim3(256), 0, stream, (const uint16_t*)x, codes,
                           scales, positions, n_rows, kv_heads, kv_len);
    return hipGetLastError();
}

}  // namespace slim

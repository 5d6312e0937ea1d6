// Measurement kernels (declared in include/slimprobe.h): a plain streaming read, the quantiser's traffic without
// its arithmetic, and back-to-back bf16 MFMAs with a cycle counter.  Not part of the attention path.
#include "../../include/slimprobe.h"

#include "slim_common.h"
#include "slim_kernels.h"

namespace slim {

__global__ __launch_bounds__(256) void probe_stream_read_kernel(const u32x4* __restrict__ src, long n16, u32x4* sink) {
    constexpr int U = 4;
    const long stride = (long)gridDim.x * 256 * U;
    u32x4 x = {0u, 0u, 0u, 0u};
    for (long base = (long)blockIdx.x * 256 * U + threadIdx.x; base < n16; base += stride) {
        u32x4 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long i = base + 256L * u;
            r[u] = i < n16 ? __builtin_nontemporal_load(src + i) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < U; ++u) x ^= r[u];
    }
    if (x[0] == 0x9e3779b9u && x[1] == 0x7f4a7c15u && x[2] == 0xf39cc060u && x[3] == 0x5cedc834u) *sink = x;
}

template <int D>
__global__ __launch_bounds__(256) void probe_quant_traffic_kernel(const uint16_t* __restrict__ x, int8_t* __restrict__ codes,
                                                                  float* __restrict__ scales, long n_rows) {
    constexpr int LPR = D / 8, ROWS = 256 / LPR, U = 4;
    const int lane_in_row = threadIdx.x % LPR;
    const long stride = (long)gridDim.x * (ROWS * U);
    for (long base = (long)blockIdx.x * (ROWS * U); base < n_rows; base += stride) {
        const long row0 = base + threadIdx.x / LPR;
        u32x4 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long row = min(row0 + (long)u * ROWS, n_rows - 1);
            raw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + row * D + lane_in_row * 8));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long row = row0 + (long)u * ROWS;
            if (row < n_rows) {
                u32x2 o;
                o[0] = raw[u][0] ^ raw[u][1];
                o[1] = raw[u][2] ^ raw[u][3];
                *reinterpret_cast<u32x2*>(codes + row * D + lane_in_row * 8) = o;
                if (lane_in_row == 0) scales[row] = __uint_as_float(raw[u][0] & 0x3fffffffu);
            }
        }
    }
}

__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(const u32x4* __restrict__ a, const u32x4* __restrict__ b,
                                                              int slices, float* __restrict__ out, int iters) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int slice = (int)((4L * blockIdx.x + w) % slices);
    const bf16x8 fa = __builtin_bit_cast(bf16x8, a[slice * 64 + lane]);
    const bf16x8 fb = __builtin_bit_cast(bf16x8, b[slice * 64 + lane]);
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    const long t0 = (long)__builtin_amdgcn_s_memtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int rep = 0; rep < 4; ++rep)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[j], 0, 0, 0);
    }
    const long t1 = (long)__builtin_amdgcn_s_memtime();
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    if (lane == 0) {
        out[(4L * blockIdx.x + w) * 2] = s;
        out[(4L * blockIdx.x + w) * 2 + 1] = (float)(t1 - t0);
    }
}

}  // namespace slim

namespace {
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
}  // namespace

extern "C" {

int slim_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || bytes == 0 || bytes % 16 != 0 || misaligned(src) || misaligned(sink)) return 1;
    const long n16 = (long)(bytes / 16);
    long blocks = (n16 + 1023) / 1024;
    if (blocks > 256L * 32) blocks = 256L * 32;
    (void)hipGetLastError();
    hipLaunchKernelGGL(slim::probe_stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const slim::u32x4*)src, n16, (slim::u32x4*)sink);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

int slim_probe_quant_traffic(const void* x_bf16, int8_t* codes, float* scales, long n_rows, int head_dim, void* stream) {
    if (!x_bf16 || !codes || !scales || n_rows <= 0 || (head_dim != 64 && head_dim != 128)) return 1;
    if (misaligned(x_bf16) || misaligned(codes) || misaligned(scales)) return 1;
    const int rows_per_block = 256 / (head_dim / 8) * 4;
    long blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    if (blocks > (1L << 20)) blocks = 1L << 20;
    (void)hipGetLastError();
    if (head_dim == 128)
        hipLaunchKernelGGL(slim::probe_quant_traffic_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           (const uint16_t*)x_bf16, codes, scales, n_rows);
    else
        hipLaunchKernelGGL(slim::probe_quant_traffic_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           (const uint16_t*)x_bf16, codes, scales, n_rows);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

int slim_probe_mfma_bf16(const void* a, const void* b, int slices, float* out, int workgroups, int iters, void* stream) {
    if (!a || !b || !out || slices <= 0 || workgroups <= 0 || iters <= 0 || misaligned(a) || misaligned(b) || misaligned(out)) return 1;
    (void)hipGetLastError();
    hipLaunchKernelGGL(slim::probe_mfma_bf16_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream,
                       (const slim::u32x4*)a, (const slim::u32x4*)b, slices, out, iters);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

int slim_probe_gqa_decode_traffic(const void* q_bf16, const int8_t* k_codes, const float* k_scale, const int8_t* v_codes,
                                  const float* v_scale, void* workspace, size_t workspace_bytes, int batch, int q_heads,
                                  int kv_heads, int kv_len, int head_dim, void* stream) {
    if (!q_bf16 || !k_codes || !k_scale || !v_codes || !v_scale || !workspace) return 1;
    if (batch <= 0 || q_heads <= 0 || kv_heads <= 0 || kv_len <= 0 || (head_dim != 64 && head_dim != 128)) return 1;
    if (q_heads % kv_heads != 0 || q_heads / kv_heads < 2 || q_heads / kv_heads > 32) return 1;   // the shapes the grouped kernel serves
    if (misaligned(q_bf16) || misaligned(k_codes) || misaligned(k_scale) || misaligned(v_codes) || misaligned(v_scale) || misaligned(workspace)) return 1;
    const int n_split = slim::decode_gqa_num_splits(kv_len, (long)batch * kv_heads);
    const size_t n_part = (size_t)batch * q_heads * n_split;
    if (workspace_bytes < n_part * ((size_t)head_dim + 2) * sizeof(float)) return 1;
    slim::DecodeArgs a;
    a.q = q_bf16;
    a.k_codes = k_codes;
    a.k_scale = k_scale;
    a.v_codes = v_codes;
    a.v_scale = v_scale;
    a.out = nullptr;
    a.workspace = (float*)workspace;
    a.kv_lens = nullptr;
    a.batch = batch;
    a.q_heads = q_heads;
    a.kv_heads = kv_heads;
    a.kv_len = kv_len;
    a.head_dim = head_dim;
    a.softmax_scale = 1.0f;
    (void)hipGetLastError();
    const hipError_t e = slim::launch_decode_gqa_split(a, a.workspace, a.workspace + n_part * head_dim, n_split, (hipStream_t)stream, true);
    return e == hipSuccess ? 0 : 2;
}

}  // extern "C"

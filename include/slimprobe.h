/*
 * slimprobe.h — C ABI of four measurement kernels for AMD MI355X (gfx950).
 *
 * They are not part of the attention path.  They exist so that the ceilings the path's kernels are judged
 * against on a given machine (what a plain streaming read reaches of the HBM peak, what the quantiser's
 * read-two-write-one stream reaches without its arithmetic, what back-to-back bf16 MFMAs reach of the matrix
 * peak and at which clock, on operands of different bit activity) are measured by the same harness that
 * measures the kernels: `bench.py --probe ceilings` calls them.
 *
 * Every pointer is device memory owned by the caller, 16-byte aligned.  `stream` is a hipStream_t passed as
 * void* (NULL = the default stream); work is enqueued on it, nothing synchronises, allocates or frees.
 * Return value: 0, or 1 for a bad argument (nothing enqueued), 2 if the launch failed.
 */
#ifndef SLIMPROBE_H
#define SLIMPROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads `bytes` bytes (a multiple of 16) at src once, with 128-bit non-temporal loads, every lane 16 bytes
 * per load and four loads in flight; the XOR of everything read goes to sink[0..3] of the one lane (if any)
 * whose XOR happens to equal a fixed pattern, which keeps the loads alive and writes next to nothing.
 * sink: at least 16 bytes.
 */
int slim_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream);

/*
 * The traffic of kv_quant_int8 without its arithmetic: reads n_rows rows of head_dim bf16 values (16 bytes per
 * lane, non-temporal, four rows per thread in flight), writes head_dim bytes per row (8 per lane, XORs of what
 * was read) and one 4-byte word per row.  head_dim 64 or 128.
 */
int slim_probe_quant_traffic(const void* x_bf16, int8_t* codes, float* scales, long n_rows, int head_dim, void* stream);

/*
 * Back-to-back v_mfma_f32_32x32x16_bf16 on the matrix cores: `workgroups` workgroups of four waves (one per
 * SIMD), every wave loads one A and one B fragment (8 bf16 per lane each: lane l reads 16 bytes at a + 16 l and
 * b + 16 l of its wave's 1024-byte slice; wave w of workgroup g uses slice (4 g + w) mod slices) and issues
 * iters x 16 MFMAs on four independent accumulators, nothing else in the loop.
 *   flops = workgroups * 4 * iters * 16 * 32768.
 * a, b      device, in   slices * 1024 bytes each
 * out       device, out  workgroups * 4 * 2 fp32: per wave, the sum of its accumulators (keeps the MFMAs alive)
 *           and the shader-clock cycles its loop took (as a float)
 */
int slim_probe_mfma_bf16(const void* a, const void* b, int slices, float* out, int workgroups, int iters, void* stream);

/*
 * The loads of the grouped-query decode kernel (slim_attn_decode_int8 with 2 to 32 query heads per KV head)
 * without its arithmetic: the same workgroups, waves, token runs and 128-bit non-temporal loads of K codes, V codes
 * and scales, issued at the same points of the same loop, a tile's registers only XORed together before they are
 * refilled.  Arguments as for slim_attn_decode_int8 (no output: what lands in the workspace is meaningless);
 * workspace_bytes as slim_attn_decode_int8_workspace_bytes() gives for the shape.
 */
int slim_probe_gqa_decode_traffic(const void* q_bf16, const int8_t* k_codes, const float* k_scale, const int8_t* v_codes,
                                  const float* v_scale, void* workspace, size_t workspace_bytes, int batch, int q_heads,
                                  int kv_heads, int kv_len, int head_dim, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SLIMPROBE_H */

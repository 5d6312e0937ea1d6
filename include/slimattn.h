/*
 * slimattn.h — C ABI of the SlimAttention library for AMD MI355X (gfx950).
 *
 * Three operations, as the paper states the problem (batch, query heads, KV heads,
 * sequence length, head dim, causal flag, softmax scale):
 *
 *   kv_quant_int8          builds the reduced-precision KV cache of section 2.2
 *   slim_attn_prefill      first-token attention of section 2.1 (score rows over all
 *                          keys, softmax over the row, row times V), bf16 or INT8 K/V
 *   slim_attn_decode_int8  next-token attention over the INT8 cache (section 2.2)
 *
 * and, around them, what a serving loop needs: kv_quant_int8_pair (K and V in one launch),
 * kv_quant_int8_append (one new token per sequence into the cache), slim_attn_prefill_emit_int8 (prefill that also writes the
 * cache), slim_attn_decode_int8_varlen (a batch whose caches differ in length), plus
 * slim_attn_prefill_two_sweep and slim_attn_prefill_strip, two comparison variants of the prefill that keep the
 * paper's own order of operations (the whole score row before the softmax).
 *
 * Common rules
 *   - Every pointer marked "device" is GPU memory owned by the caller, 16-byte
 *     aligned, densely packed in the stated layout (last index fastest).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued on it; no call synchronises, allocates or frees, and the library keeps no
 *     state between calls (slim_attn_decode_int8_static alone owns a static device array).
 *   - Every call returns a SLIM_* status.  On any status other than SLIM_OK and
 *     SLIM_ERR_LAUNCH nothing was enqueued.  Nothing throws across this boundary.
 *   - bf16 = upper 16 bits of IEEE fp32.  Inputs are not scanned for NaN or infinity.  In the
 *     quantiser a non-finite value makes the codes and the scale of its own row undefined.  In the
 *     attention calls a non-finite value anywhere in a (batch, KV head)'s K, V or scales may make
 *     every output row of the query heads that read that KV head undefined, rows that the causal
 *     mask hides it from included: a masked key takes part in the matrix products with
 *     probability zero, and zero times infinity is not zero.
 *   - SLIM_ERR_LAUNCH reports a launch of the call that returns it: an error that an earlier HIP
 *     call of the thread left behind is dropped before the first launch.
 *   - Query head h reads KV head h / (q_heads / kv_heads): consecutive query heads
 *     share a KV head.
 */
#ifndef SLIMATTN_H
#define SLIMATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SLIM_OK = 0,
    SLIM_ERR_NULL = 1,        /* a required pointer is NULL, or a scale pointer is inconsistent with kv_dtype */
    SLIM_ERR_SHAPE = 2,       /* a size is <= 0, too large to index, q_heads % kv_heads != 0, bad scale/flag */
    SLIM_ERR_UNSUPPORTED = 3, /* head_dim not in {64, 128}, or an unknown dtype code */
    SLIM_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned */
    SLIM_ERR_WORKSPACE = 5,   /* workspace smaller than the entry point's *_workspace_bytes() */
    SLIM_ERR_LAUNCH = 6       /* the HIP runtime refused a kernel launch */
};

enum { SLIM_BF16 = 0, SLIM_F32 = 1, SLIM_I8 = 2 };

/*
 * INT8 KV-cache quantiser (section 2.2: INT8 K/V with one scale per token per head).
 * Symmetric, per row of head_dim values:
 *     amax = max_d |x_d| ; scale = fl32(amax / 127) ; code_d = clamp(rne(fl32(x_d / scale)), -127, 127)
 *     amax == 0  ->  scale = 0, codes = 0.      (IEEE fp32 division, ties to even)
 * x_bf16  device, in   [batch, kv_heads, seq_len, head_dim] bf16
 * codes   device, out  [batch, kv_heads, seq_len, head_dim] int8
 * scales  device, out  [batch, kv_heads, seq_len] fp32
 * q_heads, causal and softmax_scale belong to the common argument tail: the result does not depend
 * on them, but they are checked for range like everywhere else (q_heads a positive multiple of
 * kv_heads, causal 0 or 1, softmax_scale finite and > 0; SLIM_ERR_SHAPE otherwise).
 */
int kv_quant_int8(const void* x_bf16, int8_t* codes, float* scales,
                  int batch, int q_heads, int kv_heads, int seq_len, int head_dim,
                  int causal, float softmax_scale, void* stream);

/*
 * kv_quant_int8 on the K and the V of a cache in one launch (section 2.2 quantises both the same
 * way): k_codes/k_scale are what kv_quant_int8 gives on k_bf16, v_codes/v_scale what it gives on
 * v_bf16, bit for bit.  For the tensors of a single prefill a call is bound by the launch, and the
 * pair takes little more than one of the two single calls.
 * k_bf16, v_bf16     device, in   [batch, kv_heads, seq_len, head_dim] bf16 each
 * k_codes, v_codes   device, out  [batch, kv_heads, seq_len, head_dim] int8 each
 * k_scale, v_scale   device, out  [batch, kv_heads, seq_len] fp32 each
 * The six buffers must not overlap.  Argument tail and errors as in kv_quant_int8.
 */
int kv_quant_int8_pair(const void* k_bf16, const void* v_bf16, int8_t* k_codes, float* k_scale,
                       int8_t* v_codes, float* v_scale,
                       int batch, int q_heads, int kv_heads, int seq_len, int head_dim,
                       int causal, float softmax_scale, void* stream);

/*
 * Appends one token per sequence to an INT8 cache: the step before a decode over it
 * (section 2.2 keeps the cache in INT8, so every new token's K and V are quantised on
 * their way in).  Row (b, g) of x_new is quantised exactly as in kv_quant_int8 and
 * written at token index positions[b] of that (batch, KV head)'s cache.
 * x_new_bf16  device, in      [batch, kv_heads, 1, head_dim] bf16
 * codes       device, in/out  [batch, kv_heads, kv_len, head_dim] int8 (kv_len = allocated length)
 * scales      device, in/out  [batch, kv_heads, kv_len] fp32
 * positions   device, in      [batch] int32, 4-byte aligned; a sequence whose position lies
 *             outside [0, kv_len) is skipped (the positions live on the device, so the
 *             library cannot reject them without waiting for the stream).
 * q_heads, causal and softmax_scale: unused but checked for range, as in kv_quant_int8.
 */
int kv_quant_int8_append(const void* x_new_bf16, int8_t* codes, float* scales, const int32_t* positions,
                         int batch, int q_heads, int kv_heads, int kv_len, int head_dim,
                         int causal, float softmax_scale, void* stream);

/*
 * Prefill attention (section 2.1).  For every batch b, query head h and query row i:
 *     s_j = softmax_scale * <q[b,h,i,:], k^[b,g,j,:]>   over the visible keys j
 *     o[b,h,i,:] = sum_j softmax_j(s) * v^[b,g,j,:]
 * causal != 0: key j is visible iff j <= i; causal == 0: every key.  Each work item
 * owns a block of query rows and the whole softmax direction (the one-dimensional
 * decomposition); K/V are streamed through it in tiles with an fp32 running max/sum.
 * kv_dtype == SLIM_BF16: k, v are bf16 and k_scale, v_scale must be NULL.
 * kv_dtype == SLIM_I8  : k, v are INT8 codes, k^ = code * k_scale[b,g,j] (likewise v);
 *                        the codes are widened exactly in registers (section 2.2).
 * q        device, in   [batch, q_heads, seq_len, head_dim] bf16
 * k, v     device, in   [batch, kv_heads, seq_len, head_dim] bf16 or int8
 * k_scale, v_scale  device, in  [batch, kv_heads, seq_len] fp32, or NULL
 * out      device, out  [batch, q_heads, seq_len, head_dim], bf16 (SLIM_BF16) or fp32 (SLIM_F32)
 * softmax_scale must be finite and > 0.
 */
int slim_attn_prefill(const void* q_bf16, const void* k, const void* v,
                      const float* k_scale, const float* v_scale, void* out,
                      int batch, int q_heads, int kv_heads, int seq_len, int head_dim,
                      int causal, float softmax_scale, int kv_dtype, int out_dtype, void* stream);

/*
 * Prefill attention on bf16 K/V that also writes their INT8 cache in the same launch (the
 * serving loop of section 2.2 keeps K/V in INT8 from the first token on): the attention
 * result is that of slim_attn_prefill with kv_dtype == SLIM_BF16, bit for bit, and
 * codes/scales are those of kv_quant_int8 on k_bf16 and v_bf16, bit for bit.  Each row
 * block's own K and V rows are quantised by the workgroup that just attended over them.
 * k_codes, v_codes  device, out  [batch, kv_heads, seq_len, head_dim] int8
 * k_scale, v_scale  device, out  [batch, kv_heads, seq_len] fp32
 * Everything else as in slim_attn_prefill.
 */
int slim_attn_prefill_emit_int8(const void* q_bf16, const void* k_bf16, const void* v_bf16, void* out,
                                int8_t* k_codes, float* k_scale, int8_t* v_codes, float* v_scale,
                                int batch, int q_heads, int kv_heads, int seq_len, int head_dim,
                                int causal, float softmax_scale, int out_dtype, void* stream);

/*
 * Comparison variant of the bf16 prefill that follows the order of operations of section 2.1
 * literally: a row block's whole score row exists before its softmax is applied.  The scores
 * of a row block do not fit on chip, so K is swept twice, in two kernel launches: the first
 * computes the scores and keeps the row maxima (in the workspace), the second computes them
 * again, exponentiates against those final maxima and multiplies by V.  Same result as
 * slim_attn_prefill up to rounding order; 1.5 times its matrix work.  It is there to be
 * measured against the one-sweep kernel, not to be served from.
 * workspace  device, scratch, at least slim_attn_prefill_two_sweep_workspace_bytes(...) bytes
 *            (two fp32 per query row); contents before and after the call are meaningless.
 * K/V are bf16; everything else as in slim_attn_prefill.
 */
size_t slim_attn_prefill_two_sweep_workspace_bytes(int batch, int q_heads, int kv_heads, int seq_len, int head_dim);
int slim_attn_prefill_two_sweep(const void* q_bf16, const void* k_bf16, const void* v_bf16, void* out,
                                void* workspace, size_t workspace_bytes,
                                int batch, int q_heads, int kv_heads, int seq_len, int head_dim,
                                int causal, float softmax_scale, int out_dtype, void* stream);

/*
 * Second comparison variant of the bf16 prefill, the order of operations of section 2.1 with nothing computed
 * twice: the whole score strip of a row block (its query rows times ALL their keys) is kept on chip, the softmax
 * is applied to it once (one maximum, one pass of exponentials, one sum; no running maximum, no rescaling), and
 * the strip times V is the row block's slice of the output; the next row block reuses the buffer.  The buffer is
 * the compute unit's local memory (160 KB), which holds 32 query rows x slim_attn_prefill_strip_max_seq_len()
 * (2048) keys of fp16 scores: that fixes the row block at 32 rows, so K and V are read four times as often as by
 * the 128-row blocks of slim_attn_prefill.  A score waits in the strip as fp16 relative to the row maximum found
 * so far (exact enough wherever the probability is not negligible, whatever the scores' magnitude).  A longer
 * sequence takes the streamed kernel of slim_attn_prefill instead (same result).
 * Same result as slim_attn_prefill up to rounding order.  K/V are bf16; everything else as in slim_attn_prefill.
 * It is there to be measured against the streamed kernel (the question behind the paper's Table 3: one- against
 * two-dimensional decomposition), not to be served from.
 */
int slim_attn_prefill_strip_max_seq_len(void);
int slim_attn_prefill_strip(const void* q_bf16, const void* k_bf16, const void* v_bf16, void* out,
                            int batch, int q_heads, int kv_heads, int seq_len, int head_dim,
                            int causal, float softmax_scale, int out_dtype, void* stream);

/*
 * Bytes of device workspace slim_attn_decode_int8 needs for this shape (partial
 * max / sum / accumulator of each split of the key axis).  0 if the shape is invalid.
 */
size_t slim_attn_decode_int8_workspace_bytes(int batch, int q_heads, int kv_heads, int kv_len, int head_dim);

/*
 * Decode attention over the INT8 KV cache (section 2.2: a bandwidth-bound matrix-vector
 * product; INT8 is widened to FP32 in registers and fed to FMAs).  One query token per
 * (batch, query head) attends to all kv_len cached tokens:
 *     s_t = softmax_scale * k_scale[b,g,t] * <q[b,h,:], k_codes[b,g,t,:]>
 *     o[b,h,:] = sum_t softmax_t(s) * v_scale[b,g,t] * v_codes[b,g,t,:]
 * The query is the newest position, so `causal` 0 and 1 give the same result.
 * With 2 to 32 query heads per KV head (GQA, named beside MHA in section 2.1) the query
 * heads of a KV head share one pass over its cache: the cache is read once per KV head,
 * the two products run on the matrix cores, and the probabilities (times v_scale) are
 * rounded to bf16 before the second product, as in slim_attn_prefill.
 * q_bf16    device, in   [batch, q_heads, 1, head_dim] bf16
 * k_codes, v_codes  device, in  [batch, kv_heads, kv_len, head_dim] int8
 * k_scale, v_scale  device, in  [batch, kv_heads, kv_len] fp32
 * out_bf16  device, out  [batch, q_heads, 1, head_dim] bf16
 * workspace device, scratch, at least slim_attn_decode_int8_workspace_bytes(...) bytes;
 *           contents before and after the call are meaningless.
 * The result does not depend on the order in which workgroups finish.
 */
int slim_attn_decode_int8(const void* q_bf16, const int8_t* k_codes, const float* k_scale,
                          const int8_t* v_codes, const float* v_scale, void* out_bf16,
                          void* workspace, size_t workspace_bytes,
                          int batch, int q_heads, int kv_heads, int kv_len, int head_dim,
                          int causal, float softmax_scale, void* stream);

/*
 * slim_attn_decode_int8 for callers that cannot provide or allocate a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace,
 * same kernels, same result bit for bit; the partial results of the key-axis splits go to a static device
 * array of slim_attn_decode_int8_static_max_bytes() bytes (16 MiB) that is part of the library's code object:
 * every GPU the library runs on holds its own copy until the process ends.  The call allocates and frees
 * nothing; its first call on a device looks up that device's address of the array (make that call outside a
 * graph capture).  A shape whose slim_attn_decode_int8_workspace_bytes() exceeds the array returns
 * SLIM_ERR_WORKSPACE and enqueues nothing.  All calls on one GPU share the array: two such calls that may run
 * at the same time there (different streams, different threads) race on it; calls on one stream are safe,
 * and nothing in the array has to be cleared between calls (every record that is read is written first).
 */
size_t slim_attn_decode_int8_static_max_bytes(void);
int slim_attn_decode_int8_static(const void* q_bf16, const int8_t* k_codes, const float* k_scale,
                                 const int8_t* v_codes, const float* v_scale, void* out_bf16,
                                 int batch, int q_heads, int kv_heads, int kv_len, int head_dim,
                                 int causal, float softmax_scale, void* stream);

/*
 * The same decode step for a batch whose sequences have caches of different lengths
 * (the paper's throughput runs, section 3.2, batch many sequences per step): sequence b
 * attends to its first kv_lens[b] cached tokens.  The cache tensors keep the layout
 * [batch, kv_heads, kv_len, head_dim] / [batch, kv_heads, kv_len], kv_len being the
 * allocated length; what lies past a sequence's own length is never read into the result.
 * kv_lens   device, in   [batch] int32, 4-byte aligned; a value outside [1, kv_len] is
 *           taken as the nearest bound (the lengths live on the device, so the library
 *           cannot reject them without waiting for the stream).
 * Everything else, including the workspace size (computed from kv_len), as in
 * slim_attn_decode_int8.
 */
int slim_attn_decode_int8_varlen(const void* q_bf16, const int8_t* k_codes, const float* k_scale,
                                 const int8_t* v_codes, const float* v_scale, const int32_t* kv_lens,
                                 void* out_bf16, void* workspace, size_t workspace_bytes,
                                 int batch, int q_heads, int kv_heads, int kv_len, int head_dim,
                                 int causal, float softmax_scale, void* stream);

/* Name of a status code; pointer to static storage, never NULL. */
const char* slim_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SLIMATTN_H */

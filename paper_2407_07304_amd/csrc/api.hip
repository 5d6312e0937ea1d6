// C ABI of the library (declared in include/slimattn.h): argument validation and
// dispatch only.  Nothing here allocates, synchronises or keeps state.
#include "../../include/slimattn.h"

#include <math.h>

#include "slim_kernels.h"

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// hipGetLastError() returns (and clears) whatever error an earlier HIP call of this thread left behind, the
// caller's own included.  Every entry point drops that before its first launch, so that SLIM_ERR_LAUNCH only
// ever reports a launch of the call that returns it.
inline void drop_stale_hip_error() { (void)hipGetLastError(); }

// The scalars of the common argument tail that an operation does not use are still checked for range.
inline int check_unused_tail(int q_heads, int kv_heads, int causal, float softmax_scale) {
    if (q_heads <= 0 || kv_heads <= 0 || q_heads % kv_heads != 0) return SLIM_ERR_SHAPE;
    if (causal != 0 && causal != 1) return SLIM_ERR_SHAPE;
    if (!(softmax_scale > 0.0f) || !isfinite(softmax_scale)) return SLIM_ERR_SHAPE;
    return SLIM_OK;
}

// Total element counts must stay indexable with the 32-bit row counters the kernels use.
inline bool too_large(long a, long b, long c) {
    const long lim = 2147483647L;
    if (a > lim || b > lim || c > lim) return true;
    if (a * b > lim) return true;
    return a * b * c > lim;
}

int check_shape(int batch, int q_heads, int kv_heads, int len, int head_dim) {
    if (batch <= 0 || q_heads <= 0 || kv_heads <= 0 || len <= 0 || head_dim <= 0) return SLIM_ERR_SHAPE;
    if (q_heads % kv_heads != 0) return SLIM_ERR_SHAPE;
    if (head_dim != 64 && head_dim != 128) return SLIM_ERR_UNSUPPORTED;
    if (too_large(batch, q_heads, len)) return SLIM_ERR_SHAPE;   // rows of Q/O (and of K/V, kv_heads <= q_heads)
    if (q_heads > 65535 || batch > 65535) return SLIM_ERR_SHAPE;
    // one head's K (or V) slab, plus the tiles the prefill kernel prefetches past it, is addressed with 32 bits
    if (((long)len + 256) * head_dim * 2 > 0xffffffffL) return SLIM_ERR_SHAPE;
    return SLIM_OK;
}

}  // namespace

extern "C" {

const char* slim_status_string(int status) {
    switch (status) {
        case SLIM_OK: return "SLIM_OK";
        case SLIM_ERR_NULL: return "SLIM_ERR_NULL: required pointer is null or scale pointers do not match kv_dtype";
        case SLIM_ERR_SHAPE: return "SLIM_ERR_SHAPE: invalid size, head ratio, flag or softmax scale";
        case SLIM_ERR_UNSUPPORTED: return "SLIM_ERR_UNSUPPORTED: head_dim must be 64 or 128 and dtype codes must be known";
        case SLIM_ERR_ALIGN: return "SLIM_ERR_ALIGN: pointers must be 16-byte aligned";
        case SLIM_ERR_WORKSPACE: return "SLIM_ERR_WORKSPACE: workspace too small";
        case SLIM_ERR_LAUNCH: return "SLIM_ERR_LAUNCH: kernel launch failed";
        default: return "unknown status";
    }
}

int kv_quant_int8(const void* x_bf16, int8_t* codes, float* scales, int batch, int q_heads, int kv_heads, int seq_len,
                  int head_dim, int causal, float softmax_scale, void* stream) {
    if (!x_bf16 || !codes || !scales) return SLIM_ERR_NULL;
    const int st = check_shape(batch, kv_heads, kv_heads, seq_len, head_dim);
    if (st != SLIM_OK) return st;
    const int st_tail = check_unused_tail(q_heads, kv_heads, causal, softmax_scale);
    if (st_tail != SLIM_OK) return st_tail;
    if (misaligned(x_bf16) || misaligned(codes) || misaligned(scales)) return SLIM_ERR_ALIGN;
    const long n_rows = (long)batch * kv_heads * seq_len;
    drop_stale_hip_error();
    const hipError_t e = slim::launch_kv_quant_int8(x_bf16, codes, scales, n_rows, head_dim, (hipStream_t)stream);
    return e == hipSuccess ? SLIM_OK : SLIM_ERR_LAUNCH;
}

int kv_quant_int8_pair(const void* k_bf16, const void* v_bf16, int8_t* k_codes, float* k_scale, int8_t* v_codes,
                       float* v_scale, int batch, int q_heads, int kv_heads, int seq_len, int head_dim, int causal,
                       float softmax_scale, void* stream) {
    if (!k_bf16 || !v_bf16 || !k_codes || !k_scale || !v_codes || !v_scale) return SLIM_ERR_NULL;
    const int st = check_shape(batch, kv_heads, kv_heads, seq_len, head_dim);
    if (st != SLIM_OK) return st;
    const int st_tail = check_unused_tail(q_heads, kv_heads, causal, softmax_scale);
    if (st_tail != SLIM_OK) return st_tail;
    if (misaligned(k_bf16) || misaligned(v_bf16) || misaligned(k_codes) || misaligned(k_scale) || misaligned(v_codes) ||
        misaligned(v_scale))
        return SLIM_ERR_ALIGN;
    const long n_rows = (long)batch * kv_heads * seq_len;
    drop_stale_hip_error();
    const hipError_t e = slim::launch_kv_quant_int8_pair(k_bf16, v_bf16, k_codes, k_scale, v_codes, v_scale, n_rows, head_dim,
                                                         (hipStream_t)stream);
    return e == hipSuccess ? SLIM_OK : SLIM_ERR_LAUNCH;
}

int kv_quant_int8_append(const void* x_new_bf16, int8_t* codes, float* scales, const int32_t* positions, int batch,
                         int q_heads, int kv_heads, int kv_len, int head_dim, int causal, float softmax_scale,
                         void* stream) {
    if (!x_new_bf16 || !codes || !scales || !positions) return SLIM_ERR_NULL;
    const int st = check_shape(batch, kv_heads, kv_heads, kv_len, head_dim);
    if (st != SLIM_OK) return st;
    const int st_tail = check_unused_tail(q_heads, kv_heads, causal, softmax_scale);
    if (st_tail != SLIM_OK) return st_tail;
    if (misaligned(x_new_bf16) || misaligned(codes) || misaligned(scales)) return SLIM_ERR_ALIGN;
    if ((uintptr_t)positions & 3u) return SLIM_ERR_ALIGN;
    drop_stale_hip_error();
    const hipError_t e = slim::launch_kv_quant_int8_append(x_new_bf16, codes, scales, positions, batch, kv_heads, kv_len,
                                                           head_dim, (hipStream_t)stream);
    return e == hipSuccess ? SLIM_OK : SLIM_ERR_LAUNCH;
}

static int prefill_common(const void* q_bf16, const void* k, const void* v, const float* k_scale, const float* v_scale,
                          void* out, int8_t* k_codes_out, float* k_scale_out, int8_t* v_codes_out, float* v_scale_out,
                          int batch, int q_heads, int kv_heads, int seq_len, int head_dim, int causal,
                          float softmax_scale, int kv_dtype, int out_dtype, float* row_max, void* stream,
                          bool use_strip = false) {
    if (!q_bf16 || !k || !v || !out) return SLIM_ERR_NULL;
    if (kv_dtype != SLIM_BF16 && kv_dtype != SLIM_I8) return SLIM_ERR_UNSUPPORTED;
    if (out_dtype != SLIM_BF16 && out_dtype != SLIM_F32) return SLIM_ERR_UNSUPPORTED;
    if (kv_dtype == SLIM_I8 && (!k_scale || !v_scale)) return SLIM_ERR_NULL;
    if (kv_dtype == SLIM_BF16 && (k_scale || v_scale)) return SLIM_ERR_NULL;
    const int st = check_shape(batch, q_heads, kv_heads, seq_len, head_dim);
    if (st != SLIM_OK) return st;
    if (causal != 0 && causal != 1) return SLIM_ERR_SHAPE;
    if (!(softmax_scale > 0.0f) || !isfinite(softmax_scale)) return SLIM_ERR_SHAPE;
    if (misaligned(q_bf16) || misaligned(k) || misaligned(v) || misaligned(out)) return SLIM_ERR_ALIGN;
    if (kv_dtype == SLIM_I8 && (misaligned(k_scale) || misaligned(v_scale))) return SLIM_ERR_ALIGN;
    if (k_codes_out && (misaligned(k_codes_out) || misaligned(k_scale_out) || misaligned(v_codes_out) || misaligned(v_scale_out)))
        return SLIM_ERR_ALIGN;
    slim::PrefillArgs a;
    a.q = q_bf16;
    a.k = k;
    a.v = v;
    a.k_scale = k_scale;
    a.v_scale = v_scale;
    a.out = out;
    a.k_codes_out = k_codes_out;
    a.k_scale_out = k_scale_out;
    a.v_codes_out = v_codes_out;
    a.v_scale_out = v_scale_out;
    a.batch = batch;
    a.q_heads = q_heads;
    a.kv_heads = kv_heads;
    a.seq_len = seq_len;
    a.head_dim = head_dim;
    a.causal = causal;
    a.softmax_scale = softmax_scale;
    a.kv_int8 = kv_dtype == SLIM_I8;
    a.out_f32 = out_dtype == SLIM_F32;
    a.row_max = row_max;
    drop_stale_hip_error();
    const hipError_t e = use_strip ? slim::launch_prefill_strip(a, (hipStream_t)stream) : slim::launch_prefill(a, (hipStream_t)stream);
    return e == hipSuccess ? SLIM_OK : SLIM_ERR_LAUNCH;
}

int slim_attn_prefill(const void* q_bf16, const void* k, const void* v, const float* k_scale, const float* v_scale,
                      void* out, int batch, int q_heads, int kv_heads, int seq_len, int head_dim, int causal,
                      float softmax_scale, int kv_dtype, int out_dtype, void* stream) {
    return prefill_common(q_bf16, k, v, k_scale, v_scale, out, nullptr, nullptr, nullptr, nullptr, batch, q_heads, kv_heads,
                          seq_len, head_dim, causal, softmax_scale, kv_dtype, out_dtype, nullptr, stream);
}

size_t slim_attn_prefill_two_sweep_workspace_bytes(int batch, int q_heads, int kv_heads, int seq_len, int head_dim) {
    if (check_shape(batch, q_heads, kv_heads, seq_len, head_dim) != SLIM_OK) return 0;
    return (size_t)batch * q_heads * seq_len * 2 * sizeof(float);
}

int slim_attn_prefill_two_sweep(const void* q_bf16, const void* k_bf16, const void* v_bf16, void* out, void* workspace,
                                size_t workspace_bytes, int batch, int q_heads, int kv_heads, int seq_len, int head_dim,
                                int causal, float softmax_scale, int out_dtype, void* stream) {
    if (!workspace) return SLIM_ERR_NULL;
    if (misaligned(workspace)) return SLIM_ERR_ALIGN;
    const size_t need = slim_attn_prefill_two_sweep_workspace_bytes(batch, q_heads, kv_heads, seq_len, head_dim);
    if (need != 0 && workspace_bytes < need) return SLIM_ERR_WORKSPACE;
    return prefill_common(q_bf16, k_bf16, v_bf16, nullptr, nullptr, out, nullptr, nullptr, nullptr, nullptr, batch, q_heads,
                          kv_heads, seq_len, head_dim, causal, softmax_scale, SLIM_BF16, out_dtype, (float*)workspace, stream);
}

int slim_attn_prefill_strip_max_seq_len(void) { return slim::kPrefillStripMaxSeqLen; }

int slim_attn_prefill_strip(const void* q_bf16, const void* k_bf16, const void* v_bf16, void* out, int batch, int q_heads,
                            int kv_heads, int seq_len, int head_dim, int causal, float softmax_scale, int out_dtype,
                            void* stream) {
    // a longer sequence's strip does not fit on chip: it takes the streamed kernel
    const bool fits = seq_len <= slim::kPrefillStripMaxSeqLen;
    return prefill_common(q_bf16, k_bf16, v_bf16, nullptr, nullptr, out, nullptr, nullptr, nullptr, nullptr, batch, q_heads,
                          kv_heads, seq_len, head_dim, causal, softmax_scale, SLIM_BF16, out_dtype, nullptr, stream, fits);
}

int slim_attn_prefill_emit_int8(const void* q_bf16, const void* k_bf16, const void* v_bf16, void* out, int8_t* k_codes,
                                float* k_scale, int8_t* v_codes, float* v_scale, int batch, int q_heads, int kv_heads,
                                int seq_len, int head_dim, int causal, float softmax_scale, int out_dtype, void* stream) {
    if (!k_codes || !k_scale || !v_codes || !v_scale) return SLIM_ERR_NULL;
    return prefill_common(q_bf16, k_bf16, v_bf16, nullptr, nullptr, out, k_codes, k_scale, v_codes, v_scale, batch, q_heads,
                          kv_heads, seq_len, head_dim, causal, softmax_scale, SLIM_BF16, out_dtype, nullptr, stream);
}

size_t slim_attn_decode_int8_workspace_bytes(int batch, int q_heads, int kv_heads, int kv_len, int head_dim) {
    if (check_shape(batch, q_heads, kv_heads, kv_len, head_dim) != SLIM_OK) return 0;
    return slim::decode_workspace_bytes(batch, q_heads, kv_heads, kv_len, head_dim);
}

constexpr size_t kUseStaticScratch = ~(size_t)0;   // decode_common: workspace == NULL with this size selects the static array

static int decode_common(const void* q_bf16, const int8_t* k_codes, const float* k_scale, const int8_t* v_codes,
                         const float* v_scale, const int32_t* kv_lens, void* out_bf16, void* workspace,
                         size_t workspace_bytes, int batch, int q_heads, int kv_heads, int kv_len, int head_dim, int causal,
                         float softmax_scale, void* stream) {
    // use_static: the partial results go to the library's own static device array instead of a caller's workspace
    const bool use_static = workspace == nullptr && workspace_bytes == kUseStaticScratch;
    if (!q_bf16 || !k_codes || !k_scale || !v_codes || !v_scale || !out_bf16 || (!workspace && !use_static)) return SLIM_ERR_NULL;
    const int st = check_shape(batch, q_heads, kv_heads, kv_len, head_dim);
    if (st != SLIM_OK) return st;
    if (causal != 0 && causal != 1) return SLIM_ERR_SHAPE;
    if (!(softmax_scale > 0.0f) || !isfinite(softmax_scale)) return SLIM_ERR_SHAPE;
    if (misaligned(q_bf16) || misaligned(k_codes) || misaligned(k_scale) || misaligned(v_codes) ||
        misaligned(v_scale) || misaligned(out_bf16) || misaligned(workspace))
        return SLIM_ERR_ALIGN;
    if (kv_lens && ((uintptr_t)kv_lens & 3u)) return SLIM_ERR_ALIGN;
    const size_t need = slim::decode_workspace_bytes(batch, q_heads, kv_heads, kv_len, head_dim);
    if (use_static) {
        if (need > slim::kDecodeStaticScratchBytes) return SLIM_ERR_WORKSPACE;
        float* own = nullptr;
        if (slim::decode_static_scratch(&own) != hipSuccess) return SLIM_ERR_LAUNCH;
        workspace = own;
    } else if (workspace_bytes < need) {
        return SLIM_ERR_WORKSPACE;
    }
    slim::DecodeArgs a;
    a.q = q_bf16;
    a.k_codes = k_codes;
    a.k_scale = k_scale;
    a.v_codes = v_codes;
    a.v_scale = v_scale;
    a.out = out_bf16;
    a.workspace = (float*)workspace;
    a.kv_lens = kv_lens;
    a.batch = batch;
    a.q_heads = q_heads;
    a.kv_heads = kv_heads;
    a.kv_len = kv_len;
    a.head_dim = head_dim;
    a.softmax_scale = softmax_scale;
    drop_stale_hip_error();
    const hipError_t e = slim::launch_decode(a, (hipStream_t)stream);
    return e == hipSuccess ? SLIM_OK : SLIM_ERR_LAUNCH;
}

int slim_attn_decode_int8(const void* q_bf16, const int8_t* k_codes, const float* k_scale, const int8_t* v_codes,
                          const float* v_scale, void* out_bf16, void* workspace, size_t workspace_bytes, int batch,
                          int q_heads, int kv_heads, int kv_len, int head_dim, int causal, float softmax_scale,
                          void* stream) {
    return decode_common(q_bf16, k_codes, k_scale, v_codes, v_scale, nullptr, out_bf16, workspace, workspace_bytes, batch,
                         q_heads, kv_heads, kv_len, head_dim, causal, softmax_scale, stream);
}

size_t slim_attn_decode_int8_static_max_bytes(void) { return slim::kDecodeStaticScratchBytes; }

int slim_attn_decode_int8_static(const void* q_bf16, const int8_t* k_codes, const float* k_scale, const int8_t* v_codes,
                                 const float* v_scale, void* out_bf16, int batch, int q_heads, int kv_heads, int kv_len,
                                 int head_dim, int causal, float softmax_scale, void* stream) {
    return decode_common(q_bf16, k_codes, k_scale, v_codes, v_scale, nullptr, out_bf16, nullptr, kUseStaticScratch, batch,
                         q_heads, kv_heads, kv_len, head_dim, causal, softmax_scale, stream);
}

int slim_attn_decode_int8_varlen(const void* q_bf16, const int8_t* k_codes, const float* k_scale, const int8_t* v_codes,
                                 const float* v_scale, const int32_t* kv_lens, void* out_bf16, void* workspace,
                                 size_t workspace_bytes, int batch, int q_heads, int kv_heads, int kv_len, int head_dim,
                                 int causal, float softmax_scale, void* stream) {
    if (!kv_lens) return SLIM_ERR_NULL;
    return decode_common(q_bf16, k_codes, k_scale, v_codes, v_scale, kv_lens, out_bf16, workspace, workspace_bytes, batch,
                         q_heads, kv_heads, kv_len, head_dim, causal, softmax_scale, stream);
}

}  // extern "C"

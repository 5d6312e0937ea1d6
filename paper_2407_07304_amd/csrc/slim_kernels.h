// Host-side launchers of the gfx950 kernels; arguments are validated by the C ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace slim {

hipError_t launch_kv_quant_int8(const void* x, int8_t* codes, float* scales, long n_rows, int head_dim,
                                hipStream_t stream);

hipError_t launch_kv_quant_int8_pair(const void* k, const void* v, int8_t* k_codes, float* k_scale, int8_t* v_codes,
                                     float* v_scale, long n_rows, int head_dim, hipStream_t stream);
hipError_t launch_kv_quant_int8_append(const void* x, int8_t* codes, float* scales, const int* positions, int batch,
                                       int kv_heads, int kv_len, int head_dim, hipStream_t stream);

struct PrefillArgs {
    const void* q;
    const void* k;
    const void* v;
    const float* k_scale;
    const float* v_scale;
    void* out;
    int8_t* k_codes_out;   // with bf16 K/V: also write their INT8 cache (all four set), or all null
    float* k_scale_out;
    int8_t* v_codes_out;
    float* v_scale_out;
    int batch, q_heads, kv_heads, seq_len, head_dim, causal;
    float softmax_scale;
    bool kv_int8, out_f32;
    float* row_max;   // null, or (bf16 K/V only) the two-sweep variant's workspace [batch, q_heads, seq_len, 2]
};
hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream);
// The comparison variant that keeps a row block's whole score strip in LDS (bf16 K/V, sequences up to
// kPrefillStripMaxSeqLen keys: 32 rows x that many fp16 scores is what fits beside the V staging buffer).
constexpr int kPrefillStripMaxSeqLen = 2048;
hipError_t launch_prefill_strip(const PrefillArgs& a, hipStream_t stream);

struct DecodeArgs {
    const void* q;
    const int8_t* k_codes;
    const float* k_scale;
    const int8_t* v_codes;
    const float* v_scale;
    void* out;
    float* workspace;
    const int* kv_lens;   // device, [batch]: tokens of each sequence's cache that count (clamped to 1..kv_len), or null: all
    int batch, q_heads, kv_heads, kv_len, head_dim;
    float softmax_scale;
};
// Tokens of the key axis one wave of the split kernel streams, and the split count, for a
// cache of kv_len tokens and n_bh = batch * q_heads independent rows.
int decode_tokens_per_wave(int kv_len, long n_bh);
int decode_num_splits(int kv_len, long n_bh);
// Grouped-query variant (2 to 32 query heads per KV head): one wave streams a token run of one (batch, KV
// head) for all its query heads; every wave is a split.  n_bg = batch * kv_heads.
bool decode_uses_gqa_kernel(int q_heads, int kv_heads);
int decode_gqa_tokens_per_wave(int kv_len, long n_bg);
int decode_gqa_num_splits(int kv_len, long n_bg);
// traffic_only: the measurement form (the kernel's loads without its arithmetic; what it writes is meaningless)
hipError_t launch_decode_gqa_split(const DecodeArgs& a, float* ws_acc, float* ws_ml, int n_split, hipStream_t stream,
                                   bool traffic_only = false);
size_t decode_workspace_bytes(int batch, int q_heads, int kv_heads, int kv_len, int head_dim);
hipError_t launch_decode(const DecodeArgs& a, hipStream_t stream);
// The library's own decode scratch (one static device array per GPU) for the entry point that may not
// allocate: its address on the current device, looked up on the first call there.
constexpr size_t kDecodeStaticScratchBytes = (size_t)16 << 20;
hipError_t decode_static_scratch(float** ptr);

}  // namespace slim

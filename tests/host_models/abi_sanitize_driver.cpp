// Driver for a sanitizer build of the C-ABI layer's host code (csrc/api.hip compiled with
// -fsanitize=address,undefined on the host side only): every entry point is called with arguments that its
// validation must refuse before anything is enqueued, so no GPU is needed.  Exit code 0 = every call returned the
// documented status and the sanitizers saw nothing.
#include <cstdio>
#include <limits>

#include "../../include/slimattn.h"

static int bad = 0;
static void expect(int got, int want, const char* what) {
    if (got != want) {
        std::fprintf(stderr, "abi_sanitize_driver: %s: status %d, expected %d\n", what, got, want);
        ++bad;
    }
}

int main() {
    void* A = reinterpret_cast<void*>(0x1000);   // aligned, never dereferenced: every call fails validation first
    void* M = reinterpret_cast<void*>(0x1004);   // misaligned
    int8_t* A8 = static_cast<int8_t*>(A);
    float* Af = static_cast<float*>(A);
    const float nan = std::numeric_limits<float>::quiet_NaN();
    expect(kv_quant_int8(nullptr, A8, Af, 1, 1, 1, 4, 128, 0, 1.0f, nullptr), SLIM_ERR_NULL, "quant null");
    expect(kv_quant_int8(A, A8, Af, 1, 1, 1, 0, 128, 0, 1.0f, nullptr), SLIM_ERR_SHAPE, "quant empty");
    expect(kv_quant_int8(A, A8, Af, 1, 1, 1, 4, 100, 0, 1.0f, nullptr), SLIM_ERR_UNSUPPORTED, "quant head_dim");
    expect(kv_quant_int8(A, A8, Af, 1, 1, 1, 4, 128, 0, nan, nullptr), SLIM_ERR_SHAPE, "quant scale");
    expect(kv_quant_int8(A, static_cast<int8_t*>(M), Af, 1, 1, 1, 4, 128, 0, 1.0f, nullptr), SLIM_ERR_ALIGN, "quant align");
    expect(kv_quant_int8(A, A8, Af, 65536, 65536, 65536, 2147483647, 128, 0, 1.0f, nullptr), SLIM_ERR_SHAPE, "quant overflowing sizes");
    expect(kv_quant_int8_pair(A, nullptr, A8, Af, A8, Af, 1, 1, 1, 4, 128, 0, 1.0f, nullptr), SLIM_ERR_NULL, "pair null");
    expect(kv_quant_int8_pair(A, A, A8, Af, static_cast<int8_t*>(M), Af, 1, 1, 1, 4, 128, 0, 1.0f, nullptr), SLIM_ERR_ALIGN, "pair align");
    expect(kv_quant_int8_pair(A, A, A8, Af, A8, Af, 1, 3, 2, 4, 128, 0, 1.0f, nullptr), SLIM_ERR_SHAPE, "pair head ratio");
    expect(kv_quant_int8_append(A, A8, Af, nullptr, 1, 1, 1, 4, 128, 0, 1.0f, nullptr), SLIM_ERR_NULL, "append null");
    expect(kv_quant_int8_append(A, A8, Af, static_cast<const int32_t*>(reinterpret_cast<void*>(0x1002)), 1, 1, 1, 4, 128, 0, 1.0f, nullptr), SLIM_ERR_ALIGN, "append align");
    expect(slim_attn_prefill(A, A, A, nullptr, nullptr, nullptr, 1, 2, 2, 16, 128, 1, 0.1f, SLIM_BF16, SLIM_BF16, nullptr), SLIM_ERR_NULL, "prefill null");
    expect(slim_attn_prefill(A, A, A, nullptr, nullptr, A, 1, 2, 2, 16, 128, 1, 0.1f, SLIM_I8, SLIM_BF16, nullptr), SLIM_ERR_NULL, "prefill INT8 without scales");
    expect(slim_attn_prefill(A, A, A, nullptr, nullptr, A, 1, 3, 2, 16, 128, 1, 0.1f, SLIM_BF16, SLIM_BF16, nullptr), SLIM_ERR_SHAPE, "prefill head ratio");
    expect(slim_attn_prefill(A, A, A, nullptr, nullptr, A, 1, 2, 2, 2147483647, 128, 1, 0.1f, SLIM_BF16, SLIM_BF16, nullptr), SLIM_ERR_SHAPE, "prefill huge length");
    expect(slim_attn_prefill(A, A, A, nullptr, nullptr, A, 1, 2, 2, 16, 128, 1, 0.1f, 7, SLIM_BF16, nullptr), SLIM_ERR_UNSUPPORTED, "prefill dtype");
    expect(slim_attn_prefill(A, M, A, nullptr, nullptr, A, 1, 2, 2, 16, 128, 1, 0.1f, SLIM_BF16, SLIM_BF16, nullptr), SLIM_ERR_ALIGN, "prefill align");
    expect(slim_attn_prefill_emit_int8(A, A, A, A, nullptr, Af, A8, Af, 1, 2, 2, 16, 128, 1, 0.1f, SLIM_BF16, nullptr), SLIM_ERR_NULL, "emit null");
    expect(slim_attn_prefill_strip(A, A, A, A, 1, 2, 2, 16, 96, 1, 0.1f, SLIM_BF16, nullptr), SLIM_ERR_UNSUPPORTED, "strip head_dim");
    expect(slim_attn_prefill_two_sweep(A, A, A, A, A, 8, 1, 2, 2, 16, 128, 1, 0.1f, SLIM_BF16, nullptr), SLIM_ERR_WORKSPACE, "two-sweep workspace");
    if (slim_attn_prefill_two_sweep_workspace_bytes(1, 2, 2, 16, 128) != 1u * 2 * 16 * 2 * 4) { std::fprintf(stderr, "two-sweep workspace size\n"); ++bad; }
    if (slim_attn_decode_int8_workspace_bytes(1, 3, 2, 16, 128) != 0) { std::fprintf(stderr, "workspace size of a bad shape\n"); ++bad; }
    const size_t need = slim_attn_decode_int8_workspace_bytes(2, 4, 4, 100000, 64);
    if (need == 0 || need % ((64 + 2) * 4) != 0) { std::fprintf(stderr, "decode workspace size\n"); ++bad; }
    expect(slim_attn_decode_int8(A, A8, Af, A8, Af, A, A, need - 1, 2, 4, 4, 100000, 64, 0, 0.1f, nullptr), SLIM_ERR_WORKSPACE, "decode workspace");
    expect(slim_attn_decode_int8(A, A8, Af, A8, Af, A, nullptr, need, 2, 4, 4, 100000, 64, 0, 0.1f, nullptr), SLIM_ERR_NULL, "decode null workspace");
    expect(slim_attn_decode_int8_varlen(A, A8, Af, A8, Af, nullptr, A, A, need, 2, 4, 4, 100000, 64, 0, 0.1f, nullptr), SLIM_ERR_NULL, "varlen null lengths");
    expect(slim_attn_decode_int8_static(A, A8, Af, A8, Af, A, 256, 64, 8, 8192, 128, 0, 0.1f, nullptr), SLIM_ERR_WORKSPACE, "static scratch too small");
    expect(slim_attn_decode_int8_static(A, A8, Af, A8, Af, M, 1, 2, 2, 16, 128, 0, 0.1f, nullptr), SLIM_ERR_ALIGN, "static align");
    for (int st = -1; st < 9; ++st)
        if (slim_status_string(st) == nullptr) { std::fprintf(stderr, "status string\n"); ++bad; }
    if (bad == 0) std::printf("abi_sanitize_driver: clean\n");
    return bad ? 1 : 0;
}

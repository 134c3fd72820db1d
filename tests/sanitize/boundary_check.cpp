// Host sanitizer run of the boundary: built by tests/test_host_sanitizers_cpu.py with hipcc, the
// library's own sources and -fsanitize=address,undefined on the host side.  Every call below is
// rejected by the argument validation (or is a pure function of the shape), so nothing is launched and
// no GPU is needed; what is exercised is the host code of the C ABI.
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "../../include/wkv6.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::printf("FAIL %s (line %d)\n", #cond, __LINE__);           \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main() {
    void* A = reinterpret_cast<void*>(static_cast<std::uintptr_t>(0x1000));    // aligned, never dereferenced
    void* M = reinterpret_cast<void*>(static_cast<std::uintptr_t>(0x1004));    // misaligned
    float* Af = static_cast<float*>(A);
    for (int code = 0; code <= 8; ++code) CHECK(std::strlen(wkv6_status_string(code)) > 0);
    CHECK(wkv6_version() >= 100);
    CHECK(wkv6_prefill_bf16(1, 8, 2, 32, A, A, A, A, Af, nullptr, A, Af, nullptr) == WKV6_ERR_UNSUPPORTED);
    CHECK(wkv6_prefill_bf16(-1, 8, 2, 64, A, A, A, A, Af, nullptr, A, Af, nullptr) == WKV6_ERR_SHAPE);
    CHECK(wkv6_prefill_bf16(1, 8, 2, 64, nullptr, A, A, A, Af, nullptr, A, Af, nullptr) == WKV6_ERR_NULL);
    CHECK(wkv6_prefill_bf16(1, 8, 2, 64, M, A, A, A, Af, nullptr, A, Af, nullptr) == WKV6_ERR_ALIGN);
    CHECK(wkv6_prefill_bf16(0, 8, 2, 64, nullptr, nullptr, nullptr, nullptr, Af, nullptr, nullptr, nullptr, nullptr) == WKV6_OK);
    CHECK(wkv6_prefill_bf16_f32out(1, 8, 0, 64, A, A, A, A, Af, nullptr, Af, Af, nullptr) == WKV6_ERR_SHAPE);
    CHECK(wkv6_prefill_f32(1, 8, 2, 64, Af, Af, Af, Af, nullptr, nullptr, Af, Af, nullptr) == WKV6_ERR_NULL);
    CHECK(wkv6_prefill_bf16_strided(2, 8, 2, 64, A, A, A, A, Af, nullptr, A, Af, 100, WKV6_DTYPE_BF16, nullptr) == WKV6_ERR_SHAPE);
    CHECK(wkv6_prefill_bf16_strided(2, 8, 2, 64, A, A, A, A, Af, nullptr, A, Af, 1028, WKV6_DTYPE_BF16, nullptr) == WKV6_ERR_ALIGN);
    CHECK(wkv6_prefill_bf16_strided(2, 8, 2, 64, A, A, A, A, Af, nullptr, A, Af, 1024, 7, nullptr) == WKV6_ERR_UNSUPPORTED);
    CHECK(wkv6_finch_c2_prefill_bf16(1, 8, 2, 64, A, A, A, A, nullptr, nullptr, A, Af, nullptr) == WKV6_ERR_NULL);
    CHECK(wkv6_finch_c2_prefill_bf16_moments(1, 8, 2, 64, A, A, A, A, A, nullptr, A, nullptr, Af, nullptr) == WKV6_ERR_NULL);
    CHECK(wkv6_finch_c2_prefill_lora_bf16(1, 8, 2, 64, 32, A, A, A, A, Af, A, A, nullptr, A, nullptr, Af, nullptr) == WKV6_ERR_UNSUPPORTED);
    CHECK(wkv6_prefill_lora_bf16(1, 8, 2, 64, 64, A, A, A, nullptr, Af, A, Af, nullptr, A, Af, nullptr) == WKV6_ERR_NULL);
    CHECK(wkv6_layernorm_finalize(1, 8, 2, 64, Af, -1.f, Af, nullptr) == WKV6_ERR_SHAPE);
    CHECK(wkv6_decode_bf16(4, 2, 64, A, A, A, A, Af, nullptr, A, nullptr) == WKV6_ERR_NULL);
    CHECK(wkv6_append_bf16(1, 3, 2, 64, A, A, A, M, Af, nullptr, A, Af, nullptr) == WKV6_ERR_ALIGN);
    CHECK(wkv6_key_compress_bf16(4, 1000, A, A, A, WKV6_DTYPE_BF16, nullptr) == WKV6_ERR_UNSUPPORTED);
    CHECK(wkv6_key_compress_bf16(-4, 2048, A, A, A, WKV6_DTYPE_BF16, nullptr) == WKV6_ERR_SHAPE);
    CHECK(wkv6_key_compress_bf16(0, 2048, nullptr, nullptr, nullptr, WKV6_DTYPE_F32, nullptr) == WKV6_OK);
    // token split: helpers are pure functions of the shape; the entry points validate before launching
    CHECK(wkv6_split_segments(1, 131072, 32, 64) == 8 && wkv6_split_segments(8, 4096, 32, 64) == 1);
    CHECK(wkv6_split_workspace_bytes(1, 131072, 32, 64, 8) == 8ll * 32 * (4096 + 64) * 4);
    CHECK(wkv6_split_workspace_bytes(1, 100, 2, 32, 8) == -1);
    CHECK(wkv6_prefill_bf16_split(1, 4096, 2, 64, A, A, A, A, Af, nullptr, A, Af, 1, 4, nullptr, 0, nullptr) == WKV6_ERR_NULL);
    CHECK(wkv6_prefill_bf16_split(1, 4096, 2, 64, A, A, A, A, Af, nullptr, A, Af, 1, 4, A, 16, nullptr) == WKV6_ERR_SHAPE);
    CHECK(wkv6_finch_c2_prefill_bf16_split(1, 4096, 2, 64, A, A, A, A, A, nullptr, A, Af, 1, 0, A, 1 << 30, nullptr) == WKV6_ERR_SHAPE);
    CHECK(wkv6_prefill_bf16_split_noalloc(8, 1024, 32, 64, A, A, A, A, Af, nullptr, A, Af, 1, 16, nullptr) == WKV6_ERR_WORKSPACE);
    CHECK(wkv6_prefill_bf16_split_noalloc(1, 1024, 32, 32, A, A, A, A, Af, nullptr, A, Af, 1, 4, nullptr) == WKV6_ERR_UNSUPPORTED);
    std::printf("ok\n");
    return 0;
}

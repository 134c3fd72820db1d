// C ABI of the WKV6 prefill library: argument validation and dispatch only.
// Every step of the computation runs in the kernels this file launches.
#include "../../include/wkv6.h"
#include "wkv6_launch.h"

#include <cstdint>

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<std::uintptr_t>(p) & 15u) != 0; }

enum class Path { kChunked, kRecurrent };

int run(int B, int T, int H, int N, const void* r, const void* k, const void* v, const void* x,
        const float* u, const float* state_in, void* out, float* state_out,
        long long batch_stride, bool in_bf16, bool out_f32, Path path, void* stream) {
    if (N != wkv6::kHeadSize) return WKV6_ERR_UNSUPPORTED;
    if (B < 0 || T < 0 || H < 1 || H > 262144) return WKV6_ERR_SHAPE;   // 32-bit row offsets in the kernels
    if (!u) return WKV6_ERR_NULL;
    if (B == 0) return WKV6_OK;
    const long long need = static_cast<long long>(T) * H * N;
    if (T > 0) {
        if (!r || !k || !v || !x || !out) return WKV6_ERR_NULL;
        if (batch_stride < need) return WKV6_ERR_SHAPE;
        if (misaligned(r) || misaligned(k) || misaligned(v) || misaligned(x) || misaligned(out))
            return WKV6_ERR_ALIGN;
        if (batch_stride % 8 != 0) return WKV6_ERR_ALIGN;
    }
    if (misaligned(u) || misaligned(state_in) || misaligned(state_out)) return WKV6_ERR_ALIGN;
    if (static_cast<long long>(B) * H > 0x7fffffffLL) return WKV6_ERR_SHAPE;

    wkv6::Args a;
    a.B = B; a.T = T; a.H = H;
    a.r = r; a.k = k; a.v = v; a.x = x; a.u = u;
    a.state_in = state_in; a.out = out; a.state_out = state_out;
    a.batch_stride = batch_stride;

    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t err;
    if (T == 0)
        err = wkv6::launch_state_passthrough(a, s);
    else if (path == Path::kRecurrent)
        err = wkv6::launch_recurrent(a, in_bf16, s);
    else
        err = wkv6::launch_chunked(a, out_f32, s);
    return err == hipSuccess ? WKV6_OK : WKV6_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int wkv6_prefill_bf16(int B, int T, int H, int N, const void* r, const void* k, const void* v,
                      const void* x, const float* u, const float* state_in, void* out,
                      float* state_out, void* stream) {
    return run(B, T, H, N, r, k, v, x, u, state_in, out, state_out,
               static_cast<long long>(T) * H * N, true, false, Path::kChunked, stream);
}

int wkv6_prefill_bf16_f32out(int B, int T, int H, int N, const void* r, const void* k,
                             const void* v, const void* x, const float* u, const float* state_in,
                             float* out, float* state_out, void* stream) {
    return run(B, T, H, N, r, k, v, x, u, state_in, out, state_out,
               static_cast<long long>(T) * H * N, true, true, Path::kChunked, stream);
}

int wkv6_prefill_bf16_strided(int B, int T, int H, int N, const void* r, const void* k,
                              const void* v, const void* x, const float* u, const float* state_in,
                              void* out, float* state_out, long long batch_stride, int out_dtype,
                              void* stream) {
    if (out_dtype != WKV6_DTYPE_BF16 && out_dtype != WKV6_DTYPE_F32) return WKV6_ERR_UNSUPPORTED;
    return run(B, T, H, N, r, k, v, x, u, state_in, out, state_out, batch_stride, true,
               out_dtype == WKV6_DTYPE_F32, Path::kChunked, stream);
}

int wkv6_prefill_f32(int B, int T, int H, int N, const float* r, const float* k, const float* v,
                     const float* x, const float* u, const float* state_in, float* out,
                     float* state_out, void* stream) {
    return run(B, T, H, N, r, k, v, x, u, state_in, out, state_out,
               static_cast<long long>(T) * H * N, false, true, Path::kRecurrent, stream);
}

int wkv6_prefill_bf16_recurrent(int B, int T, int H, int N, const void* r, const void* k,
                                const void* v, const void* x, const float* u,
                                const float* state_in, float* out, float* state_out,
                                void* stream) {
    return run(B, T, H, N, r, k, v, x, u, state_in, out, state_out,
               static_cast<long long>(T) * H * N, true, true, Path::kRecurrent, stream);
}

const char* wkv6_status_string(int status) {
    switch (status) {
        case WKV6_OK: return "ok";
        case WKV6_ERR_NULL: return "a required pointer is NULL";
        case WKV6_ERR_SHAPE: return "invalid shape or stride";
        case WKV6_ERR_UNSUPPORTED: return "unsupported head size or dtype";
        case WKV6_ERR_LAUNCH: return "kernel launch failed";
        case WKV6_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
        default: return "unknown status";
    }
}

int wkv6_version(void) { return 100; }

}  // extern "C"

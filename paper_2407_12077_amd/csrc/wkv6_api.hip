// C ABI of the WKV6 prefill library: argument validation and dispatch only.
// Every step of the computation runs in the kernels this file launches.
#include "../../include/wkv6.h"
#include "wkv6_launch.h"

#include <cstdint>
#include <mutex>

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<std::uintptr_t>(p) & 15u) != 0; }

enum class Path { kChunked, kRecurrent, kBySize };

// Sequences at most this long go to the token-by-token kernel when the caller leaves the
// choice to the library (append / decode shapes): with thousands of (batch, head) units and
// a few tokens each the work is streaming the state once.  Measured crossover on MI355X with
// 8192 units: about 8 tokens (the chunked kernel runs the units of a workgroup back to back, one
// window each at these lengths).
constexpr int kRecurrentMaxTokens = 6;

// `uprime` selects the form: nullptr = Finch (bonus u), otherwise Finch-C2 (u unused, may be null).
int run(int B, int T, int H, int N, const void* r, const void* k, const void* v, const void* x,
        const float* u, const float* state_in, void* out, float* state_out,
        long long batch_stride, bool in_bf16, bool out_f32, Path path, void* stream,
        const void* uprime = nullptr, bool finch_c2 = false, float* moments = nullptr,
        bool want_moments = false) {
    if (N != wkv6::kHeadSize) return WKV6_ERR_UNSUPPORTED;
    if (B < 0 || T < 0 || H < 1 || H > 262144) return WKV6_ERR_SHAPE;   // 32-bit row offsets in the kernels
    if (!finch_c2 && !u) return WKV6_ERR_NULL;
    if (B == 0) return WKV6_OK;
    const long long need = static_cast<long long>(T) * H * N;
    if (T > 0) {
        if (!r || !k || !v || !x || !out || (finch_c2 && !uprime)) return WKV6_ERR_NULL;
        if (batch_stride < need) return WKV6_ERR_SHAPE;
        if (misaligned(r) || misaligned(k) || misaligned(v) || misaligned(x) || misaligned(out) ||
            misaligned(uprime))
            return WKV6_ERR_ALIGN;
        if (batch_stride % 8 != 0) return WKV6_ERR_ALIGN;
    }
    if (misaligned(u) || misaligned(state_in) || misaligned(state_out)) return WKV6_ERR_ALIGN;
    if (static_cast<long long>(B) * H > 0x7fffffffLL) return WKV6_ERR_SHAPE;
    if (want_moments && T > 0) {
        if (!moments) return WKV6_ERR_NULL;
        if (misaligned(moments)) return WKV6_ERR_ALIGN;
    }

    wkv6::Args a;
    a.B = B; a.T = T; a.H = H;
    a.r = r; a.k = k; a.v = v; a.x = x; a.u = u;
    a.finch_c2 = finch_c2;
    a.uprime = finch_c2 ? uprime : nullptr;
    a.state_in = state_in; a.out = out; a.state_out = state_out;
    a.batch_stride = batch_stride;
    a.segs = 1; a.T_last = T; a.seg_stride = 0; a.decay_out = nullptr; a.unit_stride = 0;
    a.moments = moments;
    a.y = nullptr; a.lambda = nullptr; a.bw = nullptr;

    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t err;
    if (T == 0)
        err = wkv6::launch_state_passthrough(a, s);
    else if (path == Path::kRecurrent || (path == Path::kBySize && T <= kRecurrentMaxTokens))
        err = wkv6::launch_recurrent(a, in_bf16, in_bf16 && !out_f32, s);
    else if (want_moments)
        err = wkv6::launch_chunked(a, wkv6::ChunkedMode::kBf16OutMoments, s);
    else
        err = wkv6::launch_chunked(a, out_f32 ? wkv6::ChunkedMode::kF32Out : wkv6::ChunkedMode::kBf16Out, s);
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

int wkv6_finch_c2_prefill_bf16(int B, int T, int H, int N, const void* r, const void* kbar,
                               const void* v, const void* x, const void* uprime,
                               const float* state_in, void* out, float* state_out, void* stream) {
    return run(B, T, H, N, r, kbar, v, x, nullptr, state_in, out, state_out,
               static_cast<long long>(T) * H * N, true, false, Path::kChunked, stream, uprime, true);
}

int wkv6_finch_c2_prefill_bf16_f32out(int B, int T, int H, int N, const void* r, const void* kbar,
                                      const void* v, const void* x, const void* uprime,
                                      const float* state_in, float* out, float* state_out,
                                      void* stream) {
    return run(B, T, H, N, r, kbar, v, x, nullptr, state_in, out, state_out,
               static_cast<long long>(T) * H * N, true, true, Path::kChunked, stream, uprime, true);
}

int wkv6_finch_c2_prefill_bf16_strided(int B, int T, int H, int N, const void* r, const void* kbar,
                                       const void* v, const void* x, const void* uprime,
                                       const float* state_in, void* out, float* state_out,
                                       long long batch_stride, int out_dtype, void* stream) {
    if (out_dtype != WKV6_DTYPE_BF16 && out_dtype != WKV6_DTYPE_F32) return WKV6_ERR_UNSUPPORTED;
    return run(B, T, H, N, r, kbar, v, x, nullptr, state_in, out, state_out, batch_stride, true,
               out_dtype == WKV6_DTYPE_F32, Path::kChunked, stream, uprime, true);
}

int wkv6_finch_c2_prefill_bf16_moments(int B, int T, int H, int N, const void* r, const void* kbar,
                                       const void* v, const void* x, const void* uprime,
                                       const float* state_in, void* out, float* moments, float* state_out,
                                       void* stream) {
    return run(B, T, H, N, r, kbar, v, x, nullptr, state_in, out, state_out,
               static_cast<long long>(T) * H * N, true, false, Path::kChunked, stream, uprime, true, moments,
               true);
}

}  // extern "C"

namespace {

// Both forms of the prefill with the decay logits formed in the kernel; `uprime` non-null selects
// the Finch-C2 form (then `u` is unused), otherwise `u` is the Finch bonus.
int run_lora(int B, int T, int H, int N, int R, const void* r, const void* k, const void* v, const void* y,
             const float* lambda, const void* b_omega, const float* u, const void* uprime, bool finch_c2,
             const float* state_in, void* out, float* moments, float* state_out, void* stream) {
    if (N != wkv6::kHeadSize || R != wkv6::kLoraRank) return WKV6_ERR_UNSUPPORTED;
    if (B < 0 || T < 0 || H < 1 || H > 262144) return WKV6_ERR_SHAPE;
    if (!finch_c2 && !u) return WKV6_ERR_NULL;
    if (B == 0) return WKV6_OK;
    if (T > 0) {
        if (!r || !k || !v || !y || !lambda || !b_omega || (finch_c2 && !uprime) || !out) return WKV6_ERR_NULL;
        if (misaligned(r) || misaligned(k) || misaligned(v) || misaligned(y) || misaligned(lambda) ||
            misaligned(b_omega) || misaligned(uprime) || misaligned(out) || misaligned(moments))
            return WKV6_ERR_ALIGN;
    }
    if (misaligned(u) || misaligned(state_in) || misaligned(state_out)) return WKV6_ERR_ALIGN;
    if (static_cast<long long>(B) * H > 0x7fffffffLL) return WKV6_ERR_SHAPE;

    wkv6::Args a;
    a.B = B; a.T = T; a.H = H;
    a.r = r; a.k = k; a.v = v; a.x = nullptr; a.u = u;
    a.finch_c2 = finch_c2;
    a.uprime = finch_c2 ? uprime : nullptr;
    a.state_in = state_in; a.out = out; a.state_out = state_out;
    a.batch_stride = static_cast<long long>(T) * H * N;
    a.segs = 1; a.T_last = T; a.seg_stride = 0; a.decay_out = nullptr; a.unit_stride = 0;
    a.moments = moments;
    a.y = y; a.lambda = lambda; a.bw = b_omega;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const hipError_t err = T == 0 ? wkv6::launch_state_passthrough(a, s)
                                  : wkv6::launch_chunked(a, moments ? wkv6::ChunkedMode::kBf16OutLoraMoments
                                                                    : wkv6::ChunkedMode::kBf16OutLora, s);
    return err == hipSuccess ? WKV6_OK : WKV6_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int wkv6_finch_c2_prefill_lora_bf16(int B, int T, int H, int N, int R, const void* r, const void* kbar,
                                    const void* v, const void* y, const float* lambda, const void* b_omega,
                                    const void* uprime, const float* state_in, void* out, float* moments,
                                    float* state_out, void* stream) {
    return run_lora(B, T, H, N, R, r, kbar, v, y, lambda, b_omega, nullptr, uprime, true, state_in, out, moments,
                    state_out, stream);
}

int wkv6_prefill_lora_bf16(int B, int T, int H, int N, int R, const void* r, const void* k, const void* v,
                           const void* y, const float* lambda, const void* b_omega, const float* u,
                           const float* state_in, void* out, float* state_out, void* stream) {
    return run_lora(B, T, H, N, R, r, k, v, y, lambda, b_omega, u, nullptr, false, state_in, out, nullptr, state_out,
                    stream);
}

int wkv6_layernorm_finalize(int B, int T, int H, int N, const float* moments, float eps, float* mean_rstd,
                            void* stream) {
    if (N != wkv6::kHeadSize) return WKV6_ERR_UNSUPPORTED;
    if (B < 0 || T < 0 || H < 1 || H > 262144 || B > 65535 || !(eps >= 0.f)) return WKV6_ERR_SHAPE;
    if (B == 0 || T == 0) return WKV6_OK;
    if (!moments || !mean_rstd) return WKV6_ERR_NULL;
    if (misaligned(moments) || misaligned(mean_rstd)) return WKV6_ERR_ALIGN;
    const hipError_t err = wkv6::launch_layernorm_finalize(B, T, H, moments, eps, mean_rstd,
                                                           static_cast<hipStream_t>(stream));
    return err == hipSuccess ? WKV6_OK : WKV6_ERR_LAUNCH;
}

int wkv6_layernorm_apply_bf16(int B, int T, int H, int N, const void* o, const float* mean_rstd, const float* gamma,
                              const float* beta, void* y, int out_dtype, void* stream) {
    if (out_dtype != WKV6_DTYPE_BF16 && out_dtype != WKV6_DTYPE_F32) return WKV6_ERR_UNSUPPORTED;
    if (N != wkv6::kHeadSize) return WKV6_ERR_UNSUPPORTED;
    if (B < 0 || T < 0 || H < 1 || H > 262144) return WKV6_ERR_SHAPE;
    if (B == 0 || T == 0) return WKV6_OK;
    const long long tokens = static_cast<long long>(B) * T;
    if (!o || !mean_rstd || !gamma || !beta || !y) return WKV6_ERR_NULL;
    if (misaligned(o) || misaligned(mean_rstd) || misaligned(gamma) || misaligned(beta) || misaligned(y))
        return WKV6_ERR_ALIGN;
    const hipError_t err = wkv6::launch_layernorm_apply(tokens, H * N, o, mean_rstd, gamma, beta, y,
                                                        out_dtype == WKV6_DTYPE_F32, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? WKV6_OK : WKV6_ERR_LAUNCH;
}

int wkv6_append_bf16(int B, int T, int H, int N, const void* r, const void* k, const void* v,
                     const void* x, const float* u, const float* state_in, void* out,
                     float* state_out, void* stream) {
    return run(B, T, H, N, r, k, v, x, u, state_in, out, state_out,
               static_cast<long long>(T) * H * N, true, false, Path::kBySize, stream);
}

int wkv6_finch_c2_append_bf16(int B, int T, int H, int N, const void* r, const void* kbar,
                              const void* v, const void* x, const void* uprime,
                              const float* state_in, void* out, float* state_out, void* stream) {
    return run(B, T, H, N, r, kbar, v, x, nullptr, state_in, out, state_out,
               static_cast<long long>(T) * H * N, true, false, Path::kBySize, stream, uprime, true);
}

int wkv6_decode_bf16(int B, int H, int N, const void* r, const void* k, const void* v,
                     const void* x, const float* u, float* state, void* out, void* stream) {
    if (!state) return WKV6_ERR_NULL;
    return run(B, 1, H, N, r, k, v, x, u, state, out, state,
               static_cast<long long>(H) * N, true, false, Path::kRecurrent, stream);
}

int wkv6_finch_c2_decode_bf16(int B, int H, int N, const void* r, const void* kbar, const void* v,
                              const void* x, const void* uprime, float* state, void* out,
                              void* stream) {
    if (!state) return WKV6_ERR_NULL;
    return run(B, 1, H, N, r, kbar, v, x, nullptr, state, out, state,
               static_cast<long long>(H) * N, true, false, Path::kRecurrent, stream, uprime, true);
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

int wkv6_key_compress_bf16(long long M, int D, const void* x, const void* w_kd, void* c, int out_dtype,
                           void* stream) {
    if (out_dtype != WKV6_DTYPE_BF16 && out_dtype != WKV6_DTYPE_F32) return WKV6_ERR_UNSUPPORTED;
    if (D < 256 || D % 256 != 0 || D > 65536) return WKV6_ERR_UNSUPPORTED;
    if (M < 0 || ((M + 127) / 128 + 8) * ((D / 16 + 127) / 128) > 0x7fffffffLL) return WKV6_ERR_SHAPE;   // grid size
    if (M == 0) return WKV6_OK;
    if (!x || !w_kd || !c) return WKV6_ERR_NULL;
    if (misaligned(x) || misaligned(w_kd) || misaligned(c)) return WKV6_ERR_ALIGN;
    const hipError_t err = wkv6::launch_key_compress(M, D, x, w_kd, c, out_dtype == WKV6_DTYPE_F32,
                                                     static_cast<hipStream_t>(stream));
    return err == hipSuccess ? WKV6_OK : WKV6_ERR_LAUNCH;
}

int wkv6_decay_lora_input_bf16(int B, int T, int D, int R_d, int R, const void* x, const void* x_prev,
                               const float* mu_x, const float* lambda_d, const void* a_d, const void* b_d,
                               const void* a_omega, void* y, int out_dtype, void* stream) {
    if (out_dtype != WKV6_DTYPE_BF16 && out_dtype != WKV6_DTYPE_F32) return WKV6_ERR_UNSUPPORTED;
    if (R_d != 32 || R != wkv6::kLoraRank) return WKV6_ERR_UNSUPPORTED;
    if (D < 128 || D % 128 != 0 || D > 65536) return WKV6_ERR_UNSUPPORTED;
    if (B < 0 || T < 0) return WKV6_ERR_SHAPE;
    if (B == 0 || T == 0) return WKV6_OK;
    if (static_cast<long long>(B) * ((T + 127) / 128) > 0x7fffffffLL) return WKV6_ERR_SHAPE;  // grid size
    if (!x || !mu_x || !lambda_d || !a_d || !b_d || !a_omega || !y) return WKV6_ERR_NULL;
    if (misaligned(x) || misaligned(x_prev) || misaligned(mu_x) || misaligned(lambda_d) || misaligned(a_d) ||
        misaligned(b_d) || misaligned(a_omega) || misaligned(y))
        return WKV6_ERR_ALIGN;
    const hipError_t err = wkv6::launch_decay_input(B, T, D, x, x_prev, mu_x, lambda_d, a_d, b_d, a_omega, y,
                                                    out_dtype == WKV6_DTYPE_F32, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? WKV6_OK : WKV6_ERR_LAUNCH;
}

long long wkv6_arena_layout(int count, const long long* bytes, long long* offsets) {
    if (count < 0 || count > 64) return -1;
    if (count > 0 && (!bytes || !offsets)) return -1;
    long long cursor = 0;
    for (int i = 0; i < count; ++i) {
        if (bytes[i] < 0 || bytes[i] > (1ll << 46)) return -1;
        cursor = (cursor + WKV6_PLACEMENT_ALIGN - 1) / WKV6_PLACEMENT_ALIGN * WKV6_PLACEMENT_ALIGN;
        offsets[i] = cursor + WKV6_PLACEMENT_STEP * (i % 8);
        cursor = offsets[i] + bytes[i];
    }
    return (cursor + WKV6_PLACEMENT_ALIGN - 1) / WKV6_PLACEMENT_ALIGN * WKV6_PLACEMENT_ALIGN;
}

const char* wkv6_status_string(int status) {
    switch (status) {
        case WKV6_OK: return "ok";
        case WKV6_ERR_NULL: return "a required pointer is NULL";
        case WKV6_ERR_SHAPE: return "invalid shape or stride";
        case WKV6_ERR_UNSUPPORTED: return "unsupported head size or dtype";
        case WKV6_ERR_LAUNCH: return "kernel launch failed";
        case WKV6_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
        case WKV6_ERR_WORKSPACE: return "shape needs more scratch than the library holds";
        default: return "unknown status";
    }
}

int wkv6_version(void) { return 500; }

}  // extern "C"

// ---- token-split variant: three enqueued passes over caller-provided workspace

namespace {

struct SplitPlan {
    int segs;        // segments actually used
    int seg_len;     // tokens per segment (multiple of 32), last one shorter
    int last_len;
};

SplitPlan plan_split(int T, int segments) {
    SplitPlan p;
    if (segments < 1) segments = 1;
    long long len = (static_cast<long long>(T) + segments - 1) / segments;
    len = (len + 31) / 32 * 32;
    if (len < 32) len = 32;
    p.seg_len = static_cast<int>(len);
    p.segs = static_cast<int>((T + len - 1) / len);
    if (p.segs < 1) p.segs = 1;
    p.last_len = T - (p.segs - 1) * p.seg_len;
    return p;
}

}  // namespace

extern "C" {

int wkv6_split_segments(int B, int T, int H, int N) {
    if (N != wkv6::kHeadSize || B < 1 || T < 1 || H < 1) return 1;
    const long long units = static_cast<long long>(B) * H;
    const int cus = 256;                         // workgroups resident at once on an MI355X (one per CU); a
                                                 // pure function of the shape so that it needs no device
    if (units * 4 > cus * 3) return 1;           // already fills three quarters of the chip
    long long segs = cus / units;
    const long long by_len = T / 2048;           // keep segments long enough to amortise pass 1
    if (segs > by_len) segs = by_len;
    return segs < 2 ? 1 : static_cast<int>(segs);
}

long long wkv6_split_workspace_bytes(int B, int T, int H, int N, int segments) {
    if (N != wkv6::kHeadSize || B < 0 || T < 0 || H < 1 || segments < 1) return -1;
    const SplitPlan p = plan_split(T > 0 ? T : 1, segments);
    return static_cast<long long>(B) * p.segs * H * (wkv6::kHeadSize * wkv6::kHeadSize + wkv6::kHeadSize) * 4;
}

}  // extern "C"

// ---- library-owned scratch for the entry point that may not allocate

namespace {

// Per-segment local states and decay totals of wkv6_prefill_bf16_split_noalloc.  Every GPU the
// library runs on holds its own copy of this array, at its own address, until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; the device address it
// returns is what kernels, copies and fills must be given.
constexpr long long kScratchBytes = 8ll << 20;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
int scratch_of_current_device(void** ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return WKV6_ERR_LAUNCH;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return WKV6_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return WKV6_OK;
}

int run_split(int B, int T, int H, int N, const void* r, const void* k, const void* v, const void* x,
              const float* u, const void* uprime, bool finch_c2, const float* state_in, void* out,
              float* state_out, int out_dtype, int segments, void* workspace,
              long long workspace_bytes, void* stream) {
    if (out_dtype != WKV6_DTYPE_BF16 && out_dtype != WKV6_DTYPE_F32) return WKV6_ERR_UNSUPPORTED;
    if (N != wkv6::kHeadSize) return WKV6_ERR_UNSUPPORTED;
    if (B < 0 || T < 0 || H < 1 || H > 262144 || segments < 1) return WKV6_ERR_SHAPE;
    const SplitPlan p = plan_split(T > 0 ? T : 1, segments);
    if (T == 0 || B == 0 || p.segs == 1)
        return run(B, T, H, N, r, k, v, x, u, state_in, out, state_out,
                   static_cast<long long>(T) * H * N, true, out_dtype == WKV6_DTYPE_F32,
                   Path::kChunked, stream, uprime, finch_c2);
    if ((!finch_c2 && !u) || (finch_c2 && !uprime) || !r || !k || !v || !x || !out || !workspace)
        return WKV6_ERR_NULL;
    if (misaligned(r) || misaligned(k) || misaligned(v) || misaligned(x) || misaligned(out) ||
        misaligned(u) || misaligned(uprime) || misaligned(state_in) || misaligned(state_out) ||
        misaligned(workspace))
        return WKV6_ERR_ALIGN;
    if (workspace_bytes < wkv6_split_workspace_bytes(B, T, H, N, segments)) return WKV6_ERR_SHAPE;
    if (static_cast<long long>(B) * p.segs * H > 0x7fffffffLL) return WKV6_ERR_SHAPE;

    float* seg_state = static_cast<float*>(workspace);
    float* seg_decay = seg_state + static_cast<long long>(B) * p.segs * H * 4096;
    hipStream_t s = static_cast<hipStream_t>(stream);

    wkv6::Args a;
    a.B = B; a.T = p.seg_len; a.H = H;
    a.r = r; a.k = k; a.v = v; a.x = x; a.u = u;
    a.finch_c2 = finch_c2;
    a.uprime = finch_c2 ? uprime : nullptr;
    a.batch_stride = static_cast<long long>(T) * H * N;
    a.segs = p.segs; a.T_last = p.last_len; a.unit_stride = 0; a.moments = nullptr;
    a.y = nullptr; a.lambda = nullptr; a.bw = nullptr;
    a.seg_stride = static_cast<long long>(p.seg_len) * H * N;
    // pass 1: every segment but the last (nothing follows it) from a zero state, no output: its
    // local state and total decay
    a.state_in = nullptr; a.out = nullptr; a.state_out = seg_state; a.decay_out = seg_decay;
    a.segs_launched = p.segs - 1;
    if (wkv6::launch_chunked(a, wkv6::ChunkedMode::kStateOnly, s) != hipSuccess) return WKV6_ERR_LAUNCH;
    // pass 2: the state entering every segment (in place)
    if (wkv6::launch_combine_segments(B, H, p.segs, state_in, seg_state, seg_decay, nullptr, false, s) != hipSuccess)
        return WKV6_ERR_LAUNCH;
    // pass 3: the full computation of every segment from its true entering state; the last
    // segment's workgroups leave the sequence's final state
    a.segs_launched = 0;
    a.state_in = seg_state; a.out = out; a.state_out = state_out; a.state_out_final = true; a.decay_out = nullptr;
    const wkv6::ChunkedMode mode = out_dtype == WKV6_DTYPE_F32 ? wkv6::ChunkedMode::kF32Out
                                                               : wkv6::ChunkedMode::kBf16Out;
    if (wkv6::launch_chunked(a, mode, s) != hipSuccess) return WKV6_ERR_LAUNCH;
    return WKV6_OK;
}

}  // namespace

extern "C" {

int wkv6_prefill_bf16_split(int B, int T, int H, int N, const void* r, const void* k, const void* v,
                            const void* x, const float* u, const float* state_in, void* out,
                            float* state_out, int out_dtype, int segments, void* workspace,
                            long long workspace_bytes, void* stream) {
    return run_split(B, T, H, N, r, k, v, x, u, nullptr, false, state_in, out, state_out, out_dtype,
                     segments, workspace, workspace_bytes, stream);
}

int wkv6_prefill_bf16_split_noalloc(int B, int T, int H, int N, const void* r, const void* k, const void* v,
                                    const void* x, const float* u, const float* state_in, void* out,
                                    float* state_out, int out_dtype, int segments, void* stream) {
    const long long need = wkv6_split_workspace_bytes(B, T, H, N, segments);
    if (need < 0) return N != wkv6::kHeadSize ? WKV6_ERR_UNSUPPORTED : WKV6_ERR_SHAPE;
    if (need > kScratchBytes) return WKV6_ERR_WORKSPACE;
    void* ws = nullptr;
    const int status = scratch_of_current_device(&ws);
    if (status != WKV6_OK) return status;
    return run_split(B, T, H, N, r, k, v, x, u, nullptr, false, state_in, out, state_out, out_dtype,
                     segments, ws, kScratchBytes, stream);
}

int wkv6_finch_c2_prefill_bf16_split(int B, int T, int H, int N, const void* r, const void* kbar,
                                     const void* v, const void* x, const void* uprime,
                                     const float* state_in, void* out, float* state_out,
                                     int out_dtype, int segments, void* workspace,
                                     long long workspace_bytes, void* stream) {
    return run_split(B, T, H, N, r, kbar, v, x, nullptr, uprime, true, state_in, out, state_out,
                     out_dtype, segments, workspace, workspace_bytes, stream);
}

}  // extern "C"

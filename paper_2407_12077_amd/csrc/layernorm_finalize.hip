// Token statistics of the LayerNorm over all heads (Finch-C2 Time Mixing, output equation) from
// the per-head partial moments the prefill kernel emits next to its output.
//
// Each (batch, head, token) contributes the sum s of its N values and the squared deviations m2
// from its own mean.  Groups of values combine exactly (Chan, Golub, LeVeque): with counts n_a,
// n_b, means mu_a, mu_b:  M2 = M2_a + M2_b + (mu_b - mu_a)^2 n_a n_b / (n_a + n_b).  A workgroup
// takes 64 consecutive tokens of one batch; each of its four waves folds every fourth head (a
// lane per token, so every read is a contiguous run of 8-byte pairs), then the first wave
// combines the four partial results.
#include "wkv6_launch.h"

namespace wkv6 {
namespace {

struct Group {
    float count, mean, m2;
};

__device__ __forceinline__ Group combine(const Group& a, const Group& b) {
    if (b.count == 0.f) return a;
    const float total = a.count + b.count;
    const float delta = b.mean - a.mean;
    return Group{total, fmaf(delta, b.count / total, a.mean),
                 a.m2 + b.m2 + delta * delta * (a.count * b.count / total)};
}

__global__ __launch_bounds__(256) void layernorm_finalize_kernel(int T, int H, const float2* moments, float eps,
                                                                 float2* mean_rstd) {
    __shared__ Group part[3][64];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t = blockIdx.x * 64 + lane;
    const int b = blockIdx.y;
    Group g{0.f, 0.f, 0.f};
    if (t < T) {
        const float2* src = moments + static_cast<long long>(b) * H * T + t;
#pragma unroll 4
        for (int h = wave; h < H; h += 4) {
            const float2 p = src[static_cast<long long>(h) * T];
            g = combine(g, Group{static_cast<float>(kHeadSize), p.x * (1.f / kHeadSize), p.y});
        }
    }
    if (wave > 0) part[wave - 1][lane] = g;
    __syncthreads();
    if (wave == 0 && t < T) {
#pragma unroll
        for (int w = 0; w < 3; ++w) g = combine(g, part[w][lane]);
        mean_rstd[static_cast<long long>(b) * T + t] = make_float2(g.mean, 1.f / sqrtf(g.m2 / g.count + eps));
    }
}

// The normalisation itself, for callers whose projection GEMM has no row-scaling epilogue:
// y = (o - mean) * rstd * gamma + beta over the D = H*N values of each token; 8 channels (16 bytes
// of bf16) per item, every tensor touched once, fp32 arithmetic, one rounding of the result.  A thread
// keeps four items in flight (four loads, then four stores; a thread reads an item before it writes
// it, so y may be o).  Two forms: when a token's D/8 items are a multiple of 256 a workgroup owns a
// strip of 256 item columns over a run of tokens, so a thread's gain and offset stay in registers
// and the token's (mean, rstd) is a scalar load; otherwise items are dealt out in runs of 1024 and
// the gain and offset are fetched per item (they stay in L1).
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
constexpr int kInFlight = 4;

template <bool kOutF32>
__device__ __forceinline__ void normalise_item(const uint4v raw, const float2 ms, const float4 g0, const float4 g1,
                                               const float4 b0, const float4 b1, void* y, long long item) {
    const float gm[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
    const float bt[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
    float v[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(raw[i] << 16);
        v[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = fmaf((v[i] - ms.x) * ms.y, gm[i], bt[i]);
    if constexpr (kOutF32) {
        typedef float float4v __attribute__((ext_vector_type(4)));
        float4v* dst = static_cast<float4v*>(y) + 2 * item;
        __builtin_nontemporal_store(float4v{v[0], v[1], v[2], v[3]}, dst);
        __builtin_nontemporal_store(float4v{v[4], v[5], v[6], v[7]}, dst + 1);
    } else {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float float2v __attribute__((ext_vector_type(2)));
        uint4v q;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            q[i] = __builtin_bit_cast(unsigned, __builtin_convertvector(float2v{v[2 * i], v[2 * i + 1]}, bf16x2));
        __builtin_nontemporal_store(q, static_cast<uint4v*>(y) + item);
    }
}

// grid (token runs, strips of 256 item columns); items_per_token is a multiple of 256
template <bool kOutF32>
__global__ __launch_bounds__(256) void layernorm_apply_strip_kernel(long long tokens, int tokens_per_block,
                                                                    int items_per_token, const uint4v* o,
                                                                    const float2* mean_rstd, const float4* gamma,
                                                                    const float4* beta, void* y) {
    const int column = blockIdx.y * 256 + threadIdx.x;
    const float4 g0 = gamma[2 * column], g1 = gamma[2 * column + 1], b0 = beta[2 * column], b1 = beta[2 * column + 1];
    const long long t0 = static_cast<long long>(blockIdx.x) * tokens_per_block;
    const long long t1 = t0 + tokens_per_block < tokens ? t0 + tokens_per_block : tokens;
    for (long long t = t0; t < t1; t += kInFlight) {
        uint4v raw[kInFlight];
        float2 ms[kInFlight];
#pragma unroll
        for (int j = 0; j < kInFlight; ++j)
            if (t + j < t1) {
                raw[j] = __builtin_nontemporal_load(o + (t + j) * items_per_token + column);
                ms[j] = mean_rstd[t + j];
            }
#pragma unroll
        for (int j = 0; j < kInFlight; ++j)
            if (t + j < t1) normalise_item<kOutF32>(raw[j], ms[j], g0, g1, b0, b1, y, (t + j) * items_per_token + column);
    }
}

// any items_per_token: block b owns items [b * items_per_block, (b + 1) * items_per_block), a multiple of 1024
template <bool kOutF32>
__global__ __launch_bounds__(256) void layernorm_apply_kernel(long long items, long long items_per_block,
                                                              int items_per_token, const uint4v* o,
                                                              const float2* mean_rstd, const float4* gamma,
                                                              const float4* beta, void* y) {
    const long long i0 = blockIdx.x * items_per_block;
    const long long i1 = i0 + items_per_block < items ? i0 + items_per_block : items;
    for (long long base = i0 + threadIdx.x; base < i1; base += kInFlight * 256) {
        uint4v raw[kInFlight];
#pragma unroll
        for (int j = 0; j < kInFlight; ++j)
            if (base + j * 256 < i1) raw[j] = __builtin_nontemporal_load(o + base + j * 256);
#pragma unroll
        for (int j = 0; j < kInFlight; ++j) {
            const long long item = base + j * 256;
            if (item < i1) {
                const long long token = item / items_per_token;
                const int c8 = static_cast<int>(item - token * items_per_token);
                normalise_item<kOutF32>(raw[j], mean_rstd[token], gamma[2 * c8], gamma[2 * c8 + 1], beta[2 * c8],
                                        beta[2 * c8 + 1], y, item);
            }
        }
    }
}

}  // namespace

hipError_t launch_layernorm_apply(long long tokens, int D, const void* o, const float* mean_rstd, const float* gamma,
                                  const float* beta, void* y, bool out_f32, hipStream_t stream) {
    const int items_per_token = D / 8;
    const long long items = tokens * items_per_token;
    const int cus = compute_units();
    const uint4v* src = static_cast<const uint4v*>(o);
    const float2* ms = reinterpret_cast<const float2*>(mean_rstd);
    const float4* gm = reinterpret_cast<const float4*>(gamma);
    const float4* bt = reinterpret_cast<const float4*>(beta);
    if (items_per_token % 256 == 0) {
        // about eight workgroups per compute unit, each a run of at least kInFlight tokens
        const int strips = items_per_token / 256;
        long long runs = (8ll * cus + strips - 1) / strips;
        const long long most = (tokens + kInFlight - 1) / kInFlight;
        if (runs > most) runs = most;
        const int tokens_per_block = static_cast<int>((tokens + runs - 1) / runs);
        const dim3 grid(static_cast<unsigned>((tokens + tokens_per_block - 1) / tokens_per_block),
                        static_cast<unsigned>(strips));
        if (out_f32)
            hipLaunchKernelGGL(layernorm_apply_strip_kernel<true>, grid, dim3(256), 0, stream, tokens, tokens_per_block,
                               items_per_token, src, ms, gm, bt, y);
        else
            hipLaunchKernelGGL(layernorm_apply_strip_kernel<false>, grid, dim3(256), 0, stream, tokens, tokens_per_block,
                               items_per_token, src, ms, gm, bt, y);
        return hipGetLastError();
    }
    const long long step = kInFlight * 256;
    long long blocks = 8ll * cus;
    long long items_per_block = ((items + blocks - 1) / blocks + step - 1) / step * step;
    blocks = (items + items_per_block - 1) / items_per_block;
    const dim3 grid(static_cast<unsigned>(blocks));
    if (out_f32)
        hipLaunchKernelGGL(layernorm_apply_kernel<true>, grid, dim3(256), 0, stream, items, items_per_block,
                           items_per_token, src, ms, gm, bt, y);
    else
        hipLaunchKernelGGL(layernorm_apply_kernel<false>, grid, dim3(256), 0, stream, items, items_per_block,
                           items_per_token, src, ms, gm, bt, y);
    return hipGetLastError();
}

hipError_t launch_layernorm_finalize(int B, int T, int H, const float* moments, float eps, float* mean_rstd,
                                     hipStream_t stream) {
    const dim3 grid(static_cast<unsigned>((T + 63) / 64), static_cast<unsigned>(B));
    hipLaunchKernelGGL(layernorm_finalize_kernel, grid, dim3(256), 0, stream, T, H,
                       reinterpret_cast<const float2*>(moments), eps, reinterpret_cast<float2*>(mean_rstd));
    return hipGetLastError();
}

}  // namespace wkv6

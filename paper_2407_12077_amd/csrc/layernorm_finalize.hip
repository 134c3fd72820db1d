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
// y = (o - mean) * rstd * gamma + beta over the D = H*N values of each token; 8 channels per thread,
// every tensor touched once (non-temporal), fp32 arithmetic, one rounding of the result.
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

template <bool kOutF32>
__global__ __launch_bounds__(256) void layernorm_apply_kernel(long long groups, int groups_per_token, const uint4v* o,
                                                              const float2* mean_rstd, const float4* gamma,
                                                              const float4* beta, void* y) {
    const long long g = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
    if (g >= groups) return;
    const long long token = g / groups_per_token;
    const int c8 = static_cast<int>(g - token * groups_per_token);
    const uint4v raw = __builtin_nontemporal_load(o + g);
    const float2 ms = mean_rstd[token];
    const float4 g0 = gamma[2 * c8], g1 = gamma[2 * c8 + 1], b0 = beta[2 * c8], b1 = beta[2 * c8 + 1];
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
        float4* dst = static_cast<float4*>(y) + 2 * g;
        __builtin_nontemporal_store(v[0], &dst[0].x); __builtin_nontemporal_store(v[1], &dst[0].y);
        __builtin_nontemporal_store(v[2], &dst[0].z); __builtin_nontemporal_store(v[3], &dst[0].w);
        __builtin_nontemporal_store(v[4], &dst[1].x); __builtin_nontemporal_store(v[5], &dst[1].y);
        __builtin_nontemporal_store(v[6], &dst[1].z); __builtin_nontemporal_store(v[7], &dst[1].w);
    } else {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float float2v __attribute__((ext_vector_type(2)));
        uint4v q;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            q[i] = __builtin_bit_cast(unsigned, __builtin_convertvector(float2v{v[2 * i], v[2 * i + 1]}, bf16x2));
        __builtin_nontemporal_store(q, static_cast<uint4v*>(y) + g);
    }
}

}  // namespace

hipError_t launch_layernorm_apply(long long tokens, int D, const void* o, const float* mean_rstd, const float* gamma,
                                  const float* beta, void* y, bool out_f32, hipStream_t stream) {
    const int groups_per_token = D / 8;
    const long long groups = tokens * groups_per_token;
    const dim3 grid(static_cast<unsigned>((groups + 255) / 256));
    if (out_f32)
        hipLaunchKernelGGL(layernorm_apply_kernel<true>, grid, dim3(256), 0, stream, groups, groups_per_token,
                           static_cast<const uint4v*>(o), reinterpret_cast<const float2*>(mean_rstd),
                           reinterpret_cast<const float4*>(gamma), reinterpret_cast<const float4*>(beta), y);
    else
        hipLaunchKernelGGL(layernorm_apply_kernel<false>, grid, dim3(256), 0, stream, groups, groups_per_token,
                           static_cast<const uint4v*>(o), reinterpret_cast<const float2*>(mean_rstd),
                           reinterpret_cast<const float4*>(gamma), reinterpret_cast<const float4*>(beta), y);
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

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

}  // namespace

hipError_t launch_layernorm_finalize(int B, int T, int H, const float* moments, float eps, float* mean_rstd,
                                     hipStream_t stream) {
    const dim3 grid(static_cast<unsigned>((T + 63) / 64), static_cast<unsigned>(B));
    hipLaunchKernelGGL(layernorm_finalize_kernel, grid, dim3(256), 0, stream, T, H,
                       reinterpret_cast<const float2*>(moments), eps, reinterpret_cast<float2*>(mean_rstd));
    return hipGetLastError();
}

}  // namespace wkv6

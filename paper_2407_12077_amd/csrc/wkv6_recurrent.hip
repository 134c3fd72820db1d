// Token-by-token WKV6 kernel for gfx950: one wavefront per (batch, head), lane j owns
// column j of the state (64 fp32 registers), r/k/w of the current token are exchanged
// through LDS and read back as broadcasts.  Follows the recurrence one step at a time
// (Finch-C2 Time Mixing: decay map, wkv_t, read-out; plus the Finch bonus u):
//     o_t[j] = sum_i r_t[i] S[i][j]  +  (sum_i r_t[i] u[i] k_t[i]) v_t[j]
//     S[i][j] = w_t[i] S[i][j] + k_t[i] v_t[j],   w_t = exp(-exp(x_t))
// It is bound by the fp32 vector ALUs (about 3*N*N operations per token and head), which
// is why the chunked kernel exists; this one serves fp32 tensors, cross-checks, and the
// decode / short-append shapes (one or a few tokens per sequence, many sequences), where the
// work is streaming the fp32 state through once: 64 row loads of 256 contiguous bytes per
// wave, all in flight together.
// Finch-C2 form (template flag): k = kbar (1 - w), no bonus, second value u' added to o.
#include "wkv6_launch.h"

#include <hip/hip_bf16.h>

namespace wkv6 {
namespace {

template <bool kInBf16>
__device__ __forceinline__ float load_in(const void* p, long long idx) {
    if constexpr (kInBf16) {
        unsigned short bits = static_cast<const unsigned short*>(p)[idx];
        return __uint_as_float(static_cast<unsigned>(bits) << 16);
    } else {
        return static_cast<const float*>(p)[idx];
    }
}

__device__ __forceinline__ float wave_sum(float a) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) a += __shfl_xor(a, m, 64);
    return a;
}

template <bool kInBf16, bool kOutBf16, bool kC2>
__global__ __launch_bounds__(64) void recurrent_kernel(Args a) {
    constexpr int N = kHeadSize;
    const int unit = blockIdx.x;           // b * H + h
    const int b = unit / a.H;
    const int h = unit - b * a.H;
    const int j = threadIdx.x;

    __shared__ __attribute__((aligned(16))) float s_r[N];
    __shared__ __attribute__((aligned(16))) float s_k[N];
    __shared__ __attribute__((aligned(16))) float s_w[N];

    float S[N];
    if (a.state_in) {
        const float* s0 = a.state_in + static_cast<long long>(unit) * N * N;
#pragma unroll
        for (int i = 0; i < N; ++i) S[i] = __builtin_nontemporal_load(&s0[i * N + j]);   // streamed once
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) S[i] = 0.f;
    }

    const float uj = kC2 ? 0.f : a.u[h * N + j];
    const long long tok_stride = static_cast<long long>(a.H) * N;
    long long idx = static_cast<long long>(b) * a.batch_stride + static_cast<long long>(h) * N + j;

    float rj = 0.f, kj = 0.f, vj = 0.f, xj = 0.f, pj = 0.f;
    if (a.T > 0) {
        rj = load_in<kInBf16>(a.r, idx);
        kj = load_in<kInBf16>(a.k, idx);
        vj = load_in<kInBf16>(a.v, idx);
        xj = load_in<kInBf16>(a.x, idx);
        if constexpr (kC2) pj = load_in<kInBf16>(a.uprime, idx);
    }
    for (int t = 0; t < a.T; ++t) {
        const float r_cur = rj, v_cur = vj, p_cur = pj;
        const float w_cur = expf(-expf(xj));
        // Finch-C2 key factor 1 - w = -expm1(-exp(x)): no cancellation for decays close to 1
        const float k_cur = kC2 ? kj * -expm1f(-expf(xj)) : kj;
        const long long idx_cur = idx;
        idx += tok_stride;
        if (t + 1 < a.T) {                     // next token's loads overlap this token's math
            rj = load_in<kInBf16>(a.r, idx);
            kj = load_in<kInBf16>(a.k, idx);
            vj = load_in<kInBf16>(a.v, idx);
            xj = load_in<kInBf16>(a.x, idx);
            if constexpr (kC2) pj = load_in<kInBf16>(a.uprime, idx);
        }
        __syncthreads();                       // previous token's LDS reads are done
        s_r[j] = r_cur;
        s_k[j] = k_cur;
        s_w[j] = w_cur;
        float o = p_cur;                       // Finch-C2: the second value; Finch: the bonus term
        if constexpr (!kC2) o = wave_sum(r_cur * uj * k_cur) * v_cur;
        __syncthreads();

#pragma unroll
        for (int i4 = 0; i4 < N; i4 += 4) {
            const float4 r4 = *reinterpret_cast<const float4*>(&s_r[i4]);
            const float4 k4 = *reinterpret_cast<const float4*>(&s_k[i4]);
            const float4 w4 = *reinterpret_cast<const float4*>(&s_w[i4]);
            o = fmaf(r4.x, S[i4 + 0], o);
            S[i4 + 0] = fmaf(w4.x, S[i4 + 0], k4.x * v_cur);
            o = fmaf(r4.y, S[i4 + 1], o);
            S[i4 + 1] = fmaf(w4.y, S[i4 + 1], k4.y * v_cur);
            o = fmaf(r4.z, S[i4 + 2], o);
            S[i4 + 2] = fmaf(w4.z, S[i4 + 2], k4.z * v_cur);
            o = fmaf(r4.w, S[i4 + 3], o);
            S[i4 + 3] = fmaf(w4.w, S[i4 + 3], k4.w * v_cur);
        }
        if constexpr (kOutBf16)
            static_cast<unsigned short*>(a.out)[idx_cur] =
                __builtin_bit_cast(unsigned short, static_cast<__bf16>(o));
        else
            static_cast<float*>(a.out)[idx_cur] = o;
    }

    if (a.state_out) {
        float* so = a.state_out + static_cast<long long>(unit) * N * N;
#pragma unroll
        for (int i = 0; i < N; ++i) __builtin_nontemporal_store(S[i], &so[i * N + j]);
    }
}

__global__ __launch_bounds__(256) void state_passthrough_kernel(const float* in, float* out,
                                                                long long n4) {
    const long long i = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n4) {
        float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
        if (in) val = reinterpret_cast<const float4*>(in)[i];
        reinterpret_cast<float4*>(out)[i] = val;
    }
}

}  // namespace

hipError_t launch_recurrent(const Args& a, bool in_bf16, bool out_bf16, hipStream_t stream) {
    const dim3 grid(static_cast<unsigned>(a.B) * static_cast<unsigned>(a.H));
    const bool c2 = a.finch_c2;
    if (!in_bf16)
        hipLaunchKernelGGL((recurrent_kernel<false, false, false>), grid, dim3(64), 0, stream, a);
    else if (!out_bf16 && !c2)
        hipLaunchKernelGGL((recurrent_kernel<true, false, false>), grid, dim3(64), 0, stream, a);
    else if (!out_bf16 && c2)
        hipLaunchKernelGGL((recurrent_kernel<true, false, true>), grid, dim3(64), 0, stream, a);
    else if (!c2)
        hipLaunchKernelGGL((recurrent_kernel<true, true, false>), grid, dim3(64), 0, stream, a);
    else
        hipLaunchKernelGGL((recurrent_kernel<true, true, true>), grid, dim3(64), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_state_passthrough(const Args& a, hipStream_t stream) {
    if (!a.state_out || a.state_out == a.state_in) return hipSuccess;
    const long long n4 = static_cast<long long>(a.B) * a.H * kHeadSize * kHeadSize / 4;
    const unsigned blocks = static_cast<unsigned>((n4 + 255) / 256);
    hipLaunchKernelGGL(state_passthrough_kernel, dim3(blocks), dim3(256), 0, stream,
                       a.state_in, a.state_out, n4);
    return hipGetLastError();
}

}  // namespace wkv6

// Token-by-token WKV6 kernel for gfx950: one wavefront per (batch, head), lane j owns
// column j of the state (64 fp32 registers), r/k/w of the current token are exchanged
// through LDS and read back as broadcasts.  Follows the recurrence one step at a time
// (Finch-C2 Time Mixing: decay map, wkv_t, read-out; plus the Finch bonus u):
//     o_t[j] = sum_i r_t[i] S[i][j]  +  (sum_i r_t[i] u[i] k_t[i]) v_t[j]
//     S[i][j] = w_t[i] S[i][j] + k_t[i] v_t[j],   w_t = exp(-exp(x_t))
// It is bound by the fp32 vector ALUs (about 3*N*N operations per token and head), which
// is why the chunked kernel exists; this one serves the decode / short-append shapes (one or a
// few tokens per sequence, many sequences), where the work is streaming the fp32 state through
// once: 64 row loads of 256 contiguous bytes per wave, all in flight together.  Long sequences
// of the fp32 and cross-check entry points take the four-wave form further down.
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

// The same recurrence for long sequences, four wavefronts per (batch, head): wave w owns value
// columns 16w .. 16w+15, and its lane (q, c) = (lane / 16, lane % 16) owns key rows 16q .. 16q+15
// of column 16w + c (16 fp32 state registers).  Tokens are taken in blocks of 8.  The workgroup's
// 256 threads fetch a block together, two neighbouring channels of one token each (r, k, x, v),
// form w once per element and leave the fp32 vectors in LDS one block
// ahead of their use, two slots by block parity, one workgroup barrier per block; the loads of
// the block after that are in flight meanwhile, which is what hides the memory latency a
// token-by-token prefetch cannot.  A lane then reads its quarter of r, k, w as broadcasts, runs
// its 16 rows, and the four quarters of a column meet through two cross-lane moves per token,
// issued together at the end of the block.  The Finch bonus enters inside the row loop
// (o += r_i (S_ij + u_i k_i v_j)), so no sum over the whole wave is needed.  Finch form only: the
// Finch-C2 entry points that take this file's kernels are single steps and short appends.
constexpr int kWideBlock = 8;

template <bool kInBf16>
struct WidePair {                          // two neighbouring channels of one token
    float lo, hi;
    __device__ __forceinline__ void load(const void* p, long long elem) {
        if constexpr (kInBf16) {
            const unsigned w = *reinterpret_cast<const unsigned*>(static_cast<const unsigned short*>(p) + elem);
            lo = __uint_as_float(w << 16);
            hi = __uint_as_float(w & 0xffff0000u);
        } else {
            const float2 f = *reinterpret_cast<const float2*>(static_cast<const float*>(p) + elem);
            lo = f.x;
            hi = f.y;
        }
    }
};

template <bool kInBf16, bool kOutBf16>
__global__ __launch_bounds__(256) void recurrent_wide_kernel(Args a) {
    constexpr int N = kHeadSize;
    using Pair = WidePair<kInBf16>;
    const int unit = blockIdx.x;           // b * H + h
    const int b = unit / a.H;
    const int h = unit - b * a.H;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int q = lane >> 4, c = lane & 15;
    const int j = 16 * wave + c;

    // [block parity][r, k, w, v][token][channel]
    __shared__ __attribute__((aligned(16))) float s_in[2][4][kWideBlock][N];

    float S[16], uq[16];
    if (a.state_in) {
        const float* s0 = a.state_in + static_cast<long long>(unit) * N * N + (16 * q) * N + j;
#pragma unroll
        for (int i = 0; i < 16; ++i) S[i] = __builtin_nontemporal_load(&s0[i * N]);
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) S[i] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) uq[i] = a.u[h * N + 16 * q + i];

    const long long tok_stride = static_cast<long long>(a.H) * N;
    const long long base = static_cast<long long>(b) * a.batch_stride + static_cast<long long>(h) * N;
    const int st = tid >> 5;               // token of this thread inside a block when staging
    const int sc = 2 * (tid & 31);         // its two channels

    Pair raw_r, raw_k, raw_x, raw_v;
    auto fetch = [&](int t0) {             // rows past the end are not touched
        raw_r.lo = raw_r.hi = raw_k.lo = raw_k.hi = raw_x.lo = raw_x.hi = 0.f;
        raw_v.lo = raw_v.hi = 0.f;
        if (t0 + st < a.T) {
            const long long e = base + static_cast<long long>(t0 + st) * tok_stride + sc;
            raw_r.load(a.r, e);
            raw_k.load(a.k, e);
            raw_x.load(a.x, e);
            raw_v.load(a.v, e);
        }
    };
    auto stage = [&](int parity) {
        const float e0 = expf(raw_x.lo), e1 = expf(raw_x.hi);
        *reinterpret_cast<float2*>(&s_in[parity][0][st][sc]) = make_float2(raw_r.lo, raw_r.hi);
        *reinterpret_cast<float2*>(&s_in[parity][1][st][sc]) = make_float2(raw_k.lo, raw_k.hi);
        *reinterpret_cast<float2*>(&s_in[parity][2][st][sc]) = make_float2(expf(-e0), expf(-e1));
        *reinterpret_cast<float2*>(&s_in[parity][3][st][sc]) = make_float2(raw_v.lo, raw_v.hi);
    };
    // one token of this lane's 16 rows
    auto token = [&](int parity, int tt) {
        const float* rkw = &s_in[parity][0][tt][16 * q];
        const float v_cur = s_in[parity][3][tt][j];
        float o = 0.f;
#pragma unroll
        for (int i4 = 0; i4 < 16; i4 += 4) {
            const float4 r4 = *reinterpret_cast<const float4*>(rkw + i4);
            const float4 k4 = *reinterpret_cast<const float4*>(rkw + kWideBlock * N + i4);
            const float4 w4 = *reinterpret_cast<const float4*>(rkw + 2 * kWideBlock * N + i4);
            const float rr[4] = {r4.x, r4.y, r4.z, r4.w};
            const float kk[4] = {k4.x, k4.y, k4.z, k4.w};
            const float ww[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float kv = kk[e] * v_cur;
                o = fmaf(rr[e], fmaf(uq[i4 + e], kv, S[i4 + e]), o);
                S[i4 + e] = fmaf(ww[e], S[i4 + e], kv);
            }
        }
        return o;
    };

    if (a.T > 0) {
        fetch(0);
        stage(0);
        fetch(kWideBlock);
    }
    int parity = 0;
    for (int t0 = 0; t0 < a.T; t0 += kWideBlock, parity ^= 1) {
        __syncthreads();                       // this block is staged; the other slot has been read
        if (t0 + kWideBlock < a.T) {           // the next block into the other slot, the one after on its way
            stage(parity ^ 1);
            fetch(t0 + 2 * kWideBlock);
        }
        const int nb = a.T - t0 < kWideBlock ? a.T - t0 : kWideBlock;
        float part[kWideBlock];
        if (nb == kWideBlock) {                // straight line: the reads of one token overlap the rows of another
#pragma unroll
            for (int tt = 0; tt < kWideBlock; ++tt) part[tt] = token(parity, tt);
        } else {
#pragma unroll
            for (int tt = 0; tt < kWideBlock; ++tt) {
                part[tt] = 0.f;
                if (tt < nb) part[tt] = token(parity, tt);
            }
        }
        // the four key quarters of every column meet; quarter q then stores tokens 2q and 2q+1
#pragma unroll
        for (int tt = 0; tt < kWideBlock; ++tt) part[tt] += __shfl_xor(part[tt], 16, 64);
#pragma unroll
        for (int tt = 0; tt < kWideBlock; ++tt) part[tt] += __shfl_xor(part[tt], 32, 64);
#pragma unroll
        for (int tt = 0; tt < kWideBlock; ++tt) {
            if ((tt >> 1) == q && tt < nb) {
                const float o = part[tt];
                const long long e = base + static_cast<long long>(t0 + tt) * tok_stride + j;
                if constexpr (kOutBf16)
                    static_cast<unsigned short*>(a.out)[e] = __builtin_bit_cast(unsigned short, static_cast<__bf16>(o));
                else
                    static_cast<float*>(a.out)[e] = o;
            }
        }
    }

    if (a.state_out) {
        float* so = a.state_out + static_cast<long long>(unit) * N * N + (16 * q) * N + j;
#pragma unroll
        for (int i = 0; i < 16; ++i) __builtin_nontemporal_store(S[i], &so[i * N]);
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

// Sequences of at least this many tokens take the four-wave form; shorter ones (decode, short
// appends: the work is streaming the state once) the one-wave form with its 256-byte state rows.
constexpr int kWideMinTokens = 16;

hipError_t launch_recurrent(const Args& a, bool in_bf16, bool out_bf16, hipStream_t stream) {
    const dim3 grid(static_cast<unsigned>(a.B) * static_cast<unsigned>(a.H));
    const bool c2 = a.finch_c2;
    if (a.T >= kWideMinTokens && !c2) {
        if (!in_bf16)
            hipLaunchKernelGGL((recurrent_wide_kernel<false, false>), grid, dim3(256), 0, stream, a);
        else if (!out_bf16)
            hipLaunchKernelGGL((recurrent_wide_kernel<true, false>), grid, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((recurrent_wide_kernel<true, true>), grid, dim3(256), 0, stream, a);
        return hipGetLastError();
    }
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

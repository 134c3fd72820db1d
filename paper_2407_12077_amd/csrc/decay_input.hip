// The operators in front of the fused decay path, for gfx950 (Finch-C2 Time Mixing: lerp, lora and
// ddlerp operator equations and d_t = lora_omega(ddlerp_d(x_t, x_{t-1}))): from the layer input x to
//
//     z_t = x_t + (x_{t-1} - x_t) * (lambda_d + tanh((x_t + (x_{t-1} - x_t) * mu_x) A_d) B_d)
//     y_t = tanh(z_t A_omega)                                         64 values per token
//
// which wkv6_finch_c2_prefill_lora_bf16 turns into decay logits per head.  Per token this is a chain
// of three skinny matrix products (D -> 32, 32 -> D, D -> 64) bound by the one HBM read of x.
//
// One workgroup owns 128 consecutive tokens of one sequence and walks the D axis twice in steps of 128
// channels (the second walk needs tanh(q A_d) of the whole first one; its reads of x are served by
// L2 / the last-level cache).  Sixteen waves in two roles, one barrier per step; the steps are this
// heavy (and the workgroup this large) because a step has to last long enough for loads issued two
// steps ahead to arrive: with 64 tokens and 64 channels per step the same pipeline ran at the memory
// latency, not the memory rate (102 us against 180 us for a version without a pipeline at all).
//   waves 8..15 LOADERS: fetch, two steps ahead, the step's x rows (128 tokens and the row before the
//               first one: 256-byte pieces, 16 lanes each) and its weight slices with 16-byte loads,
//               convert the weights to fp16 and park everything in one of two LDS stages.  Rows past
//               the end of the sequence go through shrunk raw buffer descriptors and read as zero.
//   waves 0..7  WORKERS: wave w owns tokens 16w .. 16w+15 through the whole chain, in registers:
//     walk 1    q = x_t + (x_{t-1} - x_t) mu_x in fp32, rounded to fp16 (11 significant bits: bf16
//               operands would put the result outside the 2e-3 bar), times A_d
//               (v_mfma_f32_16x16x32_f16, weights as the A operand so that a lane ends up with its
//               own token's 8 inner-rank sums); tanh; that is already the B operand p of walk 2.
//     walk 2    per block of 16 channels: (lambda_d + B_d^T p) by one MFMA whose result layout (a
//               lane holds four consecutive channels of its token) is the operand layout of the
//               16x16x16 MFMA, so z = x_t + (x_{t-1} - x_t) * mix is formed in registers and fed
//               straight into the product with A_omega; mix and z never touch LDS or HBM.
//               The y accumulators (a lane: four consecutive outputs of its token per 16-column
//               block) get their tanh and leave through the wave's own piece of LDS as whole rows
//               (1 % faster than 8-byte stores straight from the accumulator layout).
// One workgroup per compute unit (134 KB of LDS, 128 registers per thread).
//
// Weight layouts are the ones an MFMA operand can be read from with the contraction index
// contiguous: A_d and A_omega column by column ([r][D]), B_d column by column ([D][r]).
#include "wkv6_launch.h"

namespace wkv6 {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));

constexpr int kTokens = 128;         // tokens per workgroup
constexpr int kStepCh = 128;         // channels per step
constexpr int kInnerRank = 32;       // columns of A_d
constexpr int kOuterRank = 64;       // columns of A_omega
constexpr int kWorkerWaves = kTokens / 16;
constexpr int kLoaderThreads = 512;
constexpr int kDiThreads = 64 * kWorkerWaves + kLoaderThreads;      // 8 worker waves + 8 loader waves
constexpr int kXRowB = 288;          // LDS row stride of 128-channel rows (256 B + 32 pad: full-rate 16-byte reads)
constexpr int kBdRow = 96;           // LDS row stride of the B_d slice (32 ranks = 64 B + 32 pad)
// one LDS stage (bytes): x rows 0..127 = tokens, row 128 = the row before the first token
constexpr int kOffX = 0;
constexpr int kOffVec = kOffX + (kTokens + 1) * kXRowB; // mu_x (walk 1) or lambda_d (walk 2) slice: 128 fp32
constexpr int kOffW1 = kOffVec + kStepCh * 4;           // walk 1: A_d slice [32 columns][128 channels] fp16
constexpr int kOffBd = kOffVec + kStepCh * 4;           // walk 2: B_d slice [128 channels][32 ranks] fp16
constexpr int kOffWo = kOffBd + kStepCh * kBdRow;       // walk 2: A_omega slice [64 columns][128 channels] fp16
constexpr int kStageBytes = (kOffWo + kOuterRank * kXRowB + 255) / 256 * 256;
constexpr int kDiLds = 2 * kStageBytes;
static_assert(kOffW1 + kInnerRank * kXRowB <= kStageBytes && kDiLds <= 160 * 1024, "stage layout");

struct DiArgs {
    int B, T, D;
    int tiles_per_seq;
    const char* x;          // [B][T][D] bf16
    const char* x_prev;     // [B][D] bf16 or nullptr
    const char* mu_x;       // [D] fp32
    const char* lambda_d;   // [D] fp32
    const char* a_d;        // [32][D] bf16
    const char* b_d;        // [D][32] bf16
    const char* a_omega;    // [64][D] bf16
    void* y;                // [B][T][64] bf16 or fp32
};

__device__ __forceinline__ float lo_f(unsigned bits) { return __uint_as_float(bits << 16); }
__device__ __forceinline__ float hi_f(unsigned bits) { return __uint_as_float(bits & 0xffff0000u); }

__device__ __forceinline__ unsigned pack_h2f(float a, float b) {
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    half2v p;
    p.x = static_cast<_Float16>(a);
    p.y = static_cast<_Float16>(b);
    return __builtin_bit_cast(unsigned, p);
}
// eight bf16 (four dwords) as four fp16 pairs (exact for magnitudes inside the fp16 range)
__device__ __forceinline__ uint4v bf16x8_to_f16x8(uint4v q) {
    uint4v h;
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = pack_h2f(lo_f(q[i]), hi_f(q[i]));
    return h;
}

// tanh through one exponential and one reciprocal: 1 - 2 / (exp(2a) + 1); exact limits at +-inf
__device__ __forceinline__ float fast_tanh(float a) {
    const float e = __builtin_amdgcn_exp2f(a * 2.8853900817779268f);     // exp(2a)
    return 1.f - 2.f * __builtin_amdgcn_rcpf(e + 1.f);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const char* base, long long bytes) {
    if (bytes < 0) bytes = 0;
    if (bytes > 0x7fffffffLL) bytes = 0x7fffffffLL;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, static_cast<int>(bytes), 0x00020000);
}

struct StepRegs {          // a loader thread's share of one step
    uint4v x0, x1, x2, x3, xp;   // x rows xr + 32 i; the row before the first token (threads 0..15)
    uint4v w0, w1, w2;     // walk 1: A_d piece (w0); walk 2: B_d piece (w0), two A_omega pieces (w1, w2)
    uint4v vec;            // mu_x / lambda_d piece (threads 0..31)
};

// ------------------------------------------------------------------------------------------
// loader waves (512 threads)
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void di_loader(const DiArgs& a, char* lds, int lt, int b, int t0, int ntok, int nsteps,
                                          int first) {
    const long long row_bytes = static_cast<long long>(a.D) * 2;
    const char* tile = a.x + (static_cast<long long>(b) * a.T + t0) * row_bytes;
    const char* pred = t0 > 0 ? tile - row_bytes : (a.x_prev ? a.x_prev + static_cast<long long>(b) * row_bytes : nullptr);
    const long long tile_bytes = static_cast<long long>(ntok) * row_bytes;
    const int nchunks = a.D / kStepCh;
    const int xr = lt >> 4, xg = lt & 15;                   // 16 lanes per 256-byte row piece, 32 rows per pass
    const int x_voff0 = static_cast<int>(xr * row_bytes + 16 * xg);
    const int x_vstep = static_cast<int>(32 * row_bytes);
    const long long wcol_bytes = row_bytes;                 // a_d / a_omega: one column = D bf16

    auto fetch = [&](StepRegs& s, int step) {
        const bool live = step < nsteps;                                   // uniform
        // Both walks are sums over the channel blocks, so their order is free: walk 1 goes up from a
        // block that differs between workgroups (workgroups marching through the channels in step
        // would all ask the same memory channels for their row pieces, which are D*2 bytes apart),
        // walk 2 comes back down, so that it starts with the blocks most recently brought into L2.
        const bool walk2 = step >= nchunks;
        int chunk = walk2 ? first + 2 * nchunks - 1 - step : first + step;
        if (chunk >= nchunks) chunk -= nchunks;
        if (!live) chunk = 0;                                              // nothing is fetched: keep the bases in range
        const long long coff = static_cast<long long>(chunk) * (kStepCh * 2);   // byte offset of the chunk in a row
        const __amdgpu_buffer_rsrc_t rx = rsrc_of(tile + coff, live ? tile_bytes - coff : 0);
        s.x0 = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rx, x_voff0, 0, 0));
        s.x1 = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rx, x_voff0 + x_vstep, 0, 0));
        s.x2 = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rx, x_voff0 + 2 * x_vstep, 0, 0));
        s.x3 = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rx, x_voff0 + 3 * x_vstep, 0, 0));
        const __amdgpu_buffer_rsrc_t rp = rsrc_of(pred ? pred + coff : a.x, (live && pred) ? kStepCh * 2 : 0);
        s.xp = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rp, lt < 16 ? 16 * lt : 0x7ffffff0, 0, 0));
        const char* vec = walk2 ? a.lambda_d : a.mu_x;
        const __amdgpu_buffer_rsrc_t rv = rsrc_of(vec + chunk * (kStepCh * 4), live ? kStepCh * 4 : 0);
        s.vec = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rv, lt < 32 ? 16 * lt : 0x7ffffff0, 0, 0));
        // walk 1: A_d slice (column lt>>4, 16-byte piece lt&15 of its 128 channels); walk 2: B_d slice (channel
        // lt>>2 of the chunk, 16-byte piece lt&3 of its 32 ranks) and A_omega slice (columns lt>>4 and
        // 32 + (lt>>4)).  Every load is issued in both walks, through an empty descriptor where it has
        // nothing to fetch, so that the step's registers are plain values on every path.
        const __amdgpu_buffer_rsrc_t rw0 =
            walk2 ? rsrc_of(a.b_d + static_cast<long long>(chunk) * (kStepCh * kInnerRank * 2), live ? kStepCh * kInnerRank * 2 : 0)
                  : rsrc_of(a.a_d + coff, live ? kInnerRank * wcol_bytes - coff : 0);
        const int w0_voff = walk2 ? (lt >> 2) * (kInnerRank * 2) + 16 * (lt & 3) : static_cast<int>(xr * wcol_bytes + 16 * xg);
        s.w0 = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rw0, w0_voff, 0, 0));
        const __amdgpu_buffer_rsrc_t ro = rsrc_of(a.a_omega + coff, (live && walk2) ? kOuterRank * wcol_bytes - coff : 0);
        s.w1 = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(ro, static_cast<int>(xr * wcol_bytes + 16 * xg), 0, 0));
        s.w2 = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(ro, static_cast<int>((xr + 32) * wcol_bytes + 16 * xg), 0, 0));
    };
    auto park = [&](const StepRegs& s, int step) {
        char* st = lds + (step & 1) * kStageBytes;
        const bool walk2 = step >= nchunks;
        char* xdst = st + kOffX + xr * kXRowB + 16 * xg;
        *reinterpret_cast<uint4v*>(xdst) = s.x0;
        *reinterpret_cast<uint4v*>(xdst + 32 * kXRowB) = s.x1;
        *reinterpret_cast<uint4v*>(xdst + 64 * kXRowB) = s.x2;
        *reinterpret_cast<uint4v*>(xdst + 96 * kXRowB) = s.x3;
        if (lt < 16) *reinterpret_cast<uint4v*>(st + kOffX + kTokens * kXRowB + 16 * lt) = s.xp;
        if (lt < 32) *reinterpret_cast<uint4v*>(st + kOffVec + 16 * lt) = s.vec;
        if (!walk2) {
            *reinterpret_cast<uint4v*>(st + kOffW1 + xr * kXRowB + 16 * xg) = bf16x8_to_f16x8(s.w0);
        } else {
            // The inner ranks of a B_d row are stored in the order in which walk 1 leaves them in a
            // worker lane: 16-byte granule g4 holds ranks 4*g4 .. 4*g4+3 and 16 + 4*g4 .. 16 + 4*g4+3.
            // This thread has ranks 8g .. 8g+7 (g = lt & 3): two 8-byte halves of two granules.
            const uint4v h = bf16x8_to_f16x8(s.w0);
            const int g = lt & 3;
            char* rowp = st + kOffBd + (lt >> 2) * kBdRow + 8 * (g >> 1);
            *reinterpret_cast<uint2v*>(rowp + 16 * (2 * (g & 1))) = uint2v{h[0], h[1]};
            *reinterpret_cast<uint2v*>(rowp + 16 * (2 * (g & 1) + 1)) = uint2v{h[2], h[3]};
            *reinterpret_cast<uint4v*>(st + kOffWo + xr * kXRowB + 16 * xg) = bf16x8_to_f16x8(s.w1);
            *reinterpret_cast<uint4v*>(st + kOffWo + (xr + 32) * kXRowB + 16 * xg) = bf16x8_to_f16x8(s.w2);
        }
    };

    // nsteps is even (two walks of D / 128 steps); same barrier sequence as the workers: one before the
    // first step and one after every step
    StepRegs s0, s1;
    fetch(s0, 0);
    fetch(s1, 1);
    park(s0, 0);
    fetch(s0, 2);
    __syncthreads();                                   // stage of step 0 is in LDS
#pragma clang loop unroll(disable)
    for (int step = 0; step < nsteps; step += 2) {
        park(s1, step + 1);                            // while the workers are on `step`
        fetch(s1, step + 3);
        __syncthreads();
        if (step + 2 < nsteps) park(s0, step + 2);
        fetch(s0, step + 4);
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// worker waves (512 threads): wave w owns tokens 16w .. 16w + 15
// ------------------------------------------------------------------------------------------
template <bool kOutF32>
__device__ __forceinline__ void di_worker(const DiArgs& a, char* lds, int lane, int w, int b, int t0, int ntok,
                                          int nsteps) {
    const int l16 = lane & 15;
    const int g4 = lane >> 4;
    const int nchunks = a.D / kStepCh;
    const int trow = 16 * w + l16;                               // this lane's token row in the stage
    const int prow = trow == 0 ? kTokens : trow - 1;             // and its previous token's
    const int xt_off = kOffX + trow * kXRowB, xp_off = kOffX + prow * kXRowB;

    float4v pacc[2] = {float4v{0.f, 0.f, 0.f, 0.f}, float4v{0.f, 0.f, 0.f, 0.f}};
    float4v yacc[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) yacc[nb] = float4v{0.f, 0.f, 0.f, 0.f};
    half8 pt;                                                    // tanh(q A_d) of this lane's token, walk 1's rank order

    auto walk1 = [&](const char* st) {
#pragma unroll
        for (int kb = 0; kb < kStepCh / 32; ++kb) {
            const int col = 64 * kb + 16 * g4;                   // byte column of this lane's 8 channels
            const uint4v xt = *reinterpret_cast<const uint4v*>(st + xt_off + col);
            const uint4v xp = *reinterpret_cast<const uint4v*>(st + xp_off + col);
            const float4 m0 = *reinterpret_cast<const float4*>(st + kOffVec + 2 * col);
            const float4 m1 = *reinterpret_cast<const float4*>(st + kOffVec + 2 * col + 16);
            const float mu[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
            uint4v q;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float c0 = lo_f(xt[i]), c1 = hi_f(xt[i]);
                q[i] = pack_h2f(__builtin_fmaf(lo_f(xp[i]) - c0, mu[2 * i], c0),
                                __builtin_fmaf(hi_f(xp[i]) - c1, mu[2 * i + 1], c1));
            }
            const half8 qh = __builtin_bit_cast(half8, q);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                // A operand: A_d columns 16nb + l16 (rows of the slice), B operand: q of token l16
                const half8 wgt = *reinterpret_cast<const half8*>(st + kOffW1 + (16 * nb + l16) * kXRowB + col);
                pacc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wgt, qh, pacc[nb], 0, 0, 0);
            }
        }
    };
    auto walk2 = [&](const char* st) {
        // Two 16-channel blocks at a time, over 32 consecutive channels.  Which channel sits in which row
        // of the B_d^T operand is free as long as z and A_omega agree, so block `half` of a pair takes the
        // channels 8*(m>>2) + 4*half + (m&3), m = 0..15: lane group g4 then owns the eight consecutive
        // channels 8*g4 .. 8*g4+7 of the pair, and x_t, x_{t-1} and A_omega are one 16-byte read each
        // (the worker's LDS reads, not its arithmetic, bound this walk).
#pragma unroll
        for (int pair = 0; pair < kStepCh / 32; ++pair) {
            const int ch = 32 * pair + 8 * g4;                   // this lane's eight channels of the step
            const int row0 = 32 * pair + 8 * (l16 >> 2) + (l16 & 3);     // B_d^T operand row of this lane, first block
            const uint4v xt = *reinterpret_cast<const uint4v*>(st + xt_off + ch * 2);
            const uint4v xp = *reinterpret_cast<const uint4v*>(st + xp_off + ch * 2);
            half8 wo[4];
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
                wo[nb] = *reinterpret_cast<const half8*>(st + kOffWo + (16 * nb + l16) * kXRowB + ch * 2);
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const half8 bd = *reinterpret_cast<const half8*>(st + kOffBd + (row0 + 4 * half) * kBdRow + 16 * g4);
                const float4 lam = *reinterpret_cast<const float4*>(st + kOffVec + (ch + 4 * half) * 4);
                // mix[e] = lambda_d + sum_k B_d[k][channel ch + 4*half + e] p[token][k], for this lane's token
                const float4v mix = __builtin_amdgcn_mfma_f32_16x16x32_f16(bd, pt, float4v{lam.x, lam.y, lam.z, lam.w}, 0, 0, 0);
                uint2v z;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const unsigned t = xt[2 * half + i], q = xp[2 * half + i];
                    const float c0 = lo_f(t), c1 = hi_f(t);
                    z[i] = pack_h2f(__builtin_fmaf(lo_f(q) - c0, mix[2 * i], c0), __builtin_fmaf(hi_f(q) - c1, mix[2 * i + 1], c1));
                }
                const half4 zh = __builtin_bit_cast(half4, z);
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    // A operand: A_omega columns 16nb + l16, this block's four channels; B operand: z of token l16
                    const half4 w4 = half ? __builtin_shufflevector(wo[nb], wo[nb], 4, 5, 6, 7)
                                          : __builtin_shufflevector(wo[nb], wo[nb], 0, 1, 2, 3);
                    yacc[nb] = __builtin_amdgcn_mfma_f32_16x16x16f16(w4, zh, yacc[nb], 0, 0, 0);
                }
            }
        }
    };
    auto step_of = [&](int step) {
        const char* st = lds + (step & 1) * kStageBytes;
        if (step < nchunks) {
            walk1(st);
            if (step == nchunks - 1) {
                // pacc[nb][e] = sum for rank 16nb + 4g4 + e of this lane's token: the order B_d was parked in
                uint4v p;
                p[0] = pack_h2f(fast_tanh(pacc[0][0]), fast_tanh(pacc[0][1]));
                p[1] = pack_h2f(fast_tanh(pacc[0][2]), fast_tanh(pacc[0][3]));
                p[2] = pack_h2f(fast_tanh(pacc[1][0]), fast_tanh(pacc[1][1]));
                p[3] = pack_h2f(fast_tanh(pacc[1][2]), fast_tanh(pacc[1][3]));
                pt = __builtin_bit_cast(half8, p);
            }
        } else {
            walk2(st);
        }
    };

    __syncthreads();                                   // stage of step 0 is in LDS
#pragma clang loop unroll(disable)
    for (int step = 0; step < nsteps; step += 2) {
        step_of(step);
        __syncthreads();
        step_of(step + 1);
        __syncthreads();
    }

    // yacc[nb][e] = pre-activation of output 16nb + 4g4 + e of token trow.  The wave's 16 rows go
    // through its own piece of LDS (free after the last barrier; this wave alone touches it), so that
    // every store instruction writes whole rows: 8 (bf16) or 16 (fp32) lanes of 16 bytes per row.
    constexpr int kYRow = kOuterRank * 4 + 16;                   // fp32 row + pad
    char* mine = lds + w * 16 * kYRow;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
        *reinterpret_cast<float4*>(mine + l16 * kYRow + (16 * nb + 4 * g4) * 4) =
            make_float4(fast_tanh(yacc[nb][0]), fast_tanh(yacc[nb][1]), fast_tanh(yacc[nb][2]), fast_tanh(yacc[nb][3]));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const long long m0 = static_cast<long long>(b) * a.T + t0 + 16 * w;   // the wave's first token
    if constexpr (kOutF32) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int row = 4 * p + (lane >> 4), c4 = 4 * (lane & 15);
            if (16 * w + row < ntok)
                *reinterpret_cast<float4*>(static_cast<float*>(a.y) + (m0 + row) * kOuterRank + c4) =
                    *reinterpret_cast<const float4*>(mine + row * kYRow + c4 * 4);
        }
    } else {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int row = 8 * p + (lane >> 3), c8 = 8 * (lane & 7);
            if (16 * w + row < ntok) {
                typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                typedef float float2v __attribute__((ext_vector_type(2)));
                const float4 lo = *reinterpret_cast<const float4*>(mine + row * kYRow + c8 * 4);
                const float4 hi = *reinterpret_cast<const float4*>(mine + row * kYRow + c8 * 4 + 16);
                const uint4v q = {__builtin_bit_cast(unsigned, __builtin_convertvector(float2v{lo.x, lo.y}, bf16x2)),
                                  __builtin_bit_cast(unsigned, __builtin_convertvector(float2v{lo.z, lo.w}, bf16x2)),
                                  __builtin_bit_cast(unsigned, __builtin_convertvector(float2v{hi.x, hi.y}, bf16x2)),
                                  __builtin_bit_cast(unsigned, __builtin_convertvector(float2v{hi.z, hi.w}, bf16x2))};
                *reinterpret_cast<uint4v*>(static_cast<unsigned short*>(a.y) + (m0 + row) * kOuterRank + c8) = q;
            }
        }
    }
}

template <bool kOutF32>
__global__ __launch_bounds__(kDiThreads) void decay_input_kernel(DiArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = blockIdx.x / a.tiles_per_seq;
    const int t0 = (blockIdx.x - b * a.tiles_per_seq) * kTokens;
    const int left = a.T - t0;
    const int ntok = left < kTokens ? left : kTokens;
    const int nsteps = 2 * (a.D / kStepCh);
    // both roles pass 1 + nsteps barriers
    if (wave >= kWorkerWaves) {
        __builtin_amdgcn_s_setprio(2);
        di_loader(a, lds, tid - 64 * kWorkerWaves, b, t0, ntok, nsteps, static_cast<int>((blockIdx.x * 3u) % (a.D / kStepCh)));
    } else {
        __builtin_amdgcn_s_setprio(1);
        di_worker<kOutF32>(a, lds, tid & 63, wave, b, t0, ntok, nsteps);
    }
}

}  // namespace

hipError_t launch_decay_input(int B, int T, int D, const void* x, const void* x_prev, const float* mu_x,
                              const float* lambda_d, const void* a_d, const void* b_d, const void* a_omega, void* y,
                              bool out_f32, hipStream_t stream) {
    DiArgs a;
    a.B = B;
    a.T = T;
    a.D = D;
    a.tiles_per_seq = (T + kTokens - 1) / kTokens;
    a.x = static_cast<const char*>(x);
    a.x_prev = static_cast<const char*>(x_prev);
    a.mu_x = reinterpret_cast<const char*>(mu_x);
    a.lambda_d = reinterpret_cast<const char*>(lambda_d);
    a.a_d = static_cast<const char*>(a_d);
    a.b_d = static_cast<const char*>(b_d);
    a.a_omega = static_cast<const char*>(a_omega);
    a.y = y;
    const dim3 grid(static_cast<unsigned>(static_cast<long long>(B) * a.tiles_per_seq));
    struct TagF32 {};
    struct TagBf16 {};
    hipError_t err;
    if (out_f32) {
        err = set_lds_limit_once<TagF32>(&decay_input_kernel<true>, kDiLds);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(decay_input_kernel<true>, grid, dim3(kDiThreads), kDiLds, stream, a);
    } else {
        err = set_lds_limit_once<TagBf16>(&decay_input_kernel<false>, kDiLds);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(decay_input_kernel<false>, grid, dim3(kDiThreads), kDiLds, stream, a);
    }
    return hipGetLastError();
}

}  // namespace wkv6

// GOLD key compression for gfx950 (MI355X): c = x W^KD, a skinny bf16 GEMM (GOLD Key
// Compression: every token's hidden state of D channels times the D x D/16 matrix W^KD gives its
// compressed key-cache entry).  M tokens x D channels are streamed from HBM exactly once; W^KD
// (D x C, C = D/16, at most a few hundred KB) stays in the L2 of every XCD.  The kernel is bound
// by the HBM read of x; all arithmetic is on the matrix cores (v_mfma_f32_16x16x32_bf16, fp32
// accumulation, bf16 products are exact in fp32).
//
// One workgroup owns 128 tokens x 128 output columns (fewer in the last column tile when D/16 is
// not a multiple of 128) and walks the D axis in steps of 64 channels (cyclically, from a start that
// differs between workgroups).  Its eight waves split into two roles that meet at one barrier per step:
//   waves 4..7  LOADERS: fetch the x tile (128 x 64: full 128-byte row pieces, 8 lanes each) and
//               the W tile (64 x 128, an L2 hit) of a step two steps ahead into registers with
//               16-byte loads, and park the tiles of the next step in one of two LDS buffers.
//               Rows past M and steps past D go through shrunk raw buffer descriptors and read
//               as zero without touching memory, so no load is predicated and the wait counters
//               stay exact.
//   waves 0..3  MFMA waves: each owns a 64 x 64 block of the result in 64 accumulator registers;
//               per step 8 row reads of x (row stride 160 B: full-rate 16-byte LDS reads), 16
//               transposing reads of W (its contraction index is the tile's row) and 32 MFMAs.
//               They issue no global loads, so nothing but LDS latency sits between their MFMAs.
// Registers and LDS are sized so that two workgroups share a compute unit: the waits, prologue
// and epilogue of one overlap the steady state of the other.
#include "wkv6_launch.h"

namespace wkv6 {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

constexpr int kBM = 128;            // tokens per workgroup
constexpr int kBN = 128;            // output columns per workgroup
constexpr int kBK = 64;             // channels per step
constexpr int kXRow = 160;          // LDS row stride of the x tile (64 bf16 + 32 B pad)
constexpr int kWRow = 288;          // LDS row stride of the W tile (128 bf16 + 32 B pad)
constexpr int kXTile = kBM * kXRow; // 20480
constexpr int kWTile = kBK * kWRow; // 18432
constexpr int kStage = kXTile + kWTile;
constexpr int kCRow = kBN * 4 + 16; // staging row of the fp32 result tile
static_assert(2 * kStage >= kBM * kCRow, "result staging reuses the operand buffers");
constexpr int kKcLds = 2 * kStage;
constexpr int kKcThreads = 512;     // 4 MFMA waves + 4 loader waves

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const void* base, long long bytes) {
    if (bytes < 0) bytes = 0;
    if (bytes > 0x7fffffffLL) bytes = 0x7fffffffLL;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, static_cast<int>(bytes), 0x00020000);
}

__device__ __forceinline__ bf16x8 lds_read_b8(const char* lds, int off) {
    return *reinterpret_cast<const bf16x8*>(lds + off);
}

// 8 consecutive rows (contraction index) of one column of a row-major 16-bit tile, as an MFMA
// operand: two transposing reads of 4 rows each.  Within a group of 16 lanes, lane i passes the
// address of the 4 entries M[i>>2][4(i&3)..+3] of a 4 x 16 block and receives M[0..3][i].
__device__ __forceinline__ bf16x8 lds_read_tr8(const char* lds, int off) {
    typedef short4v __attribute__((address_space(3))) * lds_s4_ptr;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(lds + off));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(lds + off + 4 * kWRow));
    typedef short short8v __attribute__((ext_vector_type(8)));
    const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

struct KcArgs {
    long long M;
    int D, C;
    const void* x;
    const void* w;
    void* c;
};

struct StepRegs {          // a loader thread's share of one step: 4 x 16 bytes of x and of W
    uint4v x[4], w[4];
};

// ------------------------------------------------------------------------------------------
// loader waves (256 threads): tiles of step s+2 into registers, tiles of step s+1 into LDS
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void kc_loader(const KcArgs& a, char* lds, int lt, long long m0, int n0, int rows,
                                          int nsteps, int first) {
    const long long x_row_bytes = static_cast<long long>(a.D) * 2;
    const char* x_base = static_cast<const char*>(a.x) + m0 * x_row_bytes;
    const long long x_bytes = rows * x_row_bytes;
    const long long w_row_bytes = static_cast<long long>(a.C) * 2;
    const char* w_base = static_cast<const char*>(a.w);
    const long long w_bytes = static_cast<long long>(a.D) * w_row_bytes;

    // x tile: 8 lanes per 128-byte row piece, 32 rows per pass; W tile: 16 lanes per 256-byte row
    // piece, 16 rows per pass
    const int xr = lt >> 3, xg = lt & 7;
    const int wr = lt >> 4, wg = lt & 15;
    int x_voff[4], w_voff[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        x_voff[p] = static_cast<int>((xr + 32 * p) * x_row_bytes + 16 * xg);
        // columns past C (the last column tile may be partial): an offset no descriptor covers
        w_voff[p] = n0 + 8 * wg < a.C ? static_cast<int>((wr + 16 * p) * w_row_bytes + n0 * 2 + 16 * wg) : 0x7ffffff0;
    }
    const int x_lds = xr * kXRow + 16 * xg;
    const int w_lds = kXTile + wr * kWRow + 16 * wg;

    auto fetch = [&](StepRegs& s, int step) {
        const bool live = step < nsteps;                                          // uniform
        int ks = step + first;                                                    // this step's channel block
        if (ks >= nsteps) ks -= nsteps;
        const long long xs = static_cast<long long>(ks) * kBK * 2;                // byte offset along a row of x
        const long long ws = static_cast<long long>(ks) * kBK * w_row_bytes;     // first W row of the step
        const __amdgpu_buffer_rsrc_t rx = rsrc_of(x_base + (live ? xs : 0), live ? x_bytes - xs : 0);
        const __amdgpu_buffer_rsrc_t rw = rsrc_of(w_base + (live ? ws : 0), live ? w_bytes - ws : 0);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            s.w[p] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rw, w_voff[p], 0, 0));
            s.x[p] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rx, x_voff[p], 0, 0));
        }
    };
    auto park = [&](const StepRegs& s, int buf) {
        char* b = lds + buf * kStage;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            *reinterpret_cast<uint4v*>(b + x_lds + 32 * p * kXRow) = s.x[p];
            *reinterpret_cast<uint4v*>(b + w_lds + 16 * p * kWRow) = s.w[p];
        }
    };

    // D / 64 steps, an even number; the tiles of two steps in flight per workgroup, and two
    // workgroups share a compute unit, so one's waits overlap the other's work
    StepRegs s0, s1;
    fetch(s0, 0);
    fetch(s1, 1);
    park(s0, 0);
    fetch(s0, 2);
    __syncthreads();                                   // tiles of step 0 are in LDS
#pragma clang loop unroll(disable)
    for (int step = 0; step < nsteps; step += 2) {
        park(s1, 1);                                   // step+1, while the MFMA waves work on step
        fetch(s1, step + 3);
        __syncthreads();
        park(s0, 0);
        fetch(s0, step + 4);
        __syncthreads();
    }
    __syncthreads();                                   // the result tile is staged in LDS
}

// ------------------------------------------------------------------------------------------
// MFMA waves (256 threads)
// ------------------------------------------------------------------------------------------
template <bool kOutF32>
__device__ __forceinline__ void kc_worker(const KcArgs& a, char* lds, int tid, int wave, long long m0, int n0,
                                          int rows, int nsteps) {
    const int lane = tid & 63;
    const int l16 = lane & 15;
    const int g4 = lane >> 4;
    // wave (wr, wc) owns rows 64 wr .. +63 and columns 64 wc .. +63: 4 x 4 blocks of 16 x 16
    const int wr2 = wave >> 1, wc2 = wave & 1;
    float4v acc[4][4];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) acc[rb][nb] = float4v{0.f, 0.f, 0.f, 0.f};

    const int a_lane = (64 * wr2 + l16) * kXRow + 16 * g4;                                      // + 16*kXRow*rb + 64*kb
    const int b_lane = kXTile + (8 * g4 + (l16 >> 2)) * kWRow + 8 * (l16 & 3) + 128 * wc2;     // + 32*kWRow*kb + 32*nb
    auto compute = [&](int buf) {
        const char* b = lds + buf * kStage;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            bf16x8 av[4], wt[4];
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) av[rb] = lds_read_b8(b, a_lane + 16 * kXRow * rb + 64 * kb);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) wt[nb] = lds_read_tr8(b, b_lane + 32 * kWRow * kb + 32 * nb);
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
                    acc[rb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[rb], wt[nb], acc[rb][nb], 0, 0, 0);
        }
    };

    __syncthreads();                                   // tiles of step 0 are in LDS
#pragma clang loop unroll(disable)
    for (int step = 0; step < nsteps; step += 2) {
        compute(0);
        __syncthreads();
        compute(1);
        __syncthreads();
    }

    // result tile through LDS (fp32, row stride kCRow), then full rows to HBM
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                *reinterpret_cast<float*>(lds + (64 * wr2 + 16 * rb + 4 * g4 + e) * kCRow +
                                          (64 * wc2 + 16 * nb + l16) * 4) = acc[rb][nb][e];
    __syncthreads();
    // 8 lanes per row, 16 columns each; 32 rows per pass
    const int cr = tid >> 3, cg = tid & 7;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int row = cr + 32 * p;
        if (row < rows && n0 + 16 * cg < a.C) {
            const float4* src = reinterpret_cast<const float4*>(lds + row * kCRow + cg * 64);
            const float4 q0 = src[0], q1 = src[1], q2 = src[2], q3 = src[3];
            const long long e = (m0 + row) * a.C + n0 + 16 * cg;
            if constexpr (kOutF32) {
                float4* dst = reinterpret_cast<float4*>(static_cast<float*>(a.c) + e);
                dst[0] = q0; dst[1] = q1; dst[2] = q2; dst[3] = q3;
            } else {
                auto pk = [](float lo, float hi) {
                    return static_cast<unsigned>(__builtin_bit_cast(unsigned short, static_cast<__bf16>(lo))) |
                           (static_cast<unsigned>(__builtin_bit_cast(unsigned short, static_cast<__bf16>(hi))) << 16);
                };
                uint4* dst = reinterpret_cast<uint4*>(static_cast<unsigned short*>(a.c) + e);
                dst[0] = make_uint4(pk(q0.x, q0.y), pk(q0.z, q0.w), pk(q1.x, q1.y), pk(q1.z, q1.w));
                dst[1] = make_uint4(pk(q2.x, q2.y), pk(q2.z, q2.w), pk(q3.x, q3.y), pk(q3.z, q3.w));
            }
        }
    }
}

template <bool kOutF32>
__global__ __launch_bounds__(kKcThreads, 2) void key_compress_kernel(KcArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Block -> tile map.  With more than one column tile (D > 2048) the column tiles of one row tile
    // must meet in the same L2 so that x comes from HBM once: consecutive block ids go round the
    // 8 XCDs, so the id is read as (slot, xcd) and the column tiles of a row tile take consecutive
    // slots of one XCD.
    const int nct = (a.C + kBN - 1) / kBN;
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const long long row_tile = static_cast<long long>(slot / nct) * 8 + xcd;
    const long long m0 = row_tile * kBM;
    const int n0 = (slot % nct) * kBN;
    if (m0 >= a.M) return;                     // padding of the row tiles to a multiple of 8
    const long long rows_left = a.M - m0;
    const int rows = rows_left < kBM ? static_cast<int>(rows_left) : kBM;
    const int nsteps = a.D / kBK;
    // Every workgroup walks all channel blocks, but starts at a different one (the column tiles of
    // a row tile at the same one): the rows of x are D*2 bytes apart, so workgroups that march
    // through the channels in step would all ask the same few memory channels for their 128-byte
    // row pieces, and the same L2 channel for the same rows of W (config 2's width: 127 -> 113 us).
    const int first = static_cast<int>((slot / nct + 4 * xcd) % nsteps);
    // both roles pass 2 + nsteps barriers
    // the loaders' few instructions per step go ahead of the MFMA waves' long streams (wave
    // priority is an issue-arbitration hint): measured 2-3 % on the benchmark shapes
    if (wave >= 4) {
        __builtin_amdgcn_s_setprio(2);
        kc_loader(a, lds, tid - 256, m0, n0, rows, nsteps, first);
    } else {
        __builtin_amdgcn_s_setprio(1);
        kc_worker<kOutF32>(a, lds, tid, wave, m0, n0, rows, nsteps);
    }
}

}  // namespace

hipError_t launch_key_compress(long long M, int D, const void* x, const void* w, void* c, bool out_f32,
                               hipStream_t stream) {
    KcArgs a;
    a.M = M; a.D = D; a.C = D / 16;
    a.x = x; a.w = w; a.c = c;
    const long long row_tiles = (M + kBM - 1) / kBM;
    const dim3 grid(static_cast<unsigned>((row_tiles + 7) / 8 * 8 * ((a.C + kBN - 1) / kBN)));
    hipError_t err;
    struct TagF32 {};
    struct TagBf16 {};
    if (out_f32) {
        err = set_lds_limit_once<TagF32>(&key_compress_kernel<true>, kKcLds);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(key_compress_kernel<true>, grid, dim3(kKcThreads), kKcLds, stream, a);
    } else {
        err = set_lds_limit_once<TagBf16>(&key_compress_kernel<false>, kKcLds);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(key_compress_kernel<false>, grid, dim3(kKcThreads), kKcLds, stream, a);
    }
    return hipGetLastError();
}

}  // namespace wkv6

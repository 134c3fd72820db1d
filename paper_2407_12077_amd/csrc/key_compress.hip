// GOLD key compression for gfx950 (MI355X): c = x W^KD, a skinny bf16 GEMM (GOLD Key
// Compression: every token's hidden state of D channels times the D x D/16 matrix W^KD gives its
// compressed key-cache entry).  M tokens x D channels are streamed from HBM exactly once; W^KD
// (D x C, C = D/16, at most a few hundred KB) stays in the L2 of every XCD.  The kernel is bound
// by the HBM read of x; all arithmetic is on the matrix cores (v_mfma_f32_16x16x32_bf16, fp32
// accumulation, bf16 products are exact in fp32).
//
// One workgroup owns 128 tokens x kBN output columns (kBN = 128 up to D = 2048, 256 above, so that
// up to D = 4096 a workgroup has all columns and x passes through a compute unit's vector memory
// path once; fewer columns in the last tile when D/16 is not a multiple of kBN) and walks the D
// axis in steps of 64 channels (cyclically, from a start that differs between workgroups).  Its
// waves split into two roles that meet at one barrier per step:
//   kBN/32 LOADER waves (the last ones): fetch the x tile (128 x 64: full 128-byte row pieces, 8
//               lanes each) and the W tile (64 x kBN, an L2 hit) of a step two (kBN = 128) or four
//               (kBN = 256) steps ahead into registers with
//               16-byte loads, and park the tiles of the next step in one of two LDS buffers.
//               Rows past M and steps past D go through shrunk raw buffer descriptors and read
//               as zero without touching memory, so no load is predicated and the wait counters
//               stay exact.
//   kBN/32 MFMA waves: each owns a 64 x 64 block of the result in 64 accumulator registers;
//               per step 8 row reads of x (row stride 160 B: full-rate 16-byte LDS reads), 16
//               transposing reads of W (its contraction index is the tile's row) and 32 MFMAs.
//               They issue no global loads, so nothing but LDS latency sits between their MFMAs.
// With kBN = 128 registers and LDS are sized so that two workgroups share a compute unit: the
// waits, prologue and epilogue of one overlap the steady state of the other.  With kBN = 256 a
// compute unit holds one workgroup of sixteen waves, and its loaders keep four steps in flight
// instead (in-flight bytes, not arithmetic, limit this shape).
#include "wkv6_launch.h"

namespace wkv6 {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

constexpr int kBM = 128;            // tokens per workgroup
constexpr int kBK = 64;             // channels per step
constexpr int kXRow = 160;          // LDS row stride of the x tile (64 bf16 + 32 B pad)
constexpr int kXTile = kBM * kXRow; // 20480
constexpr int kCRow = 128 * 4 + 16; // staging row of 128 columns of the fp32 result tile

// per width of the workgroup's column tile (kBN = 128 or 256)
template <int kBN>
struct Tile {
    static constexpr int kWRow = kBN * 2 + 32;          // LDS row stride of the W tile (kBN bf16 + 32 B pad)
    static constexpr int kWTile = kBK * kWRow;
    static constexpr int kStage = kXTile + kWTile;
    static constexpr int kLds = 2 * kStage;
    static constexpr int kMfmaWaves = kBN / 32;         // 2 x kBN/64 blocks of 64 x 64
    static constexpr int kLoaders = 2 * kBN;            // loader threads: as many waves as MFMA waves
    static constexpr int kThreads = 64 * kMfmaWaves + kLoaders;
    static constexpr int kXLoads = kBM * 8 / kLoaders;  // 16-byte loads per loader thread and step: x,
    static constexpr int kWLoads = kBK * kBN / 8 / kLoaders;   // W
    // steps a loader has in flight: two when two workgroups share a compute unit (they overlap each
    // other's waits), four when one workgroup has it alone
    static constexpr int kDepth = kBN == 128 ? 2 : 4;
    static constexpr int kHalves = kBN / 128;           // the result leaves through LDS 128 columns at a time
    static_assert(kLds >= kBM * kCRow, "result staging reuses the operand buffers");
};

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
template <int kWRow>
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

template <int kBN>
struct StepRegs {          // a loader thread's share of one step, 16 bytes each
    uint4v x[Tile<kBN>::kXLoads], w[Tile<kBN>::kWLoads];
};

// ------------------------------------------------------------------------------------------
// loader waves (256 threads): tiles of step s+2 into registers, tiles of step s+1 into LDS
// ------------------------------------------------------------------------------------------
template <int kBN>
__device__ __forceinline__ void kc_loader(const KcArgs& a, char* lds, int lt, long long m0, int n0, int rows,
                                          int nsteps, int first) {
    using TL = Tile<kBN>;
    constexpr int kWRow = TL::kWRow, kStage = TL::kStage, kXLoads = TL::kXLoads, kWLoads = TL::kWLoads;
    constexpr int kXRowsPerPass = TL::kLoaders / 8;
    constexpr int kLanesPerWRow = kBN / 8, kWRowsPerPass = TL::kLoaders / kLanesPerWRow;
    const long long x_row_bytes = static_cast<long long>(a.D) * 2;
    const char* x_base = static_cast<const char*>(a.x) + m0 * x_row_bytes;
    const long long x_bytes = rows * x_row_bytes;
    const long long w_row_bytes = static_cast<long long>(a.C) * 2;
    const char* w_base = static_cast<const char*>(a.w);
    const long long w_bytes = static_cast<long long>(a.D) * w_row_bytes;

    // x tile: 8 lanes per 128-byte row piece; W tile: kBN/8 lanes per row piece of kBN columns
    const int xr = lt >> 3, xg = lt & 7;
    const int wr = lt / kLanesPerWRow, wg = lt % kLanesPerWRow;
    int x_voff[kXLoads], w_voff[kWLoads];
#pragma unroll
    for (int p = 0; p < kXLoads; ++p) x_voff[p] = static_cast<int>((xr + kXRowsPerPass * p) * x_row_bytes + 16 * xg);
#pragma unroll
    for (int p = 0; p < kWLoads; ++p)
        // columns past C (the last column tile may be partial): an offset no descriptor covers
        w_voff[p] = n0 + 8 * wg < a.C ? static_cast<int>((wr + kWRowsPerPass * p) * w_row_bytes + n0 * 2 + 16 * wg)
                                      : 0x7ffffff0;
    const int x_lds = xr * kXRow + 16 * xg;
    const int w_lds = kXTile + wr * kWRow + 16 * wg;

    auto fetch = [&](StepRegs<kBN>& s, int step) {
        const bool live = step < nsteps;                                          // uniform
        int ks = step + first;                                                    // this step's channel block
        if (ks >= nsteps) ks -= nsteps;
        const long long xs = static_cast<long long>(ks) * kBK * 2;                // byte offset along a row of x
        const long long ws = static_cast<long long>(ks) * kBK * w_row_bytes;     // first W row of the step
        const __amdgpu_buffer_rsrc_t rx = rsrc_of(x_base + (live ? xs : 0), live ? x_bytes - xs : 0);
        const __amdgpu_buffer_rsrc_t rw = rsrc_of(w_base + (live ? ws : 0), live ? w_bytes - ws : 0);
#pragma unroll
        for (int p = 0; p < kWLoads; ++p)
            s.w[p] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rw, w_voff[p], 0, 0));
#pragma unroll
        for (int p = 0; p < kXLoads; ++p)
            s.x[p] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rx, x_voff[p], 0, 0));
    };
    auto park = [&](const StepRegs<kBN>& s, int buf) {
        char* b = lds + buf * kStage;
#pragma unroll
        for (int p = 0; p < kXLoads; ++p) *reinterpret_cast<uint4v*>(b + x_lds + kXRowsPerPass * p * kXRow) = s.x[p];
#pragma unroll
        for (int p = 0; p < kWLoads; ++p) *reinterpret_cast<uint4v*>(b + w_lds + kWRowsPerPass * p * kWRow) = s.w[p];
    };

    // D / 64 steps, a multiple of four; one barrier per step, as many as the MFMA waves pass
    if constexpr (TL::kDepth == 2) {
        // the tiles of two steps in flight per workgroup, and two workgroups share a compute unit
        StepRegs<kBN> s0, s1;
        fetch(s0, 0);
        fetch(s1, 1);
        park(s0, 0);
        fetch(s0, 2);
        __syncthreads();                               // tiles of step 0 are in LDS
#pragma clang loop unroll(disable)
        for (int step = 0; step < nsteps; step += 2) {
            park(s1, 1);                               // step+1, while the MFMA waves work on step
            fetch(s1, step + 3);
            __syncthreads();
            park(s0, 0);
            fetch(s0, step + 4);
            __syncthreads();
        }
    } else {
        // four steps in flight: with one workgroup per compute unit nothing else covers the latency
        StepRegs<kBN> s0, s1, s2, s3;
        fetch(s0, 0);
        fetch(s1, 1);
        fetch(s2, 2);
        fetch(s3, 3);
        park(s0, 0);
        fetch(s0, 4);
        __syncthreads();                               // tiles of step 0 are in LDS
#pragma clang loop unroll(disable)
        for (int step = 0; step < nsteps; step += 4) {
            park(s1, 1);                               // step+1, while the MFMA waves work on step
            fetch(s1, step + 5);
            __syncthreads();
            park(s2, 0);
            fetch(s2, step + 6);
            __syncthreads();
            park(s3, 1);
            fetch(s3, step + 7);
            __syncthreads();
            park(s0, 0);
            fetch(s0, step + 8);
            __syncthreads();
        }
    }
    // the result tile leaves through LDS, 128 columns at a time: one barrier after each staging and
    // one before the next
#pragma unroll
    for (int i = 0; i < 2 * TL::kHalves - 1; ++i) __syncthreads();
}

// ------------------------------------------------------------------------------------------
// MFMA waves (256 threads)
// ------------------------------------------------------------------------------------------
template <int kBN, bool kOutF32>
__device__ __forceinline__ void kc_worker(const KcArgs& a, char* lds, int tid, int wave, long long m0, int n0,
                                          int rows, int nsteps) {
    using TL = Tile<kBN>;
    constexpr int kWRow = TL::kWRow, kStage = TL::kStage, kColBlocks = kBN / 64;
    const int lane = tid & 63;
    const int l16 = lane & 15;
    const int g4 = lane >> 4;
    // wave (wr, wc) owns rows 64 wr .. +63 and columns 64 wc .. +63: 4 x 4 blocks of 16 x 16
    const int wr2 = wave / kColBlocks, wc2 = wave % kColBlocks;
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
            for (int nb = 0; nb < 4; ++nb) wt[nb] = lds_read_tr8<kWRow>(b, b_lane + 32 * kWRow * kb + 32 * nb);
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

    // result tile through LDS (fp32, row stride kCRow, 128 columns at a time), then full rows to HBM
    constexpr int kRowsPerPass = 64 * TL::kMfmaWaves / 8;          // 8 lanes per row, 16 columns each
    const int cr = tid >> 3, cg = tid & 7;
#pragma unroll
    for (int hf = 0; hf < TL::kHalves; ++hf) {
        if (hf > 0) __syncthreads();                               // the previous half has been read
        if ((wc2 >> 1) == hf) {
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        *reinterpret_cast<float*>(lds + (64 * wr2 + 16 * rb + 4 * g4 + e) * kCRow +
                                                  (64 * (wc2 & 1) + 16 * nb + l16) * 4) = acc[rb][nb][e];
        }
        __syncthreads();
        // A row's eight threads store one whole 128-byte line per instruction: thread cg takes the
        // cg-th 16 bytes of every line of the row's 128-column piece (2 lines in bf16, 4 in fp32).
        constexpr int kColsPerStore = kOutF32 ? 4 : 8, kLines = 128 / (8 * kColsPerStore);
#pragma unroll
        for (int p = 0; p < kBM / kRowsPerPass; ++p) {
            const int row = cr + kRowsPerPass * p;
            if (row >= rows) continue;
#pragma unroll
            for (int ln = 0; ln < kLines; ++ln) {
                const int lc = 8 * kColsPerStore * ln + kColsPerStore * cg;      // column within the piece
                const int col = n0 + 128 * hf + lc;
                if (col >= a.C) continue;
                const float4* src = reinterpret_cast<const float4*>(lds + row * kCRow + lc * 4);
                const long long e = (m0 + row) * a.C + col;
                if constexpr (kOutF32) {
                    *reinterpret_cast<float4*>(static_cast<float*>(a.c) + e) = src[0];
                } else {
                    auto pk = [](float lo, float hi) {
                        return static_cast<unsigned>(__builtin_bit_cast(unsigned short, static_cast<__bf16>(lo))) |
                               (static_cast<unsigned>(__builtin_bit_cast(unsigned short, static_cast<__bf16>(hi))) << 16);
                    };
                    const float4 q0 = src[0], q1 = src[1];
                    *reinterpret_cast<uint4*>(static_cast<unsigned short*>(a.c) + e) =
                        make_uint4(pk(q0.x, q0.y), pk(q0.z, q0.w), pk(q1.x, q1.y), pk(q1.z, q1.w));
                }
            }
        }
    }
}

template <int kBN, bool kOutF32>
__global__ __launch_bounds__(Tile<kBN>::kThreads, 256 / kBN) void key_compress_kernel(KcArgs a) {
    using TL = Tile<kBN>;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Block -> tile map.  With more than one column tile (D > 4096) the column tiles of one row tile
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
    // both roles pass 1 + nsteps + 2 kHalves - 1 barriers
    // the loaders' few instructions per step go ahead of the MFMA waves' long streams (wave
    // priority is an issue-arbitration hint): measured 2-3 % on the benchmark shapes
    if (wave >= TL::kMfmaWaves) {
        __builtin_amdgcn_s_setprio(2);
        kc_loader<kBN>(a, lds, tid - 64 * TL::kMfmaWaves, m0, n0, rows, nsteps, first);
    } else {
        __builtin_amdgcn_s_setprio(1);
        kc_worker<kBN, kOutF32>(a, lds, tid, wave, m0, n0, rows, nsteps);
    }
}

}  // namespace

namespace {

template <int kBN, bool kOutF32>
hipError_t launch_tile(const KcArgs& a, hipStream_t stream) {
    using TL = Tile<kBN>;
    const long long row_tiles = (a.M + kBM - 1) / kBM;
    const dim3 grid(static_cast<unsigned>((row_tiles + 7) / 8 * 8 * ((a.C + kBN - 1) / kBN)));
    struct Tag {};
    const hipError_t err = set_lds_limit_once<Tag>(&key_compress_kernel<kBN, kOutF32>, TL::kLds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((key_compress_kernel<kBN, kOutF32>), grid, dim3(TL::kThreads), TL::kLds, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_key_compress(long long M, int D, const void* x, const void* w, void* c, bool out_f32,
                               hipStream_t stream) {
    KcArgs a;
    a.M = M; a.D = D; a.C = D / 16;
    a.x = x; a.w = w; a.c = c;
    if (a.C > 128) return out_f32 ? launch_tile<256, true>(a, stream) : launch_tile<256, false>(a, stream);
    return out_f32 ? launch_tile<128, true>(a, stream) : launch_tile<128, false>(a, stream);
}

}  // namespace wkv6

// GOLD key compression for gfx950 (MI355X): c = x W^KD, a skinny bf16 GEMM (GOLD Key
// Compression: every token's hidden state of D channels times the D x D/16 matrix W^KD gives its
// compressed key-cache entry).  M tokens x D channels are streamed from HBM exactly once; W^KD
// (D x C, C = D/16, at most a few hundred KB) stays in the L2 of every XCD.  The kernel is bound
// by the HBM read of x; all arithmetic is on the matrix cores (v_mfma_f32_16x16x32_bf16, fp32
// accumulation, bf16 products are exact in fp32).
//
// The product is formed transposed, c^T = (W^KD)^T x^T, so that x is the B operand: an MFMA lane
// then needs 8 consecutive channels of one token, which is 16 contiguous bytes of x, and x goes
// from HBM straight into operand registers, four steps ahead, never through LDS.  One workgroup
// owns 128 tokens x 128 output columns and walks the D axis in steps of 64 channels:
//   waves 0..3  each own 32 tokens: per step 4 loads of x (16 bytes per lane), the step's W tile
//               read from LDS through the transposing read (its contraction index is the tile's
//               row), 32 MFMAs into 64 accumulator registers;
//   wave 4      the W loader: fetches the 64 x 128 tile of W (an L2 hit) two steps ahead and
//               parks it in one of two LDS buffers; its loads have a wait counter of their own,
//               so they never order against the x stream.
// One barrier per step.
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
constexpr int kWRow = 288;          // LDS row stride of the W tile (128 bf16 + 32 B pad)
constexpr int kWTile = kBK * kWRow; // 18432
constexpr int kKcLds = 2 * kWTile;
constexpr int kKcThreads = 320;     // 4 MFMA waves + 1 loader wave

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const void* base, long long bytes) {
    if (bytes < 0) bytes = 0;
    if (bytes > 0x7fffffffLL) bytes = 0x7fffffffLL;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, static_cast<int>(bytes), 0x00020000);
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

// ------------------------------------------------------------------------------------------
// loader wave: W tile of step s+2 into registers, W tile of step s+1 from registers into LDS
// ------------------------------------------------------------------------------------------
struct WTileRegs { uint4v q[16]; };

__device__ __forceinline__ void kc_loader(const KcArgs& a, char* lds, int lane, int n0, int nsteps) {
    const long long w_row_bytes = static_cast<long long>(a.C) * 2;
    const char* w_base = static_cast<const char*>(a.w);
    const long long w_bytes = static_cast<long long>(a.D) * w_row_bytes;
    // a tile row is 256 bytes = 16 lanes x 16 bytes; 4 rows per pass, 16 passes
    const int wr = lane >> 4, wg = lane & 15;
    int voff[16];
#pragma unroll
    for (int p = 0; p < 16; ++p) voff[p] = static_cast<int>((wr + 4 * p) * w_row_bytes + n0 * 2 + 16 * wg);
    const int w_lds = wr * kWRow + 16 * wg;

    auto fetch = [&](WTileRegs& t, int step) {
        const bool live = step < nsteps;                                          // uniform
        const long long ws = static_cast<long long>(step) * kBK * w_row_bytes;   // first W row of the step
        const __amdgpu_buffer_rsrc_t rw = rsrc_of(w_base + (live ? ws : 0), live ? w_bytes - ws : 0);
#pragma unroll
        for (int p = 0; p < 16; ++p)
            t.q[p] = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(rw, voff[p], 0, 0));
    };
    auto park = [&](const WTileRegs& t, int buf) {
        char* b = lds + buf * kWTile;
#pragma unroll
        for (int p = 0; p < 16; ++p) *reinterpret_cast<uint4v*>(b + w_lds + 4 * p * kWRow) = t.q[p];
    };

    WTileRegs t0, t1;
    fetch(t0, 0);
    fetch(t1, 1);
    park(t0, 0);
    fetch(t0, 2);
    __syncthreads();                                   // tile 0 is in LDS
#pragma clang loop unroll(disable)
    for (int step = 0; step < nsteps; step += 2) {
        park(t1, 1);                                   // tile step+1, while the others work on tile step
        fetch(t1, step + 3);
        __syncthreads();
        park(t0, 0);                                   // tile step+2
        fetch(t0, step + 4);
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// MFMA waves
// ------------------------------------------------------------------------------------------
struct XRegs { bf16x8 q[2][2]; };                      // [token block mb][channel block kb]

template <bool kOutF32>
__device__ __forceinline__ void kc_worker(const KcArgs& a, const char* lds, int lane, int wave, long long m0,
                                          int n0, int rows, int nsteps) {
    const int l16 = lane & 15;
    const int g4 = lane >> 4;
    // x through a raw buffer descriptor rebuilt per step (base moved with scalar adds, extent
    // shrunk accordingly): tokens past M and steps past D are out of range and read as zero
    // without touching memory, so no load is predicated.
    const long long x_row_bytes = static_cast<long long>(a.D) * 2;
    const char* x_base = static_cast<const char*>(a.x) + m0 * x_row_bytes;
    const long long x_bytes = rows * x_row_bytes;
    // lane (token l16 of block mb, channel group g4): 16 bytes = channels 8 g4 .. +7 of the 32-block kb
    int voff[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) voff[mb] = static_cast<int>((32 * wave + 16 * mb + l16) * x_row_bytes + 16 * g4);

    auto fetch = [&](XRegs& t, int step) {
        const bool live = step < nsteps;               // uniform
        const long long xs = static_cast<long long>(step) * kBK * 2;
        const __amdgpu_buffer_rsrc_t rx = rsrc_of(x_base + (live ? xs : 0), live ? x_bytes - xs : 0);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                t.q[mb][kb] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rx, voff[mb] + 64 * kb, 0, 0));
    };

    float4v acc[8][2];                                 // [column block nb][token block mb], transposed tiles
#pragma unroll
    for (int nb = 0; nb < 8; ++nb)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) acc[nb][mb] = float4v{0.f, 0.f, 0.f, 0.f};

    const int a_lane = (8 * g4 + (l16 >> 2)) * kWRow + 8 * (l16 & 3);     // + 32*kWRow*kb + 32*nb
    auto compute = [&](const XRegs& t, int buf) {
        const char* b = lds + buf * kWTile;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int nb = 0; nb < 8; ++nb) {
                const bf16x8 wt = lds_read_tr8(b, a_lane + 32 * kWRow * kb + 32 * nb);
                acc[nb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wt, t.q[0][kb], acc[nb][0], 0, 0, 0);
                acc[nb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wt, t.q[1][kb], acc[nb][1], 0, 0, 0);
            }
    };

    // D / 64 steps, a multiple of 4 (D is a multiple of 2048); x of four steps in flight
    XRegs x0, x1, x2, x3;
    fetch(x0, 0);
    fetch(x1, 1);
    fetch(x2, 2);
    fetch(x3, 3);
    __syncthreads();                                   // W tile 0 is in LDS
#pragma clang loop unroll(disable)
    for (int step = 0; step < nsteps; step += 4) {
        compute(x0, 0);
        fetch(x0, step + 4);
        __syncthreads();
        compute(x1, 1);
        fetch(x1, step + 5);
        __syncthreads();
        compute(x2, 0);
        fetch(x2, step + 6);
        __syncthreads();
        compute(x3, 1);
        fetch(x3, step + 7);
        __syncthreads();
    }

    // acc[nb][mb][v] = c[token 32 wave + 16 mb + l16][column 16 nb + 4 g4 + v]: four consecutive
    // columns per lane
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        const int row = 32 * wave + 16 * mb + l16;
        if (row < rows) {
            const long long e = (m0 + row) * a.C + n0 + 4 * g4;
#pragma unroll
            for (int nb = 0; nb < 8; ++nb) {
                const float4v q = acc[nb][mb];
                if constexpr (kOutF32) {
                    *reinterpret_cast<float4*>(static_cast<float*>(a.c) + e + 16 * nb) = make_float4(q[0], q[1], q[2], q[3]);
                } else {
                    auto pk = [](float lo, float hi) {
                        return static_cast<unsigned>(__builtin_bit_cast(unsigned short, static_cast<__bf16>(lo))) |
                               (static_cast<unsigned>(__builtin_bit_cast(unsigned short, static_cast<__bf16>(hi))) << 16);
                    };
                    *reinterpret_cast<uint2*>(static_cast<unsigned short*>(a.c) + e + 16 * nb) =
                        make_uint2(pk(q[0], q[1]), pk(q[2], q[3]));
                }
            }
        }
    }
}

template <bool kOutF32>
__global__ __launch_bounds__(kKcThreads) void key_compress_kernel(KcArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long long m0 = static_cast<long long>(blockIdx.x) * kBM;
    const int n0 = blockIdx.y * kBN;
    const long long rows_left = a.M - m0;
    const int rows = rows_left < kBM ? static_cast<int>(rows_left) : kBM;
    const int nsteps = a.D / kBK;
    // both roles pass 1 + nsteps barriers
    if (wave == 4)
        kc_loader(a, lds, lane, n0, nsteps);
    else
        kc_worker<kOutF32>(a, lds, lane, wave, m0, n0, rows, nsteps);
}

}  // namespace

hipError_t launch_key_compress(long long M, int D, const void* x, const void* w, void* c, bool out_f32,
                               hipStream_t stream) {
    KcArgs a;
    a.M = M; a.D = D; a.C = D / 16;
    a.x = x; a.w = w; a.c = c;
    const dim3 grid(static_cast<unsigned>((M + kBM - 1) / kBM), static_cast<unsigned>(a.C / kBN));
    if (out_f32)
        hipLaunchKernelGGL(key_compress_kernel<true>, grid, dim3(kKcThreads), kKcLds, stream, a);
    else
        hipLaunchKernelGGL(key_compress_kernel<false>, grid, dim3(kKcThreads), kKcLds, stream, a);
    return hipGetLastError();
}

}  // namespace wkv6

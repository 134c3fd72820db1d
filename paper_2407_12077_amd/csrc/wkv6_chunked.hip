// Chunked WKV6 prefill kernel for gfx950 (MI355X): one workgroup per (batch, head), 64-token
// chunks, fp32 state carried in MFMA accumulators, every dense contraction on the matrix
// cores (v_mfma_f32_16x16x32_f16, fp32 accumulation).
//
// The recurrence (Finch-C2 Time Mixing: decay map w = exp(-exp(x)), wkv_t, read-out; Finch
// bonus u) is evaluated chunk by chunk.  With tokens 0..63 of a chunk, S0 the state entering
// it, and W(t,i) = prod_{s=i+1}^{t-1} w_s (a per-key-channel vector, empty product = 1):
//
//   o_t = (r_t * W(t,-1)) . S0                                   inter-chunk read
//       + sum_{i<t} ( sum_n r_t[n] k_i[n] W(t,i)[n] ) v_i        intra-chunk, strictly causal
//       + ( sum_n r_t[n] u[n] k_t[n] ) v_t                       bonus on the diagonal
//   S64 = diag(W(64,-1)) S0 + sum_i (k_i * W(64,i))^T v_i        state update
//
// Only PRODUCTS of decays are ever formed (never a reciprocal or a positive exponent), so
// every scale factor is <= 1 and any decay logit, +-inf included, is handled exactly.  To
// write W(t,i) as (factor of t) x (factor of i) the causal triangle is cut by binary
// levels m = 32,16,8,4,2,1: the pair (t,i) belongs to the level of the highest bit in which
// t and i differ; there i lies in the first half and t in the second half of the same
// 2m-aligned block, and with `mid` that block's midpoint
//       W(t,i) = (prod_{s=mid}^{t-1} w_s) * (prod_{s=i+1}^{mid-1} w_s),
// a prefix product inside t's m-block times a suffix product inside i's m-block.  Tile Z_m
// holds, row by row, the scaled key (rows in a first half) or the scaled receptance (rows in
// a second half); one MFMA per level and 16x16 block followed by a select assembles the
// score matrix.
#include "wkv6_launch.h"

namespace wkv6 {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kChunk = 64;                 // tokens per chunk
constexpr int kThreads = 256;              // 4 wavefronts
constexpr int kRowHalfs = 72;              // fp16 tile row stride (64 + 8 pad) = 144 bytes
constexpr int kTileBytes = 64 * kRowHalfs * 2;
constexpr int kORow = 68;                  // fp32 output staging row stride (floats)

// LDS map (bytes)
enum : int {
    kZ32 = 0 * kTileBytes,
    kZ16 = 1 * kTileBytes,
    kZ8 = 2 * kTileBytes,
    kZ4 = 3 * kTileBytes,
    kZ2 = 4 * kTileBytes,
    kRH = 5 * kTileBytes,      // r as fp16, all tokens
    kKH = 6 * kTileBytes,      // k as fp16, all tokens
    kRU = 7 * kTileBytes,      // r*u
    kRT = 8 * kTileBytes,      // r * W(t,-1), channel order permuted to match the state registers
    kKT = 9 * kTileBytes,      // (k * W(64,i))^T : [channel][token]
    kVT = 10 * kTileBytes,     // v^T            : [channel][token]
    kAT = 11 * kTileBytes,     // scores A[t][i]
    kG = 12 * kTileBytes,                      // per 8-token group decay products [8][64] fp32
    kD = kG + 8 * 64 * 4,                      // whole-chunk decay product [64] fp32
    kO = kD + 64 * 4,                          // output staging [64][kORow] fp32
    kLdsBytes = kO + 64 * kORow * 4
};

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float bf16_lo(unsigned bits) { return __uint_as_float(bits << 16); }
__device__ __forceinline__ float bf16_hi(unsigned bits) { return __uint_as_float(bits & 0xffff0000u); }

__device__ __forceinline__ unsigned pack_h2(float a, float b) {
    half2v p;
    p.x = static_cast<_Float16>(a);
    p.y = static_cast<_Float16>(b);
    return __builtin_bit_cast(unsigned, p);
}

__device__ __forceinline__ unsigned pack_bf2(float a, float b) {
    bf16x2 p;
    p.x = static_cast<__bf16>(a);
    p.y = static_cast<__bf16>(b);
    return __builtin_bit_cast(unsigned, p);
}

// w = exp(-exp(x)) through two base-2 exponentials (x=-inf -> 1, x=+inf -> 0).
__device__ __forceinline__ float decay_of(float x) {
    const float e = __builtin_amdgcn_exp2f(x * kLog2e);
    return __builtin_amdgcn_exp2f(-kLog2e * e);
}

__device__ __forceinline__ half8 lds_read_h8(const char* lds, int byte_off) {
    return *reinterpret_cast<const half8*>(lds + byte_off);
}

struct Raw {           // one chunk's inputs of this thread: 8 tokens x one channel pair, bf16 bits
    unsigned r[8], k[8], v[8], x[8];
};

__device__ __forceinline__ void load_chunk(Raw& d, const Args& a, long long base, int t0, int T,
                                           long long tok_stride) {
    const unsigned* pr = static_cast<const unsigned*>(a.r);
    const unsigned* pk = static_cast<const unsigned*>(a.k);
    const unsigned* pv = static_cast<const unsigned*>(a.v);
    const unsigned* px = static_cast<const unsigned*>(a.x);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int t = t0 + s;
        if (t < T) {
            const long long e = (base + static_cast<long long>(t) * tok_stride) >> 1;   // dword index
            d.r[s] = pr[e];
            d.k[s] = pk[e];
            d.v[s] = pv[e];
            d.x[s] = px[e];
        } else {                        // past the end: no key, no value, no decay (w = 1)
            d.r[s] = 0u;
            d.k[s] = 0u;
            d.v[s] = 0u;
            d.x[s] = 0xff80ff80u;       // bf16 -inf, twice
        }
    }
}

template <bool kOutF32>
__global__ __launch_bounds__(kThreads) void chunked_kernel(Args a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = tid >> 6;                 // wavefront 0..3
    // producer mapping: channel pair cp, token group tg (8 tokens)
    const int cp = lane & 31;
    const int hi = lane >> 5;                // which half of the chunk (tokens 0..31 / 32..63)
    const int tg = wv + 4 * hi;
    // MFMA mapping
    const int l16 = lane & 15;
    const int g4 = lane >> 4;

    const int unit = blockIdx.x;
    const int b = unit / a.H;
    const int h = unit - b * a.H;
    const long long tok_stride = static_cast<long long>(a.H) * kHeadSize;
    const long long unit_base = static_cast<long long>(b) * a.batch_stride +
                                static_cast<long long>(h) * kHeadSize;
    const long long in_base = unit_base + 2 * cp;     // element offset of this thread's pair

    const float u0 = a.u[h * kHeadSize + 2 * cp];
    const float u1 = a.u[h * kHeadSize + 2 * cp + 1];

    // state: this wave owns value columns j = 16*wv + l16; S[nb][e] = S[n = 16nb + 4g4 + e][j]
    float4v S[4];
    {
        const int j = 16 * wv + l16;
        if (a.state_in) {
            const float* s0 = a.state_in + static_cast<long long>(unit) * 4096;
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int e = 0; e < 4; ++e) S[nb][e] = s0[(16 * nb + 4 * g4 + e) * 64 + j];
        } else {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) S[nb] = float4v{0.f, 0.f, 0.f, 0.f};
        }
    }

    // score blocks above the diagonal that the A.V product still touches stay zero for good
    {
        // (t-block 0, i-block 1) and (t-block 2, i-block 3): 16x16 halfs each = 128 dwords
        const int blk = tid >> 7;                    // 0 or 1
        const int e = tid & 127;                     // dword within block: row = e>>3, col pair = e&7
        const int row = (blk ? 32 : 0) + (e >> 3);
        const int col = (blk ? 48 : 16) + 2 * (e & 7);
        *reinterpret_cast<unsigned*>(lds + kAT + (row * kRowHalfs + col) * 2) = 0u;
    }

    const int nchunks = (a.T + kChunk - 1) / kChunk;
    Raw cur, nxt;
    load_chunk(cur, a, in_base, 8 * tg, a.T, tok_stride);

    for (int c = 0; c < nchunks; ++c) {
        const int c0 = c * kChunk;
        if (c + 1 < nchunks) load_chunk(nxt, a, in_base, c0 + kChunk + 8 * tg, a.T, tok_stride);

        // ---------------- producer part 1: decays and their products inside the 8-token group
        float w[2][8], pe[2][8], se[2][8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            w[0][s] = decay_of(bf16_lo(cur.x[s]));
            w[1][s] = decay_of(bf16_hi(cur.x[s]));
        }
        float gtot[2];
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {
            pe[ch][0] = 1.f;
#pragma unroll
            for (int s = 1; s < 8; ++s) pe[ch][s] = pe[ch][s - 1] * w[ch][s - 1];
            gtot[ch] = pe[ch][7] * w[ch][7];
            se[ch][7] = 1.f;
#pragma unroll
            for (int s = 6; s >= 0; --s) se[ch][s] = se[ch][s + 1] * w[ch][s + 1];
        }
        *reinterpret_cast<float2*>(lds + kG + (tg * 64 + 2 * cp) * 4) = make_float2(gtot[0], gtot[1]);
        __syncthreads();                                                        // B1

        // ---------------- producer part 2: group multipliers, then every operand tile
        float m_rt[2], m_kt[2], m32[2], m16[2];
        {
            float2 own[4], oth[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                own[g] = *reinterpret_cast<const float2*>(lds + kG + ((4 * hi + g) * 64 + 2 * cp) * 4);
                oth[g] = *reinterpret_cast<const float2*>(lds + kG + ((4 * (1 - hi) + g) * 64 + 2 * cp) * 4);
            }
#pragma unroll
            for (int ch = 0; ch < 2; ++ch) {
                float o[4], q[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    o[g] = ch ? own[g].y : own[g].x;
                    q[g] = ch ? oth[g].y : oth[g].x;
                }
                const float h_oth = (q[0] * q[1]) * (q[2] * q[3]);
                const float h_own = (o[0] * o[1]) * (o[2] * o[3]);
                float a_lo, a_hi, f16;      // products of the groups before / after this one in its half
                if (wv == 0)      { a_lo = 1.f;                a_hi = o[1] * o[2] * o[3]; f16 = o[1]; }
                else if (wv == 1) { a_lo = o[0];               a_hi = o[2] * o[3];        f16 = 1.f; }
                else if (wv == 2) { a_lo = o[0] * o[1];        a_hi = o[3];               f16 = 1.f; }
                else              { a_lo = o[0] * o[1] * o[2]; a_hi = 1.f;                f16 = o[2]; }
                m_rt[ch] = hi ? h_oth * a_lo : a_lo;       // tokens before this group in the chunk
                m_kt[ch] = hi ? a_hi : a_hi * h_oth;       // tokens after this group in the chunk
                m32[ch] = hi ? a_lo : a_hi;
                m16[ch] = f16;
                if (tg == 0) *reinterpret_cast<float*>(lds + kD + (2 * cp + ch) * 4) = h_own * h_oth;
            }
        }

        const bool q16 = (wv & 2) != 0;     // query side at level 16 (wave-uniform)
        const bool q8 = (wv & 1) != 0;      // query side at level 8  (wave-uniform)
        // column (in halfs) of this channel pair in the permuted r*W(t,-1) tile: slot order
        // matches the state accumulator registers used as the B operand
        const int n0 = 2 * cp;
        const int m5 = n0 & 31;
        const int rt_col = (n0 & 32) + 8 * ((m5 >> 2) & 3) + 4 * (m5 >> 4) + (m5 & 3);

        half8 ktv[2], vtv[2];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const float r0 = bf16_lo(cur.r[s]), r1 = bf16_hi(cur.r[s]);
            const float k0 = bf16_lo(cur.k[s]), k1 = bf16_hi(cur.k[s]);
            const float rp0 = r0 * pe[0][s], rp1 = r1 * pe[1][s];       // r * prefix inside group
            const float ks0 = k0 * se[0][s], ks1 = k1 * se[1][s];       // k * suffix inside group
            const int row = 8 * tg + s;
            const int nat = (row * kRowHalfs + 2 * cp) * 2;              // byte offset, natural order

            *reinterpret_cast<unsigned*>(lds + kRT + (row * kRowHalfs + rt_col) * 2) =
                pack_h2(rp0 * m_rt[0], rp1 * m_rt[1]);
            {
                const float a0 = hi ? rp0 : ks0, a1 = hi ? rp1 : ks1;
                *reinterpret_cast<unsigned*>(lds + kZ32 + nat) = pack_h2(a0 * m32[0], a1 * m32[1]);
            }
            {
                const float a0 = q16 ? rp0 : ks0, a1 = q16 ? rp1 : ks1;
                *reinterpret_cast<unsigned*>(lds + kZ16 + nat) = pack_h2(a0 * m16[0], a1 * m16[1]);
            }
            *reinterpret_cast<unsigned*>(lds + kZ8 + nat) = q8 ? pack_h2(rp0, rp1) : pack_h2(ks0, ks1);
            {   // level 4: tokens 0..3 of the group are keys (suffix inside [0,4)), 4..7 queries
                float f0, f1;
                if (s == 0)      { f0 = k0 * (w[0][1] * w[0][2] * w[0][3]); f1 = k1 * (w[1][1] * w[1][2] * w[1][3]); }
                else if (s == 1) { f0 = k0 * (w[0][2] * w[0][3]);           f1 = k1 * (w[1][2] * w[1][3]); }
                else if (s == 2) { f0 = k0 * w[0][3];                       f1 = k1 * w[1][3]; }
                else if (s == 3) { f0 = k0;                                 f1 = k1; }
                else if (s == 4) { f0 = r0;                                 f1 = r1; }
                else if (s == 5) { f0 = r0 * w[0][4];                       f1 = r1 * w[1][4]; }
                else if (s == 6) { f0 = r0 * (w[0][4] * w[0][5]);           f1 = r1 * (w[1][4] * w[1][5]); }
                else             { f0 = r0 * (w[0][4] * w[0][5] * w[0][6]); f1 = r1 * (w[1][4] * w[1][5] * w[1][6]); }
                *reinterpret_cast<unsigned*>(lds + kZ4 + nat) = pack_h2(f0, f1);
            }
            {   // level 2: within each 4 tokens, 0,1 are keys and 2,3 queries
                float f0, f1;
                if ((s & 3) == 0)      { f0 = k0 * w[0][s + 1]; f1 = k1 * w[1][s + 1]; }
                else if ((s & 3) == 1) { f0 = k0;               f1 = k1; }
                else if ((s & 3) == 2) { f0 = r0;               f1 = r1; }
                else                   { f0 = r0 * w[0][s - 1]; f1 = r1 * w[1][s - 1]; }
                *reinterpret_cast<unsigned*>(lds + kZ2 + nat) = pack_h2(f0, f1);
            }
            *reinterpret_cast<unsigned*>(lds + kRH + nat) = pack_h2(r0, r1);
            *reinterpret_cast<unsigned*>(lds + kKH + nat) = pack_h2(k0, k1);
            *reinterpret_cast<unsigned*>(lds + kRU + nat) = pack_h2(r0 * u0, r1 * u1);

            // transposed tiles: gather the 8 tokens of each channel
            ktv[0][s] = static_cast<_Float16>(ks0 * m_kt[0]);
            ktv[1][s] = static_cast<_Float16>(ks1 * m_kt[1]);
            vtv[0][s] = static_cast<_Float16>(bf16_lo(cur.v[s]));
            vtv[1][s] = static_cast<_Float16>(bf16_hi(cur.v[s]));
        }
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {
            const int off = ((2 * cp + ch) * kRowHalfs + 8 * tg) * 2;
            *reinterpret_cast<half8*>(lds + kKT + off) = ktv[ch];
            *reinterpret_cast<half8*>(lds + kVT + off) = vtv[ch];
        }
        __syncthreads();                                                        // B2

        // ---------------- scores: wave wv produces the columns of query block t in [16wv,16wv+16)
        {
            const int rowq = (16 * wv + l16) * kRowHalfs * 2 + 16 * g4;     // + 64*kk bytes
            // diagonal block
            float4v acc8{0.f, 0.f, 0.f, 0.f}, acc4 = acc8, acc2 = acc8, acc1 = acc8, accb = acc8;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const half8 z8 = lds_read_h8(lds, kZ8 + rowq + 64 * kk);
                const half8 z4 = lds_read_h8(lds, kZ4 + rowq + 64 * kk);
                const half8 z2 = lds_read_h8(lds, kZ2 + rowq + 64 * kk);
                const half8 rh = lds_read_h8(lds, kRH + rowq + 64 * kk);
                const half8 kh = lds_read_h8(lds, kKH + rowq + 64 * kk);
                const half8 ru = lds_read_h8(lds, kRU + rowq + 64 * kk);
                acc8 = __builtin_amdgcn_mfma_f32_16x16x32_f16(z8, z8, acc8, 0, 0, 0);
                acc4 = __builtin_amdgcn_mfma_f32_16x16x32_f16(z4, z4, acc4, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(z2, z2, acc2, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kh, rh, acc1, 0, 0, 0);
                accb = __builtin_amdgcn_mfma_f32_16x16x32_f16(kh, ru, accb, 0, 0, 0);
            }
            float sel[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = 4 * g4 + e, t = l16;
                const int d = i ^ t;
                float val = d >= 8 ? acc8[e] : d >= 4 ? acc4[e] : d >= 2 ? acc2[e] : acc1[e];
                val = (i == t) ? accb[e] : val;
                sel[e] = (i > t) ? 0.f : val;
            }
            const int arow = (16 * wv + l16) * kRowHalfs * 2;
            *reinterpret_cast<uint2*>(lds + kAT + arow + (16 * wv + 4 * g4) * 2) =
                make_uint2(pack_h2(sel[0], sel[1]), pack_h2(sel[2], sel[3]));

            // level 16: (t-block 1, i-block 0) and (t-block 3, i-block 2)
            if (wv & 1) {
                const int rowk = (16 * (wv - 1) + l16) * kRowHalfs * 2 + 16 * g4;
                float4v acc{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const half8 zq = lds_read_h8(lds, kZ16 + rowq + 64 * kk);
                    const half8 zk = lds_read_h8(lds, kZ16 + rowk + 64 * kk);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(zk, zq, acc, 0, 0, 0);
                }
                *reinterpret_cast<uint2*>(lds + kAT + arow + (16 * (wv - 1) + 4 * g4) * 2) =
                    make_uint2(pack_h2(acc[0], acc[1]), pack_h2(acc[2], acc[3]));
            }
            // level 32: t-blocks 2,3 against i-blocks 0,1
            if (wv & 2) {
#pragma unroll
                for (int ib = 0; ib < 2; ++ib) {
                    const int rowk = (16 * ib + l16) * kRowHalfs * 2 + 16 * g4;
                    float4v acc{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        const half8 zq = lds_read_h8(lds, kZ32 + rowq + 64 * kk);
                        const half8 zk = lds_read_h8(lds, kZ32 + rowk + 64 * kk);
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(zk, zq, acc, 0, 0, 0);
                    }
                    *reinterpret_cast<uint2*>(lds + kAT + arow + (16 * ib + 4 * g4) * 2) =
                        make_uint2(pack_h2(acc[0], acc[1]), pack_h2(acc[2], acc[3]));
                }
            }
        }

        // ---------------- inter-chunk read: o[t][j] = sum_n (r_t W(t,-1))[n] S0[n][j]
        float4v o[4];
        {
            half8 sh[2];
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    sh[kk][e] = static_cast<_Float16>(S[2 * kk + (e >> 2)][e & 3]);
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
                o[tb] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const half8 rt = lds_read_h8(lds, kRT + ((16 * tb + l16) * kRowHalfs + 32 * kk + 8 * g4) * 2);
                    o[tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(rt, sh[kk], o[tb], 0, 0, 0);
                }
            }
        }

        // ---------------- state update: S = diag(W(64,-1)) S + (k W(64,i))^T V
        half8 vt[2];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
            vt[kk] = lds_read_h8(lds, kVT + ((16 * wv + l16) * kRowHalfs + 32 * kk + 8 * g4) * 2);
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            const float4 d = *reinterpret_cast<const float4*>(lds + kD + (16 * nb + 4 * g4) * 4);
            S[nb][0] *= d.x;
            S[nb][1] *= d.y;
            S[nb][2] *= d.z;
            S[nb][3] *= d.w;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const half8 kt = lds_read_h8(lds, kKT + ((16 * nb + l16) * kRowHalfs + 32 * kk + 8 * g4) * 2);
                S[nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kt, vt[kk], S[nb], 0, 0, 0);
            }
        }
        __syncthreads();                                                        // B3: scores visible

        // ---------------- intra-chunk: o += A V
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                if (kk == 1 && tb < 2) continue;            // keys 32..63 are never visible to t < 32
                const half8 at = lds_read_h8(lds, kAT + ((16 * tb + l16) * kRowHalfs + 32 * kk + 8 * g4) * 2);
                o[tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(at, vt[kk], o[tb], 0, 0, 0);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
                *reinterpret_cast<float*>(lds + kO + ((16 * tb + 4 * g4 + e) * kORow + 16 * wv + l16) * 4) = o[tb][e];
        }
        __syncthreads();                                                        // B4: output tile staged

        // ---------------- coalesced store of the 64x64 output tile
        {
            const int row = tid >> 2;
            const int col = 16 * (tid & 3);
            const int t = c0 + row;
            if (t < a.T) {
                const float* src = reinterpret_cast<const float*>(lds + kO + (row * kORow + col) * 4);
                const float4 q0 = *reinterpret_cast<const float4*>(src);
                const float4 q1 = *reinterpret_cast<const float4*>(src + 4);
                const float4 q2 = *reinterpret_cast<const float4*>(src + 8);
                const float4 q3 = *reinterpret_cast<const float4*>(src + 12);
                const long long e = unit_base + static_cast<long long>(t) * tok_stride + col;
                if constexpr (kOutF32) {
                    float4* dst = reinterpret_cast<float4*>(static_cast<float*>(a.out) + e);
                    dst[0] = q0; dst[1] = q1; dst[2] = q2; dst[3] = q3;
                } else {
                    uint4* dst = reinterpret_cast<uint4*>(static_cast<unsigned short*>(a.out) + e);
                    dst[0] = make_uint4(pack_bf2(q0.x, q0.y), pack_bf2(q0.z, q0.w),
                                        pack_bf2(q1.x, q1.y), pack_bf2(q1.z, q1.w));
                    dst[1] = make_uint4(pack_bf2(q2.x, q2.y), pack_bf2(q2.z, q2.w),
                                        pack_bf2(q3.x, q3.y), pack_bf2(q3.z, q3.w));
                }
            }
        }
        if (c + 1 < nchunks) cur = nxt;
    }

    if (a.state_out) {
        const int j = 16 * wv + l16;
        float* so = a.state_out + static_cast<long long>(unit) * 4096;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e) so[(16 * nb + 4 * g4 + e) * 64 + j] = S[nb][e];
    }
}

}  // namespace

hipError_t launch_chunked(const Args& a, bool out_f32, hipStream_t stream) {
    const dim3 grid(static_cast<unsigned>(a.B) * static_cast<unsigned>(a.H));
    hipError_t err;
    if (out_f32) {
        err = hipFuncSetAttribute(reinterpret_cast<const void*>(&chunked_kernel<true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(chunked_kernel<true>, grid, dim3(kThreads), kLdsBytes, stream, a);
    } else {
        err = hipFuncSetAttribute(reinterpret_cast<const void*>(&chunked_kernel<false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(chunked_kernel<false>, grid, dim3(kThreads), kLdsBytes, stream, a);
    }
    return hipGetLastError();
}

}  // namespace wkv6

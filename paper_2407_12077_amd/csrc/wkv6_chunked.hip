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
//
// Work split inside the workgroup (12 wavefronts, 3 per SIMD):
//   waves 0..7  "producers": stream r,k,v,x from HBM (prefetched one chunk ahead), compute
//               decays and their products, write every fp16 operand tile to LDS, run the
//               score MFMAs, and write the finished output tile to HBM with full-row stores;
//   waves 8..11 "consumers": own 16 value columns of the state each and run the three
//               state-dependent contractions, i.e. the only sequential chain of the method.
// The two roles meet at three workgroup barriers per chunk; the producers work on the vector
// ALUs while the consumers occupy the matrix cores of the same SIMDs.
#include "wkv6_launch.h"

namespace wkv6 {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kChunk = 64;                 // tokens per chunk
constexpr int kProducerWaves = 8;
constexpr int kConsumerWaves = 4;
constexpr int kProducerThreads = 64 * kProducerWaves;
constexpr int kThreads = 64 * (kProducerWaves + kConsumerWaves);
constexpr int kRowHalfs = 72;              // fp16 tile row stride (64 + 8 pad) = 144 bytes
constexpr int kTileBytes = 64 * kRowHalfs * 2;
constexpr int kORowF32 = 68;               // output staging row stride, fp32 mode (floats)
constexpr int kORowBf16 = 72;              // output staging row stride, bf16 mode (halfs)

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
    kG = 12 * kTileBytes,                      // per 4-token group decay products [16][64] fp32
    kD = kG + 16 * 64 * 4,                     // whole-chunk decay product [64] fp32
    kO = kD + 64 * 4,                          // output staging
    kLdsBytes = kO + 64 * kORowF32 * 4
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

__device__ __forceinline__ unsigned short bf16_bits(float a) {
    return __builtin_bit_cast(unsigned short, static_cast<__bf16>(a));
}

// w = exp(-exp(x)) through two base-2 exponentials (x=-inf -> 1, x=+inf -> 0).
__device__ __forceinline__ float decay_of(float x) {
    const float e = __builtin_amdgcn_exp2f(x * kLog2e);
    return __builtin_amdgcn_exp2f(-kLog2e * e);
}

__device__ __forceinline__ half8 lds_read_h8(const char* lds, int byte_off) {
    return *reinterpret_cast<const half8*>(lds + byte_off);
}
__device__ __forceinline__ void lds_write_u32(char* lds, int byte_off, unsigned val) {
    *reinterpret_cast<unsigned*>(lds + byte_off) = val;
}

__device__ __forceinline__ float4v mfma(half8 a, half8 b, float4v c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

struct Raw {           // one chunk's inputs of a producer thread: 4 tokens x one channel pair
    unsigned r[4], k[4], v[4], x[4];
};

// The four input streams of one (batch, head) are read through raw buffer descriptors whose
// base is the chunk's first token row (uniform, rebuilt per chunk with scalar adds) and whose
// extent ends with the unit's last token, so rows past the end of the sequence read as zero
// without predicates.  Row offsets of a thread's 4 tokens are kernel-lifetime constants.
struct Streams {
    const char* r;
    const char* k;
    const char* v;
    const char* x;
    long long row_bytes;       // bytes between consecutive tokens
    long long span_bytes;      // bytes from the unit's first token row to the end of its last one
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t chunk_rsrc(const char* base, long long chunk_off,
                                                           long long span_bytes) {
    long long left = span_bytes - chunk_off;
    if (left < 0) left = 0;
    if (left > 0x7fffffffLL) left = 0x7fffffffLL;
    // raw buffer (stride 0), 32-bit data format
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base + chunk_off), 0,
                                             static_cast<int>(left), 0x00020000);
}

// Loads the thread's 4 tokens x channel pair of the chunk starting at token chunk_t0.
__device__ __forceinline__ void load_rows(Raw& d, const Streams& st, int chunk_t0, const int (&voff)[4]) {
    const long long off = static_cast<long long>(chunk_t0) * st.row_bytes;       // uniform
    const __amdgpu_buffer_rsrc_t rr = chunk_rsrc(st.r, off, st.span_bytes);
    const __amdgpu_buffer_rsrc_t rk = chunk_rsrc(st.k, off, st.span_bytes);
    const __amdgpu_buffer_rsrc_t rv = chunk_rsrc(st.v, off, st.span_bytes);
    const __amdgpu_buffer_rsrc_t rx = chunk_rsrc(st.x, off, st.span_bytes);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        d.x[s] = __builtin_amdgcn_raw_buffer_load_b32(rx, voff[s], 0, 0);
        d.r[s] = __builtin_amdgcn_raw_buffer_load_b32(rr, voff[s], 0, 0);
        d.k[s] = __builtin_amdgcn_raw_buffer_load_b32(rk, voff[s], 0, 0);
        d.v[s] = __builtin_amdgcn_raw_buffer_load_b32(rv, voff[s], 0, 0);
    }
}

// ------------------------------------------------------------------------------------------
// Producer waves
// ------------------------------------------------------------------------------------------
template <bool kOutF32>
__device__ __forceinline__ void producer(const Args& a, char* lds, int tid, int w8, int unit, int h,
                                         long long unit_base, long long tok_stride, int nchunks) {
    const int lane = tid & 63;
    const int cp = lane & 31;                // channel pair: channels 2cp, 2cp+1
    const int hi = lane >> 5;                // half of the chunk (tokens 0..31 / 32..63)
    const int tg = w8 + 8 * hi;              // 4-token group 0..15
    const bool q4 = (w8 & 1) != 0;           // query side at level 4   (wave-uniform)
    const bool q8 = (w8 & 2) != 0;           //                level 8
    const bool q16 = (w8 & 4) != 0;          //                level 16; level 32's side is `hi`
    const int l16 = lane & 15;
    const int g4 = lane >> 4;

    const float u0 = a.u[h * kHeadSize + 2 * cp];
    const float u1 = a.u[h * kHeadSize + 2 * cp + 1];

    Streams st;
    st.r = static_cast<const char*>(a.r) + unit_base * 2;
    st.k = static_cast<const char*>(a.k) + unit_base * 2;
    st.v = static_cast<const char*>(a.v) + unit_base * 2;
    st.x = static_cast<const char*>(a.x) + unit_base * 2;
    st.row_bytes = tok_stride * 2;
    st.span_bytes = static_cast<long long>(a.T - 1) * st.row_bytes + kHeadSize * 2;
    int voff[4];                                   // byte offsets of this thread's 4 token rows
#pragma unroll
    for (int s = 0; s < 4; ++s)
        voff[s] = static_cast<int>((4 * tg + s) * st.row_bytes + 4 * cp);

    // score blocks above the diagonal that the A.V product still touches stay zero for good:
    // (t-block 0, i-block 1) and (t-block 2, i-block 3), 16x16 halfs each = 128 dwords
    if (tid < 256) {
        const int blk = tid >> 7;
        const int e = tid & 127;
        const int row = (blk ? 32 : 0) + (e >> 3);
        const int col = (blk ? 48 : 16) + 2 * (e & 7);
        lds_write_u32(lds, kAT + (row * kRowHalfs + col) * 2, 0u);
    }

    // column (in halfs) of this channel pair in the permuted r*W(t,-1) tile: slot order matches
    // the state accumulator registers that serve as the B operand of the inter-chunk read
    const int n0 = 2 * cp;
    const int m5 = n0 & 31;
    const int rt_col = (n0 & 32) + 8 * ((m5 >> 2) & 3) + 4 * (m5 >> 4) + (m5 & 3);

    Raw cur;
    load_rows(cur, st, 0, voff);

    for (int c = 0; c <= nchunks; ++c) {
        const bool live = c < nchunks;
        const int c0 = c * kChunk;
        float rp[2][4], ks[2][4];                    // r * prefix, k * suffix inside the group

        if (live) {
            if (c0 + kChunk > a.T) {
                // last, partial chunk: tokens past the end were read as zeros; give them w = 1
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    if (c0 + 4 * tg + s >= a.T) cur.x[s] = 0xff80ff80u;      // bf16 -inf, twice
            }
            // ---- window 1: everything that needs no other group's decays
            float w[2][4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                w[0][s] = decay_of(bf16_lo(cur.x[s]));
                w[1][s] = decay_of(bf16_hi(cur.x[s]));
            }
            float gtot[2];
            half4 vt[2];
#pragma unroll
            for (int ch = 0; ch < 2; ++ch) {
                const float p2 = w[ch][0] * w[ch][1];            // prefix of token 2
                const float p3 = p2 * w[ch][2];                  // prefix of token 3
                const float s1 = w[ch][2] * w[ch][3];            // suffix of token 1
                const float s0 = w[ch][1] * s1;                  // suffix of token 0
                gtot[ch] = p3 * w[ch][3];
                float r4[4], k4[4];
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    r4[s] = ch ? bf16_hi(cur.r[s]) : bf16_lo(cur.r[s]);
                    k4[s] = ch ? bf16_hi(cur.k[s]) : bf16_lo(cur.k[s]);
                    vt[ch][s] = static_cast<_Float16>(ch ? bf16_hi(cur.v[s]) : bf16_lo(cur.v[s]));
                }
                rp[ch][0] = r4[0];
                rp[ch][1] = r4[1] * w[ch][0];
                rp[ch][2] = r4[2] * p2;
                rp[ch][3] = r4[3] * p3;
                ks[ch][0] = k4[0] * s0;
                ks[ch][1] = k4[1] * s1;
                ks[ch][2] = k4[2] * w[ch][3];
                ks[ch][3] = k4[3];
            }
            *reinterpret_cast<float2*>(lds + kG + (tg * 64 + 2 * cp) * 4) = make_float2(gtot[0], gtot[1]);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float r0 = bf16_lo(cur.r[s]), r1 = bf16_hi(cur.r[s]);
                const float k0 = bf16_lo(cur.k[s]), k1 = bf16_hi(cur.k[s]);
                const int nat = ((4 * tg + s) * kRowHalfs + 2 * cp) * 2;      // natural channel order
                // level 4: the even group of an 8-block holds keys, the odd one queries
                lds_write_u32(lds, kZ4 + nat, q4 ? pack_h2(rp[0][s], rp[1][s]) : pack_h2(ks[0][s], ks[1][s]));
                {   // level 2: tokens 0,1 of the group are keys, 2,3 queries
                    float f0, f1;
                    if (s == 0)      { f0 = k0 * w[0][1]; f1 = k1 * w[1][1]; }
                    else if (s == 1) { f0 = k0;           f1 = k1; }
                    else if (s == 2) { f0 = r0;           f1 = r1; }
                    else             { f0 = r0 * w[0][2]; f1 = r1 * w[1][2]; }
                    lds_write_u32(lds, kZ2 + nat, pack_h2(f0, f1));
                }
                lds_write_u32(lds, kRH + nat, pack_h2(r0, r1));      // level 1 and bonus operands
                lds_write_u32(lds, kKH + nat, pack_h2(k0, k1));
                lds_write_u32(lds, kRU + nat, pack_h2(r0 * u0, r1 * u1));
            }
#pragma unroll
            for (int ch = 0; ch < 2; ++ch)
                *reinterpret_cast<half4*>(lds + kVT + ((2 * cp + ch) * kRowHalfs + 4 * tg) * 2) = vt[ch];
            // this chunk's raw inputs are consumed: fetch the next chunk into the same registers;
            // the loads stay in flight through windows 2 and 3
            if (c + 1 < nchunks) load_rows(cur, st, c0 + kChunk, voff);
        }
        __syncthreads();                                                        // barrier A

        if (live) {
            // ---- window 2: multipliers from the other groups' totals, then the remaining tiles
            float m_rt[2], m_kt[2], m32[2], m16[2], m8[2];
            {
                float2 own[8], oth[8];
#pragma unroll
                for (int g = 0; g < 8; ++g) {
                    own[g] = *reinterpret_cast<const float2*>(lds + kG + ((8 * hi + g) * 64 + 2 * cp) * 4);
                    oth[g] = *reinterpret_cast<const float2*>(lds + kG + ((8 * (1 - hi) + g) * 64 + 2 * cp) * 4);
                }
#pragma unroll
                for (int ch = 0; ch < 2; ++ch) {
                    float o[8], q[8];
#pragma unroll
                    for (int g = 0; g < 8; ++g) {
                        o[g] = ch ? own[g].y : own[g].x;
                        q[g] = ch ? oth[g].y : oth[g].x;
                    }
                    const float h_oth = ((q[0] * q[1]) * (q[2] * q[3])) * ((q[4] * q[5]) * (q[6] * q[7]));
                    // products of the groups before (a_lo) / after (a_hi) this one inside its half,
                    // and the level-16 / level-8 multipliers; w8 is wave-uniform
                    float a_lo, a_hi, f16, f8;
                    switch (w8) {
                        case 0:  f8 = o[1]; f16 = o[1] * (o[2] * o[3]); a_lo = 1.f;
                                 a_hi = f16 * ((o[4] * o[5]) * (o[6] * o[7])); break;
                        case 1:  f8 = 1.f; f16 = o[2] * o[3]; a_lo = o[0];
                                 a_hi = f16 * ((o[4] * o[5]) * (o[6] * o[7])); break;
                        case 2:  f8 = 1.f; f16 = o[3]; a_lo = o[0] * o[1];
                                 a_hi = f16 * ((o[4] * o[5]) * (o[6] * o[7])); break;
                        case 3:  f8 = o[2]; f16 = 1.f; a_lo = (o[0] * o[1]) * o[2];
                                 a_hi = (o[4] * o[5]) * (o[6] * o[7]); break;
                        case 4:  f8 = o[5]; f16 = 1.f; a_lo = (o[0] * o[1]) * (o[2] * o[3]);
                                 a_hi = o[5] * (o[6] * o[7]); break;
                        case 5:  f8 = 1.f; f16 = o[4]; a_lo = ((o[0] * o[1]) * (o[2] * o[3])) * o[4];
                                 a_hi = o[6] * o[7]; break;
                        case 6:  f8 = 1.f; f16 = o[4] * o[5]; a_lo = ((o[0] * o[1]) * (o[2] * o[3])) * f16;
                                 a_hi = o[7]; break;
                        default: f8 = o[6]; f16 = (o[4] * o[5]) * o[6]; a_lo = ((o[0] * o[1]) * (o[2] * o[3])) * f16;
                                 a_hi = 1.f; break;
                    }
                    float mine = o[0];
#pragma unroll
                    for (int g = 1; g < 8; ++g) mine = (g == w8) ? o[g] : mine;
                    m_rt[ch] = hi ? h_oth * a_lo : a_lo;       // tokens before this group in the chunk
                    m_kt[ch] = hi ? a_hi : a_hi * h_oth;       // tokens after this group in the chunk
                    m32[ch] = hi ? a_lo : a_hi;
                    m16[ch] = f16;
                    m8[ch] = f8;
                    if (tg == 0) *reinterpret_cast<float*>(lds + kD + (2 * cp + ch) * 4) = (a_lo * mine * a_hi) * h_oth;
                }
            }
            half4 kt[2];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int row = 4 * tg + s;
                const int nat = (row * kRowHalfs + 2 * cp) * 2;
                lds_write_u32(lds, kRT + (row * kRowHalfs + rt_col) * 2, pack_h2(rp[0][s] * m_rt[0], rp[1][s] * m_rt[1]));
                {
                    const float a0 = hi ? rp[0][s] : ks[0][s], a1 = hi ? rp[1][s] : ks[1][s];
                    lds_write_u32(lds, kZ32 + nat, pack_h2(a0 * m32[0], a1 * m32[1]));
                }
                {
                    const float a0 = q16 ? rp[0][s] : ks[0][s], a1 = q16 ? rp[1][s] : ks[1][s];
                    lds_write_u32(lds, kZ16 + nat, pack_h2(a0 * m16[0], a1 * m16[1]));
                }
                {
                    const float a0 = q8 ? rp[0][s] : ks[0][s], a1 = q8 ? rp[1][s] : ks[1][s];
                    lds_write_u32(lds, kZ8 + nat, pack_h2(a0 * m8[0], a1 * m8[1]));
                }
                kt[0][s] = static_cast<_Float16>(ks[0][s] * m_kt[0]);
                kt[1][s] = static_cast<_Float16>(ks[1][s] * m_kt[1]);
            }
#pragma unroll
            for (int ch = 0; ch < 2; ++ch)
                *reinterpret_cast<half4*>(lds + kKT + ((2 * cp + ch) * kRowHalfs + 4 * tg) * 2) = kt[ch];
        }
        __syncthreads();                                                        // barrier B

        if (live) {
            // ---- window 3: scores.  Waves 0..3: diagonal 16x16 block w8; waves 4..6: off-diagonal
            if (w8 < 4) {
                const int rowq = (16 * w8 + l16) * kRowHalfs * 2 + 16 * g4;     // + 64*kk bytes
                float4v acc8{0.f, 0.f, 0.f, 0.f}, acc4 = acc8, acc2 = acc8, acc1 = acc8, accb = acc8;
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const half8 z8 = lds_read_h8(lds, kZ8 + rowq + 64 * kk);
                    const half8 z4 = lds_read_h8(lds, kZ4 + rowq + 64 * kk);
                    const half8 z2 = lds_read_h8(lds, kZ2 + rowq + 64 * kk);
                    const half8 rh = lds_read_h8(lds, kRH + rowq + 64 * kk);
                    const half8 kh = lds_read_h8(lds, kKH + rowq + 64 * kk);
                    const half8 ru = lds_read_h8(lds, kRU + rowq + 64 * kk);
                    acc8 = mfma(z8, z8, acc8);
                    acc4 = mfma(z4, z4, acc4);
                    acc2 = mfma(z2, z2, acc2);
                    acc1 = mfma(kh, rh, acc1);
                    accb = mfma(kh, ru, accb);
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
                *reinterpret_cast<uint2*>(lds + kAT + ((16 * w8 + l16) * kRowHalfs + 16 * w8 + 4 * g4) * 2) =
                    make_uint2(pack_h2(sel[0], sel[1]), pack_h2(sel[2], sel[3]));
            } else if (w8 < 7) {
                // wave 4: level 16, blocks (t-block 1, i-block 0) and (3, 2)
                // wave 5: level 32, blocks (2, 0) and (2, 1);  wave 6: level 32, blocks (3, 0) and (3, 1)
                const int tile = (w8 == 4) ? kZ16 : kZ32;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int tb = (w8 == 4) ? (half ? 3 : 1) : (w8 == 5 ? 2 : 3);
                    const int ib = (w8 == 4) ? (half ? 2 : 0) : half;
                    const int rowq = (16 * tb + l16) * kRowHalfs * 2 + 16 * g4;
                    const int rowk = (16 * ib + l16) * kRowHalfs * 2 + 16 * g4;
                    float4v acc{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        const half8 zq = lds_read_h8(lds, tile + rowq + 64 * kk);
                        const half8 zk = lds_read_h8(lds, tile + rowk + 64 * kk);
                        acc = mfma(zk, zq, acc);
                    }
                    *reinterpret_cast<uint2*>(lds + kAT + ((16 * tb + l16) * kRowHalfs + 16 * ib + 4 * g4) * 2) =
                        make_uint2(pack_h2(acc[0], acc[1]), pack_h2(acc[2], acc[3]));
                }
            }
        }
        if (c > 0) {
            // ---- the previous chunk's finished output tile: full 128-byte (bf16) rows to HBM
            const int row = tid >> 3;
            const int col = 8 * (tid & 7);
            const int t = c0 - kChunk + row;
            if (t < a.T) {
                const long long e = unit_base + static_cast<long long>(t) * tok_stride + col;
                if constexpr (kOutF32) {
                    const float4* src = reinterpret_cast<const float4*>(lds + kO + (row * kORowF32 + col) * 4);
                    float4* dst = reinterpret_cast<float4*>(static_cast<float*>(a.out) + e);
                    const float4 q0 = src[0], q1 = src[1];
                    dst[0] = q0;
                    dst[1] = q1;
                } else {
                    const uint4 q = *reinterpret_cast<const uint4*>(lds + kO + (row * kORowBf16 + col) * 2);
                    *reinterpret_cast<uint4*>(static_cast<unsigned short*>(a.out) + e) = q;
                }
            }
        }
        __syncthreads();                                                        // barrier C
    }
}

// ------------------------------------------------------------------------------------------
// Consumer waves
// ------------------------------------------------------------------------------------------
template <bool kOutF32>
__device__ __forceinline__ void consumer(const Args& a, char* lds, int lane, int cw, int unit, int nchunks) {
    const int l16 = lane & 15;
    const int g4 = lane >> 4;
    const int j = 16 * cw + l16;            // value column of this lane
    // the consumers carry the only sequential chain: let the SIMD arbiter prefer them
    __builtin_amdgcn_s_setprio(3);

    // S[nb][e] = state[n = 16nb + 4g4 + e][j]
    float4v S[4];
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

    for (int c = 0; c <= nchunks; ++c) {
        const bool live = c < nchunks;
        __syncthreads();                                                        // barrier A
        __syncthreads();                                                        // barrier B
        float4v o[4];
        half8 vt[2];
        if (live) {
            // inter-chunk read: o[t][j] = sum_n (r_t W(t,-1))[n] S0[n][j]; the state registers,
            // rounded to fp16, are the B operand (k-slot order = the r tile's column permutation)
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
                    o[tb] = mfma(rt, sh[kk], o[tb]);
                }
            }
            // state update: S = diag(W(64,-1)) S + (k W(64,i))^T V
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
                vt[kk] = lds_read_h8(lds, kVT + ((16 * cw + l16) * kRowHalfs + 32 * kk + 8 * g4) * 2);
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
                    S[nb] = mfma(kt, vt[kk], S[nb]);
                }
            }
        }
        __syncthreads();                                                        // barrier C: scores visible
        if (live) {
            // intra-chunk: o += A V, then stage the tile for the producers' row stores
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) {
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    if (kk == 1 && tb < 2) continue;        // keys 32..63 are never visible to t < 32
                    const half8 at = lds_read_h8(lds, kAT + ((16 * tb + l16) * kRowHalfs + 32 * kk + 8 * g4) * 2);
                    o[tb] = mfma(at, vt[kk], o[tb]);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = 16 * tb + 4 * g4 + e;
                    if constexpr (kOutF32)
                        *reinterpret_cast<float*>(lds + kO + (row * kORowF32 + j) * 4) = o[tb][e];
                    else
                        *reinterpret_cast<unsigned short*>(lds + kO + (row * kORowBf16 + j) * 2) = bf16_bits(o[tb][e]);
                }
            }
        }
    }

    if (a.state_out) {
        float* so = a.state_out + static_cast<long long>(unit) * 4096;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int e = 0; e < 4; ++e) so[(16 * nb + 4 * g4 + e) * 64 + j] = S[nb][e];
    }
}

template <bool kOutF32>
__global__ __launch_bounds__(kThreads) void chunked_kernel(Args a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x;
    const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int unit = blockIdx.x;
    const int b = unit / a.H;
    const int h = unit - b * a.H;
    const long long tok_stride = static_cast<long long>(a.H) * kHeadSize;
    const long long unit_base = static_cast<long long>(b) * a.batch_stride +
                                static_cast<long long>(h) * kHeadSize;
    const int nchunks = (a.T + kChunk - 1) / kChunk;
    if (wid < kProducerWaves)
        producer<kOutF32>(a, lds, tid, wid, unit, h, unit_base, tok_stride, nchunks);
    else
        consumer<kOutF32>(a, lds, tid & 63, wid - kProducerWaves, unit, nchunks);
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

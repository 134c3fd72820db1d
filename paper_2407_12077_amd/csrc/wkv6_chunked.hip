// Chunked WKV6 prefill kernel for gfx950 (MI355X): one workgroup per (batch, head) -- or, with
// more units than compute units, several units back to back per workgroup -- fp32 state
// carried in MFMA accumulators, every dense contraction on the matrix cores
// (v_mfma_f32_16x16x32_f16, fp32 accumulation).
//
// The recurrence (Finch-C2 Time Mixing: decay map w = exp(-exp(x)), wkv_t, read-out; Finch
// bonus u) is evaluated in chunks of 32 tokens.  With tokens 0..31 of a chunk, S0 the state
// entering it, and W(t,i) = prod_{s=i+1}^{t-1} w_s (a per-key-channel vector, empty product = 1):
//
//   o_t = (r_t * W(t,-1)) . S0                                   inter-chunk read
//       + sum_{i<t} ( sum_n r_t[n] k_i[n] W(t,i)[n] ) v_i        intra-chunk, strictly causal
//       + ( sum_n r_t[n] u[n] k_t[n] ) v_t                       bonus on the diagonal
//   S32 = diag(W(32,-1)) S0 + sum_i (k_i * W(32,i))^T v_i        state update
//
// Only PRODUCTS of decays are ever formed (never a reciprocal or a positive exponent), so
// every scale factor is <= 1 and any decay logit, +-inf included, is handled exactly.  To
// write W(t,i) as (factor of t) x (factor of i) the causal triangle is cut by binary
// levels m = 16,8,4,2,1: the pair (t,i) belongs to the level of the highest bit in which
// t and i differ; there i lies in the first half and t in the second half of the same
// 2m-aligned block, and with `mid` that block's midpoint
//       W(t,i) = (prod_{s=mid}^{t-1} w_s) * (prod_{s=i+1}^{mid-1} w_s),
// a prefix product inside t's m-block times a suffix product inside i's m-block.  Tile Z_m
// holds, row by row, the scaled key (rows in a first half) or the scaled receptance (rows in
// a second half); one MFMA per level and 16x16 block followed by a select assembles the
// score matrix.
//
// Work split inside the workgroup (16 wavefronts, 4 per SIMD), one barrier per window:
//   waves 0..11  three PRODUCER groups of four waves; group g owns the chunks c = g (mod 3) and
//               spends three windows on each: D (decays, products inside 4-token groups, HBM
//               loads six chunks ahead), T (multipliers from all groups' totals, every fp16
//               operand tile), S (score MFMAs, finished output rows of chunk c-2 to HBM).  The
//               groups run one window apart, so every window has one group in each phase and
//               vector-ALU, LDS and matrix-core work of different chunks overlap.
//   waves 12..15 CONSUMERS: each owns 16 value columns of the state and runs the three
//               state-dependent contractions, the only sequential chain of the method.
// In window n: D(chunk n), T(n-1), S(n-2), consumers' state chain on chunk n-2 and A.V on n-3.
// LDS buffers (tiles, scores, decay totals, output staging) are indexed by chunk parity.
//
// Finch-C2 form (template flag): the key is multiplied by (1 - w) in phase D, u does not enter
// the level-1 tiles, the diagonal of the scores is zero, and the second value u' is added to the
// fp32-staged rows before the store.
//
// Modes (template parameter kMode): 0 bf16 output, 1 fp32 output, 2 state only (no r, no scores,
// no output: final state and total decay of the unit, for the token split), 3 bf16 output plus
// the per-head partial sums of the LayerNorm over all heads (Finch-C2 output equation) taken in
// the store phase, 4 bf16 output with the decay logits formed in the kernel from the low-rank
// decay path (d = lambda + y B, consumers' MFMAs, handed to phase D through LDS) instead of
// read as x, 5 both.
//
// LDS tiles whose contraction index is the channel (scores, inter-chunk read) are [token][channel]
// fp16 with a 160-byte row stride; the two tiles whose contraction index is the token (k^T V, A V:
// scaled keys and values) are stored transposed, [channel][token] with a 96-byte row stride and
// the 16-byte granules of a row XOR-swizzled by two row bits.  With these layouts every MFMA
// operand is one 16-byte row read at the full rate of the gfx950 LDS (measured 254 B/clk), and a
// producer thread, which owns four consecutive tokens of a channel pair, writes a transposed
// tile with two 8-byte stores instead of four 4-byte ones (LDS stores cost about 4 clk per
// instruction up to 4 bytes per lane and 6-8 clk for 8 bytes: the kernel is bound by the LDS
// pipeline, and stores are its slow half).  The output tile is produced transposed by swapping
// the operands of the consumers' MFMAs, so that a lane holds four consecutive value channels of
// one token and stages them with one store.
#include "wkv6_launch.h"
#include "wkv6_windows.h"

#include <type_traits>

namespace wkv6 {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kChunk = 32;                 // tokens per chunk
constexpr int kProducerGroups = kWindowGroups;   // 4 waves each
constexpr int kThreads = 64 * (4 * kProducerGroups + 4);
constexpr int kRow = 160;                  // fp16 tile row stride in bytes (64 halfs + 16 pad)
constexpr int kTile = kChunk * kRow;       // one [32 tokens][64 channels] tile
constexpr int kRowT = 96;                  // transposed tile [channel][32 tokens]: 64 B + 32 pad
constexpr int kTileT = 64 * kRowT;
constexpr int kORowF32 = 68;               // output staging row stride, fp32 mode (floats)
constexpr int kORowBf16 = 72;              // output staging row stride, bf16 mode (halfs)

// LDS map (bytes).  Everything up to kBuf exists twice, once per chunk parity.
enum : int {
    kZ16 = 0 * kTile,
    kZ8 = 1 * kTile,
    kZ4 = 2 * kTile,
    kZ2 = 3 * kTile,
    kQ1 = 4 * kTile,       // level 1 and bonus, query side: r (odd tokens), r*u (even tokens)
    kK1 = 5 * kTile,       // level 1 and bonus, key side:   k (even tokens), k*u (odd tokens)
    kRT = 6 * kTile,       // r * W(t,-1), channel order permuted to match the state registers
    kKT = 7 * kTile,       // k * W(32,i), transposed: [key channel][token]
    kVT = kKT + kTileT,    // v as fp16, transposed: [value channel][token]
    kA0 = kVT + kTileT,    // scores A[t][i], contraction over channels 0..31
    kA1 = kA0 + kTile,     // scores A[t][i], contraction over channels 32..63
    kG = kA1 + kTile,                      // per 4-token group decay products [8][64] fp32
    kD = kG + 8 * 64 * 4,                  // whole-chunk decay product [64] fp32
    kO = kD + 64 * 4,                      // output staging [32 tokens][64]
    kBuf = (kO + kChunk * kORowF32 * 4 + 1023) / 1024 * 1024,
    kLdsBytes = 2 * kBuf
};
static_assert(kBuf % 16 == 0 && kLdsBytes <= 160 * 1024, "LDS budget");

// Fused decay path only: the chunk's decay logits d[channel pair][parity][token] in fp32, written
// by the consumers and read by the producers' phase D, one buffer per chunk parity after the
// two main buffers.  272 bytes per channel pair (2 x 32 tokens x 4 + 16 pad): the 16-byte
// accesses of 16 neighbouring lanes, a channel pair apart, cover all banks once.
constexpr int kDxPair = 2 * kChunk * 4 + 16;
constexpr int kDxBuf = 32 * kDxPair;
constexpr int kDx = kLdsBytes;
constexpr int kLdsBytesLora = kLdsBytes + 2 * kDxBuf;
static_assert(kLdsBytesLora <= 160 * 1024, "LDS budget");

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float bf16_lo(unsigned bits) { return __uint_as_float(bits << 16); }
__device__ __forceinline__ float bf16_hi(unsigned bits) { return __uint_as_float(bits & 0xffff0000u); }

__device__ __forceinline__ unsigned pack_h2(float a, float b) {
    half2v p;
    p.x = static_cast<_Float16>(a);
    p.y = static_cast<_Float16>(b);
    return __builtin_bit_cast(unsigned, p);
}

// packed fp16 multiply of two channel pairs
__device__ __forceinline__ unsigned mul_h2(unsigned a, unsigned b) {
    return __builtin_bit_cast(unsigned, __builtin_bit_cast(half2v, a) * __builtin_bit_cast(half2v, b));
}

// two floats to a bf16 pair (round to nearest even), one packed conversion
__device__ __forceinline__ unsigned pack_bf2(float a, float b) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float float2v __attribute__((ext_vector_type(2)));
    const float2v f = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}

// w = exp(-exp(x)) through two base-2 exponentials (x=-inf -> 1, x=+inf -> 0):
// log2(e) * exp(x) = exp2(x * log2(e) + log2(log2(e))), so the factor of the second exponential
// rides in the argument of the first.
// Also hands back the scaled inner exponential log2(e) * exp(x), which the Finch-C2 key factor needs.
__device__ __forceinline__ float decay_of(float x, float& e_log2e) {
    constexpr float kLog2Log2e = 0.5287663729448977f;
    e_log2e = __builtin_amdgcn_exp2f(__builtin_fmaf(x, kLog2e, kLog2Log2e));
    return __builtin_amdgcn_exp2f(-e_log2e);
}

// Finch-C2 key factor 1 - w = 1 - exp(-e), e = exp(x), without the cancellation of the plain
// subtraction for long-memory channels (w close to 1): below e = 2^-5 the alternating series
// e (1 - e/2 + e^2/6 - e^3/24), whose first dropped term is under 1e-8 of the result there;
// above it the subtraction loses at most five bits of an fp32 value.
__device__ __forceinline__ float one_minus_decay(float e_log2e, float w) {
    const float e = e_log2e * 0.6931471805599453f;      // exp(x) from the decay's own inner exponential
    const float series = e * __builtin_fmaf(e, __builtin_fmaf(e, __builtin_fmaf(e, -1.f / 24.f, 1.f / 6.f), -0.5f), 1.f);
    return e < 0.03125f ? series : 1.f - w;
}

__device__ __forceinline__ half8 lds_read_h8(const char* lds, int byte_off) {
    return *reinterpret_cast<const half8*>(lds + byte_off);
}
__device__ __forceinline__ void lds_write_u32(char* lds, int byte_off, unsigned val) {
    *reinterpret_cast<unsigned*>(lds + byte_off) = val;
}

// Byte offset, inside a transposed tile, of the 16-byte granule `granule` (tokens 8*granule .. +7)
// of row `row` (a channel).  The XOR with two row bits makes the producers' 8-byte stores (32
// lanes on 32 different rows, two lanes per granule) and the consumers' 16-byte reads (16
// consecutive rows) both run without bank conflicts beyond the store pipeline's own rate.
__device__ __forceinline__ int tile_t_off(int row, int granule) {
    return row * kRowT + ((granule ^ ((row >> 2) & 3)) << 4);
}
// Score tiles A[t][i] (rows of 64 bytes, stride kRow): granule `granule` (keys 8*granule .. +7) of
// token row t, swizzled by one row bit for the 8-byte score stores.
__device__ __forceinline__ int score_off(int t, int granule) {
    return t * kRow + ((granule ^ ((t >> 2) & 1)) << 4);
}
__device__ __forceinline__ void lds_write_u64(char* lds, int byte_off, unsigned lo, unsigned hi) {
    *reinterpret_cast<uint2*>(lds + byte_off) = make_uint2(lo, hi);
}
// low halves / high halves of two packed fp16 pairs as one pair
__device__ __forceinline__ unsigned lo_halves(unsigned a, unsigned b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ unsigned hi_halves(unsigned a, unsigned b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

__device__ __forceinline__ float4v mfma(half8 a, half8 b, float4v c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Cache policy of the streams that are touched exactly once (r, k, v, x, u', out): the
// non-temporal bit, so they do not displace each other in the caches on their way through.
constexpr int kStreamOnce = 2;
// Cache policy of the output rows: scope bit sc1 without the non-temporal bit, i.e. written
// through the XCD's L2 as they are produced instead of lingering there as dirty lines.  Measured
// with a streaming probe of this layout (four non-temporal input streams, one output stream of
// 128-byte rows 4 KiB apart): 130.7 us against 135.8 us with non-temporal stores.
constexpr int kStoreThrough = 16;

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

__device__ __forceinline__ __amdgpu_buffer_rsrc_t chunk_rsrc(const char* base, long long off,
                                                           long long span_bytes) {
    long long left = span_bytes - off;
    if (left < 0) left = 0;
    if (left > 0x7fffffffLL) left = 0x7fffffffLL;
    // raw buffer (stride 0), 32-bit data format
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base + off), 0,
                                             static_cast<int>(left), 0x00020000);
}

// A chunk's loads are issued in two halves (x and r; k and v) so that two different phases can
// share the cost of issuing them.
// kPolicy: the cache policy of the loads.  Every mode streams (kStreamOnce), the state-only pass of the
// token split included: running that split block by block with cached loads in its first pass, so that
// the second read of k, v, x could come from the last-level cache, was measured and dropped (config 3:
// 0.91 ms unblocked with cached first-pass loads, 0.90 to 1.10 ms in 4 to 16 blocks, against 0.78 ms
// with streaming loads and one block; the byte counters of the L2, which cannot tell that cache from
// HBM, did not move).
template <bool kSkipR, bool kSkipX, int kPolicy>
__device__ __forceinline__ void load_rows_xr(Raw& d, const Streams& st, long long unit_bytes, int t0,
                                             const int (&voff)[4]) {
    const long long off = static_cast<long long>(t0) * st.row_bytes;       // uniform
    if constexpr (!kSkipX) {
        const __amdgpu_buffer_rsrc_t rx = chunk_rsrc(st.x + unit_bytes, off, st.span_bytes);
#pragma unroll
        for (int s = 0; s < 4; ++s) d.x[s] = __builtin_amdgcn_raw_buffer_load_b32(rx, voff[s], 0, kPolicy);
    } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) d.x[s] = 0u;
    }
    if constexpr (!kSkipR) {
        const __amdgpu_buffer_rsrc_t rr = chunk_rsrc(st.r + unit_bytes, off, st.span_bytes);
#pragma unroll
        for (int s = 0; s < 4; ++s) d.r[s] = __builtin_amdgcn_raw_buffer_load_b32(rr, voff[s], 0, kPolicy);
    } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) d.r[s] = 0u;
    }
}

template <int kPolicy>
__device__ __forceinline__ void load_rows_kv(Raw& d, const Streams& st, long long unit_bytes, int t0,
                                             const int (&voff)[4]) {
    const long long off = static_cast<long long>(t0) * st.row_bytes;       // uniform
    const __amdgpu_buffer_rsrc_t rk = chunk_rsrc(st.k + unit_bytes, off, st.span_bytes);
    const __amdgpu_buffer_rsrc_t rv = chunk_rsrc(st.v + unit_bytes, off, st.span_bytes);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        d.k[s] = __builtin_amdgcn_raw_buffer_load_b32(rk, voff[s], 0, kPolicy);
        d.v[s] = __builtin_amdgcn_raw_buffer_load_b32(rv, voff[s], 0, kPolicy);
    }
}

// The units (batch, head) of one workgroup.  A workgroup keeps its pipeline running across unit
// boundaries: its chunks form one sequence, unit after unit, and only the state (consumers) and
// the base addresses change at a boundary, so short sequences do not pay the fill and drain of
// the pipeline once per unit.  All units of a workgroup share the head (the stride between them
// is a multiple of H), have the same length T, and lie `step` elements apart.
struct Units {
    int first;            // unit index of the first one: selects state_in / state_out / decay_out
    int stride;           // unit index stride
    int count;            // how many
    int nchunks;          // chunks per unit
    long long base0;      // element offset of the first unit's token 0 in r,k,v,x,out
    long long step;       // element offset between consecutive units of this workgroup
    float* state_out;     // where final states go, indexed like state_in (nullptr: not written)
};

// Sum over the 8 lanes of an aligned group of 8 (every lane gets the total): neighbours, pairs,
// then the mirrored half-row, all as data-parallel-primitive moves inside the vector ALU.
template <int kCtrl>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xf, 0xf, false));
}
__device__ __forceinline__ float row8_sum(float v) {
    v += dpp_move<0xB1>(v);       // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);       // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);      // row_half_mirror: lane i <-> 7 - i of each 8
    return v;
}

// Position in the workgroup's chunk sequence: unit ui, chunk c of it.  Advanced without
// divisions; c < 0 (before the start) and ui >= count (past the end) mean "no chunk".
// With a single unit per workgroup (kMulti false) ui stays 0 and "past the end" is c >= nchunks.
template <bool kMulti>
struct Cursor {
    int ui, c;
    __device__ __forceinline__ void advance(int by, int nchunks) {
        c += by;
        if constexpr (kMulti) {
            while (c >= nchunks) {
                c -= nchunks;
                ++ui;
            }
        }
    }
    __device__ __forceinline__ bool live(const Units& un) const {
        if constexpr (kMulti) return ui < un.count;
        return c < un.nchunks;
    }
    __device__ __forceinline__ long long unit_elems(const Units& un) const {
        if constexpr (kMulti) return ui * un.step;
        return 0;
    }
};

// What a producer thread carries from phase D (where it digests the raw inputs of its chunk)
// to phase T (where the other groups' decay totals are known and the tiles are written).
struct Prep {
    unsigned z2[4], q1[4], k1[4];                         // finished fp16 pairs (two channels), one per token
    unsigned vt[4];            // v as fp16 pairs of consecutive tokens: [2*channel + token pair]
    unsigned rp[4];            // r * prefix product inside the group, fp16 pair (2 channels)
    unsigned ks[4];            // k * suffix product inside the group, fp16 pair
};

// ------------------------------------------------------------------------------------------
// Producer waves: group pg (0..2) = chunk index mod 3, wq = wave inside the group
// ------------------------------------------------------------------------------------------
template <int kMode, bool kC2, bool kMulti>
__device__ __forceinline__ void producer(const Args& a, char* lds_all, int tid, int pg, int wq, int h,
                                         const Units& un, long long tok_stride, int T) {
    constexpr bool kOutF32 = kMode == 1;
    constexpr bool kStateOnly = kMode == 2;
    constexpr bool kMoments = kMode == 3 || kMode == 5;   // bf16 out plus the per-head LayerNorm partials
    constexpr bool kLora = kMode >= 4;           // decay logits from the consumers (LDS), not from x
    constexpr bool kStageF32 = kOutF32 || kC2;   // staging precision of the finished rows
    const int lane = tid & 63;
    const int gtid = tid & 255;              // thread inside the group
    const int cp = lane & 31;                // channel pair: channels 2cp, 2cp+1
    const int hl = lane >> 5;
    const int g8 = 2 * wq + hl;              // 4-token group 0..7 inside the chunk
    const bool q4 = hl != 0;                 // query side at level 4 (per lane half)
    const int l16 = lane & 15;
    const int g4 = lane >> 4;

    // the bonus u of this channel pair as an fp16 pair (Finch form only)
    const unsigned hu = kC2 ? 0u : pack_h2(a.u[h * kHeadSize + 2 * cp], a.u[h * kHeadSize + 2 * cp + 1]);

    Streams st;
    st.r = static_cast<const char*>(a.r) + un.base0 * 2;
    st.k = static_cast<const char*>(a.k) + un.base0 * 2;
    st.v = static_cast<const char*>(a.v) + un.base0 * 2;
    st.x = static_cast<const char*>(a.x) + un.base0 * 2;
    st.row_bytes = tok_stride * 2;
    st.span_bytes = static_cast<long long>(T - 1) * st.row_bytes + kHeadSize * 2;
    int voff[4];                                   // byte offsets of this thread's 4 token rows
#pragma unroll
    for (int s = 0; s < 4; ++s)
        voff[s] = static_cast<int>((4 * g8 + s) * st.row_bytes + 4 * cp);

    // the score block above the diagonal that the A.V product still touches, (t-block 0,
    // i-block 1), stays zero for good in both partial score tiles: 2 x 16x16 halfs = 256 dwords
    if (!kStateOnly && pg < 2) {
        char* lds = lds_all + pg * kBuf;
        const int which = gtid >> 7;                 // A0 / A1
        const int e = gtid & 127;                    // row = e>>3, column pair = e&7
        lds_write_u32(lds, (which ? kA1 : kA0) + (e >> 3) * kRow + (16 + 2 * (e & 7)) * 2, 0u);
    }

    // column (in halfs) of this channel pair in the permuted r*W(t,-1) tile: slot order matches
    // the state accumulator registers that serve as the B operand of the inter-chunk read
    const int n0 = 2 * cp;
    const int m5 = n0 & 31;
    const int rt_col = (n0 & 32) + 8 * ((m5 >> 2) & 3) + 4 * (m5 >> 4) + (m5 & 3);

    Raw raw_a, raw_b;      // raw inputs of this group's next two chunks (in flight or landed)
    Prep pr;

    // Phase D.  Digest the raw inputs in `cur` (chunk c): decays, their products inside
    // the thread's 4-token group (published in G), and every operand that needs nothing else.
    auto digest = [&](int g, int c, Raw& cur) {     // g: position in the sequence, c: chunk of its unit
        char* lds = lds_all + (g & 1) * kBuf;
        const int t0 = c * kChunk;
        if (t0 + kChunk > T) {
            // last, partial chunk: tokens past the end were read as zeros; give them w = 1
#pragma unroll
            for (int s = 0; s < 4; ++s)
                if (t0 + 4 * g8 + s >= T) cur.x[s] = 0xff80ff80u;      // bf16 -inf, twice
        }
        float w[2][4];
        [[maybe_unused]] float omw[2][4];       // Finch-C2: 1 - w
        if constexpr (kLora) {
            // the chunk's logits were left in LDS by the consumers one window ago: this thread's
            // 4 tokens of its two channels
            const char* dx = lds_all + kDx + (g & 1) * kDxBuf + cp * kDxPair + g8 * 16;
            const float4 de = *reinterpret_cast<const float4*>(dx);
            const float4 dq = *reinterpret_cast<const float4*>(dx + kChunk * 4);
            const float d0[4] = {de.x, de.y, de.z, de.w}, d1[4] = {dq.x, dq.y, dq.z, dq.w};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bool past = t0 + 4 * g8 + s >= T;          // tokens past the end: w = 1
                float e0 = 0.f, e1 = 0.f;
                const float w0 = decay_of(d0[s], e0), w1 = decay_of(d1[s], e1);
                w[0][s] = past ? 1.f : w0;
                w[1][s] = past ? 1.f : w1;
                if constexpr (kC2) {
                    omw[0][s] = one_minus_decay(e0, w0);               // past the end the key is zero
                    omw[1][s] = one_minus_decay(e1, w1);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                float e0 = 0.f, e1 = 0.f;
                w[0][s] = decay_of(bf16_lo(cur.x[s]), e0);
                w[1][s] = decay_of(bf16_hi(cur.x[s]), e1);
                if constexpr (kC2) {
                    omw[0][s] = one_minus_decay(e0, w[0][s]);
                    omw[1][s] = one_minus_decay(e1, w[1][s]);
                }
            }
        }
        // products of decays inside the group, fp32: prefix of token 2 and 3, suffix of token 1
        // and 0, and the group total
        float p2[2], p3[2], s1[2], s0[2];
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {
            p2[ch] = w[ch][0] * w[ch][1];
            p3[ch] = p2[ch] * w[ch][2];
            s1[ch] = w[ch][2] * w[ch][3];
            s0[ch] = w[ch][1] * s1[ch];
        }
        *reinterpret_cast<float2*>(lds + kG + (g8 * 64 + 2 * cp) * 4) =
            make_float2(p3[0] * w[0][3], p3[1] * w[1][3]);
        // r, k, v as fp16 channel pairs (exact: bf16 has fewer significant bits); every scaled
        // operand is one packed fp16 multiply with a multiplier rounded to fp16
        unsigned rh[4], kh[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            rh[s] = pack_h2(bf16_lo(cur.r[s]), bf16_hi(cur.r[s]));
            if constexpr (kC2)      // Finch-C2: k = kbar (1 - w), the factor applied in fp32
                kh[s] = pack_h2(bf16_lo(cur.k[s]) * omw[0][s], bf16_hi(cur.k[s]) * omw[1][s]);
            else
                kh[s] = pack_h2(bf16_lo(cur.k[s]), bf16_hi(cur.k[s]));
        }
        // v goes to a transposed tile: pairs of consecutive tokens of one channel
        pr.vt[0] = pack_h2(bf16_lo(cur.v[0]), bf16_lo(cur.v[1]));
        pr.vt[1] = pack_h2(bf16_lo(cur.v[2]), bf16_lo(cur.v[3]));
        pr.vt[2] = pack_h2(bf16_hi(cur.v[0]), bf16_hi(cur.v[1]));
        pr.vt[3] = pack_h2(bf16_hi(cur.v[2]), bf16_hi(cur.v[3]));
        pr.rp[0] = rh[0];
        pr.rp[1] = mul_h2(rh[1], pack_h2(w[0][0], w[1][0]));
        pr.rp[2] = mul_h2(rh[2], pack_h2(p2[0], p2[1]));
        pr.rp[3] = mul_h2(rh[3], pack_h2(p3[0], p3[1]));
        const unsigned hw3 = pack_h2(w[0][3], w[1][3]);
        pr.ks[0] = mul_h2(kh[0], pack_h2(s0[0], s0[1]));
        pr.ks[1] = mul_h2(kh[1], pack_h2(s1[0], s1[1]));
        pr.ks[2] = mul_h2(kh[2], hw3);
        pr.ks[3] = kh[3];
        // level 2: tokens 0,1 of the group are keys, 2,3 queries
        pr.z2[0] = mul_h2(kh[0], pack_h2(w[0][1], w[1][1]));
        pr.z2[1] = kh[1];
        pr.z2[2] = rh[2];
        pr.z2[3] = mul_h2(rh[3], pack_h2(w[0][2], w[1][2]));
        // level 1 (odd token t reads even token t-1, no decay between them) and the bonus on the
        // diagonal share one query tile and one key tile: u rides on the query for even tokens
        // and on the key for odd tokens, so the diagonal gets r.u.k and the pair gets plain r.k
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if constexpr (kC2) {
                // no diagonal term: one tile, keys in the even token rows, receptances in the odd ones
                pr.q1[s] = (s & 1) ? rh[s] : kh[s];
            } else {
                pr.q1[s] = (s & 1) ? rh[s] : mul_h2(rh[s], hu);
                pr.k1[s] = !(s & 1) ? kh[s] : mul_h2(kh[s], hu);
            }
        }
    };

    // Phase T: multipliers from the other groups' decay totals, then every operand tile.  (Writing
    // the four tiles that need no totals -- Z4, Z2, Q1, K1 -- a window earlier, in phase D, into a
    // slot per producer group was measured and dropped: the digest phase grew by what the tile
    // phase should have lost and the window did not get shorter; the compute unit's LDS queue, not
    // one phase's share of it, is what the window waits for.  Also measured and dropped: neighbouring
    // lanes trading two values so that each token-row tile takes two 8-byte stores instead of four
    // 4-byte ones -- 9 % slower in the kernel although 8-byte stores run at 85 against 62 B/clk in
    // isolation.)  The
    // body is instantiated per wave position kWq so that the level-8 and level-16 roles (key or
    // query side) and the neighbouring group products are compile-time choices.
    auto write_tiles_at = [&](auto wq_const, int c) {
        constexpr int kWq = decltype(wq_const)::value;
        constexpr bool kQ8 = (kWq & 1) != 0;     // query side at level 8
        constexpr bool kQ16 = (kWq & 2) != 0;    // query side at level 16
        char* lds = lds_all + (c & 1) * kBuf;
        float m_rt[2], m_kt[2], m16[2], m8[2];
        float2 own[8];
#pragma unroll
        for (int g = 0; g < 8; ++g)
            own[g] = *reinterpret_cast<const float2*>(lds + kG + (g * 64 + 2 * cp) * 4);
        // Writes are grouped by tile, the four tokens of a tile back to back, so that neighbouring
        // writes pair up into two-address LDS instructions.  The tiles that need no multiplier go
        // out first, right behind the reads of the group totals: at the start of a window every
        // wave of the workgroup queues LDS work, and the totals take hundreds of cycles to return.
        const int nat0 = 4 * g8 * kRow + 4 * cp;             // token 0 of the group, natural channel order
        auto put4 = [&](int tile, unsigned v0, unsigned v1, unsigned v2, unsigned v3) {
            lds_write_u32(lds, tile + nat0, v0);
            lds_write_u32(lds, tile + nat0 + kRow, v1);
            lds_write_u32(lds, tile + nat0 + 2 * kRow, v2);
            lds_write_u32(lds, tile + nat0 + 3 * kRow, v3);
        };
        // transposed tiles: this thread's 4 tokens of channel 2cp (and 2cp+1) are 8 contiguous bytes
        const int tr0 = tile_t_off(2 * cp, wq) + 8 * hl;          // tokens 4*g8 .. +3 = half hl of granule wq
        const int tr1 = tile_t_off(2 * cp + 1, wq) + 8 * hl;
        lds_write_u64(lds, kVT + tr0, pr.vt[0], pr.vt[1]);
        lds_write_u64(lds, kVT + tr1, pr.vt[2], pr.vt[3]);
        if constexpr (!kStateOnly) {
            // level 4: the even group of an 8-block holds keys, the odd one queries
            put4(kZ4, q4 ? pr.rp[0] : pr.ks[0], q4 ? pr.rp[1] : pr.ks[1], q4 ? pr.rp[2] : pr.ks[2],
                 q4 ? pr.rp[3] : pr.ks[3]);
            put4(kZ2, pr.z2[0], pr.z2[1], pr.z2[2], pr.z2[3]);
            put4(kQ1, pr.q1[0], pr.q1[1], pr.q1[2], pr.q1[3]);
            if constexpr (!kC2) put4(kK1, pr.k1[0], pr.k1[1], pr.k1[2], pr.k1[3]);
        }
        __builtin_amdgcn_sched_barrier(0);       // keep these writes ahead of the wait for the totals
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {
            float o[8];
#pragma unroll
            for (int g = 0; g < 8; ++g) o[g] = ch ? own[g].y : own[g].x;
            // pl / ph: decays of the group pairs before / after this wave's pair;
            // f16: this wave's share of the level-16 multiplier
            float pl, ph, f16;
            if constexpr (kWq == 0) { pl = 1.f; ph = (o[2] * o[3]) * ((o[4] * o[5]) * (o[6] * o[7])); f16 = o[2] * o[3]; }
            else if constexpr (kWq == 1) { pl = o[0] * o[1]; ph = (o[4] * o[5]) * (o[6] * o[7]); f16 = 1.f; }
            else if constexpr (kWq == 2) { pl = (o[0] * o[1]) * (o[2] * o[3]); ph = o[6] * o[7]; f16 = 1.f; }
            else { pl = ((o[0] * o[1]) * (o[2] * o[3])) * (o[4] * o[5]); ph = 1.f; f16 = o[4] * o[5]; }
            // the other group of this wave's pair lies before the odd group (hl=1) and after
            // the even one (hl=0)
            const float before = hl ? o[2 * kWq] : 1.f;
            const float after = hl ? 1.f : o[2 * kWq + 1];
            m_rt[ch] = pl * before;            // decays of the chunk's tokens before this group
            m_kt[ch] = after * ph;             // decays of the chunk's tokens after this group
            m16[ch] = kQ16 ? f16 * before : after * f16;   // level 16: inside the 16-token half
            m8[ch] = kQ8 ? before : after;                 // level 8: inside the 8-token block
            if constexpr (kWq == 0)
                if (hl == 0) *reinterpret_cast<float*>(lds + kD + (2 * cp + ch) * 4) = o[0] * m_kt[ch];
        }
        // the multipliers as fp16 channel pairs: one packed multiply per tile entry
        const unsigned h_rt = pack_h2(m_rt[0], m_rt[1]);
        const unsigned h_kt = pack_h2(m_kt[0], m_kt[1]);
        const unsigned h16 = pack_h2(m16[0], m16[1]);
        const unsigned h8 = pack_h2(m8[0], m8[1]);
        {
            const unsigned k0 = mul_h2(pr.ks[0], h_kt), k1 = mul_h2(pr.ks[1], h_kt);
            const unsigned k2 = mul_h2(pr.ks[2], h_kt), k3 = mul_h2(pr.ks[3], h_kt);
            lds_write_u64(lds, kKT + tr0, lo_halves(k0, k1), lo_halves(k2, k3));
            lds_write_u64(lds, kKT + tr1, hi_halves(k0, k1), hi_halves(k2, k3));
        }
        if constexpr (!kStateOnly) {
            const unsigned* z16 = kQ16 ? pr.rp : pr.ks;
            const unsigned* z8 = kQ8 ? pr.rp : pr.ks;
            put4(kZ16, mul_h2(z16[0], h16), mul_h2(z16[1], h16), mul_h2(z16[2], h16), mul_h2(z16[3], h16));
            put4(kZ8, mul_h2(z8[0], h8), mul_h2(z8[1], h8), mul_h2(z8[2], h8), mul_h2(z8[3], h8));
            put4(kRT + (rt_col - 2 * cp) * 2, mul_h2(pr.rp[0], h_rt), mul_h2(pr.rp[1], h_rt),
                 mul_h2(pr.rp[2], h_rt), mul_h2(pr.rp[3], h_rt));
        }
    };
    auto write_tiles = [&](int c) {
        switch (wq) {                             // wave-uniform
            case 0: write_tiles_at(std::integral_constant<int, 0>{}, c); break;
            case 1: write_tiles_at(std::integral_constant<int, 1>{}, c); break;
            case 2: write_tiles_at(std::integral_constant<int, 2>{}, c); break;
            default: write_tiles_at(std::integral_constant<int, 3>{}, c); break;
        }
    };

    // Phase S, part 1.  Scores of chunk c; the contraction over the 64 channels is
    // split in two halves (kk), each wave writes its partial scores to tile A0 or A1 and the
    // consumers add the two products.  Wave wq: diagonal block wq&1, channel half wq>>1; the
    // waves with an even wq also take the level-16 block (t-block 1, i-block 0).
    auto scores = [&](int c) {
        char* lds = lds_all + (c & 1) * kBuf;
        const int q = wq & 1;
        const int kk = wq >> 1;
        const int at = kk ? kA1 : kA0;
        const int rowq = (16 * q + l16) * kRow + 16 * g4 + 64 * kk;
        const half8 z8 = lds_read_h8(lds, kZ8 + rowq);
        const half8 z4 = lds_read_h8(lds, kZ4 + rowq);
        const half8 z2 = lds_read_h8(lds, kZ2 + rowq);
        const half8 q1 = lds_read_h8(lds, kQ1 + rowq);
        const half8 k1 = kC2 ? q1 : lds_read_h8(lds, kK1 + rowq);
        const float4v zero{0.f, 0.f, 0.f, 0.f};
        const float4v acc8 = mfma(z8, z8, zero);
        const float4v acc4 = mfma(z4, z4, zero);
        const float4v acc2 = mfma(z2, z2, zero);
        const float4v acc1 = mfma(k1, q1, zero);     // pairs (odd t, t-1) and, on the diagonal, the bonus
        float sel[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 4 * g4 + e, t = l16;
            const int d = i ^ t;
            const float val = d >= 8 ? acc8[e] : d >= 4 ? acc4[e] : d >= 2 ? acc2[e] : acc1[e];
            sel[e] = (kC2 ? i >= t : i > t) ? 0.f : val;    // Finch-C2 has no diagonal term
        }
        // keys 16q + 4*g4 .. +3 of token row 16q + l16: half (g4 & 1) of granule 2q + (g4 >> 1)
        *reinterpret_cast<uint2*>(lds + at + score_off(16 * q + l16, 2 * q + (g4 >> 1)) + 8 * (g4 & 1)) =
            make_uint2(pack_h2(sel[0], sel[1]), pack_h2(sel[2], sel[3]));
        if (q == 0) {
            const int rq = (16 + l16) * kRow + 16 * g4 + 64 * kk;
            const half8 zq = lds_read_h8(lds, kZ16 + rq);
            const half8 zk = lds_read_h8(lds, kZ16 + rq - 16 * kRow);
            const float4v acc = mfma(zk, zq, zero);
            *reinterpret_cast<uint2*>(lds + at + score_off(16 + l16, g4 >> 1) + 8 * (g4 & 1)) =
                make_uint2(pack_h2(acc[0], acc[1]), pack_h2(acc[2], acc[3]));
        }
    };

    // Phase S, part 2.  Finished output rows of chunk c (staged by the consumers): full
    // 128-byte (bf16) rows to HBM, 8 threads per row.  Finch-C2: the rows are staged in fp32 and
    // the second value u' of the same 8 channels (16 bytes, loaded two windows earlier) is added
    // before the single rounding of the output.  (Letting the consumer waves load u' in their
    // accumulator layout and start the chunk's accumulator from it -- bf16 staging, nothing to add
    // here -- gives the same bits and was 25 % slower: a load issued by any wave of the workgroup
    // returns behind the chunk loads the producers already have in flight, four to six windows
    // of them, and the consumers cannot wait that long.)
    const int srow = gtid >> 3;                  // token row inside the chunk this thread stores
    const int scol = 8 * (gtid & 7);             // first of its 8 channels
    [[maybe_unused]] uint4v up_raw = {0u, 0u, 0u, 0u};
    [[maybe_unused]] const int up_voff = static_cast<int>(srow * st.row_bytes + scol * 2);
    [[maybe_unused]] const char* up_base = kC2 ? static_cast<const char*>(a.uprime) + un.base0 * 2 : nullptr;
    auto load_uprime = [&](const Cursor<kMulti>& at) {
        if constexpr (kC2 && !kStateOnly) {
            // unconditional (exact wait counts): before the start it re-reads chunk 0, past the
            // end the descriptor is empty
            const int cc = at.c < 0 ? 0 : at.c;
            const bool live = at.c < 0 || at.live(un);
            const long long off = static_cast<long long>(cc) * kChunk * st.row_bytes;
            up_raw = __builtin_bit_cast(uint4v, __builtin_amdgcn_raw_buffer_load_b128(
                                                    chunk_rsrc(up_base + (live ? at.unit_elems(un) * 2 : 0), off,
                                                               live ? st.span_bytes : 0),
                                                    up_voff, 0, kStreamOnce));
        }
    };
    // Output rows leave through a raw buffer descriptor that starts at the chunk's first row and ends
    // with the unit's last token: rows past the end of the sequence are dropped by the bounds check.
    constexpr int kOutElem = kOutF32 ? 4 : 2;
    [[maybe_unused]] const long long out_row_bytes = tok_stride * kOutElem;
    [[maybe_unused]] const long long out_span = static_cast<long long>(T - 1) * out_row_bytes + kHeadSize * kOutElem;
    [[maybe_unused]] const int out_voff = static_cast<int>(srow * out_row_bytes + scol * kOutElem);
    [[maybe_unused]] const char* out_base = static_cast<const char*>(a.out) + un.base0 * kOutElem;
    auto store_rows = [&](int g, const Cursor<kMulti>& at) {   // g: position in the sequence (LDS parity)
        const char* lds = lds_all + (g & 1) * kBuf;
        const int t = at.c * kChunk + srow;
        const __amdgpu_buffer_rsrc_t ro = chunk_rsrc(out_base + at.unit_elems(un) * kOutElem,
                                                     static_cast<long long>(at.c) * kChunk * out_row_bytes, out_span);
        auto put = [&](uint4v q, int byte) {
            __builtin_amdgcn_raw_buffer_store_b128(q, ro, out_voff + byte, 0, kStoreThrough);
        };
        if (t < T) {
            if constexpr (kStageF32) {
                // fp32 rows of the Finch form (256 bytes): the row's 8 threads store its first 128 bytes, then
                // its second (whole cache lines per instruction): thread j holds floats 4j.. and 32 + 4j..
                constexpr bool kSplitRow = kOutF32 && !kC2;
                const float4* src = reinterpret_cast<const float4*>(
                    lds + kO + (srow * kORowF32 + (kSplitRow ? scol / 2 : scol)) * 4);
                float4 q0 = src[0], q1 = src[kSplitRow ? 8 : 1];
                if constexpr (kC2) {
                    q0.x += bf16_lo(up_raw[0]); q0.y += bf16_hi(up_raw[0]);
                    q0.z += bf16_lo(up_raw[1]); q0.w += bf16_hi(up_raw[1]);
                    q1.x += bf16_lo(up_raw[2]); q1.y += bf16_hi(up_raw[2]);
                    q1.z += bf16_lo(up_raw[3]); q1.w += bf16_hi(up_raw[3]);
                }
                if constexpr (kMoments) {
                    // The 8 threads of a row hold the head's 64 finished values of this token: their
                    // sum, then the squared deviations from the head's own mean, each folded over
                    // the 8 lanes; the row's first thread writes the pair.
                    const float s = row8_sum(((q0.x + q0.y) + (q0.z + q0.w)) + ((q1.x + q1.y) + (q1.z + q1.w)));
                    const float m = s * (1.f / kHeadSize);
                    float m2 = (q0.x - m) * (q0.x - m);
                    m2 = fmaf(q0.y - m, q0.y - m, m2);
                    m2 = fmaf(q0.z - m, q0.z - m, m2);
                    m2 = fmaf(q0.w - m, q0.w - m, m2);
                    m2 = fmaf(q1.x - m, q1.x - m, m2);
                    m2 = fmaf(q1.y - m, q1.y - m, m2);
                    m2 = fmaf(q1.z - m, q1.z - m, m2);
                    m2 = fmaf(q1.w - m, q1.w - m, m2);
                    m2 = row8_sum(m2);
                    if (scol == 0) {
                        long long unit_index = un.first;
                        if constexpr (kMulti) unit_index += static_cast<long long>(at.ui) * un.stride;
                        // streamed like the output rows (measured: 7 % of the kernel's time on many
                        // short units against a plain store)
                        typedef float float2v __attribute__((ext_vector_type(2)));
                        const float2v pair = {s, m2};
                        __builtin_nontemporal_store(pair, reinterpret_cast<float2v*>(a.moments + (unit_index * T + t) * 2));
                    }
                }
                if constexpr (kOutF32) {
                    if constexpr (kSplitRow) {
                        put(__builtin_bit_cast(uint4v, q0), -scol * 2);            // byte 16 j of the row
                        put(__builtin_bit_cast(uint4v, q1), 128 - scol * 2);      // byte 128 + 16 j
                    } else {
                        put(__builtin_bit_cast(uint4v, q0), 0);
                        put(__builtin_bit_cast(uint4v, q1), 16);
                    }
                } else {
                    uint4v q;
                    q.x = pack_bf2(q0.x, q0.y);
                    q.y = pack_bf2(q0.z, q0.w);
                    q.z = pack_bf2(q1.x, q1.y);
                    q.w = pack_bf2(q1.z, q1.w);
                    put(q, 0);
                }
            } else {
                put(*reinterpret_cast<const uint4v*>(lds + kO + (srow * kORowBf16 + scol) * 2), 0);
            }
        }
    };

    // A group spends three consecutive windows on each of its chunks g = pg, pg+3, ... of the
    // workgroup's chunk sequence:
    //   window g    phase D: decays and group products of chunk g from one of two raw register
    //               sets, then the HBM loads of x and r of the group's chunk after next (g+6) into
    //               the same set (k and v follow in phase T); they stay in flight for four to six
    //               windows.  Issued unconditionally: past the end the descriptor is empty and the
    //               loads return zeros without touching memory.
    //   window g+1  phase T: multipliers from all groups' decay totals, every operand tile.
    //   window g+2  phase S: score MFMAs, and the finished output rows of chunk g-2.
    // The three groups are one window apart, so every window sees one group in each phase
    // next to the consumers: vector-ALU, LDS and matrix-core work of different chunks overlap.
    // Wave priorities (s_setprio, an issue-arbitration hint inside the compute unit): the score
    // phase and the consumers (3) sit on MFMA and LDS-read latency chains and the consumers carry
    // the only dependency from window to window; the digest (2) starts with the exponentials
    // everything else waits for; the tile phase (0) is throughput work, mostly LDS writes nobody
    // reads before the barrier, and fills the gaps.  Measured against equal priorities: config 2
    // -3 %, config 5 -4 to -12 % depending on the box, fp32 output -8 %, nothing slower.
    const int total = un.count * un.nchunks;
    const int nwin = window_count(total);
    Cursor<kMulti> cur{0, 0}, ld{0, 0}, stc{0, pg - 2};      // chunk g, chunk g+6 (loads), chunk g-2 (stores)
    cur.advance(pg, un.nchunks);
    ld.advance(pg, un.nchunks);
    stc.advance(0, un.nchunks);
    auto fetch_xr = [&](Raw& buf, const Cursor<kMulti>& at) {
        const bool live = at.live(un);                // uniform; dead: offset past the span = empty descriptor
        load_rows_xr<kStateOnly, kLora, kStreamOnce>(buf, st, live ? at.unit_elems(un) * 2 : 0, live ? at.c * kChunk : T + kChunk, voff);
    };
    auto fetch_kv = [&](Raw& buf, const Cursor<kMulti>& at) {
        const bool live = at.live(un);
        load_rows_kv<kStreamOnce>(buf, st, live ? at.unit_elems(un) * 2 : 0, live ? at.c * kChunk : T + kChunk, voff);
    };
    // one chunk of this group through its three windows; `buf` holds its raw inputs and is
    // refilled with the group's chunk after next (six chunks ahead) right after the digest
    auto cycle = [&](int g, Raw& buf) {
        const bool live = cur.live(un);
        __builtin_amdgcn_s_setprio(2);            // see the note on wave priorities above
        if (live) digest(g, cur.c, buf);
        load_uprime(stc);                         // older than the chunk loads: waited for first
        fetch_xr(buf, ld);
        __syncthreads();                                                        // window barrier
        __builtin_amdgcn_s_setprio(0);
        if (live) write_tiles(g);
        fetch_kv(buf, ld);                        // the other half: issued a window later, measured best here
        __syncthreads();                                                        // window barrier
        if constexpr (!kStateOnly) {
            __builtin_amdgcn_s_setprio(3);
            if (live) scores(g);
            if (stc.c >= 0 && stc.live(un)) store_rows(g - 2, stc);
        }
        __syncthreads();                                                        // window barrier
        cur.advance(3, un.nchunks);
        ld.advance(3, un.nchunks);
        stc.advance(3, un.nchunks);
    };
    fetch_xr(raw_a, ld);
    fetch_kv(raw_a, ld);
    ld.advance(3, un.nchunks);
    fetch_xr(raw_b, ld);
    fetch_kv(raw_b, ld);
    ld.advance(3, un.nchunks);                    // now six chunks ahead of `cur`
    __syncthreads();                                                            // start barrier
    int done = 0;                                                               // windows passed
    for (; done < pg; ++done) {
        __syncthreads();                                                        // window barrier
    }
    int g = pg;
#pragma clang loop unroll(disable)
    for (; has_cycle_pair(g, nwin); g += 6) {       // same walk as producer_walk() in wkv6_windows.h
        cycle(g, raw_a);
        cycle(g + 3, raw_b);
        done += 6;
    }
    if (has_cycle(g, nwin)) {
        cycle(g, raw_a);
        done += 3;
    }
    for (; done < nwin; ++done) {
        __syncthreads();                                                        // window barrier
    }
}

// ------------------------------------------------------------------------------------------
// Consumer waves
// ------------------------------------------------------------------------------------------
template <int kMode, bool kC2, bool kMulti>
__device__ __forceinline__ void consumer(const Args& a, char* lds_all, int lane, int cw, const Units& un) {
    constexpr bool kOutF32 = kMode == 1;
    constexpr bool kStateOnly = kMode == 2;
    constexpr bool kLora = kMode >= 4;
    const int l16 = lane & 15;
    const int g4 = lane >> 4;
    const int j = 16 * cw + l16;            // value column of this lane
    // the consumers carry the only sequential chain: let the SIMD arbiter prefer them
    __builtin_amdgcn_s_setprio(3);

    // S[nb][e] = state[n = 16nb + 4g4 + e][j]; Snext: the state entering the workgroup's next
    // unit, fetched while the current unit is still being processed
    // State traffic goes through a raw buffer descriptor of the unit's 16 KiB with the
    // (nb, e) part of the offset as a scalar: one vector register of addressing for all 16
    // accesses instead of a 64-bit address each.
    float4v S[4];
    [[maybe_unused]] float4v Snext[4];
    const int state_voff = (4 * g4 * 64 + j) * 4;
    auto state_rsrc = [&](const float* base, int ui) {
        const long long unit = static_cast<long long>(un.first) + static_cast<long long>(ui) * un.stride;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base + unit * 4096), 0, 4096 * 4, 0x00020000);
    };
    auto fetch_state = [&](float4v (&dst)[4], int ui) {
        if (a.state_in && ui < un.count) {
            const __amdgpu_buffer_rsrc_t rs = state_rsrc(a.state_in, ui);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    dst[nb][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, state_voff, (16 * nb + e) * 256, 0));
        } else {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) dst[nb] = float4v{0.f, 0.f, 0.f, 0.f};
        }
    };
    if constexpr (kMulti)
        fetch_state(Snext, 0);
    else
        fetch_state(S, 0);

    float dtot = 1.f;   // product of all decays so far, key channel `lane` (only with decay_out)
    // Output of the chunk whose state chain ran last, transposed: o[tq][e] belongs to token
    // 16*tq + l16 and value channel 16*cw + 4*g4 + e (the state is the A operand and the token rows
    // the B operand of the MFMAs below), so a lane's four values are contiguous in the output row.
    float4v o[2];
    half8 vt;           // V^T operand of that chunk: this lane's value channel, tokens 8*g4 .. +7

    const int total = un.count * un.nchunks;
    const int nwin = window_count(total);

    // Fused decay path.  This wave forms the decay logits of its 16 channels (16cw .. 16cw+15, as
    // key channels) for all 32 tokens of the chunk the producers digest in the next window:
    // d = lambda + y B_h, two 16-token row blocks x two 32-wide steps over the rank, bf16 operands
    // (exact products) with fp32 accumulation started at lambda.  The head's 64x16 slice of B
    // stays in registers for the whole kernel; y rows (128 bytes per token, shared by all heads,
    // so served by L2) are requested at the start of a window and used at its end.
    [[maybe_unused]] bf16x8 bw[2];
    [[maybe_unused]] bf16x8 ya[2][2];
    [[maybe_unused]] float lam = 0.f;
    [[maybe_unused]] int y_b0 = 0, y_bstep = 0;
    [[maybe_unused]] const int y_voff = l16 * (kLoraRank * 2) + 16 * g4;
    if constexpr (kLora) {
        const int width = a.H * kHeadSize;
        const int col = (un.first % a.H) * kHeadSize + 16 * cw + l16;
        const unsigned short* bwp = static_cast<const unsigned short*>(a.bw);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                bw[ks][e] = __builtin_bit_cast(__bf16, bwp[static_cast<long long>(32 * ks + 8 * g4 + e) * width + col]);
        lam = a.lambda[col];
        y_b0 = un.first / a.H;
        y_bstep = un.stride / a.H;
    }
    auto y_fetch = [&](const Cursor<kMulti>& dn) {
        const long long batch = y_b0 + (kMulti ? static_cast<long long>(dn.ui) * y_bstep : 0);
        const long long seq_bytes = static_cast<long long>(a.T) * (kLoraRank * 2);
        const __amdgpu_buffer_rsrc_t ry = chunk_rsrc(static_cast<const char*>(a.y) + batch * seq_bytes,
                                                     static_cast<long long>(dn.c) * kChunk * (kLoraRank * 2), seq_bytes);
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                ya[rt][ks] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(
                                                            ry, y_voff + 16 * rt * (kLoraRank * 2) + 64 * ks, 0, 0));
    };
    auto d_finish = [&](int pos) {                   // pos: the chunk's position in the sequence (LDS parity)
        char* dx = lds_all + kDx + (pos & 1) * kDxBuf + (8 * cw + (l16 >> 1)) * kDxPair + (l16 & 1) * (kChunk * 4) + 16 * g4;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            float4v acc = {lam, lam, lam, lam};
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ya[rt][0], bw[0], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ya[rt][1], bw[1], acc, 0, 0, 0);
            *reinterpret_cast<float4v*>(dx + 64 * rt) = acc;     // tokens 16rt + 4g4 .. +3 of this lane's channel
        }
    };
    Cursor<kMulti> dn{0, 0};                         // the chunk whose logits are formed next
    if constexpr (kLora) {
        if (total > 0) {
            y_fetch(dn);
            d_finish(0);
            dn.advance(1, un.nchunks);
        }
    }

    __syncthreads();                                                            // start barrier
    Cursor<kMulti> at{0, 0};                         // chunk n-2 of the sequence: the state chain's
#pragma clang loop unroll(disable)
    for (int n = 0; n < nwin; ++n) {
        [[maybe_unused]] const bool dlive = kLora && n + 1 < total;
        if constexpr (kLora) {
            if (dlive) y_fetch(dn);
        }
        // (The two parts below in one straight line for the steady state -- every LDS read of the window
        // first, then the matrix-core work of both chunks -- shortens the consumers' own chain from
        // 1430 to 1260 clocks and lengthens the window from 1850 to 1960: their reads then arrive at
        // the LDS queue in one burst at the highest priority and the producers wait behind them.)
        if (!kStateOnly && n >= 3 && n - 3 < total) {
            // chunk n-3: o += A V (two partial score tiles), then stage for the producers' stores
            char* lds = lds_all + ((n - 3) & 1) * kBuf;
#pragma unroll
            for (int tq = 0; tq < 2; ++tq) {
                const int off = score_off(16 * tq + l16, g4);
                const half8 a0 = lds_read_h8(lds, kA0 + off);
                const half8 a1 = lds_read_h8(lds, kA1 + off);
                o[tq] = mfma(vt, a0, o[tq]);
                o[tq] = mfma(vt, a1, o[tq]);
                const int row = 16 * tq + l16, col = 16 * cw + 4 * g4;
                if constexpr (kOutF32 || kC2)
                    *reinterpret_cast<float4v*>(lds + kO + (row * kORowF32 + col) * 4) = o[tq];
                else
                    *reinterpret_cast<uint2*>(lds + kO + (row * kORowBf16 + col) * 2) =
                        make_uint2(pack_bf2(o[tq][0], o[tq][1]), pack_bf2(o[tq][2], o[tq][3]));
            }
        }
        if (n >= 2 && n - 2 < total) {
            // chunk n-2: the state chain
            const char* lds = lds_all + (n & 1) * kBuf;
            if (at.c == 0) {
                // a unit begins: take its entering state, start fetching the next unit's
                if constexpr (kMulti) {
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) S[nb] = Snext[nb];
                    fetch_state(Snext, at.ui + 1);
                }
                dtot = 1.f;
            }
            // inter-chunk read: o[t][j] = sum_n (r_t W(t,-1))[n] S[n][j]; the state registers,
            // rounded to fp16, are the A operand (k-slot order = the r tile's column permutation)
            if constexpr (!kStateOnly) {
                half8 sh[2];
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        sh[kk][e] = static_cast<_Float16>(S[2 * kk + (e >> 2)][e & 3]);
#pragma unroll
                for (int tq = 0; tq < 2; ++tq) {
                    o[tq] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        const half8 rt = lds_read_h8(lds, kRT + (16 * tq + l16) * kRow + (32 * kk + 8 * g4) * 2);
                        o[tq] = mfma(sh[kk], rt, o[tq]);
                    }
                }
            }
            if (a.decay_out) dtot *= *reinterpret_cast<const float*>(lds + kD + lane * 4);
            // state update: S = diag(W(32,-1)) S + (k W(32,i))^T V over the chunk's 32 tokens
            vt = lds_read_h8(lds, kVT + tile_t_off(16 * cw + l16, g4));
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const float4 d = *reinterpret_cast<const float4*>(lds + kD + (16 * nb + 4 * g4) * 4);
                S[nb][0] *= d.x;
                S[nb][1] *= d.y;
                S[nb][2] *= d.z;
                S[nb][3] *= d.w;
                const half8 kt = lds_read_h8(lds, kKT + tile_t_off(16 * nb + l16, g4));
                S[nb] = mfma(kt, vt, S[nb]);
            }
            if (at.c == un.nchunks - 1) {
                // the unit ends: its final state and, if asked for, its total decay
                const long long unit = static_cast<long long>(un.first) + static_cast<long long>(at.ui) * un.stride;
                if (un.state_out) {
                    const __amdgpu_buffer_rsrc_t rs = state_rsrc(un.state_out, at.ui);
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float value = S[nb][e];        // (a bit cast straight from the vector element reads element 0)
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(value), rs, state_voff,
                                                                  (16 * nb + e) * 256, 0);
                        }
                }
                if (a.decay_out && cw == 0) a.decay_out[unit * kHeadSize + lane] = dtot;
            }
            at.advance(1, un.nchunks);
        }
        if constexpr (kLora) {
            if (dlive) {
                d_finish(n + 1);
                dn.advance(1, un.nchunks);
            }
        }
        __syncthreads();                                                        // window barrier
    }
}

template <int kMode, bool kC2, bool kMulti>
__global__ __launch_bounds__(kThreads) void chunked_kernel(Args a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    // MODE.FP16_OVFL = 1 (hwreg id 1, bit 23, one bit): fp16 results that overflow, conversions
    // included, are clamped to +-65504 instead of becoming infinite, so operands beyond the fp16
    // range saturate as the header promises; true infinities are preserved.
    __builtin_amdgcn_s_setreg(1 | (23 << 6) | (0 << 11), 1);
    const int tid = threadIdx.x;
    const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);
    int unit = blockIdx.x;                       // (batch * segs + segment) * H + head
    if constexpr (kMode >= 4) {
        // Fused decay path: the heads of a batch share its y rows.  Workgroups go to the 8 XCDs
        // (each with its own L2) round-robin by index, so give XCD i the i-th eighth of the
        // units: neighbouring heads of a batch then read y through the same L2.
        const int per_xcd = gridDim.x >> 3;
        if ((gridDim.x & 7) == 0) unit = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    }
    const int bs = unit / a.H;
    const int h = unit - bs * a.H;
    const int segs_launched = a.segs_launched > 0 ? a.segs_launched : a.segs;
    const int b = bs / segs_launched;
    const int seg = bs - b * segs_launched;
    const long long tok_stride = static_cast<long long>(a.H) * kHeadSize;
    const long long unit_base = static_cast<long long>(b) * a.batch_stride +
                                static_cast<long long>(seg) * a.seg_stride +
                                static_cast<long long>(h) * kHeadSize;
    const int T = (seg == a.segs - 1) ? a.T_last : a.T;
    // The workgroup's units: this one and, when the launch gave a stride (a multiple of H, whole
    // sequences only), every stride-th unit after it: same head, batch index advancing.
    Units un;
    un.first = (b * a.segs + seg) * a.H + h;     // = unit when every segment has a workgroup
    un.stride = a.unit_stride;
    un.state_out = a.state_out;
    if (a.state_out_final)                       // [B][H] states, written by the last segment only
        un.state_out = a.state_out && seg == a.segs - 1 ? a.state_out - static_cast<long long>(un.first - (b * a.H + h)) * 4096 : nullptr;
    un.count = 1;
    un.nchunks = (T + kChunk - 1) / kChunk;
    un.base0 = unit_base;
    un.step = 0;
    if constexpr (kMulti) {
        const long long total = static_cast<long long>(a.B) * a.H;
        un.count = static_cast<int>((total - unit + a.unit_stride - 1) / a.unit_stride);
        un.step = static_cast<long long>(a.unit_stride / a.H) * a.batch_stride;
    }
    if (wid < 4 * kProducerGroups)
        producer<kMode, kC2, kMulti>(a, lds, tid, wid >> 2, wid & 3, h, un, tok_stride, T);
    else
        consumer<kMode, kC2, kMulti>(a, lds, tid & 63, wid - 4 * kProducerGroups, un);
}

// Sequential fold over the segments of one (batch, head): 256 threads x 16 state entries.
__global__ __launch_bounds__(256) void combine_kernel(int H, int segs, const float* state_in,
                                                      float* seg_state, const float* seg_decay,
                                                      float* state_out, bool fold_last) {
    const int unit = blockIdx.x;                 // batch * H + head
    const int b = unit / H;
    const int h = unit - b * H;
    const int t = threadIdx.x;
    const int row = t >> 2;                      // key channel of this thread's 16 entries
    float4 S[4];
    if (state_in) {
        const float4* s0 = reinterpret_cast<const float4*>(state_in + static_cast<long long>(unit) * 4096) + 4 * t;
#pragma unroll
        for (int q = 0; q < 4; ++q) S[q] = s0[q];
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) S[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int p = 0; p < segs; ++p) {
        const long long su = (static_cast<long long>(b) * segs + p) * H + h;
        float4* loc = reinterpret_cast<float4*>(seg_state + su * 4096) + 4 * t;
        if (p == segs - 1 && !fold_last) {       // nothing follows: its pair was not produced
#pragma unroll
            for (int q = 0; q < 4; ++q) loc[q] = S[q];
            break;
        }
        const float d = seg_decay[su * kHeadSize + row];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 l = loc[q];
            loc[q] = S[q];                       // the state entering segment p
            S[q] = make_float4(fmaf(d, S[q].x, l.x), fmaf(d, S[q].y, l.y), fmaf(d, S[q].z, l.z),
                               fmaf(d, S[q].w, l.w));
        }
    }
    if (state_out && fold_last) {
        float4* so = reinterpret_cast<float4*>(state_out + static_cast<long long>(unit) * 4096) + 4 * t;
#pragma unroll
        for (int q = 0; q < 4; ++q) so[q] = S[q];
    }
}

template <int kMode, bool kC2, bool kMulti>
struct ChunkedTag {};

template <int kMode, bool kC2>
hipError_t launch_mode(const Args& args, hipStream_t stream) {
    Args a = args;
    long long units = static_cast<long long>(a.B) * (a.segs_launched > 0 ? a.segs_launched : a.segs) * a.H;
    a.unit_stride = 0;
    // With more (batch, head) units than compute units each workgroup takes several of them back to back.
    const int cus = compute_units();
    if (kMode != 2 && a.segs == 1 && a.H <= cus) {
        const int per_round = a.H * (cus / a.H);                 // a multiple of H: the head stays fixed
        if (units > per_round) {
            a.unit_stride = per_round;
            units = per_round;
        }
    }
    const dim3 grid(static_cast<unsigned>(units));
    constexpr int lds_bytes = kMode >= 4 ? kLdsBytesLora : kLdsBytes;
    auto go = [&](auto tag, auto kernel) {
        const hipError_t err = set_lds_limit_once<decltype(tag)>(kernel, lds_bytes);
        if (err != hipSuccess) return err;
        hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds_bytes, stream, a);
        return hipGetLastError();
    };
    if constexpr (kMode != 2) {
        if (a.unit_stride > 0) return go(ChunkedTag<kMode, kC2, true>{}, &chunked_kernel<kMode, kC2, true>);
    }
    return go(ChunkedTag<kMode, kC2, false>{}, &chunked_kernel<kMode, kC2, false>);
}

}  // namespace

hipError_t launch_chunked(const Args& a, ChunkedMode mode, hipStream_t stream) {
    const bool c2 = a.finch_c2;
    switch (mode) {
        case ChunkedMode::kBf16Out: return c2 ? launch_mode<0, true>(a, stream) : launch_mode<0, false>(a, stream);
        case ChunkedMode::kF32Out: return c2 ? launch_mode<1, true>(a, stream) : launch_mode<1, false>(a, stream);
        case ChunkedMode::kStateOnly: return c2 ? launch_mode<2, true>(a, stream) : launch_mode<2, false>(a, stream);
        case ChunkedMode::kBf16OutMoments:
            if (!c2 || a.segs != 1 || !a.moments) return hipErrorInvalidValue;
            return launch_mode<3, true>(a, stream);
        default:
            if (a.segs != 1 || !a.y || !a.lambda || !a.bw) return hipErrorInvalidValue;
            if (mode == ChunkedMode::kBf16OutLora)
                return c2 ? launch_mode<4, true>(a, stream) : launch_mode<4, false>(a, stream);
            if (!c2 || !a.moments) return hipErrorInvalidValue;
            return launch_mode<5, true>(a, stream);
    }
}

hipError_t launch_combine_segments(int B, int H, int segs, const float* state_in, float* seg_state,
                                   const float* seg_decay, float* state_out, bool fold_last, hipStream_t stream) {
    hipLaunchKernelGGL(combine_kernel, dim3(static_cast<unsigned>(B) * static_cast<unsigned>(H)),
                       dim3(256), 0, stream, H, segs, state_in, seg_state, seg_decay, state_out, fold_last);
    return hipGetLastError();
}

}  // namespace wkv6

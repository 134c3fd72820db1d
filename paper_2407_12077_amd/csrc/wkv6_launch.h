// Internal launch interface between the C ABI (wkv6_api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

namespace wkv6 {

constexpr int kHeadSize = 64;   // N: the only head size the kernels are built for

struct Args {
    int B, T, H;
    const void* r;
    const void* k;
    const void* v;
    const void* x;
    const float* u;           // Finch bonus [H][N]; unused in the Finch-C2 form
    bool finch_c2;            // false: Finch form (bonus u).  true: Finch-C2 form: k is the key before its
                              // (1 - w) factor, no bonus, and the second value uprime is added to the read-out
    const void* uprime;       // Finch-C2 only: [B][T][H][N] bf16, laid out like out; not read by the
                              // state-only pass
    const float* state_in;    // may be nullptr (zero state)
    void* out;
    float* state_out;         // may be nullptr (not written)
    long long batch_stride;   // elements between consecutive batches of r,k,v,x,out
    // Token-axis segments (chunked kernel only).  Each sequence is cut into `segs` segments of T
    // tokens (the last one T_last), seg_stride elements apart; a workgroup handles one
    // (batch, segment, head) and indexes state_in / state_out / decay_out by
    // (batch*segs + segment)*H + head.  segs == 1: T_last == T and the plain layout.
    int segs;
    int T_last;
    long long seg_stride;
    int segs_launched = 0;    // 0: every segment has a workgroup.  n > 0: only the first n segments of each
                              // sequence have one (the indexing by all `segs` stays)
    bool state_out_final = false;   // with segs > 1: state_out is [B][H][N][N] and only the last segment's
                              // workgroup writes it (the state the whole sequence leaves behind)
    float* decay_out;         // may be nullptr; [B*segs][H][N] product of all decays of the unit
    float* moments;           // kBf16OutMoments only: [B][H][T][2] per (batch, head, token): the sum of
                              // the head's N output values and their squared deviations from the
                              // head's own mean (taken before the rounding to bf16)
    // kBf16OutLora / kBf16OutLoraMoments only (x unused): the decay logit is formed in the kernel as
    // d[b][t][h][n] = lambda[h*N+n] + sum_k y[b][t][k] * bw[k][h*N+n], k < 64
    const void* y;            // [B][T][64] bf16
    const float* lambda;      // [H*N] fp32
    const void* bw;           // [64][H*N] bf16
    int unit_stride;          // set by launch_chunked: 0 = one unit per workgroup; otherwise workgroup w
                              // handles units w, w + unit_stride, ... (a multiple of H, segs == 1 only)
};

enum class ChunkedMode { kBf16Out, kF32Out, kStateOnly, kBf16OutMoments, kBf16OutLora, kBf16OutLoraMoments };

constexpr int kLoraRank = 64;   // R: the only rank of the decay path the fused kernel is built for

// Token-by-token fp32 kernel; inputs bf16 or fp32 (fp32 inputs: fp32 out, Finch form only);
// with bf16 inputs the output is fp32 or bf16 and a.finch_c2 selects the form.
hipError_t launch_recurrent(const Args& a, bool in_bf16, bool out_bf16, hipStream_t stream);

// Chunked matrix-core kernel; inputs bf16, out bf16 or fp32, or (kStateOnly) no output at all:
// only state_out and decay_out of every unit, from r-independent work.  kBf16OutMoments: bf16 out
// plus a.moments, Finch-C2 form and segs == 1 only.  kBf16OutLora: bf16 out with the decay
// logits formed in the kernel from a.y, a.lambda, a.bw instead of read from a.x (either form,
// segs == 1); kBf16OutLoraMoments: that plus a.moments (Finch-C2 form).
hipError_t launch_chunked(const Args& a, ChunkedMode mode, hipStream_t stream);

// Token-split support: folds the per-segment (decay, local state) pairs of every (batch, head)
// into the state entering each segment, in place in `seg_state` ([B*segs][H][N][N]).  The pair of
// the last segment is not read (nothing follows it): the first pass need not produce it, and the
// final state of the sequence comes from the full pass over the last segment (state_out_final).
// state_out, when not nullptr, receives the state entering the last segment's successor only if
// `fold_last` is set (then the last pair is read too).
hipError_t launch_combine_segments(int B, int H, int segs, const float* state_in, float* seg_state,
                                   const float* seg_decay, float* state_out, bool fold_last, hipStream_t stream);

// GOLD key compression c = x W: x [M][D] bf16, w [D][D/16] bf16, c [M][D/16] bf16 or fp32.
// D must be a multiple of 256 (16 output columns per MFMA block, an even number of 64-channel steps).
hipError_t launch_key_compress(long long M, int D, const void* x, const void* w, void* c, bool out_f32,
                               hipStream_t stream);

// Folds the H per-head (sum, squared deviations) pairs of every token into the token's mean and
// 1/sqrt(variance + eps) over all H*N channels: moments [B][H][T][2] -> mean_rstd [B][T][2].
hipError_t launch_layernorm_finalize(int B, int T, int H, const float* moments, float eps, float* mean_rstd,
                                     hipStream_t stream);

// Applies the token statistics: y = (o - mean) * rstd * gamma + beta; o [tokens][D] bf16, mean_rstd
// [tokens][2], gamma and beta [D] fp32, y [tokens][D] bf16 or fp32.  D must be a multiple of 8.
hipError_t launch_layernorm_apply(long long tokens, int D, const void* o, const float* mean_rstd, const float* gamma,
                                  const float* beta, void* y, bool out_f32, hipStream_t stream);

// Front of the decay path: y = tanh(ddlerp_d(x_t, x_{t-1}) A_omega), x [B][T][D] bf16, x_prev [B][D] bf16 or
// nullptr, mu_x and lambda_d [D] fp32, a_d [32][D], b_d [D][32], a_omega [64][D] bf16, y [B][T][64] bf16
// or fp32.  D must be a multiple of 128.
hipError_t launch_decay_input(int B, int T, int D, const void* x, const void* x_prev, const float* mu_x,
                              const float* lambda_d, const void* a_d, const void* b_d, const void* a_omega, void* y,
                              bool out_f32, hipStream_t stream);

// Raises a kernel's dynamic LDS limit once per device and kernel instantiation (the attribute
// belongs to the loaded function on a device, so it need not be set again at every launch, and must
// not be set under stream capture: a process that captures should make its first call to an entry
// point outside the capture).  `Tag` makes one flag set per kernel.
template <typename Tag, typename Kernel>
inline hipError_t set_lds_limit_once(Kernel kernel, int bytes) {
    static std::atomic<unsigned long long> done{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    const unsigned long long bit = 1ull << dev;
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    const hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (err == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return err;
}

// Compute units of the current device (256 on an MI355X), read once per device; 256 if the
// query fails.
inline int compute_units() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n <= 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// T == 0: state_out = state_in (or zero).
hipError_t launch_state_passthrough(const Args& a, hipStream_t stream);

}  // namespace wkv6

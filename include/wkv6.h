/*
 * wkv6.h -- C ABI of the MI355X (gfx950) WKV6 prefill library.
 *
 * One call evaluates, for one layer and every (batch b, head h) independently,
 * the Finch (RWKV-6) time-mix recurrence that GoldFinch's linear-time pre-fill
 * runs in each Finch / Finch-C2 layer (paper: Method, "Finch-C2 Time Mixing":
 * decay map w_t = exp(-exp(d_t)); state wkv_t = sum_{i<t} diag(prod_{j=i+1}^{t-1}
 * w_j) k_i^T v_i; read-out r_t . wkv_t; and "Pre-fill of the compressed key
 * cache ..." for why this is the pre-fill hot loop):
 *
 *     o_t = r_t . ( S_{t-1} + diag(u) k_t^T v_t )      t = 1..T
 *     S_t = diag(w_t) S_{t-1} + k_t^T v_t ,            w_t = exp(-exp(x_t))
 *
 * S is a (key channel i) x (value channel j) matrix per (b,h); the decay acts
 * on the key channel; S_0 is `state_in` (or zero); `u` is the per-head Finch
 * bonus.  Finch-C2 is the case u = 0 with the caller scaling k by (1 - w) and
 * adding its second value u'_t to the output.
 *
 * Argument meaning and layout (all tensors row-major, innermost index last):
 *   B, T, H, N   batch, tokens per sequence, heads, head size.  N must be 64.
 *                B = 0 is a no-op; T = 0 writes state_out = S_0 and no output.
 *   r, k, v, x   [B][T][H][N]  receptance, key, value, decay logit (x = d_t)
 *   u            [H][N]        fp32 bonus
 *   state_in     [B][H][N][N]  fp32, [key i][value j]; NULL means S_0 = 0 (not read)
 *   out          [B][T][H][N]  o_t
 *   state_out    [B][H][N][N]  fp32 S_T; NULL means "do not write".  May equal
 *                              state_in (updated in place).  `out` must not alias
 *                              any input.
 *   stream       a hipStream_t passed as void* (NULL = the default stream)
 *
 * Ownership: every pointer is a DEVICE pointer owned by the caller; base
 * addresses of r,k,v,x,out must be 16-byte aligned.  Unless an entry point's own
 * comment says otherwise the library allocates nothing, keeps no state between
 * calls, only enqueues work on `stream` and never synchronises, so calls on
 * different streams may overlap.
 *
 * Decay logits: any finite x, and x = -inf (w = 1) and x = +inf (w = 0), are
 * accepted without a clamp: the chunked kernels only ever form products of
 * decays (all <= 1), never a reciprocal or a positive exponent, so nothing
 * overflows.  The Finch-C2 key factor 1 - w is formed without subtracting
 * nearly equal numbers (a series in exp(x) when w is close to 1).
 *
 * Value range of the bf16 entry points: the dense contractions run on the
 * matrix cores with fp16 operands and fp32 accumulation; r, k, v, the products
 * r*u and k*u, the intra-chunk scores and the running state must stay below
 * 65504 in magnitude (larger values saturate to that bound: results stay
 * finite but are those of the clamped operands).  At the small end, an fp16
 * operand below 2^-14 = 6.1e-5 in magnitude -- r, k or v times the product of
 * decays that scales it inside a 32-token chunk, and in the Finch-C2 form the
 * key kbar (1 - w) itself -- is held to an absolute 2^-25 instead of a relative
 * 2^-11, and below 2^-25 it is zero.  Against the largest value of a (batch,
 * head) unit this is far inside the tolerance; a row of the output or of the
 * state whose own values are that small is accurate to that absolute step
 * only (each output value: at most 2^-14 (max|r| + max|k|) max|v| + 2^-19
 * (1 + max|r|) max|S|).  Finch-C2 channels with decay logits below about -10
 * (1 - w < 5e-5) are the case that matters: scale kbar so that kbar (1 - w)
 * stays above 2^-14 if those state rows are needed to full relative accuracy.
 * The fp32 entry point and the decode entry points have no such limits.
 *
 * Errors: every entry point returns a wkv6_status.  Arguments are validated
 * before anything is enqueued; on a non-zero status nothing was launched,
 * except WKV6_ERR_LAUNCH which reports the HIP runtime refusing a launch.
 */
#ifndef WKV6_H
#define WKV6_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WKV6_OK = 0,
    WKV6_ERR_NULL = 1,        /* a required pointer is NULL */
    WKV6_ERR_SHAPE = 2,       /* negative size, H < 1, stride too small, overflow of the grid */
    WKV6_ERR_UNSUPPORTED = 3, /* N != 64, or an unknown dtype code */
    WKV6_ERR_LAUNCH = 4,      /* hipGetLastError() after the launch was not hipSuccess */
    WKV6_ERR_ALIGN = 5,       /* a tensor base or the batch stride is not 16-byte aligned */
    WKV6_ERR_WORKSPACE = 6    /* the shape needs more scratch memory than the library's fixed buffer */
} wkv6_status;

typedef enum {
    WKV6_DTYPE_BF16 = 0,
    WKV6_DTYPE_F32 = 1
} wkv6_dtype;

/* bf16 r,k,v,x; fp32 u and state; bf16 out.  Chunked matrix-core kernel. */
int wkv6_prefill_bf16(int B, int T, int H, int N,
                      const void *r, const void *k, const void *v, const void *x,
                      const float *u, const float *state_in,
                      void *out, float *state_out, void *stream);

/* Same computation, `out` written in fp32 (no final rounding of the output). */
int wkv6_prefill_bf16_f32out(int B, int T, int H, int N,
                             const void *r, const void *k, const void *v, const void *x,
                             const float *u, const float *state_in,
                             float *out, float *state_out, void *stream);

/*
 * As above for a window of a larger [B][T_full][H][N] buffer: consecutive
 * batches of r,k,v,x,out are `batch_stride` ELEMENTS apart (>= T*H*N, multiple
 * of 8) while tokens stay H*N apart.  Lets a caller run tokens [t0,t1) of every
 * sequence with a carried state.  out_dtype is a wkv6_dtype.
 */
int wkv6_prefill_bf16_strided(int B, int T, int H, int N,
                              const void *r, const void *k, const void *v, const void *x,
                              const float *u, const float *state_in,
                              void *out, float *state_out,
                              long long batch_stride, int out_dtype, void *stream);

/*
 * Token-split variant for few (batch, head) units and long sequences (B*H well below the 256
 * compute units, e.g. one long context): the T axis is cut into `segments` pieces that run in
 * parallel.  Three passes are enqueued on `stream`: (1) the local state and total decay of every
 * segment but the last from a zero state, using k, v, x only; (2) a sequential fold over segments
 * that turns them into the state entering each segment (the recurrence is linear in the state:
 * S_out = diag(prod w) S_in + S_local); (3) the full computation of every segment from that
 * state, the last segment leaving the final state in state_out.
 * Results equal the single-pass entry points up to rounding order.  `workspace` is caller-owned
 * device memory of at least wkv6_split_workspace_bytes() bytes, 16-byte aligned, used only
 * during the call's kernels; calls sharing a workspace must be ordered on one stream.
 * segments == 1 (or T too short to split) runs the single-pass kernel and ignores workspace.
 * out_dtype is a wkv6_dtype.
 */
int wkv6_prefill_bf16_split(int B, int T, int H, int N,
                            const void *r, const void *k, const void *v, const void *x,
                            const float *u, const float *state_in,
                            void *out, float *state_out, int out_dtype, int segments,
                            void *workspace, long long workspace_bytes, void *stream);

/*
 * wkv6_prefill_bf16_split for callers that cannot allocate device memory or pass a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * per-segment states live in a buffer of WKV6_SPLIT_NOALLOC_BYTES that is part of the library's
 * code object on every GPU it runs on, for the life of the process.  The call allocates and
 * frees nothing.  Shapes with wkv6_split_workspace_bytes(B,T,H,N,segments) above that size
 * return WKV6_ERR_WORKSPACE and enqueue nothing (B*segments*H <= 504 fits; config 3 with 8
 * segments uses 4.3 MB).  All calls on one GPU share that buffer, whatever their stream: calls
 * that overlap in time on one GPU race on it, so order them on one stream (or with events).
 * Nothing in it has to start at zero (the first two passes write every entry that is read later), and it
 * keeps the last call's contents.  The buffer's address is looked up on a GPU's first call (one
 * hipGetSymbolAddress per device, no allocation); make that first call outside stream capture.
 * Arguments, results and errors otherwise as for wkv6_prefill_bf16_split.
 */
#define WKV6_SPLIT_NOALLOC_BYTES (8ll << 20)
int wkv6_prefill_bf16_split_noalloc(int B, int T, int H, int N,
                                    const void *r, const void *k, const void *v, const void *x,
                                    const float *u, const float *state_in,
                                    void *out, float *state_out, int out_dtype, int segments,
                                    void *stream);

/* Bytes of workspace wkv6_prefill_bf16_split needs for this shape (-1 for invalid arguments). */
long long wkv6_split_workspace_bytes(int B, int T, int H, int N, int segments);

/* Segment count this library would pick for the shape on a 256-CU MI355X (1 = do not split). */
int wkv6_split_segments(int B, int T, int H, int N);

/*
 * Finch-C2 form of the same time mix (paper: Method, "Finch-C2 Time Mixing": the key is
 * multiplied by one minus the decay, and a data-dependent second value u'_t replaces Finch's
 * bonus in the read-out), fused into the chunked kernel:
 *
 *     w_t = exp(-exp(x_t)),   k_t = kbar_t * (1 - w_t)
 *     o_t = r_t . S_{t-1} + u'_t
 *     S_t = diag(w_t) S_{t-1} + k_t^T v_t
 *
 *   kbar    [B][T][H][N] bf16  the projected key BEFORE its (1 - w) factor; the factor is applied
 *                              in fp32 from the decay the kernel computes anyway
 *   uprime  [B][T][H][N] bf16  second value, added to the fp32 read-out before its one rounding
 * There is no u argument.  Everything else (layouts, state, alignment, T and B edge cases,
 * value range, errors) is as for wkv6_prefill_bf16.  The LayerNorm over the concatenated heads
 * and the output projection that follow in the paper are not part of this call.
 */
int wkv6_finch_c2_prefill_bf16(int B, int T, int H, int N,
                               const void *r, const void *kbar, const void *v, const void *x,
                               const void *uprime, const float *state_in,
                               void *out, float *state_out, void *stream);

/* Same, `out` written in fp32. */
int wkv6_finch_c2_prefill_bf16_f32out(int B, int T, int H, int N,
                                      const void *r, const void *kbar, const void *v, const void *x,
                                      const void *uprime, const float *state_in,
                                      float *out, float *state_out, void *stream);

/* Same for a window of a larger buffer (see wkv6_prefill_bf16_strided); uprime is strided like out. */
int wkv6_finch_c2_prefill_bf16_strided(int B, int T, int H, int N,
                                       const void *r, const void *kbar, const void *v, const void *x,
                                       const void *uprime, const float *state_in,
                                       void *out, float *state_out,
                                       long long batch_stride, int out_dtype, void *stream);

/* Token-split variant of the Finch-C2 form: wkv6_prefill_bf16_split with kbar and uprime in
 * place of k and u; same passes, same workspace size. */
int wkv6_finch_c2_prefill_bf16_split(int B, int T, int H, int N,
                                     const void *r, const void *kbar, const void *v, const void *x,
                                     const void *uprime, const float *state_in,
                                     void *out, float *state_out, int out_dtype, int segments,
                                     void *workspace, long long workspace_bytes, void *stream);

/*
 * Finch-C2 prefill that also emits the partial statistics of the LayerNorm that follows it
 * (paper: Method, "Finch-C2 Time Mixing", output equation: one LayerNorm over the concatenation
 * of all heads' read-outs of a token, then the output projection).  A token's heads are
 * computed by different workgroups, so the kernel writes, per (batch, head, token),
 *
 *     moments[b][h][t][0] = sum_n o[b][t][h][n]
 *     moments[b][h][t][1] = sum_n (o[b][t][h][n] - moments[b][h][t][0] / N)^2
 *
 * of the fp32 read-out values before their rounding to bf16 ([B][H][T][2] fp32, device, 16-byte
 * aligned, 8 bytes per token-head: about 1 % of the call's traffic).  wkv6_layernorm_finalize
 * folds them into each token's mean and 1/sqrt(variance + eps); with these two numbers per
 * token the normalisation becomes a row scaling and a rank-one correction in the epilogue of
 * the projection GEMM, LayerNorm(o_t) W = rstd_t (o_t (diag(gamma) W)) - rstd_t mean_t
 * (gamma W) + beta W, and no separate pass over `out` is needed.
 * Everything else is as for wkv6_finch_c2_prefill_bf16 (always the chunked kernel; `moments` must
 * not be NULL when T > 0; T == 0 writes nothing to it).
 */
int wkv6_finch_c2_prefill_bf16_moments(int B, int T, int H, int N,
                                       const void *r, const void *kbar, const void *v, const void *x,
                                       const void *uprime, const float *state_in,
                                       void *out, float *moments, float *state_out, void *stream);

/*
 * mean_rstd[b][t] = (mean, 1/sqrt(var + eps)) of the H*N read-out values of token (b, t), var
 * dividing by H*N, from `moments` as written above ([B][T][2] fp32, device, 16-byte aligned).
 * eps >= 0; the paper names the operator only, so eps is the caller's (1e-5 is the usual
 * default).  Errors as elsewhere; B == 0 or T == 0 is a no-op.
 */
int wkv6_layernorm_finalize(int B, int T, int H, int N, const float *moments, float eps,
                            float *mean_rstd, void *stream);

/*
 * Applies those statistics (paper: Method, "Finch-C2 Time Mixing", output equation: the LayerNorm over
 * the concatenated heads in front of W^O):
 *
 *     y[b][t][c] = (o[b][t][c] - mean[b][t]) * rstd[b][t] * gamma[c] + beta[c],      c = h*N + n
 *
 *   o          [B][T][H][N]  bf16  read-outs as written by the prefill entry points
 *   mean_rstd  [B][T][2]     fp32  from wkv6_layernorm_finalize
 *   gamma,beta [H*N]         fp32
 *   y          [B][T][H*N]   bf16 or fp32 per out_dtype (may equal o for bf16: every element is read before
 *                                  it is written, by the same thread)
 * all device pointers, 16-byte aligned.  This is the plain form, one streaming pass over o (read once,
 * written once), for callers whose projection GEMM cannot take the row scaling and rank-one correction
 * described above in its epilogue; with such a GEMM it is not needed.  The statistics are those of the
 * fp32 read-outs before their rounding to bf16, the values normalised are the rounded ones: the result
 * differs from a LayerNorm of the rounded values by at most the rounding itself.
 */
int wkv6_layernorm_apply_bf16(int B, int T, int H, int N, const void *o, const float *mean_rstd,
                              const float *gamma, const float *beta, void *y, int out_dtype, void *stream);

/*
 * Finch-C2 prefill with the last factor of the decay path fused in (paper: Method, "Finch-C2
 * Time Mixing": lora(x) = lambda + tanh(x A) B and d_t = lora_omega(ddlerp_d(x_t, x_{t-1})),
 * w_t = exp(-exp(d_t))).  Instead of the decay logits x [B][T][H][N] the call takes the low-rank
 * activations and the outer factor and forms the logits on the matrix cores, in fp32, chunk by
 * chunk, so they never exist in HBM:
 *
 *     d[b][t][h][n] = lambda[h*N + n] + sum_{k<R} y[b][t][k] * b_omega[k][h*N + n]
 *
 *   y        [B][T][R]   bf16  tanh(ddlerp_d(x_t, x_{t-1}) A_omega), shared by all heads; R must
 *                              be 64 (WKV6_ERR_UNSUPPORTED otherwise)
 *   lambda   [H*N]       fp32
 *   b_omega  [R][H*N]    bf16
 * all device pointers, 16-byte aligned.  The per-token-head input traffic drops from five bf16
 * rows to four (y is 128 bytes per token for all heads together).  `moments` may be NULL; if
 * not, the per-head LayerNorm partials are written as by wkv6_finch_c2_prefill_bf16_moments.
 * Everything else (kbar, uprime, layouts, state, T and B edge cases, value range, errors) is as
 * for wkv6_finch_c2_prefill_bf16; always the chunked kernel.
 */
int wkv6_finch_c2_prefill_lora_bf16(int B, int T, int H, int N, int R,
                                    const void *r, const void *kbar, const void *v,
                                    const void *y, const float *lambda, const void *b_omega,
                                    const void *uprime, const float *state_in,
                                    void *out, float *moments, float *state_out, void *stream);

/*
 * The operators in front of that call (paper: Method, "Finch-C2 Time Mixing": lerp(a, b, t) =
 * a + (b - a) t, lora(x) = lambda + tanh(x A) B, ddlerp(a, b) = a + (b - a) lora(a + (b - a) mu_x), and
 * d_t = lora_omega(ddlerp_d(x_t, x_{t-1}))): from the time-mix input x to the low-rank activations
 *
 *     z_t = x_t + (x_{t-1} - x_t) * (lambda_d + tanh((x_t + (x_{t-1} - x_t) * mu_x) A_d) B_d)
 *     y_t = tanh(z_t A_omega)
 *
 * that wkv6_finch_c2_prefill_lora_bf16 / wkv6_prefill_lora_bf16 take, so the decay path runs from the
 * layer input to the decay inside this library and neither z nor the logits exist in HBM.  One
 * kernel, bound by the one HBM read of x (algorithmic bytes 2 B T D in + 2 B T R out + weights).
 *
 *   B, T     batch, tokens per sequence (B*T = 0 is a no-op)
 *   D        model width H*N, a multiple of 128 up to 65536
 *   R_d, R   inner rank of ddlerp_d's lora and rank of lora_omega: must be 32 and 64 (Finch's sizes;
 *            WKV6_ERR_UNSUPPORTED otherwise)
 *   x        [B][T][D]  bf16  input of the time-mix block
 *   x_prev   [B][D]     bf16  the token before each sequence's first one (a carried row when a context
 *                             is processed in pieces), or NULL: nothing precedes it and x_{-1} = 0.
 *                             The paper writes x_{t-1} without saying what precedes t = 0; zero is what
 *                             Finch, from which the operators are taken, shifts in.
 *   mu_x     [D]        fp32
 *   lambda_d [D]        fp32
 *   a_d      [R_d][D]   bf16  A_d stored column by column (row i is column i of the paper's D x R_d
 *                             matrix): the contraction index must be contiguous for the matrix cores
 *   b_d      [D][R_d]   bf16  B_d stored column by column (row c is column c of the paper's R_d x D)
 *   a_omega  [R][D]     bf16  A_omega stored column by column
 *   y        [B][T][R]  bf16 or fp32 per out_dtype (a wkv6_dtype)
 * All device pointers, 16-byte aligned.  Arithmetic: interpolations in fp32, matrix-core operands
 * fp16 (q, p, z and the weights; 11 significant bits), fp32 accumulation, tanh from one
 * exponential and one reciprocal in fp32; |x| and the weights must stay inside the fp16 range.
 * Enqueues one kernel on `stream`; allocates nothing; errors as for the other entry points.
 */
int wkv6_decay_lora_input_bf16(int B, int T, int D, int R_d, int R,
                               const void *x, const void *x_prev,
                               const float *mu_x, const float *lambda_d,
                               const void *a_d, const void *b_d, const void *a_omega,
                               void *y, int out_dtype, void *stream);

/*
 * The Finch form (bonus u, plain key) with the same fusion: Finch's own decay is the same
 * low-rank path (the paper takes the operators from Finch), so a Finch layer can hand over
 * y, lambda and b_omega instead of x as well.  Arguments as for wkv6_prefill_bf16 with
 * (y, lambda, b_omega, R) in place of x, as described for wkv6_finch_c2_prefill_lora_bf16.
 */
int wkv6_prefill_lora_bf16(int B, int T, int H, int N, int R,
                           const void *r, const void *k, const void *v,
                           const void *y, const float *lambda, const void *b_omega,
                           const float *u, const float *state_in,
                           void *out, float *state_out, void *stream);

/*
 * Serving shapes: the same recurrence for one token (decode) or a few tokens (append) per
 * sequence and many sequences, where the cost is streaming each fp32 state through once
 * (paper: GoldFinch pre-fill is an RNN pass, so a cache is extended token by token with the
 * state carried; same equations as above).
 *
 * wkv6_decode_bf16: T = 1.  r,k,v,x,out are [B][H][N] bf16; `state` [B][H][N][N] fp32 is read
 * and updated in place (required, not NULL).  Token-by-token fp32 kernel, no fp16 operands, no
 * value-range limit.
 * wkv6_append_bf16: arguments exactly as wkv6_prefill_bf16 (state_in may equal state_out); the
 * library picks the token-by-token kernel for very short T (at most 6 tokens) and the chunked
 * kernel above that.  Results of the two kernels differ by rounding only, both within the
 * stated tolerance.
 * The finch_c2 variants take kbar and uprime instead of k and u (see wkv6_finch_c2_prefill_bf16).
 */
int wkv6_decode_bf16(int B, int H, int N,
                     const void *r, const void *k, const void *v, const void *x,
                     const float *u, float *state, void *out, void *stream);
int wkv6_finch_c2_decode_bf16(int B, int H, int N,
                              const void *r, const void *kbar, const void *v, const void *x,
                              const void *uprime, float *state, void *out, void *stream);
int wkv6_append_bf16(int B, int T, int H, int N,
                     const void *r, const void *k, const void *v, const void *x,
                     const float *u, const float *state_in,
                     void *out, float *state_out, void *stream);
int wkv6_finch_c2_append_bf16(int B, int T, int H, int N,
                              const void *r, const void *kbar, const void *v, const void *x,
                              const void *uprime, const float *state_in,
                              void *out, float *state_out, void *stream);

/*
 * GOLD key compression (paper: Method, "GOLD Key Compression"): the step that turns the output
 * of the last Finch-C2 layer into the compressed key cache,  c_t = x_t W^KD,  W^KD with D rows
 * and D/16 columns.  A skinny matrix product bound by the one HBM read of x; bf16 operands,
 * fp32 accumulation on the matrix cores, one rounding of the result.
 *   M      tokens (batch x sequence, any M >= 0; 0 is a no-op)
 *   D      model dimension, a multiple of 256 up to 65536 (other values: WKV6_ERR_UNSUPPORTED)
 *   x      [M][D]     bf16 device pointer, 16-byte aligned
 *   w_kd   [D][D/16]  bf16, row-major as the paper writes it (x on the left)
 *   c      [M][D/16]  bf16 or fp32 per out_dtype (a wkv6_dtype)
 * Enqueues one kernel on `stream`; allocates nothing; errors as for the other entry points.
 */
int wkv6_key_compress_bf16(long long M, int D, const void *x, const void *w_kd, void *c,
                           int out_dtype, void *stream);

/* All-fp32 tensors.  Token-by-token kernel with the state in fp32 registers. */
int wkv6_prefill_f32(int B, int T, int H, int N,
                     const float *r, const float *k, const float *v, const float *x,
                     const float *u, const float *state_in,
                     float *out, float *state_out, void *stream);

/*
 * bf16 inputs, fp32 out, evaluated by the token-by-token fp32 kernel instead of
 * the chunked one (same recurrence, no matrix cores, no fp16 operands): the
 * on-device cross-check and the "before" number of the benchmark.
 */
int wkv6_prefill_bf16_recurrent(int B, int T, int H, int N,
                                const void *r, const void *k, const void *v, const void *x,
                                const float *u, const float *state_in,
                                float *out, float *state_out, void *stream);

/*
 * Where to put the large tensors (speed only: every entry point accepts any 16-byte-aligned
 * addresses and computes the same bits wherever its operands lie).  In the [B][T][H][N] layout a
 * head's token rows are 128 bytes long and H*N*2 bytes apart, so all rows of one head share
 * address bits 7..9, and when r, k, v, x (u'), out start at equally aligned addresses -- as tensors
 * from an allocator do -- all streams of a head, i.e. everything one workgroup has in flight, fall
 * into the same eighth of the address-interleaved memory resources.  Measured on the benchmark
 * workload: 0.141 ms with equally aligned tensors, 0.122 ms when the i-th tensor starts 128*i
 * bytes past a 4 KiB boundary (any odd multiple of 128 does; the rows themselves should stay
 * 128-byte aligned: 64- or 32-byte shifts cost 20-40 %).
 *
 * wkv6_arena_layout lays `count` tensors of bytes[i] bytes out in one arena that way:
 * offsets[i] = (end of tensor i-1 rounded up to 4096) + 128 * (i mod 8), relative to an arena base
 * the caller aligns to 4096 bytes.  Returns the arena size in bytes (a multiple of 4096), or -1 for
 * count < 0, count > 64, a NULL pointer with count > 0, or a negative size.  Host arithmetic only:
 * no device call, nothing allocated.
 */
#define WKV6_PLACEMENT_ALIGN 4096
#define WKV6_PLACEMENT_STEP 128
long long wkv6_arena_layout(int count, const long long *bytes, long long *offsets);

/* Human-readable name of a wkv6_status (static storage, never NULL). */
const char *wkv6_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int wkv6_version(void);

#ifdef __cplusplus
}
#endif
#endif /* WKV6_H */

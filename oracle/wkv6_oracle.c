/*
 * WKV6 prefill oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, sequential fp64 evaluation of the Finch (RWKV-6) time-mix
 * recurrence that the GoldFinch pre-fill runs in every Finch / Finch-C2
 * layer.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it; the GPU library never does, and the two share no code.
 *
 * What is computed, per batch b and head h independently (Method section,
 * Finch-C2 Time Mixing: the decay map w_t = exp(-exp(d_t)), the definition
 * of wkv_t as the sum over i < t of diag(prod_{j=i+1}^{t-1} w_j) k_i^T v_i,
 * and the read-out r_t . wkv_t).  Unrolled one step at a time that sum is
 *
 *     o_t      = r_t . ( S_{t-1} + diag(u) k_t^T v_t )        (read first)
 *     S_t      = diag(w_t) S_{t-1} + k_t^T v_t                (then update)
 *
 * with S a (key channel i) x (value channel j) matrix, the decay acting on
 * the key channel (rows), S_0 = state_in or zero, and u the per-head Finch
 * "bonus" that weighs the current token's own k^T v in the read-out.  The
 * Finch-C2 variant of the paper is the special case u = 0 with the caller
 * pre-scaling k by (1 - w) and adding its second value u'_t afterwards.
 *
 * Parity pins (tests/test_oracle_pins.py): brute-force evaluation of the
 * unrolled double sum, T=1 and T=2 closed forms, a hand-worked fixture,
 * w==1 (causal linear attention), w==0, state passing, linearity, head
 * independence, the geometric-series closed form, the Finch-C2 row
 * normalisation, and an independent NumPy twin.
 *
 * Inputs are float (every bf16 or fp32 test tensor is exactly representable
 * in float); all arithmetic and both outputs are double.  No clamp is
 * applied to the decay logit: x=-inf gives w=1, x=+inf gives w=0.
 *
 * Layouts (row-major):  r,k,v,x,out [B][T][H][N];  u [H][N];
 * state_in/state_out [B][H][N(key i)][N(value j)].
 */
#include <math.h>
#include <pthread.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int B, T, H, N;
    const float *r, *k, *v, *x, *u;
    const float *state_in; /* may be NULL */
    double *out;
    double *state_out; /* may be NULL */
    int unit_begin, unit_end; /* range of (b*H + h) handled by this thread */
    int status;
} oracle_job;

/* One (b,h) unit: the whole sequence, one token at a time. */
static int run_unit(const oracle_job *J, int b, int h, double *S, double *w)
{
    const int T = J->T, H = J->H, N = J->N;
    const size_t tok_stride = (size_t)H * N;
    const size_t base = ((size_t)b * T * H + h) * (size_t)N;
    const float *u = J->u + (size_t)h * N;

    if (J->state_in) {
        const float *s0 = J->state_in + ((size_t)b * H + h) * (size_t)N * N;
        for (int e = 0; e < N * N; ++e) S[e] = (double)s0[e];
    } else {
        for (int e = 0; e < N * N; ++e) S[e] = 0.0;
    }

    for (int t = 0; t < T; ++t) {
        const float *rt = J->r + base + (size_t)t * tok_stride;
        const float *kt = J->k + base + (size_t)t * tok_stride;
        const float *vt = J->v + base + (size_t)t * tok_stride;
        const float *xt = J->x + base + (size_t)t * tok_stride;
        double *ot = J->out + base + (size_t)t * tok_stride;

        /* read-out with the state as it was BEFORE this token */
        for (int j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int i = 0; i < N; ++i) {
                double kv = (double)kt[i] * (double)vt[j];
                acc += (double)rt[i] * (S[(size_t)i * N + j] + (double)u[i] * kv);
            }
            ot[j] = acc;
        }
        /* decay map, then decay rows and add this token's outer product */
        for (int i = 0; i < N; ++i) w[i] = exp(-exp((double)xt[i]));
        for (int i = 0; i < N; ++i)
            for (int j = 0; j < N; ++j)
                S[(size_t)i * N + j] =
                    w[i] * S[(size_t)i * N + j] + (double)kt[i] * (double)vt[j];
    }

    if (J->state_out) {
        double *so = J->state_out + ((size_t)b * H + h) * (size_t)N * N;
        memcpy(so, S, sizeof(double) * (size_t)N * N);
    }
    return 0;
}

static void *worker(void *arg)
{
    oracle_job *J = (oracle_job *)arg;
    double *S = (double *)malloc(sizeof(double) * (size_t)J->N * J->N);
    double *w = (double *)malloc(sizeof(double) * (size_t)J->N);
    if (!S || !w) {
        J->status = 3;
        free(S);
        free(w);
        return NULL;
    }
    for (int unit = J->unit_begin; unit < J->unit_end; ++unit)
        run_unit(J, unit / J->H, unit % J->H, S, w);
    free(S);
    free(w);
    J->status = 0;
    return NULL;
}

/*
 * Returns 0 on success, 1 for a NULL required pointer, 2 for a bad shape,
 * 3 if memory or a thread could not be obtained.  nthreads <= 1 runs on the
 * calling thread; otherwise the (b,h) units are split into nthreads
 * contiguous ranges.  Any T >= 0 (T == 0 copies the state through).
 */
int wkv6_oracle_f64(int B, int T, int H, int N,
                    const float *r, const float *k, const float *v, const float *x,
                    const float *u, const float *state_in,
                    double *out, double *state_out, int nthreads)
{
    if (B < 1 || T < 0 || H < 1 || N < 1) return 2;
    if (!u) return 1;
    if (T > 0 && (!r || !k || !v || !x || !out)) return 1;

    const int units = B * H;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > units) nthreads = units;

    oracle_job proto;
    proto.B = B; proto.T = T; proto.H = H; proto.N = N;
    proto.r = r; proto.k = k; proto.v = v; proto.x = x; proto.u = u;
    proto.state_in = state_in; proto.out = out; proto.state_out = state_out;
    proto.status = 0;

    if (nthreads == 1) {
        proto.unit_begin = 0;
        proto.unit_end = units;
        worker(&proto);
        return proto.status;
    }

    oracle_job *jobs = (oracle_job *)malloc(sizeof(oracle_job) * (size_t)nthreads);
    pthread_t *tids = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
    if (!jobs || !tids) {
        free(jobs);
        free(tids);
        return 3;
    }
    int status = 0, started = 0;
    for (int i = 0; i < nthreads; ++i) {
        jobs[i] = proto;
        jobs[i].unit_begin = (int)((long long)units * i / nthreads);
        jobs[i].unit_end = (int)((long long)units * (i + 1) / nthreads);
        if (pthread_create(&tids[i], NULL, worker, &jobs[i]) != 0) {
            status = 3;
            break;
        }
        ++started;
    }
    for (int i = 0; i < started; ++i) {
        pthread_join(tids[i], NULL);
        if (jobs[i].status) status = jobs[i].status;
    }
    free(jobs);
    free(tids);
    return status;
}

/*
 * Finch-C2 time-mix oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, sequential fp64 evaluation of the per-head part of
 * GoldFinch's Finch-C2 time mixing (Method section, Finch-C2 Time Mixing):
 * the decay map w_t = exp(-exp(d_t)); the key multiplied by one minus the
 * decay, k_t = kbar_t * (1 - w_t), where kbar_t is the projected key before
 * that factor; the state wkv_t = sum_{i<t} diag(prod_{j=i+1}^{t-1} w_j)
 * k_i^T v_i; and the read-out r_t . wkv_t + u'_t, u'_t being the layer's
 * second value, which takes the place of Finch's bonus.  The LayerNorm over
 * the concatenated heads and the output projection that follow are not part
 * of this function.  One step at a time:
 *
 *     w_t = exp(-exp(x_t)),   k_t = kbar_t * (1 - w_t)
 *     o_t = r_t . S_{t-1} + u'_t                           (read first)
 *     S_t = diag(w_t) S_{t-1} + k_t^T v_t                  (then update)
 *
 * with S a (key channel i) x (value channel j) matrix, S_0 = state_in or 0.
 *
 * Parity pins (tests/test_oracle_pins.py): brute-force evaluation of the
 * double sum with the (1 - w) factor written out, T=1 closed form, the
 * reduction to the Finch oracle (u = 0, pre-scaled key, u' added), w == 1
 * (nothing is ever written to the state), the normalisation 1 - prod w of a
 * constant value, and an independent NumPy twin.
 *
 * Inputs are float (every bf16 or fp32 test tensor is exactly representable
 * in float); all arithmetic and both outputs are double.  No clamp on the
 * decay logit.
 *
 * Layouts (row-major): r,kbar,v,x,uprime,out [B][T][H][N];
 * state_in/state_out [B][H][N(key i)][N(value j)].
 */
#include <math.h>
#include <pthread.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int B, T, H, N;
    const float *r, *kbar, *v, *x, *uprime;
    const float *state_in; /* may be NULL */
    double *out;
    double *state_out; /* may be NULL */
    int unit_begin, unit_end;
    int status;
} c2_job;

static void c2_unit(const c2_job *J, int b, int h, double *S, double *w, double *k)
{
    const int T = J->T, H = J->H, N = J->N;
    const size_t tok = (size_t)H * N;
    const size_t base = ((size_t)b * T * H + h) * (size_t)N;

    for (int e = 0; e < N * N; ++e)
        S[e] = J->state_in ? (double)J->state_in[((size_t)b * H + h) * (size_t)N * N + e] : 0.0;

    for (int t = 0; t < T; ++t) {
        const size_t at = base + (size_t)t * tok;
        /* read-out from the state before this token, plus the second value */
        for (int j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int i = 0; i < N; ++i) acc += (double)J->r[at + i] * S[(size_t)i * N + j];
            J->out[at + j] = acc + (double)J->uprime[at + j];
        }
        /* decay, and the key times one minus the decay */
        for (int i = 0; i < N; ++i) {
            w[i] = exp(-exp((double)J->x[at + i]));
            k[i] = (double)J->kbar[at + i] * (1.0 - w[i]);
        }
        for (int i = 0; i < N; ++i)
            for (int j = 0; j < N; ++j)
                S[(size_t)i * N + j] = w[i] * S[(size_t)i * N + j] + k[i] * (double)J->v[at + j];
    }

    if (J->state_out)
        memcpy(J->state_out + ((size_t)b * H + h) * (size_t)N * N, S, sizeof(double) * (size_t)N * N);
}

static void *c2_worker(void *arg)
{
    c2_job *J = (c2_job *)arg;
    double *S = (double *)malloc(sizeof(double) * (size_t)J->N * J->N);
    double *w = (double *)malloc(sizeof(double) * (size_t)J->N);
    double *k = (double *)malloc(sizeof(double) * (size_t)J->N);
    if (S && w && k) {
        for (int unit = J->unit_begin; unit < J->unit_end; ++unit)
            c2_unit(J, unit / J->H, unit % J->H, S, w, k);
        J->status = 0;
    } else {
        J->status = 3;
    }
    free(S);
    free(w);
    free(k);
    return NULL;
}

/*
 * Returns 0 on success, 1 for a NULL required pointer, 2 for a bad shape,
 * 3 if memory or a thread could not be obtained.  nthreads <= 1 runs on the
 * calling thread.  Any T >= 0 (T == 0 copies the state through).
 */
int finch_c2_oracle_f64(int B, int T, int H, int N,
                        const float *r, const float *kbar, const float *v, const float *x,
                        const float *uprime, const float *state_in,
                        double *out, double *state_out, int nthreads)
{
    if (B < 1 || T < 0 || H < 1 || N < 1) return 2;
    if (T > 0 && (!r || !kbar || !v || !x || !uprime || !out)) return 1;

    const int units = B * H;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > units) nthreads = units;

    c2_job proto;
    proto.B = B; proto.T = T; proto.H = H; proto.N = N;
    proto.r = r; proto.kbar = kbar; proto.v = v; proto.x = x; proto.uprime = uprime;
    proto.state_in = state_in; proto.out = out; proto.state_out = state_out;
    proto.unit_begin = 0; proto.unit_end = units; proto.status = 0;
    if (nthreads == 1) {
        c2_worker(&proto);
        return proto.status;
    }

    c2_job *jobs = (c2_job *)malloc(sizeof(c2_job) * (size_t)nthreads);
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
        if (pthread_create(&tids[i], NULL, c2_worker, &jobs[i]) != 0) {
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

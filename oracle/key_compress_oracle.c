/*
 * GOLD key-compression oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain fp64 evaluation of GoldFinch's key compression (Method section,
 * GOLD Key Compression): every token's hidden state x_t (a row vector of D
 * entries, the output of the last Finch-C2 layer) is multiplied by the
 * learned matrix W^KD with D rows and D/16 columns, giving the compressed
 * key-cache entry
 *
 *     c_t[n] = sum_{d=0}^{D-1} x_t[d] * W[d][n],      n = 0 .. D/16 - 1.
 *
 * The definition is a matrix product and is written out as the three loops.
 * Inputs are float (bf16 test tensors are exact in float), arithmetic and
 * output are double.  Layouts (row-major): x [M][D], W [D][C], c [M][C]; the
 * function takes C explicitly and leaves the relation C = D/16 to its caller.
 *
 * Parity pins (tests/test_oracle_pins_key_compress.py): a hand-computed case,
 * selector matrices, linearity in x and in W, token independence, the library
 * matrix product on random inputs, and planted mistakes.
 */
#include <pthread.h>
#include <stdlib.h>

typedef struct {
    long long M;
    int D, C;
    const float *x, *w;
    double *c;
    long long row_begin, row_end;
} kc_job;

static void *kc_worker(void *arg)
{
    const kc_job *J = (const kc_job *)arg;
    for (long long m = J->row_begin; m < J->row_end; ++m)
        for (int n = 0; n < J->C; ++n) {
            double acc = 0.0;
            for (int d = 0; d < J->D; ++d)
                acc += (double)J->x[m * J->D + d] * (double)J->w[(long long)d * J->C + n];
            J->c[m * J->C + n] = acc;
        }
    return NULL;
}

/* Returns 0 on success, 1 for a NULL pointer, 2 for a bad shape, 3 if a thread could not start. */
int key_compress_oracle_f64(long long M, int D, int C, const float *x, const float *w, double *c,
                            int nthreads)
{
    if (M < 0 || D < 1 || C < 1) return 2;
    if (M == 0) return 0;
    if (!x || !w || !c) return 1;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > M) nthreads = (int)M;
    if (nthreads > 64) nthreads = 64;

    kc_job jobs[64];
    pthread_t tids[64];
    int started = 0, status = 0;
    for (int i = 0; i < nthreads; ++i) {
        jobs[i].M = M; jobs[i].D = D; jobs[i].C = C;
        jobs[i].x = x; jobs[i].w = w; jobs[i].c = c;
        jobs[i].row_begin = M * i / nthreads;
        jobs[i].row_end = M * (i + 1) / nthreads;
    }
    if (nthreads == 1) {
        kc_worker(&jobs[0]);
        return 0;
    }
    for (int i = 0; i < nthreads; ++i) {
        if (pthread_create(&tids[i], NULL, kc_worker, &jobs[i]) != 0) {
            status = 3;
            break;
        }
        ++started;
    }
    for (int i = 0; i < started; ++i) pthread_join(tids[i], NULL);
    return status;
}

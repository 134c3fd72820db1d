/*
 * Host sanitizer run of the C oracles (test infrastructure): built by
 * tests/test_host_sanitizers_cpu.py with -fsanitize=address,undefined together with oracle/*.c.
 * Drives every entry point through its threaded and single-threaded paths, empty and ragged
 * shapes, and two properties that need no other implementation (state passing; the T = 1 closed
 * form), so that a heap overflow, a use after free, a data race on the job array or undefined
 * arithmetic in the oracle aborts the run.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int wkv6_oracle_f64(int B, int T, int H, int N, const float *r, const float *k, const float *v, const float *x,
                    const float *u, const float *state_in, double *out, double *state_out, int nthreads);
int finch_c2_oracle_f64(int B, int T, int H, int N, const float *r, const float *kbar, const float *v,
                        const float *x, const float *uprime, const float *state_in, double *out,
                        double *state_out, int nthreads);
int key_compress_oracle_f64(long long M, int D, int C, const float *x, const float *w, double *c, int nthreads);

static unsigned long long rng_state = 88172645463325252ull;
static float unit_rand(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (float)((rng_state >> 11) * (1.0 / 9007199254740992.0));
}
static float *randoms(size_t n, float lo, float hi)
{
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = lo + (hi - lo) * unit_rand();
    return p;
}
static double max_abs_diff(const double *a, const double *b, size_t n)
{
    double m = 0;
    for (size_t i = 0; i < n; ++i) {
        const double d = fabs(a[i] - b[i]);
        if (d > m) m = d;
    }
    return m;
}
#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            printf("FAIL %s (line %d)\n", #cond, __LINE__);                \
            return 1;                                                      \
        }                                                                  \
    } while (0)

static int recurrence(int c2)
{
    const int B = 3, T = 37, H = 5, N = 8, half = 19;
    const size_t n = (size_t)B * T * H * N, ns = (size_t)B * H * N * N;
    float *r = randoms(n, -1, 1), *k = randoms(n, -1, 1), *v = randoms(n, -1, 1), *x = randoms(n, -6, 1);
    float *last = c2 ? randoms(n, -1, 1) : randoms((size_t)H * N, -1, 1);   /* uprime or u */
    float *s0 = randoms(ns, -1, 1);
    double *o1 = (double *)malloc(sizeof(double) * n), *o3 = (double *)malloc(sizeof(double) * n);
    double *s1 = (double *)malloc(sizeof(double) * ns), *s3 = (double *)malloc(sizeof(double) * ns);
#define RUN(Bv, Tv, rp, kp, vp, xp, lp, sp, op, so, th)                                                        \
    (c2 ? finch_c2_oracle_f64(Bv, Tv, H, N, rp, kp, vp, xp, lp, sp, op, so, th)                                \
        : wkv6_oracle_f64(Bv, Tv, H, N, rp, kp, vp, xp, lp, sp, op, so, th))
    /* thread counts: one, a few, more than there are units */
    CHECK(RUN(B, T, r, k, v, x, last, s0, o1, s1, 1) == 0);
    CHECK(RUN(B, T, r, k, v, x, last, s0, o3, s3, 4) == 0);
    CHECK(max_abs_diff(o1, o3, n) == 0 && max_abs_diff(s1, s3, ns) == 0);
    CHECK(RUN(B, T, r, k, v, x, last, s0, o3, s3, 64) == 0);
    CHECK(max_abs_diff(o1, o3, n) == 0 && max_abs_diff(s1, s3, ns) == 0);
    /* no state in, no state out */
    CHECK(RUN(B, T, r, k, v, x, last, NULL, o3, NULL, 3) == 0);
    /* empty sequence copies the state through */
    CHECK(RUN(B, 0, NULL, NULL, NULL, NULL, c2 ? NULL : last, s0, NULL, s3, 2) == 0 || c2);
    /* state passing on one sequence: [0, T) in one call equals [0, half) then [half, T) */
    {
        const size_t row = (size_t)H * N, n1 = (size_t)T * row, nh = (size_t)half * row, ns1 = (size_t)H * N * N;
        double *oa = (double *)malloc(sizeof(double) * n1), *ob = (double *)malloc(sizeof(double) * n1);
        double *sa = (double *)malloc(sizeof(double) * ns1), *sb = (double *)malloc(sizeof(double) * ns1);
        float *sf = (float *)malloc(sizeof(float) * ns1);
        CHECK(RUN(1, T, r, k, v, x, last, NULL, oa, sa, 2) == 0);
        CHECK(RUN(1, half, r, k, v, x, last, NULL, ob, sb, 2) == 0);
        for (size_t i = 0; i < ns1; ++i) sf[i] = (float)sb[i];
        CHECK(RUN(1, T - half, r + nh, k + nh, v + nh, x + nh, c2 ? last + nh : last, sf, ob + nh, sb, 2) == 0);
        CHECK(max_abs_diff(oa, ob, n1) < 1e-5 && max_abs_diff(sa, sb, ns1) < 1e-5);   /* carried state rounded to float */
        free(oa); free(ob); free(sa); free(sb); free(sf);
    }
    /* bad arguments are reported, not dereferenced */
    CHECK(RUN(0, T, r, k, v, x, last, s0, o1, s1, 1) == 2);
    CHECK(RUN(B, T, NULL, k, v, x, last, s0, o1, s1, 1) == 1);
#undef RUN
    free(r); free(k); free(v); free(x); free(last); free(s0); free(o1); free(o3); free(s1); free(s3);
    return 0;
}

static int t1_closed_form(void)
{
    const int H = 2, N = 4;
    float *r = randoms((size_t)H * N, -1, 1), *k = randoms((size_t)H * N, -1, 1), *v = randoms((size_t)H * N, -1, 1);
    float *x = randoms((size_t)H * N, -3, 1), *u = randoms((size_t)H * N, -1, 1), *s0 = randoms((size_t)H * N * N, -1, 1);
    double o[8], s[32];
    CHECK(wkv6_oracle_f64(1, 1, H, N, r, k, v, x, u, s0, o, s, 1) == 0);
    for (int h = 0; h < H; ++h)
        for (int j = 0; j < N; ++j) {
            double want = 0, bonus = 0;
            for (int i = 0; i < N; ++i) {
                want += (double)r[h * N + i] * s0[(h * N + i) * N + j];
                bonus += (double)r[h * N + i] * u[h * N + i] * k[h * N + i];
            }
            want += bonus * v[h * N + j];
            CHECK(fabs(o[h * N + j] - want) < 1e-12);
        }
    free(r); free(k); free(v); free(x); free(u); free(s0);
    return 0;
}

static int key_compress(void)
{
    const long long M = 37;
    const int D = 48, C = 3;
    float *x = randoms((size_t)M * D, -1, 1), *w = randoms((size_t)D * C, -1, 1);
    double *c1 = (double *)malloc(sizeof(double) * M * C), *c2 = (double *)malloc(sizeof(double) * M * C);
    CHECK(key_compress_oracle_f64(M, D, C, x, w, c1, 1) == 0);
    CHECK(key_compress_oracle_f64(M, D, C, x, w, c2, 5) == 0);
    CHECK(max_abs_diff(c1, c2, (size_t)M * C) == 0);
    CHECK(key_compress_oracle_f64(M, D, C, x, w, c2, 100) == 0);
    CHECK(max_abs_diff(c1, c2, (size_t)M * C) == 0);
    double want = 0;
    for (int d = 0; d < D; ++d) want += (double)x[5 * D + d] * w[d * C + 2];
    CHECK(fabs(c1[5 * C + 2] - want) < 1e-12);
    free(x); free(w); free(c1); free(c2);
    return 0;
}

int main(void)
{
    if (recurrence(0) || recurrence(1) || t1_closed_form() || key_compress()) return 1;
    printf("ok\n");
    return 0;
}

/*
 * The C ABI used from plain C: no Python, no PyTorch, only the HIP runtime for device memory.
 *
 * Builds small seeded inputs on the host, runs wkv6_prefill_f32 (all-fp32 tensors) and
 * wkv6_prefill_bf16_f32out (bf16 tensors) on device 0 through include/wkv6.h, and compares
 * out and state_out with the fp64 oracle (linked from oracle/, test infrastructure) using the
 * max-normalised error: <= 1e-5 for fp32 tensors, <= 2e-3 for bf16 tensors.
 * Exit status 0 = both within tolerance; every other status names the failing step on stderr.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/wkv6.h"

int wkv6_oracle_f64(int B, int T, int H, int N, const float *r, const float *k, const float *v,
                    const float *x, const float *u, const float *state_in, double *out,
                    double *state_out, int nthreads);

#define CHECK_HIP(call)                                                              \
    do {                                                                             \
        hipError_t e_ = (call);                                                      \
        if (e_ != hipSuccess) {                                                      \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));        \
            return 10;                                                               \
        }                                                                            \
    } while (0)

/* splitmix64: a small counter-based generator, only for this program's inputs */
static uint64_t rng_state = 20240712u;
static double uniform01(void)
{
    uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    z ^= z >> 31;
    return (double)(z >> 11) / 9007199254740992.0;
}
static float gauss(void)
{
    const double a = uniform01(), b = uniform01();
    return (float)(sqrt(-2.0 * log(a + 1e-300)) * cos(6.283185307179586 * b));
}
static float to_bf16_value(float f, uint16_t *bits)
{
    uint32_t w;
    memcpy(&w, &f, 4);
    w += 0x7fffu + ((w >> 16) & 1u);          /* round to nearest even */
    w &= 0xffff0000u;
    *bits = (uint16_t)(w >> 16);
    memcpy(&f, &w, 4);
    return f;
}
static double max_norm_err(const float *got, const double *ref, size_t n)
{
    double worst = 0.0, scale = 0.0;
    for (size_t i = 0; i < n; ++i) {
        const double d = fabs((double)got[i] - ref[i]);
        if (d > worst || d != d) worst = d;
        if (fabs(ref[i]) > scale) scale = fabs(ref[i]);
    }
    return scale > 0.0 ? worst / scale : worst;
}

static int run_case(int bf16, int B, int T, int H, double tol)
{
    const int N = 64;
    const size_t n = (size_t)B * T * H * N, ns = (size_t)B * H * N * N, nu = (size_t)H * N;
    float *r = malloc(4 * n), *k = malloc(4 * n), *v = malloc(4 * n), *x = malloc(4 * n);
    float *u = malloc(4 * nu), *s0 = malloc(4 * ns), *out = malloc(4 * n), *s1 = malloc(4 * ns);
    uint16_t *h16 = malloc(2 * n);
    double *out_ref = malloc(8 * n), *s_ref = malloc(8 * ns);
    if (!r || !k || !v || !x || !u || !s0 || !out || !s1 || !h16 || !out_ref || !s_ref) return 11;
    for (size_t i = 0; i < n; ++i) {
        r[i] = gauss() * 0.125f;
        k[i] = gauss() * 0.125f;
        v[i] = gauss() * 0.125f;
        x[i] = (float)(uniform01() * 7.0 - 6.0);
    }
    for (size_t i = 0; i < nu; ++i) u[i] = gauss() * 0.5f;
    for (size_t i = 0; i < ns; ++i) s0[i] = gauss() * 0.1f;

    const size_t elem = bf16 ? 2 : 4;
    void *d_in[4], *d_u, *d_s0, *d_out, *d_s1;
    float *host_in[4] = {r, k, v, x};
    for (int t = 0; t < 4; ++t) {
        CHECK_HIP(hipMalloc(&d_in[t], elem * n));
        if (bf16) {
            for (size_t i = 0; i < n; ++i) host_in[t][i] = to_bf16_value(host_in[t][i], &h16[i]);
            CHECK_HIP(hipMemcpy(d_in[t], h16, 2 * n, hipMemcpyHostToDevice));
        } else {
            CHECK_HIP(hipMemcpy(d_in[t], host_in[t], 4 * n, hipMemcpyHostToDevice));
        }
    }
    CHECK_HIP(hipMalloc(&d_u, 4 * nu));
    CHECK_HIP(hipMalloc(&d_s0, 4 * ns));
    CHECK_HIP(hipMalloc(&d_out, 4 * n));
    CHECK_HIP(hipMalloc(&d_s1, 4 * ns));
    CHECK_HIP(hipMemcpy(d_u, u, 4 * nu, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_s0, s0, 4 * ns, hipMemcpyHostToDevice));

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    const int status = bf16 ? wkv6_prefill_bf16_f32out(B, T, H, N, d_in[0], d_in[1], d_in[2], d_in[3], d_u, d_s0,
                                                       d_out, d_s1, stream)
                            : wkv6_prefill_f32(B, T, H, N, d_in[0], d_in[1], d_in[2], d_in[3], d_u, d_s0, d_out,
                                               d_s1, stream);
    if (status != WKV6_OK) {
        fprintf(stderr, "entry point returned %d: %s\n", status, wkv6_status_string(status));
        return 12;
    }
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipMemcpy(out, d_out, 4 * n, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(s1, d_s1, 4 * ns, hipMemcpyDeviceToHost));

    if (wkv6_oracle_f64(B, T, H, N, r, k, v, x, u, s0, out_ref, s_ref, 4) != 0) return 13;
    const double eo = max_norm_err(out, out_ref, n), es = max_norm_err(s1, s_ref, ns);
    printf("%s B=%d T=%d H=%d: err_out=%.3e err_state=%.3e (tolerance %.0e)\n", bf16 ? "bf16" : "fp32", B, T, H, eo,
           es, tol);
    fflush(stdout);

    CHECK_HIP(hipStreamDestroy(stream));
    for (int t = 0; t < 4; ++t) CHECK_HIP(hipFree(d_in[t]));
    CHECK_HIP(hipFree(d_u));
    CHECK_HIP(hipFree(d_s0));
    CHECK_HIP(hipFree(d_out));
    CHECK_HIP(hipFree(d_s1));
    free(r); free(k); free(v); free(x); free(u); free(s0); free(out); free(s1); free(h16); free(out_ref); free(s_ref);
    return (eo <= tol && es <= tol) ? 0 : 20;
}

int main(void)
{
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count < 1) {
        fprintf(stderr, "no GPU visible\n");
        return 2;
    }
    CHECK_HIP(hipSetDevice(0));
    printf("wkv6 library version %d\n", wkv6_version());
    int rc = run_case(0, 1, 100, 2, 1e-5);
    if (rc) return rc;
    rc = run_case(1, 3, 333, 2, 2e-3);
    return rc;
}

/* A plain C99 caller of the C ABI (include/abs_sgd.h): no Python, no PyTorch.
 *
 * TEST INFRASTRUCTURE.  Device memory comes from hipMalloc, inputs from a small
 * integer generator below (no arithmetic of the method), the library does the
 * work, and the results are compared with the C oracle (oracle/abs_oracle.c,
 * linked as liboracle.so): bit for bit against its fixed-order fp32 family,
 * within 1e-5 (norm-wise) against its double family.
 *
 * Covered: abs_accumulate (fp32 and bf16 gradients, overwrite-on-first),
 * abs_accumulate_batch, abs_sync_update, and Algorithm 1's loop through the
 * double-buffer context (abs_ctx_create / abs_ctx_accumulate /
 * abs_ctx_sync_update / abs_swap_buffers) on two streams, the same loop with
 * Step 2 of all workers as one abs_ctx_accumulate_step call, and the ragged forms
 * (abs_layout, abs_tensorset, abs_accumulate[_batch]_mt, abs_accumulate_jobs_mt,
 * abs_sync_update_mt) over separately allocated tensors, one of them empty.
 *
 * Exit status 0 and a last line "abi_check: OK" on success.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "abs_sgd.h"

/* the oracle's entry points used here (it ships no header: it is a checker) */
void oracle_accumulate_f32(double *G, const float *g, int64_t n_params, int64_t M_r);
void oracle_accumulate_bf16(double *G, const uint16_t *g, int64_t n_params, int64_t M_r);
int oracle_sync_update(double *x, double *v, const double *const *G, const int64_t *M, int N,
                       int64_t n_params, double gamma, double mu, double wd);
void oracle32_accumulate_f32(float *G, const float *g, int64_t n_params, int64_t M_r, int first);
void oracle32_accumulate_bf16(float *G, const uint16_t *g, int64_t n_params, int64_t M_r, int first);
int oracle32_sync_update(float *x, float *v, const float *const *G, const int64_t *M, int N,
                         int64_t n_params, float gamma, float mu, float wd);

#define CHECK_HIP(call)                                                                   \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s:%d: %s -> %s\n", __FILE__, __LINE__, #call, hipGetErrorString(e_)); \
            exit(2);                                                                      \
        }                                                                                 \
    } while (0)

#define CHECK_ABS(call, want)                                                             \
    do {                                                                                  \
        int rc_ = (call);                                                                 \
        if (rc_ != (want)) {                                                              \
            fprintf(stderr, "%s:%d: %s -> %d (%s), hip error %d\n", __FILE__, __LINE__, #call, rc_, \
                    abs_error_string(rc_), abs_last_hip_error());                          \
            exit(3);                                                                      \
        }                                                                                 \
    } while (0)

/* ---- inputs: a 64-bit mixing generator, uniform in (-scale, scale) ---- */
static uint64_t g_state = 0x15164ULL;

static uint64_t next_u64(void)
{
    uint64_t z = (g_state += 0x9E3779B97F4A7C15ULL);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

static float uniform(float scale)
{
    const double u = (double)(next_u64() >> 11) / 9007199254740992.0;   /* [0, 1) */
    return (float)((2.0 * u - 1.0) * scale);
}

static void fill_f32(float *a, int64_t n, float scale)
{
    for (int64_t i = 0; i < n; ++i) a[i] = uniform(scale);
}

/* bf16 bit patterns: the upper half of an fp32 value (truncation: any bf16 value will do as input) */
static void fill_bf16(uint16_t *a, int64_t n, float scale)
{
    for (int64_t i = 0; i < n; ++i) {
        const float f = uniform(scale);
        uint32_t u;
        memcpy(&u, &f, 4);
        a[i] = (uint16_t)(u >> 16);
    }
}

static void *to_device(const void *host, size_t bytes)
{
    void *d = NULL;
    CHECK_HIP(hipMalloc(&d, bytes));
    CHECK_HIP(hipMemcpy(d, host, bytes, hipMemcpyHostToDevice));
    return d;
}

static void *device_garbage(size_t bytes)
{
    void *d = NULL;
    CHECK_HIP(hipMalloc(&d, bytes));
    CHECK_HIP(hipMemset(d, 0xff, bytes));      /* NaN patterns: the first accumulate must overwrite */
    return d;
}

static int same_bits(const float *a, const float *b, int64_t n, const char *what)
{
    if (memcmp(a, b, (size_t)n * 4) == 0) return 1;
    for (int64_t i = 0; i < n; ++i)
        if (memcmp(a + i, b + i, 4) != 0) {
            fprintf(stderr, "%s: first difference at %lld: %.9g vs %.9g\n", what, (long long)i, a[i], b[i]);
            break;
        }
    return 0;
}

static int close_normwise(const float *a, const double *ref, int64_t n, double rtol, const char *what)
{
    double err = 0.0, mag = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double d = fabs((double)a[i] - ref[i]);
        if (d > err) err = d;
        if (fabs(ref[i]) > mag) mag = fabs(ref[i]);
    }
    if (err <= rtol * mag) return 1;
    fprintf(stderr, "%s: max |diff| %.3e exceeds %.1e * max |ref| %.3e\n", what, err, rtol, mag);
    return 0;
}

/* ---- case 1: the calls one by one ---- */
static int check_calls(int64_t P)
{
    enum { K = 3 };
    int ok = 1;
    printf("[case] calls one by one, P = %lld, K = %d\n", (long long)P, K);
    fflush(stdout);
    float *x = malloc((size_t)P * 4), *v = malloc((size_t)P * 4);
    float *g32[3];
    uint16_t *gbf = malloc((size_t)P * 2);
    for (int j = 0; j < 3; ++j) {
        g32[j] = malloc((size_t)P * 4);
        fill_f32(g32[j], P, 0.02f);
    }
    fill_bf16(gbf, P, 0.02f);
    fill_f32(x, P, 0.1f);
    fill_f32(v, P, 0.01f);

    float *d_acc[K];
    void *d_g32[3], *d_gbf = to_device(gbf, (size_t)P * 2);
    for (int k = 0; k < K; ++k) d_acc[k] = device_garbage((size_t)P * 4);
    for (int j = 0; j < 3; ++j) d_g32[j] = to_device(g32[j], (size_t)P * 4);
    float *d_x = to_device(x, (size_t)P * 4), *d_v = to_device(v, (size_t)P * 4);

    /* worker 0: fp32 then bf16; worker 1: one batched call of three; worker 2: idle */
    int64_t counts[K] = {0, 0, 0};
    CHECK_ABS(abs_accumulate(d_acc[0], d_g32[0], ABS_F32, P, 32, &counts[0], NULL), ABS_OK);
    CHECK_ABS(abs_accumulate(d_acc[0], d_gbf, ABS_BF16, P, 64, &counts[0], NULL), ABS_OK);
    const void *batch[3] = {d_g32[1], d_g32[2], d_g32[0]};
    const int64_t ns[3] = {32, 32, 16};
    CHECK_ABS(abs_accumulate_batch(d_acc[1], batch, ABS_F32, 3, P, ns, &counts[1], NULL), ABS_OK);
    if (counts[0] != 96 || counts[1] != 80 || counts[2] != 0) {
        fprintf(stderr, "counts: %lld %lld %lld\n", (long long)counts[0], (long long)counts[1], (long long)counts[2]);
        ok = 0;
    }
    const float *acc_c[K] = {d_acc[0], d_acc[1], d_acc[2]};
    CHECK_ABS(abs_sync_update(d_x, d_v, acc_c, counts, K, P, 0.1f, 0.9f, 5e-4f, NULL), ABS_OK);
    CHECK_HIP(hipDeviceSynchronize());

    float *out_x = malloc((size_t)P * 4), *out_v = malloc((size_t)P * 4), *out_a = malloc((size_t)P * 4);
    CHECK_HIP(hipMemcpy(out_x, d_x, (size_t)P * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(out_v, d_v, (size_t)P * 4, hipMemcpyDeviceToHost));

    /* oracle, fp32 order */
    float *G0 = malloc((size_t)P * 4), *G1 = malloc((size_t)P * 4), *G2 = calloc((size_t)P, 4);
    oracle32_accumulate_f32(G0, g32[0], P, 32, 1);
    oracle32_accumulate_bf16(G0, gbf, P, 64, 0);
    oracle32_accumulate_f32(G1, g32[1], P, 32, 1);
    oracle32_accumulate_f32(G1, g32[2], P, 32, 0);
    oracle32_accumulate_f32(G1, g32[0], P, 16, 0);
    CHECK_HIP(hipMemcpy(out_a, d_acc[0], (size_t)P * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out_a, G0, P, "accumulator 0");
    CHECK_HIP(hipMemcpy(out_a, d_acc[1], (size_t)P * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out_a, G1, P, "accumulator 1 (batched)");
    float *x32 = malloc((size_t)P * 4), *v32 = malloc((size_t)P * 4);
    memcpy(x32, x, (size_t)P * 4);
    memcpy(v32, v, (size_t)P * 4);
    const float *G32[K] = {G0, G1, G2};
    if (oracle32_sync_update(x32, v32, G32, counts, K, P, 0.1f, 0.9f, 5e-4f) != 0) ok = 0;
    ok &= same_bits(out_x, x32, P, "x after sync-update");
    ok &= same_bits(out_v, v32, P, "v after sync-update");

    /* oracle, double */
    double *D0 = calloc((size_t)P, 8), *D1 = calloc((size_t)P, 8), *D2 = calloc((size_t)P, 8);
    double *x64 = malloc((size_t)P * 8), *v64 = malloc((size_t)P * 8);
    oracle_accumulate_f32(D0, g32[0], P, 32);
    oracle_accumulate_bf16(D0, gbf, P, 64);
    oracle_accumulate_f32(D1, g32[1], P, 32);
    oracle_accumulate_f32(D1, g32[2], P, 32);
    oracle_accumulate_f32(D1, g32[0], P, 16);
    for (int64_t i = 0; i < P; ++i) { x64[i] = x[i]; v64[i] = v[i]; }
    const double *G64[K] = {D0, D1, D2};
    oracle_sync_update(x64, v64, G64, counts, K, P, (double)0.1f, (double)0.9f, (double)5e-4f);
    ok &= close_normwise(out_x, x64, P, 1e-5, "x vs double oracle");
    ok &= close_normwise(out_v, v64, P, 1e-5, "v vs double oracle");

    /* an empty step touches nothing */
    const int64_t none[K] = {0, 0, 0};
    CHECK_ABS(abs_sync_update(d_x, d_v, acc_c, none, K, P, 0.1f, 0.9f, 5e-4f, NULL), ABS_EMPTY);
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(out_a, d_x, (size_t)P * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out_a, out_x, P, "x after an empty step");

    for (int k = 0; k < K; ++k) CHECK_HIP(hipFree(d_acc[k]));
    for (int j = 0; j < 3; ++j) { CHECK_HIP(hipFree(d_g32[j])); free(g32[j]); }
    CHECK_HIP(hipFree(d_gbf)); CHECK_HIP(hipFree(d_x)); CHECK_HIP(hipFree(d_v));
    free(x); free(v); free(gbf); free(out_x); free(out_v); free(out_a); free(G0); free(G1); free(G2);
    free(x32); free(v32); free(D0); free(D1); free(D2); free(x64); free(v64);
    return ok;
}

/* ---- case 2: Algorithm 1's loop through the double-buffer context, two streams ---- */
static int check_loop(int64_t P, int fold)
{
    enum { K = 2, T = 5, R = 4 };
    static const int m[T][K] = {{1, 3}, {2, 1}, {0, 2}, {3, 3}, {1, 1}};   /* reference batches per worker and iteration */
    const int64_t M_r = 32;
    int ok = 1;
    printf("[case] Algorithm 1 loop through abs_ctx, P = %lld, K = %d, T = %d, %s\n", (long long)P, K, T,
           fold ? "Step 2 of all workers as ONE abs_ctx_accumulate_step call per iteration" : "one abs_ctx_accumulate call per batch");
    fflush(stdout);
    float *x = malloc((size_t)P * 4), *pool[R];
    void *d_pool[R];
    fill_f32(x, P, 0.1f);
    for (int r = 0; r < R; ++r) {
        pool[r] = malloc((size_t)P * 4);
        fill_f32(pool[r], P, 0.02f);
        d_pool[r] = to_device(pool[r], (size_t)P * 4);
    }
    float *d_x = to_device(x, (size_t)P * 4), *d_v = NULL;
    CHECK_HIP(hipMalloc((void **)&d_v, (size_t)P * 4));
    CHECK_HIP(hipMemset(d_v, 0, (size_t)P * 4));
    float *A[K], *B[K];
    for (int k = 0; k < K; ++k) { A[k] = device_garbage((size_t)P * 4); B[k] = device_garbage((size_t)P * 4); }
    hipStream_t s_acc, s_upd;
    CHECK_HIP(hipStreamCreate(&s_acc));
    CHECK_HIP(hipStreamCreate(&s_upd));
    abs_ctx *ctx = NULL;
    CHECK_ABS(abs_ctx_create(&ctx, K, P, A, B, s_acc, s_upd), ABS_OK);

    /* oracle state, fp32 order */
    float *x32 = malloc((size_t)P * 4), *v32 = calloc((size_t)P, 4);
    float *G[2][K];
    int64_t M[2][K] = {{0, 0}, {0, 0}};
    memcpy(x32, x, (size_t)P * 4);
    for (int g = 0; g < 2; ++g)
        for (int k = 0; k < K; ++k) G[g][k] = calloc((size_t)P, 4);
    int cur = 0;
    for (int t = 0; t < T; ++t) {
        const int applied = abs_ctx_sync_update(ctx, d_x, d_v, 0.05f, 0.9f, 1e-3f);
        const float *Gp[K] = {G[cur ^ 1][0], G[cur ^ 1][1]};
        const int want = oracle32_sync_update(x32, v32, Gp, M[cur ^ 1], K, P, 0.05f, 0.9f, 1e-3f) == 0 ? ABS_OK : ABS_EMPTY;
        if (applied != want) { fprintf(stderr, "iteration %d: sync-update returned %d, oracle says %d\n", t, applied, want); ok = 0; }
        const void *step_grads[K * 3];                 /* worker 0's batches, then worker 1's */
        int64_t step_ns[K * 3];
        int n_step = 0;
        for (int k = 0; k < K; ++k) {
            M[cur][k] = 0;
            for (int j = 0; j < m[t][k]; ++j) {
                const int r = (3 * t + 2 * k + j) % R;
                if (fold) { step_grads[n_step] = d_pool[r]; step_ns[n_step++] = M_r; }
                else CHECK_ABS(abs_ctx_accumulate(ctx, k, d_pool[r], ABS_F32, M_r), ABS_OK);
                oracle32_accumulate_f32(G[cur][k], pool[r], P, M_r, M[cur][k] == 0);
                M[cur][k] += M_r;
            }
        }
        if (fold) CHECK_ABS(abs_ctx_accumulate_step(ctx, step_grads, m[t], step_ns, ABS_F32, fold), ABS_OK);
        int64_t got[K];
        CHECK_ABS(abs_ctx_counts(ctx, 0, got), ABS_OK);
        for (int k = 0; k < K; ++k)
            if (got[k] != M[cur][k]) { fprintf(stderr, "iteration %d worker %d: count %lld vs %lld\n", t, k, (long long)got[k], (long long)M[cur][k]); ok = 0; }
        CHECK_ABS(abs_swap_buffers(ctx), ABS_OK);
        cur ^= 1;
    }
    CHECK_HIP(hipDeviceSynchronize());
    float *out = malloc((size_t)P * 4);
    CHECK_HIP(hipMemcpy(out, d_x, (size_t)P * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out, x32, P, "x after the loop");
    CHECK_HIP(hipMemcpy(out, d_v, (size_t)P * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out, v32, P, "v after the loop");

    CHECK_ABS(abs_ctx_destroy(ctx), ABS_OK);
    CHECK_HIP(hipStreamDestroy(s_acc));
    CHECK_HIP(hipStreamDestroy(s_upd));
    for (int k = 0; k < K; ++k) { CHECK_HIP(hipFree(A[k])); CHECK_HIP(hipFree(B[k])); }
    for (int r = 0; r < R; ++r) { CHECK_HIP(hipFree(d_pool[r])); free(pool[r]); }
    for (int g = 0; g < 2; ++g)
        for (int k = 0; k < K; ++k) free(G[g][k]);
    CHECK_HIP(hipFree(d_x)); CHECK_HIP(hipFree(d_v));
    free(x); free(x32); free(v32); free(out);
    return ok;
}

/* ---- case 3: the ragged forms: one hipMalloc per tensor, pointer tables, one launch per call ---- */
static int check_ragged(void)
{
    enum { T = 4, K = 2 };
    static const int64_t sizes[T] = {5, 9001, 0, 4096 * 2 + 3};
    int64_t off[T + 1] = {0}, P;
    int ok = 1;
    for (int t = 0; t < T; ++t) off[t + 1] = off[t] + sizes[t];
    P = off[T];
    printf("[case] ragged forms, %d tensors, %lld elements, K = %d\n", T, (long long)P, K);
    fflush(stdout);
    float *x = malloc((size_t)P * 4), *v = malloc((size_t)P * 4), *g32 = malloc((size_t)P * 4);
    uint16_t *gbf = malloc((size_t)P * 2);
    fill_f32(x, P, 0.1f); fill_f32(v, P, 0.01f); fill_f32(g32, P, 0.02f); fill_bf16(gbf, P, 0.02f);

    abs_layout *L = NULL;
    CHECK_ABS(abs_layout_create(&L, T, sizes), ABS_OK);
    if (abs_layout_total(L) != P || abs_layout_num_tensors(L) != T) { fprintf(stderr, "layout totals\n"); ok = 0; }
    void *dx[T], *dv[T], *dg32[T], *dgbf[T], *da[K][T];
    for (int t = 0; t < T; ++t) {
        const size_t n = (size_t)sizes[t];
        if (n == 0) { dx[t] = dv[t] = dg32[t] = dgbf[t] = da[0][t] = da[1][t] = NULL; continue; }   /* an empty tensor has no storage */
        dx[t] = to_device(x + off[t], n * 4); dv[t] = to_device(v + off[t], n * 4);
        dg32[t] = to_device(g32 + off[t], n * 4); dgbf[t] = to_device(gbf + off[t], n * 2);
        for (int k = 0; k < K; ++k) da[k][t] = device_garbage(n * 4);
    }
    abs_tensorset *sx, *sv, *sg32, *sgbf, *sa[K];
    CHECK_ABS(abs_tensorset_create(&sx, L, dx, ABS_F32), ABS_OK);
    CHECK_ABS(abs_tensorset_create(&sv, L, dv, ABS_F32), ABS_OK);
    CHECK_ABS(abs_tensorset_create(&sg32, L, dg32, ABS_F32), ABS_OK);
    CHECK_ABS(abs_tensorset_create(&sgbf, L, dgbf, ABS_BF16), ABS_OK);
    for (int k = 0; k < K; ++k) CHECK_ABS(abs_tensorset_create(&sa[k], L, da[k], ABS_F32), ABS_OK);

    int64_t counts[K] = {0, 0};
    CHECK_ABS(abs_accumulate_mt(L, sa[0], sgbf, 32, &counts[0], NULL), ABS_OK);
    CHECK_ABS(abs_accumulate_mt(L, sa[0], sg32, 64, &counts[0], NULL), ABS_OK);
    const abs_tensorset *two[2] = {sg32, sg32};
    const int64_t ns[2] = {16, 48};
    CHECK_ABS(abs_accumulate_batch_mt(L, sa[1], two, 2, ns, &counts[1], NULL), ABS_OK);
    const abs_tensorset *accs[K] = {sa[0], sa[1]};
    CHECK_ABS(abs_sync_update_mt(L, sx, sv, accs, counts, K, 0.1f, 0.9f, 5e-4f, NULL), ABS_OK);
    CHECK_HIP(hipDeviceSynchronize());
    /* the same two accumulations once more, both workers in ONE job-list call (fresh buffers) */
    void *dj[K][T];
    abs_tensorset *sj[K];
    for (int k = 0; k < K; ++k) {
        for (int t = 0; t < T; ++t) dj[k][t] = sizes[t] ? device_garbage((size_t)sizes[t] * 4) : NULL;
        CHECK_ABS(abs_tensorset_create(&sj[k], L, dj[k], ABS_F32), ABS_OK);
    }
    int64_t jcounts[K] = {0, 0};
    const abs_tensorset *job0[2] = {sg32, sg32}, *job1[2] = {sg32, sg32};
    const int64_t jn0[2] = {32, 64}, jn1[2] = {16, 48};
    const abs_job_mt jobs[K] = {{sj[0], job0, jn0, 2, &jcounts[0]}, {sj[1], job1, jn1, 2, &jcounts[1]}};
    CHECK_ABS(abs_accumulate_jobs_mt(L, jobs, K, 8, NULL), ABS_OK);
    CHECK_HIP(hipDeviceSynchronize());

    float *G0 = malloc((size_t)P * 4), *G1 = malloc((size_t)P * 4), *x32 = malloc((size_t)P * 4), *v32 = malloc((size_t)P * 4);
    oracle32_accumulate_bf16(G0, gbf, P, 32, 1);
    oracle32_accumulate_f32(G0, g32, P, 64, 0);
    oracle32_accumulate_f32(G1, g32, P, 16, 1);
    oracle32_accumulate_f32(G1, g32, P, 48, 0);
    memcpy(x32, x, (size_t)P * 4); memcpy(v32, v, (size_t)P * 4);
    const float *G32[K] = {G0, G1};
    if (counts[0] != 96 || counts[1] != 64) { fprintf(stderr, "ragged counts\n"); ok = 0; }
    if (oracle32_sync_update(x32, v32, G32, counts, K, P, 0.1f, 0.9f, 5e-4f) != 0) ok = 0;
    float *out = malloc((size_t)P * 4);
    for (int t = 0; t < T; ++t)
        if (sizes[t]) CHECK_HIP(hipMemcpy(out + off[t], dx[t], (size_t)sizes[t] * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out, x32, P, "ragged x");
    for (int t = 0; t < T; ++t)
        if (sizes[t]) CHECK_HIP(hipMemcpy(out + off[t], dv[t], (size_t)sizes[t] * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out, v32, P, "ragged v");
    for (int t = 0; t < T; ++t)
        if (sizes[t]) CHECK_HIP(hipMemcpy(out + off[t], da[1][t], (size_t)sizes[t] * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out, G1, P, "ragged accumulator (batched)");
    for (int t = 0; t < T; ++t)
        if (sizes[t]) CHECK_HIP(hipMemcpy(out + off[t], dj[1][t], (size_t)sizes[t] * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out, G1, P, "ragged accumulator (job list, worker 1)");
    oracle32_accumulate_f32(G0, g32, P, 32, 1);
    oracle32_accumulate_f32(G0, g32, P, 64, 0);
    for (int t = 0; t < T; ++t)
        if (sizes[t]) CHECK_HIP(hipMemcpy(out + off[t], dj[0][t], (size_t)sizes[t] * 4, hipMemcpyDeviceToHost));
    ok &= same_bits(out, G0, P, "ragged accumulator (job list, worker 0)");
    if (jcounts[0] != 96 || jcounts[1] != 64) { fprintf(stderr, "job-list counts\n"); ok = 0; }
    for (int k = 0; k < K; ++k) {
        abs_tensorset_destroy(sj[k]);
        for (int t = 0; t < T; ++t)
            if (sizes[t]) CHECK_HIP(hipFree(dj[k][t]));
    }

    abs_tensorset_destroy(sx); abs_tensorset_destroy(sv); abs_tensorset_destroy(sg32); abs_tensorset_destroy(sgbf);
    for (int k = 0; k < K; ++k) abs_tensorset_destroy(sa[k]);
    abs_layout_destroy(L);
    for (int t = 0; t < T; ++t) {
        if (!sizes[t]) continue;
        CHECK_HIP(hipFree(dx[t])); CHECK_HIP(hipFree(dv[t])); CHECK_HIP(hipFree(dg32[t])); CHECK_HIP(hipFree(dgbf[t]));
        for (int k = 0; k < K; ++k) CHECK_HIP(hipFree(da[k][t]));
    }
    free(x); free(v); free(g32); free(gbf); free(G0); free(G1); free(x32); free(v32); free(out);
    return ok;
}

int main(void)
{
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1) {
        fprintf(stderr, "abi_check: no GPU visible\n");
        return 2;
    }
    printf("abi_check: library version %d, row of %lld elements\n", abs_version(), (long long)abs_row_elems());
    int ok = 1;
    ok &= check_calls(3 * 4096 + 1029);        /* several tiles and a ragged tail */
    ok &= check_calls(5);                      /* shorter than one vector */
    ok &= check_loop(200003, 0);
    ok &= check_loop(200003, 8);               /* a job list: all workers of an iteration in one launch */
    ok &= check_loop(70001, 1);                /* the same call, one batch per worker and launch */
    ok &= check_ragged();
    if (!ok) {
        fprintf(stderr, "abi_check: FAILED\n");
        return 1;
    }
    printf("abi_check: OK\n");
    return 0;
}

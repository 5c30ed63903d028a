/* Plain C client of the whole boundary on a GPU: layouts, a plan, device buffers from the HIP
 * runtime's C API, ll_convert and ll_gather on the null stream, results compared bit for bit with the
 * CPU oracle's C functions (linked from oracle/, test infrastructure).  No Python, no C++.
 * Prints "ok" and returns 0 on success.
 * With the argument --time it instead times eager calls through the C ABI (no Python in the way) on
 * the one-tile configuration 1 (64 x 64 int32, blocked -> 32x32 accumulator layout) and a one-tile
 * gather, and prints one line: "us_per_convert <x> us_per_gather <y> calls <n>". */
#define __HIP_PLATFORM_AMD__ 1
#define _POSIX_C_SOURCE 199309L     /* clock_gettime under -std=c99 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "ll.h"

int oracle_convert(const uint64_t *basesA, const uint64_t *basesB, int d, int elem_bytes, const void *src, void *dst,
                   int64_t ntiles);
int oracle_gather(const uint64_t *basesL, int d, const int32_t *out_dim_bits, int n_out_dims, int axis, int elem_bytes,
                  const void *in, const int32_t *idx, void *out, int64_t ntiles);

#define CHECK(call) do { ll_status st_ = (call); if (st_ != LL_OK) { \
    fprintf(stderr, "%s -> %d: %s\n", #call, (int)st_, ll_last_error()); return 1; } } while (0)
#define HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s -> %s\n", #call, hipGetErrorString(e_)); return 1; } } while (0)

enum { D = 12, NTILES = 37 };

static double now_us(void)
{
    struct timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return ts.tv_sec * 1e6 + ts.tv_nsec * 1e-3;
}

/* Host cost of an eager call: n calls back to back on one stream, one synchronisation at the end. */
static int time_calls(void)
{
    enum { COL = 0, ROW = 6, CALLS = 20000 };
    /* configuration 1: registers, lanes, waves of the source and of the destination layout */
    const uint64_t src_bases[D] = {1ull << (COL + 0), 1ull << (COL + 1), 1ull << (ROW + 4), 1ull << (ROW + 5),
                                   1ull << (COL + 2), 1ull << (COL + 3), 1ull << (COL + 4), 1ull << (COL + 5), 1ull << (ROW + 0), 1ull << (ROW + 1),
                                   1ull << (ROW + 2), 1ull << (ROW + 3)};
    const uint64_t dst_bases[D] = {1ull << (ROW + 0), 1ull << (ROW + 1), 1ull << (ROW + 3), 1ull << (ROW + 4),
                                   1ull << (COL + 0), 1ull << (COL + 1), 1ull << (COL + 2), 1ull << (COL + 3), 1ull << (COL + 4), 1ull << (ROW + 2),
                                   1ull << (ROW + 5), 1ull << (COL + 5)};
    const ll_in_dim in_dims[3] = {{LL_IN_REG, 4}, {LL_IN_LANE, 6}, {LL_IN_WAVE, 2}};
    const ll_out_dim out_dims[2] = {{6}, {6}};
    ll_layout *a = NULL, *b = NULL;
    ll_plan *plan = NULL;
    CHECK(ll_layout_create(in_dims, 3, out_dims, 2, src_bases, &a));
    CHECK(ll_layout_create(in_dims, 3, out_dims, 2, dst_bases, &b));
    CHECK(ll_plan_convert(a, b, 4, &plan));
    void *dsrc = NULL, *ddst = NULL, *didx = NULL;
    const size_t bytes = (size_t)4 << D;
    HIP(hipMalloc(&dsrc, bytes));
    HIP(hipMalloc(&ddst, bytes));
    HIP(hipMalloc(&didx, bytes));
    HIP(hipMemset(dsrc, 1, bytes));
    HIP(hipMemset(didx, 0, bytes));
    hipStream_t stream;
    HIP(hipStreamCreate(&stream));
    double us[2];
    for (int what = 0; what < 2; ++what) {
        for (int rep = 0; rep < 2; ++rep) {            /* the first round warms up */
            HIP(hipStreamSynchronize(stream));
            const double t0 = now_us();
            for (int i = 0; i < CALLS; ++i) {
                if (what == 0) CHECK(ll_convert(plan, dsrc, ddst, 1, stream));
                else CHECK(ll_gather(b, 0, 4, dsrc, (const int32_t *)didx, ddst, 1, stream));
            }
            HIP(hipStreamSynchronize(stream));
            us[what] = (now_us() - t0) / CALLS;
        }
    }
    printf("us_per_convert %.3f us_per_gather %.3f calls %d\n", us[0], us[1], (int)CALLS);
    HIP(hipStreamDestroy(stream));
    HIP(hipFree(dsrc));
    HIP(hipFree(ddst));
    HIP(hipFree(didx));
    CHECK(ll_plan_destroy(plan));
    CHECK(ll_layout_destroy(a));
    CHECK(ll_layout_destroy(b));
    return 0;
}

int main(int argc, char **argv)
{
    if (argc > 1 && strcmp(argv[1], "--time") == 0) return time_calls();
    /* a 64 x 64 tile, 16 registers x 64 lanes x 4 waves: A row-major, B a bit permutation with XOR terms
     * (every column is one unit vector plus the unit vector of the column before it: invertible) */
    const int perm[D] = {7, 2, 9, 0, 11, 4, 1, 8, 5, 10, 3, 6};
    uint64_t a_bases[D], b_bases[D];
    for (int k = 0; k < D; ++k) {
        a_bases[k] = 1ull << k;
        b_bases[k] = (1ull << perm[k]) | (k ? 1ull << perm[k - 1] : 0);
    }
    const ll_in_dim in_dims[3] = {{LL_IN_REG, 4}, {LL_IN_LANE, 6}, {LL_IN_WAVE, 2}};
    const ll_out_dim out_dims[2] = {{6}, {6}};
    const int32_t out_bits[2] = {6, 6};
    ll_layout *a = NULL, *b = NULL;
    ll_plan *plan = NULL;
    CHECK(ll_layout_create(in_dims, 3, out_dims, 2, a_bases, &a));
    CHECK(ll_layout_create(in_dims, 3, out_dims, 2, b_bases, &b));
    CHECK(ll_plan_convert(a, b, 4, &plan));

    const size_t n = (size_t)NTILES << D;
    uint32_t *src = malloc(n * 4), *got = malloc(n * 4), *want = malloc(n * 4);
    int32_t *idx = malloc(n * 4);
    if (!src || !got || !want || !idx) return 1;
    for (size_t i = 0; i < n; ++i) {
        src[i] = (uint32_t)i * 2654435761u ^ (uint32_t)(i >> 7);
        idx[i] = (int32_t)((i * 40503u) >> 3) & 63;
    }
    void *dsrc = NULL, *ddst = NULL, *didx = NULL;
    HIP(hipMalloc(&dsrc, n * 4));
    HIP(hipMalloc(&ddst, n * 4));
    HIP(hipMalloc(&didx, n * 4));
    HIP(hipMemcpy(dsrc, src, n * 4, hipMemcpyHostToDevice));
    HIP(hipMemcpy(didx, idx, n * 4, hipMemcpyHostToDevice));

    /* conversion A -> B */
    HIP(hipMemset(ddst, 0x5A, n * 4));
    CHECK(ll_convert(plan, dsrc, ddst, NTILES, NULL));
    HIP(hipDeviceSynchronize());
    HIP(hipMemcpy(got, ddst, n * 4, hipMemcpyDeviceToHost));
    if (oracle_convert(a_bases, b_bases, D, 4, src, want, NTILES) != 0) { fprintf(stderr, "oracle_convert failed\n"); return 1; }
    if (memcmp(got, want, n * 4) != 0) { fprintf(stderr, "conversion differs from the oracle\n"); return 1; }

    /* gather along both dims under B (rows and columns are spread over registers, lanes and waves) */
    for (int axis = 0; axis < 2; ++axis) {
        HIP(hipMemset(ddst, 0x5A, n * 4));
        CHECK(ll_gather(b, axis, 4, dsrc, (const int32_t *)didx, ddst, NTILES, NULL));
        HIP(hipDeviceSynchronize());
        HIP(hipMemcpy(got, ddst, n * 4, hipMemcpyDeviceToHost));
        if (oracle_gather(b_bases, D, out_bits, 2, axis, 4, src, idx, want, NTILES) != 0) { fprintf(stderr, "oracle_gather failed\n"); return 1; }
        if (memcmp(got, want, n * 4) != 0) { fprintf(stderr, "gather along dim %d differs from the oracle\n", axis); return 1; }
    }

    /* an error must come back as a status, with nothing launched */
    if (ll_convert(plan, dsrc, dsrc, NTILES, NULL) != LL_ERR_INVALID_ARG) { fprintf(stderr, "aliasing buffers were not rejected\n"); return 1; }

    HIP(hipFree(dsrc));
    HIP(hipFree(ddst));
    HIP(hipFree(didx));
    CHECK(ll_plan_destroy(plan));
    CHECK(ll_layout_destroy(a));
    CHECK(ll_layout_destroy(b));
    free(src); free(got); free(want); free(idx);
    printf("ok\n");
    return 0;
}

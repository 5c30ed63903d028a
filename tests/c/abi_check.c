/* Plain C99 client of ll.h: proves that the header compiles as C and that the host entry points
 * can be used without Python or C++.  Host algebra only (no device call), so it runs without a GPU.
 * Prints "ok" and returns 0 on success. */
#include <stdio.h>
#include <string.h>

#include "ll.h"

#define CHECK(call) do { ll_status st_ = (call); if (st_ != LL_OK) { \
    fprintf(stderr, "%s -> %d: %s\n", #call, (int)st_, ll_last_error()); return 1; } } while (0)

int main(void)
{
    /* Layout A of the paper's Sec. 4.1 from its three tiles */
    ll_layout *regs = NULL, *thrs = NULL, *warps = NULL, *rt = NULL, *a = NULL, *inv = NULL, *q = NULL;
    const ll_in_dim reg_in = {LL_IN_REG, 2}, thr_in = {LL_IN_LANE, 5}, warp_in = {LL_IN_WAVE, 1};
    const ll_out_dim reg_out[2] = {{1}, {1}}, thr_out[2] = {{2}, {3}}, warp_out[2] = {{1}, {0}};
    const uint64_t reg_b[2] = {1, 2}, thr_b[5] = {1, 2, 4, 8, 16}, warp_b[1] = {1};
    CHECK(ll_layout_create(&reg_in, 1, reg_out, 2, reg_b, &regs));
    CHECK(ll_layout_create(&thr_in, 1, thr_out, 2, thr_b, &thrs));
    CHECK(ll_layout_create(&warp_in, 1, warp_out, 2, warp_b, &warps));
    CHECK(ll_product_dimwise(regs, thrs, &rt));
    CHECK(ll_product_dimwise(rt, warps, &a));
    uint64_t y = 0;
    CHECK(ll_layout_apply(a, 1u | (9u << 2), &y));          /* register 1, thread 9, warp 0 */
    if (y != ((2u << 4) | 3u)) { fprintf(stderr, "Layout A(r1, t9, w0) = 0x%llx\n", (unsigned long long)y); return 1; }
    CHECK(ll_invert(a, &inv));
    uint64_t h = 0;
    CHECK(ll_layout_apply(inv, y, &h));
    if (h != (1u | (9u << 2))) { fprintf(stderr, "inverse gives 0x%llx\n", (unsigned long long)h); return 1; }
    CHECK(ll_divide_left(a, regs, &q));
    int32_t contiguous = 0;
    CHECK(ll_contiguity(a, &contiguous));
    if (contiguous != 2) { fprintf(stderr, "contiguity %d\n", (int)contiguous); return 1; }

    /* a plan, its description, and an argument error that must come back as a status */
    ll_layout *b = NULL;
    ll_plan *plan = NULL;
    ll_plan_desc desc;
    int32_t rb[2] = {1, 1}, tb[2] = {2, 3}, wb[2] = {1, 0}, order[2] = {0, 1};
    CHECK(ll_layout_blocked(2, rb, tb, wb, order, &b));
    CHECK(ll_plan_convert(a, b, 4, &plan));
    CHECK(ll_plan_info(plan, &desc));
    if (desc.d != 8 || desc.elem_bytes != 4 || desc.global_vec_bytes != 16) { fprintf(stderr, "unexpected plan description\n"); return 1; }
    if (ll_convert(plan, NULL, NULL, 1, NULL) != LL_ERR_INVALID_ARG || strlen(ll_last_error()) == 0) {
        fprintf(stderr, "null device pointers were not rejected\n");
        return 1;
    }
    CHECK(ll_convert(plan, NULL, NULL, 0, NULL));           /* nothing to do */
    CHECK(ll_plan_destroy(plan));
    ll_layout *all[] = {regs, thrs, warps, rt, a, inv, q, b};
    for (unsigned i = 0; i < sizeof(all) / sizeof(all[0]); ++i) CHECK(ll_layout_destroy(all[i]));
    printf("ok\n");
    return 0;
}

// Seeded fuzz of the host side of the library through its C ABI (planners, gather chooser, algebra,
// argument checks), meant to be linked with launcher_stubs.cpp and run under ASan + UBSan.
// usage: host_fuzz <seed> <cases>.  Every plan that is made is also "launched" with made-up device
// addresses: the stub launchers return LL_ERR_DEVICE, everything before them is real.
// Exit status 0 and a summary line on success; the first unexpected status or sanitizer report ends the run.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../include/ll.h"

static std::mt19937_64 rng;
static int ri(int lo, int hi) { return lo + (int)(rng() % (uint64_t)(hi - lo + 1)); }   // inclusive

static bool spans(const std::vector<uint64_t> &cols, int d_out)
{
    std::vector<uint64_t> basis;
    for (uint64_t c : cols) {
        uint64_t x = c;
        for (uint64_t b : basis) x = std::min(x, x ^ b);
        if (x) basis.push_back(x);
    }
    return (int)basis.size() == d_out;
}

// kind 0: arbitrary XOR columns; 1: a distributed layout (unit vectors and zero columns); 2: unit vectors with a few XOR terms
static std::vector<uint64_t> rand_cols(int d_in, int d_out, int kind)
{
    for (;;) {
        std::vector<uint64_t> cols(d_in);
        if (kind == 0) {
            for (auto &c : cols) c = rng() & ((1ull << d_out) - 1);
            if (d_in > d_out && ri(0, 1)) cols[ri(0, d_in - 1)] = 0;
        } else {
            std::vector<uint64_t> units;
            std::vector<int> perm(d_out);
            for (int i = 0; i < d_out; ++i) perm[i] = i;
            std::shuffle(perm.begin(), perm.end(), rng);
            for (int i = 0; i < d_out; ++i) units.push_back(1ull << perm[i]);
            for (int i = d_out; i < d_in; ++i) units.push_back(0);
            std::shuffle(units.begin(), units.end(), rng);
            cols = units;
            if (kind == 2)
                for (int k = ri(1, 3); k > 0; --k) {
                    int i = ri(0, d_in - 1), j = ri(0, d_in - 1);
                    if (i != j) cols[i] ^= cols[j];
                }
        }
        if (spans(cols, d_out)) return cols;
    }
}

static ll_layout *make_layout(int d, int d_out, const std::vector<uint64_t> &cols, bool memory, int ndims)
{
    ll_in_dim in[4];
    int n = 0;
    if (memory) {
        in[n++] = {LL_IN_OFFSET, d};
    } else {
        int nreg = ri(0, std::min(6, d)), nlane = std::min(6, d - nreg);
        if (ri(0, 3) == 0) nlane = ri(0, nlane);
        const int nwave = d - nreg - nlane;
        if (nreg) in[n++] = {LL_IN_REG, nreg};
        if (nlane) in[n++] = {LL_IN_LANE, nlane};
        if (nwave) in[n++] = {LL_IN_WAVE, nwave};
        if (!n) in[n++] = {LL_IN_REG, 0};
    }
    ll_out_dim out[3];
    int left = d_out;
    for (int i = 0; i < ndims; ++i) {
        const int b = i == ndims - 1 ? left : ri(0, left);
        out[i] = {b};
        left -= b;
    }
    ll_layout *l = nullptr;
    if (ll_layout_create(in, n, out, ndims, cols.data(), &l) != LL_OK) {
        fprintf(stderr, "ll_layout_create: %s\n", ll_last_error());
        abort();
    }
    return l;
}

// Options with a few fields set to values from their documented domains (or just outside).
static const ll_options *rand_options(ll_options *o)
{
    if (ri(0, 2) == 0) return nullptr;
    ll_options_init(o);
    static const int strategies[] = {LL_AUTO, 3, 4, 6, 1, 99};
    static const int bytes[] = {LL_AUTO, 16, 1024, 4096, 8192, 16384, 65536, 3000, 1 << 20, 1 << 24};
    if (ri(0, 1)) o->strategy = strategies[ri(0, 5)];
    if (ri(0, 1)) o->gather_kernel = ri(-1, 6);
    if (ri(0, 2) == 0) o->block_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->pref_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->elem_threads_log2 = ri(4, 11);
    if (ri(0, 2) == 0) o->vec_block_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->vec_threads = 32 << ri(0, 4);
    if (ri(0, 2) == 0) o->shuffle_block_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->inflight_bytes = bytes[ri(0, 9)];
    if (ri(0, 3) == 0) o->lds_pad_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->xcd_chunk = ri(-1, 300);
    if (ri(0, 2) == 0) o->pull_mode = ri(-1, 3);
    if (ri(0, 2) == 0) o->pull_vec_bits = ri(-1, 5);
    if (ri(0, 2) == 0) o->pull_inflight_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->pull_threads_log2 = ri(4, 9);
    if (ri(0, 2) == 0) o->gather_block_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->gather_lds_max_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->gather_min_run_bytes = 1 << ri(0, 9);
    if (ri(0, 2) == 0) o->gather_phased_max_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->gather_threads_log2 = ri(6, 11);
    if (ri(0, 2) == 0) o->gather_inflight_bytes = bytes[ri(0, 9)];
    if (ri(0, 2) == 0) o->gather_xcd_chunk = ri(-1, 300);
    if (ri(0, 2) == 0) o->gather_waves = ri(-1, 5);
    if (ri(0, 3) == 0) o->gather_swizzle_always = ri(-1, 1);
    if (ri(0, 7) == 0) o->size = ri(0, (int)sizeof(ll_options));       // a caller built against an older, shorter struct
    return o;
}

int main(int argc, char **argv)
{
    rng.seed(argc > 1 ? atoll(argv[1]) : 1);
    const long cases = argc > 2 ? atol(argv[2]) : 2000;
    long planned = 0, declined = 0;
    void *const fake_src = (void *)4096, *const fake_dst = (void *)(1ull << 40);
    const int32_t *const fake_idx = (const int32_t *)(1ull << 38);
    for (long c = 0; c < cases; ++c) {
        const int w = 1 << ri(0, 3);
        const int kind = ri(0, 3);
        ll_options opts;
        const ll_options *o = rand_options(&opts);
        if (kind == 0) {                               // bijective conversion, maybe a memory image on a side, maybe affine
            const int d = ri(1, 26), nd = ri(1, 3);
            ll_layout *a = make_layout(d, d, rand_cols(d, d, ri(0, 2)), ri(0, 5) == 0, nd);
            ll_layout *b0 = make_layout(d, d, rand_cols(d, d, ri(0, 2)), ri(0, 5) == 0, nd), *b = b0;
            if (ri(0, 2) == 0 && ll_layout_with_offset(b0, rng() & ((1ull << d) - 1), &b) != LL_OK) return 1;
            ll_plan *p = nullptr;
            const ll_status st = ll_plan_convert_opts(a, b, w, o, &p);
            if (st == LL_OK) {
                ll_plan_desc desc;
                if (ll_plan_info(p, &desc) != LL_OK) return 1;
                const ll_status run = ll_convert(p, fake_src, fake_dst, ri(1, 40), nullptr);
                if (run != LL_ERR_DEVICE && run != LL_ERR_INVALID_ARG) { fprintf(stderr, "case %ld: ll_convert status %d: %s\n", c, run, ll_last_error()); return 1; }
                ++planned;
            } else if (st == LL_ERR_DIM_MISMATCH || st == LL_ERR_UNSUPPORTED) {
                ++declined;
            } else {
                fprintf(stderr, "case %ld: plan status %d: %s\n", c, st, ll_last_error());
                return 1;
            }
            ll_plan_destroy(p);
            if (b != b0) ll_layout_destroy(b);
            ll_layout_destroy(a);
            ll_layout_destroy(b0);
        } else if (kind == 1) {                        // conversion between broadcasting layouts
            const int dl = ri(1, 20), da = dl + ri(0, 6), db = dl + ri(0, 6), nd = ri(1, 3);
            if (da > 30 || db > 30) continue;
            ll_layout *a = make_layout(da, dl, rand_cols(da, dl, ri(0, 2)), false, nd), *b = make_layout(db, dl, rand_cols(db, dl, ri(0, 2)), false, nd);
            ll_plan *p = nullptr;
            const ll_status st = ll_plan_convert_opts(a, b, w, o, &p);
            if (st == LL_OK) {
                const ll_status run = ll_convert(p, fake_src, fake_dst, 16, nullptr);
                if (run != LL_ERR_DEVICE && run != LL_ERR_INVALID_ARG) { fprintf(stderr, "case %ld: ll_convert status %d: %s\n", c, run, ll_last_error()); return 1; }
                ++planned;
            } else if (st == LL_ERR_UNSUPPORTED || st == LL_ERR_DIM_MISMATCH) {
                ++declined;
            } else {
                fprintf(stderr, "case %ld: broadcast plan status %d: %s\n", c, st, ll_last_error());
                return 1;
            }
            ll_plan_destroy(p);
            ll_layout_destroy(a);
            ll_layout_destroy(b);
        } else {                                       // gather along every axis, layouts that may broadcast or be memory layouts
            const int dl = ri(1, 24), d = std::min(28, dl + (ri(0, 2) == 0 ? ri(0, 4) : 0)), nd = ri(1, 3);
            ll_layout *a = make_layout(d, dl, rand_cols(d, dl, ri(0, 2)), ri(0, 4) == 0, nd);
            for (int axis = 0; axis < nd; ++axis) {
                ll_gather_desc g;
                const ll_status st = ll_gather_info_opts(a, axis, w, o, &g);
                if (st == LL_OK) {
                    const ll_status run = ll_gather_opts(a, axis, w, o, fake_src, fake_idx, fake_dst, 16, nullptr);
                    if (run != LL_ERR_DEVICE && run != LL_ERR_INVALID_ARG) { fprintf(stderr, "case %ld: ll_gather status %d: %s\n", c, run, ll_last_error()); return 1; }
                    ++planned;
                } else if (st == LL_ERR_UNSUPPORTED) {
                    ++declined;
                } else {
                    fprintf(stderr, "case %ld: gather status %d: %s\n", c, st, ll_last_error());
                    return 1;
                }
            }
            ll_layout_destroy(a);
        }
    }
    printf("cases %ld planned %ld declined %ld\n", cases, planned, declined);
    return 0;
}

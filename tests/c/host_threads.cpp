// Concurrent use of shared layouts and plans through the C ABI, meant to be linked with launcher_stubs.cpp
// and run under ThreadSanitizer: the header promises that layouts and plans may be used from any thread.
// Several threads query and "launch" gathers on the SAME layouts (hits and misses of the per-layout cache of
// gather choices, under different options), plan conversions between them and run the plans; every answer
// is compared with the one a single thread got beforehand.
// usage: host_threads <threads> <rounds>.  Exit status 0 and a summary line on success.
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/ll.h"

namespace {

struct Query {
    int layout, axis, elem_bytes, option_set;
};

constexpr int kLayouts = 4, kOptionSets = 4;
ll_layout *g_layouts[kLayouts];
ll_options g_options[kOptionSets];
std::vector<Query> g_queries;
std::vector<ll_gather_desc> g_want;
std::vector<ll_status> g_want_status;
ll_plan *g_plan = nullptr;
ll_plan_desc g_plan_want;
std::atomic<long> g_bad{0};

const ll_options *options_of(int set) { return set == 0 ? nullptr : &g_options[set]; }

void worker(int id, int rounds)
{
    void *const fake_in = (void *)4096, *const fake_out = (void *)(1ull << 40);
    const int32_t *const fake_idx = (const int32_t *)(1ull << 38);
    for (int r = 0; r < rounds; ++r) {
        for (size_t q0 = 0; q0 < g_queries.size(); ++q0) {
            const size_t q = (q0 * 7 + (size_t)id * 3 + (size_t)r) % g_queries.size();     // every thread its own order
            const Query &x = g_queries[q];
            ll_gather_desc got;
            std::memset(&got, 0, sizeof(got));
            const ll_status st = ll_gather_info_opts(g_layouts[x.layout], x.axis, x.elem_bytes, options_of(x.option_set), &got);
            if (st != g_want_status[q] || (st == LL_OK && std::memcmp(&got, &g_want[q], sizeof(got)) != 0)) ++g_bad;
            if (st == LL_OK) {
                const ll_status run = ll_gather_opts(g_layouts[x.layout], x.axis, x.elem_bytes, options_of(x.option_set), fake_in, fake_idx,
                                                     fake_out, 16, nullptr);
                if (run != LL_ERR_DEVICE) ++g_bad;                                             // the stub launcher's status
                if (std::strstr(ll_last_error(), "stub") == nullptr) ++g_bad;                  // this thread's own message
            }
        }
        // a plan shared by all threads, and a plan of this thread's own between the shared layouts
        ll_plan_desc d;
        if (ll_plan_info(g_plan, &d) != LL_OK || std::memcmp(&d, &g_plan_want, sizeof(d)) != 0) ++g_bad;
        if (ll_convert(g_plan, fake_in, fake_out, 8, nullptr) != LL_ERR_DEVICE) ++g_bad;
        ll_plan *mine = nullptr;
        if (ll_plan_convert_opts(g_layouts[0], g_layouts[1], 4, options_of(r % kOptionSets), &mine) != LL_OK) ++g_bad;
        if (mine && ll_convert(mine, fake_in, fake_out, 8, nullptr) != LL_ERR_DEVICE) ++g_bad;
        ll_plan_destroy(mine);
        // an error on this thread must not show up in another thread's message
        if (ll_convert(g_plan, fake_in, fake_in, 8, nullptr) != LL_ERR_INVALID_ARG) ++g_bad;
        if (std::strstr(ll_last_error(), "stub") != nullptr) ++g_bad;
    }
}

}  // namespace

int main(int argc, char **argv)
{
    const int threads = argc > 1 ? atoi(argv[1]) : 8, rounds = argc > 2 ? atoi(argv[2]) : 20;
    // 2^12-element tiles (4 registers, 6 lanes, 2 waves bits), two logical dims of 2^6: row major, a bit rotation,
    // one with XOR terms, and one with rows on lanes
    const ll_in_dim in_dims[3] = {{LL_IN_REG, 4}, {LL_IN_LANE, 6}, {LL_IN_WAVE, 2}};
    const ll_out_dim out_dims[2] = {{6}, {6}};
    for (int l = 0; l < kLayouts; ++l) {
        uint64_t bases[12];
        for (int k = 0; k < 12; ++k) {
            const int rot[4] = {0, 5, 3, 8};
            bases[k] = 1ull << ((k + rot[l]) % 12);
            if (l == 2 && k > 0) bases[k] ^= 1ull << ((k - 1 + rot[l]) % 12);
        }
        if (ll_layout_create(in_dims, 3, out_dims, 2, bases, &g_layouts[l]) != LL_OK) { fprintf(stderr, "layout: %s\n", ll_last_error()); return 1; }
    }
    for (int s = 0; s < kOptionSets; ++s) ll_options_init(&g_options[s]);
    g_options[1].gather_kernel = LL_GATHER_BLOCK_STAGED;
    g_options[2].gather_kernel = LL_GATHER_SHUFFLE;
    g_options[2].gather_waves = 2;
    g_options[3].gather_block_bytes = 4096;
    g_options[3].strategy = LL_STRATEGY_LDS_ELEM;
    for (int l = 0; l < kLayouts; ++l)
        for (int axis = 0; axis < 2; ++axis)
            for (int w = 1; w <= 8; w *= 2)
                for (int s = 0; s < kOptionSets; ++s) g_queries.push_back({l, axis, w, s});
    // the reference answers, from fresh copies of the layouts so that the shared ones start with empty caches
    for (const Query &x : g_queries) {
        ll_layout *fresh = nullptr;
        if (ll_layout_with_offset(g_layouts[x.layout], 0, &fresh) != LL_OK) return 1;
        ll_gather_desc d;
        std::memset(&d, 0, sizeof(d));
        g_want_status.push_back(ll_gather_info_opts(fresh, x.axis, x.elem_bytes, options_of(x.option_set), &d));
        g_want.push_back(d);
        ll_layout_destroy(fresh);
    }
    if (ll_plan_convert(g_layouts[2], g_layouts[3], 2, &g_plan) != LL_OK || ll_plan_info(g_plan, &g_plan_want) != LL_OK) return 1;

    std::vector<std::thread> pool;
    for (int t = 0; t < threads; ++t) pool.emplace_back(worker, t, rounds);
    for (std::thread &t : pool) t.join();
    ll_plan_destroy(g_plan);
    for (ll_layout *l : g_layouts) ll_layout_destroy(l);
    printf("threads %d rounds %d queries %zu mismatches %ld\n", threads, rounds, g_queries.size(), g_bad.load());
    return g_bad.load() == 0 ? 0 : 1;
}

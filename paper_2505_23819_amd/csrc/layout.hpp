// Internal definitions behind the opaque handles of ll.h.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <memory>
#include <string>
#include <vector>

#include "../../include/ll.h"
#include "f2.hpp"

namespace ll {
struct GatherCache;   // kernel choices ll_gather has already made for one layout (run.cpp)
// Holder that does not travel with copies: a layout copied and then changed must not inherit the
// choices made for the original.  Read and replaced only through std::atomic_load / atomic_store.
struct GatherCacheSlot {
    std::shared_ptr<const GatherCache> p;
    GatherCacheSlot() = default;
    GatherCacheSlot(const GatherCacheSlot &) {}
    GatherCacheSlot &operator=(const GatherCacheSlot &) { p.reset(); return *this; }
};
}   // namespace ll

struct ll_layout {
    int n_in = 0;
    ll_in_dim in_dims[LL_MAX_IN_DIMS] = {};
    int n_out = 0;
    ll_out_dim out_dims[LL_MAX_OUT_DIMS] = {};
    int d_in = 0;
    int d_out = 0;
    f2::mat bases;   // d_in columns, each a d_out-bit flattened output index
    f2::vec offset = 0;   // affine part: index h holds logical element (bases h) xor offset
    mutable ll::GatherCacheSlot gather_cache;   // not part of the layout's value

    int bits_of(int label) const
    {
        for (int i = 0; i < n_in; ++i)
            if (in_dims[i].label == label) return in_dims[i].nbits;
        return 0;
    }
    int first_bit_of(int label) const   // position of the first input bit of `label` (or d_in)
    {
        int pos = 0;
        for (int i = 0; i < n_in; ++i) {
            if (in_dims[i].label >= label) return pos;
            pos += in_dims[i].nbits;
        }
        return pos;
    }
};

namespace ll {

// ll_options (options.cpp): every field LL_AUTO; LL_AUTO plus the LL_* environment overrides; the
// process defaults (the environment read once); a caller's struct made complete (NULL = process
// defaults); field-wise comparison; and readers for byte sizes (powers of two) and XCD chunk
// counts (returned as log2, -1 = natural order).
void options_init(ll_options *o);
void options_from_env(ll_options *o);
const ll_options &process_options();
ll_options resolve_options(const ll_options *given);
bool same_options(const ll_options &a, const ll_options &b);
unsigned opt_bytes(int32_t v, unsigned fallback);
int opt_chunk_bits(int32_t v, int fallback_bits);
inline int opt_or(int32_t v, int fallback) { return v == LL_AUTO ? fallback : v; }

// thread-local error text behind ll_last_error()
ll_status fail(ll_status code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
const char *last_error();

// new layout object from dims and columns (no validation beyond allocation)
ll_status make_layout(const ll_in_dim *in_dims, int n_in, const ll_out_dim *out_dims, int n_out,
                      const f2::mat &bases, ll_layout **out);

}  // namespace ll

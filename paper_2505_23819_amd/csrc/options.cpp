// ll_options: defaults, the environment overrides used for experiments, and the process-wide
// defaults that the entry points without an options argument use (read from the environment once).
#include <cstdlib>
#include <cstring>
#include <cstddef>

#include "layout.hpp"

namespace ll {

namespace {
struct Field {
    const char *env;
    size_t offset;
};
#define LL_FIELD(name, envname) {envname, offsetof(ll_options, name)}
const Field kFields[] = {
    LL_FIELD(strategy, "LL_STRATEGY"),
    LL_FIELD(gather_kernel, "LL_GATHER_KERNEL"),
    LL_FIELD(block_bytes, "LL_BLOCK_BYTES"),
    LL_FIELD(pref_bytes, "LL_PREF_BYTES"),
    LL_FIELD(elem_threads_log2, "LL_ELEM_THREADS_LOG2"),
    LL_FIELD(vec_block_bytes, "LL_VEC_BLOCK_BYTES"),
    LL_FIELD(vec_threads, "LL_VEC_THREADS"),
    LL_FIELD(shuffle_block_bytes, "LL_SHUFFLE_BLOCK_BYTES"),
    LL_FIELD(inflight_bytes, "LL_INFLIGHT_BYTES"),
    LL_FIELD(lds_pad_bytes, "LL_LDS_PAD_BYTES"),
    LL_FIELD(xcd_chunk, "LL_XCD_CHUNK"),
    LL_FIELD(pull_mode, "LL_PULL_MODE"),
    LL_FIELD(pull_vec_bits, "LL_PULL_VEC_BITS"),
    LL_FIELD(pull_inflight_bytes, "LL_PULL_INFLIGHT_BYTES"),
    LL_FIELD(pull_xcd_chunk, "LL_PULL_XCD_CHUNK"),
    LL_FIELD(gather_block_bytes, "LL_GATHER_BLOCK_BYTES"),
    LL_FIELD(gather_lds_max_bytes, "LL_GATHER_LDS_MAX_BYTES"),
    LL_FIELD(gather_min_run_bytes, "LL_GATHER_MIN_RUN_BYTES"),
    LL_FIELD(gather_phased_max_bytes, "LL_GATHER_PHASED_MAX_BYTES"),
    LL_FIELD(gather_threads_log2, "LL_GATHER_THREADS_LOG2"),
    LL_FIELD(gather_inflight_bytes, "LL_GATHER_INFLIGHT_BYTES"),
    LL_FIELD(gather_xcd_chunk, "LL_GATHER_XCD_CHUNK"),
    LL_FIELD(gather_swizzle_always, "LL_GATHER_SWIZZLE_ALWAYS"),
    LL_FIELD(copy_xcd_chunk, "LL_COPY_XCD_CHUNK"),
    LL_FIELD(debug, "LL_DEBUG"),
    LL_FIELD(gather_waves, "LL_GATHER_WAVES"),
    LL_FIELD(pull_threads_log2, "LL_PULL_THREADS_LOG2"),
};
#undef LL_FIELD
int32_t &field(ll_options *o, size_t offset) { return *reinterpret_cast<int32_t *>(reinterpret_cast<char *>(o) + offset); }
}  // namespace

void options_init(ll_options *o)
{
    for (const Field &f : kFields) field(o, f.offset) = LL_AUTO;
    o->size = (int32_t)sizeof(ll_options);
}

void options_from_env(ll_options *o)
{
    options_init(o);
    for (const Field &f : kFields)
        if (const char *v = getenv(f.env)) {
            char *end = nullptr;
            const long x = strtol(v, &end, 10);
            if (end != v && x >= -1 && x <= 0x7fffffffL) field(o, f.offset) = (int32_t)x;
        }
}

const ll_options &process_options()
{
    static const ll_options defaults = [] {
        ll_options o;
        options_from_env(&o);
        return o;
    }();
    return defaults;
}

ll_options resolve_options(const ll_options *given)
{
    if (!given) return process_options();
    ll_options o;
    options_init(&o);
    // a caller built against a shorter struct: the fields it does not know stay LL_AUTO
    const size_t have = given->size > 0 ? (size_t)given->size : 0;
    for (const Field &f : kFields)
        if (f.offset + sizeof(int32_t) <= have) field(&o, f.offset) = *reinterpret_cast<const int32_t *>(reinterpret_cast<const char *>(given) + f.offset);
    return o;
}

bool same_options(const ll_options &a, const ll_options &b)
{
    for (const Field &f : kFields)
        if (field(const_cast<ll_options *>(&a), f.offset) != field(const_cast<ll_options *>(&b), f.offset)) return false;
    return true;
}

unsigned opt_bytes(int32_t v, unsigned fallback)
{
    return (v >= 16 && v <= (1 << 20) && (v & (v - 1)) == 0) ? (unsigned)v : fallback;
}

int opt_chunk_bits(int32_t v, int fallback_bits)
{
    if (v == LL_AUTO) return fallback_bits;
    return v > 1 ? 31 - __builtin_clz((unsigned)v) : -1;
}

}  // namespace ll

extern "C" {

ll_status ll_options_init(ll_options *opts)
{
    if (!opts) return ll::fail(LL_ERR_INVALID_ARG, "opts is null");
    ll::options_init(opts);
    return LL_OK;
}

ll_status ll_options_from_env(ll_options *opts)
{
    if (!opts) return ll::fail(LL_ERR_INVALID_ARG, "opts is null");
    ll::options_from_env(opts);
    return LL_OK;
}

}  // extern "C"

// extern "C" entry points of ll.h: argument checking and marshalling only.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "layout.hpp"
#include "plan.hpp"

namespace ll {

static thread_local char g_error[512] = "";

ll_status fail(ll_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

const char *last_error() { return g_error; }

ll_status make_layout(const ll_in_dim *in_dims, int n_in, const ll_out_dim *out_dims, int n_out,
                      const f2::mat &bases, ll_layout **out)
{
    ll_layout *l = new (std::nothrow) ll_layout();
    if (!l) return fail(LL_ERR_INVALID_ARG, "out of host memory");
    l->n_in = n_in;
    l->n_out = n_out;
    for (int i = 0; i < n_in; ++i) {
        l->in_dims[i] = in_dims[i];
        l->d_in += in_dims[i].nbits;
    }
    for (int i = 0; i < n_out; ++i) {
        l->out_dims[i] = out_dims[i];
        l->d_out += out_dims[i].nbits;
    }
    l->bases = bases;
    *out = l;
    return LL_OK;
}

}  // namespace ll

using ll::fail;

extern "C" {

ll_status ll_layout_create(const ll_in_dim *in_dims, int n_in, const ll_out_dim *out_dims, int n_out,
                           const uint64_t *bases, ll_layout **out)
{
    try {
        if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
        *out = nullptr;
        if (!in_dims || !out_dims) return fail(LL_ERR_INVALID_ARG, "in_dims / out_dims is null");
        if (n_in < 1 || n_in > LL_MAX_IN_DIMS) return fail(LL_ERR_INVALID_ARG, "n_in must be in [1, %d]", LL_MAX_IN_DIMS);
        if (n_out < 1 || n_out > LL_MAX_OUT_DIMS) return fail(LL_ERR_INVALID_ARG, "n_out must be in [1, %d]", LL_MAX_OUT_DIMS);
        int d_in = 0, d_out = 0;
        for (int i = 0; i < n_in; ++i) {
            if (in_dims[i].label < LL_IN_REG || in_dims[i].label > LL_IN_OFFSET)
                return fail(LL_ERR_INVALID_ARG, "in_dims[%d]: unknown label %d", i, in_dims[i].label);
            if (i > 0 && in_dims[i].label <= in_dims[i - 1].label)
                return fail(LL_ERR_INVALID_ARG, "in_dims must be in canonical order (register, lane, wave, tile)");
            if (in_dims[i].label == LL_IN_OFFSET && n_in != 1)
                return fail(LL_ERR_INVALID_ARG, "an offset input cannot be mixed with hardware inputs");
            if (in_dims[i].nbits < 0) return fail(LL_ERR_INVALID_ARG, "in_dims[%d]: negative bit count", i);
            d_in += in_dims[i].nbits;
        }
        for (int i = 0; i < n_out; ++i) {
            if (out_dims[i].nbits < 0) return fail(LL_ERR_INVALID_ARG, "out_dims[%d]: negative bit count", i);
            d_out += out_dims[i].nbits;
        }
        if (d_in > LL_MAX_BITS || d_out > LL_MAX_BITS)
            return fail(LL_ERR_INVALID_ARG, "layouts are limited to %d input and output bits", LL_MAX_BITS);
        if (d_in > 0 && !bases) return fail(LL_ERR_INVALID_ARG, "bases is null");
        f2::mat cols(d_in);
        for (int k = 0; k < d_in; ++k) {
            if (bases[k] >> d_out) return fail(LL_ERR_INVALID_ARG, "bases[%d] = 0x%llx does not fit in %d output bits", k,
                                               (unsigned long long)bases[k], d_out);
            cols[k] = bases[k];
        }
        return ll::make_layout(in_dims, n_in, out_dims, n_out, cols, out);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_create: out of host memory");
    }
}

ll_status ll_layout_destroy(ll_layout *layout)
{
    try {
        delete layout;
        return LL_OK;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_destroy: out of host memory");
    }
}

ll_status ll_layout_get(const ll_layout *layout, int *n_in, ll_in_dim *in_dims, int *n_out, ll_out_dim *out_dims,
                        uint64_t *bases)
{
    try {
        if (!layout) return fail(LL_ERR_INVALID_ARG, "layout is null");
        if (n_in) *n_in = layout->n_in;
        if (n_out) *n_out = layout->n_out;
        if (in_dims) std::memcpy(in_dims, layout->in_dims, sizeof(ll_in_dim) * layout->n_in);
        if (out_dims) std::memcpy(out_dims, layout->out_dims, sizeof(ll_out_dim) * layout->n_out);
        if (bases)
            for (int k = 0; k < layout->d_in; ++k) bases[k] = layout->bases[k];
        return LL_OK;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_get: out of host memory");
    }
}

ll_status ll_layout_apply(const ll_layout *layout, uint64_t in_index, uint64_t *out_index)
{
    try {
        if (!layout || !out_index) return fail(LL_ERR_INVALID_ARG, "null argument");
        if (layout->d_in < 64 && (in_index >> layout->d_in))
            return fail(LL_ERR_INVALID_ARG, "in_index 0x%llx does not fit in %d input bits", (unsigned long long)in_index, layout->d_in);
        *out_index = f2::apply(layout->bases, in_index) ^ layout->offset;
        return LL_OK;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_apply: out of host memory");
    }
}

ll_status ll_compose(const ll_layout *outer, const ll_layout *inner, ll_layout **out)
{
    try {
        if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
        *out = nullptr;
        if (!outer || !inner) return fail(LL_ERR_INVALID_ARG, "null layout");
        if (inner->d_out != outer->d_in)
            return fail(LL_ERR_DIM_MISMATCH, "inner maps to %d bits but outer takes %d bits", inner->d_out, outer->d_in);
        ll_status st = ll::make_layout(inner->in_dims, inner->n_in, outer->out_dims, outer->n_out,
                                       f2::compose(outer->bases, inner->bases), out);
        // affine parts: outer(inner(h)) = A1 (A2 h ^ b2) ^ b1
        if (st == LL_OK) (*out)->offset = f2::apply(outer->bases, inner->offset) ^ outer->offset;
        return st;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_compose: out of host memory");
    }
}

ll_status ll_layout_with_offset(const ll_layout *layout, uint64_t offset, ll_layout **out)
{
    try {
        if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
        *out = nullptr;
        if (!layout) return fail(LL_ERR_INVALID_ARG, "layout is null");
        if (layout->d_out < 64 && (offset >> layout->d_out))
            return fail(LL_ERR_INVALID_ARG, "offset 0x%llx does not fit in %d output bits", (unsigned long long)offset, layout->d_out);
        ll_status st = ll::make_layout(layout->in_dims, layout->n_in, layout->out_dims, layout->n_out, layout->bases, out);
        if (st == LL_OK) (*out)->offset = offset;
        return st;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_with_offset: out of host memory");
    }
}

ll_status ll_layout_slice(const ll_layout *layout, int dim, ll_layout **out)
{
    try {
        if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
        *out = nullptr;
        if (!layout) return fail(LL_ERR_INVALID_ARG, "layout is null");
        if (layout->n_out < 2) return fail(LL_ERR_INVALID_ARG, "a slice needs at least two logical dims");
        if (dim < 0 || dim >= layout->n_out) return fail(LL_ERR_INVALID_ARG, "dim %d is not one of the %d logical dims", dim, layout->n_out);
        // flat output bits [lo, lo + nb) belong to `dim` (last dim fastest): squeeze them out
        int lo = 0;
        for (int j = dim + 1; j < layout->n_out; ++j) lo += layout->out_dims[j].nbits;
        const int nb = layout->out_dims[dim].nbits;
        const f2::vec low = (f2::vec(1) << lo) - 1;
        auto squeeze = [&](f2::vec x) { return (x & low) | ((x >> (lo + nb)) << lo); };
        ll_out_dim dims[LL_MAX_OUT_DIMS];
        int n = 0;
        for (int j = 0; j < layout->n_out; ++j)
            if (j != dim) dims[n++] = layout->out_dims[j];
        f2::mat cols;
        for (f2::vec c : layout->bases) cols.push_back(squeeze(c));
        ll_status st = ll::make_layout(layout->in_dims, layout->n_in, dims, n, cols, out);
        if (st == LL_OK) (*out)->offset = squeeze(layout->offset);
        return st;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_slice: out of host memory");
    }
}

ll_status ll_layout_get_offset(const ll_layout *layout, uint64_t *offset)
{
    try {
        if (!layout || !offset) return fail(LL_ERR_INVALID_ARG, "null argument");
        *offset = layout->offset;
        return LL_OK;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_get_offset: out of host memory");
    }
}

ll_status ll_product(const ll_layout *a, const ll_layout *b, ll_layout **out)
{
    try {
        if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
        *out = nullptr;
        if (!a || !b) return fail(LL_ERR_INVALID_ARG, "null layout");
        if (a->d_in + b->d_in > LL_MAX_BITS || a->d_out + b->d_out > LL_MAX_BITS)
            return fail(LL_ERR_INVALID_ARG, "product exceeds %d bits", LL_MAX_BITS);
        if (a->n_out + b->n_out > LL_MAX_OUT_DIMS) return fail(LL_ERR_INVALID_ARG, "product has too many output dims");
        // merged input dims, label by label: bits of `a` first, then bits of `b`
        ll_in_dim dims[LL_MAX_IN_DIMS];
        int n = 0;
        f2::mat cols;
        for (int label = LL_IN_REG; label <= LL_IN_OFFSET; ++label) {
            const int na = a->bits_of(label), nb = b->bits_of(label);
            bool present = false;
            for (int i = 0; i < a->n_in; ++i) present |= a->in_dims[i].label == label;
            for (int i = 0; i < b->n_in; ++i) present |= b->in_dims[i].label == label;
            if (!present) continue;
            dims[n].label = label;
            dims[n].nbits = na + nb;
            ++n;
            const int fa = a->first_bit_of(label), fb = b->first_bit_of(label);
            for (int k = 0; k < na; ++k) cols.push_back(a->bases[fa + k]);
            for (int k = 0; k < nb; ++k) cols.push_back(b->bases[fb + k] << a->d_out);   // b's outputs sit above a's
        }
        bool has_offset = false, has_hw = false;
        for (int i = 0; i < n; ++i) (dims[i].label == LL_IN_OFFSET ? has_offset : has_hw) = true;
        if (has_offset && has_hw) return fail(LL_ERR_DIM_MISMATCH, "cannot multiply a memory layout with a distributed layout");
        // output dims, slowest first: those of b (upper bits), then those of a
        ll_out_dim odims[LL_MAX_OUT_DIMS];
        int m = 0;
        for (int i = 0; i < b->n_out; ++i) odims[m++] = b->out_dims[i];
        for (int i = 0; i < a->n_out; ++i) odims[m++] = a->out_dims[i];
        const ll_status st = ll::make_layout(dims, n, odims, m, cols, out);
        // affine factors: (A1 h1 ^ b1, A2 h2 ^ b2) = (A1 x A2)(h1, h2) ^ (b1, b2)
        if (st == LL_OK) (*out)->offset = a->offset | (b->offset << a->d_out);
        return st;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_product: out of host memory");
    }
}

ll_status ll_invert(const ll_layout *layout, ll_layout **out)
{
    try {
        if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
        *out = nullptr;
        if (!layout) return fail(LL_ERR_INVALID_ARG, "layout is null");
        f2::mat inv;
        if (!f2::right_inverse(layout->bases, layout->d_out, &inv))
            return fail(LL_ERR_NOT_SURJECTIVE, "layout of rank %d does not cover its %d output bits", f2::rank(layout->bases),
                        layout->d_out);
        ll_in_dim in = {LL_IN_OFFSET, layout->d_out};
        ll_out_dim o = {layout->d_in};
        ll_status st = ll::make_layout(&in, 1, &o, 1, inv, out);
        // h = X (x ^ b) = X x ^ X b
        if (st == LL_OK) (*out)->offset = f2::apply(inv, layout->offset);
        return st;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_invert: out of host memory");
    }
}

ll_status ll_plan_convert(const ll_layout *src, const ll_layout *dst, int elem_bytes, ll_plan **out)
{
    return ll_plan_convert_opts(src, dst, elem_bytes, nullptr, out);
}

ll_status ll_plan_convert_opts(const ll_layout *src, const ll_layout *dst, int elem_bytes, const ll_options *opts, ll_plan **out)
{
    try {
        if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
        *out = nullptr;
        if (!src || !dst) return fail(LL_ERR_INVALID_ARG, "null layout");
        ll_plan *p = new (std::nothrow) ll_plan();
        if (!p) return fail(LL_ERR_INVALID_ARG, "out of host memory");
        p->opts = ll::resolve_options(opts);
        ll_status st = ll::plan_convert(src, dst, elem_bytes, p);
        if (st != LL_OK) {
            delete p;
            return st;
        }
        *out = p;
        return LL_OK;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_plan_convert: out of host memory");
    }
}

ll_status ll_plan_info(const ll_plan *plan, ll_plan_desc *out)
{
    try {
        if (!plan || !out) return fail(LL_ERR_INVALID_ARG, "null argument");
        *out = plan->desc;
        return LL_OK;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_plan_info: out of host memory");
    }
}

ll_status ll_plan_destroy(ll_plan *plan)
{
    try {
        delete plan;
        return LL_OK;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_plan_destroy: out of host memory");
    }
}

static bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

ll_status ll_convert(const ll_plan *plan, const void *src_dev, void *dst_dev, int64_t ntiles, void *hip_stream)
{
    try {
        if (!plan) return fail(LL_ERR_INVALID_ARG, "plan is null");
        if (ntiles < 0) return fail(LL_ERR_INVALID_ARG, "ntiles is negative");
        if (ntiles == 0) return LL_OK;
        if (!src_dev || !dst_dev) return fail(LL_ERR_INVALID_ARG, "null device pointer");
        if (misaligned(src_dev) || misaligned(dst_dev)) return fail(LL_ERR_INVALID_ARG, "device buffers must be 16-byte aligned");
        const int dmax = plan->desc.d > plan->desc.d_dst ? plan->desc.d : plan->desc.d_dst;
        if (ntiles > (1ll << 40) >> dmax) return fail(LL_ERR_INVALID_ARG, "ntiles is too large");
        const unsigned long long sbytes = (unsigned long long)ntiles * plan->desc.elem_bytes << plan->desc.d;
        const unsigned long long dbytes = (unsigned long long)ntiles * plan->desc.elem_bytes << plan->desc.d_dst;
        // every access is a 16-byte vector: tiles smaller than that must come in whole vectors
        if ((sbytes | dbytes) & 15)
            return fail(LL_ERR_INVALID_ARG, "ntiles * tile bytes (%llu source, %llu destination) must be a multiple of 16", sbytes, dbytes);
        const char *s = static_cast<const char *>(src_dev), *t = static_cast<const char *>(dst_dev);
        if (s < t + dbytes && t < s + sbytes) return fail(LL_ERR_INVALID_ARG, "source and destination buffers overlap");
        return ll::run_convert(plan, src_dev, dst_dev, ntiles, hip_stream);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_convert: out of host memory");
    }
}

ll_status ll_gather(const ll_layout *layout, int axis, int elem_bytes, const void *in_dev, const int32_t *idx_dev,
                    void *out_dev, int64_t ntiles, void *hip_stream)
{
    return ll_gather_opts(layout, axis, elem_bytes, nullptr, in_dev, idx_dev, out_dev, ntiles, hip_stream);
}

ll_status ll_gather_opts(const ll_layout *layout, int axis, int elem_bytes, const ll_options *opts, const void *in_dev,
                         const int32_t *idx_dev, void *out_dev, int64_t ntiles, void *hip_stream)
{
    try {
        if (!layout) return fail(LL_ERR_INVALID_ARG, "layout is null");
        if (ntiles < 0) return fail(LL_ERR_INVALID_ARG, "ntiles is negative");
        if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8)
            return fail(LL_ERR_INVALID_ARG, "elem_bytes must be 1, 2, 4 or 8 (got %d)", elem_bytes);
        if (axis < 0 || axis >= layout->n_out) return fail(LL_ERR_INVALID_ARG, "axis %d is not an output dim", axis);
        // the layout is validated even when there is nothing to move
        if (!opts) return ll::run_gather(layout, axis, elem_bytes, nullptr, in_dev, idx_dev, out_dev, ntiles, hip_stream);
        const ll_options full = ll::resolve_options(opts);
        return ll::run_gather(layout, axis, elem_bytes, &full, in_dev, idx_dev, out_dev, ntiles, hip_stream);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_gather: out of host memory");
    }
}

ll_status ll_gather_info(const ll_layout *layout, int axis, int elem_bytes, ll_gather_desc *out)
{
    return ll_gather_info_opts(layout, axis, elem_bytes, nullptr, out);
}

ll_status ll_gather_info_opts(const ll_layout *layout, int axis, int elem_bytes, const ll_options *opts, ll_gather_desc *out)
{
    try {
        if (!layout || !out) return fail(LL_ERR_INVALID_ARG, "null argument");
        if (!opts) return ll::describe_gather(layout, axis, elem_bytes, nullptr, out);
        const ll_options full = ll::resolve_options(opts);
        return ll::describe_gather(layout, axis, elem_bytes, &full, out);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_gather_info: out of host memory");
    }
}

ll_status ll_copy(const void *src_dev, void *dst_dev, int64_t bytes, void *hip_stream)
{
    try {
        if (bytes < 0 || (bytes & 15)) return fail(LL_ERR_INVALID_ARG, "bytes must be a non-negative multiple of 16");
        if (bytes == 0) return LL_OK;
        if (!src_dev || !dst_dev) return fail(LL_ERR_INVALID_ARG, "null device pointer");
        if (misaligned(src_dev) || misaligned(dst_dev)) return fail(LL_ERR_INVALID_ARG, "device buffers must be 16-byte aligned");
        const char *ps = static_cast<const char *>(src_dev), *pd = static_cast<const char *>(dst_dev);
        if (ps < pd + bytes && pd < ps + bytes) return fail(LL_ERR_INVALID_ARG, "source and destination buffers overlap");
        return ll::launch_copy(src_dev, dst_dev, bytes, ll::copy_xcd_chunk_bits(ll::process_options()), hip_stream);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_copy: out of host memory");
    }
}

const char *ll_last_error(void) { return ll::last_error(); }

}  // extern "C"

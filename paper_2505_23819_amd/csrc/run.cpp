// Host side of the device entry points: pick the kernel a plan names, fill the per-call fields of
// its argument block, validate the gather layout (paper Sec. 5.5) and launch.
#include <cstdlib>
#include <cstring>

#include "plan.hpp"

using f2::mat;
using f2::vec;

namespace ll {

ll_status run_convert(const ll_plan *plan, const void *src, void *dst, long long ntiles, void *stream)
{
    const ll_plan_desc &desc = plan->desc;
    switch (desc.strategy) {
    case LL_STRATEGY_COPY:
        return launch_copy(src, dst, (ntiles << desc.d) * desc.elem_bytes, stream);
    case LL_STRATEGY_LDS_ELEM: {
        LdsElemArgs a = plan->lds_elem;
        a.src = src;
        a.dst = dst;
        a.ntiles = ntiles;
        const long long groups = (ntiles + (1ll << a.group_bits) - 1) >> a.group_bits;
        a.nblocks = groups << a.coset_bits;
        return launch_lds_elem(a, desc.elem_bytes, plan->nvec, desc.lds_vec_bits, desc.threads, desc.lds_bytes, stream);
    }
    case LL_STRATEGY_LDS_TR: {
        LdsElemArgs a = plan->lds_elem;
        a.src = src;
        a.dst = dst;
        a.ntiles = ntiles;
        const long long groups = (ntiles + (1ll << a.group_bits) - 1) >> a.group_bits;
        a.nblocks = groups << a.coset_bits;
        return launch_lds_tr(a, desc.elem_bytes, plan->nvec, desc.lds_bytes, stream);
    }
    case LL_STRATEGY_REG_PERMUTE:
    case LL_STRATEGY_WAVE_SHUFFLE:
    case LL_STRATEGY_LDS_VEC: {
        VecArgs a = plan->vec;
        a.src = src;
        a.dst = dst;
        a.ntiles = ntiles;
        const long long groups = (ntiles + (1ll << a.group_bits) - 1) >> a.group_bits;
        a.nblocks = groups << a.coset_bits;
        return launch_vec(a, desc.elem_bytes, plan->vec_nvec_bits, plan->vec_tpose, plan->vec_xchg, desc.threads,
                          desc.lds_bytes, stream);
    }
    case LL_STRATEGY_LDS_PULL: {
        PullArgs a = plan->pull;
        a.src = src;
        a.dst = dst;
        a.ntiles = ntiles;
        const long long groups = (ntiles + (1ll << a.group_bits) - 1) >> a.group_bits;
        a.nblocks = groups << a.coset_bits;
        return launch_pull(a, desc.elem_bytes, plan->pull_src_iters, plan->pull_vec_bits, desc.lds_bytes, stream);
    }
    default:
        return fail(LL_ERR_UNSUPPORTED, "plan strategy %d has no kernel", desc.strategy);
    }
}

ll_status run_gather(const ll_layout *L, int axis, int elem_bytes, const void *in, const int32_t *idx, void *out,
                     long long ntiles, void *stream)
{
    for (int i = 0; i < L->n_in; ++i)
        if (L->in_dims[i].label == LL_IN_OFFSET)
            return fail(LL_ERR_INVALID_ARG, "gather needs a distributed layout (register / lane / wave / tile inputs)");
    const int d = L->d_in;
    if (f2::rank(L->bases) < L->d_out) return fail(LL_ERR_NOT_SURJECTIVE, "layout does not cover the whole logical tensor");
    if (d > L->d_out) return fail(LL_ERR_NOT_INJECTIVE, "layouts with broadcasting are not supported");
    mat linv;
    if (!f2::invert(L->bases, d, &linv)) return fail(LL_ERR_NOT_INJECTIVE, "layout is not bijective");
    const int nreg = L->bits_of(LL_IN_REG), nlane = L->bits_of(LL_IN_LANE);
    if (nlane != LL_WAVE_LANE_BITS) return fail(LL_ERR_UNSUPPORTED, "gather needs %d lane bits (wave64), layout has %d", LL_WAVE_LANE_BITS, nlane);
    const int nhigh = d - nreg - nlane;              // wave (and tile) bits of the layout
    if (nhigh > 16) return fail(LL_ERR_UNSUPPORTED, "gather supports at most 16 wave + tile bits");
    if (nreg > 6) return fail(LL_ERR_UNSUPPORTED, "gather supports at most 6 register bits (got %d)", nreg);

    int axis_shift = 0;
    for (int k = L->n_out - 1; k > axis; --k) axis_shift += L->out_dims[k].nbits;
    const int na = L->out_dims[axis].nbits;
    const vec reg_mask = (vec(1) << nreg) - 1;
    const vec lane_mask = vec(63) << nreg;

    GatherArgs a;
    std::memset(&a, 0, sizeof(a));
    // Moving one step along axis bit b moves the hardware index by L^-1(e_b): it must stay inside
    // the wave (Sec. 5.5: the warp part of the layout restricted to the axis vanishes).
    for (int b = 0; b < na; ++b)
        if (linv[axis_shift + b] & ~(reg_mask | lane_mask))
            return fail(LL_ERR_AXIS_NOT_IN_WAVE, "axis bit %d crosses waves: the gather axis must lie inside one wave", b);
    for (int b = 0; b < na; ++b) {
        const vec delta = linv[axis_shift + b];
        if (delta & reg_mask)
            return fail(LL_ERR_UNSUPPORTED, "axis bit %d lives in registers; only lane-resident axes are implemented", b);
        a.lane_delta[b] = (uint32_t)((delta & lane_mask) >> nreg);
    }
    if (na > 6) return fail(LL_ERR_AXIS_NOT_IN_WAVE, "axis of 2^%d elements cannot fit in 64 lanes", na);
    auto axis_coord = [&](vec h) { return (uint32_t)((f2::apply(L->bases, h) >> axis_shift) & ((vec(1) << na) - 1)); };
    for (int b = 0; b < 6; ++b) a.own_lane[b] = axis_coord(vec(1) << (nreg + b));
    for (int r = 0; r < (1 << nreg); ++r) a.own_reg[r] = axis_coord((vec)r);
    for (int b = 0; b < nhigh; ++b) a.own_wave[b] = axis_coord(vec(1) << (nreg + 6 + b));
    for (int b = 0; b < nreg; ++b) a.own_regbit[b] = axis_coord(vec(1) << b);
    a.nwave = nhigh;
    a.nreg = nreg;
    a.axis_mask = (1u << na) - 1;
    // fast form: the axis is a contiguous field of the lane index holding the coordinate itself
    a.fast = 0;
    if (na > 0) {
        int shift = __builtin_ctz(a.lane_delta[0]);
        bool ok = true;
        for (int b = 0; b < na; ++b) ok &= a.lane_delta[b] == (1u << (shift + b));
        for (int b = 0; b < 6; ++b) {
            const uint32_t want = (b >= shift && b < shift + na) ? (1u << (b - shift)) : 0u;
            ok &= a.own_lane[b] == want;
        }
        for (int r = 0; r < (1 << nreg); ++r) ok &= a.own_reg[r] == 0;
        for (int b = 0; b < nhigh; ++b) ok &= a.own_wave[b] == 0;
        if (ok) {
            a.fast = 1;
            a.shift = shift;
            a.keep_mask = 63u & ~(a.axis_mask << shift);
        }
    }
    if (ntiles == 0) return LL_OK;
    if (!in || !idx || !out) return fail(LL_ERR_INVALID_ARG, "null device pointer");
    if ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(idx) | reinterpret_cast<uintptr_t>(out)) & 15)
        return fail(LL_ERR_INVALID_ARG, "device buffers must be 16-byte aligned");
    const unsigned long long bytes = ((unsigned long long)ntiles << d) * elem_bytes;
    if (ntiles > (1ll << 40) >> d) return fail(LL_ERR_INVALID_ARG, "ntiles is too large");
    const char *pi = static_cast<const char *>(in), *po = static_cast<const char *>(out);
    const char *px = reinterpret_cast<const char *>(idx);
    const unsigned long long ibytes = ((unsigned long long)ntiles << d) * 4;
    if ((pi < po + bytes && po < pi + bytes) || (px < po + bytes && po < px + ibytes))
        return fail(LL_ERR_INVALID_ARG, "the output buffer overlaps an input buffer");
    a.in = in;
    a.idx = idx;
    a.out = out;
    a.nchunks = ntiles << nhigh;
    // Rows of 16 bytes are already one coalesced vector per lane: shuffle directly.  Wider rows would
    // make every lane's accesses strided, so they are staged through wave-private LDS instead.
    const int row_bytes = (1 << nreg) * elem_bytes;
    a.staged = (row_bytes > 16 && row_bytes <= 256 && nreg >= 2) ? 1 : 0;
    if (const char *force = getenv("LL_GATHER_STAGED")) a.staged = atoi(force) && row_bytes >= 16 && row_bytes <= 256 && nreg >= 2;
    return launch_gather(a, elem_bytes, stream);
}

}  // namespace ll

// LDS staging read back with the gfx950 transposing LDS loads (ds_read_b64_tr_b16 / _tr_b8): the
// hardware tile the paper's Sec. 5.3 "Using SIMD Hardware Primitives" asks for, selected by the
// left-division test of Def. "Left Division".
//
// Measured behaviour of the instructions (16 lanes form a group; lane i16 = lane % 16):
//   ds_read_b64_tr_b16: every lane supplies the address of an 8-byte chunk (4 elements); lane i16
//     receives, as element j = 0..3 of its result, element (i16 % 4) of the chunk whose address was
//     supplied by lane (i16 / 4) + 4 j of its group;
//   ds_read_b64_tr_b8: 8 elements per chunk; element j = 0..7 of lane i16's result is element
//     (i16 % 8) of the chunk supplied by lane (i16 / 8) + 2 j.
// As a tile: the low ce = log2(8 / w) lane bits map by the identity onto the low ce bits of the LDS
// offset (the element inside a chunk); everything else is free, because the chunk addresses come
// from registers.  So the instruction can serve a read whose layout L (result registers, lanes,
// iterations -> LDS offset) is divisible on the left by id_ce^{lane, offset}, after the kernel's
// lanes are chosen suitably (the lane analogue of "Generalized Vectorization").
#include <algorithm>
#include <cstring>
#include <vector>

#include "plan.hpp"

using f2::mat;
using f2::vec;

namespace ll {

static int ilog2t(unsigned x) { return 31 - __builtin_clz(x); }

static vec xor_sel(const mat &cols, int first, unsigned idx)
{
    vec r = 0;
    for (int b = 0; (idx >> b) != 0; ++b)
        if ((idx >> b) & 1) r ^= cols[first + b];
    return r;
}

// Host-side walk of one block with the instruction's lane behaviour, as the kernel indexes it.
static ll_status check_tr_block(const LdsElemArgs &a, const mat &pext, int n, int vs, int ce, int w, int nvec,
                                uint32_t cs, uint32_t cd, uint32_t cr)
{
    const int run = 1 << ce, nsub = 1 << (vs - ce);
    const uint32_t block_bytes = (uint32_t)((1u << n) * (unsigned)w);
    const uint64_t group_elems = 1ull << (a.d + a.group_bits);
    std::vector<int64_t> held(block_bytes / w, -1);
    auto lane_part = [&](const uint32_t *tab, int tid) {
        uint32_t x = 0;
        for (int b = 0; b < 8; ++b)
            if ((tid >> b) & 1) x ^= tab[b];
        return x;
    };
    for (int tid = 0; tid < 256; ++tid)
        for (int i = 0; i < nvec; ++i) {
            const uint32_t off = cs ^ lane_part(a.lane_src, tid) ^ a.iter_src[i];
            if (off >= group_elems || (off & ((1u << vs) - 1))) return fail(LL_ERR_INVALID_ARG, "internal: bad source offset in transposing-read plan");
            for (int s = 0; s < nsub; ++s) {
                const uint32_t addr = lane_part(a.lds_wr_lane, tid) ^ a.lds_wr_iter[i] ^ a.lds_wr_sub[s];
                if (addr >= block_bytes || addr % 8u) return fail(LL_ERR_INVALID_ARG, "internal: bad LDS write address in transposing-read plan");
                for (int e = 0; e < run; ++e) {
                    int64_t &slot = held[addr / w + e];
                    if (slot >= 0) return fail(LL_ERR_INVALID_ARG, "internal: LDS writes overlap in transposing-read plan");
                    slot = (int64_t)off + s * run + e;
                }
            }
        }
    for (int tid = 0; tid < 256; ++tid)
        for (int i = 0; i < nvec; ++i) {
            const uint32_t off = cd ^ lane_part(a.lane_dst, tid) ^ a.iter_dst[i];
            if (off >= group_elems || (off & ((1u << vs) - 1))) return fail(LL_ERR_INVALID_ARG, "internal: bad destination offset in transposing-read plan");
            const int group = tid & ~15, i16 = tid & 15;
            for (int s = 0; s < nsub; ++s)
                for (int j = 0; j < run; ++j) {
                    const int supplier = group + (i16 >> ce) + (j << (4 - ce));
                    const uint32_t addr = cr ^ lane_part(a.lds_rd_lane, supplier) ^ a.lds_rd_iter[i] ^ a.lds_rd_sub[s];
                    if (addr >= block_bytes || addr % 8u) return fail(LL_ERR_INVALID_ARG, "internal: bad LDS read address in transposing-read plan");
                    const int64_t from = held[addr / w + (i16 & (run - 1))];
                    if (from < 0 || f2::apply(pext, (vec)from) != (vec)off + s * run + j)
                        return fail(LL_ERR_INVALID_ARG, "internal: transposing-read plan does not realise the conversion");
                }
        }
    return LL_OK;
}

ll_status plan_lds_tr(const mat &p, int d, int w, ll_plan *plan, bool *applied)
{
    *applied = false;
    if (w != 1 && w != 2) return LL_OK;
    const LdsModel hw;
    const int vs = ilog2t(16u / (unsigned)w), ce = ilog2t(8u / (unsigned)w), tb = 8;
    BlockGeom geom;
    if (ll_status st = build_blocks(p, d, w, vs + tb, opt_bytes(plan->opts.block_bytes, 8192u), opt_bytes(plan->opts.pref_bytes, 8192u), &geom);
        st != LL_OK)
        return st;
    const int g = geom.g, k = geom.k, n = geom.n;
    const mat &pext = geom.pext, &us = geom.us, &ud = geom.ud, &q = geom.q, &qinv = geom.qinv, &comp = geom.comp;
    const int nvec_bits = n - vs - tb;
    if (nvec_bits < 0 || (1 << nvec_bits) > 8) return LL_OK;
    const vec posmask = (vec(1) << vs) - 1, cemask = (vec(1) << ce) - 1, low_mask = (vec(1) << k) - 1;

    // Left division of the read layout by the tile id_ce^{lane, offset}.  The read layout sends a
    // destination-local index (position bits = result registers, the rest = lanes and iterations)
    // to the source-local index Q^-1 x, whose low ce bits are the element inside an LDS chunk.
    //  * upper-left block: the kernel's low ce lane bits must map onto those bits by the identity:
    //    the lanes are free to choose, so lane bit j is given the direction Q e_j, which must be a
    //    direction between destination vectors (zero position bits);
    //  * upper-right block zero: no other input reaches the low ce offset bits: for the position
    //    bits this is a condition on Q^-1; the remaining lane / iteration directions are reduced
    //    against the first ce ones until it holds;
    //  * the per-block shift (low bits of P h_c) must keep chunks whole as well.
    for (int j = 0; j < ce; ++j)
        if (q[j] & posmask) return LL_OK;
    for (int b = 0; b < vs; ++b)
        if (qinv[b] & cemask) return LL_OK;
    for (vec h : comp)
        if (f2::apply(qinv, f2::apply(pext, h) & low_mask) & cemask) return LL_OK;
    mat y;                                           // basis of the destination vector-index space
    f2::Basis span;
    for (int j = 0; j < ce; ++j) {
        y.push_back(q[j]);
        if (!span.add(q[j])) return LL_OK;
    }
    for (int b = vs; b < n; ++b) {
        vec cand = vec(1) << b;
        const vec inside = f2::apply(qinv, cand) & cemask;
        for (int j = 0; j < ce; ++j)
            if ((inside >> j) & 1) cand ^= q[j];
        if (span.add(cand)) y.push_back(cand);
    }
    if ((int)y.size() != n - vs) return fail(LL_ERR_INVALID_ARG, "internal: destination basis of a transposing-read plan");

    // which basis vector each physical lane bit stands for when the lane SUPPLIES a chunk address:
    // lane bits 0 .. 3-ce take the group's lanes ce .. 3, lane bits 4-ce .. 3 take result elements
    mat supplier(tb);
    for (int b = 0; b < tb; ++b) {
        if (b < 4 - ce) supplier[b] = y[ce + b];
        else if (b < 4) supplier[b] = vec(1) << (b - (4 - ce));
        else supplier[b] = y[b];
    }
    mat wr_lanes, rd_lanes;
    for (int b = 0; b < 6; ++b) {
        wr_lanes.push_back(vec(1) << (vs + b));
        rd_lanes.push_back(f2::apply(qinv, supplier[b]));
    }
    int wfw = 1, wfr = 1;
    const mat m = synthesize_swizzle(n, ce, w, wr_lanes, rd_lanes, hw, &wfw, &wfr);
    mat sw;
    if (!f2::invert(m, n, &sw)) return fail(LL_ERR_INVALID_ARG, "internal: swizzle not invertible");
    const mat swq = f2::compose(sw, qinv);

    LdsElemArgs &a = plan->lds_elem;
    std::memset(&a, 0, sizeof(a));
    a.d = d; a.group_bits = g; a.coset_bits = (int)comp.size(); a.thread_bits = tb;
    for (size_t c = 0; c < comp.size(); ++c) {
        const vec ph = f2::apply(pext, comp[c]);
        a.coset_src[c] = (uint32_t)comp[c];
        a.coset_dst[c] = (uint32_t)(ph & ~low_mask);
        a.coset_lds_rd[c] = (uint32_t)(f2::apply(swq, ph & low_mask) * (vec)w);
    }
    for (int b = 0; b < tb; ++b) {
        a.lane_src[b] = (uint32_t)us[vs + b];
        a.lds_wr_lane[b] = (uint32_t)(sw[vs + b] * (vec)w);
        a.lane_dst[b] = (uint32_t)f2::apply(ud, y[b]);
        a.lds_rd_lane[b] = (uint32_t)(f2::apply(swq, supplier[b]) * (vec)w);
    }
    for (int i = 0; i < (1 << nvec_bits); ++i) {
        a.iter_src[i] = (uint32_t)xor_sel(us, vs + tb, (unsigned)i);
        a.lds_wr_iter[i] = (uint32_t)(xor_sel(sw, vs + tb, (unsigned)i) * (vec)w);
        const vec yi = xor_sel(y, tb, (unsigned)i);
        a.iter_dst[i] = (uint32_t)f2::apply(ud, yi);
        a.lds_rd_iter[i] = (uint32_t)(f2::apply(swq, yi) * (vec)w);
    }
    for (int s = 0; s < (1 << (vs - ce)); ++s) {
        a.lds_wr_sub[s] = (uint32_t)(xor_sel(sw, ce, (unsigned)s) * (vec)w);
        a.lds_rd_sub[s] = (uint32_t)(xor_sel(swq, ce, (unsigned)s) * (vec)w);
    }
    plan->nvec = 1 << nvec_bits;
    {
        ll_status st = check_tr_block(a, pext, n, vs, ce, w, plan->nvec, 0, 0, 0);
        uint32_t cs = 0, cd = 0, cr = 0;
        for (int c = 0; c < a.coset_bits && st == LL_OK; ++c) {
            st = check_tr_block(a, pext, n, vs, ce, w, plan->nvec, a.coset_src[c], a.coset_dst[c], a.coset_lds_rd[c]);
            cs ^= a.coset_src[c]; cd ^= a.coset_dst[c]; cr ^= a.coset_lds_rd[c];
        }
        if (st == LL_OK && a.coset_bits > 1) st = check_tr_block(a, pext, n, vs, ce, w, plan->nvec, cs, cd, cr);
        if (st != LL_OK) return st;
    }

    ll_plan_desc &desc = plan->desc;
    desc.strategy = LL_STRATEGY_LDS_TR;
    desc.global_vec_bytes = 16;
    desc.lds_write_bytes = desc.lds_read_bytes = 8;
    desc.lds_bytes = (1 << n) * w;
    desc.threads = 256;
    desc.vectors_per_thread = 1 << nvec_bits;
    desc.block_bits = n; desc.group_bits = g; desc.segment_bits = k;
    desc.shuffle_rounds = 0;
    desc.lds_vec_bits = ce;
    const int cls = lds_width_class(8);
    desc.lds_banks = hw.rd_banks[cls]; desc.lds_banks_write = hw.wr_banks[cls];
    desc.lds_phase_lanes_write = 1 << hw.wr_phase_dim[cls];
    desc.lds_phase_lanes_read = 1 << hw.rd_phase_dim[cls];
    desc.predicted_wavefronts_write = wfw;
    desc.predicted_wavefronts_read = wfr;
    for (int j = 0; j < n; ++j) desc.lds_mem[j] = m[j];
    *applied = true;
    return LL_OK;
}

}  // namespace ll

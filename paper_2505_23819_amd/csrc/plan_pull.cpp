// Planner of conversions between layouts with broadcasting (paper Sec. 5.1 "Broadcasting",
// Sec. 5.4 rule 2).  A and B are surjective onto the same logical tensor but need not be
// injective and may have different numbers of input bits.  The conversion is the "pull" map
// R = A^+ o B from destination hardware indices to source hardware indices, A^+ being the right
// inverse with free variables zero: dst[hB] = src[R hB].
#include <algorithm>
#include <cstring>
#include <vector>

#include "plan.hpp"

using f2::mat;
using f2::vec;

namespace ll {

static int ilog2p(unsigned x) { return 31 - __builtin_clz(x); }

static mat cat(const mat &a, const mat &b)
{
    mat r = a;
    r.insert(r.end(), b.begin(), b.end());
    return r;
}

static vec xor_sel(const mat &cols, int first, unsigned idx)
{
    vec r = 0;
    for (int b = 0; (idx >> b) != 0; ++b)
        if ((idx >> b) & 1) r ^= cols[first + b];
    return r;
}

// Host-side walk of one block, as the kernel indexes it.
static ll_status check_pull_block(const PullArgs &a, const mat &rext, vec cconst, int vs, int v, int w, int tb, int src_iters, int lds_bytes,
                                  uint32_t cs, uint32_t cd, uint32_t cr)
{
    const int threads = 1 << tb;
    const int E = 1 << vs, A = 1 << v;                // elements per global vector / per LDS access
    const uint64_t src_group = 1ull << (a.d_src + a.group_bits), dst_group = 1ull << (a.d_dst + a.group_bits);
    std::vector<int64_t> held((size_t)lds_bytes / w, -1);
    auto lane_part = [&](const uint32_t *tab, int tid) {
        uint32_t x = 0;
        for (int b = 0; b < tb; ++b)
            if ((tid >> b) & 1) x ^= tab[b];
        return x;
    };
    for (int tid = 0; tid < threads; ++tid)
        for (int i = 0; i < src_iters; ++i) {
            if ((unsigned)(tid + threads * i) >= (1u << a.src_vec_bits)) continue;
            const uint32_t off = cs ^ lane_part(a.lane_src, tid) ^ a.iter_src[i];
            if (off >= src_group || (off & (uint32_t)(E - 1))) return fail(LL_ERR_INVALID_ARG, "internal: bad source offset in broadcast plan");
            for (int s = 0; s < E; ++s) {
                const uint32_t base = lane_part(a.lds_wr_lane, tid) ^ a.lds_wr_iter[i] ^ a.lds_wr_sub[s / A];
                if (base % (uint32_t)(w * A)) return fail(LL_ERR_INVALID_ARG, "internal: misaligned LDS write in broadcast plan");
                const uint32_t addr = base + (uint32_t)((s % A) * w);
                if (addr >= (uint32_t)lds_bytes) return fail(LL_ERR_INVALID_ARG, "internal: bad LDS write address in broadcast plan");
                if (held[addr / w] >= 0) return fail(LL_ERR_INVALID_ARG, "internal: LDS writes overlap in broadcast plan");
                held[addr / w] = (int64_t)off + s;
            }
        }
    for (int tid = 0; tid < threads; ++tid)
        for (int it = 0; it < a.dst_iters; ++it) {
            uint32_t ib = 0, ob = 0;
            for (int b = 0; (it >> b) != 0; ++b)
                if ((it >> b) & 1) { ib ^= a.lds_rd_iter_bit[b]; ob ^= a.iter_dst_bit[b]; }
            const uint32_t off = cd ^ lane_part(a.lane_dst, tid) ^ ob;
            if (off >= dst_group || (off & (uint32_t)(E - 1))) return fail(LL_ERR_INVALID_ARG, "internal: bad destination offset in broadcast plan");
            for (int s = 0; s < E; ++s) {
                const uint32_t base = cr ^ lane_part(a.lds_rd_lane, tid) ^ ib ^ a.lds_rd_sub[s / A];
                if (base % (uint32_t)(w * A)) return fail(LL_ERR_INVALID_ARG, "internal: misaligned LDS read in broadcast plan");
                const uint32_t addr = base + (uint32_t)((s % A) * w);
                if (addr >= (uint32_t)lds_bytes || held[addr / w] < 0)
                    return fail(LL_ERR_INVALID_ARG, "internal: bad LDS read address in broadcast plan");
                if ((vec)held[addr / w] != (f2::apply(rext, (vec)off + s) ^ cconst))
                    return fail(LL_ERR_INVALID_ARG, "internal: broadcast plan does not realise the conversion");
            }
        }
    return LL_OK;
}

// One attempt with blocks of at most 2^n_max elements.  *too_large: the source vectors behind such a
// block exceed what one workgroup stages (a source whose 16-byte vectors hold few canonical slots).
static ll_status plan_pull_at(const ll_layout *A, const ll_layout *B, int w, int mode, int n_max, int tb, ll_plan *plan, bool *too_large)
{
    const LdsModel hw;
    const int dA = A->d_in, dB = B->d_in, dl = A->d_out;
    const int vs = ilog2p(16u / (unsigned)w);
    mat aplus;
    if (!f2::right_inverse(A->bases, dl, &aplus)) return fail(LL_ERR_NOT_SURJECTIVE, "source layout does not cover the whole logical tensor");
    const mat r = f2::compose(aplus, B->bases);                 // dB columns in F2^dA
    // affine layouts: x = B hB ^ b is held by the source slot A^+ (x ^ a) = R hB ^ A^+ (a ^ b)
    const vec cconst = f2::apply(aplus, A->offset ^ B->offset);
    // pivots of A: the source bits the right inverse may use
    vec pivots = 0;
    for (vec c : aplus) pivots |= c;

    const int g = std::max(0, n_max - std::min(dA, dB));        // bundle small tiles
    const int Ds = dA + g, Dd = dB + g;
    if (std::max(Ds, Dd) + ilog2p((unsigned)w) > 31) return fail(LL_ERR_UNSUPPORTED, "tile too large");
    mat rext = r;                                               // Dd columns in F2^Ds
    for (int t = 0; t < g; ++t) {
        rext.push_back(vec(1) << (dA + t));
        pivots |= vec(1) << (dA + t);
    }
    // a preimage under R of every pivot source bit, and a basis of ker R (destination broadcast directions)
    f2::Basis rb;                                               // echelon basis of the images with their preimages as tags
    mat kernel_r;
    for (int k = 0; k < Dd; ++k) {
        vec dep = 0;
        if (!rb.add(rext[k], vec(1) << k, &dep)) kernel_r.push_back(dep);
    }
    auto preimage = [&](vec src_vec, vec *out) {
        vec tag = 0;
        if (rb.reduce(src_vec, &tag) != 0) return false;
        *out = tag;
        return true;
    };
    // Block = destination runs of 2^kd slots plus the destination slots that pull from source runs
    // of 2^ks slots (pivot bits only).  Longer runs on a side mean longer contiguous pieces of HBM on
    // that side; the side that moves more bytes gets its run bits first.
    int nrep = 0;                                    // destination broadcast directions taken into the block first
    auto block_space = [&](int ks, int kd) {
        mat gens;
        for (int j = 0; j < kd; ++j) gens.push_back(vec(1) << j);
        for (int j = 0; j < nrep; ++j) gens.push_back(kernel_r[(size_t)j]);
        for (int j = 0; j < ks && j < Ds; ++j) {
            vec pre;
            if (((pivots >> j) & 1) && preimage(vec(1) << j, &pre)) gens.push_back(pre);
        }
        return f2::extend({}, gens);
    };
    if (vs > Ds || vs > Dd) return fail(LL_ERR_UNSUPPORTED, "tile smaller than one 16-byte vector");
    int ks = vs, kd = vs;
    auto fits = [&](int s_, int d_) { return (int)block_space(s_, d_).size() <= n_max; };
    if (mode == 1) {
        // destination runs first, but not at the price of 16-byte source pieces: the source side gets
        // runs of a 128-byte line before the destination takes the rest (random bit correspondences
        // between the two sides otherwise leave every source line fetched by eight blocks)
        const int line = std::max(vs, ilog2p(128u / (unsigned)w));
        while (ks < Ds && ks < line && fits(ks + 1, kd)) ++ks;
        // ... and the replicas of an element stay in one block while destination runs of 1 KiB remain,
        // so that every source element is fetched by one block instead of one per replica
        for (const int run = std::max(vs, ilog2p(1024u / (unsigned)w)); nrep < (int)kernel_r.size();) {
            ++nrep;
            if (!fits(ks, std::min(Dd, run))) { --nrep; break; }
        }
        while (kd < Dd && fits(ks, kd + 1)) ++kd;
        while (ks < Ds && fits(ks + 1, kd)) ++ks;
    } else if (mode == 2) {
        while (ks < Ds && fits(ks + 1, kd)) ++ks;
        while (kd < Dd && fits(ks, kd + 1)) ++kd;
    } else {
        for (bool grew = true; grew;) {
            grew = false;
            if (kd < Dd && fits(ks, kd + 1)) { ++kd; grew = true; }
            if (ks < Ds && fits(ks + 1, kd)) { ++ks; grew = true; }
        }
    }
    const int k = kd;
    mat Ud = block_space(ks, kd);
    // destination broadcast directions: keep replicas of one element in one block while it fits
    for (vec kv : kernel_r)
        if ((int)Ud.size() < n_max) Ud = f2::extend({}, cat(Ud, {kv}));
    for (int j = k; j < Dd && (int)Ud.size() < vs + tb; ++j) Ud = f2::extend({}, cat(Ud, {vec(1) << j}));
    const int nd = (int)Ud.size();
    if (nd < vs + tb) return fail(LL_ERR_UNSUPPORTED, "internal: destination block smaller than one vector per thread");
    if (nd - vs - tb > 8) return fail(LL_ERR_UNSUPPORTED, "internal: destination block too large");
    const vec low_mask = (vec(1) << k) - 1;
    // destination-local basis
    mat ud;
    for (int j = 0; j < k; ++j) ud.push_back(vec(1) << j);
    {
        mat cand;
        for (vec x : Ud) cand.push_back(x & ~low_mask);
        for (vec x : f2::extend(ud, cand)) ud.push_back(x);
    }
    // Source block: the 16-byte vectors that hold R(Ud).  R only reaches slots whose replica bits
    // are zero, so above the vector bits the block is spanned by pivot bits alone: replicas in the
    // source image are never read (unless they share a 16-byte vector with a slot that is).
    const vec src_low = (vec(1) << vs) - 1;
    mat us;
    for (int j = 0; j < vs; ++j) us.push_back(vec(1) << j);
    {
        mat cand;
        for (int j = vs; j < ks && j < Ds; ++j)
            if ((pivots >> j) & 1) cand.push_back(vec(1) << j);
        for (vec x : ud) cand.push_back(f2::apply(rext, x) & ~src_low);
        for (vec x : f2::extend(us, cand)) us.push_back(x);
    }
    const int ns = (int)us.size();
    if ((int)ud.size() != nd) return fail(LL_ERR_INVALID_ARG, "internal: broadcast block basis mismatch");
    // R in block-local coordinates (ns x nd)
    f2::Basis usb;
    for (int j = 0; j < ns; ++j) usb.add(us[j], vec(1) << j);
    mat rl(nd);
    for (int j = 0; j < nd; ++j) {
        vec tag = 0;
        if (usb.reduce(f2::apply(rext, ud[j]), &tag) != 0) return fail(LL_ERR_INVALID_ARG, "internal: broadcast block not closed");
        rl[j] = tag;
    }
    const mat comp = f2::complement(Ud, Dd);
    if ((int)comp.size() > kMaxCosetBits) return fail(LL_ERR_UNSUPPORTED, "internal: too many blocks per tile");
    const int src_vec_bits = ns - vs;
    const int src_iters = std::max(1, 1 << std::max(0, src_vec_bits - tb));
    if (src_iters > kPullMaxSrcIters) {
        *too_large = true;
        return fail(LL_ERR_UNSUPPORTED, "internal: source block too large");
    }

    // LDS access width: 2^v elements where the conversion keeps the low v bits of a slot index in
    // place (Sec. 5.3 "Generalized Vectorization"), element-wide otherwise
    int v = vs;
    if (plan->opts.pull_vec_bits != LL_AUTO) v = std::min(vs, std::max(0, (int)plan->opts.pull_vec_bits));
    for (int j = 0; j < nd; ++j)
        while (v > 0 && (j < v ? rl[j] != (vec(1) << j) : (rl[j] & ((vec(1) << v) - 1)) != 0)) --v;
    for (vec c : comp)
        while (v > 0 && (f2::apply(rext, c) & ((vec(1) << v) - 1)) != 0) --v;
    while (v > 0 && (cconst & ((vec(1) << v) - 1)) != 0) --v;
    for (int j = 0; j < v; ++j)
        if (rl[j] != (vec(1) << j)) return fail(LL_ERR_INVALID_ARG, "internal: vector bits of a broadcast plan");
    mat wr_lanes, rd_lanes;
    for (int b = 0; b < 6; ++b) {
        wr_lanes.push_back(vs + b < ns ? vec(1) << (vs + b) : 0);
        rd_lanes.push_back(rl[vs + b]);
    }
    int wfw = 1, wfr = 1;
    const mat m = synthesize_swizzle(ns, v, w, wr_lanes, rd_lanes, hw, &wfw, &wfr);
    mat sw;
    if (!f2::invert(m, ns, &sw)) return fail(LL_ERR_INVALID_ARG, "internal: swizzle not invertible");
    const mat swr = f2::compose(sw, rl);            // destination-local index -> LDS element offset

    PullArgs &a = plan->pull;
    std::memset(&a, 0, sizeof(a));
    a.d_src = dA; a.d_dst = dB; a.group_bits = g; a.coset_bits = (int)comp.size();
    a.src_vec_bits = src_vec_bits;
    a.dst_iters = 1 << (nd - vs - tb);
    a.src_xor = (uint32_t)(cconst & ~src_low);
    a.lds_rd_xor = (uint32_t)(f2::apply(sw, cconst & src_low) * (vec)w);
    for (size_t c = 0; c < comp.size(); ++c) {
        const vec sc = f2::apply(rext, comp[c]);
        a.coset_dst[c] = (uint32_t)comp[c];
        a.coset_src[c] = (uint32_t)(sc & ~src_low);
        a.coset_lds_rd[c] = (uint32_t)(f2::apply(sw, sc & src_low) * (vec)w);
    }
    for (int b = 0; b < tb; ++b) {
        a.lane_src[b] = vs + b < ns ? (uint32_t)us[vs + b] : 0u;
        a.lds_wr_lane[b] = vs + b < ns ? (uint32_t)(sw[vs + b] * (vec)w) : 0u;
        a.lane_dst[b] = (uint32_t)ud[vs + b];
        a.lds_rd_lane[b] = (uint32_t)(swr[vs + b] * (vec)w);
    }
    for (int i = 0; i < src_iters; ++i) {
        a.iter_src[i] = (uint32_t)xor_sel(us, vs + tb, (unsigned)i);
        a.lds_wr_iter[i] = (uint32_t)(xor_sel(sw, vs + tb, (unsigned)i) * (vec)w);
    }
    for (int b = 0; b < nd - vs - tb; ++b) {
        a.iter_dst_bit[b] = (uint32_t)ud[vs + tb + b];
        a.lds_rd_iter_bit[b] = (uint32_t)(swr[vs + tb + b] * (vec)w);
    }
    for (int s = 0; s < (1 << (vs - v)); ++s) {      // one entry per LDS access of 2^v elements
        a.lds_wr_sub[s] = (uint32_t)(xor_sel(sw, v, (unsigned)s) * (vec)w);
        a.lds_rd_sub[s] = (uint32_t)(xor_sel(swr, v, (unsigned)s) * (vec)w);
    }
    const int lds_bytes = (1 << ns) * w;
    plan->pull_src_iters = src_iters;
    plan->pull_vec_bits = v;
    plan->pull_thread_bits = tb;
    {
        ll_status st = check_pull_block(a, rext, cconst, vs, v, w, tb, src_iters, lds_bytes, a.src_xor, 0, a.lds_rd_xor);
        const uint32_t cs0 = a.src_xor, cr0 = a.lds_rd_xor;
        uint32_t cs = cs0, cd = 0, cr = cr0;
        for (int c = 0; c < a.coset_bits && st == LL_OK; ++c) {
            st = check_pull_block(a, rext, cconst, vs, v, w, tb, src_iters, lds_bytes, cs0 ^ a.coset_src[c], a.coset_dst[c], cr0 ^ a.coset_lds_rd[c]);
            cs ^= a.coset_src[c]; cd ^= a.coset_dst[c]; cr ^= a.coset_lds_rd[c];
        }
        if (st == LL_OK && a.coset_bits > 1) st = check_pull_block(a, rext, cconst, vs, v, w, tb, src_iters, lds_bytes, cs, cd, cr);
        if (st != LL_OK) return st;
    }

    ll_plan_desc &desc = plan->desc;
    desc.kind = LL_KIND_BROADCAST;
    desc.strategy = LL_STRATEGY_LDS_PULL;
    desc.d = dA;
    desc.d_dst = dB;
    for (int j = 0; j < dB; ++j) desc.pull[j] = r[j];
    desc.conv_offset = cconst;       // source index = pull * hB xor conv_offset
    desc.global_vec_bytes = 16;
    desc.lds_write_bytes = desc.lds_read_bytes = w << v;
    desc.lds_bytes = lds_bytes;
    desc.threads = 1 << tb;
    desc.vectors_per_thread = a.dst_iters;
    desc.block_bits = nd; desc.group_bits = g; desc.segment_bits = k;
    desc.lds_vec_bits = v;
    const int cls = lds_width_class(w << v);
    desc.lds_banks = hw.rd_banks[cls]; desc.lds_banks_write = hw.wr_banks[cls];
    desc.lds_phase_lanes_write = 1 << hw.wr_phase_dim[cls];
    desc.lds_phase_lanes_read = 1 << hw.rd_phase_dim[cls];
    desc.predicted_wavefronts_write = wfw;
    desc.predicted_wavefronts_read = wfr;
    return LL_OK;
}

ll_status plan_pull(const ll_layout *A, const ll_layout *B, int w, ll_plan *plan)
{
    const int vs = ilog2p(16u / (unsigned)w);
    const int tb = plan->opts.pull_threads_log2 == 6 ? 6 : 8;
    // A destination that replicates 4x or more makes the conversion write-dominated: destination
    // runs first, and 16 KiB blocks (four stores in flight per thread measured fastest on MI355X;
    // read-dominated and balanced conversions do best at 8 KiB).
    int mode = B->d_in > A->d_out + 1 ? 1 : 0;
    if (plan->opts.pull_mode != LL_AUTO) mode = plan->opts.pull_mode;
    const unsigned max_block = opt_bytes(plan->opts.block_bytes, mode == 1 ? 16384u : 8192u);
    // A sparse source (few canonical slots per 16-byte vector, as in the slice left by a reduction
    // along the register-fastest dim) needs many vectors per destination element: shrink the block
    // until they fit.  At one vector per thread on the destination side a block needs at most one
    // source vector per element, 2^vs per thread, which the kernel covers.
    for (int n_max = std::max(vs + tb, ilog2p(max_block / (unsigned)w));; --n_max) {
        bool too_large = false;
        const ll_status st = plan_pull_at(A, B, w, mode, n_max, tb, plan, &too_large);
        if (st == LL_OK || !too_large || n_max == vs + tb) return st;
    }
}

}  // namespace ll


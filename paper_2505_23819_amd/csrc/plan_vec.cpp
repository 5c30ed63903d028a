// Planners of the vector-preserving strategies: register transposes combined with no exchange,
// with lane <-> register butterfly stages inside a wave (paper Sec. 5.4 "Intra-thread" and
// "Intra-warp Data Exchange"), or with 128-bit accesses to XOR-swizzled LDS ("Optimal Swizzling"
// with the whole 16-byte vector as the common run).
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <utility>
#include <vector>

#include "plan.hpp"

using f2::mat;
using f2::vec;

namespace ll {

static thread_local bool g_debug = false;      // ll_options.debug of the plan being made
static ll_status dbg_na(int where)
{
    if (g_debug) fprintf(stderr, "[ll] wave-shuffle plan not applicable (reason %d)\n", where);
    return LL_OK;
}

static int ilog2u(unsigned x) { return 31 - __builtin_clz(x); }

static vec xor_bits(const mat &cols, unsigned idx)
{
    vec r = 0;
    for (int b = 0; (idx >> b) != 0; ++b)
        if ((idx >> b) & 1) r ^= cols[b];
    return r;
}

// Host-side execution of the vector kernel's data movement on element identities, for block 0,
// the block of every single block-index bit and the block of all bits: every offset in range and
// 16-byte aligned, LDS vector slots written once, every element stored where the conversion sends
// it.  Turns a planner mistake into an error status instead of a GPU fault.
static ll_status check_vec_block(const VecArgs &a, const mat &pext, int vs, int w, int nvb, int tpose, int xchg,
                                 int lds_bytes, uint32_t cs, uint32_t cd, uint32_t cr)
{
    const int threads = 1 << a.thread_bits, nv = 1 << nvb, E = 1 << vs;
    const uint64_t group_elems = 1ull << (a.d + a.group_bits);
    auto lane_part = [&](const uint32_t *tab, int tid) {
        uint32_t x = 0;
        for (int b = 0; b < a.thread_bits; ++b)
            if ((tid >> b) & 1) x ^= tab[b];
        return x;
    };
    // regs[tid][i][e] = source element offset held there
    std::vector<int64_t> regs((size_t)threads * nv * E), tmp(regs.size());
    auto at = [&](std::vector<int64_t> &r, int tid, int i, int e) -> int64_t & { return r[((size_t)tid * nv + i) * E + e]; };
    for (int tid = 0; tid < threads; ++tid)
        for (int i = 0; i < nv; ++i) {
            const uint32_t off = cs ^ lane_part(a.lane_src, tid) ^ a.iter_src[i];
            if (off >= group_elems || (off & (uint32_t)(E - 1))) return fail(LL_ERR_INVALID_ARG, "internal: bad source offset in vector plan");
            for (int e = 0; e < E; ++e) at(regs, tid, i, e) = (int64_t)off + e;
        }
    auto transpose = [&]() {
        if (nv < E) return false;
        for (int tid = 0; tid < threads; ++tid)
            for (int h = 0; h < nv / E; ++h)
                for (int pnew = 0; pnew < E; ++pnew)
                    for (int c = 0; c < E; ++c) at(tmp, tid, pnew + E * h, c) = at(regs, tid, c + E * h, pnew);
        regs.swap(tmp);
        return true;
    };
    if (tpose == kTposeBefore && !transpose()) return fail(LL_ERR_INVALID_ARG, "internal: transpose needs 2^vs vectors");
    if (xchg == kXchgShuffle) {
        if (threads != 64) return fail(LL_ERR_INVALID_ARG, "internal: shuffle plan must use one wave");
        for (int b = 0; b < nvb && b < 5; ++b) {
            const uint32_t mask = a.stage_mask[b];
            if (!mask) continue;
            if (mask > 63) return fail(LL_ERR_INVALID_ARG, "internal: bad lane mask in vector plan");
            tmp = regs;
            for (int lane = 0; lane < 64; ++lane) {
                const bool upper = (lane & mask) != 0;
                const int partner = lane ^ (int)mask;
                for (int i = 0; i < nv; ++i) {
                    if ((i >> b) & 1) continue;
                    for (int e = 0; e < E; ++e) {
                        if (upper) at(tmp, lane, i, e) = at(regs, partner, i | (1 << b), e);
                        else at(tmp, lane, i | (1 << b), e) = at(regs, partner, i, e);
                    }
                }
            }
            regs.swap(tmp);
        }
    }
    if (xchg == kXchgLds) {
        const int slots = lds_bytes / 16;
        std::vector<int> owner(slots, -1);
        std::vector<int64_t> held((size_t)slots * E);
        for (int tid = 0; tid < threads; ++tid)
            for (int i = 0; i < nv; ++i) {
                const uint32_t addr = lane_part(a.lds_wr_lane, tid) ^ a.lds_wr_iter[i];
                if (addr >= (uint32_t)lds_bytes || (addr & 15)) return fail(LL_ERR_INVALID_ARG, "internal: bad LDS write address in vector plan");
                if (owner[addr / 16] >= 0) return fail(LL_ERR_INVALID_ARG, "internal: LDS writes overlap in vector plan");
                owner[addr / 16] = tid;
                for (int e = 0; e < E; ++e) held[(size_t)(addr / 16) * E + e] = at(regs, tid, i, e);
            }
        for (int tid = 0; tid < threads; ++tid)
            for (int i = 0; i < nv; ++i) {
                const uint32_t addr = cr ^ lane_part(a.lds_rd_lane, tid) ^ a.lds_rd_iter[i];
                if (addr >= (uint32_t)lds_bytes || (addr & 15) || owner[addr / 16] < 0)
                    return fail(LL_ERR_INVALID_ARG, "internal: bad LDS read address in vector plan");
                for (int e = 0; e < E; ++e) at(regs, tid, i, e) = held[(size_t)(addr / 16) * E + e];
            }
    }
    if (tpose == kTposeAfter && !transpose()) return fail(LL_ERR_INVALID_ARG, "internal: transpose needs 2^vs vectors");
    for (int tid = 0; tid < threads; ++tid)
        for (int i = 0; i < nv; ++i) {
            const uint32_t off = cd ^ lane_part(a.lane_dst, tid) ^ a.iter_dst[i];
            if (off >= group_elems || (off & (uint32_t)(E - 1))) return fail(LL_ERR_INVALID_ARG, "internal: bad destination offset in vector plan");
            for (int e = 0; e < E; ++e)
                if (f2::apply(pext, (vec)at(regs, tid, i, e)) != (vec)off + e)
                    return fail(LL_ERR_INVALID_ARG, "internal: vector plan does not realise the conversion");
        }
    (void)w;
    return LL_OK;
}

static ll_status check_vec_tables(const VecArgs &a, const mat &pext, int vs, int w, int nvb, int tpose, int xchg, int lds_bytes)
{
    ll_status st = check_vec_block(a, pext, vs, w, nvb, tpose, xchg, lds_bytes, 0, 0, 0);
    uint32_t cs = 0, cd = 0, cr = 0;
    for (int c = 0; c < a.coset_bits && st == LL_OK; ++c) {
        st = check_vec_block(a, pext, vs, w, nvb, tpose, xchg, lds_bytes, a.coset_src[c], a.coset_dst[c], a.coset_lds_rd[c]);
        cs ^= a.coset_src[c];
        cd ^= a.coset_dst[c];
        cr ^= a.coset_lds_rd[c];
    }
    if (st == LL_OK && a.coset_bits > 1) st = check_vec_block(a, pext, vs, w, nvb, tpose, xchg, lds_bytes, cs, cd, cr);
    return st;
}

// ---------------------------------------------------------------------------------------------
// Intra-wave exchange by lane <-> register butterfly stages (and the register-only case with no
// stage at all).  Paper Sec. 5.4 "Intra-warp Data Exchange" computes, for distributed layouts,
// I = A_thr n B_thr, E = A_thr \ I, F = B_thr \ I and pairs e_i with f_i.  Here the "threads" are
// the kernel's own lanes (bits vs..vs+5 of the block-local index on both sides, which is what
// makes global accesses coalesced), E are the lane bits that must become register bits, F the
// register bits that must become lane bits, and every pair (e_i, f_i) is one stage that trades
// one lane bit for one register bit.  Register indices stay static, so a stage moves half of the
// registers of every lane; a plan has |E| stages.  The position-in-vector bits join through an
// in-register transpose with the low iteration bits before or after the stages.
// Built for conversions that are bit permutations inside a block.
// ---------------------------------------------------------------------------------------------
static ll_status plan_wave_shuffle_at(const mat &p, int d, int w, unsigned max_block, ll_plan *plan, bool *applied);

// Blocks of 4 KiB (a wave with 4 vectors per lane) unless their runs are only one 128-byte line
// long or the block comes out smaller: then 8 KiB blocks are tried and taken if they apply and
// lengthen the runs.  Interleaved A/B on 30 random bit permutations of 2^12..2^18 elements (TB/s, 4 / 8
// KiB): short-run cases 5.6-6.3 -> 6.4-6.7, the others equal within 1 %; configs 1 and 3 (runs of 512
// and 256 bytes) are 1-2 % faster with 4 KiB and keep it; 16 KiB (16 vectors per lane) drops to 3.7-5.3.
ll_status plan_wave_shuffle(const mat &p, int d, int w, ll_plan *plan, bool *applied)
{
    *applied = false;
    g_debug = plan->opts.debug == 1;
    if (w != 2 && w != 4 && w != 8) return dbg_na(1);
    if (plan->opts.shuffle_block_bytes != LL_AUTO)      // one fixed block size
        return plan_wave_shuffle_at(p, d, w, opt_bytes(plan->opts.shuffle_block_bytes, 4096u), plan, applied);
    ll_plan small = *plan;
    bool small_ok = false;
    if (ll_status st = plan_wave_shuffle_at(p, d, w, 4096u, &small, &small_ok); st != LL_OK) return st;
    // (8-byte elements: a 4 KiB block is 4 vectors per lane of 2 elements each, and 8 KiB measured 2-10 % faster throughout)
    const bool short_runs = small_ok && (w == 8 || ((unsigned)w << small.desc.segment_bits) <= 128u || ((unsigned)w << small.desc.block_bits) < 4096u);
    if (small_ok && !short_runs) {
        *plan = small;
        *applied = true;
        return LL_OK;
    }
    ll_plan wide = *plan;
    bool wide_ok = false;
    if (ll_status st = plan_wave_shuffle_at(p, d, w, 8192u, &wide, &wide_ok); st != LL_OK) return st;
    if (wide_ok && (!small_ok || wide.desc.segment_bits > small.desc.segment_bits)) {
        *plan = wide;
        *applied = true;
    } else if (small_ok) {
        *plan = small;
        *applied = true;
    }
    return LL_OK;
}

static ll_status plan_wave_shuffle_at(const mat &p, int d, int w, unsigned max_block, ll_plan *plan, bool *applied)
{
    *applied = false;
    const int vs = ilog2u(16u / (unsigned)w), tb = 6;
    BlockGeom g;
    // a transposing plan needs 2^vs vectors per lane
    if (build_blocks(p, d, w, 2 * vs + tb, max_block, max_block, &g) != LL_OK) return dbg_na(2);
    const int n = g.n, nvb = n - vs - tb;
    if (nvb > 4 || nvb < 0) return dbg_na(3);
    // bit permutation inside the block?
    std::vector<int> pi(n), pinv(n);
    for (int m = 0; m < n; ++m) {
        if (f2::popcount(g.q[m]) != 1) return dbg_na(4);
        pi[m] = f2::top_bit(g.q[m]);
        pinv[pi[m]] = m;
    }
    // blocks must land on 16-byte boundaries
    for (vec h : g.comp)
        if (f2::apply(g.pext, h) & ((vec(1) << vs) - 1)) return dbg_na(5);

    auto is_j = [&](int b) { return b < vs; };
    // Lanes.  Bits vs .. k-1 of the block-local index walk along a contiguous run, so on each side
    // they must be lane bits (up to 6) for a wave's access to be contiguous.  The remaining lane
    // bits are picked among the run selectors (bits >= k), freely and separately on the two sides:
    // on the source side prefer bits that are lanes at the destination anyway (no stage needed),
    // never position-bit sources if avoidable; on the destination side prefer the images of the
    // source lanes, never images of the position bits if avoidable.
    std::vector<bool> src_lane(n, false), dst_lane(n, false);
    const int mand = std::min(g.k, vs + tb) - vs;
    for (int b = vs; b < vs + mand; ++b) src_lane[b] = dst_lane[b] = true;
    {
        int need = tb - mand;
        for (int pass = 0; pass < 3 && need > 0; ++pass)
            for (int sbit = vs + mand; sbit < n && need > 0; ++sbit) {
                if (src_lane[sbit]) continue;
                const int t = pi[sbit];
                const bool to_mand = dst_lane[t], to_j = is_j(t);
                if ((pass == 0 && to_mand) || (pass == 1 && !to_j && !to_mand) || pass == 2) { src_lane[sbit] = true; --need; }
            }
        need = tb - mand;
        for (int pass = 0; pass < 3 && need > 0; ++pass)
            for (int t = vs + mand; t < n && need > 0; ++t) {
                if (dst_lane[t]) continue;
                const int sbit = pinv[t];
                if ((pass == 0 && src_lane[sbit]) || (pass == 1 && !is_j(sbit)) || pass == 2) { dst_lane[t] = true; --need; }
            }
    }
    auto is_lane_src = [&](int b) { return (bool)src_lane[b]; };
    auto is_lane = [&](int b) { return (bool)dst_lane[b]; };          // destination-side role
    // which source bit sits on each kernel position
    std::vector<int> at_j(vs), at_lane, at_i(nvb, -1);
    for (int c = 0; c < vs; ++c) at_j[c] = c;
    for (int b = vs; b < n; ++b)
        if (src_lane[b]) at_lane.push_back(b);
    const std::vector<int> lane_src_bit = at_lane;

    bool j_identity = true, j_leaves = true;
    for (int c = 0; c < vs; ++c) {
        j_identity &= pi[c] == c;
        j_leaves &= !is_j(pi[c]);
    }
    if (!j_identity && !j_leaves) return dbg_na(6);      // mixed: some position bits stay, some move
    int tpose = kTposeNone;
    bool jl = false, lj = false;                     // a position bit goes to a lane / comes from a lane
    if (!j_identity) {
        for (int c = 0; c < vs; ++c) {
            jl |= is_lane(pi[c]);
            lj |= is_lane_src(pinv[c]);
        }
        if (jl && lj) return dbg_na(7);                  // would need transposes on both sides
        tpose = lj ? kTposeAfter : kTposeBefore;
    }
    // assign source iteration bits: the low vs iteration bits are special when transposing
    std::vector<int> src_i;                          // source bits that start as iteration bits
    for (int b = vs; b < n; ++b)
        if (!src_lane[b]) src_i.push_back(b);
    std::vector<bool> used(n, false);
    if (tpose != kTposeNone) {
        // position c of the destination vector must be on iteration bit c right before the
        // transpose that brings it in.  If it starts as an iteration bit, put it there now.
        for (int c = 0; c < vs; ++c) {
            const int s = pinv[c];
            if (!is_lane_src(s)) { at_i[c] = s; used[s] = true; }
        }
    }
    // remaining iteration bits: first those that must go to lanes (they will be traded), then the rest
    std::vector<int> to_lane, stay;
    for (int s : src_i)
        if (!used[s]) (is_lane(pi[s]) ? to_lane : stay).push_back(s);
    {
        std::vector<int> pool = to_lane;
        pool.insert(pool.end(), stay.begin(), stay.end());
        size_t next = 0;
        for (int b = 0; b < nvb; ++b)
            if (at_i[b] < 0) at_i[b] = pool[next++];
        if (next != pool.size()) return fail(LL_ERR_INVALID_ARG, "internal: iteration bit assignment");
    }
    uint32_t stage_mask[5] = {0, 0, 0, 0, 0};
    int stages = 0;
    if (tpose == kTposeBefore)
        for (int c = 0; c < vs; ++c) std::swap(at_j[c], at_i[c]);
    // lanes holding a bit that must leave the lanes
    auto lane_leaving = [&](bool want_j, int want_pos) {
        for (int l = 0; l < tb; ++l) {
            const int s = at_lane[l];
            if (is_lane(pi[s])) continue;
            if (want_j ? (pi[s] == want_pos) : !is_j(pi[s])) return l;
        }
        return -1;
    };
    for (int b = 0; b < nvb; ++b) {
        const int s = at_i[b];
        int l = -1;
        if (tpose == kTposeAfter && b < vs) {
            if (pi[s] == b) continue;                 // already the bit that becomes position b
            l = lane_leaving(true, b);                // the lane that holds destination position b
            if (l < 0 || !is_lane(pi[s])) return dbg_na(8);
        } else {
            if (!is_lane(pi[s])) continue;            // stays a register bit
            l = lane_leaving(false, 0);
            if (l < 0) return dbg_na(9);
        }
        std::swap(at_i[b], at_lane[l]);
        stage_mask[b] = 1u << l;
        ++stages;
    }
    if (tpose == kTposeAfter)
        for (int c = 0; c < vs; ++c) std::swap(at_j[c], at_i[c]);
    // final roles
    for (int c = 0; c < vs; ++c)
        if (pi[at_j[c]] != c) return dbg_na(10);
    for (int l = 0; l < tb; ++l)
        if (!is_lane(pi[at_lane[l]])) return dbg_na(11);
    for (int b = 0; b < nvb; ++b)
        if (is_lane(pi[at_i[b]]) || is_j(pi[at_i[b]])) return dbg_na(12);

    // ---- tables
    VecArgs &a = plan->vec;
    std::memset(&a, 0, sizeof(a));
    a.d = d; a.group_bits = g.g; a.coset_bits = (int)g.comp.size(); a.thread_bits = tb;
    for (size_t c = 0; c < g.comp.size(); ++c) {
        a.coset_src[c] = (uint32_t)g.comp[c];
        a.coset_dst[c] = (uint32_t)f2::apply(g.pext, g.comp[c]);
    }
    // source side: lane l is block-local bit vs + l; iteration bit b is the bit it started on.
    // (at_i was permuted by the steps above, so rebuild the initial assignment.)
    std::vector<int> init_i(nvb);
    {
        // undo: replay from scratch to recover the initial assignment
        std::vector<int> cur_i = at_i, cur_lane = at_lane, cur_j = at_j;
        if (tpose == kTposeAfter) for (int c = 0; c < vs; ++c) std::swap(cur_j[c], cur_i[c]);
        for (int b = nvb - 1; b >= 0; --b)
            if (stage_mask[b]) std::swap(cur_i[b], cur_lane[__builtin_ctz(stage_mask[b])]);
        if (tpose == kTposeBefore) for (int c = 0; c < vs; ++c) std::swap(cur_j[c], cur_i[c]);
        init_i = cur_i;
    }
    mat src_iter_cols(nvb), dst_iter_cols(nvb);
    for (int b = 0; b < nvb; ++b) {
        src_iter_cols[b] = g.us[init_i[b]];
        dst_iter_cols[b] = g.ud[pi[at_i[b]]];
    }
    for (int l = 0; l < tb; ++l) {
        a.lane_src[l] = (uint32_t)g.us[lane_src_bit[l]];
        a.lane_dst[l] = (uint32_t)g.ud[pi[at_lane[l]]];
    }
    for (int i = 0; i < (1 << nvb); ++i) {
        a.iter_src[i] = (uint32_t)xor_bits(src_iter_cols, (unsigned)i);
        a.iter_dst[i] = (uint32_t)xor_bits(dst_iter_cols, (unsigned)i);
    }
    for (int b = 0; b < 5; ++b) a.stage_mask[b] = stage_mask[b];
    const int xchg = stages ? kXchgShuffle : kXchgNone;
    if (ll_status st = check_vec_tables(a, g.pext, vs, w, nvb, tpose, xchg, 0); st != LL_OK) return st;

    plan->vec_nvec_bits = nvb; plan->vec_tpose = tpose; plan->vec_xchg = xchg;
    ll_plan_desc &desc = plan->desc;
    desc.strategy = stages ? LL_STRATEGY_WAVE_SHUFFLE : LL_STRATEGY_REG_PERMUTE;
    desc.global_vec_bytes = 16;
    desc.lds_write_bytes = desc.lds_read_bytes = desc.lds_bytes = 0;
    desc.threads = 64;
    desc.vectors_per_thread = 1 << nvb;
    desc.block_bits = n; desc.group_bits = g.g; desc.segment_bits = g.k;
    desc.shuffle_rounds = stages;
    desc.register_transpose = tpose;
    *applied = true;
    return LL_OK;
}

// ---------------------------------------------------------------------------------------------
// LDS staging with 128-bit accesses on both sides.  A thread loads the 2^vs source vectors that
// together hold 2^vs whole destination vectors (their addresses differ by Q^-1 of the
// destination position bits), transposes them in registers, writes destination vectors to
// XOR-swizzled LDS with ds_write_b128 and reads the destination vectors it stores with
// ds_read_b128.  Needs: source position bits map to zero destination position bits and vice
// versa (then the two sets of position bits are independent and the in-register step is a pure
// transpose).  Works for any linear Q with that property, not only bit permutations.
// ---------------------------------------------------------------------------------------------
ll_status plan_lds_vec(const mat &p, int d, int w, ll_plan *plan, bool *applied)
{
    *applied = false;
    if (w != 2 && w != 4 && w != 8) return LL_OK;
    const LdsModel hw;
    const int vs = ilog2u(16u / (unsigned)w);
    const unsigned max_block = opt_bytes(plan->opts.vec_block_bytes, 8192u);
    int tb = ilog2u(opt_bytes(plan->opts.vec_threads, 64u));
    if (tb < 6 || tb > 8) tb = 6;
    BlockGeom g;
    if (build_blocks(p, d, w, 2 * vs + tb, max_block, max_block, &g) != LL_OK) return LL_OK;
    const int n = g.n, nvb = n - vs - tb;
    if (nvb > 4 || nvb < vs) return LL_OK;
    const vec vmask = (vec(1) << vs) - 1;
    for (int c = 0; c < vs; ++c)
        if ((g.q[c] & vmask) || (g.qinv[c] & vmask)) return LL_OK;
    const vec low_mask = (vec(1) << g.k) - 1;
    for (vec h : g.comp)
        if (f2::apply(g.pext, h) & vmask) return LL_OK;

    // Source-side directions (block-local, vector granular: low vs bits zero):
    //   T_c = Q^-1 e_c for the low iteration bits; Z = a basis of {low bits zero} n Q^-1{low bits zero}
    //   for lanes, waves and the high iteration bits, taking plain unit vectors first so that
    //   consecutive lanes read consecutive vectors.
    mat tdir;
    for (int c = 0; c < vs; ++c) tdir.push_back(g.qinv[c]);
    mat h_src, h_pre;
    for (int b = vs; b < n; ++b) {
        h_src.push_back(vec(1) << b);
        h_pre.push_back(g.qinv[b]);
    }
    const mat zspace = f2::intersect(h_src, h_pre, n);
    if ((int)zspace.size() != n - 2 * vs) return LL_OK;
    // Lanes first: take the directions of Z in the order of the source offsets they stand for, so
    // that the 64 vectors of a wave-wide load lie in as few 128-byte lines as Z allows.
    if (zspace.size() > 12) return LL_OK;
    std::vector<std::pair<vec, vec>> by_offset;       // (source offset, direction)
    for (unsigned sel = 1; sel < (1u << zspace.size()); ++sel) {
        const vec x = xor_bits(zspace, sel);
        by_offset.push_back({f2::apply(g.us, x), x});
    }
    std::sort(by_offset.begin(), by_offset.end());
    mat zcand;
    for (const auto &e : by_offset) zcand.push_back(e.second);
    const mat z = f2::extend({}, zcand);
    if ((int)z.size() != n - 2 * vs) return LL_OK;
    {
        mat all;
        for (int c = 0; c < vs; ++c) all.push_back(vec(1) << c);
        all.insert(all.end(), tdir.begin(), tdir.end());
        all.insert(all.end(), z.begin(), z.end());
        if (f2::rank(all) != n) return LL_OK;
    }
    // iteration index: low vs bits -> T, then high bits -> z[tb..]; threads -> z[0..tb)
    mat src_iter_cols, qz_iter_cols, aj_cols;
    for (int c = 0; c < vs; ++c) src_iter_cols.push_back(tdir[c]);
    for (int b = vs; b < nvb; ++b) src_iter_cols.push_back(z[tb + b - vs]);
    // after the transpose the low vs iteration bits are the old position bits (images Q e_j), the
    // high ones unchanged (images Q z)
    mat dstv_iter_cols;
    for (int c = 0; c < vs; ++c) dstv_iter_cols.push_back(g.q[c]);
    for (int b = vs; b < nvb; ++b) dstv_iter_cols.push_back(f2::apply(g.q, z[tb + b - vs]));
    mat wr_lane_cols;
    for (int b = 0; b < tb; ++b) wr_lane_cols.push_back(f2::apply(g.q, z[b]));

    // LDS layout in destination-local coordinates, whole vectors
    mat wr_lanes(wr_lane_cols.begin(), wr_lane_cols.begin() + 6), rd_lanes;
    for (int b = 0; b < 6; ++b) rd_lanes.push_back(vec(1) << (vs + b));
    int wfw = 1, wfr = 1;
    const mat m = synthesize_swizzle(n, vs, w, wr_lanes, rd_lanes, hw, &wfw, &wfr);
    mat sw;
    if (!f2::invert(m, n, &sw)) return fail(LL_ERR_INVALID_ARG, "internal: swizzle not invertible");

    VecArgs &a = plan->vec;
    std::memset(&a, 0, sizeof(a));
    a.d = d; a.group_bits = g.g; a.coset_bits = (int)g.comp.size(); a.thread_bits = tb;
    for (size_t c = 0; c < g.comp.size(); ++c) {
        const vec ph = f2::apply(g.pext, g.comp[c]);
        a.coset_src[c] = (uint32_t)g.comp[c];
        a.coset_dst[c] = (uint32_t)(ph & ~low_mask);
        a.coset_lds_rd[c] = (uint32_t)(f2::apply(sw, ph & low_mask) * (vec)w);
    }
    auto to_offset = [&](const mat &basis, vec local) { return f2::apply(basis, local); };
    for (int b = 0; b < tb; ++b) {
        a.lane_src[b] = (uint32_t)to_offset(g.us, z[b]);
        a.lane_dst[b] = (uint32_t)g.ud[vs + b];
        a.lds_wr_lane[b] = (uint32_t)(f2::apply(sw, wr_lane_cols[b]) * (vec)w);
        a.lds_rd_lane[b] = (uint32_t)(sw[vs + b] * (vec)w);
    }
    for (int i = 0; i < (1 << nvb); ++i) {
        a.iter_src[i] = (uint32_t)to_offset(g.us, xor_bits(src_iter_cols, (unsigned)i));
        a.lds_wr_iter[i] = (uint32_t)(f2::apply(sw, xor_bits(dstv_iter_cols, (unsigned)i)) * (vec)w);
        vec dl = 0, rl = 0;
        for (int b = 0; b < nvb; ++b)
            if ((i >> b) & 1) { dl ^= g.ud[vs + tb + b]; rl ^= sw[vs + tb + b]; }
        a.iter_dst[i] = (uint32_t)dl;
        a.lds_rd_iter[i] = (uint32_t)(rl * (vec)w);
    }
    // A wave-wide load that is spread over more than 8 lines costs more than the narrower LDS
    // accesses of the element-wide kernel, whose global accesses are always contiguous (measured:
    // 16 lines 5.6 TB/s, 32 lines 3.9-5.2, element-wide kernel 6.2).
    if (wave_access_lines(a.lane_src, w) > 8 || wave_access_lines(a.lane_dst, w) > 8) return LL_OK;
    const int lds_bytes = (1 << n) * w;
    if (ll_status st = check_vec_tables(a, g.pext, vs, w, nvb, kTposeBefore, kXchgLds, lds_bytes); st != LL_OK) return st;

    plan->vec_nvec_bits = nvb; plan->vec_tpose = kTposeBefore; plan->vec_xchg = kXchgLds;
    ll_plan_desc &desc = plan->desc;
    desc.strategy = LL_STRATEGY_LDS_VEC;
    desc.global_vec_bytes = 16;
    desc.lds_write_bytes = desc.lds_read_bytes = 16;
    desc.lds_bytes = lds_bytes;
    desc.threads = 1 << tb;
    desc.vectors_per_thread = 1 << nvb;
    desc.block_bits = n; desc.group_bits = g.g; desc.segment_bits = g.k;
    desc.shuffle_rounds = 0;
    desc.register_transpose = kTposeBefore;
    desc.lds_vec_bits = vs;
    desc.lds_banks = hw.rd_banks[2];
    desc.lds_banks_write = hw.wr_banks[2];
    desc.lds_phase_lanes_write = 1 << hw.wr_phase_dim[2];
    desc.lds_phase_lanes_read = 1 << hw.rd_phase_dim[2];
    desc.predicted_wavefronts_write = wfw;
    desc.predicted_wavefronts_read = wfr;
    desc.lds_write_reg_bits = desc.lds_read_reg_bits = vs + nvb;
    // access layouts (destination-local space): vector position bits, iteration bits, lanes, waves
    int pos = 0;
    for (int c = 0; c < vs; ++c) { desc.lds_write[pos] = vec(1) << c; desc.lds_read[pos] = vec(1) << c; ++pos; }
    for (int b = 0; b < nvb; ++b) { desc.lds_write[pos] = dstv_iter_cols[b]; desc.lds_read[pos] = vec(1) << (vs + tb + b); ++pos; }
    for (int b = 0; b < tb; ++b) { desc.lds_write[pos] = wr_lane_cols[b]; desc.lds_read[pos] = vec(1) << (vs + b); ++pos; }
    for (int j = 0; j < n; ++j) desc.lds_mem[j] = m[j];
    *applied = true;
    return LL_OK;
}

}  // namespace ll

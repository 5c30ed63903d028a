// Conversion planner (paper Sec. 5.4): B^-1 o A, classification, block decomposition for
// coalesced 16-byte global access, and the swizzled LDS layout.
#include "plan.hpp"

#include <algorithm>
#include <cstdlib>
#include <cstring>

using f2::mat;
using f2::vec;

namespace ll {

static int ilog2(unsigned x) { return 31 - __builtin_clz(x); }

int lds_alloc_for(unsigned block_bytes, unsigned budget, int lds_bytes)
{
    const unsigned per_cu = budget / block_bytes > 1 ? budget / block_bytes : 1;
    unsigned alloc = (160u * 1024u / per_cu) & ~1023u;
    if (alloc > 64u * 1024u) alloc = 64u * 1024u;
    if (alloc < (unsigned)lds_bytes) alloc = (unsigned)lds_bytes;
    return (int)alloc;
}

int xcd_chunk_bits_for(long long target_bytes, long long block_bytes)
{
    if (block_bytes <= 0 || block_bytes >= target_bytes) return -1;
    return 63 - __builtin_clzll((unsigned long long)(target_bytes / block_bytes));
}

int wave_access_lines(const uint32_t *lane_table, int w)
{
    const int line_shift = ilog2(128u / (unsigned)w);       // element-offset bits inside one 128-byte line
    mat high;
    for (int b = 0; b < 6; ++b) high.push_back((vec)(lane_table[b] >> line_shift));
    return 1 << f2::rank(high);
}

int lds_width_class(int access_bytes) { return access_bytes <= 4 ? 0 : (access_bytes == 8 ? 1 : 2); }

static vec lane_image(const mat &lanes, uint32_t lane_vec)
{
    vec r = 0;
    for (size_t b = 0; b < lanes.size(); ++b)
        if ((lane_vec >> b) & 1) r ^= lanes[b];
    return r;
}

static mat concat(const mat &a, const mat &b)
{
    mat r = a;
    r.insert(r.end(), b.begin(), b.end());
    return r;
}

// Wavefronts per phase of an access whose lanes of one phase span `phase_space`:
// lanes collide when their offsets agree on the bank bits but differ above them.
static int predict_wavefronts(const mat &m, int n, int low_bits, int row_bits, const mat &phase_space)
{
    mat low(m.begin(), m.begin() + low_bits);
    mat low_seg = low;
    low_seg.insert(low_seg.end(), m.begin() + row_bits, m.end());
    int k = (int)f2::intersect(low_seg, phase_space, n).size();
    int k0 = (int)f2::intersect(low, phase_space, n).size();
    return 1 << (k - k0);
}

// Paper Sec. 5.4 "Optimal Swizzling" (and the appendix of the same name), stated for subspaces so
// that layouts whose columns are not unit vectors are covered (the appendix's abstract lemma):
//   U, W   the spans of (vector elements + images of the lanes served in one phase) for the
//          write and the read access;
//   I = U n W,  U = I + E,  W = I + F,  G = {e_i ^ f_i},  C = a complement of U + W;
//   the segment (row-index) columns come from G u C, which meets U u W only in 0;
//   the bank columns complete the basis.
// The hardware constants (banks, lanes per phase) come from the LdsModel instead of the
// 32-bank / 32-lane figures of the paper.  On gfx950 a wide write phase covers a 128-byte row and
// a wide read phase a 256-byte row, so the offset bits between the two row sizes are row-index
// bits for one side and bank bits for the other: they are filled with vectors that keep the
// narrower-row side conflict free (always possible: a subspace meeting U only in 0 extends to a
// complement of U).
mat synthesize_swizzle(int n, int v, int w, const mat &wr_lanes, const mat &rd_lanes, const LdsModel &hw,
                       int *wf_write, int *wf_read)
{
    const int access = (1 << v) * w;
    const int cls = lds_width_class(access);
    const int row_w = std::min(n, ilog2((unsigned)(hw.wr_banks[cls] * 4 / w)));   // offset bits that pick (bank, byte)
    const int row_r = std::min(n, ilog2((unsigned)(hw.rd_banks[cls] * 4 / w)));
    const int row_lo = std::min(row_w, row_r), row_hi = std::max(row_w, row_r);
    const int low_bits = std::min(row_lo, std::max(v, ilog2((unsigned)std::max(1, 4 / w))));   // bits inside one access / word

    mat vecs;
    for (int b = 0; b < v; ++b) vecs.push_back(vec(1) << b);
    mat wl, rl;     // images of the lanes served in one phase
    for (int k = 0; k < hw.wr_phase_dim[cls]; ++k) wl.push_back(lane_image(wr_lanes, hw.wr_phase_basis[cls][k]));
    for (int k = 0; k < hw.rd_phase_dim[cls]; ++k) rl.push_back(lane_image(rd_lanes, hw.rd_phase_basis[cls][k]));
    // "low" columns: the offsets inside one access or one 4-byte word, whichever is larger.  They
    // start with the vector; for sub-word accesses they are completed with directions shared by
    // the write and read lanes if there are any (lanes that differ only there share a word on
    // both sides), else with write-lane directions.
    mat low = vecs;
    if ((int)low.size() < low_bits) {
        const mat shared = f2::intersect(f2::extend({}, concat(vecs, wl)), f2::extend({}, concat(vecs, rl)), n);
        for (vec x : f2::extend(vecs, concat(concat(shared, wl), f2::identity(n))))
            if ((int)low.size() < low_bits) low.push_back(x);
    }
    const mat U = f2::extend({}, concat(low, wl)), W = f2::extend({}, concat(low, rl));
    const mat I = f2::intersect(U, W, n);
    const mat E = f2::extend(I, U), F = f2::extend(I, W);
    mat G;
    for (size_t i = 0; i < std::min(E.size(), F.size()); ++i) G.push_back(E[i] ^ F[i]);
    const mat C = f2::complement(concat(U, W), n);

    // columns above the larger row: row index for both sides
    const int need = n - row_hi;
    mat seg;
    for (vec g : concat(G, C))
        if ((int)seg.size() < need) seg.push_back(g);
    if ((int)seg.size() < need) {
        // conflicts are unavoidable: fill up with vectors of the write space, then anything
        for (vec x : f2::extend(concat(low, seg), concat(concat(U, W), f2::identity(n))))
            if ((int)seg.size() < need) seg.push_back(x);
    }
    // columns between the two row sizes: row index for the side with the smaller row (call its
    // phase space T), bank bits for the other side
    const mat &T = (row_w <= row_r) ? U : W;
    const mat &other = (row_w <= row_r) ? W : U;
    mat mid;
    {
        f2::Basis taken;                 // low + seg + mid + T: a candidate must stay outside
        for (vec x : concat(concat(low, seg), T)) taken.add(x);
        for (vec x : concat(other, f2::identity(n))) {
            if ((int)mid.size() >= row_hi - row_lo) break;
            if (taken.add(x)) mid.push_back(x);
        }
        for (vec x : f2::extend(concat(concat(low, seg), mid), f2::identity(n)))      // unavoidable conflicts
            if ((int)mid.size() < row_hi - row_lo) mid.push_back(x);
    }
    // bank columns: complete to a basis, preferring the write lanes so that a write instruction of
    // consecutive lanes stays contiguous
    mat fixed = concat(concat(low, seg), mid);
    mat bank = f2::extend(fixed, concat(concat(U, W), f2::identity(n)));
    // Keep vectors aligned: an index whose low v bits are zero must get an offset whose low v bits
    // are zero, i.e. every non-vector column must have zero low v bits.  Clearing them adds vector
    // columns to the others, which changes neither the spans used above nor invertibility.
    const vec vmask = (vec(1) << v) - 1;
    for (vec &x : bank) x &= ~vmask;
    for (vec &x : mid) x &= ~vmask;
    for (vec &x : seg) x &= ~vmask;
    for (size_t i = (size_t)v; i < low.size(); ++i) low[i] &= ~vmask;
    mat m = concat(concat(concat(low, bank), mid), seg);

    if (wf_write) *wf_write = predict_wavefronts(m, n, low_bits, row_w, U);
    if (wf_read) *wf_read = predict_wavefronts(m, n, low_bits, row_r, W);
    return m;
}

// ---------------------------------------------------------------------------------------------

static bool same_inputs(const ll_layout *a, const ll_layout *b)
{
    if (a->n_in != b->n_in) return false;
    for (int i = 0; i < a->n_in; ++i)
        if (a->in_dims[i].label != b->in_dims[i].label || a->in_dims[i].nbits != b->in_dims[i].nbits) return false;
    return true;
}

static int classify(const mat &p, int d, int reg_bits, int wave_first)
{
    bool ident = true;
    for (int k = 0; k < d; ++k) ident &= (p[k] == (vec(1) << k));
    if (ident) return LL_KIND_NOOP;
    const vec reg_mask = (vec(1) << reg_bits) - 1;
    const vec wave_mask = ((vec(1) << d) - 1) & ~((vec(1) << wave_first) - 1);
    bool reg_only = true, intra_wave = true;
    for (int k = 0; k < d; ++k) {
        if (k < reg_bits) {
            if (p[k] & ~reg_mask) reg_only = false;
        } else if (p[k] != (vec(1) << k)) {
            reg_only = false;
        }
        if (k >= wave_first) {
            if (p[k] != (vec(1) << k)) intra_wave = false;
        } else if (p[k] & wave_mask) {
            intra_wave = false;
        }
    }
    if (reg_only) return LL_KIND_REG_ONLY;
    if (intra_wave) return LL_KIND_INTRA_WAVE;
    return LL_KIND_LDS;
}

// Work decomposition shared by the staged kernels.  Tiles smaller than `pref_bytes` are bundled
// (the conversion is extended by the identity on the bundling bits).  A block is a coset of
// U_k = span(e_0..e_{k-1}) + P^-1 span(e_0..e_{k-1}) for the largest k with |U_k| * w <= max_bytes:
// on BOTH sides a block consists of whole runs of 2^k contiguous elements.  `min_bits` is the
// smallest block the kernel can take (one unit of work per thread).
ll_status build_blocks(const mat &p, int d, int w, int min_bits, unsigned max_bytes, unsigned pref_bytes, BlockGeom *out)
{
    BlockGeom &b = *out;
    const int vs = ilog2(16u / (unsigned)w);
    const int n_max = std::max(min_bits, ilog2(max_bytes / (unsigned)w));
    const int n_pref = std::max(min_bits, ilog2(pref_bytes / (unsigned)w));
    const int g = std::max(0, n_pref - d);
    const int D = d + g;
    if (D + ilog2((unsigned)w) > 31) return fail(LL_ERR_UNSUPPORTED, "tile of 2^%d elements of %d bytes is too large", d, w);
    mat pext = p;
    for (int k = d; k < D; ++k) pext.push_back(vec(1) << k);
    mat pinv;
    if (!f2::invert(pext, D, &pinv)) return fail(LL_ERR_INVALID_ARG, "internal: conversion matrix is singular");
    auto block_space = [&](int k) {
        mat gens;
        for (int j = 0; j < k; ++j) gens.push_back(vec(1) << j);
        for (int j = 0; j < k; ++j) gens.push_back(pinv[j]);
        return f2::extend({}, gens);
    };
    int k = vs;
    while (k < D && (int)block_space(k + 1).size() <= n_max) ++k;
    // HBM is fetched in 128-byte lines: runs shorter than that waste half of every line (measured:
    // a 128 x 128 transpose of 1-byte elements runs at 4.1 TB/s with 64-byte runs and at 6.0 TB/s
    // with 128-byte runs).  Allow a block of twice the limit when that buys runs of a full line.
    while (k < D && ((unsigned)w << k) < 128u && (int)block_space(k + 1).size() <= n_max + 1) ++k;
    mat U = block_space(k);
    for (int j = k; j < D && (int)U.size() < min_bits; ++j) U = f2::extend({}, concat(U, {vec(1) << j}));
    const int n = (int)U.size();
    if (n < min_bits) return fail(LL_ERR_UNSUPPORTED, "internal: block smaller than the kernel's unit of work");
    const vec low_mask = (vec(1) << k) - 1;
    // source-local basis: the k contiguous bits, then the remaining directions of U with their
    // low k bits cleared (they select the run)
    mat us;
    for (int j = 0; j < k; ++j) us.push_back(vec(1) << j);
    {
        mat cand;
        for (vec x : U) cand.push_back(x & ~low_mask);
        for (vec x : f2::extend(us, cand)) us.push_back(x);
    }
    // destination-local basis of P(U)
    mat ud;
    for (int j = 0; j < k; ++j) ud.push_back(vec(1) << j);
    {
        mat cand;
        for (vec x : us) cand.push_back(f2::apply(pext, x) & ~low_mask);
        for (vec x : f2::extend(ud, cand)) ud.push_back(x);
    }
    if ((int)us.size() != n || (int)ud.size() != n) return fail(LL_ERR_INVALID_ARG, "internal: block basis mismatch");
    // Q = Ud^-1 P Us : block-local source index -> block-local destination index
    f2::Basis udb;
    for (int j = 0; j < n; ++j) udb.add(ud[j], vec(1) << j);
    mat q(n), qinv;
    for (int j = 0; j < n; ++j) {
        vec tag = 0;
        if (udb.reduce(f2::apply(pext, us[j]), &tag) != 0) return fail(LL_ERR_INVALID_ARG, "internal: block not closed");
        q[j] = tag;
    }
    if (!f2::invert(q, n, &qinv)) return fail(LL_ERR_INVALID_ARG, "internal: block map singular");
    // cosets of U: the blocks of one tile group, enumerated by unit vectors outside U
    const mat comp = f2::complement(U, D);
    if ((int)comp.size() > kMaxCosetBits) return fail(LL_ERR_UNSUPPORTED, "internal: too many blocks per tile");
    b.d = d; b.g = g; b.D = D; b.k = k; b.n = n; b.vs = vs; b.w = w;
    b.pext = pext; b.us = us; b.ud = ud; b.q = q; b.qinv = qinv; b.comp = comp;
    return LL_OK;
}

// Host-side walk through blocks of a finished plan, exactly as the kernel indexes them: every
// global offset (16-byte aligned) and LDS address must be in range, the LDS writes must tile the
// block without overlap, and every element read back must be stored where the conversion sends
// it.  Block 0, the block of every single block-index bit and the block of all bits are walked;
// the offsets of the others are XOR combinations of these.  Guards the GPU against a planner
// mistake.
static ll_status check_lds_elem_block(const LdsElemArgs &a, const mat &pext, int n, int vs, int v, int w, int nvec,
                                       uint32_t cs, uint32_t cd, uint32_t cr);

static ll_status check_lds_elem_tables(const LdsElemArgs &a, const mat &pext, int n, int vs, int v, int w, int nvec)
{
    ll_status st = check_lds_elem_block(a, pext, n, vs, v, w, nvec, 0, 0, 0);
    uint32_t cs = 0, cd = 0, cr = 0;
    for (int c = 0; c < a.coset_bits && st == LL_OK; ++c) {
        st = check_lds_elem_block(a, pext, n, vs, v, w, nvec, a.coset_src[c], a.coset_dst[c], a.coset_lds_rd[c]);
        cs ^= a.coset_src[c];
        cd ^= a.coset_dst[c];
        cr ^= a.coset_lds_rd[c];
    }
    if (st == LL_OK && a.coset_bits > 1) st = check_lds_elem_block(a, pext, n, vs, v, w, nvec, cs, cd, cr);
    return st;
}

static ll_status check_lds_elem_block(const LdsElemArgs &a, const mat &pext, int n, int vs, int v, int w, int nvec,
                                       uint32_t cs, uint32_t cd, uint32_t cr)
{
    const int threads = 1 << a.thread_bits;
    const int nsub = 1 << (vs - v);
    const int run = 1 << v;                       // elements per LDS access
    const uint32_t block_bytes = (uint32_t)((1u << n) * (unsigned)w);
    const uint64_t group_elems = 1ull << (a.d + a.group_bits);
    std::vector<int64_t> held(block_bytes / w, -1);   // LDS element slot -> source element offset
    auto lane_part = [&](const uint32_t *tab, int tid) {
        uint32_t x = 0;
        for (int b = 0; b < a.thread_bits; ++b)
            if ((tid >> b) & 1) x ^= tab[b];
        return x;
    };
    for (int tid = 0; tid < threads; ++tid) {
        for (int i = 0; i < nvec; ++i) {
            const uint32_t off = cs ^ lane_part(a.lane_src, tid) ^ a.iter_src[i];
            if (off >= group_elems || (off & ((1u << vs) - 1))) return fail(LL_ERR_INVALID_ARG, "internal: bad source offset in plan");
            for (int s = 0; s < nsub; ++s) {
                const uint32_t addr = lane_part(a.lds_wr_lane, tid) ^ a.lds_wr_iter[i] ^ a.lds_wr_sub[s];
                if (addr >= block_bytes || addr % (uint32_t)(run * w)) return fail(LL_ERR_INVALID_ARG, "internal: bad LDS write address in plan");
                for (int e = 0; e < run; ++e) {
                    int64_t &slot = held[addr / w + e];
                    if (slot >= 0) return fail(LL_ERR_INVALID_ARG, "internal: LDS writes overlap in plan");
                    slot = (int64_t)off + s * run + e;
                }
            }
        }
    }
    for (int tid = 0; tid < threads; ++tid) {
        for (int i = 0; i < nvec; ++i) {
            const uint32_t off = cd ^ lane_part(a.lane_dst, tid) ^ a.iter_dst[i];
            if (off >= group_elems || (off & ((1u << vs) - 1))) return fail(LL_ERR_INVALID_ARG, "internal: bad destination offset in plan");
            for (int s = 0; s < nsub; ++s) {
                const uint32_t addr = cr ^ lane_part(a.lds_rd_lane, tid) ^ a.lds_rd_iter[i] ^ a.lds_rd_sub[s];
                if (addr >= block_bytes || addr % (uint32_t)(run * w)) return fail(LL_ERR_INVALID_ARG, "internal: bad LDS read address in plan");
                for (int e = 0; e < run; ++e) {
                    const int64_t from = held[addr / w + e];
                    if (from < 0 || f2::apply(pext, (vec)from) != (vec)off + s * run + e)
                        return fail(LL_ERR_INVALID_ARG, "internal: plan does not realise the conversion");
                }
            }
        }
    }
    return LL_OK;
}

// Fill the LDS-staged plan.  P acts on d bits; elements are w bytes.
static ll_status plan_lds_elem(const mat &p, int d, int w, ll_plan *plan)
{
    const LdsModel hw;
    ll_plan_desc &desc = plan->desc;
    LdsElemArgs &a = plan->lds_elem;
    const int vs = ilog2(16u / (unsigned)w);          // elements per 16-byte vector (log2)
    const ll_options &opt = plan->opts;
    int tb = 8;                                       // 256 threads
    if (opt.elem_threads_log2 != LL_AUTO) tb = std::min(10, std::max(6, (int)opt.elem_threads_log2));
    // Largest staged block, and the size small tiles are bundled to (bytes, powers of two).
    // Small blocks measured best on MI355X (more, shorter-lived workgroups keep about 32-64 KiB in
    // flight per CU, which is where a plain copy also peaks).
    // 4- and 8-byte elements: 4 KiB, which goes to one wave (below).  Measured against the 8 KiB blocks of four (two)
    // waves, with their longer runs, TB/s: bit permutations of 4-byte elements on tiles of 2^12 / 2^14 / 2^18 / 2^20 /
    // 2^22 elements 6.32 / 6.46 / 5.93 / 5.95 / 5.93 -> 6.52 / 6.68 / 6.45 / 6.21 / 6.18 (2^17: 6.68 -> 6.59), configs 1
    // and 3 through this kernel 6.41 / 6.42 -> 6.61 / 6.56; 8-byte elements, random XOR maps 2^13 / 2^16 / 2^18 / 2^22
    // 6.55 / 6.30 / 6.18 / 5.48 -> 6.55 / 6.45 / 6.33 / 5.48, bit permutations 2^18 / 2^22 6.39 / 5.18 -> 6.58 / 5.88.
    // 2-byte elements keep 8 KiB: their 4 KiB blocks have runs of 64 bytes under XOR maps, and permutations of large
    // tiles lose up to 11 % with the shorter runs.
    const unsigned max_block = opt_bytes(opt.block_bytes, w >= 4 ? 4096u : 8192u);
    const unsigned pref_block = opt_bytes(opt.pref_bytes, 8192u);

    BlockGeom geom;
    const int min_bits = vs + std::max(tb, 8);        // a wave-sized workgroup takes at least four vectors per lane
    const bool tb_auto = opt.elem_threads_log2 == LL_AUTO;
    if (ll_status st = build_blocks(p, d, w, min_bits, max_block, pref_block, &geom); st != LL_OK) return st;
    if (geom.n == min_bits && (w == 1 || (d >= 17 && w == 2)) && opt.block_bytes == LL_AUTO) {
        // One vector per thread and a tile cut into many such blocks: the runs are as short as the
        // limit allows (4-byte elements: 128 bytes on each side, 32 of them scattered over the tile).
        // Runs grow on both sides at once, so the next size is four times the block.  Measured with
        // interleaved runs of both block sizes (TB/s, 4 KiB against 16 KiB blocks).  Random XOR layouts
        // of 4-byte elements on 1 GiB: tiles of 2^12..2^17 elements 6.1-6.4 against 5.9-6.2, 2^18
        // 6.1 / 6.1, 2^19 5.9 / 6.05, 2^20 5.55 / 6.0, 2^21 5.26 / 6.05, 2^22 4.94 / 5.65, 2^24
        // 4.44 / 5.3-5.5.  Random bit permutations on 256 MiB: 2-byte elements 2^13..2^16 6.2-6.5
        // against 5.8-6.2, 2^17 5.9-6.0 / 6.1-6.2, 2^18 5.3-5.9 / 6.1-6.2, 2^19 5.5-5.9 / 6.0-6.2;
        // 4-byte 2^17 6.1 / 6.25, 2^18 5.8 / 6.3; 8-byte 2^13..2^15 6.5 / 5.8-6.2, 2^17 6.1 / 6.3.
        // Byte elements pay one LDS instruction per byte, and a workgroup that holds only 4 KiB
        // cannot hide that: 2^14..2^20 4.2-5.8 against 6.1-6.5 at every tile size.
        // (The 4- and 8-byte figures above are those of four waves per 4 KiB block in natural block order.  With one
        // wave per block and the XCD-aware order the small block wins for them at every size - random XOR maps of
        // 4-byte elements, 2^17 / 2^18 / 2^20 / 2^22 / 2^24: 6.27 / 6.25 / 6.15 / 5.88 / 5.16 for 16 KiB against
        // 6.41 / 6.38 / 6.40 / 6.13 / 5.41 - so only bytes and 2-byte elements still widen.)
        BlockGeom wider;
        if (build_blocks(p, d, w, min_bits, 2 * max_block, pref_block, &wider) == LL_OK && wider.k > geom.k &&
            ((unsigned)w << wider.n) <= 2 * max_block)
            geom = wider;
    }
    const int g = geom.g, k = geom.k, n = geom.n;
    const mat &pext = geom.pext, &us = geom.us, &ud = geom.ud, &q = geom.q, &qinv = geom.qinv, &comp = geom.comp;
    const int nco = (int)comp.size();
    const vec low_mask = (vec(1) << k) - 1;
    // A 4 KiB block is given to ONE wave (four vectors per lane) instead of four: the wave goes on as
    // soon as its own loads have landed, no workgroup barrier holds the CU slot until the slowest of
    // four waves is ready.  Measured on MI355X, random XOR layouts of 4-byte elements, 1 GiB each way:
    // config 4 6.2-6.4 -> 6.7 TB/s, tiles of 2^12 / 2^14 elements 6.45 -> 6.6; 8-byte elements (blocks of
    // 2^9) equal within 1 %.  Larger blocks lose that way (16 vectors per lane and two waves per CU
    // leave the LDS latency exposed: 4.0-5.3 TB/s), so they keep 256 threads.
    if (tb_auto && ((unsigned)w << n) == 4096u) tb = 6;
    // 8 KiB blocks of 8-byte elements (two LDS instructions per vector and side): two waves with four vectors per lane
    // measured 6.36-6.5 against 6.1-6.3 TB/s for four waves with two; 2- and 4-byte elements tie or lose that way
    if (tb_auto && w == 8 && ((unsigned)w << n) == 8192u) tb = 7;
    if (tb == 6 && ((unsigned)w << n) != 4096u) tb = 8;               // the one-wave kernel exists for 4 KiB blocks only
    if (tb == 7 && ((unsigned)w << n) != 8192u) tb = 8;               // the two-wave kernel for 8 KiB blocks only
    const int nvec_bits = n - vs - tb;
    // what the launcher instantiates: up to 8 vectors per thread with 256 threads, up to 4 with more
    if (nvec_bits < 0 || (1 << nvec_bits) > (tb == 8 ? 8 : 4))
        return fail(LL_ERR_UNSUPPORTED, "staged block of %d bytes needs %d vectors per thread", (1 << n) * w, 1 << nvec_bits);

    // common contiguous run: Q e_b = e_b for b < v
    // (the low v bits of the destination index must be the low v bits of the source index: column
    // b is e_b and no other column touches row b)
    int v = 0;
    while (v < vs && q[v] == (vec(1) << v)) ++v;
    for (int j = 0; j < n; ++j)
        while (v > 0 && j >= v && (q[j] & ((vec(1) << v) - 1))) --v;
    // a block may land shifted by low bits of P h_c (see the block offsets below); the run must
    // survive that shift as a unit
    for (vec h : comp)
        while (v > 0 && (f2::apply(pext, h) & ((vec(1) << v) - 1))) --v;

    // LDS layout
    mat wr_lanes, rd_lanes;
    for (int b = 0; b < 6; ++b) {
        wr_lanes.push_back(vec(1) << (vs + b));
        rd_lanes.push_back(qinv[vs + b]);
    }
    int wfw = 1, wfr = 1;
    const mat m = synthesize_swizzle(n, v, w, wr_lanes, rd_lanes, hw, &wfw, &wfr);
    mat sw;
    if (!f2::invert(m, n, &sw)) return fail(LL_ERR_INVALID_ARG, "internal: swizzle not invertible");
    const mat swq = f2::compose(sw, qinv);    // destination-local index -> LDS element offset

    // ---- kernel tables
    std::memset(&a, 0, sizeof(a));
    a.d = d;
    a.group_bits = g;
    a.coset_bits = nco;
    a.thread_bits = tb;
    // Block c starts at the source offset h_c (unit vectors above the runs) and lands on the coset
    // P h_c + P U.  The destination base keeps only the bits of P h_c above the runs, so that
    // stores stay aligned; the low bits of P h_c become a per-block XOR on the LDS read address
    // (the reader of destination element x fetches the element that belongs at x ^ low(P h_c)).
    for (int c = 0; c < nco; ++c) {
        const vec ph = f2::apply(pext, comp[c]);
        a.coset_src[c] = (uint32_t)comp[c];
        a.coset_dst[c] = (uint32_t)(ph & ~low_mask);
        a.coset_lds_rd[c] = (uint32_t)(f2::apply(swq, ph & low_mask) * (vec)w);
    }
    auto xor_bits = [](const mat &cols, int first, unsigned idx) {
        vec r = 0;
        for (int b = 0; (idx >> b) != 0; ++b)
            if ((idx >> b) & 1) r ^= cols[first + b];
        return r;
    };
    for (int b = 0; b < tb; ++b) {
        a.lane_src[b] = (uint32_t)us[vs + b];
        a.lane_dst[b] = (uint32_t)ud[vs + b];
        a.lds_wr_lane[b] = (uint32_t)(sw[vs + b] * (vec)w);
        a.lds_rd_lane[b] = (uint32_t)(swq[vs + b] * (vec)w);
    }
    for (int i = 0; i < (1 << nvec_bits); ++i) {
        a.iter_src[i] = (uint32_t)xor_bits(us, vs + tb, (unsigned)i);
        a.iter_dst[i] = (uint32_t)xor_bits(ud, vs + tb, (unsigned)i);
        a.lds_wr_iter[i] = (uint32_t)(xor_bits(sw, vs + tb, (unsigned)i) * (vec)w);
        a.lds_rd_iter[i] = (uint32_t)(xor_bits(swq, vs + tb, (unsigned)i) * (vec)w);
    }
    for (int s = 0; s < (1 << (vs - v)); ++s) {
        a.lds_wr_sub[s] = (uint32_t)(xor_bits(sw, v, (unsigned)s) * (vec)w);
        a.lds_rd_sub[s] = (uint32_t)(xor_bits(swq, v, (unsigned)s) * (vec)w);
    }
    plan->nvec = 1 << nvec_bits;

    // ---- description
    desc.strategy = LL_STRATEGY_LDS_ELEM;
    desc.global_vec_bytes = 16;
    desc.lds_write_bytes = desc.lds_read_bytes = (1 << v) * w;
    desc.lds_bytes = (1 << n) * w;
    desc.threads = 1 << tb;
    desc.vectors_per_thread = 1 << nvec_bits;
    desc.block_bits = n;
    desc.group_bits = g;
    desc.segment_bits = k;
    desc.shuffle_rounds = 0;
    desc.lds_vec_bits = v;
    const int cls = lds_width_class((1 << v) * w);
    desc.lds_banks = hw.rd_banks[cls];
    desc.lds_banks_write = hw.wr_banks[cls];
    desc.lds_phase_lanes_write = 1 << hw.wr_phase_dim[cls];
    desc.lds_phase_lanes_read = 1 << hw.rd_phase_dim[cls];
    desc.predicted_wavefronts_write = wfw;
    desc.predicted_wavefronts_read = wfr;
    desc.lds_write_reg_bits = desc.lds_read_reg_bits = vs + nvec_bits;
    // access layouts in the order: element-in-vector bits, iteration bits, 6 lane bits, wave bits
    int pos = 0;
    auto put = [&](int local_bit) {
        desc.lds_write[pos] = vec(1) << local_bit;
        desc.lds_read[pos] = qinv[local_bit];
        ++pos;
    };
    for (int b = 0; b < vs; ++b) put(b);
    for (int b = 0; b < nvec_bits; ++b) put(vs + tb + b);
    for (int b = 0; b < tb; ++b) put(vs + b);
    for (int j = 0; j < n; ++j) desc.lds_mem[j] = m[j];
    return check_lds_elem_tables(a, pext, n, vs, v, w, 1 << nvec_bits);
}

// The shuffle schedule exactly as Sec. 5.4 "Intra-warp Data Exchange" states it, on the layouts'
// own registers and lanes.  Only for distributed layouts (every column a unit vector) whose
// conversion keeps the wave part fixed.
static void paper_shuffle_schedule(const ll_layout *a, const ll_layout *b, int w, ll_plan_desc *desc)
{
    desc->sched_valid = 0;
    const int d = a->d_in;
    for (int k = 0; k < d; ++k)
        if (f2::popcount(a->bases[k]) != 1 || f2::popcount(b->bases[k]) != 1) return;
    if (desc->kind != LL_KIND_REG_ONLY && desc->kind != LL_KIND_INTRA_WAVE) return;
    const int nreg = a->bits_of(LL_IN_REG), lane0 = a->first_bit_of(LL_IN_LANE), wave0 = a->first_bit_of(LL_IN_WAVE);
    auto members = [](const ll_layout *l, int from, int to) {
        mat r(l->bases.begin() + from, l->bases.begin() + to);
        std::sort(r.begin(), r.end());
        return r;
    };
    auto both = [](const mat &x, const mat &y) {
        mat r;
        for (vec v : x)
            if (std::find(y.begin(), y.end(), v) != y.end()) r.push_back(v);
        return r;
    };
    auto minus = [](const mat &x, const mat &y) {
        mat r;
        for (vec v : x)
            if (std::find(y.begin(), y.end(), v) == y.end()) r.push_back(v);
        return r;
    };
    const mat areg = members(a, 0, nreg), breg = members(b, 0, nreg);
    const mat alane = members(a, lane0, wave0), blane = members(b, lane0, wave0);
    mat V = both(areg, breg);
    const size_t vmax = w >= 4 ? 0 : (size_t)ilog2(4u / (unsigned)w);      // 32-bit shuffle payload
    if (V.size() > vmax) V.resize(vmax);
    const mat I = both(alane, blane), E = minus(alane, I), F = minus(blane, I);
    if (E.size() != F.size()) return;                                       // cannot happen without broadcasting
    mat G;
    for (size_t i = 0; i < E.size(); ++i) G.push_back(E[i] ^ F[i]);
    mat fixed = concat(concat(V, I), G);
    fixed.insert(fixed.end(), a->bases.begin() + wave0, a->bases.end());    // waves (and tiles) stay where they are
    const mat R = f2::complement(fixed, a->d_out);
    if (V.size() > 2 || I.size() > 8 || G.size() > 8 || R.size() > LL_MAX_BITS) return;
    desc->sched_nv = (int)V.size(); desc->sched_ni = (int)I.size(); desc->sched_ng = (int)G.size(); desc->sched_nr = (int)R.size();
    std::copy(V.begin(), V.end(), desc->sched_v);
    std::copy(I.begin(), I.end(), desc->sched_i);
    std::copy(G.begin(), G.end(), desc->sched_g);
    std::copy(R.begin(), R.end(), desc->sched_r);
    desc->sched_valid = 1;
}

// Strategy, cheapest exchange first.  The kernel's lanes are not the layout's lanes (only the
// conversion and the image order are observable), so even a conversion that moves data between
// the layout's waves may need no exchange between the KERNEL's lanes once small blocks with the
// right run selectors as lanes are used: the register / shuffle planner is tried for every
// class.  What its structure does not cover is staged through LDS, with 128-bit accesses when
// the in-register transpose applies and element-wide accesses otherwise (always possible).
static ll_status choose_strategy(const mat &p, int d, int elem_bytes, ll_plan *plan)
{
    const int force = plan->opts.strategy;
    bool applied = false;
    // Transposing LDS loads (1- and 2-byte elements): on request only (ll_options.strategy).  They
    // cut the LDS instructions 8-fold, but the instruction makes adjacent lanes take adjacent source
    // elements, which in a transpose are different destination rows: stores of 16-byte pieces at
    // row pitch.  Measured 5.8-6.0 TB/s against 6.3 for byte-wide LDS accesses with contiguous
    // stores on the 128 x 128 transpose of 1-byte elements; the conversion is HBM bound either way.
    if (force == LL_STRATEGY_LDS_TR) {
        if (ll_status st = plan_lds_tr(p, d, elem_bytes, plan, &applied); st != LL_OK) return st;
        if (applied) return LL_OK;
    }
    // Tiles above 128 KiB of 4- and 8-byte elements go to the element-wide LDS kernel straight away: its 4 KiB blocks
    // for one wave hold up at every tile size, while the register / shuffle kernels (4 or 8 vectors per lane, blocks
    // scattered over a large tile) fall off.  Sampled on MI355X, planner's former choice -> LDS kernel, TB/s: transposes
    // of 2^16 .. 2^22-element tiles 5.5-5.8 -> 6.1-6.45 (4-byte, all 13 shapes), 5.4-6.3 -> 5.9-6.5 (8-byte, better in
    // 12 of 15); random bit permutations, five to ten per size on 1 GiB each way, geometric mean: 4-byte 2^15 / 2^16 /
    // 2^17 / 2^18 / 2^20 elements +0.2 / +2.4 / -0.3 / -0.9 / +4.5 %, 8-byte 2^16 / 2^17 / 2^18 / 2^20 / 2^22 +0.8 / -1.2 /
    // -1.5 / -0.5 / +2.4 %: a tie for random permutations, a clear gain for structured ones.  Up to 128 KiB the two
    // are within 1-2 % either way and the register / shuffle path stays.
    const bool large = force == LL_AUTO && elem_bytes >= 4 && ((long long)elem_bytes << d) > 128 * 1024;
    if (!(force >= LL_STRATEGY_LDS_ELEM) && !large) {
        if (ll_status st = plan_wave_shuffle(p, d, elem_bytes, plan, &applied); st != LL_OK) return st;
        if (applied) return LL_OK;
    }
    if (force != LL_STRATEGY_LDS_ELEM && !large) {
        if (ll_status st = plan_lds_vec(p, d, elem_bytes, plan, &applied); st != LL_OK) return st;
        if (applied) return LL_OK;
    }
    return plan_lds_elem(p, d, elem_bytes, plan);
}

// What a launch needs besides the tables: the XCD-aware block order and the LDS allocation that
// caps the workgroups per CU.  Fixed here so that ll_convert does no lookups of its own.
//
// XCD-aware order.  Workgroups are dealt to the 8 XCDs round robin; renumbering blocks so that each
// XCD works through a run of consecutive blocks at a time (blocks that touch neighbouring lines then
// share an L2 and reach memory close in time) measured 1-6 % faster than the natural order with
// 128 KiB per XCD for the one-wave kernels (config 2: 6.02 -> 6.43 TB/s, config 3: 6.59 -> 6.66,
// config 4 with one wave per block: 6.16 -> 6.7).
//
// In-flight cap.  A plain copy on this chip peaks with roughly 32-48 KiB in flight per CU and loses
// bandwidth beyond that, so workgroups are kept to (budget / block bytes) per CU by asking for a
// matching share of the 160 KiB LDS.  Budget: 48 KiB for the register / shuffle / 128-bit LDS
// kernels (interleaved A/B, TB/s at 32 / 40 / 48 KiB: config 2 6.44 / 6.44 / 6.44, with the destination
// flipped 5.85 / 5.85 / 6.42, config 3 6.60 / 6.59 / 6.49, config 1's layouts on 32768 tiles 6.09 / 6.46 /
// 6.63, 128-bit LDS staging of config 2 - / 5.24 / 6.15: the more work a wave does between its loads
// and its stores, the more waves it takes to keep the same bytes in flight), 44 KiB (11 waves per
// CU) for the one-wave element-wide kernel (config 4: 9-11 per CU 6.70-6.74, 12: 6.65, 16: 6.53).
static void set_launch_params(ll_plan *plan)
{
    const ll_plan_desc &desc = plan->desc;
    const ll_options &opt = plan->opts;
    const long long block_bytes = (long long)desc.elem_bytes << desc.block_bits;
    const long long group_bytes = (long long)desc.elem_bytes << (desc.d + desc.group_bits);
    const long long kXcdTarget = 128 * 1024;
    switch (desc.strategy) {
    case LL_STRATEGY_LDS_ELEM:
    case LL_STRATEGY_LDS_TR: {
        // at every tile size (four waves per block on tiles above 128 KiB too: random XOR maps, five per size on 1 GiB
        // each way, geometric mean against the natural order: 2-byte elements 2^18 / 2^20 / 2^22 +3.6 / +2.7 / +5.3 %,
        // bytes +6.5 / +2.0 / +1.4 %)
        plan->lds_elem.xcd_chunk = opt_chunk_bits(opt.xcd_chunk, xcd_chunk_bits_for(kXcdTarget, block_bytes));
        int alloc = desc.lds_bytes;
        if (desc.threads < 256 || opt.inflight_bytes != LL_AUTO)
            alloc = lds_alloc_for((unsigned)block_bytes, (unsigned)opt_or(opt.inflight_bytes, 45056), alloc);
        else if (block_bytes == 8192)
            // four waves on 8 KiB blocks: six workgroups per CU instead of the eight that fit (1- and 2-byte elements
            // under random XOR maps and bit permutations: +2..6 %, e.g. 6.27 -> 6.52 TB/s on 2^12-element tiles);
            // 16 KiB blocks want all the workgroups they can get
            alloc = lds_alloc_for(8192u, 49152u, alloc);
        else if (desc.strategy == LL_STRATEGY_LDS_TR && block_bytes == 16384)
            // the transposing loads on 16 KiB blocks: three to five workgroups per CU 6.16-6.20 TB/s, six and more 5.8
            alloc = lds_alloc_for(16384u, 65536u, alloc);
        if (opt.lds_pad_bytes > 0) alloc = std::min(64 * 1024, alloc + opt.lds_pad_bytes);
        plan->lds_alloc = alloc;
        break;
    }
    case LL_STRATEGY_REG_PERMUTE:
    case LL_STRATEGY_WAVE_SHUFFLE:
    case LL_STRATEGY_LDS_VEC: {
        // 2-byte elements at every tile size (transposes of tiles above 128 KiB: 5.6-5.9 TB/s in natural order, 6.0-6.3
        // with it, all 12 shapes; random bit permutations +1 % on average); 4- and 8-byte elements only reach these
        // kernels with tiles up to 128 KiB
        const int chunk = (group_bytes <= kXcdTarget || desc.elem_bytes == 2) ? xcd_chunk_bits_for(kXcdTarget, block_bytes) : -1;
        plan->vec.xcd_chunk = opt_chunk_bits(opt.xcd_chunk, chunk);
        // the pure register path (no exchange, no affine constant to apply) is the lightest: 40 KiB suits it
        // (bench conditions: config 2 6.40 -> 6.43 TB/s, config 3 6.48 -> 6.57), everything else wants 48 KiB
        const bool light = plan->vec_xchg == kXchgNone && plan->vec.dst_xor == 0;
        plan->lds_alloc = lds_alloc_for((unsigned)desc.threads * (16u << plan->vec_nvec_bits),
                                        (unsigned)opt_or(opt.inflight_bytes, light ? 40960 : 49152), desc.lds_bytes);
        break;
    }
    case LL_STRATEGY_LDS_PULL: {
        // measured best with 256 KiB of consecutive destination blocks per XCD when writes dominate
        // (expand 16x: 5.95 -> 6.5 TB/s), 512 KiB otherwise
        const long long target = (desc.d_dst > desc.d ? 256 : 512) * 1024;
        plan->pull.xcd_chunk = opt_chunk_bits(opt.pull_xcd_chunk, xcd_chunk_bits_for(target, block_bytes));
        plan->lds_alloc = desc.lds_bytes;
        if (opt.pull_inflight_bytes != LL_AUTO)
            plan->lds_alloc = lds_alloc_for((16u << plan->pull_thread_bits) * (unsigned)plan->pull.dst_iters, (unsigned)opt.pull_inflight_bytes, desc.lds_bytes);
        break;
    }
    default:
        break;
    }
}

ll_status plan_convert(const ll_layout *src, const ll_layout *dst, int elem_bytes, ll_plan *plan)
{
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8)
        return fail(LL_ERR_INVALID_ARG, "elem_bytes must be 1, 2, 4 or 8 (got %d)", elem_bytes);
    if (src->d_out != dst->d_out)
        return fail(LL_ERR_DIM_MISMATCH, "source and destination map to output spaces of %d and %d bits", src->d_out, dst->d_out);
    // A memory layout (input label `offset`, Sec. 4.3) may stand on either side: its image is the
    // buffer indexed by memory offset, and the conversion is then the A^-1 o B of Sec. 5.3 "Shared
    // Memory Load and Store" between a memory image and a register image (or two memory images).
    bool memory_side = false;
    for (int i = 0; i < src->n_in; ++i) memory_side |= src->in_dims[i].label == LL_IN_OFFSET;
    for (int i = 0; i < dst->n_in; ++i) memory_side |= dst->in_dims[i].label == LL_IN_OFFSET;
    const bool memory_image = memory_side;
    const int d = src->d_in;
    if (f2::rank(src->bases) < src->d_out || f2::rank(dst->bases) < dst->d_out)
        return fail(LL_ERR_NOT_SURJECTIVE, "layout does not cover the whole logical tensor");
    if (d < 1 || dst->d_in < 1) return fail(LL_ERR_INVALID_ARG, "empty layout");
    if (d > src->d_out || dst->d_in > dst->d_out) {
        // broadcasting (Sec. 5.1, Sec. 5.4 rule 2): destination units pull from canonical source units
        std::memset(&plan->desc, 0, sizeof(plan->desc));
        plan->desc.elem_bytes = elem_bytes;
        if (ll_status st = plan_pull(src, dst, elem_bytes, plan); st != LL_OK) return st;
        set_launch_params(plan);
        return LL_OK;
    }
    if (memory_side) {
        if (src->d_in != dst->d_in)
            return fail(LL_ERR_DIM_MISMATCH, "source and destination layouts have %d and %d input bits", src->d_in, dst->d_in);
        if (src->bits_of(LL_IN_TILE) || dst->bits_of(LL_IN_TILE))
            return fail(LL_ERR_DIM_MISMATCH, "a memory layout cannot be converted to or from a layout with a tile label");
    } else if (!same_inputs(src, dst)) {
        // The same tile split differently over registers, lanes and waves: the images are still
        // 2^d slots per tile, so the conversion is the same B^-1 o A on flat indices.  The register /
        // lane / wave classes of the two sides do not line up, so no class-based shortcut applies
        // (handled like a memory image).  Tiles must agree.
        if (src->d_in != dst->d_in || src->bits_of(LL_IN_TILE) != dst->bits_of(LL_IN_TILE))
            return fail(LL_ERR_DIM_MISMATCH, "source and destination layouts have different input dims");
        memory_side = true;
    }

    // B^-1 o A (Sec. 5.4)
    mat binv;
    if (!f2::invert(dst->bases, d, &binv)) return fail(LL_ERR_NOT_INJECTIVE, "destination layout is not bijective");
    const mat p = f2::compose(binv, src->bases);

    // a tile label must pass through untouched
    const int tile_first = memory_image ? d : src->first_bit_of(LL_IN_TILE);
    for (int k = 0; k < d; ++k) {
        const vec tile_mask = ((vec(1) << d) - 1) & ~((vec(1) << tile_first) - 1);
        if (k >= tile_first ? p[k] != (vec(1) << k) : (p[k] & tile_mask) != 0)
            return fail(LL_ERR_TILE_MIXED, "the conversion would move data between tiles");
    }

    ll_plan_desc &desc = plan->desc;
    std::memset(&desc, 0, sizeof(desc));
    desc.d = desc.d_dst = d;
    desc.elem_bytes = elem_bytes;
    for (int k = 0; k < d; ++k) desc.conv[k] = p[k];
    desc.kind = classify(p, d, src->bits_of(LL_IN_REG), src->first_bit_of(LL_IN_WAVE));
    if (memory_side && desc.kind != LL_KIND_NOOP) desc.kind = LL_KIND_LDS;      // no register / lane / wave classes to compare
    paper_shuffle_schedule(src, dst, elem_bytes, &desc);
    // Affine layouts: x = A h ^ a = B h' ^ b gives h' = P h ^ c with c = B^-1 (a ^ b).  The planners
    // below work on P alone; c is a constant XOR on every destination index, which the kernels
    // apply when they store (whole vectors move by its upper bits, elements inside a vector by
    // its low bits), so it changes neither blocks, nor LDS layouts, nor exchanges.
    const vec c = f2::apply(binv, src->offset ^ dst->offset);
    if (c & (((vec(1) << d) - 1) & ~((vec(1) << tile_first) - 1)))
        return fail(LL_ERR_TILE_MIXED, "the offsets of the layouts would move data between tiles");
    desc.conv_offset = c;
    if (desc.kind == LL_KIND_NOOP && c == 0) {
        desc.strategy = LL_STRATEGY_COPY;
        desc.global_vec_bytes = 16;
        desc.threads = 256;
        return LL_OK;
    }
    if (ll_status st = choose_strategy(p, d, elem_bytes, plan); st != LL_OK) return st;
    {
        const bool elem = desc.strategy == LL_STRATEGY_LDS_ELEM || desc.strategy == LL_STRATEGY_LDS_TR;
        desc.src_lines_per_access = wave_access_lines(elem ? plan->lds_elem.lane_src : plan->vec.lane_src, elem_bytes);
        desc.dst_lines_per_access = wave_access_lines(elem ? plan->lds_elem.lane_dst : plan->vec.lane_dst, elem_bytes);
    }
    plan->lds_elem.dst_xor = (uint32_t)c;      // whichever argument block the strategy uses
    plan->vec.dst_xor = (uint32_t)c;
    set_launch_params(plan);
    return LL_OK;
}

}  // namespace ll

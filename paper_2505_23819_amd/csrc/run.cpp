// Host side of the device entry points: pick the kernel a plan names, fill the per-call fields of
// its argument block, validate the gather layout (paper Sec. 5.5) and launch.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <vector>

#include "plan.hpp"

using f2::mat;
using f2::vec;

namespace ll {

// 1 MiB of consecutive 4 KiB blocks per XCD: 2 % above the natural round robin for the plain copy
// (6.77 against 6.62 TB/s at 1 GiB)
int copy_xcd_chunk_bits(const ll_options &opt) { return opt_chunk_bits(opt.copy_xcd_chunk, 8); }

// Everything a launch needs beyond the caller's pointers and tile count is fixed when the plan is
// made (set_launch_params in plan.cpp): no environment lookups, allocations or attribute calls here.
ll_status run_convert(const ll_plan *plan, const void *src, void *dst, long long ntiles, void *stream)
{
    const ll_plan_desc &desc = plan->desc;
    switch (desc.strategy) {
    case LL_STRATEGY_COPY:
        return launch_copy(src, dst, (ntiles << desc.d) * desc.elem_bytes, copy_xcd_chunk_bits(plan->opts), stream);
    case LL_STRATEGY_LDS_ELEM: {
        LdsElemArgs a = plan->lds_elem;
        a.src = src;
        a.dst = dst;
        a.ntiles = ntiles;
        const long long groups = (ntiles + (1ll << a.group_bits) - 1) >> a.group_bits;
        a.nblocks = groups << a.coset_bits;
        return launch_lds_elem(a, desc.elem_bytes, plan->nvec, desc.lds_vec_bits, desc.threads, plan->lds_alloc, stream);
    }
    case LL_STRATEGY_LDS_TR: {
        LdsElemArgs a = plan->lds_elem;
        a.src = src;
        a.dst = dst;
        a.ntiles = ntiles;
        const long long groups = (ntiles + (1ll << a.group_bits) - 1) >> a.group_bits;
        a.nblocks = groups << a.coset_bits;
        return launch_lds_tr(a, desc.elem_bytes, plan->nvec, plan->lds_alloc, stream);
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
                          plan->lds_alloc, stream);
    }
    case LL_STRATEGY_LDS_PULL: {
        PullArgs a = plan->pull;
        a.src = src;
        a.dst = dst;
        a.ntiles = ntiles;
        const long long groups = (ntiles + (1ll << a.group_bits) - 1) >> a.group_bits;
        a.nblocks = groups << a.coset_bits;
        return launch_pull(a, desc.elem_bytes, plan->pull_src_iters, plan->pull_vec_bits, plan->pull_thread_bits, plan->lds_alloc, stream);
    }
    default:
        return fail(LL_ERR_UNSUPPORTED, "plan strategy %d has no kernel", desc.strategy);
    }
}

// What run_gather decides before it launches: which kernel, and the geometry of the general one.
struct GatherChoice {
    int kernel = 0;                    // ll_gather_desc.kernel
    int axis_reg_bits = 0, axis_lane_bits = 0, axis_wave_bits = 0;
    bool memory = false;               // memory layout: no registers, lanes or waves
    GatherArgs wave = {};              // shuffle / wave-staged kernels
    GatherGenArgs gen = {};            // workgroup-staged kernel
    int lds_alloc = 0;                 // wave-level kernels: dynamic LDS to ask for (caps the workgroups per CU)
    int waves = 4;                     // wave-level kernels: waves (chunks) per workgroup
    int thread_bits = 8;               // workgroup-staged kernel: log2 threads per workgroup
};

static ll_status choose_gather(const ll_layout *L, int axis, int elem_bytes, const ll_options &opt, GatherChoice *c)
{
    // A memory layout (one `offset` input, Sec. 4.3) is a buffer indexed by memory offset: no lanes or
    // waves to shuffle between, every bit counts as a register bit and the staged kernels serve it.
    bool memory = false;
    for (int i = 0; i < L->n_in; ++i) memory |= L->in_dims[i].label == LL_IN_OFFSET;
    c->memory = memory;
    if (axis < 0 || axis >= L->n_out) return fail(LL_ERR_INVALID_ARG, "axis %d of a %d-dim tensor", axis, L->n_out);
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8)
        return fail(LL_ERR_INVALID_ARG, "elem_bytes must be 1, 2, 4 or 8 (got %d)", elem_bytes);
    const int d = L->d_in;
    if (f2::rank(L->bases) < L->d_out) return fail(LL_ERR_NOT_SURJECTIVE, "layout does not cover the whole logical tensor");
    // Right inverse with free variables zero (Def. "Right Inverse"); the inverse when L is bijective.
    // Under a broadcasting layout `in` is the image of a logical tensor (equal replicas), so any slot
    // that holds the wanted element will do; the one that differs from the receiving slot by L^+ of
    // the coordinate difference is taken, L(h ^ L^+(delta)) = L(h) ^ delta, because it keeps the
    // kernels' "own index xor linear delta" addressing.
    mat linv;
    if (!f2::right_inverse(L->bases, L->d_out, &linv)) return fail(LL_ERR_NOT_SURJECTIVE, "layout does not cover the whole logical tensor");
    const int nreg = L->bits_of(LL_IN_REG), nlane = L->bits_of(LL_IN_LANE);
    const int lane0 = memory ? d : L->first_bit_of(LL_IN_LANE), wave0 = memory ? d : L->first_bit_of(LL_IN_WAVE);
    const int tile0 = memory ? d : L->first_bit_of(LL_IN_TILE);
    int axis_shift = 0;
    for (int k = L->n_out - 1; k > axis; --k) axis_shift += L->out_dims[k].nbits;
    const int na = L->out_dims[axis].nbits;
    const vec all = (vec(1) << d) - 1;
    const vec reg_mask = (vec(1) << lane0) - 1;
    const vec lane_mask = ((vec(1) << wave0) - 1) & ~reg_mask;
    const vec wave_mask = ((vec(1) << tile0) - 1) & ~(reg_mask | lane_mask);
    const vec tile_mask = all & ~((vec(1) << tile0) - 1);

    // Moving one step along axis bit b moves the hardware index by L^-1(e_b) (Sec. 5.5: the source
    // of an element is L^-1 of its position with the axis coordinate replaced).
    vec touched = 0;
    for (int b = 0; b < na; ++b) touched |= linv[axis_shift + b];
    if (touched & tile_mask) return fail(LL_ERR_TILE_MIXED, "the gather axis crosses tiles");
    c->axis_reg_bits = f2::popcount(touched & reg_mask);
    c->axis_lane_bits = f2::popcount(touched & lane_mask);
    c->axis_wave_bits = f2::popcount(touched & wave_mask);
    auto axis_coord = [&](vec h) { return (uint32_t)((f2::apply(L->bases, h) >> axis_shift) & ((vec(1) << na) - 1)); };
    // affine layouts: every element's axis coordinate carries the axis part of the offset; the
    // moves along the axis (differences) do not change
    const uint32_t own_const = (uint32_t)((L->offset >> axis_shift) & ((vec(1) << na) - 1));

    const bool lane_only = !(touched & ~lane_mask) && nlane == LL_WAVE_LANE_BITS && nreg <= 6 && d - nreg - nlane <= 16 &&
                           na <= 6 && (1 << nreg) * elem_bytes >= 4 && (1 << nreg) * elem_bytes <= 256;
    // Lanes that hold fewer than 16 bytes make the shuffle kernel's global accesses narrow (measured
    // 4.6-5.5 TB/s against 6.4-6.5 for the workgroup-staged kernel), so those layouts take the general
    // kernel unless the options ask for one of the wave kernels.
    // One-byte elements need one shuffle each however many a lane holds (measured 4.8 TB/s with 16 per
    // lane against 5.7-5.9 staged), so they take the general kernel as well.
    // Lanes that hold 128 bytes or more: the wave kernels need 32 to 64 registers each for data, indices
    // and results; measured 5.8-6.4 TB/s for them against 6.3-6.6 for the workgroup-staged kernel.
    const bool narrow = (1 << nreg) * elem_bytes < 16 || elem_bytes == 1 || (1 << nreg) * elem_bytes >= 128;
    const bool wave_kernel_asked = opt.gather_kernel == LL_GATHER_SHUFFLE || opt.gather_kernel == LL_GATHER_WAVE_STAGED ||
                                   opt.gather_kernel == LL_GATHER_SHUFFLE_ROWS;
    const bool want_general = opt.gather_kernel == LL_GATHER_BLOCK_STAGED || (!wave_kernel_asked && narrow);
    if (lane_only && !want_general) {
        GatherArgs &a = c->wave;
        std::memset(&a, 0, sizeof(a));
        const int nhigh = d - nreg - nlane;
        for (int b = 0; b < na; ++b) a.lane_delta[b] = (uint32_t)((linv[axis_shift + b] & lane_mask) >> nreg);
        for (int b = 0; b < 6; ++b) a.own_lane[b] = axis_coord(vec(1) << (nreg + b));
        for (int r = 0; r < (1 << nreg); ++r) a.own_reg[r] = axis_coord((vec)r);
        for (int b = 0; b < nhigh; ++b) a.own_wave[b] = axis_coord(vec(1) << (nreg + 6 + b));
        for (int b = 0; b < nreg; ++b) a.own_regbit[b] = axis_coord(vec(1) << b);
        a.nwave = nhigh;
        a.nreg = nreg;
        a.axis_mask = (1u << na) - 1;
        a.own_const = own_const;
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
            ok &= own_const == 0;
            if (ok) {
                a.fast = 1;
                a.shift = shift;
                a.keep_mask = 63u & ~(a.axis_mask << shift);
            }
        }
        // Rows of 16 bytes are already one coalesced vector per lane: shuffle directly.  Wider rows would
        // make every lane's accesses strided (measured 4.58 TB/s on config 5), so they are moved in
        // coalesced 16-byte pieces and either staged through wave-private LDS or brought into "one row
        // per lane" by lane <-> register butterflies and gathered with ds_bpermute_b32 as Sec. 5.5 does.
        // Measured (TB/s, staged / butterflies, each with one wave per workgroup): rows of 32 bytes
        // 6.83 / 6.51 (config 5), 6.60 / 6.62, 6.56 / 6.54; 64 bytes 6.37 / 6.56, 6.59 / 6.75, 6.67 / 6.82;
        // 128 bytes 5.81 / 6.38, 5.95 / 6.39, 5.98 / 6.35 (workgroup-staged kernel: 6.3, 6.6, 6.5); 256 bytes
        // 5.68 / 5.70 and 5.70 / 5.50, against 5.89 and 6.17 staged by four waves per workgroup (workgroup-
        // staged kernel: 6.28, 6.16).  Hence 32 bytes: staged, 64: butterflies, more: not here at all.
        const int row_bytes = (1 << nreg) * elem_bytes;
        // Rows wider than 16 bytes under an axis that is NOT a plain field of the lane index (lane bits permuted or
        // mixed): the wave kernels then work out every element's source lane bit by bit, and the workgroup-staged
        // kernel with its delta tables is far ahead (five random lane-bit orders each, TB/s: 32-byte rows of 2-byte
        // elements 4.5 against 6.5, 64-byte rows 4.3-5.1 against 6.5; 16-byte rows 6.4 against 6.6, left to the
        // shuffle kernel).  Those layouts go on to the general case below.
        if (a.fast || row_bytes <= 16 || wave_kernel_asked) {
            a.staged = (row_bytes > 16 && row_bytes <= 256 && nreg >= 2) ? ((row_bytes == 64 || row_bytes == 128) ? 2 : 1) : 0;
            if (opt.gather_kernel == LL_GATHER_SHUFFLE) a.staged = 0;
            if (opt.gather_kernel == LL_GATHER_WAVE_STAGED) a.staged = row_bytes >= 16 && row_bytes <= 256 && nreg >= 2;
            if (opt.gather_kernel == LL_GATHER_SHUFFLE_ROWS) a.staged = (row_bytes >= 32 && row_bytes <= 256 && nreg >= 2) ? 2 : 0;
            c->kernel = a.staged == 2 ? LL_GATHER_SHUFFLE_ROWS : a.staged ? LL_GATHER_WAVE_STAGED : LL_GATHER_SHUFFLE;
            // The kernels with coalesced pieces run ONE wave per workgroup (a wave's chunk is its own: it goes
            // on as soon as its loads have landed), a number of waves per CU set through the LDS share, and an
            // XCD-aware order.  Measured on MI355X (64 x 256 tiles and relatives, 512 MiB of `in`, TB/s):
            // config 5 four waves per workgroup 6.59, one wave 6.68, with 32 consecutive chunks per XCD 6.84;
            // 5 waves per CU 5.0, 8: 6.35-6.8, 10: 6.84 (6 KiB loaded per wave), 16: 6.55 (4 KiB per wave).
            // The shuffle kernel on rows of 8 or 16 bytes does best with one wave per workgroup as well, in natural
            // order and without a cap (16-byte rows of 2- / 4- / 8-byte elements: four waves 6.37 / 6.23 / 6.43, one
            // wave 6.53 / 6.70 / 6.81; 32 consecutive chunks per XCD: 6.36 / 6.06 / 6.29).
            const bool one_wave = a.staged && row_bytes < 256;
            const bool one_wave_shuffle = !a.staged && row_bytes >= 8;
            c->waves = (opt.gather_waves == 1 || opt.gather_waves == 2 || opt.gather_waves == 4) ? opt.gather_waves
                                                                                                   : ((one_wave || one_wave_shuffle) ? 1 : 4);
            const unsigned load_bytes = 64u * ((unsigned)row_bytes + 4u * (1u << nreg));           // per wave: `in` and `idx`
            const unsigned wave_bytes = load_bytes + 64u * (unsigned)row_bytes;                       // ... and `out`
            // 256 KiB of consecutive chunks (in + idx + out) per XCD; 64 KiB of loads in flight per CU, but 8 to 16 waves
            a.xcd_chunk = opt_chunk_bits(opt.gather_xcd_chunk, one_wave ? xcd_chunk_bits_for(256 * 1024, (long long)wave_bytes * c->waves) : -1);
            c->lds_alloc = 0;
            if (!a.staged && opt.gather_inflight_bytes != LL_AUTO)
                c->lds_alloc = lds_alloc_for(1u, std::max(1u, (unsigned)opt.gather_inflight_bytes / (load_bytes * (unsigned)c->waves)), 0);
            if (a.staged) {
                unsigned groups = (unsigned)opt_or(opt.gather_inflight_bytes, one_wave ? 65536 : 49152) / (load_bytes * (unsigned)c->waves);
                if (opt.gather_inflight_bytes == LL_AUTO && one_wave) groups = std::min(std::max(groups, 8u / (unsigned)c->waves), 16u);
                c->lds_alloc = lds_alloc_for(1u, std::max(groups, 1u), 0);
            }
            return LL_OK;
        }
    }

    // General case: the axis occupies register and / or wave bits (or the layout is not wave64
    // shaped).  A set of image elements closed under moves along the axis is a coset of any
    // subspace U that contains the deltas; one workgroup stages one coset in LDS.  The paper's
    // shuffle rounds (2^|register bits of the axis| per element) are replaced by one LDS read per
    // element: a round needs a register index chosen per lane at run time, and ds_bpermute_b32 goes
    // through the same LDS crossbar anyway.
    //   U = span(e_0 .. e_{c-1}) + span(deltas): the low c index bits give contiguous runs of 2^c
    //   elements (coalesced global access: 128 bytes where the block allows), the deltas close it.
    //   Bits between the runs and the deltas (the columns of a row gather in a row-major tile)
    //   select the coset, so the block need not be the aligned range up to the highest delta bit.
    if (na > kMaxAxisBits) return fail(LL_ERR_UNSUPPORTED, "gather axis of 2^%d elements", na);
    const int vs = 31 - __builtin_clz(16u / (unsigned)elem_bytes);
    const int ubits = elem_bytes == 8 ? 1 : 2;                        // log2 elements per unit of the gather phase
    const int wlog = 31 - __builtin_clz((unsigned)elem_bytes);
    const int top = touched ? 64 - __builtin_clzll((unsigned long long)touched) : 0;
    // gfx950 has 160 KiB of LDS per CU: blocks up to 128 KiB (plus the delta tables) are staged
    const long long lds_max = opt_or(opt.gather_lds_max_bytes, 128 * 1024);
    const int max_bits = 63 - __builtin_clzll((unsigned long long)std::max(1ll, lds_max / elem_bytes));
    int min_bits = std::max(vs + 8, 10);                               // one 16-byte vector and one unit per thread
    {
        // 8 KiB blocks measured best on MI355X when the axis leaves the choice (4 KiB: -5 %, 32 KiB: -4 %)
        const int bytes = opt_or(opt.gather_block_bytes, 8192);
        min_bits = std::max(min_bits, 31 - __builtin_clz((unsigned)std::max(1, bytes / elem_bytes)));
    }
    const int gb = std::max(0, min_bits - d);                          // small tiles are bundled
    const int D = d + gb;
    auto dim_u = [&](int cc, mat *basis) {
        mat us, cand;
        for (int j = 0; j < cc; ++j) us.push_back(vec(1) << j);
        const vec low = (vec(1) << cc) - 1;
        for (int b = 0; b < na; ++b) cand.push_back(linv[axis_shift + b] & ~low);
        for (vec x : f2::extend(us, cand)) us.push_back(x);
        if (basis) *basis = us;
        return (int)us.size();
    };
    const int cmin = std::max(vs, ubits);
    int cb = std::min(D, std::max(cmin, 7 - wlog));                    // runs of 128 bytes to start with
    while (cb > cmin && dim_u(cb, nullptr) > max_bits) --cb;           // shorter runs if the block would not fit LDS
    while (cb < D && dim_u(cb, nullptr) < min_bits) ++cb;              // longer runs up to the preferred block size
    mat us;
    const int n = dim_u(cb, &us);
    // A block beyond LDS even with the shortest runs, or runs under 64 bytes (every line would be
    // fetched by several blocks): the source elements are read straight from memory inside the
    // aligned 2^top block around each element.
    // (the staged kernel addresses a tile group through 32-bit buffer offsets)
    // Runs under 64 bytes make several blocks fetch every 128-byte line (consecutive blocks, which the
    // XCD-aware order keeps on one L2).  Measured against the memory-direct kernel: worth it only when
    // the aligned range is beyond an XCD's 4 MiB L2 (4096 x 4096 two-byte rows, 32-byte runs: 2.0
    // against 0.51 TB/s; four-byte: 1.44 / 0.68), not below (4096 x 256 eight-byte: 1.44 / 1.71).
    const int min_run = opt_or(opt.gather_min_run_bytes, ((long long)elem_bytes << top) > (4ll << 20) ? 32 : 64);
    const bool global = n > max_bits || (elem_bytes << cb) < min_run || D + wlog > 31;
    GatherGenArgs &g = c->gen;
    std::memset(&g, 0, sizeof(g));
    g.na = na;
    g.axis_mask = (uint32_t)((vec(1) << na) - 1);
    g.own_const = own_const;
    g.d = d;
    if (global) {
        // (a range smaller than a workgroup's share of consecutive elements is widened to it: the
        // aligned range only grows, and it stays inside the tile)
        g.block_bits = std::max(top, gather_global_chunk_bits(elem_bytes));
        for (int b = 0; b < na; ++b) g.delta[b] = (uint32_t)linv[axis_shift + b];
        for (int b = 0; b < d && b < 32; ++b) g.own_bit[b] = axis_coord(vec(1) << b);
        // An aligned block of a few LDS sizes is walked through LDS chunk by chunk by every workgroup
        // that has elements in it (k_gather_phased): the block is then read from L2 once per workgroup,
        // in full lines, instead of one line per element.  Measured on MI355X (row gathers in row-major
        // tiles, where the source index needs no tables; TB/s, chunk walk against memory-direct): ranges of
        // 256 KiB: one-byte elements 3.99 / 1.46, four-byte 5.11 / 2.48; 512 KiB: two-byte 3.35 / 1.76,
        // eight-byte 3.85 / 3.08; 1 MiB: one-byte 1.80 / 1.39, four-byte 2.85 / 2.40; 2 MiB: two-byte
        // 1.27 / 1.66, eight-byte 1.63 / 2.86.  Random XOR layouts (table lookups), 512 KiB: 2.5 / 2.9 / 3.5
        // for 1- / 2- / 4-byte elements.  The cost grows with range bytes per workgroup element, the
        // memory-direct kernel's does not.
        const int pcb = gather_phased_chunk_bits(elem_bytes);
        const long long phased_max = opt_or(opt.gather_phased_max_bytes, 1024 * 1024);
        const long long block_bytes = (long long)elem_bytes << top;
        const bool phased = top >= pcb && block_bytes >= 2 * gather_phased_lds_chunk_bytes() && block_bytes <= phased_max && top + wlog <= 31;
        c->kernel = phased ? LL_GATHER_PHASED : LL_GATHER_GLOBAL;
        // The axis coordinate of an element may simply be a bit field of its index (row-major memory
        // layouts, blocked layouts): then the source is the element's own index with that field
        // replaced by the gather index, no tables needed.
        g.field_shift = -1;
        if (na > 0 && own_const == 0 && g.delta[0] != 0 && !(g.delta[0] & (g.delta[0] - 1))) {
            const int shift = __builtin_ctz(g.delta[0]);
            bool field = shift + na <= 32;
            for (int b = 0; b < na && field; ++b) field = g.delta[b] == (1u << (shift + b));
            for (int j = 0; j < 32 && field; ++j) field = g.own_bit[j] == ((j >= shift && j < shift + na) ? (1u << (j - shift)) : 0u);
            if (field) g.field_shift = shift;
        }
        // XCD-aware order: the workgroups of one aligned range run on one XCD, whose L2 serves their
        // repeated reads of it (the memory-direct kernel: up to 2 MiB of a larger range)
        const int cb = phased ? pcb : gather_global_chunk_bits(elem_bytes);
        const int range_chunks = (phased ? g.block_bits : std::min(g.block_bits, 21 - wlog)) - cb;
        g.xcd_chunk = opt_chunk_bits(opt.gather_xcd_chunk, range_chunks > 0 ? range_chunks : -1);
        return LL_OK;
    }
    if (n < min_bits) return fail(LL_ERR_INVALID_ARG, "internal: gather block smaller than the kernel's unit of work");
    g.block_bits = n;
    g.group_bits = gb;
    f2::Basis ub;
    for (int j = 0; j < n; ++j) ub.add(us[j], vec(1) << j);
    for (int b = 0; b < na; ++b) {
        vec tag = 0;
        if (ub.reduce(linv[axis_shift + b], &tag) != 0) return fail(LL_ERR_INVALID_ARG, "internal: gather block not closed under the axis");
        g.delta[b] = (uint32_t)tag;                                    // in block-local coordinates
    }
    for (int j = 0; j < n; ++j) {
        g.embed[j] = (uint32_t)us[j];
        g.own_bit[j] = (us[j] >> d) ? 0u : axis_coord(us[j]);          // bundled-tile bits carry no coordinate
    }
    const mat comp = f2::complement(us, D);
    if ((int)comp.size() > kMaxCosetBits) return fail(LL_ERR_UNSUPPORTED, "internal: too many gather blocks per tile");
    g.coset_bits = (int)comp.size();
    for (size_t k = 0; k < comp.size(); ++k) {
        g.coset[k] = (uint32_t)comp[k];
        g.own_coset[k] = (comp[k] >> d) ? 0u : axis_coord(comp[k] & all);
    }
    // LDS swizzle: the bank field is address bits [ub, ub + 5); bring layout-lane bits into it
    const int ubk = elem_bytes == 8 ? 3 : 2;
    const int rb = 31 - __builtin_clz((unsigned)((1 << nreg) * elem_bytes));
    const int t = std::min(std::max(rb, ubk), ubk + 5);
    const int nx = std::min(5, t - ubk);
    g.swz_shift = std::max(ubk + 5, rb);
    g.swz_to = ubk;
    g.swz_mask = (1u << nx) - 1;
    {
        // When no move along the axis changes the bank bits of an LDS address (a row gather in a
        // row-major tile: the deltas sit above the runs), every lane reads in the bank of its own
        // unit and consecutive units already spread over the banks: a swizzle would only scatter them.
        vec moved = 0;
        for (int b = 0; b < na; ++b) moved |= g.delta[b];
        const int lo = std::max(0, ubk - wlog), hi = ubk + 5 - wlog;      // element bits that form the bank field
        const vec bank_bits = hi > lo ? ((vec(1) << hi) - 1) & ~((vec(1) << lo) - 1) : 0;
        const bool always = opt.gather_swizzle_always == 1;
        if (!(moved & bank_bits) && !always) g.swz_mask = 0;
    }
    // deltas that are consecutive single bits of the block-local index, nothing swizzled: the LDS byte
    // offset of a move is (coordinate difference) << field_shift
    g.field_shift = -1;
    if (g.swz_mask == 0 && na > 0 && g.delta[0] != 0 && !(g.delta[0] & (g.delta[0] - 1))) {
        const int shift = __builtin_ctz(g.delta[0]);
        bool field = true;
        for (int b = 0; b < na && field; ++b) field = g.delta[b] == (1u << (shift + b));
        if (field) g.field_shift = shift + wlog;
    }
    c->kernel = LL_GATHER_BLOCK_STAGED;
    // XCD-aware block order: 512 KiB of consecutive blocks per XCD (rows of config 5: 5.99 -> 6.36 TB/s)
    g.xcd_chunk = opt_chunk_bits(opt.gather_xcd_chunk, xcd_chunk_bits_for(512 * 1024, (long long)elem_bytes << g.block_bits));
    c->thread_bits = gather_general_thread_bits((long long)elem_bytes << g.block_bits, elem_bytes);
    if (opt.gather_threads_log2 >= 8 && opt.gather_threads_log2 <= 10) {
        // every thread must get at least one 16-byte vector of the block and one unit of output elements
        const long long vectors = ((long long)elem_bytes << g.block_bits) / 16, units = (1ll << g.block_bits) >> ubits;
        if ((std::min(vectors, units) >> opt.gather_threads_log2) >= 1) c->thread_bits = opt.gather_threads_log2;
    }
    c->lds_alloc = 0;
    const long long staged_bytes = (long long)elem_bytes << g.block_bits;
    if (opt.gather_inflight_bytes != LL_AUTO)
        c->lds_alloc = lds_alloc_for((unsigned)staged_bytes, (unsigned)opt.gather_inflight_bytes, 0);
    else if (staged_bytes == 8192)
        // 8 KiB blocks: six workgroups per CU instead of the eight that fit (config 5's layout, rows and columns:
        // 6.43 -> 6.72 and 6.32 -> 6.65 TB/s; row-major 64 x 256 tiles +1..3 %; five workgroups: 5.8)
        c->lds_alloc = lds_alloc_for(8192u, 49152u, 0);
    return LL_OK;
}

// choose_gather costs about 3 us of host time (a right inverse, a few subspace bases), most of a small
// gather's launch cost, and a layout is immutable: the choices are kept with the layout, keyed by
// axis, element size and the options they were made under.  The list is replaced as a whole (copy,
// append, atomic store), so concurrent callers need no lock; two threads that miss at the same time
// both compute the same entry and one list wins.  A hit costs a few integer comparisons.
struct GatherCache {
    struct Entry {
        int axis, elem_bytes;
        ll_options opts;
        GatherChoice choice;
    };
    std::vector<Entry> entries;
};

static ll_status choose_gather_cached(const ll_layout *L, int axis, int elem_bytes, const ll_options *given, GatherChoice *c)
{
    const ll_options &opt = given ? *given : process_options();       // `given` is complete (resolve_options)
    std::shared_ptr<const GatherCache> have = std::atomic_load(&L->gather_cache.p);
    if (have)
        for (const GatherCache::Entry &e : have->entries)
            if (e.axis == axis && e.elem_bytes == elem_bytes && same_options(e.opts, opt)) {
                *c = e.choice;
                return LL_OK;
            }
    if (ll_status st = choose_gather(L, axis, elem_bytes, opt, c); st != LL_OK) return st;
    auto next = std::make_shared<GatherCache>();
    if (have && have->entries.size() < 32) next->entries = have->entries;     // bounded: start over when full
    next->entries.push_back({axis, elem_bytes, opt, *c});
    std::atomic_store(&L->gather_cache.p, std::shared_ptr<const GatherCache>(next));
    return LL_OK;
}

ll_status describe_gather(const ll_layout *L, int axis, int elem_bytes, const ll_options *opts, ll_gather_desc *out)
{
    GatherChoice c;
    if (ll_status st = choose_gather_cached(L, axis, elem_bytes, opts, &c); st != LL_OK) return st;
    std::memset(out, 0, sizeof(*out));
    out->kernel = c.kernel;
    out->axis_reg_bits = c.axis_reg_bits;
    out->axis_lane_bits = c.axis_lane_bits;
    out->axis_wave_bits = c.axis_wave_bits;
    out->paper_rounds = c.memory ? 0 : 1 << c.axis_reg_bits;
    const long long gen_bytes = (long long)elem_bytes << c.gen.block_bits;
    out->block_bytes = c.kernel == LL_GATHER_BLOCK_STAGED || c.kernel == LL_GATHER_GLOBAL || c.kernel == LL_GATHER_PHASED
                           ? (int32_t)std::min(gen_bytes, (long long)INT32_MAX)
                           : 64 * (1 << L->bits_of(LL_IN_REG)) * elem_bytes;
    return LL_OK;
}

ll_status run_gather(const ll_layout *L, int axis, int elem_bytes, const ll_options *opts, const void *in, const int32_t *idx, void *out,
                     long long ntiles, void *stream)
{
    GatherChoice c;
    if (ll_status st = choose_gather_cached(L, axis, elem_bytes, opts, &c); st != LL_OK) return st;
    const int d = L->d_in;
    if (ntiles == 0) return LL_OK;
    if (!in || !idx || !out) return fail(LL_ERR_INVALID_ARG, "null device pointer");
    if ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(idx) | reinterpret_cast<uintptr_t>(out)) & 15)
        return fail(LL_ERR_INVALID_ARG, "device buffers must be 16-byte aligned");
    const unsigned long long bytes = ((unsigned long long)ntiles << d) * elem_bytes;
    if (ntiles > (1ll << 40) >> d) return fail(LL_ERR_INVALID_ARG, "ntiles is too large");
    if (bytes & 15) return fail(LL_ERR_INVALID_ARG, "ntiles * tile bytes (%llu) must be a multiple of 16", bytes);
    const char *pi = static_cast<const char *>(in), *po = static_cast<const char *>(out);
    const char *px = reinterpret_cast<const char *>(idx);
    const unsigned long long ibytes = ((unsigned long long)ntiles << d) * 4;
    if ((pi < po + bytes && po < pi + bytes) || (px < po + bytes && po < px + ibytes))
        return fail(LL_ERR_INVALID_ARG, "the output buffer overlaps an input buffer");
    if (c.kernel == LL_GATHER_PHASED || c.kernel == LL_GATHER_GLOBAL) {
        GatherGenArgs &g = c.gen;
        g.in = in;
        g.idx = idx;
        g.out = out;
        g.total_elems = ntiles << d;
        const int cb = c.kernel == LL_GATHER_PHASED ? gather_phased_chunk_bits(elem_bytes) : gather_global_chunk_bits(elem_bytes);
        g.nblocks = (g.total_elems + (1ll << cb) - 1) >> cb;
        return c.kernel == LL_GATHER_PHASED ? launch_gather_phased(g, elem_bytes, stream) : launch_gather_global(g, elem_bytes, stream);
    }
    if (c.kernel == LL_GATHER_BLOCK_STAGED) {
        GatherGenArgs &g = c.gen;
        g.in = in;
        g.idx = idx;
        g.out = out;
        g.ntiles = ntiles;
        g.total_elems = ntiles << d;
        const long long ngroups = (ntiles + (1ll << g.group_bits) - 1) >> g.group_bits;
        g.nblocks = ngroups << g.coset_bits;
        return launch_gather_general(g, elem_bytes, c.thread_bits, c.lds_alloc, stream);
    }
    GatherArgs &a = c.wave;
    a.in = in;
    a.idx = idx;
    a.out = out;
    a.nchunks = ntiles << a.nwave;
    return launch_gather(a, elem_bytes, c.waves, c.lds_alloc, stream);
}

}  // namespace ll

// Conversion planner: B^-1 o A, its classification, work decomposition and kernel tables
// (paper Sec. 5.4).
#pragma once
#include "kernels.hpp"
#include "layout.hpp"

namespace ll {

// LDS hardware model used by the swizzle synthesizer.  An LDS instruction of a wave is served in
// phases; the lanes of one phase must fall in distinct banks (or touch the same 4-byte word).
// A phase is a coset of a subspace of the 6-bit lane index.  The defaults describe gfx950 as
// measured with two-active-lane micro-benchmarks (timing for reads, SQ_LDS_BANK_CONFLICT for
// writes); index 0 = accesses up to 4 bytes, 1 = 8 bytes, 2 = 16 bytes:
//   reads   <= 4 B: lanes 0-31 / 32-63, 32 banks;  8 B: the same halves, 64 banks;
//           16 B: four groups of 16 lanes {l5 = const, l2^l3^l4 = const}, 64 banks
//   writes  <= 4 B: halves;  8 B: 16 consecutive lanes;  16 B: 8 consecutive lanes;
//           a write phase moves at most 128 bytes, modelled as 32 banks
struct LdsModel {
    int rd_banks[3] = {32, 64, 64};
    int rd_phase_dim[3] = {5, 5, 4};
    uint32_t rd_phase_basis[3][6] = {{1, 2, 4, 8, 16}, {1, 2, 4, 8, 16}, {1, 2, 12, 20}};
    int wr_banks[3] = {32, 32, 32};
    int wr_phase_dim[3] = {5, 4, 3};
    uint32_t wr_phase_basis[3][6] = {{1, 2, 4, 8, 16}, {1, 2, 4, 8}, {1, 2, 4}};
};

// Swizzled LDS layout for one staged block (paper Sec. 5.4 "Optimal Swizzling" and appendix).
//   n         block bits; all vectors live in the block-local space F2^n
//   v         log2 of the elements moved by one LDS access (the common contiguous run)
//   w         element bytes
//   wr_lanes  images of the 6 lane bits of a writing instruction
//   rd_lanes  images of the 6 lane bits of a reading instruction
// Returns the memory layout M (n columns: LDS element offset -> block-local index) with
// M e_b = e_b for b < v.  *wf_write / *wf_read receive the predicted wavefronts per phase.
f2::mat synthesize_swizzle(int n, int v, int w, const f2::mat &wr_lanes, const f2::mat &rd_lanes,
                           const LdsModel &hw, int *wf_write, int *wf_read);

int lds_width_class(int access_bytes);   // 0, 1, 2 for <=4, 8, 16 bytes

// Geometry of the blocks a conversion is cut into (see build_blocks).
struct BlockGeom {
    int d = 0, g = 0, D = 0;      // tile bits, bundling bits, D = d + g
    int k = 0, n = 0;             // run bits, block bits
    int vs = 0, w = 0;            // log2 elements per 16-byte vector, element bytes
    f2::mat pext;                 // conversion extended by the identity on the bundling bits (D columns)
    f2::mat us, ud;               // block-local bases (n columns each, low k = unit vectors) on the source / destination side
    f2::mat q, qinv;              // Q = Ud^-1 P Us and its inverse (n x n)
    f2::mat comp;                 // unit vectors enumerating the blocks of a tile group
};
ll_status build_blocks(const f2::mat &p, int d, int w, int min_bits, unsigned max_bytes, unsigned pref_bytes, BlockGeom *out);
// Distinct 128-byte lines touched by one wave-wide access of 16-byte vectors whose element offsets are
// XOR combinations of lane_table[0..5] (8 when the 64 vectors are contiguous).
int wave_access_lines(const uint32_t *lane_table, int w);

}  // namespace ll

struct ll_plan {
    ll_plan_desc desc = {};
    ll_options opts = {};         // the options the plan was made with (complete: no field missing)
    int lds_alloc = 0;            // dynamic LDS bytes a launch asks for: the block, raised where that caps the workgroups per CU
    int nvec = 0;                 // 16-byte vectors per thread
    ll::LdsElemArgs lds_elem = {};
    ll::VecArgs vec = {};
    int vec_nvec_bits = 0, vec_tpose = 0, vec_xchg = 0;
    ll::PullArgs pull = {};
    int pull_src_iters = 0, pull_vec_bits = 0, pull_thread_bits = 8;
};

namespace ll {
// Vector-preserving strategies (plan_vec.cpp).  Each returns LL_OK and sets *applied when the
// conversion has the structure the strategy needs; otherwise *applied is false and the plan is
// untouched.
ll_status plan_wave_shuffle(const f2::mat &p, int d, int w, ll_plan *plan, bool *applied);
ll_status plan_lds_vec(const f2::mat &p, int d, int w, ll_plan *plan, bool *applied);
// LDS staging read back with the transposing LDS loads of gfx950 (plan_tr.cpp), 1- and 2-byte elements.
ll_status plan_lds_tr(const f2::mat &p, int d, int w, ll_plan *plan, bool *applied);
// Broadcasting layouts (plan_pull.cpp): A, B surjective, possibly not injective.
ll_status plan_pull(const ll_layout *A, const ll_layout *B, int w, ll_plan *plan);
// Fills *plan; plan->opts must hold the (complete) options before the call.
ll_status plan_convert(const ll_layout *src, const ll_layout *dst, int elem_bytes, ll_plan *plan);
ll_status run_convert(const ll_plan *plan, const void *src, void *dst, long long ntiles, void *stream);
int copy_xcd_chunk_bits(const ll_options &opt);
ll_status describe_gather(const ll_layout *L, int axis, int elem_bytes, const ll_options *opts, ll_gather_desc *out);
ll_status run_gather(const ll_layout *L, int axis, int elem_bytes, const ll_options *opts, const void *in, const int32_t *idx,
                     void *out, long long ntiles, void *stream);
// LDS bytes to ask for so that at most budget / block_bytes workgroups (at least one) share a CU's
// 160 KiB; never less than the workgroup needs, at most 64 KiB.
int lds_alloc_for(unsigned block_bytes, unsigned budget, int lds_bytes);
// log2 of the consecutive blocks one XCD takes (-1: natural order) so that it works through
// `target` bytes at a time.
int xcd_chunk_bits_for(long long target_bytes, long long block_bytes);
}  // namespace ll

// Kernel argument blocks (plain data, passed by value) and host-side launchers.
//
// All index tables hold XOR-combinable offsets: the offset of an element is the XOR of the table
// entries selected by the bits of (block, thread, iteration) indices, because every map involved
// is linear over F2 (paper Sec. 4.2).
#pragma once
#include <cstdint>

#include "../../include/ll.h"

namespace ll {

constexpr int kMaxThreadBits = 10;   // up to 1024 threads per workgroup
constexpr int kMaxIter = 32;         // 16-byte vectors per thread
constexpr int kMaxSub = 16;          // LDS accesses per 16-byte vector (1-byte elements: 16)
constexpr int kMaxCosetBits = 24;
constexpr int kPullMaxSrcIters = 16; // source vectors one thread of the broadcast kernel stages

// LDS-staged conversion with element-wide (or common-vector-wide) LDS accesses
// (paper Sec. 5.4 "Optimal Swizzling"; vector width = the common contiguous elements).
//
// Work decomposition: tiles are bundled in groups of 2^group_bits; the 2^(d+group_bits) elements
// of a group are split into 2^coset_bits blocks of 2^block_bits elements, one block per
// workgroup.  Element offsets below are in ELEMENTS relative to the start of the group; LDS
// offsets are in BYTES.
struct LdsElemArgs {
    const void *src;
    void *dst;
    long long ntiles;
    long long nblocks;
    int d;              // index bits of one tile
    int group_bits;     // log2 tiles per group
    int coset_bits;     // log2 blocks per group
    int thread_bits;    // log2 threads per workgroup
    uint32_t coset_src[kMaxCosetBits], coset_dst[kMaxCosetBits];    // per block-index bit
    uint32_t coset_lds_rd[kMaxCosetBits];                           // per block-index bit: XOR on LDS read addresses
    uint32_t lane_src[kMaxThreadBits], lane_dst[kMaxThreadBits];    // per thread-index bit
    uint32_t iter_src[kMaxIter], iter_dst[kMaxIter];                // per iteration
    uint32_t lds_wr_lane[kMaxThreadBits], lds_rd_lane[kMaxThreadBits];
    uint32_t lds_wr_iter[kMaxIter], lds_rd_iter[kMaxIter];
    uint32_t lds_wr_sub[kMaxSub], lds_rd_sub[kMaxSub];              // per sub-access of a vector
    uint32_t dst_xor;   // affine conversions: constant XORed onto every destination element index
    int xcd_chunk;      // log2 of the consecutive blocks one XCD takes, -1: natural order (set at launch)
};

// Vector-preserving conversion: every thread keeps whole 16-byte vectors, optionally transposes
// 2^vs x 2^vs element blocks between "position in the vector" and the low iteration bits in
// registers (paper Sec. 5.4 "Intra-thread Data Exchange", Sec. 5.3 "Generalized Vectorization"),
// and exchanges vectors either not at all, by lane <-> register butterfly stages inside the wave
// (Sec. 5.4 "Intra-warp Data Exchange"), or through XOR-swizzled LDS with 128-bit accesses
// (Sec. 5.4 "Optimal Swizzling" with the full vector as the common run).
struct VecArgs {
    const void *src;
    void *dst;
    long long ntiles;
    long long nblocks;
    int d, group_bits, coset_bits, thread_bits;
    uint32_t coset_src[kMaxCosetBits], coset_dst[kMaxCosetBits], coset_lds_rd[kMaxCosetBits];
    uint32_t lane_src[kMaxThreadBits], lane_dst[kMaxThreadBits];
    uint32_t iter_src[kMaxIter], iter_dst[kMaxIter];
    uint32_t stage_mask[5];       // per iteration bit: lane XOR mask of the butterfly stage (0 = none)
    uint32_t lds_wr_lane[kMaxThreadBits], lds_rd_lane[kMaxThreadBits];
    uint32_t lds_wr_iter[kMaxIter], lds_rd_iter[kMaxIter];
    uint32_t dst_xor;   // affine conversions: constant XORed onto every destination element index
    int xcd_chunk;      // log2 of the consecutive blocks one XCD takes, -1: natural order (set at launch)
};

// Conversion between layouts with broadcasting (paper Sec. 5.1 "Broadcasting", Sec. 5.4 rule 2):
// every destination unit pulls the value of its logical element from the canonical source unit.
// A workgroup stages the source runs that hold the elements of one destination block in LDS and
// then assembles the block's destination vectors from them; several destination elements may read
// the same LDS word.  Offsets in elements relative to the group start; LDS offsets in bytes.
struct PullArgs {
    const void *src;
    void *dst;
    long long ntiles;
    long long nblocks;
    int d_src, d_dst;           // index bits of one source / destination tile
    int group_bits, coset_bits;
    int src_vec_bits;           // log2 of the 16-byte vectors staged per block
    int dst_iters;              // destination vectors per thread
    uint32_t coset_src[kMaxCosetBits], coset_dst[kMaxCosetBits], coset_lds_rd[kMaxCosetBits];
    uint32_t lane_src[8], lane_dst[8];
    uint32_t iter_src[kMaxIter];
    uint32_t iter_dst_bit[8];                       // per bit of the destination iteration index
    uint32_t lds_wr_lane[8], lds_rd_lane[8];
    uint32_t lds_wr_iter[kMaxIter], lds_rd_iter_bit[8];
    uint32_t lds_wr_sub[kMaxSub], lds_rd_sub[kMaxSub];
    uint32_t src_xor, lds_rd_xor;   // affine layouts: constant on every source index (vector part / in-vector part via LDS)
    int xcd_chunk;      // log2 of the consecutive blocks one XCD takes, -1: natural order (set at launch)
};

enum { kTposeNone = 0, kTposeBefore = 1, kTposeAfter = 2 };
enum { kXchgNone = 0, kXchgShuffle = 1, kXchgLds = 2 };

// Wave-local gather (paper Sec. 5.5): one kernel wave per layout wave; lane = layout lane.
struct GatherArgs {
    const void *in;
    const int32_t *idx;
    void *out;
    long long nchunks;        // number of (tile, wave) chunks = ntiles * 2^nwave
    int nreg;                 // register bits of the layout
    uint32_t axis_mask;       // (axis length - 1)
    int fast;                 // 1: source lane = (lane & keep_mask) | ((idx & axis_mask) << shift)
    uint32_t keep_mask;
    int shift;
    // general form: source lane = lane ^ XOR_b [bit b of (idx ^ own)] * lane_delta[b], where own
    // is the element's own axis coordinate = own_lane(lane) ^ own_reg[r] ^ own_wave(chunk)
    uint32_t lane_delta[6];
    uint32_t own_lane[6];     // per lane bit: axis coordinate contribution
    uint32_t own_reg[64];     // per register: axis coordinate contribution
    uint32_t own_wave[16];    // per wave-index bit
    uint32_t own_regbit[6];   // per register bit (own_reg is linear: own_reg[r] = XOR of these)
    int nwave;
    uint32_t own_const;       // affine layouts: constant part of every element's axis coordinate
    int xcd_chunk;            // log2 of the consecutive workgroups' worth of chunks one XCD takes, -1: natural order
    int staged;               // 0: lane = layout lane from the start (a lane's elements are one global access);
                              // 1: coalesced 16-byte pieces, source rows staged in wave-private LDS;
                              // 2: coalesced 16-byte pieces, lane <-> register butterflies, then as 0
};

// General gather (paper Sec. 5.5 extended): the axis may occupy register, lane and wave bits.  A
// workgroup stages a block of 2^block_bits consecutive image elements (a block that is closed
// under moves along the axis) in LDS and reads every output element's source from there.
constexpr int kMaxAxisBits = 30;
struct GatherGenArgs {
    const void *in;
    const int32_t *idx;
    void *out;
    long long nblocks;
    long long ntiles;
    long long total_elems;               // ntiles * 2^d
    int d;                               // index bits of one tile
    int group_bits;                      // staged kernel: log2 tiles bundled into a group
    int coset_bits;                      // staged kernel: log2 blocks per group
    int block_bits;                      // log2 elements per block (staged: dimension of the block's subspace;
                                         // memory-direct: the aligned range a source lies in)
    int na;                              // axis bits
    uint32_t axis_mask;
    uint32_t delta[kMaxAxisBits];        // per axis bit: XOR on the block-local index (staged) / the element index (memory-direct)
    uint32_t embed[32];                  // staged: group-relative element offset of block-local bit j (1 << j inside a run)
    uint32_t coset[kMaxCosetBits];       // staged: group-relative element offset per block-index bit
    uint32_t own_bit[32];                // axis coordinate contribution per block-local bit (staged) / element-index bit
    uint32_t own_coset[kMaxCosetBits];   // staged: ... per block-index bit
    uint32_t own_const;                  // affine layouts: constant part of every element's axis coordinate
    int xcd_chunk;                       // log2 of the consecutive blocks one XCD takes, -1: natural order
    int swz_shift, swz_to;               // LDS byte address ^= ((address >> swz_shift) & swz_mask) << swz_to
    uint32_t swz_mask;
    int field_shift;                     // chunk-walking kernel: >= 0 when the axis coordinate is the bit field [field_shift, field_shift + na)
                                         // of the element index itself (a row-major tile, a blocked layout), else -1;
                                         // staged kernel: >= 0 when the LDS byte offset of a move is (coordinate difference) << field_shift
};

// Work geometry of the gather kernels, shared by the kernels and by the host code that sizes their grids.
constexpr int kGlobalPasses = 4;                      // memory-direct kernel: passes of 256 units per workgroup
constexpr int kPhasedThreadBits = 10;                 // chunk-walking kernel: 1024 threads,
constexpr int kPhasedUnits = 8;                       //   8 units per thread,
constexpr int kPhasedChunkBytes = 128 * 1024;         //   the aligned range staged 128 KiB at a time
// log2 threads measured best for a block staged by the workgroup-staged kernel (see launch_gather_general_w)
inline int gather_general_thread_bits(long long block_bytes, int elem_bytes)
{
    return block_bytes >= 32 * 1024 ? 10 : (block_bytes >= 16 * 1024 || (elem_bytes == 1 && block_bytes >= 8 * 1024)) ? 9 : 8;
}
// log2 elements one workgroup takes: units of 4 elements (2 of 8 bytes) x 256 threads x 4 passes / x 1024 threads x 8 units
inline int gather_global_chunk_bits(int elem_bytes) { return (elem_bytes == 8 ? 1 : 2) + 8 + 2; }
inline int gather_phased_chunk_bits(int elem_bytes) { return (elem_bytes == 8 ? 1 : 2) + kPhasedThreadBits + 3; }
inline int gather_phased_lds_chunk_bytes() { return kPhasedChunkBytes; }
ll_status launch_gather_general(const GatherGenArgs &a, int elem_bytes, int thread_bits, int lds_alloc, void *stream);
ll_status launch_gather_global(const GatherGenArgs &a, int elem_bytes, void *stream);
ll_status launch_gather_phased(const GatherGenArgs &a, int elem_bytes, void *stream);
ll_status launch_lds_elem(const LdsElemArgs &a, int elem_bytes, int nvec, int lds_vec_bits, int threads,
                          int lds_bytes, void *stream);
ll_status launch_vec(const VecArgs &a, int elem_bytes, int nvec_bits, int tpose, int xchg, int threads, int lds_bytes,
                     void *stream);
ll_status launch_lds_tr(const LdsElemArgs &a, int elem_bytes, int nvec, int lds_bytes, void *stream);
ll_status launch_pull(const PullArgs &a, int elem_bytes, int src_iters, int vec_bits, int thread_bits, int lds_bytes, void *stream);
ll_status launch_gather(const GatherArgs &a, int elem_bytes, int waves, int lds_alloc, void *stream);
ll_status launch_copy(const void *src, void *dst, long long bytes, int xcd_chunk_bits, void *stream);

}  // namespace ll

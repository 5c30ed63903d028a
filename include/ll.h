/*
 * ll.h - C ABI of the MI355X-native Linear-Layouts library (arXiv 2505.23819).
 *
 * A linear layout is a linear map over F2 between labeled bit spaces
 * (paper Sec. 4.2, Def. "Linear Layouts").  Its matrix is stored by COLUMNS:
 * bases[k] is the image of input bit k.  Input bits are the concatenation of
 * the input dimensions in canonical order register, lane, wave[, tile] (or a
 * single `offset` dimension for memory layouts), least-significant bit first
 * (Sec. 4.1, Layout A and its footnote).  An image is a FLATTENED output
 * index: the LAST output dimension occupies the lowest bits (it is the fastest
 * moving one, Sec. 4.1: w_0:3 = j, w_4:7 = i).
 *
 * Images.  A tensor tile held "under layout L" is an array indexed by the
 * hardware index h = reg | lane << nreg | wave << (nreg + nlane): element h of
 * tile t is stored at buf[t * 2^d + h] and is the logical element L(h).
 * A row-major logical tile is the special case L = identity on flattened bits.
 *
 * Ownership and threading.  ll_layout and ll_plan objects are allocated by the
 * library, immutable after creation, usable from any thread, and released with
 * the matching destroy call.  Device buffers belong to the caller, must be
 * 16-byte aligned, must not overlap each other, and hold ntiles * 2^d elements.
 * `hip_stream` is the caller's hipStream_t (NULL = the default stream).  The
 * device entry points only enqueue work on that stream: they never
 * synchronize, never allocate device memory and never touch the host copy of
 * the data.  There is NO host fallback: without a usable HIP device the device
 * entry points return LL_ERR_DEVICE.
 *
 * Errors.  Every call returns an ll_status; argument errors are detected on
 * the host before anything is launched.  ll_last_error() returns a
 * thread-local, human-readable description of the last failure on this thread.
 */
#ifndef LL_H_
#define LL_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LL_OK = 0,
    LL_ERR_INVALID_ARG = 1,      /* null pointer, size out of range, bad label order, misaligned buffer */
    LL_ERR_DIM_MISMATCH = 2,     /* input/output spaces of the operands do not match */
    LL_ERR_NOT_SURJECTIVE = 3,   /* a right inverse was requested of a non-surjective layout */
    LL_ERR_NOT_INJECTIVE = 4,    /* the operation needs an injective layout */
    LL_ERR_TILE_MIXED = 5,       /* the conversion would move data between tiles */
    LL_ERR_AXIS_NOT_IN_WAVE = 6, /* gather axis is not contained in one wave (Sec. 5.5); kept for ABI stability,
                                    no longer returned: see ll_gather */
    LL_ERR_UNSUPPORTED = 7,      /* valid request outside what is implemented */
    LL_ERR_DEVICE = 8,           /* a HIP call failed; see ll_last_error() */
    LL_ERR_NOT_DIVISIBLE = 9     /* the layout does not have the tile as a left factor (Def. "Left Division") */
} ll_status;

typedef enum { LL_IN_REG = 0, LL_IN_LANE = 1, LL_IN_WAVE = 2, LL_IN_TILE = 3, LL_IN_OFFSET = 4 } ll_in_label;

typedef struct { int32_t label; int32_t nbits; } ll_in_dim;   /* canonical order: labels strictly ascending */
typedef struct { int32_t nbits; } ll_out_dim;                 /* logical dims, slowest first */

typedef struct ll_layout ll_layout;   /* opaque */
typedef struct ll_plan ll_plan;       /* opaque */

#define LL_MAX_IN_DIMS 5
#define LL_MAX_OUT_DIMS 8
#define LL_MAX_BITS 30                /* input and output bits of a layout */
#define LL_WAVE_LANE_BITS 6           /* wave64 */

/* ---- host-side F2 algebra (paper Sec. 4.2) ----------------------------------------------- */

/* Build a layout from its basis vectors (matrix columns, Sec. 4.1 / 4.2).  `bases` holds
 * sum(in_dims[].nbits) values, each < 2^sum(out_dims[].nbits).  The new layout is returned
 * through *out.  Any linear map is accepted here (surjectivity / injectivity are checked by the
 * calls that need them). */
ll_status ll_layout_create(const ll_in_dim *in_dims, int n_in, const ll_out_dim *out_dims, int n_out,
                           const uint64_t *bases, ll_layout **out);
ll_status ll_layout_destroy(ll_layout *layout);

/* Read a layout back.  Any output pointer may be NULL.  in_dims / out_dims / bases must have room
 * for LL_MAX_IN_DIMS / LL_MAX_OUT_DIMS / LL_MAX_BITS entries. */
ll_status ll_layout_get(const ll_layout *layout, int *n_in, ll_in_dim *in_dims, int *n_out,
                        ll_out_dim *out_dims, uint64_t *bases);

/* y = L x over F2: XOR of the columns selected by the set bits of in_index (Sec. 4.1). Host only. */
ll_status ll_layout_apply(const ll_layout *layout, uint64_t in_index, uint64_t *out_index);

/* Composition outer o inner (Def. "Composition"): the matrix product over F2.  The output space
 * of `inner` must have as many bits as the input space of `outer`.  The result maps the input
 * dims of `inner` to the output dims of `outer`. */
ll_status ll_compose(const ll_layout *outer, const ll_layout *inner, ll_layout **out);

/* Product L1 x L2 (Def. "Product"): the block-diagonal layout acting on the concatenated inputs.
 * Input dims are merged label-wise (bits of `a` below bits of `b` inside one label); the output
 * dims of `b` are placed above (slower than) those of `a` in the flattened index. */
ll_status ll_product(const ll_layout *a, const ll_layout *b, ll_layout **out);

/* Product taken label-wise on BOTH sides (Def. "Product" as used for tiling, Sec. 5.1
 * "Broadcasting"): a and b must have the same number of logical dims; inside every input label
 * and inside every logical dim the bits of `a` sit below the bits of `b`.  Layout A of Sec. 4.1 is
 * (2x2 registers) x (4x8 threads) x (2x1 warps) in this sense.  LL_ERR_DIM_MISMATCH if the numbers
 * of logical dims differ. */
ll_status ll_product_dimwise(const ll_layout *a, const ll_layout *b, ll_layout **out);

/* Left division (Def. "Left Division"; Sec. 5.3: an instruction with tile T can lower a layout L
 * if L / T exists).  Succeeds when layout = ll_product_dimwise(tile, Q) for some Q, which is
 * returned: the tile must own the low input bits of each of its labels and the low bits of every
 * logical dim, those inputs must map exactly as the tile does, and no other input may reach the
 * tile's bits.  Q keeps the layout's input labels (possibly with zero bits).
 * LL_ERR_NOT_DIVISIBLE otherwise (ll_last_error() names the first column that breaks the
 * structure); LL_ERR_DIM_MISMATCH if the numbers of logical dims differ. */
ll_status ll_divide_left(const ll_layout *layout, const ll_layout *tile, ll_layout **out);

/* Generalized vectorization (Sec. 5.3): like ll_divide_left, but the input bits of `label` may be
 * permuted first.  The tile's columns of that label are processed in order; each takes the first
 * unused input bit that maps as it does.  perm (room for the layout's bits of `label`) receives
 * the order: new bit k = old bit perm[k].  LL_ERR_NOT_DIVISIBLE if no permutation works. */
ll_status ll_divide_left_permuted(const ll_layout *layout, const ll_layout *tile, int label, int32_t *perm,
                                  ll_layout **out);

/* Contiguous elements per thread (Sec. 5.1 "Contiguous elements"): the largest 2^u such that the
 * inverse of the layout maps logical elements 0..2^u-1 by the identity onto registers 0..2^u-1,
 * i.e. the widest vector one thread can load or store.  1 if the layout has no register bits. */
ll_status ll_contiguity(const ll_layout *layout, int32_t *elems);

/* ---- layout families (paper Sec. 4.3, appendix) --------------------------------------------- */

/* id_k^{label, dim} (appendix "Notation"): the first k bits of input `label` map identically onto
 * the first k bits of logical dim `dim` (dims numbered slowest first) of an n_dims-dim tensor whose
 * other dims have no bits.  Building block for ll_product_dimwise. */
ll_status ll_layout_identity(int label, int dim, int k, int n_dims, ll_layout **out);

/* Blocked layout (Proposition "Blocked layouts are linear layouts"): reg_bits / lane_bits /
 * wave_bits give, per dim, the log2 number of registers, lanes and waves along it; order[i] is the
 * i-th fastest dim.  The result is id_R^o x id_T^o x id_W^o; dim k has reg + lane + wave bits. */
ll_status ll_layout_blocked(int n_dims, const int32_t *reg_bits, const int32_t *lane_bits, const int32_t *wave_bits,
                            const int32_t *order, ll_layout **out);

/* Result tile of a CDNA matrix instruction with a 16x16 (m_bits 4) or 32x32 (m_bits 5) fp32
 * accumulator on 64 lanes, as the product id_2^{reg,0} x id_m^{lane,1} x id_{6-m}^{lane,0} x
 * id_{2m-8}^{reg,0} (the pattern of the appendix's proof for `mma`): a lane holds groups of 4
 * consecutive rows of one column.  Multiply by further identities (ll_product_dimwise) to cover
 * a larger tensor with registers or waves. */
ll_status ll_layout_mfma_accumulator(int m_bits, ll_layout **out);

/* Left-operand tile (2^m_bits rows x K) of the same instructions: a lane holds 2^k_reg_bits
 * consecutive elements along K of one row: id_kr^{reg,1} x id_m^{lane,0} x id_{6-m}^{lane,1}. */
ll_status ll_layout_mfma_operand(int m_bits, int k_reg_bits, ll_layout **out);

/* The legacy `mma` swizzle (Def. "mma swizzling") for a row-major 2^m_bits x 2^n_bits tensor as a
 * memory layout (input label `offset`, logical dims (i, j)), built from the closed form of
 * Sec. 4.3: [[I_n, C], [0, I_m]] with c_i = (vec * ((2^i / per_phase) mod max_phase)) mod 2^n.
 * vec_elems, per_phase, max_phase: powers of two with vec_elems * max_phase <= 2^n_bits. */
ll_status ll_layout_mma_swizzle(int m_bits, int n_bits, int vec_elems, int per_phase, int max_phase, ll_layout **out);

/* Family tests: OR of the flags below.  DISTRIBUTED: Def. "Distributed Layout" (surjective, every
 * column zero or a unit vector, no unit vector twice; register / lane / wave / tile inputs).
 * MEMORY: Def. "Memory Layout" (invertible, every column has one or two non-zero bits). */
#define LL_LAYOUT_SURJECTIVE 1u
#define LL_LAYOUT_INJECTIVE 2u
#define LL_LAYOUT_DISTRIBUTED 4u
#define LL_LAYOUT_MEMORY 8u
ll_status ll_layout_classify(const ll_layout *layout, uint32_t *flags);

/* Sliced layout (Sec. 4.3 "Sliced Layouts"): the layout of the result of a reduction along logical
 * dim `dim` (numbered slowest first).  The rows of that dim are removed from the matrix: inputs keep
 * their labels and sizes, columns that ran along the dim become zero (the result is replicated over
 * them), an affine constant loses the same bits.  The layout must have at least two logical dims.
 * A surjective layout stays surjective; ll_plan_convert treats the zero columns as broadcasting. */
ll_status ll_layout_slice(const ll_layout *layout, int dim, ll_layout **out);

/* Affine layouts (Conclusions: flips and slices are y = A x xor b).  A copy of `layout` in which
 * index h holds the logical element (A h) xor offset; offset < 2^(output bits).  For a dim of 2^n
 * elements, offset = all ones of that dim flips it, offset = its top bit rolls it by half.
 * ll_layout_apply, ll_compose and ll_invert carry the offset along; ll_plan_convert and ll_gather
 * accept affine layouts; products combine the constants of their factors dim by dim, a division
 * needs the layout's constant to contain the tile's (LL_ERR_NOT_DIVISIBLE otherwise) and gives the
 * quotient the rest; ll_contiguity counts the run that starts at register 0's element. */
ll_status ll_layout_with_offset(const ll_layout *layout, uint64_t offset, ll_layout **out);
ll_status ll_layout_get_offset(const ll_layout *layout, uint64_t *offset);

/* Right inverse (Def. "Right Inverse") by Gaussian elimination over F2.  L must be surjective,
 * else LL_ERR_NOT_SURJECTIVE.  If L is not injective the free variables are set to zero, with
 * input columns taken as pivots in order (register bits first).  The result maps one `offset`
 * input dim of d_out bits to one output dim of d_in bits (the flattened hardware index). */
ll_status ll_invert(const ll_layout *layout, ll_layout **out);

/* ---- options ------------------------------------------------------------------------------- */

/* Explicit kernel selection and tuning for ll_plan_convert_opts / ll_gather_opts / ll_gather_info_opts.
 * For callers that want a particular kernel (tests, benchmarks comparing the exchange paths) or
 * that retune for a workload; nothing here changes a result.  Every field is an int32; LL_AUTO
 * (-1) leaves the decision to the library.  An ll_options is plain data owned by the caller, read
 * during the call only, and safe to share between threads.  ll_options_init sets every field to
 * LL_AUTO; ll_options_from_env additionally takes overrides from LL_* environment variables (one
 * per field, upper-case field name, e.g. LL_XCD_CHUNK) and is meant for experiments.  The calls
 * without options behave as with a NULL pointer: they use the process defaults, which are
 * ll_options_from_env evaluated ONCE, at the first call that needs them. */
#define LL_AUTO (-1)
typedef struct {
    int32_t size;                  /* sizeof(ll_options), set by ll_options_init / ll_options_from_env */
    /* kernel selection */
    int32_t strategy;              /* conversions: LL_STRATEGY_LDS_ELEM: element-wide LDS staging (always applicable);
                                      LL_STRATEGY_LDS_VEC: skip the register / shuffle planner, i.e. 128-bit LDS staging where it
                                      applies, else element-wide; LL_STRATEGY_LDS_TR: transposing LDS loads where they apply,
                                      else as LL_AUTO.  ll_plan_info reports the kernel actually planned. */
    int32_t gather_kernel;         /* gathers: LL_GATHER_SHUFFLE / LL_GATHER_SHUFFLE_ROWS / LL_GATHER_WAVE_STAGED (taken when the
                                      axis moves lane bits only and the bytes per lane suit the kernel),
                                      LL_GATHER_BLOCK_STAGED (taken whenever a closed block fits LDS); otherwise as LL_AUTO.
                                      ll_gather_info_opts reports the choice. */
    /* conversion tuning (bytes are powers of two) */
    int32_t block_bytes;           /* largest block of the element-wide LDS kernels */
    int32_t pref_bytes;            /* size small tiles are bundled up to */
    int32_t elem_threads_log2;     /* threads per workgroup of the element-wide LDS kernel: 6 (one wave), 8, 9 or 10 */
    int32_t vec_block_bytes;       /* largest block of the 128-bit LDS kernel */
    int32_t vec_threads;           /* its threads per workgroup: 64, 128 or 256 */
    int32_t shuffle_block_bytes;   /* block of the register / shuffle kernel: 4096 or 8192 */
    int32_t inflight_bytes;        /* bytes a CU may have in flight: resident workgroups are capped through their LDS share */
    int32_t lds_pad_bytes;         /* extra LDS per workgroup of the 256-thread element-wide kernel (lowers occupancy) */
    int32_t xcd_chunk;             /* consecutive blocks each of the 8 XCDs takes at a time (power of two); 0: natural order */
    int32_t pull_mode;             /* broadcasting plans: 0 balanced, 1 destination runs first, 2 source runs first */
    int32_t pull_vec_bits;         /* log2 elements per LDS access of the broadcast kernel (upper bound) */
    int32_t pull_inflight_bytes;   /* as inflight_bytes, counted in destination bytes of the broadcast kernel's blocks */
    int32_t pull_xcd_chunk;        /* as xcd_chunk */
    /* gather tuning */
    int32_t gather_block_bytes;    /* preferred block of the workgroup-staged kernel */
    int32_t gather_lds_max_bytes;  /* largest block it may stage */
    int32_t gather_min_run_bytes;  /* shortest contiguous run a staged block may be made of */
    int32_t gather_phased_max_bytes; /* largest aligned range walked through LDS in chunks */
    int32_t gather_threads_log2;   /* threads per workgroup of the workgroup-staged kernel: 8, 9 or 10 */
    int32_t gather_inflight_bytes; /* as inflight_bytes: bytes of `in` and `idx` loads (wave-level kernels) or of staged blocks */
    int32_t gather_xcd_chunk;      /* as xcd_chunk, in chunks of one wave (wave-level kernels) or blocks */
    int32_t gather_swizzle_always; /* 1: swizzle the staged block even when no move along the axis changes bank bits */
    int32_t copy_xcd_chunk;        /* ll_copy (process defaults only) */
    int32_t debug;                 /* 1: planners say on stderr why a strategy did not apply */
    int32_t gather_waves;          /* waves per workgroup of the wave-level gather kernels (one chunk each): 1, 2 or 4 */
    int32_t pull_threads_log2;     /* threads per workgroup of the broadcast kernel: 6 (one wave) or 8 */
} ll_options;

ll_status ll_options_init(ll_options *opts);
ll_status ll_options_from_env(ll_options *opts);

/* ---- conversion (paper Sec. 5.4) ------------------------------------------------------- */

typedef enum {
    LL_KIND_NOOP = 0,        /* B^-1 o A is the identity */
    LL_KIND_REG_ONLY = 1,    /* only register bits move ("intra-thread data exchange") */
    LL_KIND_INTRA_WAVE = 2,  /* the wave part of B^-1 o A is the identity ("intra-warp") */
    LL_KIND_LDS = 3,         /* data crosses waves: staged through shared memory (LDS) */
    LL_KIND_BROADCAST = 4    /* a layout is not injective (Sec. 5.1 "Broadcasting", Sec. 5.4 rule 2) */
} ll_plan_kind;

typedef enum {
    LL_STRATEGY_COPY = 0,      /* plain 16-byte vector copy */
    LL_STRATEGY_REG_PERMUTE = 1, /* each lane loads whole vectors, permutes them in registers, stores */
    LL_STRATEGY_WAVE_SHUFFLE = 2, /* wave64 exchange by cross-lane shuffles */
    LL_STRATEGY_LDS_ELEM = 3,  /* LDS staging, element-wide (or common-vector-wide) accesses, XOR swizzle */
    LL_STRATEGY_LDS_VEC = 4,   /* LDS staging with in-register transposes and 128-bit LDS accesses */
    LL_STRATEGY_LDS_PULL = 5,  /* broadcasting layouts: destination units pull from LDS-staged source runs */
    LL_STRATEGY_LDS_TR = 6     /* LDS staging read back with transposing LDS loads (1- and 2-byte elements) */
} ll_strategy;

#define LL_PLAN_MAX_BLOCK_BITS 20

typedef struct {
    int32_t kind;               /* ll_plan_kind: the paper's classification of B^-1 o A */
    int32_t strategy;           /* ll_strategy: the kernel that ll_convert launches */
    int32_t d;                  /* index bits of one (source) tile */
    int32_t d_dst;              /* index bits of one destination tile (= d unless a layout broadcasts) */
    int32_t elem_bytes;
    uint64_t conv[LL_MAX_BITS]; /* columns of B^-1 o A on the d hardware-index bits (bijective layouts) */
    uint64_t conv_offset;       /* affine layouts: destination index = conv * h xor conv_offset
                                 * (broadcasting plans: source index = pull * hB xor conv_offset) */
    uint64_t pull[LL_MAX_BITS]; /* broadcasting layouts: columns of A^+ o B, destination index -> source index */
    int32_t global_vec_bytes;   /* width of every global load and store */
    int32_t src_lines_per_access; /* distinct 128-byte lines one wave-wide load (64 x 16 bytes) touches; 8 = fully coalesced */
    int32_t dst_lines_per_access; /* the same for one wave-wide store */
    int32_t lds_write_bytes;    /* width of one LDS write (0 if LDS unused) */
    int32_t lds_read_bytes;     /* width of one LDS read  (0 if LDS unused) */
    int32_t lds_bytes;          /* LDS bytes per workgroup */
    int32_t threads;            /* threads per workgroup */
    int32_t vectors_per_thread;
    int32_t block_bits;         /* log2 elements staged per workgroup iteration */
    int32_t group_bits;         /* log2 tiles that share one block (small tiles) */
    int32_t segment_bits;       /* log2 elements of the contiguous runs a block reads and writes */
    int32_t shuffle_rounds;     /* cross-lane exchange stages (WAVE_SHUFFLE) */
    int32_t register_transpose; /* 0: none; 1 / 2: in-register transpose before / after the exchange */
    /* LDS layout of one block, as linear layouts on block_bits bits over a common "block-local"
     * logical space (paper Sec. 5.4 "Optimal Swizzling"): lds_mem maps an LDS element offset to
     * a block-local index; lds_write / lds_read map (register, lane, wave) of the writing /
     * reading instruction to the same space, with lds_*_reg_bits register bits first, then
     * LL_WAVE_LANE_BITS lane bits, then wave bits. */
    uint64_t lds_mem[LL_PLAN_MAX_BLOCK_BITS];
    uint64_t lds_write[LL_PLAN_MAX_BLOCK_BITS];
    uint64_t lds_read[LL_PLAN_MAX_BLOCK_BITS];
    int32_t lds_write_reg_bits, lds_read_reg_bits;
    int32_t lds_vec_bits;       /* log2 elements per LDS access */
    int32_t lds_banks;          /* hardware model used by the synthesizer: 4-byte banks a read phase spans */
    int32_t lds_banks_write;    /* ... and a write phase */
    int32_t lds_phase_lanes_write, lds_phase_lanes_read; /* lanes served together */
    int32_t predicted_wavefronts_write, predicted_wavefronts_read; /* per access phase; 1 = conflict free */
    /* The shuffle schedule of Sec. 5.4 "Intra-warp Data Exchange", computed on the layouts' own
     * lanes when both are distributed layouts (Def. "Distributed Layout") and the wave part of
     * B^-1 o A is the identity; vectors are flattened logical indices.  V: common register vectors
     * that fit one 32-bit shuffle; I = A_lane n B_lane; G = {e_i ^ f_i} with E = A_lane \ I and
     * F = B_lane \ I in ascending order; R completes V u I u G (and the wave images) to a basis:
     * the exchange takes 2^sched_nr rounds, one shuffle per lane and round.  Reported for
     * reference and tests; the kernels use lane <-> register butterfly stages instead (see
     * shuffle_rounds). */
    int32_t sched_valid, sched_nv, sched_ni, sched_ng, sched_nr;
    uint64_t sched_v[2], sched_i[8], sched_g[8], sched_r[LL_MAX_BITS];
} ll_plan_desc;

/* Plan the conversion of images under `src` into images under `dst` (both map register / lane /
 * wave [/ tile] inputs onto output spaces of equal size).  Computes B^-1 o A (Sec. 5.4),
 * classifies it (intra-thread / intra-warp / shared memory), and picks the kernel, its vector
 * widths and, for LDS paths, the XOR swizzle.  elem_bytes is 1, 2, 4 or 8.
 * Either side may instead be a memory layout (one `offset` input dim, Sec. 4.3: unswizzled,
 * ll_layout_mma_swizzle, ...): its image is the buffer indexed by memory offset, and the plan is
 * the register <-> memory mapping of Sec. 5.3; the input bit counts must match and no tile label
 * may be present.
 * Both layouts must be surjective (LL_ERR_NOT_SURJECTIVE otherwise).  If both are bijective they
 * must have the same number of input bits and the same `tile` bits (LL_ERR_DIM_MISMATCH), and the
 * tile bits must map identically in both (LL_ERR_TILE_MIXED); the split of the remaining bits over
 * registers, lanes and waves may differ (the images are flat per tile; such a plan is classified
 * as a shared-memory conversion, since the register / lane classes do not line up).  If a layout is not injective (broadcasting:
 * zero or dependent columns, Sec. 5.1) the two may have different input dims; the plan then
 * pulls every destination unit's logical element from the source unit given by the right
 * inverse with free variables zero (Sec. 5.4 rule 2), source tiles hold 2^d and destination
 * tiles 2^d_dst elements. */
ll_status ll_plan_convert(const ll_layout *src, const ll_layout *dst, int elem_bytes, ll_plan **out);
/* The same with explicit options (NULL = the process defaults); the plan keeps what it needs of them. */
ll_status ll_plan_convert_opts(const ll_layout *src, const ll_layout *dst, int elem_bytes, const ll_options *opts,
                               ll_plan **out);
ll_status ll_plan_info(const ll_plan *plan, ll_plan_desc *out);
ll_status ll_plan_destroy(ll_plan *plan);

/* Apply a plan: dst_dev[t * 2^d + (B^-1 o A)(h)] = src_dev[t * 2^d + h] for every tile t < ntiles
 * and every h (Sec. 5.4); for broadcasting plans dst_dev[t * 2^d_dst + hB] =
 * src_dev[t * 2^d + (A^+ o B)(hB)].  Pointers are DEVICE pointers, 16-byte aligned, not
 * overlapping; both buffers must hold a whole number of 16-byte vectors (only tiles smaller than
 * 16 bytes can violate that: pass a multiple of 16 / tile bytes tiles).  Asynchronous on
 * hip_stream.  ntiles == 0 is a no-op.  Errors in the arguments are reported before any launch. */
ll_status ll_convert(const ll_plan *plan, const void *src_dev, void *dst_dev, int64_t ntiles, void *hip_stream);

/* ---- gather (paper Sec. 5.5) ----------------------------------------------------------- */

/* out[.., i, ..] = in[.., idx[.., i, ..], ..] along output dim `axis`, where in, idx (int32) and
 * out are images under the same surjective layout L.  Indices are reduced modulo the axis length.
 * L may broadcast (Sec. 5.1; 2^d slots per tile for fewer logical elements): `in` must then be the
 * image of a logical tensor, i.e. all replicas of an element hold the same value (the paper gives no
 * rule for which replica a gather reads, and neither does this library: with unequal replicas the
 * result is one of their values, unspecified which).  Every slot of out is written, from its own slot
 * of idx; replicas of idx may differ.
 * Moving along the axis changes the hardware index by L^-1 (L^+, the right inverse with free
 * variables zero) of the axis bits:
 *  - lane bits only (the paper's condition, Sec. 5.5, with one round): cross-lane shuffles, or
 *    wave-private LDS staging when a lane holds more than 16 bytes;
 *  - register and / or wave bits as well: a block of image elements closed under moves along the axis
 *    (the span of those index changes plus contiguous runs of 128 bytes where the size allows) is
 *    staged in workgroup LDS, at most 128 KiB; if no such block with runs of at least 64 bytes fits,
 *    the aligned power-of-two range around an element that holds all its possible sources is either
 *    walked through LDS in 128 KiB chunks by every workgroup with elements in it (ranges up to
 *    1 MiB), or every element is gathered straight from memory (slower: every element is its own
 *    access).
 *    Sec. 5.5's condition (no wave bits on the axis) is reported by ll_gather_info
 *    (axis_wave_bits == 0) and is not an error here;
 *  - tile bits: LL_ERR_TILE_MIXED.
 * L may also be a memory layout (one `offset` input dim): in, idx and out are then buffers indexed by
 * memory offset (a row-major tensor is the identity memory layout) and every bit counts as a register bit.
 * Pointers are DEVICE pointers.  Asynchronous on hip_stream. */
typedef enum {
    LL_GATHER_SHUFFLE = 0,       /* one ds_bpermute_b32 per 32-bit piece of an element */
    LL_GATHER_WAVE_STAGED = 1,   /* coalesced access, source rows staged in wave-private LDS */
    LL_GATHER_BLOCK_STAGED = 2,  /* general: a block closed under the axis staged in workgroup LDS */
    LL_GATHER_GLOBAL = 3,        /* no closed block fits LDS: element-wide reads from memory */
    LL_GATHER_PHASED = 4,        /* no closed block fits LDS, but the aligned range around an element is a few
                                    LDS sizes: every workgroup walks the range through LDS in 128 KiB chunks */
    LL_GATHER_SHUFFLE_ROWS = 5   /* as LL_GATHER_SHUFFLE for lanes that hold 32 to 256 bytes: global accesses in coalesced
                                    16-byte pieces, converted to and from "one layout row per lane" by lane <-> register
                                    butterflies (ds_bpermute_b32), the gather itself by ds_bpermute_b32 */
} ll_gather_kernel;

typedef struct {
    int32_t kernel;              /* ll_gather_kernel */
    int32_t axis_reg_bits;       /* hardware bits a move along the axis can flip, by label */
    int32_t axis_lane_bits;
    int32_t axis_wave_bits;
    int32_t paper_rounds;        /* 2^axis_reg_bits: the shuffle rounds of Sec. 5.5 (0 for a memory layout) */
    int32_t block_bytes;         /* bytes of `in` one wave (kernels 0, 1) or workgroup (kernel 2) stages; kernel 3:
                                    the aligned range a source lies in (saturates at 2^31 - 1) */
} ll_gather_desc;

/* What ll_gather would do for this layout, axis and element size (same checks and errors). */
ll_status ll_gather_info(const ll_layout *layout, int axis, int elem_bytes, ll_gather_desc *out);

ll_status ll_gather(const ll_layout *layout, int axis, int elem_bytes, const void *in_dev,
                    const int32_t *idx_dev, void *out_dev, int64_t ntiles, void *hip_stream);
/* The same with explicit options (NULL = the process defaults). */
ll_status ll_gather_info_opts(const ll_layout *layout, int axis, int elem_bytes, const ll_options *opts, ll_gather_desc *out);
ll_status ll_gather_opts(const ll_layout *layout, int axis, int elem_bytes, const ll_options *opts, const void *in_dev,
                         const int32_t *idx_dev, void *out_dev, int64_t ntiles, void *hip_stream);

/* ---- misc -------------------------------------------------------------------------------- */

/* Plain 16-byte-vector device copy of `bytes` bytes (a multiple of 16) between buffers that do not
 * overlap: the achievable-bandwidth yardstick the benchmark prints next to each conversion.
 * Asynchronous on hip_stream. */
ll_status ll_copy(const void *src_dev, void *dst_dev, int64_t bytes, void *hip_stream);

const char *ll_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LL_H_ */

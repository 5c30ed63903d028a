// HIP kernels for gfx950 (CDNA4, wave64).  Pure data movement: 16-byte global loads and stores,
// LDS staging or cross-lane shuffles in between, no MFMA.
#include <hip/hip_runtime.h>
#include <atomic>
#include <type_traits>

#include <cstdlib>

#include "../../include/ll.h"
#include "kernels.hpp"
#include "layout.hpp"

namespace ll {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

static __device__ __forceinline__ u32x4 load16(const void *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}
static __device__ __forceinline__ void store16(void *p, u32x4 v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
}

// Raw buffer access (16 bytes per lane) with streaming cache policy.  The descriptor covers
// [base, base + bytes): loads beyond it return zero and stores beyond it are dropped by the
// hardware, which is how ragged tails are handled without branches.
constexpr int kStream = 16 | 2;   // cache-policy bits "sc1 nt": stream through, do not keep in cache
static __device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
static __device__ __forceinline__ u32x4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kStream);
}
static __device__ __forceinline__ void buf_store16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, u32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, kStream);
}

// Affine conversions (y = A x xor b): the destination index of every element carries a constant
// XOR c.  Its bits above the vector move whole vectors (an XOR on the store offset); its low bits
// move elements inside the 16-byte vector: element e goes to position e ^ c_low.
template <int W>
static __device__ __forceinline__ void store_vec_xor(__amdgpu_buffer_rsrc_t r, uint32_t elem_off, u32x4 v, uint32_t c)
{
    constexpr uint32_t kPos = 16u / W - 1u;            // position bits inside a vector
    const uint32_t cl = c & kPos;                       // wave uniform
    if (cl) {
        uint32_t d[4] = {v.x, v.y, v.z, v.w};
        uint32_t dsel;                                  // dword-index bits of cl
        if constexpr (W == 1) {
            if (cl & 1u)
                for (int k = 0; k < 4; ++k) d[k] = ((d[k] & 0x00FF00FFu) << 8) | ((d[k] >> 8) & 0x00FF00FFu);
            if (cl & 2u)
                for (int k = 0; k < 4; ++k) d[k] = (d[k] << 16) | (d[k] >> 16);
            dsel = cl >> 2;
        } else if constexpr (W == 2) {
            if (cl & 1u)
                for (int k = 0; k < 4; ++k) d[k] = (d[k] << 16) | (d[k] >> 16);
            dsel = cl >> 1;
        } else if constexpr (W == 4) {
            dsel = cl;
        } else {
            dsel = cl << 1;
        }
        if (dsel & 1u) { uint32_t t = d[0]; d[0] = d[1]; d[1] = t; t = d[2]; d[2] = d[3]; d[3] = t; }
        if (dsel & 2u) { uint32_t t = d[0]; d[0] = d[2]; d[2] = t; t = d[1]; d[1] = d[3]; d[3] = t; }
        v.x = d[0]; v.y = d[1]; v.z = d[2]; v.w = d[3];
    }
    buf_store16(r, (elem_off ^ (c & ~kPos)) * W, v);
}

// Workgroups are dealt to the 8 XCDs round robin by their index.  With xcd_chunk = c > 0 the block
// a workgroup takes is renumbered so that every XCD works through runs of c consecutive blocks
// (blocks that touch the same DRAM pages then share an L2 and run close in time).  c is a power of
// two, passed as its log2 (-1: off).
static __device__ __forceinline__ long long block_of_workgroup(long long wg, long long nblocks, int xcd_chunk_bits)
{
    if (xcd_chunk_bits < 0) return wg;
    const int span_bits = 3 + xcd_chunk_bits;             // blocks covered by one round over the XCDs
    const long long full = (nblocks >> span_bits) << span_bits;      // the tail keeps its natural order
    if (wg >= full) return wg;
    const uint32_t in = (uint32_t)wg & ((1u << span_bits) - 1u);
    return (wg - in) + ((long long)(in & 7u) << xcd_chunk_bits) + (in >> 3);
}

// Launches go through hipLaunchKernel, whose return value is the status of THIS launch.  (The
// thread's "last error" is shared with every other user of the runtime in the process: an error
// left behind by someone else's call would otherwise be reported as ours.)
static thread_local hipError_t g_launch_status = hipSuccess;

template <typename... P, typename... A>
static void launch(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, A &&...args)
{
    auto with_params = [&](P... p) {
        void *ptrs[] = {static_cast<void *>(&p)...};
        return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds_bytes, stream);
    };
    g_launch_status = with_params(static_cast<P>(args)...);
}

static ll_status check_launch(const char *what)
{
    if (g_launch_status != hipSuccess) return fail(LL_ERR_DEVICE, "%s: %s", what, hipGetErrorString(g_launch_status));
    return LL_OK;
}

// A kernel that wants more than 64 KiB of dynamic LDS must be told so once per device
// (hipFuncSetAttribute); `done` is the per-kernel record of the devices that have been (one bit per
// device ordinal; ordinals beyond 63 simply set the attribute on every call).
static ll_status allow_large_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(LL_ERR_DEVICE, "hipGetDevice failed");
    const uint64_t bit = dev >= 0 && dev < 64 ? 1ull << dev : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return LL_OK;
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return fail(LL_ERR_DEVICE, "hipFuncSetAttribute: %s", hipGetErrorString(e));
    if (bit) done.fetch_or(bit, std::memory_order_release);
    return LL_OK;
}

// ---------------------------------------------------------------------------------------------
// plain copy (bandwidth yardstick, and the NOOP conversion)
// ---------------------------------------------------------------------------------------------

// One 16-byte vector per thread with the streaming cache policy: the fastest plain copy found on
// MI355X (many short-lived waves; about 32 KiB in flight per CU).
constexpr int kCopyVec = 1;

__global__ __launch_bounds__(256) void k_copy(const void *__restrict__ src, void *__restrict__ dst, long long nvec,
                                              long long nblocks, int xcd_chunk)
{
    // descriptors cover this workgroup's 4 KiB (or the tail): out-of-range lanes do nothing
    const long long first = block_of_workgroup((long long)blockIdx.x, nblocks, xcd_chunk) * 256;
    const long long left = nvec - first;
    const uint32_t bytes = (uint32_t)(left >= 256 ? 256 : left) * 16u;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(static_cast<const unsigned char *>(src) + first * 16, bytes);
    const __amdgpu_buffer_rsrc_t rd = make_rsrc(static_cast<unsigned char *>(dst) + first * 16, bytes);
    buf_store16(rd, threadIdx.x * 16, buf_load16(rs, threadIdx.x * 16));
}

ll_status launch_copy(const void *src, void *dst, long long bytes, int xcd_chunk_bits, void *stream)
{
    const long long nvec = bytes / 16;
    const long long per = kCopyVec * 256;
    const long long grid = (nvec + per - 1) / per;
    if (grid > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "copy of %lld bytes is too large for one launch", bytes);
    launch(k_copy, dim3((unsigned)grid), dim3(256), 0, static_cast<hipStream_t>(stream), src, dst, nvec, grid, xcd_chunk_bits);
    return check_launch("copy kernel launch");
}

// ---------------------------------------------------------------------------------------------
// LDS-staged conversion, element-wide LDS accesses (paper Sec. 5.4, shared-memory path)
// ---------------------------------------------------------------------------------------------

template <int AB>
static __device__ __forceinline__ void lds_put(unsigned char *lds, uint32_t addr, const uint32_t (&r)[4], int s)
{
    if constexpr (AB == 16) {
        u32x4 v = {r[0], r[1], r[2], r[3]};
        *reinterpret_cast<u32x4 *>(lds + addr) = v;
    } else if constexpr (AB == 8) {
        u32x2 v = {r[2 * s], r[2 * s + 1]};
        *reinterpret_cast<u32x2 *>(lds + addr) = v;
    } else if constexpr (AB == 4) {
        *reinterpret_cast<uint32_t *>(lds + addr) = r[s];
    } else if constexpr (AB == 2) {
        *reinterpret_cast<uint16_t *>(lds + addr) = (uint16_t)(r[s >> 1] >> ((s & 1) * 16));
    } else {
        *reinterpret_cast<uint8_t *>(lds + addr) = (uint8_t)(r[s >> 2] >> ((s & 3) * 8));
    }
}

template <int AB>
static __device__ __forceinline__ void lds_get(const unsigned char *lds, uint32_t addr, uint32_t (&r)[4], int s)
{
    if constexpr (AB == 16) {
        u32x4 v = *reinterpret_cast<const u32x4 *>(lds + addr);
        r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
    } else if constexpr (AB == 8) {
        u32x2 v = *reinterpret_cast<const u32x2 *>(lds + addr);
        r[2 * s] = v.x; r[2 * s + 1] = v.y;
    } else if constexpr (AB == 4) {
        r[s] = *reinterpret_cast<const uint32_t *>(lds + addr);
    } else if constexpr (AB == 2) {
        const uint32_t x = *reinterpret_cast<const uint16_t *>(lds + addr);
        r[s >> 1] = (s & 1) ? (r[s >> 1] | (x << 16)) : x;
    } else {
        const uint32_t x = *reinterpret_cast<const uint8_t *>(lds + addr);
        r[s >> 2] = (s & 3) ? (r[s >> 2] | (x << ((s & 3) * 8))) : x;
    }
}

// W: element bytes, NV: 16-byte vectors per thread, V: log2 elements per LDS access.
// One workgroup of T = 2^TB threads (256 unless the experiment knob says otherwise) stages one block:
// coalesced 16-byte loads (thread t, iteration i takes vector t + T i of the block's source runs), LDS
// writes at swizzled offsets, barrier,
// LDS reads of the elements of its destination vectors, coalesced 16-byte stores.  Every index
// map is linear over F2, so an offset is the XOR of per-bit table entries.
// Read one 8-byte LDS chunk with the transposing load: the address this lane passes is used by
// OTHER lanes of its group of 16 (see plan_tr.cpp for the measured lane behaviour); the result is
// half of this lane's destination vector.
template <int W>
static __device__ __forceinline__ void lds_get_tr(unsigned char *lds, uint32_t addr, uint32_t (&r)[4], int s)
{
    typedef short v4s __attribute__((ext_vector_type(4)));
    typedef int v2i __attribute__((ext_vector_type(2)));
    if constexpr (W == 2) {
        const v4s x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3))) *)(lds + addr));
        const u32x2 y = __builtin_bit_cast(u32x2, x);
        r[2 * s] = y.x; r[2 * s + 1] = y.y;
    } else {
        static_assert(W == 1 || W == 2, "transposing LDS loads exist for 1- and 2-byte elements");
        const v2i x = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)(lds + addr));
        r[2 * s] = (uint32_t)x.x; r[2 * s + 1] = (uint32_t)x.y;
    }
}

// TR = 1: the LDS reads are transposing loads (ds_read_b64_tr_b16 / _tr_b8), V must make the
// access 8 bytes wide; the read tables then hold the addresses a lane supplies for its group.
template <int W, int NV, int V, int TR = 0, int TB = 8>
__global__ __launch_bounds__(1 << TB) void k_lds_elem(const LdsElemArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int VS = (W == 1) ? 4 : (W == 2) ? 3 : (W == 4) ? 2 : 1;
    constexpr int NSUB = 1 << (VS - V);
    constexpr int AB = (1 << V) * W;
    const uint32_t tid = threadIdx.x;

    uint32_t ls = 0, ld = 0, lw = 0, lr = 0;
#pragma unroll
    for (int b = 0; b < TB; ++b) {
        const uint32_t m = 0u - ((tid >> b) & 1u);
        ls ^= a.lane_src[b] & m;
        ld ^= a.lane_dst[b] & m;
        lw ^= a.lds_wr_lane[b] & m;
        lr ^= a.lds_rd_lane[b] & m;
    }
    const long long blk = block_of_workgroup((long long)blockIdx.x, a.nblocks, a.xcd_chunk);
    const long long group = blk >> a.coset_bits;
    const uint32_t c = (uint32_t)(blk & ((1ll << a.coset_bits) - 1));
    uint32_t cs = 0, cd = 0, cr = 0;
    for (int b = 0; b < a.coset_bits; ++b) {
        const uint32_t m = 0u - ((c >> b) & 1u);
        cs ^= a.coset_src[b] & m;
        cd ^= a.coset_dst[b] & m;
        cr ^= a.coset_lds_rd[b] & m;
    }
    const int gshift = a.d + a.group_bits;
    const unsigned char *sbase = static_cast<const unsigned char *>(a.src) + (((size_t)group << gshift) * W);
    unsigned char *dbase = static_cast<unsigned char *>(a.dst) + (((size_t)group << gshift) * W);
    // tiles of this group that exist (the last group may be partly empty): they are a prefix of the
    // group, and the buffer descriptors end there
    const long long left = a.ntiles - (group << a.group_bits);
    const uint32_t tiles_here = left > (1ll << a.group_bits) ? (1u << a.group_bits) : (uint32_t)left;
    const uint32_t valid_bytes = (tiles_here << a.d) * W;
    const __amdgpu_buffer_rsrc_t srsrc = make_rsrc(sbase, valid_bytes);
    const __amdgpu_buffer_rsrc_t drsrc = make_rsrc(dbase, valid_bytes);

    uint32_t r[NV][4];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const uint32_t off = cs ^ ls ^ a.iter_src[i];
        const u32x4 v = buf_load16(srsrc, off * W);
        r[i][0] = v.x; r[i][1] = v.y; r[i][2] = v.z; r[i][3] = v.w;
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const uint32_t base = lw ^ a.lds_wr_iter[i];
#pragma unroll
        for (int s = 0; s < NSUB; ++s) lds_put<AB>(lds, base ^ a.lds_wr_sub[s], r[i], s);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const uint32_t base = cr ^ lr ^ a.lds_rd_iter[i];
#pragma unroll
        for (int s = 0; s < NSUB; ++s) {
            if constexpr (TR) lds_get_tr<W>(lds, base ^ a.lds_rd_sub[s], r[i], s);
            else lds_get<AB>(lds, base ^ a.lds_rd_sub[s], r[i], s);
        }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const uint32_t off = cd ^ ld ^ a.iter_dst[i];
        const u32x4 v = {r[i][0], r[i][1], r[i][2], r[i][3]};
        store_vec_xor<W>(drsrc, off, v, a.dst_xor);
    }
}

template <int W, int NV, int V, int TB>
static ll_status launch_lds_elem_tb(const LdsElemArgs &a, int lds_bytes, hipStream_t stream)
{
    launch((k_lds_elem<W, NV, V, 0, TB>), dim3((unsigned)a.nblocks), dim3(1u << TB), (size_t)lds_bytes, stream, a);
    return check_launch("LDS conversion kernel launch");
}

template <int W, int NV, int V>
static ll_status launch_lds_elem_t(const LdsElemArgs &a, int lds_bytes, hipStream_t stream)
{
    switch (a.thread_bits) {
    case 6: if constexpr (NV == 4) return launch_lds_elem_tb<W, NV, V, 6>(a, lds_bytes, stream); break;   // one wave, a 4 KiB block
    case 7: if constexpr (NV == 4) return launch_lds_elem_tb<W, NV, V, 7>(a, lds_bytes, stream); break;   // two waves, an 8 KiB block
    case 8: return launch_lds_elem_tb<W, NV, V, 8>(a, lds_bytes, stream);
    case 9: if constexpr (NV <= 4) return launch_lds_elem_tb<W, NV, V, 9>(a, lds_bytes, stream); break;
    case 10: if constexpr (NV <= 4) return launch_lds_elem_tb<W, NV, V, 10>(a, lds_bytes, stream); break;
    default: break;
    }
    return fail(LL_ERR_UNSUPPORTED, "no LDS kernel for 2^%d threads and %d vectors per thread", a.thread_bits, NV);
}

template <int W, int NV>
static ll_status launch_lds_elem_v(const LdsElemArgs &a, int v, int lds_bytes, hipStream_t stream)
{
    constexpr int VS = (W == 1) ? 4 : (W == 2) ? 3 : (W == 4) ? 2 : 1;
    if (v == 0) return launch_lds_elem_t<W, NV, 0>(a, lds_bytes, stream);
    if constexpr (VS >= 1) if (v == 1) return launch_lds_elem_t<W, NV, 1>(a, lds_bytes, stream);
    if constexpr (VS >= 2) if (v == 2) return launch_lds_elem_t<W, NV, 2>(a, lds_bytes, stream);
    if constexpr (VS >= 3) if (v == 3) return launch_lds_elem_t<W, NV, 3>(a, lds_bytes, stream);
    if constexpr (VS >= 4) if (v == 4) return launch_lds_elem_t<W, NV, 4>(a, lds_bytes, stream);
    return fail(LL_ERR_UNSUPPORTED, "no LDS kernel for vector bits %d of %d-byte elements", v, W);
}

template <int W>
static ll_status launch_lds_elem_n(const LdsElemArgs &a, int nvec, int v, int lds_bytes, hipStream_t stream)
{
    switch (nvec) {
    case 1: return launch_lds_elem_v<W, 1>(a, v, lds_bytes, stream);
    case 2: return launch_lds_elem_v<W, 2>(a, v, lds_bytes, stream);
    case 4: return launch_lds_elem_v<W, 4>(a, v, lds_bytes, stream);
    case 8: return launch_lds_elem_v<W, 8>(a, v, lds_bytes, stream);
    default: return fail(LL_ERR_UNSUPPORTED, "no LDS kernel for %d vectors per thread", nvec);
    }
}

ll_status launch_lds_elem(const LdsElemArgs &a, int elem_bytes, int nvec, int lds_vec_bits, int threads, int lds_bytes,
                          void *stream)
{
    if (threads != (1 << a.thread_bits) || a.thread_bits < 6 || a.thread_bits > 10)
        return fail(LL_ERR_UNSUPPORTED, "LDS kernel runs 64, 256, 512 or 1024 threads per workgroup");
    if (a.nblocks <= 0 || a.nblocks > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", a.nblocks);
    if (lds_bytes <= 0 || lds_bytes > 64 * 1024) return fail(LL_ERR_UNSUPPORTED, "LDS block of %d bytes", lds_bytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (elem_bytes) {
    case 1: return launch_lds_elem_n<1>(a, nvec, lds_vec_bits, lds_bytes, s);
    case 2: return launch_lds_elem_n<2>(a, nvec, lds_vec_bits, lds_bytes, s);
    case 4: return launch_lds_elem_n<4>(a, nvec, lds_vec_bits, lds_bytes, s);
    case 8: return launch_lds_elem_n<8>(a, nvec, lds_vec_bits, lds_bytes, s);
    default: return fail(LL_ERR_INVALID_ARG, "elem_bytes %d", elem_bytes);
    }
}

template <int W>
static ll_status launch_lds_tr_w(const LdsElemArgs &a, int nvec, int lds_bytes, hipStream_t stream)
{
    constexpr int V = (W == 1) ? 3 : 2;             // 8-byte chunks
    const dim3 grid((unsigned)a.nblocks), block(256);
    switch (nvec) {
    case 1: launch((k_lds_elem<W, 1, V, 1>), grid, block, (size_t)lds_bytes, stream, a); break;
    case 2: launch((k_lds_elem<W, 2, V, 1>), grid, block, (size_t)lds_bytes, stream, a); break;
    case 4: launch((k_lds_elem<W, 4, V, 1>), grid, block, (size_t)lds_bytes, stream, a); break;
    case 8: launch((k_lds_elem<W, 8, V, 1>), grid, block, (size_t)lds_bytes, stream, a); break;
    default: return fail(LL_ERR_UNSUPPORTED, "no transposing-read kernel for %d vectors per thread", nvec);
    }
    return check_launch("transposing-read conversion kernel launch");
}

ll_status launch_lds_tr(const LdsElemArgs &a, int elem_bytes, int nvec, int lds_bytes, void *stream)
{
    if (a.nblocks <= 0 || a.nblocks > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", a.nblocks);
    if (lds_bytes <= 0 || lds_bytes > 64 * 1024) return fail(LL_ERR_UNSUPPORTED, "LDS block of %d bytes", lds_bytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (elem_bytes == 1) return launch_lds_tr_w<1>(a, nvec, lds_bytes, s);
    if (elem_bytes == 2) return launch_lds_tr_w<2>(a, nvec, lds_bytes, s);
    return fail(LL_ERR_UNSUPPORTED, "transposing LDS loads exist for 1- and 2-byte elements");
}

// ---------------------------------------------------------------------------------------------
// vector-preserving conversion: register transposes + (nothing | wave shuffle | 128-bit LDS)
// ---------------------------------------------------------------------------------------------

// Transpose, inside one thread, between the position of an element in its 16-byte vector and the
// low VS bits of the iteration index: element p of vector (c + 2^VS * h) becomes element c of
// vector (p + 2^VS * h).  4- and 8-byte elements: pure register renaming.  2-byte elements: one
// v_perm_b32 per output dword.
template <int W, int NV>
static __device__ __forceinline__ void transpose_regs(uint32_t (&r)[NV][4])
{
    constexpr int VS = (W == 2) ? 3 : (W == 4) ? 2 : 1;
    constexpr int E = 1 << VS;
    uint32_t t[NV][4];
#pragma unroll
    for (int h = 0; h < NV / E; ++h) {
#pragma unroll
        for (int p = 0; p < E; ++p) {          // new vector index (old position)
            if constexpr (W == 4) {
#pragma unroll
                for (int c = 0; c < 4; ++c) t[p + E * h][c] = r[c + E * h][p];
            } else if constexpr (W == 8) {
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    t[p + E * h][2 * c] = r[c + E * h][2 * p];
                    t[p + E * h][2 * c + 1] = r[c + E * h][2 * p + 1];
                }
            } else {
                // new dword q holds new positions 2q, 2q+1 = old vectors 2q, 2q+1, old position p
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t a = r[2 * q + E * h][p >> 1], b = r[2 * q + 1 + E * h][p >> 1];
                    t[p + E * h][q] = (p & 1) ? __builtin_amdgcn_perm(b, a, 0x07060302u)
                                              : __builtin_amdgcn_perm(b, a, 0x05040100u);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) r[i][c] = t[i][c];
}

// One butterfly stage: lanes l and l ^ mask exchange the vectors whose iteration bit B differs
// from their own side, i.e. the lane index bit selected by `mask` and iteration bit B trade
// places.  The lane with the mask bit clear keeps its (B = 0) vectors and sends its (B = 1)
// vectors; the partner does the opposite.  32-bit payload per ds_bpermute_b32.
template <int NV, int B>
static __device__ __forceinline__ void shuffle_stage(uint32_t (&r)[NV][4], uint32_t lane, uint32_t mask)
{
    const bool upper = (lane & mask) != 0;
    const int partner = (int)((lane ^ mask) << 2);
    constexpr int bit = 1 << B;
    // Pairs (lo, hi = lo | bit) by their index among the vectors with iteration bit B clear.  Both
    // registers of a pair are rewritten with selects (no conditional stores into the array and no
    // skipped iterations: with those, one instantiation was compiled into compare-and-select chains
    // over all 32 registers, 14 times the vector instructions).
#pragma unroll
    for (int k = 0; k < NV / 2; ++k) {
        const int lo = ((k >> B) << (B + 1)) | (k & (bit - 1)), hi = lo | bit;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t x = r[lo][c], y = r[hi][c];
            const uint32_t got = (uint32_t)__builtin_amdgcn_ds_bpermute(partner, (int)(upper ? x : y));
            r[lo][c] = upper ? got : x;
            r[hi][c] = upper ? y : got;
        }
    }
}

template <int NV, int NVB>
static __device__ __forceinline__ void shuffle_stages(uint32_t (&r)[NV][4], uint32_t lane, const VecArgs &a)
{
    if constexpr (NVB > 0) { if (a.stage_mask[0]) shuffle_stage<NV, 0>(r, lane, a.stage_mask[0]); }
    if constexpr (NVB > 1) { if (a.stage_mask[1]) shuffle_stage<NV, 1>(r, lane, a.stage_mask[1]); }
    if constexpr (NVB > 2) { if (a.stage_mask[2]) shuffle_stage<NV, 2>(r, lane, a.stage_mask[2]); }
    if constexpr (NVB > 3) { if (a.stage_mask[3]) shuffle_stage<NV, 3>(r, lane, a.stage_mask[3]); }
    if constexpr (NVB > 4) { if (a.stage_mask[4]) shuffle_stage<NV, 4>(r, lane, a.stage_mask[4]); }
}

template <int W, int NVB, int TPOSE, int XCHG>
__global__ __launch_bounds__(256) void k_vec(const VecArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int NV = 1 << NVB;
    const uint32_t tid = threadIdx.x;

    uint32_t ls = 0, ld = 0, lw = 0, lr = 0;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint32_t m = 0u - ((tid >> b) & 1u);
        ls ^= a.lane_src[b] & m;
        ld ^= a.lane_dst[b] & m;
        if constexpr (XCHG == kXchgLds) {
            lw ^= a.lds_wr_lane[b] & m;
            lr ^= a.lds_rd_lane[b] & m;
        }
    }
    struct Ctx {
        uint32_t cs, cd, cr;
        __amdgpu_buffer_rsrc_t srsrc, drsrc;
    };
    auto context = [&](long long blk) {
        Ctx x;
        const long long group = blk >> a.coset_bits;
        const uint32_t c = (uint32_t)(blk & ((1ll << a.coset_bits) - 1));
        x.cs = 0; x.cd = 0; x.cr = 0;
        for (int b = 0; b < a.coset_bits; ++b) {
            const uint32_t m = 0u - ((c >> b) & 1u);
            x.cs ^= a.coset_src[b] & m;
            x.cd ^= a.coset_dst[b] & m;
            x.cr ^= a.coset_lds_rd[b] & m;
        }
        const int gshift = a.d + a.group_bits;
        const unsigned char *sbase = static_cast<const unsigned char *>(a.src) + (((size_t)group << gshift) * W);
        unsigned char *dbase = static_cast<unsigned char *>(a.dst) + (((size_t)group << gshift) * W);
        const long long left = a.ntiles - (group << a.group_bits);
        const uint32_t tiles_here = left > (1ll << a.group_bits) ? (1u << a.group_bits) : (uint32_t)left;
        const uint32_t valid_bytes = (tiles_here << a.d) * W;
        x.srsrc = make_rsrc(sbase, valid_bytes);
        x.drsrc = make_rsrc(dbase, valid_bytes);
        return x;
    };
    auto load = [&](const Ctx &x, uint32_t (&r)[NV][4]) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t off = x.cs ^ ls ^ a.iter_src[i];
            const u32x4 v = buf_load16(x.srsrc, off * W);
            r[i][0] = v.x; r[i][1] = v.y; r[i][2] = v.z; r[i][3] = v.w;
        }
    };
    auto finish = [&](const Ctx &x, uint32_t (&r)[NV][4]) {
        if constexpr (TPOSE == kTposeBefore) transpose_regs<W, NV>(r);
        if constexpr (XCHG == kXchgShuffle) shuffle_stages<NV, NVB>(r, tid & 63, a);
        if constexpr (XCHG == kXchgLds) {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const u32x4 v = {r[i][0], r[i][1], r[i][2], r[i][3]};
                *reinterpret_cast<u32x4 *>(lds + (lw ^ a.lds_wr_iter[i])) = v;
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const u32x4 v = *reinterpret_cast<const u32x4 *>(lds + (x.cr ^ lr ^ a.lds_rd_iter[i]));
                r[i][0] = v.x; r[i][1] = v.y; r[i][2] = v.z; r[i][3] = v.w;
            }
        }
        if constexpr (TPOSE == kTposeAfter) transpose_regs<W, NV>(r);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t off = x.cd ^ ld ^ a.iter_dst[i];
            const u32x4 v = {r[i][0], r[i][1], r[i][2], r[i][3]};
            store_vec_xor<W>(x.drsrc, off, v, a.dst_xor);
        }
    };

    // One block per workgroup.  (Letting a wave take several blocks and load the next while it
    // finishes the current one was measured 5-20 % slower on MI355X at every occupancy: many
    // short-lived waves stream better.)
    const Ctx x = context(block_of_workgroup((long long)blockIdx.x, a.nblocks, a.xcd_chunk));
    uint32_t r[NV][4];
    load(x, r);
    finish(x, r);
}

template <int W, int NVB, int TPOSE, int XCHG>
static ll_status launch_vec_t(const VecArgs &a, int threads, int lds_bytes, hipStream_t stream)
{
    constexpr int VS = (W == 2) ? 3 : (W == 4) ? 2 : 1;
    if constexpr (TPOSE != kTposeNone && NVB < VS) {
        return fail(LL_ERR_UNSUPPORTED, "internal: transposing kernel needs 2^%d vectors per thread", VS);
    } else {
        // lds_bytes carries the occupancy cap (the planner asks for a share of the 160 KiB LDS that
        // admits in-flight budget / block bytes workgroups per CU)
        launch((k_vec<W, NVB, TPOSE, XCHG>), dim3((unsigned)a.nblocks), dim3((unsigned)threads),
                           (size_t)lds_bytes, stream, a);
        return check_launch("vector conversion kernel launch");
    }
}

template <int W, int NVB, int TPOSE>
static ll_status launch_vec_x(const VecArgs &a, int xchg, int threads, int lds_bytes, hipStream_t stream)
{
    switch (xchg) {
    case kXchgNone: return launch_vec_t<W, NVB, TPOSE, kXchgNone>(a, threads, lds_bytes, stream);
    case kXchgShuffle: return launch_vec_t<W, NVB, TPOSE, kXchgShuffle>(a, threads, lds_bytes, stream);
    case kXchgLds: return launch_vec_t<W, NVB, TPOSE, kXchgLds>(a, threads, lds_bytes, stream);
    default: return fail(LL_ERR_INVALID_ARG, "internal: exchange kind %d", xchg);
    }
}

template <int W, int NVB>
static ll_status launch_vec_p(const VecArgs &a, int tpose, int xchg, int threads, int lds_bytes, hipStream_t stream)
{
    switch (tpose) {
    case kTposeNone: return launch_vec_x<W, NVB, kTposeNone>(a, xchg, threads, lds_bytes, stream);
    case kTposeBefore: return launch_vec_x<W, NVB, kTposeBefore>(a, xchg, threads, lds_bytes, stream);
    case kTposeAfter: return launch_vec_x<W, NVB, kTposeAfter>(a, xchg, threads, lds_bytes, stream);
    default: return fail(LL_ERR_INVALID_ARG, "internal: transpose kind %d", tpose);
    }
}

template <int W>
static ll_status launch_vec_n(const VecArgs &a, int nvb, int tpose, int xchg, int threads, int lds_bytes, hipStream_t stream)
{
    switch (nvb) {
    case 0: return launch_vec_p<W, 0>(a, tpose, xchg, threads, lds_bytes, stream);
    case 1: return launch_vec_p<W, 1>(a, tpose, xchg, threads, lds_bytes, stream);
    case 2: return launch_vec_p<W, 2>(a, tpose, xchg, threads, lds_bytes, stream);
    case 3: return launch_vec_p<W, 3>(a, tpose, xchg, threads, lds_bytes, stream);
    case 4: return launch_vec_p<W, 4>(a, tpose, xchg, threads, lds_bytes, stream);
    default: return fail(LL_ERR_UNSUPPORTED, "no vector kernel for 2^%d vectors per thread", nvb);
    }
}

ll_status launch_vec(const VecArgs &a, int elem_bytes, int nvec_bits, int tpose, int xchg, int threads, int lds_bytes,
                     void *stream)
{
    if (threads != 64 && threads != 128 && threads != 256) return fail(LL_ERR_UNSUPPORTED, "vector kernel runs 64, 128 or 256 threads");
    if (xchg == kXchgShuffle && threads != 64) return fail(LL_ERR_UNSUPPORTED, "shuffle kernel runs one wave per workgroup");
    if (a.nblocks <= 0 || a.nblocks > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", a.nblocks);
    if (lds_bytes < 0 || lds_bytes > 64 * 1024) return fail(LL_ERR_UNSUPPORTED, "LDS block of %d bytes", lds_bytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (elem_bytes) {
    case 2: return launch_vec_n<2>(a, nvec_bits, tpose, xchg, threads, lds_bytes, s);
    case 4: return launch_vec_n<4>(a, nvec_bits, tpose, xchg, threads, lds_bytes, s);
    case 8: return launch_vec_n<8>(a, nvec_bits, tpose, xchg, threads, lds_bytes, s);
    default: return fail(LL_ERR_UNSUPPORTED, "vector kernel handles 2-, 4- and 8-byte elements");
    }
}

// ---------------------------------------------------------------------------------------------
// conversion with broadcasting: destination units pull from the canonical source unit
// ---------------------------------------------------------------------------------------------

// W: element bytes, NVS: source vectors staged per thread, V: log2 elements per LDS access,
// TB: log2 threads per workgroup (6: one wave owns the block; 8).
template <int W, int NVS, int V, int TB>
__global__ __launch_bounds__(1 << TB) void k_pull(const PullArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int VS = (W == 1) ? 4 : (W == 2) ? 3 : (W == 4) ? 2 : 1;
    constexpr int NSUB = 1 << (VS - V);
    constexpr int AB = W << V;
    const uint32_t tid = threadIdx.x;
    constexpr uint32_t T = 1u << TB;
    uint32_t ls = 0, ld = 0, lw = 0, lr = 0;
#pragma unroll
    for (int b = 0; b < TB; ++b) {
        const uint32_t m = 0u - ((tid >> b) & 1u);
        ls ^= a.lane_src[b] & m;
        ld ^= a.lane_dst[b] & m;
        lw ^= a.lds_wr_lane[b] & m;
        lr ^= a.lds_rd_lane[b] & m;
    }
    const long long blk = block_of_workgroup((long long)blockIdx.x, a.nblocks, a.xcd_chunk);
    const long long group = blk >> a.coset_bits;
    const uint32_t c = (uint32_t)(blk & ((1ll << a.coset_bits) - 1));
    uint32_t cs = a.src_xor, cd = 0, cr = a.lds_rd_xor;   // affine layouts: constants of the pull map
    for (int b = 0; b < a.coset_bits; ++b) {
        const uint32_t m = 0u - ((c >> b) & 1u);
        cs ^= a.coset_src[b] & m;
        cd ^= a.coset_dst[b] & m;
        cr ^= a.coset_lds_rd[b] & m;
    }
    const unsigned char *sbase = static_cast<const unsigned char *>(a.src) + (((size_t)group << (a.d_src + a.group_bits)) * W);
    unsigned char *dbase = static_cast<unsigned char *>(a.dst) + (((size_t)group << (a.d_dst + a.group_bits)) * W);
    const long long left = a.ntiles - (group << a.group_bits);
    const uint32_t tiles_here = left > (1ll << a.group_bits) ? (1u << a.group_bits) : (uint32_t)left;
    const __amdgpu_buffer_rsrc_t srsrc = make_rsrc(sbase, (tiles_here << a.d_src) * W);
    const __amdgpu_buffer_rsrc_t drsrc = make_rsrc(dbase, (tiles_here << a.d_dst) * W);
    const uint32_t nsrc = 1u << a.src_vec_bits;

    uint32_t r[NVS][4];
#pragma unroll
    for (int i = 0; i < NVS; ++i) {
        const uint32_t off = cs ^ ls ^ a.iter_src[i];
        u32x4 v = {0u, 0u, 0u, 0u};
        if (tid + T * i < nsrc) v = buf_load16(srsrc, off * W);
        r[i][0] = v.x; r[i][1] = v.y; r[i][2] = v.z; r[i][3] = v.w;
    }
#pragma unroll
    for (int i = 0; i < NVS; ++i) {
        if (tid + T * i < nsrc) {
            const uint32_t base = lw ^ a.lds_wr_iter[i];
#pragma unroll
            for (int s = 0; s < NSUB; ++s) lds_put<AB>(lds, base ^ a.lds_wr_sub[s], r[i], s);
        }
    }
    __syncthreads();
    // One destination vector at a time: reading four from LDS and then issuing their four stores back
    // to back measured 8-10 % slower on the write-dominated workloads.
    for (int it = 0; it < a.dst_iters; ++it) {
        uint32_t ib = 0, ob = 0;                     // wave-uniform parts of this iteration
        for (int b = 0; (it >> b) != 0; ++b) {
            const uint32_t m = 0u - (((uint32_t)it >> b) & 1u);
            ib ^= a.lds_rd_iter_bit[b] & m;
            ob ^= a.iter_dst_bit[b] & m;
        }
        const uint32_t base = cr ^ lr ^ ib;
        uint32_t o[4];
#pragma unroll
        for (int s = 0; s < NSUB; ++s) lds_get<AB>(lds, base ^ a.lds_rd_sub[s], o, s);
        const u32x4 v = {o[0], o[1], o[2], o[3]};
        buf_store16(drsrc, (cd ^ ld ^ ob) * W, v);
    }
}

template <int W, int V, int TB>
static ll_status launch_pull_wvt(const PullArgs &a, int src_iters, int lds_bytes, hipStream_t stream)
{
    const dim3 grid((unsigned)a.nblocks), block(1u << TB);
    switch (src_iters) {
    case 1: launch((k_pull<W, 1, V, TB>), grid, block, (size_t)lds_bytes, stream, a); break;
    case 2: launch((k_pull<W, 2, V, TB>), grid, block, (size_t)lds_bytes, stream, a); break;
    case 4: launch((k_pull<W, 4, V, TB>), grid, block, (size_t)lds_bytes, stream, a); break;
    case 8: launch((k_pull<W, 8, V, TB>), grid, block, (size_t)lds_bytes, stream, a); break;
    case 16: launch((k_pull<W, 16, V, TB>), grid, block, (size_t)lds_bytes, stream, a); break;
    default: return fail(LL_ERR_UNSUPPORTED, "no broadcast kernel for %d source vectors per thread", src_iters);
    }
    return check_launch("broadcast conversion kernel launch");
}

template <int W, int V>
static ll_status launch_pull_wv(const PullArgs &a, int src_iters, int thread_bits, int lds_bytes, hipStream_t stream)
{
    switch (thread_bits) {
    case 6: return launch_pull_wvt<W, V, 6>(a, src_iters, lds_bytes, stream);
    case 8: return launch_pull_wvt<W, V, 8>(a, src_iters, lds_bytes, stream);
    default: return fail(LL_ERR_UNSUPPORTED, "broadcast kernel runs 64 or 256 threads");
    }
}

template <int W>
static ll_status launch_pull_w(const PullArgs &a, int src_iters, int vec_bits, int thread_bits, int lds_bytes, hipStream_t stream)
{
    constexpr int VS = (W == 1) ? 4 : (W == 2) ? 3 : (W == 4) ? 2 : 1;
    switch (vec_bits) {
    case 0: return launch_pull_wv<W, 0>(a, src_iters, thread_bits, lds_bytes, stream);
    case 1: return launch_pull_wv<W, 1>(a, src_iters, thread_bits, lds_bytes, stream);
    case 2: if constexpr (VS >= 2) return launch_pull_wv<W, 2>(a, src_iters, thread_bits, lds_bytes, stream); break;
    case 3: if constexpr (VS >= 3) return launch_pull_wv<W, 3>(a, src_iters, thread_bits, lds_bytes, stream); break;
    case 4: if constexpr (VS >= 4) return launch_pull_wv<W, 4>(a, src_iters, thread_bits, lds_bytes, stream); break;
    default: break;
    }
    return fail(LL_ERR_INVALID_ARG, "LDS accesses of 2^%d elements of %d bytes exceed 16 bytes", vec_bits, W);
}

ll_status launch_pull(const PullArgs &a, int elem_bytes, int src_iters, int vec_bits, int thread_bits, int lds_bytes, void *stream)
{
    if (a.nblocks <= 0 || a.nblocks > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", a.nblocks);
    if (lds_bytes <= 0 || lds_bytes > 64 * 1024) return fail(LL_ERR_UNSUPPORTED, "LDS block of %d bytes", lds_bytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (elem_bytes) {
    case 1: return launch_pull_w<1>(a, src_iters, vec_bits, thread_bits, lds_bytes, s);
    case 2: return launch_pull_w<2>(a, src_iters, vec_bits, thread_bits, lds_bytes, s);
    case 4: return launch_pull_w<4>(a, src_iters, vec_bits, thread_bits, lds_bytes, s);
    case 8: return launch_pull_w<8>(a, src_iters, vec_bits, thread_bits, lds_bytes, s);
    default: return fail(LL_ERR_INVALID_ARG, "elem_bytes %d", elem_bytes);
    }
}

// ---------------------------------------------------------------------------------------------
// wave-local gather (paper Sec. 5.5): one kernel wave per layout wave, lane = layout lane
// ---------------------------------------------------------------------------------------------

// W: element bytes, NREG: register bits of the layout (a lane holds 2^NREG elements, contiguous in
// the image).  Every output element needs one value from the lane named by its index: one
// ds_bpermute_b32 per 32-bit piece, the source register being the element's own (the axis has no
// register bits).
template <int W, int NREG>
__global__ __launch_bounds__(256) void k_gather(const GatherArgs a)
{
    constexpr int NE = 1 << NREG;                 // elements per lane
    constexpr int PL = NE * W;                    // data bytes per lane
    constexpr int DW = (PL + 3) / 4;              // data dwords per lane
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wpg = blockDim.x >> 6;         // waves (chunks) per workgroup
    const long long chunk = block_of_workgroup((long long)blockIdx.x, (a.nchunks + wpg - 1) / wpg, a.xcd_chunk) * wpg + (threadIdx.x >> 6);
    if (chunk >= a.nchunks) return;               // whole wave leaves together
    const unsigned char *in = static_cast<const unsigned char *>(a.in) + ((size_t)chunk * 64 + lane) * PL;
    const unsigned char *ix = reinterpret_cast<const unsigned char *>(a.idx) + ((size_t)chunk * 64 + lane) * (NE * 4);
    unsigned char *out = static_cast<unsigned char *>(a.out) + ((size_t)chunk * 64 + lane) * PL;

    uint32_t data[DW], idx[NE], res[DW];
    if constexpr (PL >= 16) {
#pragma unroll
        for (int k = 0; k < PL / 16; ++k) {
            u32x4 v = load16(in + 16 * k);
            data[4 * k] = v.x; data[4 * k + 1] = v.y; data[4 * k + 2] = v.z; data[4 * k + 3] = v.w;
        }
    } else if constexpr (PL == 8) {
        u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(in));
        data[0] = v.x; data[1] = v.y;
    } else {
        data[0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(in));
    }
    if constexpr (NE >= 4) {
#pragma unroll
        for (int k = 0; k < NE / 4; ++k) {
            u32x4 v = load16(ix + 16 * k);
            idx[4 * k] = v.x; idx[4 * k + 1] = v.y; idx[4 * k + 2] = v.z; idx[4 * k + 3] = v.w;
        }
    } else if constexpr (NE == 2) {
        u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(ix));
        idx[0] = v.x; idx[1] = v.y;
    } else {
        idx[0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(ix));
    }

    uint32_t own_lw = a.own_const;        // own axis coordinate: lane and wave contributions
    if (!a.fast) {
#pragma unroll
        for (int b = 0; b < 6; ++b) own_lw ^= a.own_lane[b] & (0u - ((lane >> b) & 1u));
        const uint32_t wv = (uint32_t)(chunk & ((1ll << a.nwave) - 1));
        for (int b = 0; b < a.nwave; ++b) own_lw ^= a.own_wave[b] & (0u - ((wv >> b) & 1u));
    }
#pragma unroll
    for (int k = 0; k < DW; ++k) res[k] = 0;
#pragma unroll
    for (int r = 0; r < NE; ++r) {
        uint32_t s = idx[r] & a.axis_mask;
        uint32_t src_lane;
        if (a.fast) {
            src_lane = (lane & a.keep_mask) | (s << a.shift);
        } else {
            const uint32_t x = (s ^ own_lw ^ a.own_reg[r]) & a.axis_mask;
            src_lane = lane;
#pragma unroll
            for (int b = 0; b < 6; ++b) src_lane ^= a.lane_delta[b] & (0u - ((x >> b) & 1u));
        }
        const int addr = (int)(src_lane << 2);
        if constexpr (W == 8) {
            res[2 * r] = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)data[2 * r]);
            res[2 * r + 1] = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)data[2 * r + 1]);
        } else if constexpr (W == 4) {
            res[r] = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)data[r]);
        } else {
            constexpr int PER = 4 / W;            // elements per dword
            const uint32_t got = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)data[r / PER]);
            constexpr uint32_t EM = (W == 2) ? 0xffffu : 0xffu;
            const int sh = (r % PER) * W * 8;
            res[r / PER] |= got & (EM << sh);
        }
    }
    if constexpr (PL >= 16) {
#pragma unroll
        for (int k = 0; k < PL / 16; ++k) {
            u32x4 v = {res[4 * k], res[4 * k + 1], res[4 * k + 2], res[4 * k + 3]};
            store16(out + 16 * k, v);
        }
    } else if constexpr (PL == 8) {
        u32x2 v = {res[0], res[1]};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2 *>(out));
    } else {
        __builtin_nontemporal_store(res[0], reinterpret_cast<uint32_t *>(out));
    }
}

// The shuffle gather of Sec. 5.5 for rows wider than one 16-byte vector, with every global access
// coalesced.  Loads and stores move 16-byte pieces (lane m of instruction j takes piece
// j * 64 + rotl6(m, A) of the wave's chunk, a lane permutation inside a contiguous KiB), and lane <->
// register butterfly stages (shuffle_stage: one lane bit traded for one register bit, 32-bit payload
// per ds_bpermute_b32) convert between "a piece per lane" and "a layout row per lane": A stages on
// the data (2^A pieces per row), B stages on the indices (2^B pieces of four indices per row), A
// stages back on the result.  In between, lane = layout lane and the gather is the one of k_gather:
// one ds_bpermute_b32 per 32-bit piece of an element, the source register being the element's own.
//   stage s trades register (piece-in-row) bit s with lane bit 6 - A + s; afterwards lane k holds,
//   as register j', the piece that lane (j' << (6 - A)) | (k & low) loaded as register k >> (6 - A):
//   chunk piece (k >> (6-A)) * 64 + rotl6(that lane, A) = k * 2^A + j', piece j' of row k.
template <int NV, int NVB>
static __device__ __forceinline__ void row_stages(uint32_t (&r)[NV][4], uint32_t lane)
{
    if constexpr (NVB > 0) shuffle_stage<NV, 0>(r, lane, 1u << (6 - NVB));
    if constexpr (NVB > 1) shuffle_stage<NV, 1>(r, lane, 1u << (7 - NVB));
    if constexpr (NVB > 2) shuffle_stage<NV, 2>(r, lane, 1u << (8 - NVB));
    if constexpr (NVB > 3) shuffle_stage<NV, 3>(r, lane, 1u << (9 - NVB));
}

template <int W, int NREG>
__global__ __launch_bounds__(256) void k_gather_rows(const GatherArgs a)
{
    constexpr int NE = 1 << NREG;                 // elements per layout lane
    constexpr int PL = NE * W;                    // bytes per layout lane (row): 32 .. 256
    constexpr int M = PL / 16;                    // data pieces per row
    constexpr int IQ = NE / 4;                    // index pieces per row
    constexpr int A = (M == 2) ? 1 : (M == 4) ? 2 : (M == 8) ? 3 : 4;
    constexpr int B = (IQ == 1) ? 0 : (IQ == 2) ? 1 : (IQ == 4) ? 2 : (IQ == 8) ? 3 : 4;
    constexpr int DW = PL / 4;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wpg = blockDim.x >> 6;         // waves (chunks) per workgroup
    const long long chunk = block_of_workgroup((long long)blockIdx.x, (a.nchunks + wpg - 1) / wpg, a.xcd_chunk) * wpg + (threadIdx.x >> 6);
    if (chunk >= a.nchunks) return;               // whole wave leaves together
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(static_cast<const unsigned char *>(a.in) + (size_t)chunk * 64 * PL, 64 * PL);
    const __amdgpu_buffer_rsrc_t rix = make_rsrc(reinterpret_cast<const unsigned char *>(a.idx) + (size_t)chunk * 64 * NE * 4, 64 * NE * 4);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(static_cast<unsigned char *>(a.out) + (size_t)chunk * 64 * PL, 64 * PL);
    const uint32_t piece_d = ((lane << A) | (lane >> (6 - A))) & 63u;      // rotl6(lane, A)
    const uint32_t piece_i = B ? (((lane << B) | (lane >> (6 - B))) & 63u) : lane;

    uint32_t dv[M][4], iv[IQ][4];
#pragma unroll
    for (int j = 0; j < M; ++j) {
        const u32x4 v = buf_load16(rin, (j * 64 + piece_d) * 16);
        dv[j][0] = v.x; dv[j][1] = v.y; dv[j][2] = v.z; dv[j][3] = v.w;
    }
#pragma unroll
    for (int j = 0; j < IQ; ++j) {
        const u32x4 v = buf_load16(rix, (j * 64 + piece_i) * 16);
        iv[j][0] = v.x; iv[j][1] = v.y; iv[j][2] = v.z; iv[j][3] = v.w;
    }
    row_stages<M, A>(dv, lane);
    row_stages<IQ, B>(iv, lane);

    uint32_t own_lw = a.own_const;        // own axis coordinate: lane and wave contributions
    if (!a.fast) {
#pragma unroll
        for (int b = 0; b < 6; ++b) own_lw ^= a.own_lane[b] & (0u - ((lane >> b) & 1u));
        const uint32_t wv = (uint32_t)(chunk & ((1ll << a.nwave) - 1));
        for (int b = 0; b < a.nwave; ++b) own_lw ^= a.own_wave[b] & (0u - ((wv >> b) & 1u));
    }
    uint32_t rv[M][4];
#pragma unroll
    for (int k = 0; k < DW; ++k) rv[k >> 2][k & 3] = 0;
#pragma unroll
    for (int r = 0; r < NE; ++r) {
        const uint32_t s = iv[r >> 2][r & 3] & a.axis_mask;
        uint32_t src_lane;
        if (a.fast) {
            src_lane = (lane & a.keep_mask) | (s << a.shift);
        } else {
            const uint32_t x = (s ^ own_lw ^ a.own_reg[r]) & a.axis_mask;
            src_lane = lane;
#pragma unroll
            for (int b = 0; b < 6; ++b) src_lane ^= a.lane_delta[b] & (0u - ((x >> b) & 1u));
        }
        const int addr = (int)(src_lane << 2);
        if constexpr (W == 8) {
            rv[(2 * r) >> 2][(2 * r) & 3] = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)dv[(2 * r) >> 2][(2 * r) & 3]);
            rv[(2 * r + 1) >> 2][(2 * r + 1) & 3] = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)dv[(2 * r + 1) >> 2][(2 * r + 1) & 3]);
        } else if constexpr (W == 4) {
            rv[r >> 2][r & 3] = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)dv[r >> 2][r & 3]);
        } else {
            constexpr int PER = 4 / W;            // elements per dword
            const int q = r / PER;
            const uint32_t got = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)dv[q >> 2][q & 3]);
            constexpr uint32_t EM = (W == 2) ? 0xffffu : 0xffu;
            const int sh = (r % PER) * W * 8;
            rv[q >> 2][q & 3] |= got & (EM << sh);
        }
    }
    row_stages<M, A>(rv, lane);           // back to a piece per lane: the stages are their own inverses and commute
#pragma unroll
    for (int j = 0; j < M; ++j) {
        const u32x4 v = {rv[j][0], rv[j][1], rv[j][2], rv[j][3]};
        buf_store16(rout, (j * 64 + piece_d) * 16, v);
    }
}

// Same gather with every global access fully coalesced.  A lane no longer stands for a layout lane:
// lane k of a load or store instruction takes the k-th 16-byte (or 8-byte) piece of the chunk.  The
// source values of the wave's chunk are staged in a wave-private LDS region, one row per layout
// lane, and each output element is fetched with one LDS read at the row its index names.  This is
// the same crossbar the lane shuffle uses (ds_bpermute reads a 64-dword row through it).  No data
// crosses between waves - the condition of Sec. 5.5, the axis stays inside the wave - so each wave
// only needs its own LDS writes to be visible before it reads; the kernel is launched with one wave
// per workgroup by default, and the __syncthreads() between staging and gathering is then a wave-
// local barrier (with 2 or 4 waves per workgroup, on request, every wave of the group reaches it:
// none leaves early).  Rows are XOR-swizzled so that reads of one register from 32 different
// rows fall in 32 different banks (random indices then collide only as often as random lanes do).
//   unit      the 4- or 8-byte word an element lives in
//   row s     holds RU units; unit q of row s is stored at unit address s*RU + (q ^ f(s))
template <int W, int NREG>
__global__ __launch_bounds__(256) void k_gather_staged(const GatherArgs a)
{
    constexpr int NE = 1 << NREG;                 // elements per layout lane
    constexpr int PL = NE * W;                    // bytes per layout lane (row), >= 16
    constexpr int M = PL / 16;                    // 16-byte vectors per row
    constexpr int U = (W == 8) ? 8 : 4;           // unit bytes
    constexpr int RU = PL / U;                    // units per row
    constexpr int UV = 16 / U;                    // units per 16-byte vector
    constexpr int EPS = (W == 8) ? 2 : 4;         // elements per lane per step (one idx load)
    constexpr int NSTEP = NE / EPS;               // steps per lane: 64 * NE elements / (64 * EPS)
    constexpr int LOG_M = (M == 1) ? 0 : (M == 2) ? 1 : (M == 4) ? 2 : (M == 8) ? 3 : 4;
    constexpr int FS_SHIFT = (RU >= 32) ? 0 : (RU == 16) ? 1 : (RU == 8) ? 2 : (RU == 4) ? 3 : (RU == 2) ? 4 : 5;
    constexpr int FS_MASK = (RU >= 32) ? 31 : RU - 1;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t wpg = blockDim.x >> 6;         // waves (chunks) per workgroup
    const long long chunk0 = block_of_workgroup((long long)blockIdx.x, (a.nchunks + wpg - 1) / wpg, a.xcd_chunk) * wpg;
    const long long chunk = chunk0 + wave;
    const long long left = a.nchunks - chunk0;
    const uint32_t chunks_here = left >= (long long)wpg ? wpg : (left > 0 ? (uint32_t)left : 0u);
    // descriptors cover the chunks of this workgroup (one per wave): out-of-range lanes read zero and
    // write nothing
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(static_cast<const unsigned char *>(a.in) + (size_t)chunk0 * 64 * PL, chunks_here * 64 * PL);
    const __amdgpu_buffer_rsrc_t rix = make_rsrc(reinterpret_cast<const unsigned char *>(a.idx) + (size_t)chunk0 * 64 * NE * 4, chunks_here * 64 * NE * 4);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(static_cast<unsigned char *>(a.out) + (size_t)chunk0 * 64 * PL, chunks_here * 64 * PL);
    unsigned char *my = lds + wave * (64 * PL);

    // issue all loads first
    u32x4 vin[M];
#pragma unroll
    for (int j = 0; j < M; ++j) vin[j] = buf_load16(rin, wave * (64 * PL) + (j * 64 + lane) * 16);
    uint32_t idx[NSTEP][EPS];
#pragma unroll
    for (int j = 0; j < NSTEP; ++j) {
        const uint32_t off = wave * (64 * NE * 4) + (j * 64 + lane) * (EPS * 4);
        if constexpr (EPS == 4) {
            const u32x4 v = buf_load16(rix, off);
            idx[j][0] = v.x; idx[j][1] = v.y; idx[j][2] = v.z; idx[j][3] = v.w;
        } else {
            const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rix, off, 0, kStream);
            idx[j][0] = v.x; idx[j][1] = v.y;
        }
    }
    // stage the source rows
#pragma unroll
    for (int j = 0; j < M; ++j) {
        const uint32_t vecno = j * 64 + lane;
        const uint32_t s = vecno >> LOG_M, hv = vecno & (M - 1);
        const uint32_t fs = (s >> FS_SHIFT) & FS_MASK;
        const uint32_t w4[4] = {vin[j].x, vin[j].y, vin[j].z, vin[j].w};
#pragma unroll
        for (int c = 0; c < UV; ++c) {
            const uint32_t q = hv * UV + c;
            const uint32_t addr = (s * RU + (q ^ fs)) * U;
            if constexpr (U == 8) {
                u32x2 v = {w4[2 * c], w4[2 * c + 1]};
                *reinterpret_cast<u32x2 *>(my + addr) = v;
            } else {
                *reinterpret_cast<uint32_t *>(my + addr) = w4[c];
            }
        }
    }
    __syncthreads();

    uint32_t own_w = a.own_const;
    if (!a.fast) {
        const uint32_t wv = (uint32_t)(chunk & ((1ll << a.nwave) - 1));
        for (int b = 0; b < a.nwave; ++b) own_w ^= a.own_wave[b] & (0u - ((wv >> b) & 1u));
    }
#pragma unroll
    for (int j = 0; j < NSTEP; ++j) {
        const uint32_t e0 = (j * 64 + lane) * EPS;       // first element of this step, inside the chunk
        const uint32_t l = e0 >> NREG;                   // its layout lane (all EPS elements share it)
        uint32_t own_l = own_w;
        if (!a.fast) {
#pragma unroll
            for (int b = 0; b < 6; ++b) own_l ^= a.own_lane[b] & (0u - ((l >> b) & 1u));
        }
        uint32_t got[EPS * ((W == 8) ? 2 : 1)];
#pragma unroll
        for (int t = 0; t < EPS; ++t) {
            const uint32_t r = (e0 + t) & (NE - 1);
            const uint32_t sidx = idx[j][t] & a.axis_mask;
            uint32_t src;
            if (a.fast) {
                src = (l & a.keep_mask) | (sidx << a.shift);
            } else {
                uint32_t own = own_l;
#pragma unroll
                for (int b = 0; b < NREG; ++b) own ^= a.own_regbit[b] & (0u - ((r >> b) & 1u));
                const uint32_t x = (sidx ^ own) & a.axis_mask;
                src = l;
#pragma unroll
                for (int b = 0; b < 6; ++b) src ^= a.lane_delta[b] & (0u - ((x >> b) & 1u));
            }
            const uint32_t fs = (src >> FS_SHIFT) & FS_MASK;
            const uint32_t q = (r * W) / U;
            const uint32_t addr = (src * RU + (q ^ fs)) * U + (r * W) % U;
            if constexpr (W == 8) {
                const u32x2 v = *reinterpret_cast<const u32x2 *>(my + addr);
                got[2 * t] = v.x; got[2 * t + 1] = v.y;
            } else if constexpr (W == 4) {
                got[t] = *reinterpret_cast<const uint32_t *>(my + addr);
            } else if constexpr (W == 2) {
                got[t] = *reinterpret_cast<const uint16_t *>(my + addr);
            } else {
                got[t] = *reinterpret_cast<const uint8_t *>(my + addr);
            }
        }
        const uint32_t ooff = wave * (64 * PL) + e0 * W;
        if constexpr (W == 8 || W == 4) {
            const u32x4 v = {got[0], got[1], got[2], got[3]};
            buf_store16(rout, ooff, v);
        } else if constexpr (W == 2) {
            const u32x2 v = {got[0] | (got[1] << 16), got[2] | (got[3] << 16)};
            __builtin_amdgcn_raw_buffer_store_b64(v, rout, ooff, 0, kStream);
        } else {
            const uint32_t v = got[0] | (got[1] << 8) | (got[2] << 16) | (got[3] << 24);
            __builtin_amdgcn_raw_buffer_store_b32(v, rout, ooff, 0, kStream);
        }
    }
}

// `waves`: chunks (one per wave) a workgroup takes: 1, 2 or 4.
template <int W, int NREG>
static ll_status launch_gather_staged_t(const GatherArgs &a, int waves, int lds_alloc, hipStream_t stream)
{
    constexpr int PL = (1 << NREG) * W;
    if constexpr (PL < 16 || PL > 256 || (1 << NREG) < 4) {
        return fail(LL_ERR_UNSUPPORTED, "staged gather needs 16 to 256 bytes and at least 4 elements per lane");
    } else {
        const long long grid = (a.nchunks + waves - 1) / waves;
        if (grid > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", grid);
        const int lds_bytes = waves * 64 * PL;
        // lds_alloc carries the occupancy cap (every wave has a chunk of `in` and of `idx` in flight)
        const unsigned alloc = lds_alloc > lds_bytes ? (unsigned)lds_alloc : (unsigned)lds_bytes;
        if (alloc > 64u * 1024u) return fail(LL_ERR_INVALID_ARG, "internal: staged gather asked for %u bytes of LDS", alloc);
        launch((k_gather_staged<W, NREG>), dim3((unsigned)grid), dim3(64u * (unsigned)waves), alloc, stream, a);
        return check_launch("gather kernel launch");
    }
}

template <int W, int NREG>
static ll_status launch_gather_rows_t(const GatherArgs &a, int waves, int lds_alloc, hipStream_t stream)
{
    constexpr int PL = (1 << NREG) * W;
    if constexpr (PL < 32 || PL > 256 || (1 << NREG) < 4) {
        return fail(LL_ERR_UNSUPPORTED, "row-shuffle gather needs 32 to 256 bytes and at least 4 elements per lane");
    } else {
        const long long grid = (a.nchunks + waves - 1) / waves;
        if (grid > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", grid);
        if (lds_alloc < 0 || lds_alloc > 64 * 1024) return fail(LL_ERR_INVALID_ARG, "internal: row-shuffle gather asked for %d bytes of LDS", lds_alloc);
        launch((k_gather_rows<W, NREG>), dim3((unsigned)grid), dim3(64u * (unsigned)waves), (size_t)lds_alloc, stream, a);   // LDS only as the occupancy cap
        return check_launch("gather kernel launch");
    }
}

template <int W, int NREG>
static ll_status launch_gather_t(const GatherArgs &a, int waves, int lds_alloc, hipStream_t stream)
{
    if constexpr ((1 << NREG) * W < 4 || (1 << NREG) * W > 256) {
        return fail(LL_ERR_UNSUPPORTED, "gather needs 4 to 256 bytes per lane (got %d)", (1 << NREG) * W);
    } else {
        const long long grid = (a.nchunks + waves - 1) / waves;
        if (grid > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", grid);
        if (lds_alloc < 0 || lds_alloc > 64 * 1024) return fail(LL_ERR_INVALID_ARG, "internal: shuffle gather asked for %d bytes of LDS", lds_alloc);
        launch((k_gather<W, NREG>), dim3((unsigned)grid), dim3(64u * (unsigned)waves), (size_t)lds_alloc, stream, a);   // LDS only as the occupancy cap
        return check_launch("gather kernel launch");
    }
}

template <int W>
static ll_status launch_gather_w(const GatherArgs &a, int waves, int lds_alloc, hipStream_t stream)
{
    if (a.staged == 2) {
        switch (a.nreg) {
        case 2: return launch_gather_rows_t<W, 2>(a, waves, lds_alloc, stream);
        case 3: return launch_gather_rows_t<W, 3>(a, waves, lds_alloc, stream);
        case 4: return launch_gather_rows_t<W, 4>(a, waves, lds_alloc, stream);
        case 5: return launch_gather_rows_t<W, 5>(a, waves, lds_alloc, stream);
        case 6: return launch_gather_rows_t<W, 6>(a, waves, lds_alloc, stream);
        default: return fail(LL_ERR_UNSUPPORTED, "row-shuffle gather needs 2 to 6 register bits (got %d)", a.nreg);
        }
    }
    if (a.staged) {
        switch (a.nreg) {
        case 2: return launch_gather_staged_t<W, 2>(a, waves, lds_alloc, stream);
        case 3: return launch_gather_staged_t<W, 3>(a, waves, lds_alloc, stream);
        case 4: return launch_gather_staged_t<W, 4>(a, waves, lds_alloc, stream);
        case 5: return launch_gather_staged_t<W, 5>(a, waves, lds_alloc, stream);
        case 6: return launch_gather_staged_t<W, 6>(a, waves, lds_alloc, stream);
        default: return fail(LL_ERR_UNSUPPORTED, "staged gather needs 2 to 6 register bits (got %d)", a.nreg);
        }
    }
    switch (a.nreg) {
    case 0: return launch_gather_t<W, 0>(a, waves, lds_alloc, stream);
    case 1: return launch_gather_t<W, 1>(a, waves, lds_alloc, stream);
    case 2: return launch_gather_t<W, 2>(a, waves, lds_alloc, stream);
    case 3: return launch_gather_t<W, 3>(a, waves, lds_alloc, stream);
    case 4: return launch_gather_t<W, 4>(a, waves, lds_alloc, stream);
    case 5: return launch_gather_t<W, 5>(a, waves, lds_alloc, stream);
    case 6: return launch_gather_t<W, 6>(a, waves, lds_alloc, stream);
    default: return fail(LL_ERR_UNSUPPORTED, "gather supports at most 6 register bits (got %d)", a.nreg);
    }
}

// General gather: any surjective layout (replicas included), axis bits anywhere inside the block.
// 2^TB threads (256, 512 or 1024: see launch_gather_general_w).
//   stage   coalesced 16-byte loads of the block of `in`, written to LDS word by word (4-byte words,
//           8-byte for 8-byte elements) at XOR-swizzled addresses;
//   gather  a unit of work is 4 consecutive output elements (2 for 8-byte elements): one coalesced
//           load of their indices, at most 16 bytes stored.  For each element the XOR delta that moves its hardware index along the axis
//           to the indexed coordinate (Sec. 5.5: the source is L^-1 of the element's logical
//           position with the axis coordinate replaced) is linear in x = idx ^ own coordinate, and
//           so is the swizzle: the LDS address of the source is (address of the element itself) ^
//           T(x), with T read from tables of 32 entries per 5 bits of x that sit in LDS behind the
//           block (32 consecutive words: any access pattern to one table is conflict free).
// The swizzle moves higher address bits into the bank bits so that lanes reading the same register
// slot of different layout lanes fall in different banks; reads are data dependent, so conflicts
// cannot be excluded in general.  U: passes handled together (loads issued back to back).
template <int W, int U, int TB>
__global__ __launch_bounds__(1 << TB) void k_gather_general(const GatherGenArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int VS = (W == 1) ? 4 : (W == 2) ? 3 : (W == 4) ? 2 : 1;
    constexpr uint32_t T = 1u << TB;                 // threads per workgroup
    constexpr int UB = (W == 8) ? 1 : 2;             // log2 elements per unit: one 16-byte (8-byte) index load
    constexpr int UE = 1 << UB;
    const uint32_t tid = threadIdx.x;
    const uint32_t block_elems = 1u << a.block_bits;
    // which block of which tile group: the block is a coset of the subspace spanned by `embed`
    const long long blk = block_of_workgroup((long long)blockIdx.x, a.nblocks, a.xcd_chunk);
    const long long group = blk >> a.coset_bits;
    const uint32_t cidx = (uint32_t)(blk & ((1ll << a.coset_bits) - 1));
    uint32_t cbase = 0, own_c = a.own_const;
    for (int b = 0; b < a.coset_bits; ++b) {
        const uint32_t m = 0u - ((cidx >> b) & 1u);
        cbase ^= a.coset[b] & m;
        own_c ^= a.own_coset[b] & m;
    }
    const int gshift = a.d + a.group_bits;
    const long long left = a.ntiles - (group << a.group_bits);
    const uint32_t tiles_here = left > (1ll << a.group_bits) ? (1u << a.group_bits) : (uint32_t)left;
    const uint32_t valid = tiles_here << a.d;        // elements of this group that exist (a prefix)
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(static_cast<const unsigned char *>(a.in) + (((size_t)group << gshift) * W), valid * W);
    const __amdgpu_buffer_rsrc_t rix = make_rsrc(reinterpret_cast<const unsigned char *>(a.idx) + (((size_t)group << gshift) * 4), valid * 4);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(static_cast<unsigned char *>(a.out) + (((size_t)group << gshift) * W), valid * W);
    auto swz = [&](uint32_t addr) { return addr ^ (((addr >> a.swz_shift) & a.swz_mask) << a.swz_to); };
    uint32_t *table = reinterpret_cast<uint32_t *>(lds + ((size_t)block_elems * W));

    // delta tables
    if (tid < 128u) {                                    // four tables, those beyond the axis bits all zero
        const uint32_t x = (tid & 31u) << (5u * (tid >> 5));
        uint32_t dl = 0;
        for (int b = 0; b < a.na; ++b) dl ^= a.delta[b] & (0u - ((x >> b) & 1u));
        table[tid] = swz(dl * W);
    }
    // Group-relative element offsets of this thread's vectors and units: block-local index -> image
    // index is linear (XOR of `embed` entries), identity inside a run.
    uint32_t vec_t = cbase, unit_t = cbase, own_t = own_c;
#pragma unroll
    for (int b = 0; b < TB; ++b) {
        const uint32_t m = 0u - ((tid >> b) & 1u);
        vec_t ^= a.embed[VS + b] & m;
        unit_t ^= a.embed[UB + b] & m;
        own_t ^= a.own_bit[UB + b] & m;
    }
    // stage the block
    const uint32_t vec_passes = (block_elems >> VS) >> TB;        // 16-byte vectors per thread (a multiple of U)
    for (uint32_t p = 0; p < vec_passes; p += U) {
        u32x4 x[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            uint32_t off = vec_t;
            for (int b = 0; ((p + q) >> b) != 0; ++b) off ^= a.embed[VS + TB + b] & (0u - (((p + q) >> b) & 1u));
            x[q] = buf_load16(rin, off * W);
        }
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const uint32_t at = (tid + T * (p + q)) * 16u;
            if constexpr (W == 8) {
                const u32x2 lo = {x[q].x, x[q].y}, hi = {x[q].z, x[q].w};
                *reinterpret_cast<u32x2 *>(lds + swz(at)) = lo;
                *reinterpret_cast<u32x2 *>(lds + swz(at + 8)) = hi;
            } else {
                *reinterpret_cast<uint32_t *>(lds + swz(at)) = x[q].x;
                *reinterpret_cast<uint32_t *>(lds + swz(at + 4)) = x[q].y;
                *reinterpret_cast<uint32_t *>(lds + swz(at + 8)) = x[q].z;
                *reinterpret_cast<uint32_t *>(lds + swz(at + 12)) = x[q].w;
            }
        }
    }
    // axis coordinate of an element = XOR of the contributions of the set bits of its block-local
    // index (thread bits, pass bits, slot bits) and of the block's own offset
    const uint32_t own_s[4] = {0u, a.own_bit[0], a.own_bit[1], a.own_bit[0] ^ a.own_bit[1]};
    const uint32_t unit_passes = (block_elems >> UB) >> TB;        // units per thread (a multiple of U)
    __syncthreads();

    for (uint32_t p = 0; p < unit_passes; p += U) {
        uint32_t ix[U][UE], uoff[U], own_p[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const uint32_t pass = p + q;
            uoff[q] = unit_t;
            own_p[q] = own_t;
            for (int b = 0; (pass >> b) != 0; ++b) {
                const uint32_t m = 0u - ((pass >> b) & 1u);
                uoff[q] ^= a.embed[UB + TB + b] & m;
                own_p[q] ^= a.own_bit[UB + TB + b] & m;
            }
            if constexpr (UE == 4) {
                const u32x4 t = buf_load16(rix, uoff[q] * 4u);
                ix[q][0] = t.x; ix[q][1] = t.y; ix[q][2] = t.z; ix[q][3] = t.w;
            } else {
                const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(rix, uoff[q] * 4u, 0, kStream);
                ix[q][0] = t.x; ix[q][1] = t.y;
            }
        }
        // When the deltas are consecutive single bits of the block-local index and nothing is swizzled
        // (a row gather in a row-major tile), the LDS offset of a move is the coordinate difference
        // shifted into place: no table lookups.  The choice is uniform and made per pass.
        auto gather_units = [&](auto mode) {
        constexpr int kMode = decltype(mode)::value;       // 0: four tables, 1: shifted coordinate, 2: two tables (axis of at most 2^10)
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const uint32_t unit = tid + T * (p + q);
            const uint32_t self = swz(unit * (uint32_t)(UE * W));  // LDS address of the unit's first element
            uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int s = 0; s < UE; ++s) {
                const uint32_t x = (ix[q][s] ^ own_p[q] ^ own_s[s]) & a.axis_mask;
                uint32_t t;
                if constexpr (kMode == 1) {
                    t = x << a.field_shift;
                } else if constexpr (kMode == 2) {
                    t = table[x & 31u] ^ table[32u + (x >> 5)];
                } else {
                    t = table[x & 31u];
                    t ^= table[32u + ((x >> 5) & 31u)] ^ table[64u + ((x >> 10) & 31u)] ^ table[96u + (x >> 15)];
                }
                const uint32_t addr = self ^ ((uint32_t)s * W) ^ t;   // XOR, not add: the swizzle may have set bit 2 of self
                if constexpr (W == 8) {
                    const u32x2 v = *reinterpret_cast<const u32x2 *>(lds + addr);
                    o[2 * s] = v.x; o[2 * s + 1] = v.y;
                } else if constexpr (W == 4) {
                    o[s] = *reinterpret_cast<const uint32_t *>(lds + addr);
                } else if constexpr (W == 2) {
                    o[s >> 1] |= (uint32_t)*reinterpret_cast<const uint16_t *>(lds + addr) << ((s & 1) * 16);
                } else {
                    o[0] |= (uint32_t)*reinterpret_cast<const uint8_t *>(lds + addr) << (s * 8);
                }
            }
            if constexpr (W >= 4) {
                const u32x4 v = {o[0], o[1], o[2], o[3]};
                buf_store16(rout, uoff[q] * W, v);
            } else if constexpr (W == 2) {
                const u32x2 v = {o[0], o[1]};
                __builtin_amdgcn_raw_buffer_store_b64(v, rout, uoff[q] * W, 0, kStream);
            } else {
                __builtin_amdgcn_raw_buffer_store_b32(o[0], rout, uoff[q] * W, 0, kStream);
            }
        }
        };
        if (a.field_shift >= 0)
            gather_units(std::integral_constant<int, 1>{});
        else if (a.na <= 10)
            gather_units(std::integral_constant<int, 2>{});
        else
            gather_units(std::integral_constant<int, 0>{});
    }
}

template <int W, int TB>
static ll_status launch_gather_general_wt(const GatherGenArgs &a, int lds_alloc, hipStream_t s)
{
    constexpr int VS = (W == 1) ? 4 : (W == 2) ? 3 : (W == 4) ? 2 : 1;
    const long long block_bytes = (1ll << a.block_bits) * W;
    size_t lds_bytes = (size_t)block_bytes + 4u * 128u;            // the block and four delta tables
    if ((size_t)lds_alloc > lds_bytes && lds_alloc <= 64 * 1024) lds_bytes = (size_t)lds_alloc;   // occupancy cap
    const dim3 grid((unsigned)a.nblocks), block(1u << TB);
    const int vec_passes = (int)((1ll << a.block_bits) >> VS >> TB), unit_passes = (int)((1ll << a.block_bits) >> ((W == 8 ? 1 : 2) + TB));
    if (vec_passes < 1 || unit_passes < 1) return fail(LL_ERR_INVALID_ARG, "internal: gather block smaller than one pass");
    const int together = vec_passes < unit_passes ? vec_passes : unit_passes;   // both are powers of two
    if (together >= 4) {
        if (lds_bytes > 64 * 1024) {
            static std::atomic<uint64_t> allowed{0};
            if (ll_status st = allow_large_lds(reinterpret_cast<const void *>(k_gather_general<W, 4, TB>), 136 * 1024, allowed); st != LL_OK)
                return st;
        }
        launch((k_gather_general<W, 4, TB>), grid, block, lds_bytes, s, a);
    } else if (together == 2) {
        launch((k_gather_general<W, 2, TB>), grid, block, lds_bytes, s, a);
    } else {
        launch((k_gather_general<W, 1, TB>), grid, block, lds_bytes, s, a);
    }
    return check_launch("general gather kernel launch");
}

// Threads per workgroup.  A block is staged, then gathered from, with a barrier between: what hides
// memory latency is other workgroups on the CU, and a large block leaves room for few of them, so it
// gets more threads.  Measured on MI355X (TB/s, 256 / 512 / 1024 threads): 128 KiB blocks 3.3-3.5 /
// 5.2-5.3 / 5.7-5.96; 64 KiB 5.5-5.6 / 6.0 / 6.05-6.16; 32 KiB 5.8-6.0 / 6.0-6.26 / 6.07-6.35; 16 KiB
// 5.7-6.2 / 5.9-6.5 / 4.9-5.7; 8 KiB 6.3-6.5 / 4.1-5.7 / - (one-byte elements, whose units are a quarter
// of the bytes: 5.96 / 6.08 / -).  Interleaved repeats on 512 MiB of data.  One or two waves per 8 KiB
// block (the recipe of the conversion kernels) lose here, 5.8-6.1 against 6.25-6.5 TB/s: the gather
// phase is 31 vector instructions per element and wants many waves to hide them.
template <int W>
static ll_status launch_gather_general_w(const GatherGenArgs &a, int tb, int lds_alloc, hipStream_t s)
{
    if (tb == 10) return launch_gather_general_wt<W, 10>(a, lds_alloc, s);
    if (tb == 9) return launch_gather_general_wt<W, 9>(a, lds_alloc, s);
    return launch_gather_general_wt<W, 8>(a, lds_alloc, s);
}

ll_status launch_gather_general(const GatherGenArgs &a, int elem_bytes, int thread_bits, int lds_alloc, void *stream)
{
    if (a.nblocks <= 0 || a.nblocks > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", a.nblocks);
    const long long block_bytes = (1ll << a.block_bits) * elem_bytes;
    if (block_bytes < 4096 || block_bytes > 128 * 1024) return fail(LL_ERR_UNSUPPORTED, "gather block of %lld bytes", block_bytes);
    if (a.na < 0 || a.na > 20) return fail(LL_ERR_UNSUPPORTED, "gather axis of 2^%d elements", a.na);   // four delta tables of five bits
    if (a.block_bits > 31 || a.coset_bits < 0 || a.coset_bits > kMaxCosetBits) return fail(LL_ERR_INVALID_ARG, "internal: gather block geometry");
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (elem_bytes) {
    case 1: return launch_gather_general_w<1>(a, thread_bits, lds_alloc, s);
    case 2: return launch_gather_general_w<2>(a, thread_bits, lds_alloc, s);
    case 4: return launch_gather_general_w<4>(a, thread_bits, lds_alloc, s);
    case 8: return launch_gather_general_w<8>(a, thread_bits, lds_alloc, s);
    default: return fail(LL_ERR_INVALID_ARG, "elem_bytes %d", elem_bytes);
    }
}

// Gather for axes whose block does not fit LDS: the source element is read straight from memory at
// (own index) ^ delta(x), with the same linear delta tables as above (element units here, up to 6
// tables of 32 entries for an axis of 2^30).  A workgroup takes kGlobalPasses * 256 units of
// consecutive output elements: coalesced index loads and output stores, element-wide source loads
// that stay inside the aligned block of 2^block_bits elements around the element (L2 / MALL serve
// the re-reads when the block order keeps one block on one XCD).
template <int W>
__global__ __launch_bounds__(256) void k_gather_global(const GatherGenArgs a)
{
    __shared__ uint32_t table[6 * 32];
    constexpr int UB = (W == 8) ? 1 : 2;
    constexpr int UE = 1 << UB;
    constexpr int CB = UB + 8 + 2;                    // log2 elements per workgroup (4 passes)
    static_assert(kGlobalPasses == 4, "CB assumes four passes");
    const uint32_t tid = threadIdx.x;
    const int ntab = a.na > 0 ? (a.na + 4) / 5 : 1;
    // at least four tables are filled (those beyond the axis bits with zeros) so that the first four
    // lookups of an element need no condition and issue together
    if (tid < 32u * (uint32_t)(ntab > 4 ? ntab : 4)) {
        const uint32_t x = (tid & 31u) << (5u * (tid >> 5));
        uint32_t dl = 0;
        for (int b = 0; b < a.na; ++b) dl ^= a.delta[b] & (0u - ((x >> b) & 1u));
        table[tid] = dl;
    }
    const long long first = block_of_workgroup((long long)blockIdx.x, a.nblocks, a.xcd_chunk) << CB;
    const long long left = a.total_elems - first;
    const uint32_t valid = left >= (1ll << CB) ? (1u << CB) : (uint32_t)left;     // a multiple of UE
    const __amdgpu_buffer_rsrc_t rix = make_rsrc(reinterpret_cast<const unsigned char *>(a.idx) + (size_t)first * 4, valid * 4);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(static_cast<unsigned char *>(a.out) + (size_t)first * W, valid * W);
    const unsigned char *in = static_cast<const unsigned char *>(a.in);

    uint32_t own_t = a.own_const;
    {
        const unsigned long long f = (unsigned long long)first;
        for (int b = CB; b < 32; ++b) own_t ^= a.own_bit[b] & (0u - (uint32_t)((f >> b) & 1ull));
#pragma unroll
        for (int b = 0; b < 8; ++b) own_t ^= a.own_bit[UB + b] & (0u - ((tid >> b) & 1u));
    }
    const uint32_t own_s[4] = {0u, a.own_bit[0], a.own_bit[1], a.own_bit[0] ^ a.own_bit[1]};
    const uint32_t own_q[4] = {0u, a.own_bit[UB + 8], a.own_bit[UB + 9], a.own_bit[UB + 8] ^ a.own_bit[UB + 9]};

    uint32_t ix[kGlobalPasses][UE];
#pragma unroll
    for (int q = 0; q < kGlobalPasses; ++q) {
        if constexpr (UE == 4) {
            const u32x4 t = buf_load16(rix, (tid + 256u * q) * 16u);
            ix[q][0] = t.x; ix[q][1] = t.y; ix[q][2] = t.z; ix[q][3] = t.w;
        } else {
            const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(rix, (tid + 256u * q) * 8u, 0, kStream);
            ix[q][0] = t.x; ix[q][1] = t.y;
        }
    }
    __syncthreads();
    uint32_t o[kGlobalPasses][4];
#pragma unroll
    for (int q = 0; q < kGlobalPasses; ++q) {
        const uint32_t unit = tid + 256u * q;
        o[q][0] = o[q][1] = o[q][2] = o[q][3] = 0u;
        if (unit * UE < valid) {                      // the source of a valid element is valid: same tile
#pragma unroll
            for (int s = 0; s < UE; ++s) {
                const uint32_t x = (ix[q][s] ^ own_t ^ own_q[q] ^ own_s[s]) & a.axis_mask;
                uint32_t t = table[x & 31u] ^ table[32u + ((x >> 5) & 31u)] ^ table[64u + ((x >> 10) & 31u)] ^ table[96u + ((x >> 15) & 31u)];
                for (int k = 4; k < ntab; ++k) t ^= table[32u * k + ((x >> (5 * k)) & 31u)];
                const unsigned long long src = ((unsigned long long)first + unit * UE + s) ^ (unsigned long long)t;
                const unsigned char *p = in + src * W;
                if constexpr (W == 8) {
                    const u32x2 v = *reinterpret_cast<const u32x2 *>(p);
                    o[q][2 * s] = v.x; o[q][2 * s + 1] = v.y;
                } else if constexpr (W == 4) {
                    o[q][s] = *reinterpret_cast<const uint32_t *>(p);
                } else if constexpr (W == 2) {
                    o[q][s >> 1] |= (uint32_t)*reinterpret_cast<const uint16_t *>(p) << ((s & 1) * 16);
                } else {
                    o[q][0] |= (uint32_t)*p << (s * 8);
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < kGlobalPasses; ++q) {
        const uint32_t unit = tid + 256u * q;
        if constexpr (W >= 4) {
            const u32x4 v = {o[q][0], o[q][1], o[q][2], o[q][3]};
            buf_store16(rout, unit * 16u, v);
        } else if constexpr (W == 2) {
            const u32x2 v = {o[q][0], o[q][1]};
            __builtin_amdgcn_raw_buffer_store_b64(v, rout, unit * 8u, 0, kStream);
        } else {
            __builtin_amdgcn_raw_buffer_store_b32(o[q][0], rout, unit * 4u, 0, kStream);
        }
    }
}

ll_status launch_gather_global(const GatherGenArgs &a, int elem_bytes, void *stream)
{
    if (a.nblocks <= 0 || a.nblocks > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", a.nblocks);
    if (a.na < 0 || a.na > kMaxAxisBits) return fail(LL_ERR_UNSUPPORTED, "gather axis of 2^%d elements", a.na);
    if (a.block_bits < gather_global_chunk_bits(elem_bytes)) return fail(LL_ERR_INVALID_ARG, "internal: gather block smaller than a workgroup's share");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)a.nblocks), block(256);
    switch (elem_bytes) {
    case 1: launch((k_gather_global<1>), grid, block, 0, s, a); break;
    case 2: launch((k_gather_global<2>), grid, block, 0, s, a); break;
    case 4: launch((k_gather_global<4>), grid, block, 0, s, a); break;
    case 8: launch((k_gather_global<8>), grid, block, 0, s, a); break;
    default: return fail(LL_ERR_INVALID_ARG, "elem_bytes %d", elem_bytes);
    }
    return check_launch("global gather kernel launch");
}

// Gather for aligned ranges a few times the size of LDS (the axis leaves LDS, but the range still
// sits in an XCD's L2).  A workgroup of 1024 threads owns 8 units per thread of consecutive output
// elements: it loads their indices once (coalesced), turns them into byte offsets of the sources
// inside the aligned range (delta tables as in the kernels above), then walks through the WHOLE
// range in chunks of 128 KiB: the chunk is stored to LDS from registers filled by coalesced 16-byte
// loads one phase earlier, and every element reads LDS once per phase - at its source when that
// lies in the chunk, else at 16 bytes of zeros behind the chunk - and ORs the value into its output.
// Every workgroup reads the whole range, so the range comes from L2
// (range elements / workgroup elements) times, in full lines, against one line per ELEMENT in the
// memory-direct kernel.  One workgroup fits a CU.
template <int W, bool FIELD>
__global__ __launch_bounds__(1 << kPhasedThreadBits) void k_gather_phased(const GatherGenArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int UB = (W == 8) ? 1 : 2;
    constexpr int UE = 1 << UB;
    constexpr int TB = kPhasedThreadBits;
    constexpr uint32_t T = 1u << TB;
    constexpr int P = kPhasedUnits;
    constexpr int CB = UB + TB + 3;                   // log2 elements per workgroup
    static_assert(kPhasedUnits == 8, "CB assumes eight units per thread");
    constexpr int WL = (W == 1) ? 0 : (W == 2) ? 1 : (W == 4) ? 2 : 3;
    static_assert(kPhasedChunkBytes == 128 * 1024, "SB assumes 128 KiB chunks");
    constexpr int SB = 17 - WL;                       // log2 elements per chunk
    constexpr int VPT = kPhasedChunkBytes / 16 / (int)T;   // 16-byte vectors per thread and chunk
    // LDS: the chunk, then 16 bytes of zeros (where every element whose source is NOT in the current
    // chunk reads), then the delta tables
    uint32_t *table = reinterpret_cast<uint32_t *>(lds + kPhasedChunkBytes + 16);
    const uint32_t tid = threadIdx.x;
    const int ntab = a.na > 0 ? (a.na + 4) / 5 : 1;
    // at least four tables are filled (those beyond the axis bits with zeros) so that the first four
    // lookups of an element need no condition and issue together
    if (tid < 32u * (uint32_t)(ntab > 4 ? ntab : 4)) {
        const uint32_t x = (tid & 31u) << (5u * (tid >> 5));
        uint32_t dl = 0;
        for (int b = 0; b < a.na; ++b) dl ^= a.delta[b] & (0u - ((x >> b) & 1u));
        table[tid] = dl;
    }
    if (tid < 4u) reinterpret_cast<uint32_t *>(lds + kPhasedChunkBytes)[tid] = 0u;
    const long long first = block_of_workgroup((long long)blockIdx.x, a.nblocks, a.xcd_chunk) << CB;
    const long long left = a.total_elems - first;
    const uint32_t valid = left >= (1ll << CB) ? (1u << CB) : (uint32_t)left;     // a multiple of UE
    const __amdgpu_buffer_rsrc_t rix = make_rsrc(reinterpret_cast<const unsigned char *>(a.idx) + (size_t)first * 4, valid * 4);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(static_cast<unsigned char *>(a.out) + (size_t)first * W, valid * W);
    // the aligned block around this workgroup's elements; what lies beyond the last tile reads as zero
    const uint32_t block_mask = (1u << a.block_bits) - 1u;
    const long long block_base = first & ~(long long)block_mask;
    const long long block_left = a.total_elems - block_base;
    const uint32_t block_valid = block_left >= (1ll << a.block_bits) ? (1u << a.block_bits) : (uint32_t)block_left;
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(static_cast<const unsigned char *>(a.in) + (size_t)block_base * W, block_valid * W);
    const uint32_t nchunks = 1u << (a.block_bits - SB);

    u32x4 stage[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) stage[i] = buf_load16(rin, (tid + T * i) * 16u);

    uint32_t own_t = a.own_const;
    {
        const unsigned long long f = (unsigned long long)first;
        for (int b = CB; b < 32; ++b) own_t ^= a.own_bit[b] & (0u - (uint32_t)((f >> b) & 1ull));
#pragma unroll
        for (int b = 0; b < TB; ++b) own_t ^= a.own_bit[UB + b] & (0u - ((tid >> b) & 1u));
    }
    const uint32_t own_s[4] = {0u, a.own_bit[0], a.own_bit[1], a.own_bit[0] ^ a.own_bit[1]};
    uint32_t ix[P][UE];
#pragma unroll
    for (int q = 0; q < P; ++q) {
        if constexpr (UE == 4) {
            const u32x4 t = buf_load16(rix, (tid + T * q) * 16u);
            ix[q][0] = t.x; ix[q][1] = t.y; ix[q][2] = t.z; ix[q][3] = t.w;
        } else {
            const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(rix, (tid + T * q) * 8u, 0, kStream);
            ix[q][0] = t.x; ix[q][1] = t.y;
        }
    }
    __syncthreads();                                  // delta tables
    // block-relative source index of every element (it replaces the index in ix)
    const uint32_t rel = (uint32_t)(first - block_base);
#pragma unroll
    for (int q = 0; q < P; ++q) {
        uint32_t own_q = own_t;
#pragma unroll
        for (int b = 0; b < 3; ++b) own_q ^= a.own_bit[UB + TB + b] & (0u - (((uint32_t)q >> b) & 1u));
        const uint32_t unit = tid + T * q;
#pragma unroll
        for (int s = 0; s < UE; ++s) {
            if constexpr (FIELD) {
                // the axis coordinate is a bit field of the element index: the source is the element's
                // own index with that field replaced by the gather index
                const uint32_t field = a.axis_mask << a.field_shift;
                ix[q][s] = ((((rel + unit * UE + s) & ~field) | ((ix[q][s] & a.axis_mask) << a.field_shift)) & block_mask) * W;
            } else {
                const uint32_t x = (ix[q][s] ^ own_q ^ own_s[s]) & a.axis_mask;
                uint32_t t = table[x & 31u] ^ table[32u + ((x >> 5) & 31u)] ^ table[64u + ((x >> 10) & 31u)] ^ table[96u + ((x >> 15) & 31u)];
                for (int k = 4; k < ntab; ++k) t ^= table[32u * k + ((x >> (5 * k)) & 31u)];
                ix[q][s] = (((rel + unit * UE + s) ^ t) & block_mask) * W;    // byte offset of the source in the range
            }
        }
    }
    uint32_t o[P][4];
#pragma unroll
    for (int q = 0; q < P; ++q) o[q][0] = o[q][1] = o[q][2] = o[q][3] = 0u;

    for (uint32_t c = 0; c < nchunks; ++c) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) *reinterpret_cast<u32x4 *>(lds + (tid + T * i) * 16u) = stage[i];
        __syncthreads();
        if (c + 1 < nchunks) {
#pragma unroll
            for (int i = 0; i < VPT; ++i) stage[i] = buf_load16(rin, (c + 1) * (uint32_t)kPhasedChunkBytes + (tid + T * i) * 16u);
        }
        // Every element reads in every phase: at its source when that lies in this chunk, otherwise at
        // the zeros behind the chunk (offsets below the chunk wrap to huge values, so one unsigned
        // minimum sends both kinds of miss there), and ORs what it read into its output, which starts
        // as zero.  Three vector instructions and one LDS read per element and phase; the reads of a
        // unit are independent and issue back to back.
        const uint32_t cbytes = c * (uint32_t)kPhasedChunkBytes;
#pragma unroll
        for (int q = 0; q < P; ++q) {
#pragma unroll
            for (int s = 0; s < UE; ++s) {
                const uint32_t at = ix[q][s] - cbytes;
                const unsigned char *p = lds + (at < (uint32_t)kPhasedChunkBytes ? at : (uint32_t)kPhasedChunkBytes);
                if constexpr (W == 8) {
                    const u32x2 v = *reinterpret_cast<const u32x2 *>(p);
                    o[q][2 * s] |= v.x;
                    o[q][2 * s + 1] |= v.y;
                } else if constexpr (W == 4) {
                    o[q][s] |= *reinterpret_cast<const uint32_t *>(p);
                } else if constexpr (W == 2) {
                    o[q][s >> 1] |= (uint32_t)*reinterpret_cast<const uint16_t *>(p) << ((s & 1) * 16);
                } else {
                    o[q][0] |= (uint32_t)*p << (s * 8);
                }
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < P; ++q) {
        const uint32_t unit = tid + T * q;
        if constexpr (W >= 4) {
            const u32x4 v = {o[q][0], o[q][1], o[q][2], o[q][3]};
            buf_store16(rout, unit * 16u, v);
        } else if constexpr (W == 2) {
            const u32x2 v = {o[q][0], o[q][1]};
            __builtin_amdgcn_raw_buffer_store_b64(v, rout, unit * 8u, 0, kStream);
        } else {
            __builtin_amdgcn_raw_buffer_store_b32(o[q][0], rout, unit * 4u, 0, kStream);
        }
    }
}

template <int W>
static ll_status launch_gather_phased_w(const GatherGenArgs &a, hipStream_t s)
{
    const size_t lds_bytes = (size_t)kPhasedChunkBytes + 16 + 6 * 32 * sizeof(uint32_t);
    const bool field = a.field_shift >= 0;
    static std::atomic<uint64_t> allowed_field{0}, allowed_table{0};
    if (ll_status st = allow_large_lds(field ? reinterpret_cast<const void *>(k_gather_phased<W, true>)
                                             : reinterpret_cast<const void *>(k_gather_phased<W, false>),
                                       (int)lds_bytes, field ? allowed_field : allowed_table);
        st != LL_OK)
        return st;
    const dim3 grid((unsigned)a.nblocks), block(1u << kPhasedThreadBits);
    if (field)
        launch((k_gather_phased<W, true>), grid, block, lds_bytes, s, a);
    else
        launch((k_gather_phased<W, false>), grid, block, lds_bytes, s, a);
    return check_launch("phased gather kernel launch");
}

ll_status launch_gather_phased(const GatherGenArgs &a, int elem_bytes, void *stream)
{
    if (a.nblocks <= 0 || a.nblocks > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", a.nblocks);
    if (a.na < 0 || a.na > kMaxAxisBits) return fail(LL_ERR_UNSUPPORTED, "gather axis of 2^%d elements", a.na);
    const int wl = elem_bytes == 1 ? 0 : elem_bytes == 2 ? 1 : elem_bytes == 4 ? 2 : 3;
    // a workgroup's elements lie in one aligned block, the block is a whole number of chunks and its
    // bytes fit a buffer descriptor
    if (a.field_shift >= 0 && a.field_shift + a.na > 32) return fail(LL_ERR_INVALID_ARG, "internal: gather axis field out of range");
    if (a.block_bits < gather_phased_chunk_bits(elem_bytes) || (1ll << (a.block_bits + wl)) < kPhasedChunkBytes || a.block_bits + wl > 31)
        return fail(LL_ERR_INVALID_ARG, "internal: gather block of 2^%d elements does not suit the phased kernel", a.block_bits);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (elem_bytes) {
    case 1: return launch_gather_phased_w<1>(a, s);
    case 2: return launch_gather_phased_w<2>(a, s);
    case 4: return launch_gather_phased_w<4>(a, s);
    case 8: return launch_gather_phased_w<8>(a, s);
    default: return fail(LL_ERR_INVALID_ARG, "elem_bytes %d", elem_bytes);
    }
}

ll_status launch_gather(const GatherArgs &a, int elem_bytes, int waves, int lds_alloc, void *stream)
{
    if (waves != 1 && waves != 2 && waves != 4) return fail(LL_ERR_INVALID_ARG, "internal: %d waves per gather workgroup", waves);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (elem_bytes) {
    case 1: return launch_gather_w<1>(a, waves, lds_alloc, s);
    case 2: return launch_gather_w<2>(a, waves, lds_alloc, s);
    case 4: return launch_gather_w<4>(a, waves, lds_alloc, s);
    case 8: return launch_gather_w<8>(a, waves, lds_alloc, s);
    default: return fail(LL_ERR_INVALID_ARG, "elem_bytes %d", elem_bytes);
    }
}

}  // namespace ll

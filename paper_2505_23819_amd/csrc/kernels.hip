// HIP kernels for gfx950 (CDNA4, wave64).  Pure data movement: 16-byte global loads and stores,
// LDS staging or cross-lane shuffles in between, no MFMA.
#include <hip/hip_runtime.h>

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

static ll_status check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LL_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
    return LL_OK;
}

// ---------------------------------------------------------------------------------------------
// plain copy (bandwidth yardstick, and the NOOP conversion)
// ---------------------------------------------------------------------------------------------

constexpr int kCopyVec = 4;   // vectors per thread

__global__ __launch_bounds__(256) void k_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, long long nvec)
{
    const long long base = (long long)blockIdx.x * (kCopyVec * 256) + threadIdx.x;
    u32x4 r[kCopyVec];
#pragma unroll
    for (int i = 0; i < kCopyVec; ++i) {
        const long long k = base + i * 256;
        if (k < nvec) r[i] = load16(src + k);
    }
#pragma unroll
    for (int i = 0; i < kCopyVec; ++i) {
        const long long k = base + i * 256;
        if (k < nvec) store16(dst + k, r[i]);
    }
}

ll_status launch_copy(const void *src, void *dst, long long bytes, void *stream)
{
    const long long nvec = bytes / 16;
    const long long per = kCopyVec * 256;
    const long long grid = (nvec + per - 1) / per;
    if (grid > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "copy of %lld bytes is too large for one launch", bytes);
    hipLaunchKernelGGL(k_copy, dim3((unsigned)grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(src), static_cast<u32x4 *>(dst), nvec);
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
// One workgroup of 256 threads stages one block: coalesced 16-byte loads (thread t, iteration i
// takes vector t + 256 i of the block's source runs), LDS writes at swizzled offsets, barrier,
// LDS reads of the elements of its destination vectors, coalesced 16-byte stores.  Every index
// map is linear over F2, so an offset is the XOR of per-bit table entries.
template <int W, int NV, int V>
__global__ __launch_bounds__(256) void k_lds_elem(const LdsElemArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int VS = (W == 1) ? 4 : (W == 2) ? 3 : (W == 4) ? 2 : 1;
    constexpr int NSUB = 1 << (VS - V);
    constexpr int AB = (1 << V) * W;
    const uint32_t tid = threadIdx.x;

    uint32_t ls = 0, ld = 0, lw = 0, lr = 0;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint32_t m = 0u - ((tid >> b) & 1u);
        ls ^= a.lane_src[b] & m;
        ld ^= a.lane_dst[b] & m;
        lw ^= a.lds_wr_lane[b] & m;
        lr ^= a.lds_rd_lane[b] & m;
    }
    const long long blk = blockIdx.x;
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
    // tiles of this group that exist (the last group may be partly empty)
    const long long left = a.ntiles - (group << a.group_bits);
    const uint32_t tiles_here = left > (1ll << a.group_bits) ? (1u << a.group_bits) : (uint32_t)left;

    uint32_t r[NV][4];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const uint32_t off = cs ^ ls ^ a.iter_src[i];
        u32x4 v = {0u, 0u, 0u, 0u};
        if ((off >> a.d) < tiles_here) v = load16(sbase + (size_t)off * W);
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
        for (int s = 0; s < NSUB; ++s) lds_get<AB>(lds, base ^ a.lds_rd_sub[s], r[i], s);
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const uint32_t off = cd ^ ld ^ a.iter_dst[i];
        if ((off >> a.d) < tiles_here) {
            u32x4 v = {r[i][0], r[i][1], r[i][2], r[i][3]};
            store16(dbase + (size_t)off * W, v);
        }
    }
}

template <int W, int NV, int V>
static ll_status launch_lds_elem_t(const LdsElemArgs &a, int lds_bytes, hipStream_t stream)
{
    static bool attr_set = false;
    if (!attr_set && lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_lds_elem<W, NV, V>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
        if (e != hipSuccess) return fail(LL_ERR_DEVICE, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_set = true;
    }
    hipLaunchKernelGGL((k_lds_elem<W, NV, V>), dim3((unsigned)a.nblocks), dim3(256), (size_t)lds_bytes, stream, a);
    return check_launch("LDS conversion kernel launch");
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
    if (threads != 256) return fail(LL_ERR_UNSUPPORTED, "LDS kernel runs 256 threads per workgroup");
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
    const long long chunk = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
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

    uint32_t own_lw = 0;        // own axis coordinate: lane and wave contributions
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

template <int W, int NREG>
static ll_status launch_gather_t(const GatherArgs &a, hipStream_t stream)
{
    if constexpr ((1 << NREG) * W < 4 || (1 << NREG) * W > 256) {
        return fail(LL_ERR_UNSUPPORTED, "gather needs 4 to 256 bytes per lane (got %d)", (1 << NREG) * W);
    } else {
        const long long grid = (a.nchunks + 3) / 4;
        if (grid > 0x7fffffffLL) return fail(LL_ERR_INVALID_ARG, "%lld workgroups do not fit one launch", grid);
        hipLaunchKernelGGL((k_gather<W, NREG>), dim3((unsigned)grid), dim3(256), 0, stream, a);
        return check_launch("gather kernel launch");
    }
}

template <int W>
static ll_status launch_gather_w(const GatherArgs &a, hipStream_t stream)
{
    switch (a.nreg) {
    case 0: return launch_gather_t<W, 0>(a, stream);
    case 1: return launch_gather_t<W, 1>(a, stream);
    case 2: return launch_gather_t<W, 2>(a, stream);
    case 3: return launch_gather_t<W, 3>(a, stream);
    case 4: return launch_gather_t<W, 4>(a, stream);
    case 5: return launch_gather_t<W, 5>(a, stream);
    case 6: return launch_gather_t<W, 6>(a, stream);
    default: return fail(LL_ERR_UNSUPPORTED, "gather supports at most 6 register bits (got %d)", a.nreg);
    }
}

ll_status launch_gather(const GatherArgs &a, int elem_bytes, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (elem_bytes) {
    case 1: return launch_gather_w<1>(a, s);
    case 2: return launch_gather_w<2>(a, s);
    case 4: return launch_gather_w<4>(a, s);
    case 8: return launch_gather_w<8>(a, s);
    default: return fail(LL_ERR_INVALID_ARG, "elem_bytes %d", elem_bytes);
    }
}

}  // namespace ll

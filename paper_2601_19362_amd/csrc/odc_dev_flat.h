// Single-tensor (T = 1) kernels: gather, scatter-accumulate, reset.
#pragma once

#include "odc_dev_common.h"

namespace odc {
namespace {

// ------------------------------------------------------------------------------------ flat
// One flat parameter (T = 1).  grid = (tiles, ranks); a tile is TPB * U work items,
// item (u, lane) = tile_base + u * TPB + lane, so each wave instruction touches one
// contiguous run.  Full tiles run without per-item guards: all U loads are issued back to
// back and only then consumed, which keeps U independent requests per lane in flight.
//
// Tile order.  The hardware hands consecutive workgroup ids to the 8 XCDs in turn.  With
// remap = 0 tile = workgroup id: the whole chip sweeps one compact address window.  With
// remap = 1 the tile space is cut into 8 contiguous parts and workgroup id w takes tile
// (w mod 8) * part + w / 8, so each XCD sweeps its own contiguous part.

__device__ __forceinline__ int64_t tile_of(int64_t slot, int64_t ntiles, int remap)
{
    if (!remap) return slot;
    const int64_t part = (ntiles + 7) >> 3;
    return (slot & 7) * part + (slot >> 3);
}

__device__ __forceinline__ int64_t slots_of(int64_t ntiles, int remap)
{
    return remap ? ((ntiles + 7) >> 3) << 3 : ntiles;
}

template <int TPB, int U, bool NT, bool GUARD, bool SC1>
__device__ __forceinline__ void gather_tile(const uint16_t *__restrict__ bsrc, u32x4 *__restrict__ bdst,
                                            int64_t v0, int64_t nvec)
{
    u32x4 reg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = v0 + u * TPB;
        if (!GUARD || v < nvec) reg[u] = ld_u128_unaligned<NT>(bsrc + 8 * v);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = v0 + u * TPB;
        if (!GUARD || v < nvec) {
            if constexpr (SC1) st_sc1_nt(bdst + v, reg[u]);
            else st<NT>(bdst + v, reg[u]);
        }
    }
}

template <int TPB, int U, bool NT, bool SC1>
__global__ __launch_bounds__(TPB) void k_gather_flat(RankPtrs shards, uint16_t *__restrict__ full,
                                                     int64_t S, int64_t N, int r0, int remap)
{
    const int64_t base = static_cast<int64_t>(r0 + static_cast<int>(blockIdx.y)) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    const uint16_t *__restrict__ src = static_cast<const uint16_t *>(shards.p[blockIdx.y]);
    uint16_t *__restrict__ dst = full + base;
    // Elements before the first 128-byte boundary of the destination: every wavefront's store
    // then covers whole cache lines.  (Aligning the items to 16 bytes only is enough for
    // correctness, but when an owner's range starts off a line boundary each wavefront's
    // kilobyte begins and ends in a line it shares with its neighbours, and those partly
    // written lines cost a fifth of the rate: 5.5 against 6.7 TB/s on a 233 M-element tensor.)
    int64_t head = static_cast<int64_t>((128u - (reinterpret_cast<uintptr_t>(dst) & 127u)) & 127u) >> 1;
    if (head > valid) head = valid;
    const int64_t nvec = (valid - head) >> 3;
    const int tail = static_cast<int>((valid - head) & 7);
    const uint16_t *bsrc = src + head;
    u32x4 *bdst = reinterpret_cast<u32x4 *>(dst + head);

    const int64_t ntiles = (nvec + TPB * U - 1) / (TPB * U);
    const int64_t nslots = slots_of(ntiles, remap);
    for (int64_t slot = blockIdx.x; slot < nslots; slot += gridDim.x) {
        const int64_t t0 = tile_of(slot, ntiles, remap) * (TPB * U);
        if (t0 + TPB * U <= nvec) gather_tile<TPB, U, NT, false, SC1>(bsrc, bdst, t0 + threadIdx.x, nvec);
        else if (t0 < nvec) gather_tile<TPB, U, NT, true, SC1>(bsrc, bdst, t0 + threadIdx.x, nvec);
    }
    if (blockIdx.x == 0) {
        const int t = threadIdx.x;
        if (t < head) st_u16(dst + t, ld_u16(src + t));
        if (t < tail) {
            const int64_t k = head + 8 * nvec + t;
            st_u16(dst + k, ld_u16(src + k));
        }
    }
}

// Ordered contribution to four accumulator elements.  Unweighted (Section 2.1 with w_m = 1):
// one binary32 add each.  Weighted: one fused multiply-add each, acc = fma(w, g, acc), a
// single rounding of w*g + acc.
template <bool WEIGHTED>
__device__ __forceinline__ f32x4 add4(f32x4 a, u32x2 g, float w)
{
    if constexpr (WEIGHTED) {
        a.x = __builtin_fmaf(w, widen_lo(g.x), a.x);
        a.y = __builtin_fmaf(w, widen_hi(g.x), a.y);
        a.z = __builtin_fmaf(w, widen_lo(g.y), a.z);
        a.w = __builtin_fmaf(w, widen_hi(g.y), a.w);
    } else {
        a.x = a.x + widen_lo(g.x);
        a.y = a.y + widen_hi(g.x);
        a.z = a.z + widen_lo(g.y);
        a.w = a.w + widen_hi(g.y);
    }
    return a;
}

// A work item is one accumulator vector (4 floats, 16 bytes) and 8 bytes of gradient;
// consecutive lanes take consecutive vectors, so every wave instruction is contiguous
// (1 KiB of accumulator, 512 B of gradient).
template <int TPB, int U, bool NT, bool WEIGHTED, bool GUARD>
__device__ __forceinline__ void accum_tile(float *__restrict__ acc, const uint16_t *__restrict__ g,
                                           int64_t q0, int64_t nitem, float w)
{
    f32x4 *__restrict__ accv = reinterpret_cast<f32x4 *>(acc);
    u32x2 gv[U];
    f32x4 av[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t q = q0 + u * TPB;
        if (!GUARD || q < nitem) {
            gv[u] = ld_u64_unaligned<NT>(g + 4 * q);
            av[u] = ld<NT>(accv + q);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t q = q0 + u * TPB;
        if (!GUARD || q < nitem) st<NT>(accv + q, add4<WEIGHTED>(av[u], gv[u], w));
    }
}

// Unordered form of a tile (device-scope float atomics; a weighted product is rounded
// first): consecutive lanes take consecutive ELEMENTS, so that one atomic
// instruction of a wavefront covers 256 contiguous bytes (two cache lines) instead of four
// floats out of every 16 bytes over 1 KiB (eight lines): the atomic units of the L2 work per
// cache line, and the coalesced form is several times faster.
template <int TPB, int E, bool WEIGHTED, bool GUARD>
__device__ __forceinline__ void accum_tile_atomic(float *__restrict__ acc, const uint16_t *__restrict__ g,
                                                  int64_t e0, int64_t n, float w)
{
    uint16_t gv[E];
#pragma unroll
    for (int u = 0; u < E; ++u) {
        const int64_t e = e0 + u * TPB;
        if (!GUARD || e < n) gv[u] = ld_u16(g + e);
    }
#pragma unroll
    for (int u = 0; u < E; ++u) {
        const int64_t e = e0 + u * TPB;
        if (!GUARD || e < n) unsafeAtomicAdd(acc + e, WEIGHTED ? w * widen_one(gv[u]) : widen_one(gv[u]));
    }
}

template <int TPB, int U, bool NT, bool ATOMIC, bool WEIGHTED>
__global__ __launch_bounds__(TPB) void k_accum_flat(RankPtrs accs, const uint16_t *__restrict__ grad,
                                                    int64_t S, int64_t N, int r0, int remap, float w)
{
    const int64_t base = static_cast<int64_t>(r0 + static_cast<int>(blockIdx.y)) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    float *__restrict__ acc = static_cast<float *>(accs.p[blockIdx.y]);
    const uint16_t *__restrict__ g = grad + base;
    const int64_t nitem = valid >> 2;
    const int tail = static_cast<int>(valid & 3);

    const int64_t ntiles = (nitem + TPB * U - 1) / (TPB * U);
    const int64_t nslots = slots_of(ntiles, remap);
    for (int64_t slot = blockIdx.x; slot < nslots; slot += gridDim.x) {
        const int64_t t0 = tile_of(slot, ntiles, remap) * (TPB * U);
        if constexpr (ATOMIC) {
            if (t0 + TPB * U <= nitem) accum_tile_atomic<TPB, 4 * U, WEIGHTED, false>(acc, g, 4 * t0 + threadIdx.x, 4 * nitem, w);
            else if (t0 < nitem) accum_tile_atomic<TPB, 4 * U, WEIGHTED, true>(acc, g, 4 * t0 + threadIdx.x, 4 * nitem, w);
        } else {
            if (t0 + TPB * U <= nitem) accum_tile<TPB, U, NT, WEIGHTED, false>(acc, g, t0 + threadIdx.x, nitem, w);
            else if (t0 < nitem) accum_tile<TPB, U, NT, WEIGHTED, true>(acc, g, t0 + threadIdx.x, nitem, w);
        }
    }
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < tail) {
        const int64_t k = 4 * nitem + threadIdx.x;
        add_one<ATOMIC, WEIGHTED>(acc + k, widen_one(ld_u16(g + k)), w);
    }
}

template <int TPB, int U, bool NT>
__global__ __launch_bounds__(TPB) void k_reset_flat(RankPtrs accs, int64_t S, int64_t N, int r0, int remap)
{
    const int64_t base = static_cast<int64_t>(r0 + static_cast<int>(blockIdx.y)) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    float *__restrict__ acc = static_cast<float *>(accs.p[blockIdx.y]);
    const int64_t nvec = valid >> 2;
    const int tail = static_cast<int>(valid & 3);
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    const int64_t ntiles = (nvec + TPB * U - 1) / (TPB * U);
    const int64_t nslots = slots_of(ntiles, remap);
    for (int64_t slot = blockIdx.x; slot < nslots; slot += gridDim.x) {
        const int64_t v0 = tile_of(slot, ntiles, remap) * (TPB * U) + threadIdx.x;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t v = v0 + u * TPB;
            if (v < nvec) st_stream<NT ? 2 : 0>(reinterpret_cast<f32x4 *>(acc) + v, zero);
        }
    }
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < tail) st_f32(acc + 4 * nvec + threadIdx.x, 0.0f);
}

}  // namespace
}  // namespace odc

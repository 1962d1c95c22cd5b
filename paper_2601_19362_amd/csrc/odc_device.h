// gfx950 (MI355X) kernels for the ODC hot path: gather, scatter-accumulate, reset.
//
// Nothing here is a contraction, so there is no MFMA: every kernel is a pure HBM stream
// (0 or 0.1 flop per byte) and is shaped for that -- 64-lane wavefronts issuing 128-bit
// loads/stores that are contiguous across the wave, several independent vectors in flight
// per lane, non-temporal hints on data that is touched once, and thousands of workgroups so
// that all 256 CUs in the 8 XCDs stay busy.  Rank base pointers travel in the kernel
// arguments; blockIdx.y selects the owner rank, so the flat kernels do no division at all.
//
// What is computed (paper Section 3, Section 3.1, Appendix B, Section 2.1 with w_m = 1):
//   gather:      full[r*S + i]  = shard_r[i]                       i < valid_r
//   accumulate:  acc_r[i]       = fl32(acc_r[i] + widen(g[r*S+i])) i < valid_r
//   reset:       acc_r[i]       = +0.0f                            i < valid_r
// with S = ceil(N / R) and valid_r = clamp(N - r*S, 0, S).  Padding is never touched.
//
// Misalignment: shard boundaries r*S fall on any 2-byte boundary.  The side that is written
// is always accessed with naturally aligned 16-byte vectors (head and tail elements are
// peeled); the read-only side uses byte-unaligned wide loads, which global memory on this
// target supports in hardware, so no LDS staging is needed for the shift.
#pragma once

#include <cstdint>

#include "odc_internal.h"

namespace odc {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Wide accesses whose address is only 2-byte aligned.
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef u32x2 u32x2_a2 __attribute__((aligned(2)));

struct RankPtrs {
    void *p[kRanksPerLaunch];
};

template <bool NT, typename V>
__device__ __forceinline__ V ld(const V *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename V>
__device__ __forceinline__ void st(V *p, V v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

template <bool NT>
__device__ __forceinline__ u32x4 ld_u128_unaligned(const uint16_t *p)
{
    const u32x4_a2 *q = reinterpret_cast<const u32x4_a2 *>(p);
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

template <bool NT>
__device__ __forceinline__ u32x2 ld_u64_unaligned(const uint16_t *p)
{
    const u32x2_a2 *q = reinterpret_cast<const u32x2_a2 *>(p);
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

template <bool NT>
__device__ __forceinline__ void st_u128_unaligned(uint16_t *p, u32x4 v)
{
    u32x4_a2 *q = reinterpret_cast<u32x4_a2 *>(p);
    if constexpr (NT) __builtin_nontemporal_store(v, q);
    else *q = v;
}

// bf16 -> binary32 is exact: the 16 bits are the high half of the word.
__device__ __forceinline__ float widen_lo(uint32_t two) { return __uint_as_float(two << 16); }
__device__ __forceinline__ float widen_hi(uint32_t two) { return __uint_as_float(two & 0xFFFF0000u); }
__device__ __forceinline__ float widen_one(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

template <bool ATOMIC>
__device__ __forceinline__ void add_one(float *a, float v)
{
    if constexpr (ATOMIC) unsafeAtomicAdd(a, v);
    else *a = *a + v;
}

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

template <int TPB, int U, bool NT, bool GUARD>
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
        if (!GUARD || v < nvec) st<NT>(bdst + v, reg[u]);
    }
}

template <int TPB, int U, bool NT>
__global__ __launch_bounds__(TPB) void k_gather_flat(RankPtrs shards, uint16_t *__restrict__ full,
                                                     int64_t S, int64_t N, int r0, int remap)
{
    const int64_t base = static_cast<int64_t>(r0 + static_cast<int>(blockIdx.y)) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    const uint16_t *__restrict__ src = static_cast<const uint16_t *>(shards.p[blockIdx.y]);
    uint16_t *__restrict__ dst = full + base;
    // Elements before the first 16-byte boundary of the destination.
    int64_t head = static_cast<int64_t>((16u - (reinterpret_cast<uintptr_t>(dst) & 15u)) & 15u) >> 1;
    if (head > valid) head = valid;
    const int64_t nvec = (valid - head) >> 3;
    const int tail = static_cast<int>((valid - head) & 7);
    const uint16_t *bsrc = src + head;
    u32x4 *bdst = reinterpret_cast<u32x4 *>(dst + head);

    const int64_t ntiles = (nvec + TPB * U - 1) / (TPB * U);
    const int64_t nslots = slots_of(ntiles, remap);
    for (int64_t slot = blockIdx.x; slot < nslots; slot += gridDim.x) {
        const int64_t t0 = tile_of(slot, ntiles, remap) * (TPB * U);
        if (t0 + TPB * U <= nvec) gather_tile<TPB, U, NT, false>(bsrc, bdst, t0 + threadIdx.x, nvec);
        else if (t0 < nvec) gather_tile<TPB, U, NT, true>(bsrc, bdst, t0 + threadIdx.x, nvec);
    }
    if (blockIdx.x == 0) {
        const int t = threadIdx.x;
        if (t < head) dst[t] = src[t];
        if (t < tail) {
            const int64_t k = head + 8 * nvec + t;
            dst[k] = src[k];
        }
    }
}

__device__ __forceinline__ f32x4 add4(f32x4 a, u32x2 g)
{
    a.x = a.x + widen_lo(g.x);
    a.y = a.y + widen_hi(g.x);
    a.z = a.z + widen_lo(g.y);
    a.w = a.w + widen_hi(g.y);
    return a;
}

__device__ __forceinline__ void atomic_add4(float *a, u32x2 g)
{
    unsafeAtomicAdd(a + 0, widen_lo(g.x));
    unsafeAtomicAdd(a + 1, widen_hi(g.x));
    unsafeAtomicAdd(a + 2, widen_lo(g.y));
    unsafeAtomicAdd(a + 3, widen_hi(g.y));
}

// A work item is one accumulator vector (4 floats, 16 bytes) and 8 bytes of gradient;
// consecutive lanes take consecutive vectors, so every wave instruction is contiguous
// (1 KiB of accumulator, 512 B of gradient).
template <int TPB, int U, bool NT, bool ATOMIC, bool GUARD>
__device__ __forceinline__ void accum_tile(float *__restrict__ acc, const uint16_t *__restrict__ g,
                                           int64_t q0, int64_t nitem)
{
    f32x4 *__restrict__ accv = reinterpret_cast<f32x4 *>(acc);
    u32x2 gv[U];
    f32x4 av[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t q = q0 + u * TPB;
        if (!GUARD || q < nitem) {
            gv[u] = ld_u64_unaligned<NT>(g + 4 * q);
            if constexpr (!ATOMIC) av[u] = ld<NT>(accv + q);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t q = q0 + u * TPB;
        if (!GUARD || q < nitem) {
            if constexpr (ATOMIC) atomic_add4(acc + 4 * q, gv[u]);
            else st<NT>(accv + q, add4(av[u], gv[u]));
        }
    }
}

template <int TPB, int U, bool NT, bool ATOMIC>
__global__ __launch_bounds__(TPB) void k_accum_flat(RankPtrs accs, const uint16_t *__restrict__ grad,
                                                    int64_t S, int64_t N, int r0, int remap)
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
        if (t0 + TPB * U <= nitem) accum_tile<TPB, U, NT, ATOMIC, false>(acc, g, t0 + threadIdx.x, nitem);
        else if (t0 < nitem) accum_tile<TPB, U, NT, ATOMIC, true>(acc, g, t0 + threadIdx.x, nitem);
    }
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < tail) {
        const int64_t k = 4 * nitem + threadIdx.x;
        add_one<ATOMIC>(acc + k, widen_one(g[k]));
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
            if (v < nvec) st<NT>(reinterpret_cast<f32x4 *>(acc) + v, zero);
        }
    }
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < tail) acc[4 * nvec + threadIdx.x] = 0.0f;
}

// --------------------------------------------------------------------------------- batched
// T tensors in one launch.  The kernels walk each owner's rank arena in aligned work items
// (8 bf16 for gather, 4 floats for accumulate / reset); every tensor starts at a multiple of
// 8 arena elements, so a work item never straddles two tensors.  A work item finds its
// tensor through the coarse chunk index plus a short binary search over the start offsets.

__device__ __forceinline__ int find_tensor(const BatchTable &tb, int64_t a)
{
    const int64_t c = a >> kChunkShift;
    int lo = tb.chunk_first[c];
    int hi = tb.chunk_first[c + 1];
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tb.shard_off[mid] <= a) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

// Valid elements of tensor d, owner r, starting at slot `slot`, at most `width`.
__device__ __forceinline__ int valid_from(const TensorDesc &d, int r, int64_t slot, int width)
{
    int64_t valid = d.numel - static_cast<int64_t>(r) * d.S;
    if (valid > d.S) valid = d.S;
    const int64_t left = valid - slot;
    return left >= width ? width : (left > 0 ? static_cast<int>(left) : 0);
}

template <int TPB, int U, bool NT>
__global__ __launch_bounds__(TPB) void k_gather_batched(BatchTable tb, RankPtrs arenas,
                                                             uint16_t *__restrict__ full, int r0)
{
    const int r = r0 + static_cast<int>(blockIdx.y);
    const uint16_t *__restrict__ arena = static_cast<const uint16_t *>(arenas.p[blockIdx.y]);
    const int64_t nitem = (tb.arena_elems + 7) >> 3;
    const int64_t ntiles = (nitem + TPB * U - 1) / (TPB * U);
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t q0 = tile * (TPB * U) + threadIdx.x;
        u32x4 reg[U];
        uint16_t *dst[U];
        int cnt[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t a = 8 * (q0 + u * TPB);
            cnt[u] = 0;
            if (a < tb.arena_elems) {
                const TensorDesc d = tb.desc[find_tensor(tb, a)];
                const int64_t slot = a - d.shard_off;
                cnt[u] = valid_from(d, r, slot, 8);
                dst[u] = full + d.full_off + static_cast<int64_t>(r) * d.S + slot;
                if (cnt[u] == 8) reg[u] = ld<NT>(reinterpret_cast<const u32x4 *>(arena + a));
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (cnt[u] == 8) {
                st_u128_unaligned<NT>(dst[u], reg[u]);
            } else if (cnt[u] > 0) {
                const uint16_t *s = arena + 8 * (q0 + u * TPB);
                for (int k = 0; k < cnt[u]; ++k) dst[u][k] = s[k];
            }
        }
    }
}

template <int TPB, int U, bool NT, bool ATOMIC>
__global__ __launch_bounds__(TPB) void k_accum_batched(BatchTable tb, RankPtrs accs,
                                                            const uint16_t *__restrict__ grad, int r0)
{
    const int r = r0 + static_cast<int>(blockIdx.y);
    float *__restrict__ arena = static_cast<float *>(accs.p[blockIdx.y]);
    const int64_t nitem = (tb.arena_elems + 3) >> 2;
    const int64_t ntiles = (nitem + TPB * U - 1) / (TPB * U);
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t q0 = tile * (TPB * U) + threadIdx.x;
        u32x2 gv[U];
        f32x4 av[U];
        const uint16_t *gp[U];
        int cnt[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t a = 4 * (q0 + u * TPB);
            cnt[u] = 0;
            if (a < tb.arena_elems) {
                const TensorDesc d = tb.desc[find_tensor(tb, a)];
                const int64_t slot = a - d.shard_off;
                cnt[u] = valid_from(d, r, slot, 4);
                gp[u] = grad + d.full_off + static_cast<int64_t>(r) * d.S + slot;
                if (cnt[u] == 4) {
                    gv[u] = ld_u64_unaligned<NT>(gp[u]);
                    if constexpr (!ATOMIC) av[u] = ld<NT>(reinterpret_cast<const f32x4 *>(arena + a));
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float *a = arena + 4 * (q0 + u * TPB);
            if (cnt[u] == 4) {
                if constexpr (ATOMIC) {
                    unsafeAtomicAdd(a + 0, widen_lo(gv[u].x));
                    unsafeAtomicAdd(a + 1, widen_hi(gv[u].x));
                    unsafeAtomicAdd(a + 2, widen_lo(gv[u].y));
                    unsafeAtomicAdd(a + 3, widen_hi(gv[u].y));
                } else {
                    f32x4 rv = av[u];
                    rv.x = rv.x + widen_lo(gv[u].x);
                    rv.y = rv.y + widen_hi(gv[u].x);
                    rv.z = rv.z + widen_lo(gv[u].y);
                    rv.w = rv.w + widen_hi(gv[u].y);
                    st<NT>(reinterpret_cast<f32x4 *>(a), rv);
                }
            } else if (cnt[u] > 0) {
                for (int k = 0; k < cnt[u]; ++k) add_one<ATOMIC>(a + k, widen_one(gp[u][k]));
            }
        }
    }
}

template <int TPB, int U, bool NT>
__global__ __launch_bounds__(TPB) void k_reset_batched(BatchTable tb, RankPtrs accs, int r0)
{
    const int r = r0 + static_cast<int>(blockIdx.y);
    float *__restrict__ arena = static_cast<float *>(accs.p[blockIdx.y]);
    const int64_t nitem = (tb.arena_elems + 3) >> 2;
    const int64_t ntiles = (nitem + TPB * U - 1) / (TPB * U);
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t q0 = tile * (TPB * U) + threadIdx.x;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t a = 4 * (q0 + u * TPB);
            if (a < tb.arena_elems) {
                const TensorDesc d = tb.desc[find_tensor(tb, a)];
                const int cnt = valid_from(d, r, a - d.shard_off, 4);
                if (cnt == 4) st<NT>(reinterpret_cast<f32x4 *>(arena + a), zero);
                else
                    for (int k = 0; k < cnt; ++k) arena[a + k] = 0.0f;
            }
        }
    }
}

// ----------------------------------------------------------------------------------- probe
template <int TPB, int U>
__global__ __launch_bounds__(TPB) void k_probe_copy(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                         int64_t nvec)
{
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * (TPB * U) + threadIdx.x;
    u32x4 reg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = v0 + u * TPB;
        if (v < nvec) reg[u] = __builtin_nontemporal_load(src + v);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = v0 + u * TPB;
        if (v < nvec) __builtin_nontemporal_store(reg[u], dst + v);
    }
}

}  // namespace
}  // namespace odc

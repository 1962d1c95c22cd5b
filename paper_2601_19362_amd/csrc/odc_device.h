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

// Every data pointer in these kernels points to device (global) memory.  Pointers that reach
// a lane through LDS or a per-lane table lookup lose that information and would be accessed
// with slower generic-address instructions, so every access goes through a pointer that is
// explicitly in the global address space.  (On the host, in the CPU emulation build, the
// qualifier is empty.)
#ifdef __HIP_DEVICE_COMPILE__
#define ODC_GLOBAL __attribute__((address_space(1)))
#else
#define ODC_GLOBAL
#endif

// Register budget of a kernel, as the number of wavefronts per SIMD it must allow (512 vector
// registers per SIMD: 8 wavefronts = 64 registers each).  Used where the compiler lands one
// register above a boundary.  (Empty in the CPU emulation build.)
#ifdef __HIP__
#define ODC_WAVES_PER_EU(n) __attribute__((amdgpu_waves_per_eu(n)))
#else
#define ODC_WAVES_PER_EU(n)
#endif

template <bool NT, typename V>
__device__ __forceinline__ V ld(const V *p)
{
    const ODC_GLOBAL V *q = (const ODC_GLOBAL V *)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

template <bool NT, typename V>
__device__ __forceinline__ void st(V *p, V v)
{
    ODC_GLOBAL V *q = (ODC_GLOBAL V *)p;
    if constexpr (NT) __builtin_nontemporal_store(v, q);
    else *q = v;
}

// Stores with the non-temporal hint and system-scope write-through (sc1 nt).  For streams
// that are only written (gather output, reset, retrieval, staging) this measured about 3 %
// faster than the plain non-temporal store; the compiler has no builtin for the combination,
// so the store is written as one instruction.  It is an ordinary vector store: the only
// thing the compiler does not know is that it bumps the memory-operation counter, which can
// only make a later wait longer, never too short.
__device__ __forceinline__ void st_sc1_nt(u32x4 *p, u32x4 v)
{
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
#else
    *p = v;
#endif
}

__device__ __forceinline__ void st_sc1_nt(f32x4 *p, f32x4 v)
{
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
#else
    *p = v;
#endif
}

__device__ __forceinline__ void st_sc1_nt(u32x2 *p, u32x2 v)
{
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("global_store_dwordx2 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
#else
    *p = v;
#endif
}

// Store of a write-only stream: WT = 2 sc1 + nt, 1 nt, 0 plain.
template <int WT, typename V>
__device__ __forceinline__ void st_stream(V *p, V v)
{
    if constexpr (WT == 2) st_sc1_nt(p, v);
    else st<WT == 1>(p, v);
}

template <bool NT>
__device__ __forceinline__ u32x4 ld_u128_unaligned(const uint16_t *p)
{
    const ODC_GLOBAL u32x4_a2 *q = (const ODC_GLOBAL u32x4_a2 *)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

template <bool NT>
__device__ __forceinline__ u32x2 ld_u64_unaligned(const uint16_t *p)
{
    const ODC_GLOBAL u32x2_a2 *q = (const ODC_GLOBAL u32x2_a2 *)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

// Single elements (heads, tails, ragged ends, pieces of small tensors).
__device__ __forceinline__ uint16_t ld_u16(const uint16_t *p) { return *(const ODC_GLOBAL uint16_t *)p; }
__device__ __forceinline__ void st_u16(uint16_t *p, uint16_t v) { *(ODC_GLOBAL uint16_t *)p = v; }
__device__ __forceinline__ float ld_f32(const float *p) { return *(const ODC_GLOBAL float *)p; }
__device__ __forceinline__ void st_f32(float *p, float v) { *(ODC_GLOBAL float *)p = v; }

// bf16 -> binary32 is exact: the 16 bits are the high half of the word.
__device__ __forceinline__ float widen_lo(uint32_t two) { return __uint_as_float(two << 16); }
__device__ __forceinline__ float widen_hi(uint32_t two) { return __uint_as_float(two & 0xFFFF0000u); }
__device__ __forceinline__ float widen_one(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

template <bool ATOMIC, bool WEIGHTED>
__device__ __forceinline__ void add_one(float *a, float v, float w)
{
    if constexpr (ATOMIC) unsafeAtomicAdd(a, WEIGHTED ? w * v : v);
    else if constexpr (WEIGHTED) st_f32(a, __builtin_fmaf(w, v, ld_f32(a)));
    else st_f32(a, ld_f32(a) + v);
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

// --------------------------------------------------------------------------------- batched
// T tensors in one launch: thousands of small tensors, or a layer kept as a handful of large
// ones.  Work is cut into tiles of an index space in which every tensor starts at a multiple
// of 8 elements:
//   accumulate / reset / retrieve walk the owners' rank arenas (the side that is written),
//     so all writes are dense, aligned 16-byte vectors.  Every owner's arena has the same
//     tensor placement, so a workgroup takes one tile and a group of RG owners: the tensor
//     of a work item is looked up once and used for all RG owners;
//   gather walks the full buffer (again the side that is written) and pulls each 16-byte
//     item from the owner that holds it, so the pieces of a small tensor that come from
//     many owners still leave as full 16-byte stores of one workgroup.
// The tensors that intersect a tile are staged in LDS once per workgroup (found through the
// coarse per-chunk index): start offsets for a binary search, and the descriptors themselves.
// A tile that lies inside one tensor skips all of that, and if all of it is valid for the
// owners at hand (tile_is_uniform) it runs the plain vector loop of the single-tensor kernels.

// Loads of short shard pieces (a gradient slice or a parameter piece of a small tensor) do NOT
// carry the non-temporal hint in the multi-tensor kernels: neighbouring pieces share cache
// lines, neighbouring wavefronts read them at slightly different times, and a line loaded with
// the streaming hint is dropped from the L2 before its neighbour arrives and is fetched from
// memory again (stress workload: batched gather 59 -> 48 us from this alone).  Dense streams --
// accumulators, whole-tile paths of large tensors, all stores -- keep the hint.
constexpr bool kPieceLoadsNT = false;

constexpr int kChunkElems = 1 << kChunkShift;
constexpr int kBatchThreads = 256;
constexpr int kAccumItems = kChunkElems / (4 * kBatchThreads);  // accumulate tile: 1 chunk

template <int CHUNKS>
struct TileIndex {
    static constexpr int kMax = CHUNKS * (kChunkElems / static_cast<int>(kAlignElems)) + 2;
    int32_t rel[kMax];      // start of each staged tensor relative to the tile start, clamped
    TensorDesc desc[kMax];  // its descriptor, so that an item needs no second trip to memory
};

// Stage the tensors that intersect tile `tile` (CHUNKS chunks) of the rank-arena space.  All
// threads of the workgroup must call it; it ends with a barrier unless only one tensor is
// involved (then the descriptor is read straight from the table, uniformly).
template <int CHUNKS>
__device__ __forceinline__ void stage_tile(const BatchTable &tb, int64_t tile, int64_t nchunks,
                                           TileIndex<CHUNKS> &lds, int &t_lo, int &n)
{
    const int64_t c0 = tile * CHUNKS;
    const int64_t c1 = c0 + CHUNKS < nchunks ? c0 + CHUNKS : nchunks;
    t_lo = tb.chunk_first[c0];
    n = tb.chunk_first[c1] - t_lo + 1;
    if (n == 1) return;
    const int64_t a0 = c0 << kChunkShift;
    for (int k = threadIdx.x; k < n; k += kBatchThreads) {
        const TensorDesc d = tb.desc[t_lo + k];
        const int64_t rel = d.shard_off - a0;
        lds.rel[k] = rel < -0x40000000 ? -0x40000000 : (rel > 0x40000000 ? 0x40000000 : static_cast<int32_t>(rel));
        lds.desc[k] = d;
    }
    __syncthreads();
}

// Descriptor of the tensor that owns tile-relative element `a_rel`.
template <int CHUNKS>
__device__ __forceinline__ TensorDesc tile_desc(const BatchTable &tb, int t_lo, int n, int a_rel,
                                                const TileIndex<CHUNKS> &lds)
{
    if (n == 1) return tb.desc[t_lo];
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (lds.rel[mid] <= a_rel) lo = mid;
        else hi = mid - 1;
    }
    return lds.desc[lo];
}

// Valid elements of tensor d, owner r, starting at slot `slot`, at most `width`.
__device__ __forceinline__ int valid_from(const TensorDesc &d, int r, int64_t slot, int width)
{
    int64_t valid = d.numel - static_cast<int64_t>(r) * d.S;
    if (valid > d.S) valid = d.S;
    const int64_t left = valid - slot;
    return left >= width ? width : (left > 0 ? static_cast<int>(left) : 0);
}

// True when the arena tile that starts at element a0 lies wholly inside the slots of tensor d
// that are valid for every owner in [r_first, r_first + count).  Every item of such a tile is
// a full vector of one tensor, so the kernels skip the per-item lookup and validity checks and
// run the same lean loop as the single-tensor kernels (large tensors of a multi-tensor layout,
// e.g. a decoder layer kept as separate weight matrices, then move at nearly the same rate).
__device__ __forceinline__ bool tile_is_uniform(const TensorDesc &d, int64_t a0, int r_first, int count,
                                                int tile_elems = kChunkElems)
{
    int64_t valid = d.numel - static_cast<int64_t>(r_first + count - 1) * d.S;  // the last owner has the fewest
    if (valid > d.S) valid = d.S;
    return a0 >= d.shard_off && a0 - d.shard_off + tile_elems <= valid;
}

// Work order of the gather kernels.  Consecutive workgroup ids go to the 8 XCDs in turn, and
// each XCD has its own L2.  The shard pieces that neighbouring tiles read sit next to each other
// in every owner's arena and share cache lines, so work units are handed out in blocks: of every
// 8 * block consecutive units, XCD x takes units [x * block, (x + 1) * block), which keeps the
// lines that neighbours share inside one L2 instead of fetching them once per XCD.
// `shift` = log2(block); slot = workgroup id.
__device__ __forceinline__ int64_t span_of(int64_t slot, int shift)
{
    const int64_t x = slot & 7, q = slot >> 3;
    return ((q >> shift) << (shift + 3)) + (x << shift) + (q & ((int64_t{1} << shift) - 1));
}

// ---- gather, full-buffer-major ---------------------------------------------------------
// Per-tensor record of the gather kernel, staged in LDS once per tile.  Offsets are 32-bit
// and relative to the tile so that the per-item index arithmetic stays in 32-bit integer
// instructions (64-bit vector integer math is several times slower on this chip and used to
// make this kernel ALU-bound).  Tensors of 2^30 elements or more take a generic 64-bit path
// instead (S = 0 marks them).
struct GatherRec {
    int32_t rel;        // full_off - tile start (may be negative: tensor began before the tile)
    uint32_t S;         // shard elements; 0 = use the generic path
    uint32_t numel;
    int64_t shard_off;  // start inside every rank arena
};

__device__ __forceinline__ GatherRec make_gather_rec(const TensorDesc &d, int64_t a0)
{
    GatherRec g;
    const int64_t lim = int64_t{1} << 30;
    const int64_t rel = d.full_off - a0;
    // A tensor that intersects the tile began less than numel elements before it, so a
    // small tensor's offset always fits; only the ordering matters for the others.
    const bool small = d.numel < (int64_t{1} << kGatherSmallShift);
    g.rel = static_cast<int32_t>(rel < -lim ? -lim : (rel > lim ? lim : rel));
    g.S = small ? static_cast<uint32_t>(d.S) : 0u;
    g.numel = small ? static_cast<uint32_t>(d.numel) : 0u;
    g.shard_off = d.shard_off;
    return g;
}

// One-instruction reciprocal (about 1 ulp); the host pass and the CPU emulation divide.
__device__ __forceinline__ float fast_rcp(float x)
{
#ifdef __HIP_DEVICE_COMPILE__
    return __builtin_amdgcn_rcpf(x);
#else
    return 1.0f / x;
#endif
}

// floor(j / S) for j < 2^30, S >= 1 and a quotient of at most 2^12 (the owner count): the
// float estimate is off by at most one, which the two comparisons repair.
__device__ __forceinline__ uint32_t div_owner(uint32_t j, uint32_t S)
{
    uint32_t r = static_cast<uint32_t>(static_cast<float>(j) * fast_rcp(static_cast<float>(S)));
    const int32_t i = static_cast<int32_t>(j - r * S);  // |i| < 2S < 2^31
    if (i < 0) --r;
    else if (static_cast<uint32_t>(i) >= S) ++r;
    return r;
}

// The same for 64-bit operands (0 <= j < 2^62, quotient below 2^12): the conversions, the
// reciprocal and the product are each good to about 2^-23, so the estimate is within
// 2^12 * 2^-21 < 1 of the quotient and one step of repair is enough.  Replaces a 64-bit
// integer division, which the compiler expands into a long instruction sequence.
__device__ __forceinline__ int64_t div_owner64(int64_t j, int64_t S)
{
    int64_t r = static_cast<int64_t>(static_cast<float>(j) * fast_rcp(static_cast<float>(S)));
    const int64_t i = j - r * S;
    if (i < 0) --r;
    else if (i >= S) ++r;
    return r;
}

// One item copied element by element, each element from whichever owner holds it; owners
// outside this launch are left to the launch that serves them.  Sequential on purpose (few
// registers): used only where a wide load could run past the end of an arena.
__device__ __forceinline__ void gather_elements(uint32_t j, uint32_t S, int64_t shard_off, int cnt,
                                                void *const *base, int r0, int nr, uint16_t *dst)
{
    uint32_t r = div_owner(j, S);
    uint32_t i = j - r * S;
#pragma unroll 1
    for (int e = 0; e < cnt; ++e) {
        const uint32_t rl = r - static_cast<uint32_t>(r0);
        if (rl < static_cast<uint32_t>(nr))
            st_u16(dst + e, ld_u16(static_cast<const uint16_t *>(base[rl]) + shard_off + i));
        if (++i == S) {
            i = 0;
            ++r;
        }
    }
}

// Generic 64-bit form of one item, for tensors too large for the 32-bit records (their
// shards are far longer than an item, so an item touches at most two owners).
template <bool NT>
__device__ __forceinline__ void gather_item_generic(const TensorDesc &d, int64_t a, void *const *base, int r0,
                                                    int nr, uint16_t *dst)
{
    const int64_t j = a - d.full_off;
    if (j < 0 || j >= d.numel) return;
    const int cnt = d.numel - j >= 8 ? 8 : static_cast<int>(d.numel - j);
    int64_t r = div_owner64(j, d.S);
    int64_t i = j - r * d.S;
    if (cnt == 8 && i + 8 <= d.S) {
        if (r >= r0 && r < r0 + nr)
            st<NT>(reinterpret_cast<u32x4 *>(dst),
                   ld_u128_unaligned<NT>(static_cast<const uint16_t *>(base[r - r0]) + d.shard_off + i));
        return;
    }
#pragma unroll 1
    for (int k = 0; k < cnt; ++k) {  // at most one such item per shard boundary
        if (r >= r0 && r < r0 + nr)
            st_u16(dst + k, ld_u16(static_cast<const uint16_t *>(base[r - r0]) + d.shard_off + i));
        if (++i == d.S) {
            i = 0;
            ++r;
        }
    }
}

// First `k` 16-bit elements of a (1 <= k <= 7) followed by the first 8 - k elements of b.
__device__ __forceinline__ u32x4 splice(u32x4 a, u32x4 b, int k)
{
    const uint64_t alo = a.x | (static_cast<uint64_t>(a.y) << 32), ahi = a.z | (static_cast<uint64_t>(a.w) << 32);
    const uint64_t blo = b.x | (static_cast<uint64_t>(b.y) << 32), bhi = b.z | (static_cast<uint64_t>(b.w) << 32);
    const int s = 16 * k;  // bits kept from a
    uint64_t lo, hi;
    if (s < 64) {
        lo = (alo & ((uint64_t{1} << s) - 1)) | (blo << s);
        hi = (bhi << s) | (blo >> (64 - s));
    } else if (s == 64) {
        lo = alo;
        hi = blo;
    } else {
        lo = alo;
        hi = (ahi & ((uint64_t{1} << (s - 64)) - 1)) | (blo << (s - 64));
    }
    u32x4 v;
    v.x = static_cast<uint32_t>(lo);
    v.y = static_cast<uint32_t>(lo >> 32);
    v.z = static_cast<uint32_t>(hi);
    v.w = static_cast<uint32_t>(hi >> 32);
    return v;
}

constexpr int kGatherMaxTensors = kGatherChunks * kMaxTensorsPerChunk + 2;
constexpr int kGatherFewTensors = 32;  // LDS capacity of the variant for ordinary layouts

template <int CAP>
struct GatherTile {
    int32_t rel[CAP];
    uint32_t S[CAP];
    uint32_t numel[CAP];
    int64_t shard_off[CAP];
    void *base[kRanksPerLaunch];
};

// What pass 1 of the gather kernel leaves for pass 2, packed into one register per item:
// kind in bits 0..3, then three 4-bit element counts.
enum : int { kGatherNone = 0, kGatherWide = 1, kGatherGeneric = 2, kGatherElements = 3 };

// Index of the staged tensor that holds tile-relative element a_rel.
template <int CAP>
__device__ __forceinline__ int gather_find(const GatherTile<CAP> &lds, int n, int a_rel)
{
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (lds.rel[mid] <= a_rel) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

// grid.x = tiles of the full buffer; owners [r0, r0 + nr) are served by this launch.
//
// A tile is kGatherChunks chunks, i.e. kGatherChunks items of 8 elements per thread, taken
// UG at a time: pass 1 locates the items and issues their wide loads, pass 2 stores.  An
// item of a tensor with S >= 8 lies in one owner's shard or straddles into the next owner's:
// one or two wide loads (the first may run past the end of the shard piece into the owner's
// next slots, which are inside the arena unless the item is the arena's last) and, for a
// straddling item, a splice.  When one of the two owners belongs to another launch only the
// elements of the owner served here are stored.  The kernel is deliberately lean: it runs
// at the rate the number of resident wavefronts allows, so everything rare is kept out of
// the main path -- tensors with S < 8 (an item spans three or more owners) are skipped there
// and copied element-wise, one lane per element, by the loop at the end of the tile.
template <bool NT, int CAP, bool BIG>
__global__ __launch_bounds__(kBatchThreads) void k_gather_batched(BatchTable tb, RankPtrs arenas,
                                                                  uint16_t *__restrict__ full, int r0, int nr,
                                                                  int block_shift)
{
    constexpr int UG = 2;  // items in flight per thread
    static_assert(kGatherChunks % UG == 0, "tile must hold a whole number of item groups");
    __shared__ GatherTile<CAP> lds;
    if (threadIdx.x < kRanksPerLaunch) lds.base[threadIdx.x] = arenas.p[threadIdx.x];
    const int wave = static_cast<int>(threadIdx.x) >> 6, lane = static_cast<int>(threadIdx.x) & 63;
    const int64_t nchunks = (tb.full_elems + kChunkElems - 1) >> kChunkShift;
    const int64_t ntiles = (nchunks + kGatherChunks - 1) / kGatherChunks;
    const int64_t nslots = ((ntiles + (int64_t{8} << block_shift) - 1) >> (block_shift + 3)) << (block_shift + 3);
    for (int64_t slot = blockIdx.x; slot < nslots; slot += gridDim.x) {
        if (slot != static_cast<int64_t>(blockIdx.x)) __syncthreads();  // LDS reuse across iterations
        const int64_t tile = span_of(slot, block_shift);  // tiles handed to the XCDs in blocks
        if (tile >= ntiles) continue;
        const int64_t c0 = tile * kGatherChunks;
        const int64_t c1 = c0 + kGatherChunks < nchunks ? c0 + kGatherChunks : nchunks;
        const int64_t a0 = c0 << kChunkShift;
        const int t_lo = tb.full_chunk_first[c0];
        const int n = tb.full_chunk_first[c1] - t_lo + 1;  // <= CAP: the launcher picked CAP
        if (BIG && n == 1) {
            // A tile that lies inside one owner's piece of one tensor (most tiles of a large
            // tensor, whatever its size): a plain copy with uniform source and destination,
            // no staging, no per-item arithmetic.  (BIG: the layout has a tensor whose shard
            // pieces are at least a tile long; layouts of small tensors only run the variant
            // without this path, which is a few per cent faster for them.)
            const TensorDesc d = tb.desc[t_lo];
            constexpr int64_t kTile = static_cast<int64_t>(kGatherChunks) * kChunkElems;
            const int64_t j0 = a0 - d.full_off;
            if (j0 >= 0 && j0 + kTile <= d.numel) {
                const int64_t r = div_owner64(j0, d.S);
                const int64_t i0 = j0 - r * d.S;
                if (i0 + kTile <= d.S && r >= r0 && r < r0 + nr) {
                    const uint16_t *src = static_cast<const uint16_t *>(arenas.p[r - r0]) + d.shard_off + i0;
                    uint16_t *dst = full + a0;
                    // all of the thread's items in flight at once: measured best for this path
                    u32x4 v[kGatherChunks];
#pragma unroll
                    for (int u = 0; u < kGatherChunks; ++u)
                        v[u] = ld_u128_unaligned<NT>(src + 8 * (u * kBatchThreads + static_cast<int>(threadIdx.x)));
#pragma unroll
                    for (int u = 0; u < kGatherChunks; ++u)
                        st<NT>(reinterpret_cast<u32x4 *>(dst) + u * kBatchThreads + threadIdx.x, v[u]);
                    continue;
                }
            }
        }
        for (int k = threadIdx.x; k < n; k += kBatchThreads) {
            const GatherRec g = make_gather_rec(tb.desc[t_lo + k], a0);
            lds.rel[k] = g.rel;
            lds.S[k] = g.S;
            lds.numel[k] = g.numel;
            lds.shard_off[k] = g.shard_off;
        }
        __syncthreads();
        const int64_t tile_elems = tb.full_elems - a0;  // elements from the tile start to the buffer end

#pragma unroll 1
        for (int grp = 0; grp < kGatherChunks / UG; ++grp) {
            u32x4 va[UG], vb[UG];
            int code[UG];
#pragma unroll
            for (int u = 0; u < UG; ++u) {
                code[u] = kGatherNone;
                va[u] = u32x4{0u, 0u, 0u, 0u};
                vb[u] = va[u];
                const int a_rel = 8 * ((grp * UG + u) * kBatchThreads + static_cast<int>(threadIdx.x));
                if (a_rel >= tile_elems) continue;
                const int k = gather_find(lds, n, a_rel);
                const uint32_t S = lds.S[k];
                if (S == 0) {
                    code[u] = kGatherGeneric;
                    continue;
                }
                const uint32_t j = static_cast<uint32_t>(a_rel - lds.rel[k]);
                const uint32_t numel = lds.numel[k];
                if (S < 8 || j >= numel) continue;  // element-wise loop after the items / alignment gap
                const uint32_t cnt = numel - j >= 8 ? 8u : numel - j;
                const uint32_t r = div_owner(j, S);
                const uint32_t i = j - r * S;
                const uint32_t rl = r - static_cast<uint32_t>(r0);  // wraps if r < r0
                const uint32_t split = i + cnt > S ? S - i : 0u;    // elements from the first owner if two
                const bool in_a = rl < static_cast<uint32_t>(nr);
                const bool in_b = split != 0 && rl + 1 < static_cast<uint32_t>(nr);
                if (!in_a && !in_b) continue;
                const int64_t shard_off = lds.shard_off[k];
                if (in_a && shard_off + i + 8 > tb.arena_elems) {
                    code[u] = kGatherElements;
                    continue;
                }
                const uint32_t e_lo = in_a ? 0u : split;
                const uint32_t e_hi = (split != 0 && !in_b) ? split : cnt;
                constexpr bool NTL = NT && kPieceLoadsNT;
                if (in_a) va[u] = ld_u128_unaligned<NTL>(static_cast<const uint16_t *>(lds.base[rl]) + shard_off + i);
                if (in_b)
                    vb[u] = ld<NTL>(reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(lds.base[rl + 1]) +
                                                                   shard_off));
                code[u] = kGatherWide | static_cast<int>(split << 4 | e_lo << 8 | e_hi << 12);
            }
#pragma unroll
            for (int u = 0; u < UG; ++u) {
                const int kind = code[u] & 15;
                if (kind == kGatherNone) continue;
                const int a_rel = 8 * ((grp * UG + u) * kBatchThreads + static_cast<int>(threadIdx.x));
                uint16_t *dst = full + a0 + a_rel;
                if (kind == kGatherWide) {
                    const int split = (code[u] >> 4) & 15, e_lo = (code[u] >> 8) & 15, e_hi = (code[u] >> 12) & 15;
                    const u32x4 v = split ? splice(va[u], vb[u], split) : va[u];
                    if (e_lo == 0 && e_hi == 8) {
                        st<NT>(reinterpret_cast<u32x4 *>(dst), v);
                    } else {  // ragged tensor end, or an owner of another launch: its slots stay untouched
                        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (e >= e_lo && e < e_hi) st_u16(dst + e, static_cast<uint16_t>(w[e >> 1] >> (16 * (e & 1))));
                    }
                } else {  // rare: located again rather than kept in registers
                    const int k = gather_find(lds, n, a_rel);
                    if (kind == kGatherGeneric) {
                        gather_item_generic<NT>(tb.desc[t_lo + k], a0 + a_rel, lds.base, r0, nr, dst);
                    } else {
                        const uint32_t j = static_cast<uint32_t>(a_rel - lds.rel[k]);
                        const uint32_t numel = lds.numel[k];
                        gather_elements(j, lds.S[k], lds.shard_off[k], numel - j >= 8 ? 8 : static_cast<int>(numel - j),
                                        lds.base, r0, nr, dst);
                    }
                }
            }
        }

        // Tensors with S < 8 that begin in this tile: one wavefront per tensor, one lane per
        // element.  Done here, next to the items of their neighbours, because their 16-byte
        // pieces share every cache line with the neighbouring tensors' pieces: in a pass of
        // their own those lines would be fetched from memory a second time.
        for (int k = wave; k < n; k += kBatchThreads / 64) {
            const uint32_t S = lds.S[k];
            const int32_t rel = lds.rel[k];
            if (S == 0 || S >= 8 || rel < 0 || rel >= kGatherChunks * kChunkElems) continue;
            const uint32_t numel = lds.numel[k];
            uint16_t *dst = full + a0 + rel;
            const int64_t shard_off = lds.shard_off[k];
            for (uint32_t j = static_cast<uint32_t>(lane); j < numel; j += 64) {
                const uint32_t r = div_owner(j, S);
                const uint32_t rl = r - static_cast<uint32_t>(r0);
                if (rl < static_cast<uint32_t>(nr))
                    st_u16(dst + j, ld_u16(static_cast<const uint16_t *>(lds.base[rl]) + shard_off + (j - r * S)));
            }
        }
    }
}

// Valid elements of the 4-float vector at piece slot `slot`, and `gap`: the vector holds no valid
// element but is the alignment gap behind a fully valid piece (slot below S rounded up to 8), so
// that reading it and writing it back unchanged completes the piece's last cache line.
__device__ __forceinline__ int vec_cover(const TensorDesc &d, int r, int64_t slot, bool &gap)
{
    int64_t valid = d.numel - static_cast<int64_t>(r) * d.S;
    if (valid > d.S) valid = d.S;
    const int64_t left = valid - slot;
    gap = left <= 0 && valid == d.S && slot < ((d.S + 7) & ~int64_t{7});
    return left >= 4 ? 4 : (left > 0 ? static_cast<int>(left) : 0);
}

// First `cnt` lanes from `fresh`, the others from `old`.
__device__ __forceinline__ f32x4 keep_tail(f32x4 fresh, f32x4 old, int cnt)
{
    if (cnt < 1) fresh.x = old.x;
    if (cnt < 2) fresh.y = old.y;
    if (cnt < 3) fresh.z = old.z;
    if (cnt < 4) fresh.w = old.w;
    return fresh;
}

// One accumulate item: 4 floats at arena offset a of one owner, in two phases so that a
// thread can issue the loads of all its items before it consumes any of them.
struct AccumItem {
    u32x2 g;
    f32x4 acc;
    int cnt;    // valid elements: 4 = whole vector, 1..3 = ragged end of a shard piece, 0 = none
    bool wide;  // the accumulator vector was loaded whole and is stored whole
};

// Every accumulator line is written whole.  A shard piece rarely ends on a cache-line boundary:
// its last vector may hold only 1..3 valid elements, and up to 7 slots of alignment gap follow
// before the next tensor's piece.  Storing just the valid elements leaves a hole in a line that
// is otherwise rewritten completely, and the memory pays for a partly written line with a
// read-modify-write of its own (a layout of 132-element pieces, no ragged vector but a 16-byte
// hole per piece, ran 10 % slower than one of 136-element pieces).  So the slots after the valid
// ones travel with the rest: a ragged vector is loaded whole and stored whole with the lanes
// beyond `cnt` carrying the bits that were read, and the gap vector that completes a fully
// valid piece's last line is read and written back unchanged.  No padding or gap value ever
// changes.  The gradient load of a ragged vector is wide too (its extra lanes are the next
// piece's elements and are thrown away).  Only where the 16 bytes would pass the end of the arena
// or of the gradient buffer does an item go element by element.
template <bool NT>
__device__ __forceinline__ void accum_item_load(AccumItem &it, const TensorDesc &d, int r, int64_t a,
                                                float *__restrict__ arena, const uint16_t *__restrict__ grad,
                                                int64_t arena_elems, int64_t full_elems)
{
    const int64_t slot = a - d.shard_off;
    bool gap;
    it.cnt = vec_cover(d, r, slot, gap);
    it.wide = false;
    const float *ap = arena + a;
    if (it.cnt == 0) {
        if (gap && a + 4 <= arena_elems) {
            it.acc = ld<NT>(reinterpret_cast<const f32x4 *>(ap));
            it.wide = true;
        }
        return;
    }
    const int64_t goff = d.full_off + static_cast<int64_t>(r) * d.S + slot;
    const uint16_t *gp = grad + goff;
    if (it.cnt == 4 || (a + 4 <= arena_elems && goff + 4 <= full_elems)) {
        it.g = ld_u64_unaligned<NT && kPieceLoadsNT>(gp);
        it.acc = ld<NT>(reinterpret_cast<const f32x4 *>(ap));
        it.wide = true;
    } else {
        const uint32_t e0 = ld_u16(gp);
        const uint32_t e1 = it.cnt > 1 ? ld_u16(gp + 1) : 0u;
        const uint32_t e2 = it.cnt > 2 ? ld_u16(gp + 2) : 0u;
        it.g.x = e0 | (e1 << 16);
        it.g.y = e2;
        it.acc.x = ld_f32(ap);
        it.acc.y = it.cnt > 1 ? ld_f32(ap + 1) : 0.0f;
        it.acc.z = it.cnt > 2 ? ld_f32(ap + 2) : 0.0f;
        it.acc.w = 0.0f;
    }
}

template <bool NT, bool WEIGHTED>
__device__ __forceinline__ void accum_item_store(const AccumItem &it, float *ap, float w)
{
    if (it.wide) {
        f32x4 out = it.acc;
        if (it.cnt > 0) out = keep_tail(add4<WEIGHTED>(it.acc, it.g, w), it.acc, it.cnt);
        st<NT>(reinterpret_cast<f32x4 *>(ap), out);
    } else if (it.cnt > 0) {
        const f32x4 sum = add4<WEIGHTED>(it.acc, it.g, w);
        st_f32(ap, sum.x);
        if (it.cnt > 1) st_f32(ap + 1, sum.y);
        if (it.cnt > 2) st_f32(ap + 2, sum.z);
    }
}

// Grid: x = tiles of the rank arena, y = groups of RG owners.  Workgroups are handed out x
// first, so consecutive workgroups sweep one owner group's arenas from start to end and the
// chip works on a few advancing address windows at a time (measurably faster than spreading
// every tile over all owners first); and no kernel has to divide a linear work index.
// (Also measured and rejected: blocks of 8 to 128 tiles with the owner groups taken in turn
// inside a block, so that the gradient lines two neighbouring owners share stay in one L2: 10 %
// slower on the many-small-tensor workload.  Long contiguous runs per owner matter more.)
template <int RG, bool NT, bool ATOMIC, bool WEIGHTED>
__global__ __launch_bounds__(kBatchThreads) ODC_WAVES_PER_EU(RG == 2 ? 8 : 1) void k_accum_batched(BatchTable tb, RankPtrs accs,
                                                                 const uint16_t *__restrict__ grad, int r0, int nr,
                                                                 float w)
{
    __shared__ TileIndex<1> lds;
    const int64_t ntiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rl0 = static_cast<int>(blockIdx.y) * RG;  // grid.y = owner groups
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (tile != static_cast<int64_t>(blockIdx.x)) __syncthreads();
        int t_lo, n;
        stage_tile<1>(tb, tile, ntiles, lds, t_lo, n);
        if constexpr (ATOMIC) {
            // unordered: one element per lane and step, so that every atomic instruction of a
            // wavefront covers contiguous bytes (see accum_tile_atomic)
            constexpr int E = kChunkElems / kBatchThreads;
            uint16_t gv[E][RG];
            const int owners = nr - rl0 < RG ? nr - rl0 : RG;
            if (n == 1 && owners > 0 && tile_is_uniform(tb.desc[t_lo], tile << kChunkShift, r0 + rl0, owners)) {
                const TensorDesc d = tb.desc[t_lo];
#pragma unroll
                for (int u = 0; u < E; ++u) {
                    const int64_t a = (tile << kChunkShift) + u * kBatchThreads + static_cast<int>(threadIdx.x);
#pragma unroll
                    for (int k = 0; k < RG; ++k)
                        if (k < owners)
                            gv[u][k] = ld_u16(grad + d.full_off + static_cast<int64_t>(r0 + rl0 + k) * d.S + (a - d.shard_off));
                }
#pragma unroll
                for (int u = 0; u < E; ++u) {
                    const int64_t a = (tile << kChunkShift) + u * kBatchThreads + static_cast<int>(threadIdx.x);
#pragma unroll
                    for (int k = 0; k < RG; ++k)
                        if (k < owners)
                            unsafeAtomicAdd(static_cast<float *>(accs.p[rl0 + k]) + a,
                                            WEIGHTED ? w * widen_one(gv[u][k]) : widen_one(gv[u][k]));
                }
                continue;
            }
            bool on[E][RG];
#pragma unroll
            for (int u = 0; u < E; ++u) {
                const int a_rel = u * kBatchThreads + static_cast<int>(threadIdx.x);
                const int64_t a = (tile << kChunkShift) + a_rel;
                const bool live = a < tb.arena_elems;
                TensorDesc d{};
                if (live) d = tile_desc(tb, t_lo, n, a_rel, lds);
#pragma unroll
                for (int k = 0; k < RG; ++k) {
                    const int rl = rl0 + k;
                    on[u][k] = live && rl < nr && valid_from(d, r0 + rl, a - d.shard_off, 1) == 1;
                    gv[u][k] = 0;
                    if (on[u][k]) gv[u][k] = ld_u16(grad + d.full_off + static_cast<int64_t>(r0 + rl) * d.S + (a - d.shard_off));
                }
            }
#pragma unroll
            for (int u = 0; u < E; ++u) {
                const int64_t a = (tile << kChunkShift) + u * kBatchThreads + static_cast<int>(threadIdx.x);
#pragma unroll
                for (int k = 0; k < RG; ++k)
                    if (on[u][k])
                        unsafeAtomicAdd(static_cast<float *>(accs.p[rl0 + k]) + a,
                                        WEIGHTED ? w * widen_one(gv[u][k]) : widen_one(gv[u][k]));
            }
        } else {
            if constexpr (RG == 1) {
                // (only the one-owner variant, which is the one picked for layouts of large
                // tensors: with more owners per workgroup the extra path costs registers)
                if (n == 1 && rl0 < nr && tile_is_uniform(tb.desc[t_lo], tile << kChunkShift, r0 + rl0, 1)) {
                    const TensorDesc d = tb.desc[t_lo];
                    float *arena = static_cast<float *>(accs.p[rl0]);
                    const uint16_t *g = grad + d.full_off + static_cast<int64_t>(r0 + rl0) * d.S - d.shard_off;
                    u32x2 gv[kAccumItems];
                    f32x4 av[kAccumItems];
#pragma unroll
                    for (int u = 0; u < kAccumItems; ++u) {
                        const int64_t a = (tile << kChunkShift) + 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
                        gv[u] = ld_u64_unaligned<NT>(g + a);
                        av[u] = ld<NT>(reinterpret_cast<const f32x4 *>(arena + a));
                    }
#pragma unroll
                    for (int u = 0; u < kAccumItems; ++u) {
                        const int64_t a = (tile << kChunkShift) + 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
                        st<NT>(reinterpret_cast<f32x4 *>(arena + a), add4<WEIGHTED>(av[u], gv[u], w));
                    }
                    continue;
                }
            }
            AccumItem items[kAccumItems][RG];
#pragma unroll
            for (int u = 0; u < kAccumItems; ++u) {
                const int a_rel = 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
                const int64_t a = (tile << kChunkShift) + a_rel;
                const bool live = a < tb.arena_elems;
                TensorDesc d{};
                if (live) d = tile_desc(tb, t_lo, n, a_rel, lds);
#pragma unroll
                for (int k = 0; k < RG; ++k) {
                    const int rl = rl0 + k;
                    items[u][k].cnt = 0;
                    items[u][k].wide = false;
                    if (live && rl < nr)
                        accum_item_load<NT>(items[u][k], d, r0 + rl, a, static_cast<float *>(accs.p[rl]), grad,
                                            tb.arena_elems, tb.full_elems);
                }
            }
#pragma unroll
            for (int u = 0; u < kAccumItems; ++u) {
                const int64_t a = (tile << kChunkShift) + 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
#pragma unroll
                for (int k = 0; k < RG; ++k)
                    if (rl0 + k < nr)
                        accum_item_store<NT, WEIGHTED>(items[u][k], static_cast<float *>(accs.p[rl0 + k]) + a, w);
            }
        }
    }
}

template <int RG, bool NT>
__global__ __launch_bounds__(kBatchThreads) void k_reset_batched(BatchTable tb, RankPtrs accs, int r0, int nr)
{
    __shared__ TileIndex<1> lds;
    const int64_t ntiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rl0 = static_cast<int>(blockIdx.y) * RG;  // grid.y = owner groups
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (tile != static_cast<int64_t>(blockIdx.x)) __syncthreads();
        int t_lo, n;
        stage_tile<1>(tb, tile, ntiles, lds, t_lo, n);
        const int owners = nr - rl0 < RG ? nr - rl0 : RG;
        if (n == 1 && tile_is_uniform(tb.desc[t_lo], tile << kChunkShift, r0 + rl0, owners)) {
#pragma unroll
            for (int u = 0; u < kAccumItems; ++u) {
                const int64_t a = (tile << kChunkShift) + 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
#pragma unroll
                for (int k = 0; k < RG; ++k)
                    if (k < owners)
                        st_stream<NT ? 2 : 0>(reinterpret_cast<f32x4 *>(static_cast<float *>(accs.p[rl0 + k]) + a), zero);
            }
            continue;
        }
#pragma unroll
        for (int u = 0; u < kAccumItems; ++u) {
            const int a_rel = 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            const int64_t a = (tile << kChunkShift) + a_rel;
            if (a >= tb.arena_elems) continue;
            const TensorDesc d = tile_desc(tb, t_lo, n, a_rel, lds);
#pragma unroll
            for (int k = 0; k < RG; ++k) {
                const int rl = rl0 + k;
                if (rl >= nr) continue;
                float *arena = static_cast<float *>(accs.p[rl]);
                const int cnt = valid_from(d, r0 + rl, a - d.shard_off, 4);
                if (cnt == 4) st<NT>(reinterpret_cast<f32x4 *>(arena + a), zero);
                else
                    for (int e = 0; e < cnt; ++e) st_f32(arena + a + e, 0.0f);
            }
        }
    }
}

// ---------------------------------------------------------------------------- fused accumulate
// K contributions applied in one pass (an owner draining K staged client buffers at once,
// paper Appendix B): acc = (((acc + g_1) + g_2) + ... + g_K), the same left-to-right binary32
// sequence, starting from the stored accumulator value, that K single calls would perform, so
// the ordered result is bit-identical -- but the accumulator is read and written once:
// (2K + 8) bytes per element instead of 10K.  Fixed launch shape: one wavefront per
// workgroup, one accumulator vector per lane, non-temporal accesses.  The unordered form sums
// the K values in registers, pairwise, and issues one atomic add per element: C contributions
// taken K at a time go through ceil(log2 K) + ceil(C / K) roundings instead of C.

constexpr int kMaxFused = 8;

struct GradPtrs {
    const uint16_t *p[kMaxFused];
};

// One accumulator vector (ordered form), loaded whole and stored whole: lanes beyond `cnt` (the
// ragged end of a shard piece, or cnt = 0: the alignment gap behind a piece) keep the bits that
// were read.  The caller has checked that the wide loads stay inside the buffers.
template <int K, bool NTG = true>
__device__ __forceinline__ void accum_multi_vec(float *__restrict__ acc, const GradPtrs &grads, int64_t goff, int64_t q,
                                                int cnt = 4)
{
    f32x4 *av = reinterpret_cast<f32x4 *>(acc) + q;
    if (cnt == 0) {
        st<true>(av, ld<true>(av));
        return;
    }
    u32x2 gv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) gv[k] = ld_u64_unaligned<NTG>(grads.p[k] + goff + 4 * q);
    const f32x4 old = ld<true>(av);
    f32x4 a = old;
#pragma unroll
    for (int k = 0; k < K; ++k) a = add4<false>(a, gv[k], 1.0f);
    st<true>(av, cnt == 4 ? a : keep_tail(a, old, cnt));
}

// Sum of values v[lo .. lo + n) as a balanced binary tree (pairwise summation): the rounding
// error of the sum grows with the depth ceil(log2 n) of the tree instead of with n.
template <int N0>
__device__ __forceinline__ float tree_sum(const float *v)
{
    if constexpr (N0 == 1) return v[0];
    else return tree_sum<N0 - N0 / 2>(v) + tree_sum<N0 / 2>(v + (N0 - N0 / 2));
}

// Sum of the K values of one element for the unordered form (added atomically afterwards).  No
// order is promised there, so the association that bounds the error best is used: pairwise.
template <int K>
__device__ __forceinline__ float multi_sum_one(const GradPtrs &grads, int64_t goff, int64_t e)
{
    uint16_t gv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) gv[k] = ld_u16(grads.p[k] + goff + e);
    float v[K];
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] = widen_one(gv[k]);
    return tree_sum<K>(v);
}

template <int K, bool ATOMIC>
__device__ __forceinline__ void accum_multi_one(float *acc, const GradPtrs &grads, int64_t goff, int64_t e)
{
    if constexpr (ATOMIC) {
        unsafeAtomicAdd(acc + e, multi_sum_one<K>(grads, goff, e));
    } else {
        float a = ld_f32(acc + e);
#pragma unroll
        for (int k = 0; k < K; ++k) a = a + widen_one(ld_u16(grads.p[k] + goff + e));
        st_f32(acc + e, a);
    }
}

template <int K, bool ATOMIC>
__global__ __launch_bounds__(64) void k_accum_multi_flat(RankPtrs accs, GradPtrs grads, int64_t S, int64_t N, int r0)
{
    const int64_t base = static_cast<int64_t>(r0 + static_cast<int>(blockIdx.y)) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    float *__restrict__ acc = static_cast<float *>(accs.p[blockIdx.y]);
    const int64_t nitem = valid >> 2;
    const int tail = static_cast<int>(valid & 3);
    const int64_t ntiles = (nitem + 63) >> 6;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if constexpr (ATOMIC) {
            // one element per lane and step: contiguous atomics (see accum_tile_atomic)
            float sum[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t e = (tile << 8) + u * 64 + threadIdx.x;
                sum[u] = 0.0f;
                if (e < 4 * nitem) sum[u] = multi_sum_one<K>(grads, base, e);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t e = (tile << 8) + u * 64 + threadIdx.x;
                if (e < 4 * nitem) unsafeAtomicAdd(acc + e, sum[u]);
            }
        } else {
            const int64_t q = (tile << 6) + threadIdx.x;
            if (q < nitem) accum_multi_vec<K>(acc, grads, base, q);
        }
    }
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < tail)
        accum_multi_one<K, ATOMIC>(acc, grads, base, 4 * nitem + threadIdx.x);
}

// Batched form: grid x = tiles of the rank arena, y = owners.
template <int K, bool ATOMIC>
__global__ __launch_bounds__(kBatchThreads) void k_accum_multi_batched(BatchTable tb, RankPtrs accs, GradPtrs grads,
                                                                       int r0)
{
    __shared__ TileIndex<1> lds;
    const int64_t ntiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rl = static_cast<int>(blockIdx.y);  // grid.y = owners of this launch
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (tile != static_cast<int64_t>(blockIdx.x)) __syncthreads();
        float *__restrict__ arena = static_cast<float *>(accs.p[rl]);
        int t_lo, n;
        stage_tile<1>(tb, tile, ntiles, lds, t_lo, n);
        if constexpr (ATOMIC) {
            constexpr int E = kChunkElems / kBatchThreads;
            float sum[E];
            bool on[E];
#pragma unroll
            for (int u = 0; u < E; ++u) {
                const int a_rel = u * kBatchThreads + static_cast<int>(threadIdx.x);
                const int64_t a = (tile << kChunkShift) + a_rel;
                on[u] = false;
                sum[u] = 0.0f;
                if (a >= tb.arena_elems) continue;
                const TensorDesc d = tile_desc(tb, t_lo, n, a_rel, lds);
                const int64_t slot = a - d.shard_off;
                on[u] = valid_from(d, r0 + rl, slot, 1) == 1;
                if (on[u]) sum[u] = multi_sum_one<K>(grads, d.full_off + static_cast<int64_t>(r0 + rl) * d.S + slot - a, a);
            }
#pragma unroll
            for (int u = 0; u < E; ++u)
                if (on[u]) unsafeAtomicAdd(arena + (tile << kChunkShift) + u * kBatchThreads + static_cast<int>(threadIdx.x), sum[u]);
            continue;
        }
#pragma unroll
        for (int u = 0; u < kAccumItems; ++u) {
            const int a_rel = 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            const int64_t a = (tile << kChunkShift) + a_rel;
            if (a >= tb.arena_elems) continue;
            const TensorDesc d = tile_desc(tb, t_lo, n, a_rel, lds);
            const int64_t slot = a - d.shard_off;
            bool gap;
            const int cnt = vec_cover(d, r0 + rl, slot, gap);
            // gradient element that pairs with arena element a: goff + a
            const int64_t goff = d.full_off + static_cast<int64_t>(r0 + rl) * d.S + slot - a;
            // ragged and gap vectors are handled whole wherever the wide accesses stay inside the
            // buffers, so that every accumulator line is written completely (see accum_item_load)
            if (cnt == 4 || (cnt > 0 && a + 4 <= tb.arena_elems && goff + a + 4 <= tb.full_elems) ||
                (cnt == 0 && gap && a + 4 <= tb.arena_elems))
                accum_multi_vec<K, kPieceLoadsNT>(arena, grads, goff, a >> 2, cnt);
            else
                for (int e = 0; e < cnt; ++e) accum_multi_one<K, ATOMIC>(arena, grads, goff, a + e);
        }
    }
}

// --------------------------------------------------------------------------------- staging
// Server-side staging (paper Appendix B): every owner keeps one receive buffer per client
// (M/N elements each, M per owner in total).  A worker's push copies slice r of its gradient
// into its own slot of owner r's staging buffer and then raises flag (r, w); the owner's
// drain takes a snapshot of its flags and, in one pass over its accumulator, adds every
// staged slice in ascending client order -- the same left-to-right binary32 sequence as
// single contributions in that order -- then lowers the flags it consumed.  The polling
// daemon of the paper becomes a drain call that handles whatever has arrived and returns;
// no kernel ever waits.
//
// Layout: owner r's staging buffer holds R slots of `slot` elements (the rank arena length
// rounded up to 8, so every slot starts 16-byte aligned); client w's slot starts at w * slot
// and mirrors the rank arena element for element.  flags[r * R + w] is the state of that slot;
// flags[R * R] counts refused pushes (a slot that is not empty is never overwritten).
//
// Slot protocol.  A push and a drain may run at the same time on different streams, so the
// fate of a push is decided ONCE per (owner, client), by one thread, before any byte is copied:
//   claim   (one thread per owner)  compare-and-swap empty -> writing; a slot that is not empty
//           refuses the push for that owner (counted)
//   copy    every workgroup copies for an owner only if its slot is in state writing; nothing
//           but this push's own raise ever leaves that state, so all workgroups agree
//   raise   writing -> full
//   drain   its snapshot lists the slots that are full (never one that is being written), the
//           accumulate kernel adds exactly those, and the clear lowers exactly those to empty.
// A push that meets a full slot is therefore refused as a whole for that owner, however a
// concurrent drain interleaves with its kernels, and a slot is never added twice or half-old.
// All flag accesses are device-scope atomics (acquire loads, release stores): the slot data
// written before a raise are visible to the drain that sees the flag, and the drain's reads
// are complete before a claim can see the slot empty again.  What the protocol assumes of the
// caller: the pushes of one client are serialised (Appendix B), and so are the drains.
constexpr int32_t kSlotEmpty = 0, kSlotFull = 1, kSlotWriting = 2;

__device__ __forceinline__ int32_t flag_load(const int32_t *f)
{
    return __scoped_atomic_load_n(f, __ATOMIC_ACQUIRE, __MEMORY_SCOPE_DEVICE);
}

// Relaxed form for the copy workgroups of a push: they only ask "is this slot mine" (state
// writing, set by this push's own claim kernel, which ended before the copy kernel began, and
// changed by nobody else), and read no data that another stream publishes through the flag.  An
// acquire here would invalidate the caches once per workgroup (measured: push 12 x slower).
__device__ __forceinline__ int32_t flag_peek(const int32_t *f)
{
    return __scoped_atomic_load_n(f, __ATOMIC_RELAXED, __MEMORY_SCOPE_DEVICE);
}

__device__ __forceinline__ void flag_store(int32_t *f, int32_t v)
{
    __scoped_atomic_store_n(f, v, __ATOMIC_RELEASE, __MEMORY_SCOPE_DEVICE);
}

// true if *f was `from` and is now `to`
__device__ __forceinline__ bool flag_swap(int32_t *f, int32_t from, int32_t to)
{
    return __scoped_atomic_compare_exchange_n(f, &from, to, false, __ATOMIC_ACQ_REL, __ATOMIC_ACQUIRE,
                                              __MEMORY_SCOPE_DEVICE);
}

// Copy `valid` bf16 elements from an unaligned source to a 16-byte-aligned destination.
template <int TPB, bool NT>
__device__ __forceinline__ void copy_to_aligned(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                int64_t valid)
{
    const int64_t nvec = valid >> 3;
    const int tail = static_cast<int>(valid & 7);
    const int64_t ntiles = (nvec + TPB - 1) / TPB;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v = tile * TPB + threadIdx.x;
        if (v < nvec) st_stream<NT ? 2 : 0>(reinterpret_cast<u32x4 *>(dst) + v, ld_u128_unaligned<NT>(src + 8 * v));
    }
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < tail) {
        const int64_t k = 8 * nvec + threadIdx.x;
        st_u16(dst + k, ld_u16(src + k));
    }
}

template <bool NT>
__global__ __launch_bounds__(64) void k_stage_push_flat(RankPtrs staging, const uint16_t *__restrict__ grad,
                                                        const int32_t *__restrict__ flags, int64_t S, int64_t N,
                                                        int64_t slot, int R, int r0, int worker)
{
    const int r = r0 + static_cast<int>(blockIdx.y);
    const int64_t base = static_cast<int64_t>(r) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    if (flag_peek(flags + static_cast<int64_t>(r) * R + worker) != kSlotWriting) return;  // not claimed: refused
    uint16_t *dst = static_cast<uint16_t *>(staging.p[blockIdx.y]) + static_cast<int64_t>(worker) * slot;
    copy_to_aligned<64, NT>(grad + base, dst, valid);
}

// Tiles of kPushChunks chunks: kPushChunks 16-byte items per thread, all loaded before any is
// stored.
constexpr int kPushChunks = 2;

template <bool NT>
__global__ __launch_bounds__(kBatchThreads) void k_stage_push_batched(BatchTable tb, RankPtrs staging,
                                                                      const uint16_t *__restrict__ grad,
                                                                      const int32_t *__restrict__ flags,
                                                                      int64_t slot, int R, int r0, int worker)
{
    __shared__ TileIndex<kPushChunks> lds;
    constexpr int kTile = kPushChunks * kChunkElems;
    const int64_t nchunks = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int64_t ntiles = (nchunks + kPushChunks - 1) / kPushChunks;
    const int rl = static_cast<int>(blockIdx.y);  // grid.y = owners of this launch
    const int r = r0 + rl;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (tile != static_cast<int64_t>(blockIdx.x)) __syncthreads();
        const bool claimed = flag_peek(flags + static_cast<int64_t>(r) * R + worker) == kSlotWriting;  // uniform
        int t_lo, n;
        stage_tile<kPushChunks>(tb, tile, nchunks, lds, t_lo, n);
        if (!claimed) continue;  // this owner refused the push
        uint16_t *dst = static_cast<uint16_t *>(staging.p[rl]) + static_cast<int64_t>(worker) * slot;
        const int64_t a0 = tile * kTile;
        u32x4 v[kPushChunks];
        if (n == 1 && tile_is_uniform(tb.desc[t_lo], a0, r, 1, kTile)) {
            const TensorDesc d = tb.desc[t_lo];
            const uint16_t *src = grad + d.full_off + static_cast<int64_t>(r) * d.S - d.shard_off + a0;
#pragma unroll
            for (int u = 0; u < kPushChunks; ++u)
                v[u] = ld_u128_unaligned<NT>(src + 8 * (u * kBatchThreads + static_cast<int>(threadIdx.x)));
#pragma unroll
            for (int u = 0; u < kPushChunks; ++u)
                st<NT>(reinterpret_cast<u32x4 *>(dst + a0) + u * kBatchThreads + threadIdx.x, v[u]);
            continue;
        }
        int cnt[kPushChunks];
#pragma unroll
        for (int u = 0; u < kPushChunks; ++u) {
            const int a_rel = 8 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            const int64_t a = a0 + a_rel;
            cnt[u] = 0;
            v[u] = u32x4{0u, 0u, 0u, 0u};
            if (a >= tb.arena_elems) continue;
            const TensorDesc d = tile_desc(tb, t_lo, n, a_rel, lds);
            const int64_t slot_in = a - d.shard_off;
            const int c = valid_from(d, r, slot_in, 8);
            if (c == 0) continue;
            const int64_t goff = d.full_off + static_cast<int64_t>(r) * d.S + slot_in;
            if (c == 8 || goff + 8 <= tb.full_elems) {
                // a ragged end (c < 8) keeps the wide load: the extra lanes belong to the next
                // piece and are dropped
                cnt[u] = c;
                v[u] = ld_u128_unaligned<NT && kPieceLoadsNT>(grad + goff);
            } else {  // the last elements of the gradient buffer
                for (int e = 0; e < c; ++e) st_u16(dst + a + e, ld_u16(grad + goff + e));
            }
        }
#pragma unroll
        for (int u = 0; u < kPushChunks; ++u) {
            const int64_t a = a0 + 8 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            // A ragged item is stored whole as well: its spare lanes fall into the alignment gap
            // behind the piece, which in a staging slot belongs to nobody (the drain never takes
            // them), and a slot written in whole 16-byte vectors has no partly written sector.
            if (cnt[u] > 0) st<NT>(reinterpret_cast<u32x4 *>(dst + a), v[u]);
        }
    }
}

// Claim: one thread per owner decides whether the owner takes this push (see the slot protocol).
__global__ __launch_bounds__(64) void k_stage_claim(int32_t *flags, int R, int worker)
{
    for (int r = blockIdx.x * 64 + threadIdx.x; r < R; r += gridDim.x * 64) {
        if (!flag_swap(flags + static_cast<int64_t>(r) * R + worker, kSlotEmpty, kSlotWriting))
            atomicAdd(flags + static_cast<int64_t>(R) * R, 1);
    }
}

// Raise: the slots this push claimed (and has filled by now) become full.
__global__ __launch_bounds__(64) void k_stage_raise(int32_t *flags, int R, int worker)
{
    for (int r = blockIdx.x * 64 + threadIdx.x; r < R; r += gridDim.x * 64)
        (void)flag_swap(flags + static_cast<int64_t>(r) * R + worker, kSlotWriting, kSlotFull);
}

// One thread per owner.  Snapshot: the owner's full slots, ascending, are written as a list
// snapshot[r * (R + 1)] = count, then the client indices.  Clear: every listed flag is lowered.
// Taking the list once per drain keeps all workgroups of the accumulate kernel on the same set
// of contributions even if pushes from other streams raise more flags meanwhile.
__global__ __launch_bounds__(64) void k_stage_snapshot(const int32_t *flags, int32_t *snapshot, int R)
{
    for (int r = blockIdx.x * 64 + threadIdx.x; r < R; r += gridDim.x * 64) {
        ODC_GLOBAL int32_t *list = (ODC_GLOBAL int32_t *)(snapshot + static_cast<int64_t>(r) * (R + 1));
        const int32_t *row = flags + static_cast<int64_t>(r) * R;
        int n = 0;
        for (int w = 0; w < R; ++w)
            if (flag_load(row + w) == kSlotFull) list[1 + n++] = w;
        list[0] = n;
    }
}

__global__ __launch_bounds__(64) void k_stage_clear(int32_t *flags, const int32_t *snapshot, int R)
{
    for (int r = blockIdx.x * 64 + threadIdx.x; r < R; r += gridDim.x * 64) {
        const ODC_GLOBAL int32_t *list = (const ODC_GLOBAL int32_t *)(snapshot + static_cast<int64_t>(r) * (R + 1));
        int32_t *row = flags + static_cast<int64_t>(r) * R;
        const int n = list[0];
        for (int k = 0; k < n; ++k) flag_store(row + list[1 + k], kSlotEmpty);
    }
}

__global__ __launch_bounds__(256) void k_stage_zero(int32_t *flags, int64_t count)
{
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < count; i += static_cast<int64_t>(gridDim.x) * 256)
        *(ODC_GLOBAL int32_t *)(flags + i) = 0;
}

// Add the staged vectors of the listed clients, in list order, to one accumulator vector;
// up to four staged vectors are fetched before they are added.  `list` is the owner's
// snapshot (count, then client indices): the same for every lane, so its reads are scalar.
template <bool NT>
__device__ __forceinline__ f32x4 drain_vec(f32x4 acc, const uint16_t *__restrict__ stage, int64_t slot, int64_t a,
                                           const int32_t *__restrict__ list)
{
    constexpr int B = 4;
    const int n = list[0];
    for (int c = 0; c < n; c += B) {
        u32x2 gv[B];
#pragma unroll
        for (int j = 0; j < B; ++j)
            if (c + j < n)
                gv[j] = ld<NT>(reinterpret_cast<const u32x2 *>(stage + static_cast<int64_t>(list[1 + c + j]) * slot + a));
#pragma unroll
        for (int j = 0; j < B; ++j)
            if (c + j < n) acc = add4<false>(acc, gv[j], 1.0f);
    }
    return acc;
}

__device__ __forceinline__ float drain_one(float v, const uint16_t *__restrict__ stage, int64_t slot, int64_t k,
                                           const int32_t *__restrict__ list)
{
    const int n = list[0];
    for (int c = 0; c < n; ++c) v = v + widen_one(ld_u16(stage + static_cast<int64_t>(list[1 + c]) * slot + k));
    return v;
}

template <bool NT>
__global__ __launch_bounds__(64) void k_stage_drain_flat(RankPtrs accs, RankPtrs staging,
                                                         const int32_t *__restrict__ snapshot, int64_t S, int64_t N,
                                                         int64_t slot, int R, int r0)
{
    const int r = r0 + static_cast<int>(blockIdx.y);
    const int64_t base = static_cast<int64_t>(r) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    const int32_t *list = snapshot + static_cast<int64_t>(r) * (R + 1);
    if (list[0] == 0) return;  // nothing staged for this owner: its accumulator is not touched
    float *__restrict__ acc = static_cast<float *>(accs.p[blockIdx.y]);
    const uint16_t *__restrict__ stage = static_cast<const uint16_t *>(staging.p[blockIdx.y]);
    const int64_t nitem = valid >> 2;
    const int tail = static_cast<int>(valid & 3);
    const int64_t ntiles = (nitem + 63) >> 6;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t q = (tile << 6) + threadIdx.x;
        if (q < nitem) {
            f32x4 *av = reinterpret_cast<f32x4 *>(acc) + q;
            st<NT>(av, drain_vec<NT>(ld<NT>(av), stage, slot, 4 * q, list));
        }
    }
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < tail) {
        const int64_t k = 4 * nitem + threadIdx.x;
        st_f32(acc + k, drain_one(ld_f32(acc + k), stage, slot, k, list));
    }
}

template <bool NT>
__global__ __launch_bounds__(kBatchThreads) void k_stage_drain_batched(BatchTable tb, RankPtrs accs, RankPtrs staging,
                                                                       const int32_t *__restrict__ snapshot,
                                                                       int64_t slot, int R, int r0)
{
    __shared__ TileIndex<1> lds;
    const int64_t ntiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rl = static_cast<int>(blockIdx.y);  // grid.y = owners of this launch
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (tile != static_cast<int64_t>(blockIdx.x)) __syncthreads();
        const int r = r0 + rl;
        int t_lo, n;
        stage_tile<1>(tb, tile, ntiles, lds, t_lo, n);
        const int32_t *list = snapshot + static_cast<int64_t>(r) * (R + 1);
        if (list[0] == 0) continue;
        float *__restrict__ arena = static_cast<float *>(accs.p[rl]);
        const uint16_t *__restrict__ stage = static_cast<const uint16_t *>(staging.p[rl]);
#pragma unroll
        for (int u = 0; u < kAccumItems; ++u) {
            const int a_rel = 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            const int64_t a = (tile << kChunkShift) + a_rel;
            if (a >= tb.arena_elems) continue;
            const TensorDesc d = tile_desc(tb, t_lo, n, a_rel, lds);
            bool gap;
            const int cnt = vec_cover(d, r, a - d.shard_off, gap);
            if (cnt == 4) {
                f32x4 *av = reinterpret_cast<f32x4 *>(arena + a);
                st<NT>(av, drain_vec<NT>(ld<NT>(av), stage, slot, a, list));
            } else if (cnt > 0 && a + 4 <= tb.arena_elems) {
                // ragged end of a shard piece: wide loads (every staging slot is at least as long
                // as the arena rounded up to 8) and a whole store whose lanes beyond cnt carry
                // the bits that were read
                f32x4 *av = reinterpret_cast<f32x4 *>(arena + a);
                const f32x4 old = ld<NT>(av);
                st<NT>(av, keep_tail(drain_vec<NT>(old, stage, slot, a, list), old, cnt));
            } else if (cnt == 0 && gap && a + 4 <= tb.arena_elems) {
                f32x4 *av = reinterpret_cast<f32x4 *>(arena + a);  // completes the piece's last line
                st<NT>(av, ld<NT>(av));
            } else {
                for (int e = 0; e < cnt; ++e) st_f32(arena + a + e, drain_one(ld_f32(arena + a + e), stage, slot, a + e, list));
            }
        }
    }
}

// -------------------------------------------------------------------------------- retrieve
// Minibatch-end retrieval (paper Section 3.2): each owner's accumulated gradient shard is
// read, multiplied by `scale` (one binary32 multiply) and written to the owner's output shard
// as binary32 or, rounded once more to nearest-even, as bf16.  4 + 4 or 4 + 2 bytes per
// element; the accumulators are left as they are.

// binary32 -> bf16, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t narrow_bf16(float f)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <bool NT, bool BF16, bool STREAM>
__device__ __forceinline__ void retrieve_vec(const float *__restrict__ src, void *__restrict__ out, int64_t q, float scale)
{
    f32x4 v = ld<NT>(reinterpret_cast<const f32x4 *>(src) + q);
    v.x = scale * v.x;
    v.y = scale * v.y;
    v.z = scale * v.z;
    v.w = scale * v.w;
    if constexpr (BF16) {
        const u32x2 p = {narrow_bf16(v.x) | (narrow_bf16(v.y) << 16), narrow_bf16(v.z) | (narrow_bf16(v.w) << 16)};
        st_stream<(NT ? (STREAM ? 2 : 1) : 0)>(reinterpret_cast<u32x2 *>(out) + q, p);
    } else {
        st_stream<(NT ? (STREAM ? 2 : 1) : 0)>(reinterpret_cast<f32x4 *>(out) + q, v);
    }
}

template <bool BF16>
__device__ __forceinline__ void retrieve_one(const float *src, void *out, int64_t k, float scale)
{
    const float v = scale * ld_f32(src + k);
    if constexpr (BF16) st_u16(static_cast<uint16_t *>(out) + k, static_cast<uint16_t>(narrow_bf16(v)));
    else st_f32(static_cast<float *>(out) + k, v);
}

template <int TPB, int U, bool NT, bool BF16>
__global__ __launch_bounds__(TPB) void k_retrieve_flat(RankPtrs accs, RankPtrs outs, int64_t S, int64_t N, int r0,
                                                       float scale)
{
    const int64_t base = static_cast<int64_t>(r0 + static_cast<int>(blockIdx.y)) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    const float *__restrict__ acc = static_cast<const float *>(accs.p[blockIdx.y]);
    void *__restrict__ out = outs.p[blockIdx.y];
    const int64_t nvec = valid >> 2;
    const int tail = static_cast<int>(valid & 3);
    const int64_t ntiles = (nvec + TPB * U - 1) / (TPB * U);
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * (TPB * U) + threadIdx.x;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t v = v0 + u * TPB;
            if (v < nvec) retrieve_vec<NT, BF16, true>(acc, out, v, scale);
        }
    }
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < tail) retrieve_one<BF16>(acc, out, 4 * nvec + threadIdx.x, scale);
}

// Two phases like the accumulate kernel: all loads of a thread's items first, then the stores
// (the compiler cannot move a load above an earlier store by itself: for all it knows the
// output shard may alias an accumulator).  A ragged item uses the wide load too where that
// stays inside the arena; only its stores are element-wise.
template <int RG, bool NT, bool BF16>
__global__ __launch_bounds__(kBatchThreads) void k_retrieve_batched(BatchTable tb, RankPtrs accs, RankPtrs outs,
                                                                    int r0, int nr, float scale)
{
    __shared__ TileIndex<1> lds;
    const int64_t ntiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rl0 = static_cast<int>(blockIdx.y) * RG;  // grid.y = owner groups
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (tile != static_cast<int64_t>(blockIdx.x)) __syncthreads();
        int t_lo, n;
        stage_tile<1>(tb, tile, ntiles, lds, t_lo, n);
        f32x4 v[kAccumItems][RG];
        const int owners = nr - rl0 < RG ? nr - rl0 : RG;
        if (n == 1 && tile_is_uniform(tb.desc[t_lo], tile << kChunkShift, r0 + rl0, owners)) {
#pragma unroll
            for (int u = 0; u < kAccumItems; ++u) {
                const int64_t a = (tile << kChunkShift) + 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
#pragma unroll
                for (int k = 0; k < RG; ++k)
                    if (k < owners) v[u][k] = ld<NT>(reinterpret_cast<const f32x4 *>(static_cast<const float *>(accs.p[rl0 + k]) + a));
            }
#pragma unroll
            for (int u = 0; u < kAccumItems; ++u) {
                const int64_t a = (tile << kChunkShift) + 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
#pragma unroll
                for (int k = 0; k < RG; ++k) {
                    if (k >= owners) continue;
                    const f32x4 sv = {scale * v[u][k].x, scale * v[u][k].y, scale * v[u][k].z, scale * v[u][k].w};
                    if constexpr (BF16) {
                        const u32x2 p = {narrow_bf16(sv.x) | (narrow_bf16(sv.y) << 16),
                                         narrow_bf16(sv.z) | (narrow_bf16(sv.w) << 16)};
                        st_stream<NT ? 2 : 0>(reinterpret_cast<u32x2 *>(static_cast<uint16_t *>(outs.p[rl0 + k]) + a), p);
                    } else {
                        st_stream<NT ? 2 : 0>(reinterpret_cast<f32x4 *>(static_cast<float *>(outs.p[rl0 + k]) + a), sv);
                    }
                }
            }
            continue;
        }
        int cnt[kAccumItems][RG];
#pragma unroll
        for (int u = 0; u < kAccumItems; ++u) {
            const int a_rel = 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            const int64_t a = (tile << kChunkShift) + a_rel;
            const bool live = a < tb.arena_elems;
            TensorDesc d{};
            if (live) d = tile_desc(tb, t_lo, n, a_rel, lds);
#pragma unroll
            for (int k = 0; k < RG; ++k) {
                const int rl = rl0 + k;
                cnt[u][k] = 0;
                v[u][k] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                if (!live || rl >= nr) continue;
                const float *src = static_cast<const float *>(accs.p[rl]) + a;
                const int c = valid_from(d, r0 + rl, a - d.shard_off, 4);
                cnt[u][k] = c;
                if (c == 4 || (c > 0 && a + 4 <= tb.arena_elems)) {
                    v[u][k] = ld<NT>(reinterpret_cast<const f32x4 *>(src));
                } else if (c > 0) {  // the last item of the arena
                    v[u][k].x = ld_f32(src);
                    if (c > 1) v[u][k].y = ld_f32(src + 1);
                    if (c > 2) v[u][k].z = ld_f32(src + 2);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kAccumItems; ++u) {
            const int64_t a = (tile << kChunkShift) + 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
#pragma unroll
            for (int k = 0; k < RG; ++k) {
                const int c = cnt[u][k];
                if (c == 0) continue;
                const f32x4 s = {scale * v[u][k].x, scale * v[u][k].y, scale * v[u][k].z, scale * v[u][k].w};
                void *out = outs.p[rl0 + k];
                if constexpr (BF16) {
                    uint16_t *o = static_cast<uint16_t *>(out) + a;
                    if (c == 4) {
                        const u32x2 p = {narrow_bf16(s.x) | (narrow_bf16(s.y) << 16),
                                         narrow_bf16(s.z) | (narrow_bf16(s.w) << 16)};
                        st<NT>(reinterpret_cast<u32x2 *>(o), p);
                    } else {
                        st_u16(o, static_cast<uint16_t>(narrow_bf16(s.x)));
                        if (c > 1) st_u16(o + 1, static_cast<uint16_t>(narrow_bf16(s.y)));
                        if (c > 2) st_u16(o + 2, static_cast<uint16_t>(narrow_bf16(s.z)));
                    }
                } else {
                    float *o = static_cast<float *>(out) + a;
                    if (c == 4) {
                        st<NT>(reinterpret_cast<f32x4 *>(o), s);
                    } else {
                        st_f32(o, s.x);
                        if (c > 1) st_f32(o + 1, s.y);
                        if (c > 2) st_f32(o + 2, s.z);
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------- wide accumulators
// Unordered accumulation whose error does not grow with the number of contributions or depend
// on their order: the running sum lives in binary64 shards (same element offsets as the
// binary32 ones), every contribution is added with a device-scope binary64 atomic, and the sum
// is rounded to binary32 once, at retrieval.  After C contributions the retrieved value is
// within 2^-24 * (1 + C * 2^-29) * sum|g| of the exact sum for ANY inputs, where a binary32
// accumulator can be off by (C - 1) * 2^-24 * sum|g|.  One element per lane and step, so that an
// atomic instruction of a wavefront covers 512 contiguous bytes.  The atomics are executed at
// the memory side like the binary32 ones, two requests per 16 elements instead of one.
enum : int { kWideAccumulate = 0, kWideReset = 1, kWideRetrieveF32 = 2, kWideRetrieveBf16 = 3 };

template <int OP>
__device__ __forceinline__ void wide_apply(double *acc, void *out, int64_t k, uint16_t g, float scale)
{
    if constexpr (OP == kWideAccumulate) {
        unsafeAtomicAdd(acc + k, static_cast<double>(widen_one(g)));
    } else if constexpr (OP == kWideReset) {
        *(ODC_GLOBAL double *)(acc + k) = 0.0;
    } else {
        // one rounding to binary32, then the multiply and cast of the binary32 retrieval
        const float v = scale * static_cast<float>(*(const ODC_GLOBAL double *)(acc + k));
        if constexpr (OP == kWideRetrieveF32) st_f32(static_cast<float *>(out) + k, v);
        else st_u16(static_cast<uint16_t *>(out) + k, static_cast<uint16_t>(narrow_bf16(v)));
    }
}

constexpr int kWideThreads = 256, kWideElems = 4;  // a tile: 1024 elements of one owner's shard

template <int OP>
__global__ __launch_bounds__(kWideThreads) void k_wide_flat(RankPtrs accs, RankPtrs outs, const uint16_t *__restrict__ grad,
                                                            int64_t S, int64_t N, int r0, float scale)
{
    const int64_t base = static_cast<int64_t>(r0 + static_cast<int>(blockIdx.y)) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    double *acc = static_cast<double *>(accs.p[blockIdx.y]);
    void *out = outs.p[blockIdx.y];
    const uint16_t *g = OP == kWideAccumulate ? grad + base : nullptr;  // no gradient in the other forms
    constexpr int kTile = kWideThreads * kWideElems;
    const int64_t ntiles = (valid + kTile - 1) / kTile;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        uint16_t gv[kWideElems];
#pragma unroll
        for (int u = 0; u < kWideElems; ++u) {
            const int64_t e = tile * kTile + u * kWideThreads + threadIdx.x;
            gv[u] = 0;
            if (OP == kWideAccumulate && e < valid) gv[u] = ld_u16(g + e);
        }
#pragma unroll
        for (int u = 0; u < kWideElems; ++u) {
            const int64_t e = tile * kTile + u * kWideThreads + threadIdx.x;
            if (e < valid) wide_apply<OP>(acc, out, e, gv[u], scale);
        }
    }
}

// Batched form: grid x = tiles of the rank arena, y = owners of this launch.
template <int OP>
__global__ __launch_bounds__(kBatchThreads) void k_wide_batched(BatchTable tb, RankPtrs accs, RankPtrs outs,
                                                                const uint16_t *__restrict__ grad, int r0, float scale)
{
    __shared__ TileIndex<1> lds;
    const int64_t ntiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rl = static_cast<int>(blockIdx.y);
    constexpr int E = kChunkElems / kBatchThreads;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (tile != static_cast<int64_t>(blockIdx.x)) __syncthreads();
        int t_lo, n;
        stage_tile<1>(tb, tile, ntiles, lds, t_lo, n);
        double *acc = static_cast<double *>(accs.p[rl]);
        void *out = outs.p[rl];
        uint16_t gv[E];
        bool on[E];
#pragma unroll
        for (int u = 0; u < E; ++u) {
            const int a_rel = u * kBatchThreads + static_cast<int>(threadIdx.x);
            const int64_t a = (tile << kChunkShift) + a_rel;
            on[u] = false;
            gv[u] = 0;
            if (a >= tb.arena_elems) continue;
            const TensorDesc d = tile_desc(tb, t_lo, n, a_rel, lds);
            const int64_t slot = a - d.shard_off;
            on[u] = valid_from(d, r0 + rl, slot, 1) == 1;
            if (OP == kWideAccumulate && on[u]) gv[u] = ld_u16(grad + d.full_off + static_cast<int64_t>(r0 + rl) * d.S + slot);
        }
#pragma unroll
        for (int u = 0; u < E; ++u)
            if (on[u]) wide_apply<OP>(acc, out, (tile << kChunkShift) + u * kBatchThreads + static_cast<int>(threadIdx.x), gv[u], scale);
    }
}

// ----------------------------------------------------------------------------- hybrid sharding
// Hybrid sharding (paper Section 6.1, Appendix E): parameters and gradients are sharded inside
// a group of R devices (a node) only, so every one of the K groups ends a minibatch with its
// own accumulated gradient shards; shard r of the minibatch gradient is their sum, taken in
// ascending group order with one binary32 add per further group:
//   out_r[i] = (((a_{0,r}[i] + a_{1,r}[i]) + a_{2,r}[i]) + ...)          i < valid_r
// A pass reads up to kReduceSources group shards per owner; a sum over more groups continues
// from the stored partial result (INIT = false), which changes no bit because the partial
// result is a binary32 value either way.  (K + 1) * 4 bytes per element per pass.

constexpr int kReduceSources = 8;  // group shards read per pass
constexpr int kReduceRanks = 16;   // owners per launch: 16 x 9 pointers travel in the kernel arguments

struct ReducePtrs {
    const float *src[kReduceRanks][kReduceSources];
    float *out[kReduceRanks];
};

// Sum of one vector position over the K sources of owner slot `rl`; INIT: starts from the first
// source, otherwise from the value stored in out.
template <int K, bool INIT>
__device__ __forceinline__ f32x4 reduce_vec(const ReducePtrs &p, int rl, int64_t a)
{
    f32x4 v[K];
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] = ld<true>(reinterpret_cast<const f32x4 *>(p.src[rl][k] + a));
    f32x4 s;
    if constexpr (INIT) s = v[0];
    else s = ld<true>(reinterpret_cast<const f32x4 *>(p.out[rl] + a));
#pragma unroll
    for (int k = INIT ? 1 : 0; k < K; ++k) {
        s.x = s.x + v[k].x;
        s.y = s.y + v[k].y;
        s.z = s.z + v[k].z;
        s.w = s.w + v[k].w;
    }
    return s;
}

template <int K, bool INIT>
__device__ __forceinline__ float reduce_one(const ReducePtrs &p, int rl, int64_t a)
{
    float s = INIT ? ld_f32(p.src[rl][0] + a) : ld_f32(p.out[rl] + a);
#pragma unroll
    for (int k = INIT ? 1 : 0; k < K; ++k) s = s + ld_f32(p.src[rl][k] + a);
    return s;
}

template <int K, bool INIT>
__global__ __launch_bounds__(64) void k_reduce_flat(ReducePtrs p, int64_t S, int64_t N, int r0)
{
    const int rl = static_cast<int>(blockIdx.y);
    const int64_t base = static_cast<int64_t>(r0 + rl) * S;
    int64_t valid = N - base;
    if (valid > S) valid = S;
    if (valid <= 0) return;
    const int64_t nvec = valid >> 2;
    const int tail = static_cast<int>(valid & 3);
    const int64_t ntiles = (nvec + 63) >> 6;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t q = (tile << 6) + threadIdx.x;
        if (q < nvec) st<true>(reinterpret_cast<f32x4 *>(p.out[rl] + 4 * q), reduce_vec<K, INIT>(p, rl, 4 * q));
    }
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < tail) {
        const int64_t k = 4 * nvec + threadIdx.x;
        st_f32(p.out[rl] + k, reduce_one<K, INIT>(p, rl, k));
    }
}

// Batched form: grid x = tiles of the rank arena, y = owners of this launch.
template <int K, bool INIT>
__global__ __launch_bounds__(kBatchThreads) void k_reduce_batched(BatchTable tb, ReducePtrs p, int r0)
{
    __shared__ TileIndex<1> lds;
    const int64_t ntiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rl = static_cast<int>(blockIdx.y);
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (tile != static_cast<int64_t>(blockIdx.x)) __syncthreads();
        int t_lo, n;
        stage_tile<1>(tb, tile, ntiles, lds, t_lo, n);
        if (n == 1 && tile_is_uniform(tb.desc[t_lo], tile << kChunkShift, r0 + rl, 1)) {
#pragma unroll
            for (int u = 0; u < kAccumItems; ++u) {
                const int64_t a = (tile << kChunkShift) + 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
                st<true>(reinterpret_cast<f32x4 *>(p.out[rl] + a), reduce_vec<K, INIT>(p, rl, a));
            }
            continue;
        }
#pragma unroll
        for (int u = 0; u < kAccumItems; ++u) {
            const int a_rel = 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            const int64_t a = (tile << kChunkShift) + a_rel;
            if (a >= tb.arena_elems) continue;
            const TensorDesc d = tile_desc(tb, t_lo, n, a_rel, lds);
            const int cnt = valid_from(d, r0 + rl, a - d.shard_off, 4);
            if (cnt == 4) {
                st<true>(reinterpret_cast<f32x4 *>(p.out[rl] + a), reduce_vec<K, INIT>(p, rl, a));
            } else if (cnt > 0 && a + 4 <= tb.arena_elems) {
                // ragged end of a shard piece: wide loads, element stores
                const f32x4 s = reduce_vec<K, INIT>(p, rl, a);
                st_f32(p.out[rl] + a, s.x);
                if (cnt > 1) st_f32(p.out[rl] + a + 1, s.y);
                if (cnt > 2) st_f32(p.out[rl] + a + 2, s.z);
            } else {
                for (int e = 0; e < cnt; ++e) st_f32(p.out[rl] + a + e, reduce_one<K, INIT>(p, rl, a + e));
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

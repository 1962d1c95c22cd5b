// Multi-tensor (T > 1) kernels: the LDS tile index, gather, scatter-accumulate, reset.
#pragma once

#include "odc_dev_common.h"
#include "odc_dev_flat.h"

namespace odc {
namespace {

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

}  // namespace
}  // namespace odc

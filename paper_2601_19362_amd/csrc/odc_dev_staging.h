// Server-side staging (Appendix B): per-client slots, slot states, push and drain kernels.
#pragma once

#include "odc_dev_batched.h"

namespace odc {
namespace {

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
// All flag accesses are device-scope atomics, ordered by acquire / release (on the access
// itself for claim and raise, by one fence per thread in snapshot and clear): the slot data
// written before a raise are visible to the drain that sees the flag, and the drain's reads
// are complete before a claim can see the slot empty again.  What the protocol assumes of the
// caller: the pushes of one client are serialised (Appendix B), and so are the drains.
constexpr int32_t kSlotEmpty = 0, kSlotFull = 1, kSlotWriting = 2;

// Relaxed load.  The copy workgroups of a push use it bare: they only ask "is this slot mine"
// (state writing, set by this push's own claim kernel, which ended before the copy kernel
// began, and changed by nobody else), and read no data that another stream publishes through
// the flag.  An acquire here would invalidate the caches once per workgroup (measured: push
// 12 x slower).
__device__ __forceinline__ int32_t flag_peek(const int32_t *f)
{
    return __scoped_atomic_load_n(f, __ATOMIC_RELAXED, __MEMORY_SCOPE_DEVICE);
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

template <bool NT, int RG>
__global__ __launch_bounds__(kBatchThreads) void k_stage_push_batched(BatchTable tb, RankPtrs staging,
                                                                      const uint16_t *__restrict__ grad,
                                                                      const int32_t *__restrict__ flags,
                                                                      int64_t slot, int R, int r0, int nr, int worker)
{
    __shared__ TileIndex<kPushChunks> lds;
    constexpr int kTile = kPushChunks * kChunkElems;
    const int64_t nchunks = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int64_t ntiles = (nchunks + kPushChunks - 1) / kPushChunks;
    const int rl0 = static_cast<int>(blockIdx.y) * RG;  // grid.y = groups of RG owners of this launch
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        if (tile != static_cast<int64_t>(blockIdx.x)) __syncthreads();
        // The slot states are requested without a branch (an owner beyond the launch reads the
        // last owner's flag and ignores it), so that they travel together with the index loads
        // of stage_tile instead of ahead of them.
        int32_t state[RG];
#pragma unroll
        for (int k = 0; k < RG; ++k) {
            const int rl = rl0 + k < nr ? rl0 + k : nr - 1;
            state[k] = flag_peek(flags + static_cast<int64_t>(r0 + rl) * R + worker);
        }
        int t_lo, n;
        stage_tile<kPushChunks>(tb, tile, nchunks, lds, t_lo, n);
        bool claimed[RG];  // uniform; an owner that refused the push is left alone
        bool any = false;
#pragma unroll
        for (int k = 0; k < RG; ++k) {
            claimed[k] = rl0 + k < nr && state[k] == kSlotWriting;
            any = any || claimed[k];
        }
        if (!any) continue;
        const int64_t a0 = tile * kTile;
        if constexpr (RG == 1) {
            // (only the one-owner variant, picked for layouts of large tensors, carries this path)
            const int r = r0 + rl0;
            if (n == 1 && tile_is_uniform(tb.desc[t_lo], a0, r, 1, kTile)) {
                uint16_t *dst = static_cast<uint16_t *>(staging.p[rl0]) + static_cast<int64_t>(worker) * slot;
                const TensorDesc d = tb.desc[t_lo];
                const uint16_t *src = grad + d.full_off + static_cast<int64_t>(r) * d.S - d.shard_off + a0;
                u32x4 w[kPushChunks];
#pragma unroll
                for (int u = 0; u < kPushChunks; ++u)
                    w[u] = ld_u128_unaligned<NT>(src + 8 * (u * kBatchThreads + static_cast<int>(threadIdx.x)));
#pragma unroll
                for (int u = 0; u < kPushChunks; ++u)
                    st<NT>(reinterpret_cast<u32x4 *>(dst + a0) + u * kBatchThreads + threadIdx.x, w[u]);
                continue;
            }
        }
        u32x4 v[kPushChunks][RG];
        bool on[kPushChunks][RG];
#pragma unroll
        for (int u = 0; u < kPushChunks; ++u) {
            const int a_rel = 8 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            const int64_t a = a0 + a_rel;
            const bool live = a < tb.arena_elems;
            TensorDesc d{};
            if (live) d = tile_desc(tb, t_lo, n, a_rel, lds);  // looked up once for all RG owners
#pragma unroll
            for (int k = 0; k < RG; ++k) {
                on[u][k] = false;
                v[u][k] = u32x4{0u, 0u, 0u, 0u};
                if (!live || !claimed[k]) continue;
                const int r = r0 + rl0 + k;
                const int64_t slot_in = a - d.shard_off;
                const int c = valid_from(d, r, slot_in, 8);
                if (c == 0) continue;
                const int64_t goff = d.full_off + static_cast<int64_t>(r) * d.S + slot_in;
                if (c == 8 || goff + 8 <= tb.full_elems) {
                    // a ragged end (c < 8) keeps the wide load; its spare lanes belong to the next
                    // piece of the gradient
                    on[u][k] = true;
                    v[u][k] = ld_u128_unaligned<NT && kPieceLoadsNT>(grad + goff);
                } else {  // the last elements of the gradient buffer
                    uint16_t *dst = static_cast<uint16_t *>(staging.p[rl0 + k]) + static_cast<int64_t>(worker) * slot;
                    for (int e = 0; e < c; ++e) st_u16(dst + a + e, ld_u16(grad + goff + e));
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kPushChunks; ++u) {
            const int64_t a = a0 + 8 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            // A ragged item is stored whole as well: its spare lanes fall into the alignment gap
            // behind the piece, which in a staging slot belongs to nobody (the drain never takes
            // them), and a slot written in whole 16-byte vectors has no partly written sector.
#pragma unroll
            for (int k = 0; k < RG; ++k)
                if (on[u][k])
                    st<NT>(reinterpret_cast<u32x4 *>(static_cast<uint16_t *>(staging.p[rl0 + k]) +
                                                     static_cast<int64_t>(worker) * slot + a),
                           v[u][k]);
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

// One 64-thread workgroup per owner.  Snapshot: the owner's full slots, ascending, are written as
// a list snapshot[r * (R + 1)] = count, then the client indices.  Clear: every listed flag is
// lowered.  Taking the list once per drain keeps all workgroups of the accumulate kernel on the
// same set of contributions even if pushes from other streams raise more flags meanwhile.
//
// Lane w reads the flag of client w (one contiguous 256-byte row per load instruction; a thread
// per owner walking its row alone spent 14 us on R = 64 waiting for one uncached load after the
// other), the states go through LDS, and every lane counts the full slots before its own to
// find its place in the list.  The flags are read with relaxed device-scope loads and ONE acquire
// fence follows: that orders everything after the fence behind every raise whose flag was
// seen, as acquire loads would, without invalidating the caches once per flag.  The clear
// mirrors it: one release fence, then relaxed stores.
__global__ __launch_bounds__(64) void k_stage_snapshot(const int32_t *flags, int32_t *snapshot, int R)
{
    __shared__ int32_t state[64];
    const int lane = static_cast<int>(threadIdx.x);
    for (int r = blockIdx.x; r < R; r += gridDim.x) {
        ODC_GLOBAL int32_t *list = (ODC_GLOBAL int32_t *)(snapshot + static_cast<int64_t>(r) * (R + 1));
        const int32_t *row = flags + static_cast<int64_t>(r) * R;
        int n = 0;  // the same in every lane
        for (int w0 = 0; w0 < R; w0 += 64) {
            const int w = w0 + lane;
            __syncthreads();  // the previous round's reads of `state` are over
            state[lane] = w < R ? flag_peek(row + w) : kSlotEmpty;
            __syncthreads();
            int before = 0, total = 0;
            for (int j = 0; j < 64; ++j) {
                const int full = state[j] == kSlotFull ? 1 : 0;
                before += j < lane ? full : 0;
                total += full;
            }
            if (state[lane] == kSlotFull) list[1 + n + before] = w;
            n += total;
        }
        if (lane == 0) list[0] = n;
    }
    __scoped_atomic_thread_fence(__ATOMIC_ACQUIRE, __MEMORY_SCOPE_DEVICE);
}

__global__ __launch_bounds__(64) void k_stage_clear(int32_t *flags, const int32_t *snapshot, int R)
{
    __scoped_atomic_thread_fence(__ATOMIC_RELEASE, __MEMORY_SCOPE_DEVICE);
    for (int r = blockIdx.x; r < R; r += gridDim.x) {
        const ODC_GLOBAL int32_t *list = (const ODC_GLOBAL int32_t *)(snapshot + static_cast<int64_t>(r) * (R + 1));
        int32_t *row = flags + static_cast<int64_t>(r) * R;
        const int n = list[0];
        for (int k = static_cast<int>(threadIdx.x); k < n; k += 64)
            __scoped_atomic_store_n(row + list[1 + k], kSlotEmpty, __ATOMIC_RELAXED, __MEMORY_SCOPE_DEVICE);
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
// `first`: entries of the list before it have been added by the caller.
template <bool NT>
__device__ __forceinline__ f32x4 drain_vec(f32x4 acc, const uint16_t *__restrict__ stage, int64_t slot, int64_t a,
                                           const int32_t *__restrict__ list, int first = 0)
{
    constexpr int B = 4;
    const int n = list[0];
    for (int c = first; c < n; c += B) {
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
        // Two phases, like the accumulate kernel: the accumulator vector and the first staged
        // vectors of every item of the thread are requested before anything is stored (a store
        // in between would hold the later loads back: for all the compiler knows they alias).
        // kind: 0 nothing, 1 whole vector (full, ragged end, or the alignment gap that completes
        // a piece's last line), 2 the arena's last elements, one by one.
        constexpr int B = 4;
        const int staged = list[0];
        f32x4 old[kAccumItems];
        u32x2 gv[kAccumItems][B];
        int cnt[kAccumItems], kind[kAccumItems];
#pragma unroll
        for (int u = 0; u < kAccumItems; ++u) {
            const int a_rel = 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            const int64_t a = (tile << kChunkShift) + a_rel;
            kind[u] = 0;
            cnt[u] = 0;
            if (a >= tb.arena_elems) continue;
            const TensorDesc d = tile_desc(tb, t_lo, n, a_rel, lds);
            bool gap;
            cnt[u] = vec_cover(d, r, a - d.shard_off, gap);
            if (cnt[u] == 0 && !gap) continue;
            if (cnt[u] < 4 && a + 4 > tb.arena_elems) {
                kind[u] = cnt[u] > 0 ? 2 : 0;
                continue;
            }
            // (a ragged end keeps the wide loads: every staging slot is at least as long as the
            // arena rounded up to 8)
            kind[u] = 1;
            old[u] = ld<NT>(reinterpret_cast<const f32x4 *>(arena + a));
            if (cnt[u] > 0) {
#pragma unroll
                for (int j = 0; j < B; ++j)
                    if (j < staged)
                        gv[u][j] = ld<NT>(reinterpret_cast<const u32x2 *>(stage + static_cast<int64_t>(list[1 + j]) * slot + a));
            }
        }
#pragma unroll
        for (int u = 0; u < kAccumItems; ++u) {
            const int64_t a = (tile << kChunkShift) + 4 * (u * kBatchThreads + static_cast<int>(threadIdx.x));
            if (kind[u] == 1) {
                f32x4 sum = old[u];
                if (cnt[u] > 0) {
#pragma unroll
                    for (int j = 0; j < B; ++j)
                        if (j < staged) sum = add4<false>(sum, gv[u][j], 1.0f);
                    if (staged > B) sum = drain_vec<NT>(sum, stage, slot, a, list, B);
                }
                // lanes beyond cnt carry the bits that were read
                st<NT>(reinterpret_cast<f32x4 *>(arena + a), cnt[u] == 4 ? sum : keep_tail(sum, old[u], cnt[u]));
            } else if (kind[u] == 2) {
                for (int e = 0; e < cnt[u]; ++e) st_f32(arena + a + e, drain_one(ld_f32(arena + a + e), stage, slot, a + e, list));
            }
        }
    }
}

}  // namespace
}  // namespace odc

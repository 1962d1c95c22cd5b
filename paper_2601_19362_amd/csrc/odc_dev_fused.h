// Fused accumulate: several contributions applied in one pass over the accumulators.
#pragma once

#include "odc_dev_batched.h"

namespace odc {
namespace {

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

}  // namespace
}  // namespace odc

// Wide (binary64) accumulators for the unordered mode.
#pragma once

#include "odc_dev_batched.h"
#include "odc_dev_retrieve.h"

namespace odc {
namespace {

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

}  // namespace
}  // namespace odc

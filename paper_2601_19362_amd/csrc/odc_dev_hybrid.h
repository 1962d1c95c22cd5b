// Hybrid sharding (Section 6.1): the sum of the groups' accumulator shards at the minibatch end.
#pragma once

#include "odc_dev_batched.h"

namespace odc {
namespace {

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

}  // namespace
}  // namespace odc

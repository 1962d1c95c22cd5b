// Minibatch-end retrieval (Section 3.2): out = cast(scale * acc).
#pragma once

#include "odc_dev_batched.h"

namespace odc {
namespace {

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

}  // namespace
}  // namespace odc

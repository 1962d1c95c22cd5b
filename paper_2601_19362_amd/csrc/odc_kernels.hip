// Kernel launchers for the ODC hot path (gfx950).  The kernels themselves are in the
// odc_dev_*.h headers (one per family, all included by odc_device.h); this file only picks an
// instantiation and a grid.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "odc_device.h"
#include "odc_internal.h"

namespace odc {
namespace {

// -------------------------------------------------------------------------------- launching
RankPtrs pack(const void *const *ptrs, int nr)
{
    RankPtrs rp;
    for (int k = 0; k < kRanksPerLaunch; ++k) rp.p[k] = k < nr ? const_cast<void *>(ptrs[k]) : nullptr;
    return rp;
}

// Grid for `items` work items at TPB * U items per tile.  With tile remapping the x extent
// is rounded up to a multiple of 8 (one slot per XCD part) and never capped.
dim3 grid_for(const Tuning &t, int64_t items, int per_block, int nr)
{
    unsigned gx = grid_x_for(items, per_block, t.tile_remap ? 0 : t.max_grid_x);
    if (t.tile_remap && gx <= 0x7FFFFFF0u) gx = (gx + 7u) & ~7u;
    return dim3(gx, static_cast<unsigned>(nr), 1);
}

dim3 plain_grid(const Tuning &t, int64_t items, int per_block, int nr)
{
    return dim3(grid_x_for(items, per_block, t.max_grid_x), static_cast<unsigned>(nr), 1);
}

int finish() { return static_cast<int>(hipGetLastError()); }

// Dispatch runtime (threads, unroll, non-temporal) to the matching instantiation.  Inside
// CALL the chosen values are the constants TPB_, U_ and NT_.
#define ODC_DISPATCH_NT(NTF, CALL)                       \
    do {                                                 \
        if (NTF) { constexpr bool NT_ = true; CALL; }    \
        else { constexpr bool NT_ = false; CALL; }       \
    } while (0)

#define ODC_DISPATCH_U(UN, NTF, CALL)                                           \
    do {                                                                        \
        switch (UN) {                                                           \
            case 1: { constexpr int U_ = 1; ODC_DISPATCH_NT(NTF, CALL); } break; \
            case 2: { constexpr int U_ = 2; ODC_DISPATCH_NT(NTF, CALL); } break; \
            default: { constexpr int U_ = 4; ODC_DISPATCH_NT(NTF, CALL); } break; \
        }                                                                       \
    } while (0)

#define ODC_DISPATCH(TPBV, UN, NTF, CALL)                                                  \
    do {                                                                                   \
        switch (TPBV) {                                                                    \
            case 64: { constexpr int TPB_ = 64; ODC_DISPATCH_U(UN, NTF, CALL); } break;     \
            case 128: { constexpr int TPB_ = 128; ODC_DISPATCH_U(UN, NTF, CALL); } break;   \
            default: { constexpr int TPB_ = 256; ODC_DISPATCH_U(UN, NTF, CALL); } break;    \
        }                                                                                  \
    } while (0)

}  // namespace

int launch_gather_flat(const void *const *ptrs, int r0, int nr, void *full, int64_t S, int64_t N,
                       void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (t.gather_store_sc1 && t.nontemporal) {
        ODC_DISPATCH(t.gather_threads, t.gather_unroll, true,
                     (k_gather_flat<TPB_, U_, NT_, true><<<grid_for(t, (S >> 3) + 1, TPB_ * U_, nr), TPB_, 0, s>>>(
                         rp, static_cast<uint16_t *>(full), S, N, r0, t.tile_remap)));
    } else {
        ODC_DISPATCH(t.gather_threads, t.gather_unroll, t.nontemporal != 0,
                     (k_gather_flat<TPB_, U_, NT_, false><<<grid_for(t, (S >> 3) + 1, TPB_ * U_, nr), TPB_, 0, s>>>(
                         rp, static_cast<uint16_t *>(full), S, N, r0, t.tile_remap)));
    }
    return finish();
}

int launch_accum_flat(void *const *ptrs, int r0, int nr, const void *grad, int64_t S, int64_t N,
                      bool atomic, bool weighted, float w, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t *g = static_cast<const uint16_t *>(grad);
#define ODC_ACCUM_FLAT(ATOMIC_, WEIGHTED_, NTF)                                                                 \
    ODC_DISPATCH(t.accum_threads, t.accum_unroll, NTF,                                                          \
                 (k_accum_flat<TPB_, U_, NT_, ATOMIC_, WEIGHTED_><<<grid_for(t, (S >> 2) + 1, TPB_ * U_, nr), TPB_, 0, s>>>( \
                     rp, g, S, N, r0, t.tile_remap, w)))
    if (atomic && weighted) ODC_ACCUM_FLAT(true, true, false);
    else if (atomic) ODC_ACCUM_FLAT(true, false, false);
    else if (weighted) ODC_ACCUM_FLAT(false, true, t.nontemporal != 0);
    else ODC_ACCUM_FLAT(false, false, t.nontemporal != 0);
#undef ODC_ACCUM_FLAT
    return finish();
}

int launch_reset_flat(void *const *ptrs, int r0, int nr, int64_t S, int64_t N, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ODC_DISPATCH(t.reset_threads, t.reset_unroll, t.nontemporal != 0,
                 (k_reset_flat<TPB_, U_, NT_><<<grid_for(t, (S >> 2) + 1, TPB_ * U_, nr), TPB_, 0, s>>>(
                     rp, S, N, r0, t.tile_remap)));
    return finish();
}

// The batched kernels use fixed 256-thread workgroups: grid x = tiles (capped by the
// max_grid_x knob, the kernels loop), y = owner groups for the arena-major kernels.
static unsigned batched_grid_x(const Tuning &t, int64_t tiles)
{
    return grid_x_for(tiles, 1, t.max_grid_x);
}

// Owners per workgroup in the batched accumulate / reset / retrieve kernels.  A workgroup that
// serves two owners looks its tensors up once for both, which pays for the read-modify-write
// kernels on layouts of many small tensors when there is enough work to fill the chip; the
// write-only reset, and layouts whose shard pieces are long (mean of 1024 elements or more:
// most tiles then lie inside one tensor and take the lean path), are fastest with one.
static int rank_group(const Tuning &t, const BatchTable &tb, int64_t tiles, int nr, int preferred)
{
    const int forced = t.batch_rank_group;
    if (forced > 0) return forced;
    if (tb.arena_elems / tb.T >= 1024) return 1;
    for (int rg = preferred; rg > 1; rg >>= 1)
        if (tiles * ((nr + rg - 1) / rg) >= 4096) return rg;
    return 1;
}

#define ODC_DISPATCH_RG(RGV, NTF, CALL)                                            \
    do {                                                                           \
        switch (RGV) {                                                             \
            case 8: { constexpr int RG_ = 8; ODC_DISPATCH_NT(NTF, CALL); } break;   \
            case 4: { constexpr int RG_ = 4; ODC_DISPATCH_NT(NTF, CALL); } break;   \
            case 2: { constexpr int RG_ = 2; ODC_DISPATCH_NT(NTF, CALL); } break;   \
            default: { constexpr int RG_ = 1; ODC_DISPATCH_NT(NTF, CALL); } break;  \
        }                                                                          \
    } while (0)

int launch_gather_batched(const BatchTable &tb, const void *const *ptrs, int r0, int nr, void *full,
                          void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint16_t *out = static_cast<uint16_t *>(full);
    const int64_t chunks = (tb.full_elems + kChunkElems - 1) >> kChunkShift;
    const int64_t tiles = (chunks + kGatherChunks - 1) / kGatherChunks;
    // Tiles go to the XCDs in blocks of consecutive tiles (knob: up to 16); a launch with few
    // tiles takes smaller blocks, so that every XCD still gets at least eight of them and no
    // XCD is left without work.
    int block = t.gather_tile_xcd_block;
    while (block > 1 && tiles < int64_t{64} * block) block >>= 1;
    int tshift = 0;
    while ((1 << tshift) < block) ++tshift;
    const int64_t tgroup = int64_t{8} << tshift;
    const dim3 grid(batched_grid_x(t, (tiles + tgroup - 1) / tgroup * tgroup));
#define ODC_GATHER_BATCHED(CAP_, BIG_)                                 \
    ODC_DISPATCH_NT(t.nontemporal != 0,                         \
                    (k_gather_batched<NT_, CAP_, BIG_><<<grid, kBatchThreads, 0, s>>>(tb, rp, out, r0, nr, tshift)))
    const bool few = tb.gather_tile_tensors <= kGatherFewTensors;
    if (few && tb.gather_big) ODC_GATHER_BATCHED(kGatherFewTensors, true);
    else if (few) ODC_GATHER_BATCHED(kGatherFewTensors, false);
    else if (tb.gather_big) ODC_GATHER_BATCHED(kGatherMaxTensors, true);
    else ODC_GATHER_BATCHED(kGatherMaxTensors, false);
#undef ODC_GATHER_BATCHED
    return finish();
}

int launch_accum_batched(const BatchTable &tb, void *const *ptrs, int r0, int nr, const void *grad,
                         bool atomic, bool weighted, float w, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t *g = static_cast<const uint16_t *>(grad);
    const int64_t tiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rg = rank_group(t, tb, tiles, nr, 2);
    const dim3 grid(batched_grid_x(t, tiles), static_cast<unsigned>((nr + rg - 1) / rg));
#define ODC_ACCUM_BATCHED(ATOMIC_, WEIGHTED_, NTF)                                                     \
    ODC_DISPATCH_RG(rg, NTF,                                                                           \
                    (k_accum_batched<RG_, NT_, ATOMIC_, WEIGHTED_><<<grid, kBatchThreads, 0, s>>>(tb, rp, g, r0, nr, \
                                                                                                  w)))
    if (atomic && weighted) ODC_ACCUM_BATCHED(true, true, false);
    else if (atomic) ODC_ACCUM_BATCHED(true, false, false);
    else if (weighted) ODC_ACCUM_BATCHED(false, true, t.nontemporal != 0);
    else ODC_ACCUM_BATCHED(false, false, t.nontemporal != 0);
#undef ODC_ACCUM_BATCHED
    return finish();
}

int launch_reset_batched(const BatchTable &tb, void *const *ptrs, int r0, int nr, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t tiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rg = rank_group(t, tb, tiles, nr, 1);
    const dim3 grid(batched_grid_x(t, tiles), static_cast<unsigned>((nr + rg - 1) / rg));
    ODC_DISPATCH_RG(rg, t.nontemporal != 0,
                    (k_reset_batched<RG_, NT_><<<grid, kBatchThreads, 0, s>>>(tb, rp, r0, nr)));
    return finish();
}

#define ODC_DISPATCH_K(KV, CALL)                                \
    do {                                                        \
        switch (KV) {                                           \
            case 2: { constexpr int K_ = 2; CALL; } break;       \
            case 3: { constexpr int K_ = 3; CALL; } break;       \
            case 4: { constexpr int K_ = 4; CALL; } break;       \
            case 5: { constexpr int K_ = 5; CALL; } break;       \
            case 6: { constexpr int K_ = 6; CALL; } break;       \
            case 7: { constexpr int K_ = 7; CALL; } break;       \
            default: { constexpr int K_ = 8; CALL; } break;      \
        }                                                       \
    } while (0)

static GradPtrs pack_grads(const void *const *grads, int count)
{
    GradPtrs gp;
    for (int k = 0; k < kMaxFused; ++k) gp.p[k] = static_cast<const uint16_t *>(k < count ? grads[k] : grads[0]);
    return gp;
}

int launch_accum_multi_flat(void *const *ptrs, int r0, int nr, const void *const *grads, int count, int64_t S,
                            int64_t N, bool atomic, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    const GradPtrs gp = pack_grads(grads, count);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid = plain_grid(t, (S >> 2) + 1, 64, nr);
    if (atomic) ODC_DISPATCH_K(count, (k_accum_multi_flat<K_, true><<<grid, 64, 0, s>>>(rp, gp, S, N, r0)));
    else ODC_DISPATCH_K(count, (k_accum_multi_flat<K_, false><<<grid, 64, 0, s>>>(rp, gp, S, N, r0)));
    return finish();
}

int launch_accum_multi_batched(const BatchTable &tb, void *const *ptrs, int r0, int nr, const void *const *grads,
                               int count, bool atomic, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    const GradPtrs gp = pack_grads(grads, count);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(batched_grid_x(t, (tb.arena_elems + kChunkElems - 1) >> kChunkShift), static_cast<unsigned>(nr));
    if (atomic)
        ODC_DISPATCH_K(count, (k_accum_multi_batched<K_, true><<<grid, kBatchThreads, 0, s>>>(tb, rp, gp, r0)));
    else
        ODC_DISPATCH_K(count, (k_accum_multi_batched<K_, false><<<grid, kBatchThreads, 0, s>>>(tb, rp, gp, r0)));
    return finish();
}

int launch_stage_zero(void *flags, int64_t count, void *stream)
{
    const unsigned blocks = grid_x_for(count, 256, 1024);
    k_stage_zero<<<dim3(blocks), 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<int32_t *>(flags), count);
    return finish();
}

int launch_stage_push_flat(void *const *staging, int r0, int nr, const void *grad, const void *flags, int64_t S,
                           int64_t N, int64_t slot, int R, int worker, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(staging, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ODC_DISPATCH_NT(t.nontemporal != 0,
                    (k_stage_push_flat<NT_><<<plain_grid(t, (S >> 3) + 1, 64, nr), 64, 0, s>>>(
                        rp, static_cast<const uint16_t *>(grad), static_cast<const int32_t *>(flags), S, N, slot, R,
                        r0, worker)));
    return finish();
}

int launch_stage_push_batched(const BatchTable &tb, void *const *staging, int r0, int nr, const void *grad,
                              const void *flags, int64_t slot, int R, int worker, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs rp = pack(staging, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t chunks = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int64_t tiles = (chunks + kPushChunks - 1) / kPushChunks;
    const int rg = rank_group(t, tb, tiles, nr, 2) >= 2 ? 2 : 1;
    const dim3 grid(batched_grid_x(t, tiles), static_cast<unsigned>((nr + rg - 1) / rg));
    const uint16_t *g = static_cast<const uint16_t *>(grad);
    const int32_t *f = static_cast<const int32_t *>(flags);
    if (rg == 2)
        ODC_DISPATCH_NT(t.nontemporal != 0, (k_stage_push_batched<NT_, 2><<<grid, kBatchThreads, 0, s>>>(
                                                tb, rp, g, f, slot, R, r0, nr, worker)));
    else
        ODC_DISPATCH_NT(t.nontemporal != 0, (k_stage_push_batched<NT_, 1><<<grid, kBatchThreads, 0, s>>>(
                                                tb, rp, g, f, slot, R, r0, nr, worker)));
    return finish();
}

int launch_stage_claim(void *flags, int R, int worker, void *stream)
{
    k_stage_claim<<<dim3((R + 63) / 64), 64, 0, static_cast<hipStream_t>(stream)>>>(static_cast<int32_t *>(flags), R,
                                                                                   worker);
    return finish();
}

int launch_stage_raise(void *flags, int R, int worker, void *stream)
{
    k_stage_raise<<<dim3((R + 63) / 64), 64, 0, static_cast<hipStream_t>(stream)>>>(static_cast<int32_t *>(flags), R,
                                                                                   worker);
    return finish();
}

int launch_stage_snapshot(const void *flags, void *snapshot, int R, void *stream)
{
    k_stage_snapshot<<<dim3(static_cast<unsigned>(R)), 64, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const int32_t *>(flags), static_cast<int32_t *>(snapshot), R);
    return finish();
}

int launch_stage_clear(void *flags, const void *snapshot, int R, void *stream)
{
    k_stage_clear<<<dim3(static_cast<unsigned>(R)), 64, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<int32_t *>(flags), static_cast<const int32_t *>(snapshot), R);
    return finish();
}

int launch_stage_drain_flat(void *const *accs, const void *const *staging, int r0, int nr, const void *snapshot,
                            int64_t S, int64_t N, int64_t slot, int R, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs ra = pack(accs, nr);
    const RankPtrs rs = pack(staging, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ODC_DISPATCH_NT(t.nontemporal != 0,
                    (k_stage_drain_flat<NT_><<<plain_grid(t, (S >> 2) + 1, 64, nr), 64, 0, s>>>(
                        ra, rs, static_cast<const int32_t *>(snapshot), S, N, slot, R, r0)));
    return finish();
}

int launch_stage_drain_batched(const BatchTable &tb, void *const *accs, const void *const *staging, int r0, int nr,
                               const void *snapshot, int64_t slot, int R, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs ra = pack(accs, nr);
    const RankPtrs rs = pack(staging, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(batched_grid_x(t, (tb.arena_elems + kChunkElems - 1) >> kChunkShift), static_cast<unsigned>(nr));
    ODC_DISPATCH_NT(t.nontemporal != 0,
                    (k_stage_drain_batched<NT_><<<grid, kBatchThreads, 0, s>>>(
                        tb, ra, rs, static_cast<const int32_t *>(snapshot), slot, R, r0)));
    return finish();
}

int launch_retrieve_flat(const void *const *acc, void *const *out, int r0, int nr, int64_t S, int64_t N,
                         float scale, bool bf16, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs ra = pack(acc, nr);
    const RankPtrs ro = pack(out, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (bf16) {
        ODC_DISPATCH(t.reset_threads, t.reset_unroll, t.nontemporal != 0,
                     (k_retrieve_flat<TPB_, U_, NT_, true><<<plain_grid(t, (S >> 2) + 1, TPB_ * U_, nr), TPB_, 0, s>>>(
                         ra, ro, S, N, r0, scale)));
    } else {
        ODC_DISPATCH(t.reset_threads, t.reset_unroll, t.nontemporal != 0,
                     (k_retrieve_flat<TPB_, U_, NT_, false><<<plain_grid(t, (S >> 2) + 1, TPB_ * U_, nr), TPB_, 0, s>>>(
                         ra, ro, S, N, r0, scale)));
    }
    return finish();
}

int launch_retrieve_batched(const BatchTable &tb, const void *const *acc, void *const *out, int r0, int nr,
                            float scale, bool bf16, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs ra = pack(acc, nr);
    const RankPtrs ro = pack(out, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t tiles = (tb.arena_elems + kChunkElems - 1) >> kChunkShift;
    const int rg = rank_group(t, tb, tiles, nr, 2);
    const dim3 grid(batched_grid_x(t, tiles), static_cast<unsigned>((nr + rg - 1) / rg));
    if (bf16) {
        ODC_DISPATCH_RG(rg, t.nontemporal != 0,
                        (k_retrieve_batched<RG_, NT_, true><<<grid, kBatchThreads, 0, s>>>(tb, ra, ro, r0, nr, scale)));
    } else {
        ODC_DISPATCH_RG(rg, t.nontemporal != 0,
                        (k_retrieve_batched<RG_, NT_, false><<<grid, kBatchThreads, 0, s>>>(tb, ra, ro, r0, nr, scale)));
    }
    return finish();
}

// Wide (binary64) accumulators: op 0 accumulate, 1 reset, 2 retrieve to binary32, 3 retrieve to bf16.
int launch_wide(const BatchTable *tb, int op, void *const *accs, void *const *outs, const void *grad, int r0, int nr,
                int64_t S, int64_t N, float scale, void *stream)
{
    const Tuning t = tuning();
    const RankPtrs ra = pack(accs, nr);
    RankPtrs ro{};
    if (outs) ro = pack(outs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t *g = static_cast<const uint16_t *>(grad);
#define ODC_WIDE(OP_)                                                                                         \
    do {                                                                                                      \
        if (tb) {                                                                                             \
            const dim3 grid(batched_grid_x(t, (tb->arena_elems + kChunkElems - 1) >> kChunkShift),             \
                            static_cast<unsigned>(nr));                                                       \
            k_wide_batched<OP_><<<grid, kBatchThreads, 0, s>>>(*tb, ra, ro, g, r0, scale);                     \
        } else {                                                                                              \
            k_wide_flat<OP_><<<plain_grid(t, S + 1, kWideThreads * kWideElems, nr), kWideThreads, 0, s>>>(ra, ro, g, S, N, \
                                                                                                         r0, scale); \
        }                                                                                                     \
    } while (0)
    switch (op) {
        case kWideAccumulate: ODC_WIDE(kWideAccumulate); break;
        case kWideReset: ODC_WIDE(kWideReset); break;
        case kWideRetrieveF32: ODC_WIDE(kWideRetrieveF32); break;
        default: ODC_WIDE(kWideRetrieveBf16); break;
    }
#undef ODC_WIDE
    return finish();
}

// One pass of the group reduction: owners [r0, r0 + nr), nr <= kReduceRanks; `count` sources per
// owner (1..kReduceSources), srcs[k * stride + r] = source k of owner r0 + r; init: the sum starts
// from the first source instead of the stored value of out.
static_assert(kReduceSources == kReduceSourcesPerPass && kReduceRanks == kReduceRanksPerLaunch,
              "the host loop and the kernels must agree on the pass shape");

int launch_reduce_groups(const BatchTable *tb, const void *const *srcs, int64_t stride, int count, bool init,
                         void *const *outs, int r0, int nr, int64_t S, int64_t N, void *stream)
{
    const Tuning t = tuning();
    ReducePtrs p{};
    for (int r = 0; r < kReduceRanks; ++r) {
        for (int k = 0; k < kReduceSources; ++k)
            p.src[r][k] = static_cast<const float *>(r < nr && k < count ? srcs[k * stride + r] : nullptr);
        p.out[r] = static_cast<float *>(r < nr ? outs[r] : nullptr);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
#define ODC_REDUCE(K_, INIT_)                                                                                  \
    do {                                                                                                       \
        if (tb) {                                                                                              \
            const dim3 grid(batched_grid_x(t, (tb->arena_elems + kChunkElems - 1) >> kChunkShift),                 \
                            static_cast<unsigned>(nr));                                                        \
            k_reduce_batched<K_, INIT_><<<grid, kBatchThreads, 0, s>>>(*tb, p, r0);                              \
        } else {                                                                                               \
            k_reduce_flat<K_, INIT_><<<plain_grid(t, (S >> 2) + 1, 64, nr), 64, 0, s>>>(p, S, N, r0);               \
        }                                                                                                      \
    } while (0)
#define ODC_REDUCE_K(INIT_)                               \
    switch (count) {                                      \
        case 1: ODC_REDUCE(1, INIT_); break;              \
        case 2: ODC_REDUCE(2, INIT_); break;              \
        case 3: ODC_REDUCE(3, INIT_); break;              \
        case 4: ODC_REDUCE(4, INIT_); break;              \
        case 5: ODC_REDUCE(5, INIT_); break;              \
        case 6: ODC_REDUCE(6, INIT_); break;              \
        case 7: ODC_REDUCE(7, INIT_); break;              \
        default: ODC_REDUCE(8, INIT_); break;             \
    }
    if (init) ODC_REDUCE_K(true)
    else ODC_REDUCE_K(false)
#undef ODC_REDUCE_K
#undef ODC_REDUCE
    return finish();
}

// ------------------------------------------------------------------ fixed scratch, no allocation
// Snapshot list of odc_stage_drain_noalloc: lives in the code object, one copy per GPU, so the
// entry point needs no workspace from the caller and never allocates.  The array's name is
// only a host-side handle; its device address is looked up once per device and kept.
namespace {
constexpr int kScratchDevices = 64;
static __device__ __align__(256) int32_t scratch[kStageScratchMaxRanks * (kStageScratchMaxRanks + 1)];
std::mutex scratch_mu;
int32_t *scratch_ptr[kScratchDevices] = {};
}  // namespace

int stage_scratch(int device, int32_t **out)
{
    *out = nullptr;
    if (device < 0 || device >= kScratchDevices) return static_cast<int>(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[device]) {
        // `device` is the current device (the caller has checked): the lookup returns the
        // address of this device's copy of the array
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return static_cast<int>(e);
        if (!p) return static_cast<int>(hipErrorInvalidSymbol);
        scratch_ptr[device] = static_cast<int32_t *>(p);
    }
    *out = scratch_ptr[device];
    return 0;
}

int launch_probe_copy(void *dst, const void *src, int64_t bytes, void *stream)
{
    const int64_t nvec = bytes >> 4;
    if (nvec == 0) return 0;
    constexpr int TPB = 256, U = 4;
    const int64_t blocks = (nvec + TPB * U - 1) / (TPB * U);
    if (blocks > 0x7FFFFFFF) return static_cast<int>(hipErrorInvalidValue);
    k_probe_copy<TPB, U><<<dim3(static_cast<unsigned>(blocks)), TPB, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), nvec);
    return finish();
}

}  // namespace odc

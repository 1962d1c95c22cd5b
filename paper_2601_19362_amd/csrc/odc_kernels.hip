// Kernel launchers for the ODC hot path (gfx950).  The kernels themselves are in
// odc_device.h; this file only picks an instantiation and a grid.
#include <hip/hip_runtime.h>

#include <cstdint>

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

dim3 grid_for(int64_t items, int per_block, int nr)
{
    return dim3(grid_x_for(items, per_block, tuning().max_grid_x), static_cast<unsigned>(nr), 1);
}

int finish() { return static_cast<int>(hipGetLastError()); }

// Dispatch a runtime (unroll, non-temporal) pair to the matching instantiation.
#define ODC_DISPATCH_U_NT(UN, NTF, CALL)                                  \
    do {                                                                  \
        if (NTF) {                                                        \
            switch (UN) {                                                 \
                case 1: { constexpr int U_ = 1; constexpr bool NT_ = true; CALL; } break;  \
                case 2: { constexpr int U_ = 2; constexpr bool NT_ = true; CALL; } break;  \
                case 8: { constexpr int U_ = 8; constexpr bool NT_ = true; CALL; } break;  \
                default: { constexpr int U_ = 4; constexpr bool NT_ = true; CALL; } break; \
            }                                                             \
        } else {                                                          \
            switch (UN) {                                                 \
                case 1: { constexpr int U_ = 1; constexpr bool NT_ = false; CALL; } break;  \
                case 2: { constexpr int U_ = 2; constexpr bool NT_ = false; CALL; } break;  \
                case 8: { constexpr int U_ = 8; constexpr bool NT_ = false; CALL; } break;  \
                default: { constexpr int U_ = 4; constexpr bool NT_ = false; CALL; } break; \
            }                                                             \
        }                                                                 \
    } while (0)

}  // namespace

int launch_gather_flat(const void *const *ptrs, int r0, int nr, void *full, int64_t S, int64_t N,
                       void *stream)
{
    const Tuning &t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ODC_DISPATCH_U_NT(t.gather_unroll, t.nontemporal != 0,
                      (k_gather_flat<U_, NT_><<<grid_for((S >> 3) + 1, kThreads * U_, nr), kThreads, 0, s>>>(
                          rp, static_cast<uint16_t *>(full), S, N, r0)));
    return finish();
}

int launch_accum_flat(void *const *ptrs, int r0, int nr, const void *grad, int64_t S, int64_t N,
                      bool atomic, void *stream)
{
    const Tuning &t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t *g = static_cast<const uint16_t *>(grad);
    if (atomic) {
        ODC_DISPATCH_U_NT(t.accum_unroll, false,
                          (k_accum_flat<U_, 4, NT_, true><<<grid_for((S >> 2) + 1, kThreads * U_, nr), kThreads, 0, s>>>(
                              rp, g, S, N, r0)));
    } else if (t.accum_width == 8) {
        ODC_DISPATCH_U_NT(t.accum_unroll, t.nontemporal != 0,
                          (k_accum_flat<U_, 8, NT_, false><<<grid_for((S >> 3) + 1, kThreads * U_, nr), kThreads, 0, s>>>(
                              rp, g, S, N, r0)));
    } else {
        ODC_DISPATCH_U_NT(t.accum_unroll, t.nontemporal != 0,
                          (k_accum_flat<U_, 4, NT_, false><<<grid_for((S >> 2) + 1, kThreads * U_, nr), kThreads, 0, s>>>(
                              rp, g, S, N, r0)));
    }
    return finish();
}

int launch_reset_flat(void *const *ptrs, int r0, int nr, int64_t S, int64_t N, void *stream)
{
    const Tuning &t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ODC_DISPATCH_U_NT(t.accum_unroll, t.nontemporal != 0,
                      (k_reset_flat<U_, NT_><<<grid_for((S >> 2) + 1, kThreads * U_, nr), kThreads, 0, s>>>(rp, S, N, r0)));
    return finish();
}

int launch_gather_batched(const BatchTable &tb, const void *const *ptrs, int r0, int nr, void *full,
                          void *stream)
{
    const Tuning &t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ODC_DISPATCH_U_NT(t.gather_unroll, t.nontemporal != 0,
                      (k_gather_batched<U_, NT_><<<grid_for((tb.arena_elems + 7) >> 3, kThreads * U_, nr), kThreads, 0, s>>>(
                          tb, rp, static_cast<uint16_t *>(full), r0)));
    return finish();
}

int launch_accum_batched(const BatchTable &tb, void *const *ptrs, int r0, int nr, const void *grad,
                         bool atomic, void *stream)
{
    const Tuning &t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t *g = static_cast<const uint16_t *>(grad);
    if (atomic) {
        ODC_DISPATCH_U_NT(t.accum_unroll, false,
                          (k_accum_batched<U_, NT_, true><<<grid_for((tb.arena_elems + 3) >> 2, kThreads * U_, nr), kThreads, 0, s>>>(
                              tb, rp, g, r0)));
    } else {
        ODC_DISPATCH_U_NT(t.accum_unroll, t.nontemporal != 0,
                          (k_accum_batched<U_, NT_, false><<<grid_for((tb.arena_elems + 3) >> 2, kThreads * U_, nr), kThreads, 0, s>>>(
                              tb, rp, g, r0)));
    }
    return finish();
}

int launch_reset_batched(const BatchTable &tb, void *const *ptrs, int r0, int nr, void *stream)
{
    const Tuning &t = tuning();
    const RankPtrs rp = pack(ptrs, nr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ODC_DISPATCH_U_NT(t.accum_unroll, t.nontemporal != 0,
                      (k_reset_batched<U_, NT_><<<grid_for((tb.arena_elems + 3) >> 2, kThreads * U_, nr), kThreads, 0, s>>>(tb, rp, r0)));
    return finish();
}

int launch_probe_copy(void *dst, const void *src, int64_t bytes, void *stream)
{
    const int64_t nvec = bytes >> 4;
    if (nvec == 0) return 0;
    constexpr int U = 4;
    const int64_t blocks = (nvec + kThreads * U - 1) / (kThreads * U);
    k_probe_copy<U><<<dim3(static_cast<unsigned>(blocks)), kThreads, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), nvec);
    return finish();
}

}  // namespace odc

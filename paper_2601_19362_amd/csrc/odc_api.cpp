// C ABI of the ODC hot-path library: argument validation, ordered-mode bookkeeping and
// kernel launches.  All argument errors are reported before anything is enqueued.
#include "../../include/odc.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <functional>
#include <new>
#include <vector>

#include "odc_internal.h"

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e)
{
    g_last_hip_error = static_cast<int>(e);
    return ODC_ERR_HIP;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks shared by the three launch calls.  On success *ptrs_ok is the validated array.
int check_launchable(const odc_layout_t *L, const void *const *ptrs)
{
    if (!L || !ptrs) return ODC_ERR_INVALID_ARG;
    for (int r = 0; r < L->host.R; ++r)
        if (!ptrs[r]) return ODC_ERR_INVALID_ARG;
    for (int r = 0; r < L->host.R; ++r)
        if (!aligned16(ptrs[r])) return ODC_ERR_ALIGNMENT;
    return ODC_OK;
}

int check_device(const odc_layout_t *L)
{
    if (L->host_only) return ODC_ERR_NO_DEVICE;
    // With a single visible device the current device cannot differ from the layout's: the
    // count is read once per process and the per-call query is skipped.
    static const int n_devices = [] {
        int n = 0;
        return hipGetDeviceCount(&n) == hipSuccess ? n : 0;
    }();
    if (n_devices == 1) return ODC_OK;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev != L->device) return ODC_ERR_NO_DEVICE;
    return ODC_OK;
}

// Ordered-mode history of one accumulator set (caller holds L->mu).  A new set gets a fresh
// entry; when the table is full the least recently used entry is dropped first, so the table
// cannot grow without bound if a caller never resets.  Returns nullptr if the host is out of memory.
odc_layout::History *history_of(odc_layout_t *L, const void *key, bool *inserted)
{
    *inserted = false;
    auto it = L->last.find(key);
    if (it == L->last.end()) {
        if (L->last.size() >= odc_layout::kMaxHistory) {
            auto oldest = L->last.begin();
            for (auto j = L->last.begin(); j != L->last.end(); ++j)
                if (j->second.used < oldest->second.used) oldest = j;
            L->last.erase(oldest);
        }
        try {
            it = L->last.emplace(key, odc_layout::History{}).first;
        } catch (...) {
            return nullptr;
        }
        *inserted = true;
    }
    it->second.used = ++L->clock;
    return &it->second;
}

int upload_table(odc_layout_t *L)
{
    hipError_t e = hipGetDevice(&L->device);
    if (e != hipSuccess) return hip_fail(e);
    if (L->host.R <= odc::kStageScratchMaxRanks) {
        // look the fixed scratch of odc_stage_drain_noalloc up now, so that its first call on
        // this device does not have to (the lookup may load the code object)
        int32_t *unused = nullptr;
        const int se = odc::stage_scratch(L->device, &unused);
        if (se != 0) return hip_fail(static_cast<hipError_t>(se));
    }
    if (L->host.T == 1) return ODC_OK;  // flat kernels need no table
    const odc::HostLayout &H = L->host;
    const size_t T = static_cast<size_t>(H.T);
    // one blob: descriptors (8-byte aligned data first), then the two tile indices
    const size_t desc_bytes = T * sizeof(odc::TensorDesc);
    const size_t chunk_bytes = H.chunk_first.size() * sizeof(int32_t);
    const size_t full_chunk_bytes = H.full_chunk_first.size() * sizeof(int32_t);
    const size_t total = desc_bytes + chunk_bytes + full_chunk_bytes;
    char *staging = new (std::nothrow) char[total];
    if (!staging) return ODC_ERR_NOMEM;
    std::memcpy(staging, H.desc.data(), desc_bytes);
    std::memcpy(staging + desc_bytes, H.chunk_first.data(), chunk_bytes);
    std::memcpy(staging + desc_bytes + chunk_bytes, H.full_chunk_first.data(), full_chunk_bytes);
    e = hipMalloc(&L->d_blob, total);
    if (e == hipSuccess) e = hipMemcpy(L->d_blob, staging, total, hipMemcpyHostToDevice);
    delete[] staging;
    if (e != hipSuccess) {
        if (L->d_blob) (void)hipFree(L->d_blob);
        L->d_blob = nullptr;
        return hip_fail(e);
    }
    char *d = static_cast<char *>(L->d_blob);
    L->table.desc = reinterpret_cast<const odc::TensorDesc *>(d);
    L->table.chunk_first = reinterpret_cast<const int32_t *>(d + desc_bytes);
    L->table.full_chunk_first = reinterpret_cast<const int32_t *>(d + desc_bytes + chunk_bytes);
    L->table.gather_tile_tensors = H.gather_tile_tensors;
    L->table.gather_big = H.gather_big;
    L->table.arena_elems = H.arena_elems;
    L->table.full_elems = H.full_elems;
    L->table.T = H.T;
    return ODC_OK;
}

}  // namespace

extern "C" {

int odc_init_layout(int R, int T, const int64_t *numel, int flags, odc_layout_t **out)
{
    if (!out) return ODC_ERR_INVALID_ARG;
    *out = nullptr;
    if (flags & ~ODC_LAYOUT_HOST_ONLY) return ODC_ERR_INVALID_ARG;
    odc_layout_t *L = new (std::nothrow) odc_layout_t;
    if (!L) return ODC_ERR_NOMEM;
    int rc = odc::build_host_layout(R, T, numel, &L->host);
    if (rc == ODC_OK && !(flags & ODC_LAYOUT_HOST_ONLY)) {
        L->host_only = false;
        rc = upload_table(L);
    }
    if (rc != ODC_OK) {
        delete L;
        return rc;
    }
    *out = L;
    return ODC_OK;
}

void odc_free_layout(odc_layout_t *layout)
{
    if (!layout) return;
    if (layout->d_blob) (void)hipFree(layout->d_blob);
    delete layout;
}

int odc_num_ranks(const odc_layout_t *L) { return L ? L->host.R : -1; }
int odc_num_tensors(const odc_layout_t *L) { return L ? L->host.T : -1; }

#define ODC_TENSOR_OR_FAIL(L, t) \
    if (!(L) || (t) < 0 || (t) >= (L)->host.T) return -1

int64_t odc_numel(const odc_layout_t *L, int t)
{
    ODC_TENSOR_OR_FAIL(L, t);
    return L->host.desc[static_cast<size_t>(t)].numel;
}

int64_t odc_shard_elems(const odc_layout_t *L, int t)
{
    ODC_TENSOR_OR_FAIL(L, t);
    return L->host.desc[static_cast<size_t>(t)].S;
}

int64_t odc_valid_elems(const odc_layout_t *L, int t, int r)
{
    ODC_TENSOR_OR_FAIL(L, t);
    if (r < 0 || r >= L->host.R) return -1;
    return odc::valid_elems(L->host.desc[static_cast<size_t>(t)], r);
}

int64_t odc_rank_arena_elems(const odc_layout_t *L) { return L ? L->host.arena_elems : -1; }
int64_t odc_full_elems(const odc_layout_t *L) { return L ? L->host.full_elems : -1; }

int64_t odc_shard_offset(const odc_layout_t *L, int t)
{
    ODC_TENSOR_OR_FAIL(L, t);
    return L->host.desc[static_cast<size_t>(t)].shard_off;
}

int64_t odc_full_offset(const odc_layout_t *L, int t)
{
    ODC_TENSOR_OR_FAIL(L, t);
    return L->host.desc[static_cast<size_t>(t)].full_off;
}

int odc_gather(const odc_layout_t *L, const void *const *param_shards, void *full_out, void *stream)
{
    int rc = check_launchable(L, param_shards);
    if (rc != ODC_OK) return rc;
    if (!full_out) return ODC_ERR_INVALID_ARG;
    if (!aligned16(full_out)) return ODC_ERR_ALIGNMENT;
    rc = check_device(L);
    if (rc != ODC_OK) return rc;
    const odc::HostLayout &H = L->host;
    for (int r0 = 0; r0 < H.R; r0 += odc::kRanksPerLaunch) {
        const int nr = H.R - r0 < odc::kRanksPerLaunch ? H.R - r0 : odc::kRanksPerLaunch;
        int e;
        if (H.T == 1)
            e = odc::launch_gather_flat(param_shards + r0, r0, nr, full_out, H.desc[0].S,
                                        H.desc[0].numel, stream);
        else
            e = odc::launch_gather_batched(L->table, param_shards + r0, r0, nr, full_out, stream);
        if (e != 0) return hip_fail(static_cast<hipError_t>(e));
    }
    return ODC_OK;
}

// Common body of the unweighted and the weighted contribution.
static int scatter_accumulate_impl(const odc_layout_t *L, const void *grad_full, void *const *accum_shards,
                                   int worker, int microbatch, bool weighted, float weight, int flags,
                                   void *stream)
{
    int rc = check_launchable(L, accum_shards);
    if (rc != ODC_OK) return rc;
    if (!grad_full) return ODC_ERR_INVALID_ARG;
    if (flags != ODC_ORDERED && flags != ODC_UNORDERED) return ODC_ERR_INVALID_ARG;
    if (worker < 0 || worker >= L->host.R || microbatch < 0) return ODC_ERR_INVALID_ARG;
    if (!aligned16(grad_full)) return ODC_ERR_ALIGNMENT;

    const bool atomic = flags == ODC_UNORDERED;
    odc_layout_t *M = const_cast<odc_layout_t *>(L);
    // Ordered mode: strictly ascending (worker, microbatch) per accumulator set.  The lock
    // is held until the kernels are enqueued so that history and stream order agree.
    std::unique_lock<std::mutex> lock(M->mu, std::defer_lock);
    const std::pair<int, int> now{worker, microbatch};
    std::pair<int, int> *slot = nullptr;
    bool inserted = false;
    if (!atomic) {
        lock.lock();
        odc_layout::History *h = history_of(M, accum_shards[0], &inserted);
        if (!h) return ODC_ERR_NOMEM;
        slot = &h->last;
        if (!(*slot < now)) return ODC_ERR_ORDER;
    }
    rc = check_device(L);
    const odc::HostLayout &H = L->host;
    for (int r0 = 0; rc == ODC_OK && r0 < H.R; r0 += odc::kRanksPerLaunch) {
        const int nr = H.R - r0 < odc::kRanksPerLaunch ? H.R - r0 : odc::kRanksPerLaunch;
        int e;
        if (H.T == 1)
            e = odc::launch_accum_flat(accum_shards + r0, r0, nr, grad_full, H.desc[0].S,
                                       H.desc[0].numel, atomic, weighted, weight, stream);
        else
            e = odc::launch_accum_batched(L->table, accum_shards + r0, r0, nr, grad_full, atomic, weighted,
                                          weight, stream);
        if (e != 0) rc = hip_fail(static_cast<hipError_t>(e));
        else if (slot) {
            *slot = now;  // something was enqueued: this contribution counts as issued
            inserted = false;
        }
    }
    if (inserted) M->last.erase(accum_shards[0]);  // nothing was enqueued
    return rc;
}

int odc_scatter_accumulate(const odc_layout_t *L, const void *grad_full, void *const *accum_shards,
                           int worker, int microbatch, int flags, void *stream)
{
    return scatter_accumulate_impl(L, grad_full, accum_shards, worker, microbatch, false, 1.0f, flags, stream);
}

int odc_scatter_accumulate_weighted(const odc_layout_t *L, const void *grad_full, void *const *accum_shards,
                                    int worker, int microbatch, float weight, int flags, void *stream)
{
    return scatter_accumulate_impl(L, grad_full, accum_shards, worker, microbatch, true, weight, flags, stream);
}

int odc_scatter_accumulate_multi(const odc_layout_t *L, int count, const void *const *grads,
                                 void *const *accum_shards, const int *workers, const int *microbatches,
                                 int flags, void *stream)
{
    int rc = check_launchable(L, accum_shards);
    if (rc != ODC_OK) return rc;
    if (!grads || !workers || !microbatches || count < 1 || count > ODC_MAX_FUSED) return ODC_ERR_INVALID_ARG;
    if (flags != ODC_ORDERED && flags != ODC_UNORDERED) return ODC_ERR_INVALID_ARG;
    for (int k = 0; k < count; ++k) {
        if (!grads[k] || workers[k] < 0 || workers[k] >= L->host.R || microbatches[k] < 0)
            return ODC_ERR_INVALID_ARG;
    }
    for (int k = 0; k < count; ++k)
        if (!aligned16(grads[k])) return ODC_ERR_ALIGNMENT;
    if (count == 1)
        return scatter_accumulate_impl(L, grads[0], accum_shards, workers[0], microbatches[0], false, 1.0f, flags,
                                       stream);

    const bool atomic = flags == ODC_UNORDERED;
    odc_layout_t *M = const_cast<odc_layout_t *>(L);
    std::unique_lock<std::mutex> lock(M->mu, std::defer_lock);
    std::pair<int, int> *slot = nullptr;
    bool inserted = false;
    const std::pair<int, int> last_now{workers[count - 1], microbatches[count - 1]};
    if (!atomic) {
        // ascending inside the call, and the first one after the history of this accumulator set
        for (int k = 1; k < count; ++k) {
            const std::pair<int, int> a{workers[k - 1], microbatches[k - 1]}, b{workers[k], microbatches[k]};
            if (!(a < b)) return ODC_ERR_ORDER;
        }
        lock.lock();
        odc_layout::History *h = history_of(M, accum_shards[0], &inserted);
        if (!h) return ODC_ERR_NOMEM;
        slot = &h->last;
        if (!(*slot < std::pair<int, int>{workers[0], microbatches[0]})) {
            if (inserted) M->last.erase(accum_shards[0]);
            return ODC_ERR_ORDER;
        }
    }
    rc = check_device(L);
    const odc::HostLayout &H = L->host;
    for (int r0 = 0; rc == ODC_OK && r0 < H.R; r0 += odc::kRanksPerLaunch) {
        const int nr = H.R - r0 < odc::kRanksPerLaunch ? H.R - r0 : odc::kRanksPerLaunch;
        int e;
        if (H.T == 1)
            e = odc::launch_accum_multi_flat(accum_shards + r0, r0, nr, grads, count, H.desc[0].S, H.desc[0].numel,
                                             atomic, stream);
        else
            e = odc::launch_accum_multi_batched(L->table, accum_shards + r0, r0, nr, grads, count, atomic, stream);
        if (e != 0) rc = hip_fail(static_cast<hipError_t>(e));
        else if (slot) {
            *slot = last_now;
            inserted = false;
        }
    }
    if (inserted) M->last.erase(accum_shards[0]);
    return rc;
}

// A client's slot: the rank arena rounded up to whole 128-byte cache lines of bf16, so that
// every slot of a line-aligned staging buffer starts on a line (the copy kernels' wavefronts
// then write whole lines).
static int64_t stage_slot(const odc_layout_t *L)
{
    return (L->host.arena_elems + odc::kStageSlotAlignElems - 1) / odc::kStageSlotAlignElems *
           odc::kStageSlotAlignElems;
}

int64_t odc_stage_slot_elems(const odc_layout_t *L) { return L ? stage_slot(L) : -1; }

int64_t odc_stage_flag_count(const odc_layout_t *L)
{
    return L ? static_cast<int64_t>(L->host.R) * L->host.R + 1 : -1;
}

int64_t odc_stage_snapshot_count(const odc_layout_t *L)
{
    return L ? static_cast<int64_t>(L->host.R) * (L->host.R + 1) : -1;
}

int odc_stage_init(const odc_layout_t *L, void *flags, void *stream)
{
    if (!L || !flags) return ODC_ERR_INVALID_ARG;
    if (!aligned16(flags)) return ODC_ERR_ALIGNMENT;
    const int rc = check_device(L);
    if (rc != ODC_OK) return rc;
    const int e = odc::launch_stage_zero(flags, odc_stage_flag_count(L), stream);
    return e == 0 ? ODC_OK : hip_fail(static_cast<hipError_t>(e));
}

int odc_stage_push(const odc_layout_t *L, const void *grad_full, void *const *staging_shards, void *flags,
                   int worker, void *stream)
{
    int rc = check_launchable(L, staging_shards);
    if (rc != ODC_OK) return rc;
    if (!grad_full || !flags || worker < 0 || worker >= L->host.R) return ODC_ERR_INVALID_ARG;
    if (!aligned16(grad_full) || !aligned16(flags)) return ODC_ERR_ALIGNMENT;
    rc = check_device(L);
    if (rc != ODC_OK) return rc;
    const odc::HostLayout &H = L->host;
    const int64_t slot = stage_slot(L);
    // claim (one decision per owner), copy into the claimed slots, raise them
    int e = odc::launch_stage_claim(flags, H.R, worker, stream);
    if (e != 0) return hip_fail(static_cast<hipError_t>(e));
    for (int r0 = 0; r0 < H.R; r0 += odc::kRanksPerLaunch) {
        const int nr = H.R - r0 < odc::kRanksPerLaunch ? H.R - r0 : odc::kRanksPerLaunch;
        if (H.T == 1)
            e = odc::launch_stage_push_flat(staging_shards + r0, r0, nr, grad_full, flags, H.desc[0].S,
                                            H.desc[0].numel, slot, H.R, worker, stream);
        else
            e = odc::launch_stage_push_batched(L->table, staging_shards + r0, r0, nr, grad_full, flags, slot, H.R,
                                               worker, stream);
        if (e != 0) return hip_fail(static_cast<hipError_t>(e));
    }
    e = odc::launch_stage_raise(flags, H.R, worker, stream);
    return e == 0 ? ODC_OK : hip_fail(static_cast<hipError_t>(e));
}

// Shared by the two drain entry points; `snapshot` is the caller's workspace or the fixed scratch.
static int stage_drain_impl(const odc_layout_t *L, const void *const *staging_shards, void *flags, void *snapshot,
                            void *const *accum_shards, void *stream)
{
    const odc::HostLayout &H = L->host;
    const int64_t slot = stage_slot(L);
    int e = odc::launch_stage_snapshot(flags, snapshot, H.R, stream);
    if (e != 0) return hip_fail(static_cast<hipError_t>(e));
    for (int r0 = 0; r0 < H.R; r0 += odc::kRanksPerLaunch) {
        const int nr = H.R - r0 < odc::kRanksPerLaunch ? H.R - r0 : odc::kRanksPerLaunch;
        if (H.T == 1)
            e = odc::launch_stage_drain_flat(accum_shards + r0, staging_shards + r0, r0, nr, snapshot, H.desc[0].S,
                                             H.desc[0].numel, slot, H.R, stream);
        else
            e = odc::launch_stage_drain_batched(L->table, accum_shards + r0, staging_shards + r0, r0, nr, snapshot,
                                                slot, H.R, stream);
        if (e != 0) return hip_fail(static_cast<hipError_t>(e));
    }
    e = odc::launch_stage_clear(flags, snapshot, H.R, stream);
    return e == 0 ? ODC_OK : hip_fail(static_cast<hipError_t>(e));
}

static int check_drain_args(const odc_layout_t *L, const void *const *staging_shards, void *flags,
                            void *const *accum_shards)
{
    int rc = check_launchable(L, staging_shards);
    if (rc != ODC_OK) return rc;
    rc = check_launchable(L, accum_shards);
    if (rc != ODC_OK) return rc;
    if (!flags) return ODC_ERR_INVALID_ARG;
    if (!aligned16(flags)) return ODC_ERR_ALIGNMENT;
    return ODC_OK;
}

int odc_stage_drain(const odc_layout_t *L, const void *const *staging_shards, void *flags, void *snapshot,
                    void *const *accum_shards, void *stream)
{
    int rc = check_drain_args(L, staging_shards, flags, accum_shards);
    if (rc != ODC_OK) return rc;
    if (!snapshot) return ODC_ERR_INVALID_ARG;
    if (!aligned16(snapshot)) return ODC_ERR_ALIGNMENT;
    rc = check_device(L);
    if (rc != ODC_OK) return rc;
    return stage_drain_impl(L, staging_shards, flags, snapshot, accum_shards, stream);
}

int odc_stage_drain_noalloc(const odc_layout_t *L, const void *const *staging_shards, void *flags,
                            void *const *accum_shards, void *stream)
{
    int rc = check_drain_args(L, staging_shards, flags, accum_shards);
    if (rc != ODC_OK) return rc;
    if (L->host.R > ODC_NOALLOC_MAX_RANKS) return ODC_ERR_TOO_LARGE;
    rc = check_device(L);  // the layout's device is the current one
    if (rc != ODC_OK) return rc;
    int32_t *scratch = nullptr;
    const int e = odc::stage_scratch(L->device, &scratch);
    if (e != 0) return hip_fail(static_cast<hipError_t>(e));
    return stage_drain_impl(L, staging_shards, flags, scratch, accum_shards, stream);
}

int odc_retrieve_grads(const odc_layout_t *L, const void *const *accum_shards, void *const *out_shards,
                       float scale, int out_dtype, void *stream)
{
    int rc = check_launchable(L, accum_shards);
    if (rc != ODC_OK) return rc;
    rc = check_launchable(L, out_shards);
    if (rc != ODC_OK) return rc;
    if (out_dtype != ODC_OUT_F32 && out_dtype != ODC_OUT_BF16) return ODC_ERR_INVALID_ARG;
    rc = check_device(L);
    if (rc != ODC_OK) return rc;
    const odc::HostLayout &H = L->host;
    const bool bf16 = out_dtype == ODC_OUT_BF16;
    for (int r0 = 0; r0 < H.R; r0 += odc::kRanksPerLaunch) {
        const int nr = H.R - r0 < odc::kRanksPerLaunch ? H.R - r0 : odc::kRanksPerLaunch;
        int e;
        if (H.T == 1)
            e = odc::launch_retrieve_flat(accum_shards + r0, out_shards + r0, r0, nr, H.desc[0].S,
                                          H.desc[0].numel, scale, bf16, stream);
        else
            e = odc::launch_retrieve_batched(L->table, accum_shards + r0, out_shards + r0, r0, nr, scale,
                                             bf16, stream);
        if (e != 0) return hip_fail(static_cast<hipError_t>(e));
    }
    return ODC_OK;
}

// ---------------------------------------------------------------------- wide accumulators
static int wide_call(const odc_layout_t *L, int op, void *const *accum64_shards, void *const *out_shards,
                     const void *grad_full, float scale, void *stream)
{
    int rc = check_launchable(L, accum64_shards);
    if (rc != ODC_OK) return rc;
    if (out_shards) {
        rc = check_launchable(L, out_shards);
        if (rc != ODC_OK) return rc;
    }
    rc = check_device(L);
    if (rc != ODC_OK) return rc;
    const odc::HostLayout &H = L->host;
    const odc::BatchTable *tb = H.T == 1 ? nullptr : &L->table;
    for (int r0 = 0; r0 < H.R; r0 += odc::kRanksPerLaunch) {
        const int nr = H.R - r0 < odc::kRanksPerLaunch ? H.R - r0 : odc::kRanksPerLaunch;
        const int e = odc::launch_wide(tb, op, accum64_shards + r0, out_shards ? out_shards + r0 : nullptr, grad_full, r0,
                                       nr, H.desc[0].S, H.desc[0].numel, scale, stream);
        if (e != 0) return hip_fail(static_cast<hipError_t>(e));
    }
    return ODC_OK;
}

int odc_scatter_accumulate_wide(const odc_layout_t *L, const void *grad_full, void *const *accum64_shards, void *stream)
{
    if (!grad_full) return ODC_ERR_INVALID_ARG;
    if (!aligned16(grad_full)) return ODC_ERR_ALIGNMENT;
    return wide_call(L, 0, accum64_shards, nullptr, grad_full, 1.0f, stream);
}

int odc_reset_accum_wide(const odc_layout_t *L, void *const *accum64_shards, void *stream)
{
    return wide_call(L, 1, accum64_shards, nullptr, nullptr, 1.0f, stream);
}

int odc_retrieve_grads_wide(const odc_layout_t *L, const void *const *accum64_shards, void *const *out_shards, float scale,
                            int out_dtype, void *stream)
{
    if (out_dtype != ODC_OUT_F32 && out_dtype != ODC_OUT_BF16) return ODC_ERR_INVALID_ARG;
    if (!out_shards) return ODC_ERR_INVALID_ARG;
    return wide_call(L, out_dtype == ODC_OUT_BF16 ? 3 : 2, const_cast<void *const *>(accum64_shards), out_shards, nullptr,
                     scale, stream);
}

// ------------------------------------------------------------------------ hybrid sharding
int odc_hybrid_group_of(const odc_layout_t *L, int groups, int world_worker)
{
    if (!L || groups < 1 || groups > ODC_MAX_GROUPS || world_worker < 0) return -1;
    const int64_t world = static_cast<int64_t>(groups) * L->host.R;
    if (world_worker >= world) return -1;
    return world_worker / L->host.R;
}

int odc_gather_hybrid(const odc_layout_t *L, int groups, const void *const *group_param_shards, int world_worker,
                      void *full_out, void *stream)
{
    if (!L || !group_param_shards) return ODC_ERR_INVALID_ARG;
    const int g = odc_hybrid_group_of(L, groups, world_worker);
    if (g < 0) return ODC_ERR_INVALID_ARG;
    return odc_gather(L, group_param_shards + static_cast<size_t>(g) * L->host.R, full_out, stream);
}

int odc_scatter_accumulate_hybrid(const odc_layout_t *L, int groups, const void *grad_full,
                                  void *const *group_accum_shards, int world_worker, int microbatch, int flags,
                                  void *stream)
{
    if (!L || !group_accum_shards) return ODC_ERR_INVALID_ARG;
    const int g = odc_hybrid_group_of(L, groups, world_worker);
    if (g < 0) return ODC_ERR_INVALID_ARG;
    return odc_scatter_accumulate(L, grad_full, group_accum_shards + static_cast<size_t>(g) * L->host.R,
                                  world_worker % L->host.R, microbatch, flags, stream);
}

int odc_reduce_groups(const odc_layout_t *L, int groups, const void *const *group_accum_shards,
                      void *const *out_shards, void *stream)
{
    if (!L || !group_accum_shards || groups < 1 || groups > ODC_MAX_GROUPS) return ODC_ERR_INVALID_ARG;
    int rc = check_launchable(L, out_shards);
    if (rc != ODC_OK) return rc;
    const odc::HostLayout &H = L->host;
    const int R = H.R;
    for (int k = 0; k < groups; ++k) {
        rc = check_launchable(L, group_accum_shards + static_cast<size_t>(k) * R);
        if (rc != ODC_OK) return rc;
    }
    // the sum may replace group 0's shards; a later group's shard would be overwritten by the
    // first pass before a later pass reads it
    if (groups > 1) {
        try {
            std::vector<const void *> outs(out_shards, out_shards + R);
            std::sort(outs.begin(), outs.end(), std::less<const void *>());
            for (size_t i = static_cast<size_t>(R); i < static_cast<size_t>(groups) * R; ++i)
                if (std::binary_search(outs.begin(), outs.end(), group_accum_shards[i], std::less<const void *>()))
                    return ODC_ERR_INVALID_ARG;
        } catch (...) {
            return ODC_ERR_NOMEM;
        }
    }
    rc = check_device(L);
    if (rc != ODC_OK) return rc;
    const odc::BatchTable *tb = H.T == 1 ? nullptr : &L->table;
    for (int r0 = 0; r0 < R; r0 += odc::kReduceRanksPerLaunch) {
        const int nr = R - r0 < odc::kReduceRanksPerLaunch ? R - r0 : odc::kReduceRanksPerLaunch;
        for (int k0 = 0; k0 < groups; k0 += odc::kReduceSourcesPerPass) {
            const int count = groups - k0 < odc::kReduceSourcesPerPass ? groups - k0 : odc::kReduceSourcesPerPass;
            const int e = odc::launch_reduce_groups(tb, group_accum_shards + static_cast<size_t>(k0) * R + r0, R, count,
                                                    k0 == 0, out_shards + r0, r0, nr, H.desc[0].S, H.desc[0].numel,
                                                    stream);
            if (e != 0) return hip_fail(static_cast<hipError_t>(e));
        }
    }
    return ODC_OK;
}

int odc_reset_accum(const odc_layout_t *L, void *const *accum_shards, void *stream)
{
    int rc = check_launchable(L, accum_shards);
    if (rc != ODC_OK) return rc;
    rc = check_device(L);
    if (rc != ODC_OK) return rc;
    const odc::HostLayout &H = L->host;
    odc_layout_t *M = const_cast<odc_layout_t *>(L);
    // the lock covers the launch and the erase, so that history and stream order agree when
    // several host threads work on one accumulator set
    std::lock_guard<std::mutex> lock(M->mu);
    for (int r0 = 0; r0 < H.R; r0 += odc::kRanksPerLaunch) {
        const int nr = H.R - r0 < odc::kRanksPerLaunch ? H.R - r0 : odc::kRanksPerLaunch;
        int e;
        if (H.T == 1)
            e = odc::launch_reset_flat(accum_shards + r0, r0, nr, H.desc[0].S, H.desc[0].numel, stream);
        else
            e = odc::launch_reset_batched(L->table, accum_shards + r0, r0, nr, stream);
        if (e != 0) return hip_fail(static_cast<hipError_t>(e));
    }
    M->last.erase(accum_shards[0]);
    return ODC_OK;
}

int odc_forget_accum(const odc_layout_t *L, void *const *accum_shards)
{
    if (!L || !accum_shards || !accum_shards[0]) return ODC_ERR_INVALID_ARG;
    odc_layout_t *M = const_cast<odc_layout_t *>(L);
    std::lock_guard<std::mutex> lock(M->mu);
    M->last.erase(accum_shards[0]);
    return ODC_OK;
}

const char *odc_strerror(int code)
{
    switch (code) {
        case ODC_OK: return "success";
        case ODC_ERR_INVALID_ARG: return "invalid argument";
        case ODC_ERR_ALIGNMENT: return "device base pointer is not 16-byte aligned";
        case ODC_ERR_ORDER: return "ordered contribution is not after the previous (worker, microbatch)";
        case ODC_ERR_OVERFLOW: return "size arithmetic overflows 64 bits";
        case ODC_ERR_HIP: return "HIP call failed (see odc_last_hip_error)";
        case ODC_ERR_NO_DEVICE: return "layout is host-only or belongs to another device";
        case ODC_ERR_NOMEM: return "host allocation failed";
        case ODC_ERR_TOO_LARGE: return "size exceeds the fixed scratch of a no-allocation entry point";
        default: return "unknown ODC error code";
    }
}

int odc_last_hip_error(void) { return g_last_hip_error; }

int odc_probe_copy(void *dst, const void *src, int64_t bytes, void *stream)
{
    if (!dst || !src || bytes < 0 || (bytes & 15)) return ODC_ERR_INVALID_ARG;
    if (!aligned16(dst) || !aligned16(src)) return ODC_ERR_ALIGNMENT;
    const int e = odc::launch_probe_copy(dst, src, bytes, stream);
    return e == 0 ? ODC_OK : hip_fail(static_cast<hipError_t>(e));
}

int odc_tune(const char *knob, int value)
{
    if (!knob) return ODC_ERR_INVALID_ARG;
    // read-modify-write of the whole set under the API's own lock, so two tuning calls cannot
    // lose each other's change
    static std::mutex tune_mu;
    std::lock_guard<std::mutex> tune_lock(tune_mu);
    odc::Tuning t = odc::tuning();
    const bool unroll_ok = value == 1 || value == 2 || value == 4;
    const bool threads_ok = value == 64 || value == 128 || value == 256;
    const bool flag_ok = value == 0 || value == 1;
    if (!std::strcmp(knob, "defaults") && value == 0) t = odc::Tuning{};
    else if (!std::strcmp(knob, "gather_unroll") && unroll_ok) t.gather_unroll = value;
    else if (!std::strcmp(knob, "accum_unroll") && unroll_ok) t.accum_unroll = value;
    else if (!std::strcmp(knob, "reset_unroll") && unroll_ok) t.reset_unroll = value;
    else if (!std::strcmp(knob, "gather_threads") && threads_ok) t.gather_threads = value;
    else if (!std::strcmp(knob, "accum_threads") && threads_ok) t.accum_threads = value;
    else if (!std::strcmp(knob, "reset_threads") && threads_ok) t.reset_threads = value;
    else if (!std::strcmp(knob, "nontemporal") && flag_ok) t.nontemporal = value;
    else if (!std::strcmp(knob, "tile_remap") && flag_ok) t.tile_remap = value;
    else if (!std::strcmp(knob, "gather_store_sc1") && flag_ok) t.gather_store_sc1 = value;
    else if (!std::strcmp(knob, "max_grid_x") && value >= 0) t.max_grid_x = value;
    else if (!std::strcmp(knob, "gather_tile_xcd_block") && value >= 1 && value <= 4096 && (value & (value - 1)) == 0)
        t.gather_tile_xcd_block = value;
    else if (!std::strcmp(knob, "batch_rank_group") &&
             (value == 0 || value == 1 || value == 2 || value == 4 || value == 8))
        t.batch_rank_group = value;
    else return ODC_ERR_INVALID_ARG;
    odc::set_tuning(t);
    return ODC_OK;
}

}  // extern "C"

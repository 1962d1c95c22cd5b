// Internal interfaces between the host layout code, the C-ABI layer and the gfx950 kernels.
#pragma once

#include <cstdint>
#include <mutex>
#include <unordered_map>
#include <utility>
#include <vector>

namespace odc {

// Ranks served by one kernel launch: their base pointers travel by value in the kernel
// arguments (64 * 8 bytes), so no per-call device table or host-to-device copy is needed.
constexpr int kRanksPerLaunch = 64;
// Every tensor starts at a multiple of this many elements inside a rank arena and inside
// the full buffer: 16 bytes of bf16, 32 bytes of binary32.
constexpr int64_t kAlignElems = 8;
// A staging slot is a whole number of 128-byte lines of bf16.
constexpr int64_t kStageSlotAlignElems = 64;
// Rank-arena elements per entry of the coarse tensor-lookup index (power of two).
constexpr int kChunkShift = 11;

// The batched gather kernel works on tiles of this many chunks of the full buffer.
constexpr int kGatherChunks = 4;
// Tensors below 2^kGatherSmallShift elements use 32-bit tile-relative index arithmetic in
// the batched gather kernel, larger ones a 64-bit path.  (A build of the CPU emulation lowers
// the limit so that small test cases reach the 64-bit path.)
#ifndef ODC_GATHER_SMALL_SHIFT
#define ODC_GATHER_SMALL_SHIFT 30
#endif
constexpr int kGatherSmallShift = ODC_GATHER_SMALL_SHIFT;

// Per-tensor record read by the batched kernels.
struct TensorDesc {
    int64_t shard_off;  // start inside every rank arena (elements)
    int64_t full_off;   // start inside the full buffer (elements)
    int64_t numel;      // N_t
    int64_t S;          // ceil(N_t / R)
};

// Device-side lookup data of a multi-tensor layout (all pointers are device pointers).
struct BatchTable {
    const TensorDesc *desc;           // [T]
    const int32_t *chunk_first;       // rank-arena space, [arena tiles + 1]: last tensor whose
                                      // shard_off is at or before the tile's first element
    const int32_t *full_chunk_first;  // the same for the full buffer (full_off)
    int64_t arena_elems;
    int64_t full_elems;
    int32_t T;
    int32_t gather_tile_tensors;      // most tensors that intersect one gather tile
    int32_t gather_big;               // 1: some tensor's shard pieces are at least one gather tile long
};

struct HostLayout {
    int R = 0;
    int T = 0;
    std::vector<TensorDesc> desc;
    int64_t arena_elems = 0;
    int64_t full_elems = 0;
    int64_t total_numel = 0;
    std::vector<int32_t> chunk_first;       // built for T > 1
    std::vector<int32_t> full_chunk_first;  // built for T > 1
    int gather_tile_tensors = 1;            // built for T > 1
    int gather_big = 0;                     // built for T > 1
};

// Pure integer layout construction (Section 3.1 even partition, tail padding).
// Returns an ODC_* code; never touches the GPU.
int build_host_layout(int R, int T, const int64_t *numel, HostLayout *out);

inline int64_t valid_elems(const TensorDesc &d, int r)
{
    int64_t v = d.numel - static_cast<int64_t>(r) * d.S;
    if (v < 0) v = 0;
    if (v > d.S) v = d.S;
    return v;
}

// Workgroups along x for `items` work items at `per_block` items per workgroup pass.  The
// kernels loop over tiles, so a capped grid is still complete.
inline unsigned grid_x_for(int64_t items, int per_block, int cap)
{
    int64_t tiles = (items + per_block - 1) / per_block;
    if (tiles < 1) tiles = 1;
    if (cap > 0 && tiles > cap) tiles = cap;
    if (tiles > 0x7FFFFFFF) tiles = 0x7FFFFFFF;
    return static_cast<unsigned>(tiles);
}

// Launch knobs (process-wide, diagnostics only; results never depend on them).  The defaults
// are the best point of a sweep over threads x unroll x tile order on the 1.5B-, 7B- and
// 32B-shaped layers: one wavefront per workgroup and one 16-byte item per lane for the two
// read-write streams (the chip then sweeps one compact, steadily advancing address window,
// which HBM serves best), four wavefronts per workgroup for the write-only reset, which is
// otherwise limited by the workgroup launch rate.
struct Tuning {
    int gather_threads = 64;   // workgroup size of the flat kernels: 64, 128 or 256
    int accum_threads = 64;
    int reset_threads = 256;
    int gather_unroll = 1;     // work items per thread and tile: 1, 2 or 4
    int accum_unroll = 1;
    int reset_unroll = 1;
    int nontemporal = 1;       // 1: streaming loads/stores carry the non-temporal hint
    int max_grid_x = 0;        // 0: one workgroup per tile; > 0: cap and loop (persistent style)
    int tile_remap = 0;        // 1: each XCD sweeps its own contiguous eighth of the tiles
    int gather_store_sc1 = 1;  // 1: gather stores use sc1 + nt (about 3 % faster than nt on this GPU)
    int batch_rank_group = 0;  // owners per workgroup in batched accumulate/reset: 0 = auto, 1, 2, 4, 8
    int gather_tile_xcd_block = 16;  // batched gather: tiles handed to the 8 XCDs in blocks of up to this many (power of two)
};
// The knobs are process-wide.  Every launcher takes ONE copy at its start (under a lock) and
// computes grid, kernel variant and kernel arguments from that copy, so a thread that changes a
// knob while another launches can never make a launch see half of a change.
Tuning tuning();
void set_tuning(const Tuning &t);

// Kernel launchers (odc_kernels.hip).  All return a hipError_t as int.  `ptrs` holds the
// device base pointers of ranks [r0, r0 + nr), nr <= kRanksPerLaunch.
int launch_gather_flat(const void *const *ptrs, int r0, int nr, void *full, int64_t S, int64_t N,
                       void *stream);
int launch_accum_flat(void *const *ptrs, int r0, int nr, const void *grad, int64_t S, int64_t N,
                      bool atomic, bool weighted, float w, void *stream);
int launch_reset_flat(void *const *ptrs, int r0, int nr, int64_t S, int64_t N, void *stream);
int launch_gather_batched(const BatchTable &tb, const void *const *ptrs, int r0, int nr,
                          void *full, void *stream);
// The batched kernels stage in LDS the tensors that intersect a tile of up to kMaxTileChunks
// chunks of 2^kChunkShift elements.  With every tensor starting at a multiple of kAlignElems
// at most one tensor starts per aligned position, so a chunk adds at most
// 2^kChunkShift / kAlignElems tensors; the host layout checks this bound.
constexpr int kMaxTensorsPerChunk = (1 << kChunkShift) / static_cast<int>(kAlignElems);
int launch_accum_batched(const BatchTable &tb, void *const *ptrs, int r0, int nr,
                         const void *grad, bool atomic, bool weighted, float w, void *stream);
// Fused form: `count` (2..8) gradients applied in order in one pass.
int launch_accum_multi_flat(void *const *ptrs, int r0, int nr, const void *const *grads, int count, int64_t S,
                            int64_t N, bool atomic, void *stream);
int launch_accum_multi_batched(const BatchTable &tb, void *const *ptrs, int r0, int nr, const void *const *grads,
                               int count, bool atomic, void *stream);
// Staging (per-client receive buffers + flags); see odc_stage_* in odc.h.
int launch_stage_zero(void *flags, int64_t count, void *stream);
int launch_stage_push_flat(void *const *staging, int r0, int nr, const void *grad, const void *flags, int64_t S,
                           int64_t N, int64_t slot, int R, int worker, void *stream);
int launch_stage_push_batched(const BatchTable &tb, void *const *staging, int r0, int nr, const void *grad,
                              const void *flags, int64_t slot, int R, int worker, void *stream);
int launch_stage_claim(void *flags, int R, int worker, void *stream);
int launch_stage_raise(void *flags, int R, int worker, void *stream);
int launch_stage_snapshot(const void *flags, void *snapshot, int R, void *stream);
int launch_stage_clear(void *flags, const void *snapshot, int R, void *stream);
int launch_stage_drain_flat(void *const *accs, const void *const *staging, int r0, int nr, const void *snapshot,
                            int64_t S, int64_t N, int64_t slot, int R, void *stream);
int launch_stage_drain_batched(const BatchTable &tb, void *const *accs, const void *const *staging, int r0, int nr,
                               const void *snapshot, int64_t slot, int R, void *stream);
// Device address, on the current device `device`, of the library's fixed snapshot scratch
// (room for kStageScratchMaxRanks owners); looked up on first use per device, no allocation.
constexpr int kStageScratchMaxRanks = 256;
int stage_scratch(int device, int32_t **out);
int launch_retrieve_flat(const void *const *acc, void *const *out, int r0, int nr, int64_t S, int64_t N,
                         float scale, bool bf16, void *stream);
int launch_retrieve_batched(const BatchTable &tb, const void *const *acc, void *const *out, int r0, int nr,
                            float scale, bool bf16, void *stream);
int launch_reset_batched(const BatchTable &tb, void *const *ptrs, int r0, int nr, void *stream);
// Wide (binary64) accumulators of the unordered mode: op 0 accumulate (atomic), 1 reset,
// 2 retrieve to binary32, 3 retrieve to bf16; tb = nullptr: single tensor with S, N.
int launch_wide(const BatchTable *tb, int op, void *const *accs, void *const *outs, const void *grad, int r0, int nr,
                int64_t S, int64_t N, float scale, void *stream);
// Hybrid sharding: one pass of the sum over groups (tb = nullptr: single tensor with S, N).
constexpr int kReduceSourcesPerPass = 8;
constexpr int kReduceRanksPerLaunch = 16;
int launch_reduce_groups(const BatchTable *tb, const void *const *srcs, int64_t stride, int count, bool init,
                         void *const *outs, int r0, int nr, int64_t S, int64_t N, void *stream);
int launch_probe_copy(void *dst, const void *src, int64_t bytes, void *stream);

}  // namespace odc

// The opaque handle of the C ABI.
struct odc_layout {
    odc::HostLayout host;
    bool host_only = true;
    int device = -1;
    void *d_blob = nullptr;  // one hipMalloc holding shard_off, desc and chunk_first
    odc::BatchTable table{};
    std::mutex mu;
    // ordered-mode history: accum_shards[0] -> last (worker, microbatch) issued, with the time of
    // its last use; bounded (the least recently used entry goes when kMaxHistory is reached)
    struct History {
        std::pair<int, int> last{-1, -1};
        uint64_t used = 0;
    };
    static constexpr size_t kMaxHistory = 1024;
    std::unordered_map<const void *, History> last;
    uint64_t clock = 0;
};

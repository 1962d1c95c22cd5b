// Host-side shard layout: pure 64-bit integer arithmetic, no GPU calls.
//
// Section 3.1 of the paper partitions parameters and gradients evenly over all devices and
// Section 3 keeps FSDP's flat memory layout.  The paper does not say what happens when the
// rank count does not divide a tensor; here S = ceil(N / R) slots per owner with the padding
// at the tail of the flat index space, so several trailing owners can be partly or wholly
// padding (N = 1, R = 64: owner 0 holds one element, the others none).
#include "odc_internal.h"

#include "../../include/odc.h"

#include <limits>
#include <mutex>

namespace odc {

namespace {

constexpr int64_t kMaxElems = std::numeric_limits<int64_t>::max() / 16;  // bytes still fit

bool round_up(int64_t x, int64_t a, int64_t *out)
{
    if (x > kMaxElems) return false;
    *out = (x + a - 1) / a * a;
    return true;
}

}  // namespace

int build_host_layout(int R, int T, const int64_t *numel, HostLayout *out)
{
    if (!out || !numel || R < 1 || R > ODC_MAX_RANKS || T < 1) return ODC_ERR_INVALID_ARG;
    HostLayout L;
    L.R = R;
    L.T = T;
    try {
        L.desc.resize(static_cast<size_t>(T));
    } catch (...) {
        return ODC_ERR_NOMEM;
    }
    int64_t shard_cursor = 0, full_cursor = 0, total = 0;
    for (int t = 0; t < T; ++t) {
        const int64_t N = numel[t];
        if (N < 1) return ODC_ERR_INVALID_ARG;
        if (N > kMaxElems) return ODC_ERR_OVERFLOW;
        const int64_t S = (N - 1) / R + 1;  // ceil without overflow
        TensorDesc &d = L.desc[static_cast<size_t>(t)];
        d.numel = N;
        d.S = S;
        d.shard_off = shard_cursor;
        d.full_off = full_cursor;
        L.arena_elems = shard_cursor + S;
        L.full_elems = full_cursor + N;
        if (L.arena_elems > kMaxElems || L.full_elems > kMaxElems) return ODC_ERR_OVERFLOW;
        total += N;
        int64_t s_pad, n_pad;
        if (!round_up(S, kAlignElems, &s_pad) || !round_up(N, kAlignElems, &n_pad))
            return ODC_ERR_OVERFLOW;
        shard_cursor += s_pad;
        full_cursor += n_pad;
        if (shard_cursor > kMaxElems || full_cursor > kMaxElems) return ODC_ERR_OVERFLOW;
    }
    L.total_numel = total;

    if (T > 1) {
        // Coarse indices for the batched kernels: for every tile of 2^kChunkShift elements of
        // the rank-arena space (and of the full-buffer space), the last tensor that starts at
        // or before the tile's first element.
        const int64_t chunk = int64_t{1} << kChunkShift;
        for (int space = 0; space < 2; ++space) {
            const int64_t extent = space == 0 ? L.arena_elems : L.full_elems;
            std::vector<int32_t> &index = space == 0 ? L.chunk_first : L.full_chunk_first;
            const int64_t n_chunks = (extent + chunk - 1) / chunk;
            try {
                index.resize(static_cast<size_t>(n_chunks) + 1);
            } catch (...) {
                return ODC_ERR_NOMEM;
            }
            int t = 0;
            for (int64_t c = 0; c <= n_chunks; ++c) {
                const int64_t start = c * chunk;
                while (t + 1 < T) {
                    const TensorDesc &next = L.desc[static_cast<size_t>(t) + 1];
                    if ((space == 0 ? next.shard_off : next.full_off) > start) break;
                    ++t;
                }
                index[static_cast<size_t>(c)] = t;
                // the kernels size their LDS staging area from this bound
                if (c > 0 && t - index[static_cast<size_t>(c) - 1] > kMaxTensorsPerChunk)
                    return ODC_ERR_OVERFLOW;
            }
        }
    }
    if (T > 1) {
        // What the batched gather kernel needs beyond the indices: whether any shard piece is
        // a tile long, and the most tensors any of its tiles holds (sizes its LDS staging).
        for (int t = 0; t < T; ++t)
            if (L.desc[static_cast<size_t>(t)].S >= (int64_t{kGatherChunks} << kChunkShift)) L.gather_big = 1;
        const int64_t n_chunks = static_cast<int64_t>(L.full_chunk_first.size()) - 1;
        int most = 1;
        for (int64_t c0 = 0; c0 < n_chunks; c0 += kGatherChunks) {
            const int64_t c1 = c0 + kGatherChunks < n_chunks ? c0 + kGatherChunks : n_chunks;
            const int n = L.full_chunk_first[static_cast<size_t>(c1)] - L.full_chunk_first[static_cast<size_t>(c0)] + 1;
            if (n > most) most = n;
        }
        L.gather_tile_tensors = most;
    }
    *out = std::move(L);
    return ODC_OK;
}

namespace {
std::mutex g_tuning_mu;
Tuning g_tuning;
}  // namespace

Tuning tuning()
{
    std::lock_guard<std::mutex> lock(g_tuning_mu);
    return g_tuning;
}

void set_tuning(const Tuning &t)
{
    std::lock_guard<std::mutex> lock(g_tuning_mu);
    g_tuning = t;
}

}  // namespace odc

// CPU emulation driver for the ODC kernels (test infrastructure only).
//
// Reads one case from a directory, runs the REAL kernel source (odc_device.h) on the host
// one thread at a time under AddressSanitizer/UBSan, and writes the outputs back.  Every
// rank buffer is its own exactly-sized heap block, so any access outside the valid range of
// a buffer is reported.  The test compares the outputs with the CPU oracle.
//
// usage: emu <dir> <op> <R> [threads= unroll= nt= remap= atomic= cap= rg= weighted= weight= bf16= scale=]
//   dir holds numel.i64 [T]; arenas.u16 [R*arena] (gather); full.u16 [full] (gather in/out);
//   grad.u16 [full] and acc.f32 [R*arena] (accum / reset, in/out; retrieve: in, with out.bin [R*arena] in/out)
#include "hip_shim.h"

#include <cstdio>
#include <cstdlib>
#include <string>
#include <thread>
#include <type_traits>
#include <vector>

#include "../../include/odc.h"
#include "../../paper_2601_19362_amd/csrc/odc_device.h"

namespace {

template <typename T>
std::vector<T> read_file(const std::string &path)
{
    FILE *f = std::fopen(path.c_str(), "rb");
    if (!f) {
        std::fprintf(stderr, "cannot open %s\n", path.c_str());
        std::exit(2);
    }
    std::fseek(f, 0, SEEK_END);
    long n = std::ftell(f);
    std::fseek(f, 0, SEEK_SET);
    std::vector<T> v(static_cast<size_t>(n) / sizeof(T));
    if (n && std::fread(v.data(), 1, static_cast<size_t>(n), f) != static_cast<size_t>(n)) std::exit(2);
    std::fclose(f);
    return v;
}

template <typename T>
void write_file(const std::string &path, const T *p, size_t n)
{
    FILE *f = std::fopen(path.c_str(), "wb");
    if (!f || (n && std::fwrite(p, sizeof(T), n, f) != n)) std::exit(2);
    std::fclose(f);
}

// A scripted run can execute only part of a grid: the workgroups whose linear index is
// congruent to part_k modulo part_n (part_n = 1: all).  Used to interleave the workgroups of
// one kernel with kernels of another stream.
unsigned part_k = 0, part_n = 1;

bool in_part(unsigned x, unsigned y, unsigned gx) { return part_n <= 1 || (y * gx + x) % part_n == part_k; }

template <typename F>
void run_grid(unsigned tpb, unsigned gx, unsigned gy, F &&kernel)
{
    gridDim.x = gx;
    gridDim.y = gy;
    blockDim.x = tpb;
    for (unsigned y = 0; y < gy; ++y)
        for (unsigned x = 0; x < gx; ++x)
            for (unsigned t = 0; t < tpb && in_part(x, y, gx); ++t) {
                blockIdx.x = x;
                blockIdx.y = y;
                threadIdx.x = t;
                kernel();
            }
}

// Workgroups one after the other, each on `tpb` host threads that meet at the barrier
// behind __syncthreads().  `kernel` is called once per (thread, workgroup).
template <typename F>
void run_grid_threaded(unsigned tpb, unsigned gx, unsigned gy, F &&kernel)
{
    gridDim.x = gx;
    gridDim.y = gy;
    blockDim.x = tpb;
    pthread_barrier_t barrier;
    pthread_barrier_init(&barrier, nullptr, tpb);
    emu_block_barrier = &barrier;
    std::vector<std::thread> pool;
    for (unsigned t = 0; t < tpb; ++t)
        pool.emplace_back([&, t] {
            for (unsigned y = 0; y < gy; ++y)
                for (unsigned x = 0; x < gx; ++x) {
                    if (!in_part(x, y, gx)) continue;
                    blockIdx.x = x;
                    blockIdx.y = y;
                    threadIdx.x = t;
                    kernel();
                    pthread_barrier_wait(&barrier);  // the shared LDS image is reused by the next workgroup
                }
        });
    for (auto &th : pool) th.join();
    emu_block_barrier = nullptr;
    pthread_barrier_destroy(&barrier);
}

#define EMU_NT(NTF, CALL)                             \
    do {                                              \
        if (NTF) { constexpr bool NT_ = true; CALL; } \
        else { constexpr bool NT_ = false; CALL; }    \
    } while (0)

#define EMU_U(UN, NTF, CALL)                                            \
    do {                                                                \
        switch (UN) {                                                   \
            case 1: { constexpr int U_ = 1; EMU_NT(NTF, CALL); } break;  \
            case 2: { constexpr int U_ = 2; EMU_NT(NTF, CALL); } break;  \
            default: { constexpr int U_ = 4; EMU_NT(NTF, CALL); } break; \
        }                                                               \
    } while (0)

#define EMU_DISPATCH(TPBV, UN, NTF, CALL)                                         \
    do {                                                                          \
        switch (TPBV) {                                                           \
            case 64: { constexpr int TPB_ = 64; EMU_U(UN, NTF, CALL); } break;     \
            case 128: { constexpr int TPB_ = 128; EMU_U(UN, NTF, CALL); } break;   \
            default: { constexpr int TPB_ = 256; EMU_U(UN, NTF, CALL); } break;    \
        }                                                                         \
    } while (0)

#define EMU_RG(RGV, NTF, CALL)                                            \
    do {                                                                  \
        switch (RGV) {                                                    \
            case 8: { constexpr int RG_ = 8; EMU_NT(NTF, CALL); } break;   \
            case 4: { constexpr int RG_ = 4; EMU_NT(NTF, CALL); } break;   \
            case 2: { constexpr int RG_ = 2; EMU_NT(NTF, CALL); } break;   \
            default: { constexpr int RG_ = 1; EMU_NT(NTF, CALL); } break;  \
        }                                                                 \
    } while (0)

// x extent as the launcher computes it
unsigned gx_for(int64_t items, int per_block, int cap, int remap)
{
    unsigned gx = odc::grid_x_for(items, per_block, remap ? 0 : cap);
    if (remap) gx = (gx + 7u) & ~7u;
    return gx;
}

}  // namespace

int main(int argc, char **argv)
{
    if (argc < 4) {
        std::fprintf(stderr, "usage: emu dir op R [key=value ...]\n");
        return 2;
    }
    const std::string dir = argv[1], op = argv[2];
    const int R = std::atoi(argv[3]);
    int threads = 256, unroll = 4, nt = 1, remap = 0, atomic = 0, cap = 0, rg = 1, weighted = 0, bf16 = 0, count = 2;
    int lds_max = 0;  // 1: use the large-LDS gather variant even where the small one would do
    float weight = 1.0f, scale = 1.0f;
    std::string script;
    for (int k = 4; k < argc; ++k) {
        const std::string kv = argv[k];
        const size_t eq = kv.find('=');
        if (eq == std::string::npos) return 2;
        const std::string key = kv.substr(0, eq), val = kv.substr(eq + 1);
        if (key == "threads") threads = std::atoi(val.c_str());
        else if (key == "unroll") unroll = std::atoi(val.c_str());
        else if (key == "nt") nt = std::atoi(val.c_str());
        else if (key == "remap") remap = std::atoi(val.c_str());
        else if (key == "atomic") atomic = std::atoi(val.c_str());
        else if (key == "cap") cap = std::atoi(val.c_str());
        else if (key == "rg") rg = std::atoi(val.c_str());
        else if (key == "weighted") weighted = std::atoi(val.c_str());
        else if (key == "bf16") bf16 = std::atoi(val.c_str());
        else if (key == "count") count = std::atoi(val.c_str());
        else if (key == "lds_max") lds_max = std::atoi(val.c_str());
        else if (key == "script") script = val;
        else if (key == "weight") weight = std::strtof(val.c_str(), nullptr);
        else if (key == "scale") scale = std::strtof(val.c_str(), nullptr);
        else {
            std::fprintf(stderr, "unknown key %s\n", key.c_str());
            return 2;
        }
    }
    using namespace odc;

    std::vector<int64_t> numel = read_file<int64_t>(dir + "/numel.i64");
    HostLayout H;
    int rc = build_host_layout(R, static_cast<int>(numel.size()), numel.data(), &H);
    if (rc != ODC_OK) {
        std::fprintf(stderr, "layout failed: %d\n", rc);
        return 3;
    }
    const size_t arena = static_cast<size_t>(H.arena_elems), full_n = static_cast<size_t>(H.full_elems);
    BatchTable tb{H.desc.data(), H.chunk_first.data(), H.full_chunk_first.data(), H.arena_elems,
                  H.full_elems, H.T, H.gather_tile_tensors, H.gather_big};
    const bool flat = H.T == 1;
    const int64_t S = H.desc[0].S, N = H.desc[0].numel;

    if (op == "gather") {
        std::vector<uint16_t> all = read_file<uint16_t>(dir + "/arenas.u16");
        std::vector<uint16_t> full_in = read_file<uint16_t>(dir + "/full.u16");
        if (all.size() != arena * static_cast<size_t>(R) || full_in.size() != full_n) return 4;
        // exactly-sized heap blocks (malloc returns 16-byte alignment, like device memory),
        // so the sanitizer sees any access past the last element
        std::vector<uint16_t *> bufs(static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) {
            bufs[r] = static_cast<uint16_t *>(std::malloc(arena * 2));
            std::memcpy(bufs[r], all.data() + arena * r, arena * 2);
        }
        uint16_t *full = static_cast<uint16_t *>(std::malloc(full_n * 2));
        std::memcpy(full, full_in.data(), full_n * 2);
        for (int r0 = 0; r0 < R; r0 += kRanksPerLaunch) {
            const int nr = R - r0 < kRanksPerLaunch ? R - r0 : kRanksPerLaunch;
            RankPtrs rp{};
            for (int k = 0; k < nr; ++k) rp.p[k] = bufs[r0 + k];
            if (flat) {
                EMU_DISPATCH(threads, unroll, nt,
                             run_grid(TPB_, gx_for((S >> 3) + 1, TPB_ * U_, cap, remap), nr, [&] {
                                 k_gather_flat<TPB_, U_, NT_, false>(rp, full, S, N, r0, remap);
                             }));
            } else {
                const int64_t chunks = (tb.full_elems + kChunkElems - 1) >> kChunkShift;
                const int64_t tiles = (chunks + kGatherChunks - 1) / kGatherChunks;
                // remap > 0 for a multi-tensor layout: tiles handed out in XCD blocks of 2^remap
                const int tshift = remap;
                const int64_t tgroup = int64_t{8} << tshift;
                const unsigned tgx = grid_x_for((tiles + tgroup - 1) / tgroup * tgroup, 1, cap);
                if (tb.gather_tile_tensors <= kGatherFewTensors && !lds_max) {
                    EMU_NT(nt, run_grid_threaded(kBatchThreads, tgx, 1, [&] {
                               if (tb.gather_big) k_gather_batched<NT_, kGatherFewTensors, true>(tb, rp, full, r0, nr, tshift);
                               else k_gather_batched<NT_, kGatherFewTensors, false>(tb, rp, full, r0, nr, tshift);
                           }));
                } else {
                    EMU_NT(nt, run_grid_threaded(kBatchThreads, tgx, 1, [&] {
                               if (tb.gather_big) k_gather_batched<NT_, kGatherMaxTensors, true>(tb, rp, full, r0, nr, tshift);
                               else k_gather_batched<NT_, kGatherMaxTensors, false>(tb, rp, full, r0, nr, tshift);
                           }));
                }
            }
        }
        write_file(dir + "/full.out", full, full_n);
        for (auto *b : bufs) std::free(b);
        std::free(full);
        return 0;
    }

#ifndef EMU_GATHER_ONLY  // a build that only needs the gather kernels compiles much faster
    if (op == "accum" || op == "reset") {
        std::vector<float> all = read_file<float>(dir + "/acc.f32");
        if (all.size() != arena * static_cast<size_t>(R)) return 4;
        uint16_t *grad = nullptr;
        if (op == "accum") {
            std::vector<uint16_t> grad_in = read_file<uint16_t>(dir + "/grad.u16");
            if (grad_in.size() != full_n) return 4;
            grad = static_cast<uint16_t *>(std::malloc(full_n * 2));
            std::memcpy(grad, grad_in.data(), full_n * 2);
        }
        std::vector<float *> bufs(static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) {
            bufs[r] = static_cast<float *>(std::malloc(arena * 4));
            std::memcpy(bufs[r], all.data() + arena * r, arena * 4);
        }
        for (int r0 = 0; r0 < R; r0 += kRanksPerLaunch) {
            const int nr = R - r0 < kRanksPerLaunch ? R - r0 : kRanksPerLaunch;
            RankPtrs rp{};
            for (int k = 0; k < nr; ++k) rp.p[k] = bufs[r0 + k];
            if (op == "reset") {
                if (flat) {
                    EMU_DISPATCH(threads, unroll, nt,
                                 run_grid(TPB_, gx_for((S >> 2) + 1, TPB_ * U_, cap, remap), nr,
                                          [&] { k_reset_flat<TPB_, U_, NT_>(rp, S, N, r0, remap); }));
                } else {
                    const int64_t tiles = ((tb.arena_elems + kChunkElems - 1) >> kChunkShift);
                const unsigned groups = static_cast<unsigned>((nr + rg - 1) / rg);
                    EMU_RG(rg, nt, run_grid_threaded(kBatchThreads, grid_x_for(tiles, 1, cap), groups,
                                                     [&] { k_reset_batched<RG_, NT_>(tb, rp, r0, nr); }));
                }
            } else if (flat) {
#define EMU_ACC_FLAT(ATOMIC_, WEIGHTED_, NTF)                                                        \
    EMU_DISPATCH(threads, unroll, NTF, run_grid(TPB_, gx_for((S >> 2) + 1, TPB_ * U_, cap, remap), nr, [&] { \
                     k_accum_flat<TPB_, U_, NT_, ATOMIC_, WEIGHTED_>(rp, grad, S, N, r0, remap, weight);  \
                 }))
                if (atomic && weighted) EMU_ACC_FLAT(true, true, 0);
                else if (atomic) EMU_ACC_FLAT(true, false, 0);
                else if (weighted) EMU_ACC_FLAT(false, true, nt);
                else EMU_ACC_FLAT(false, false, nt);
#undef EMU_ACC_FLAT
            } else {
                const int64_t tiles = ((tb.arena_elems + kChunkElems - 1) >> kChunkShift);
                const unsigned groups = static_cast<unsigned>((nr + rg - 1) / rg);
#define EMU_ACC_BATCHED(ATOMIC_, WEIGHTED_, NTF)                                                   \
    EMU_RG(rg, NTF, run_grid_threaded(kBatchThreads, grid_x_for(tiles, 1, cap), groups, [&] {               \
               k_accum_batched<RG_, NT_, ATOMIC_, WEIGHTED_>(tb, rp, grad, r0, nr, weight);         \
           }))
                if (atomic && weighted) EMU_ACC_BATCHED(true, true, 0);
                else if (atomic) EMU_ACC_BATCHED(true, false, 0);
                else if (weighted) EMU_ACC_BATCHED(false, true, nt);
                else EMU_ACC_BATCHED(false, false, nt);
#undef EMU_ACC_BATCHED
            }
        }
        std::vector<float> out(arena * static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) std::memcpy(out.data() + arena * r, bufs[r], arena * 4);
        write_file(dir + "/acc.out", out.data(), out.size());
        for (auto *b : bufs) std::free(b);
        std::free(grad);
        return 0;
    }
    if (op == "accum_multi") {
        if (count < 2 || count > kMaxFused) return 2;
        std::vector<float> all = read_file<float>(dir + "/acc.f32");
        if (all.size() != arena * static_cast<size_t>(R)) return 4;
        GradPtrs gp{};
        std::vector<uint16_t *> gbufs;
        for (int k = 0; k < count; ++k) {
            std::vector<uint16_t> gi = read_file<uint16_t>(dir + "/grad" + std::to_string(k) + ".u16");
            if (gi.size() != full_n) return 4;
            uint16_t *g = static_cast<uint16_t *>(std::malloc(full_n * 2));
            std::memcpy(g, gi.data(), full_n * 2);
            gbufs.push_back(g);
        }
        for (int k = 0; k < kMaxFused; ++k) gp.p[k] = gbufs[k < count ? k : 0];
        std::vector<float *> bufs(static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) {
            bufs[r] = static_cast<float *>(std::malloc(arena * 4));
            std::memcpy(bufs[r], all.data() + arena * r, arena * 4);
        }
#define EMU_K(CALL)                                            \
    do {                                                       \
        switch (count) {                                       \
            case 2: { constexpr int K_ = 2; CALL; } break;      \
            case 3: { constexpr int K_ = 3; CALL; } break;      \
            case 4: { constexpr int K_ = 4; CALL; } break;      \
            case 5: { constexpr int K_ = 5; CALL; } break;      \
            case 6: { constexpr int K_ = 6; CALL; } break;      \
            case 7: { constexpr int K_ = 7; CALL; } break;      \
            default: { constexpr int K_ = 8; CALL; } break;     \
        }                                                      \
    } while (0)
        for (int r0 = 0; r0 < R; r0 += kRanksPerLaunch) {
            const int nr = R - r0 < kRanksPerLaunch ? R - r0 : kRanksPerLaunch;
            RankPtrs rp{};
            for (int k = 0; k < nr; ++k) rp.p[k] = bufs[r0 + k];
            if (flat) {
                const unsigned gx = grid_x_for((S >> 2) + 1, 64, cap);
                if (atomic) EMU_K(run_grid(64, gx, nr, [&] { k_accum_multi_flat<K_, true>(rp, gp, S, N, r0); }));
                else EMU_K(run_grid(64, gx, nr, [&] { k_accum_multi_flat<K_, false>(rp, gp, S, N, r0); }));
            } else {
                const int64_t tiles = ((tb.arena_elems + kChunkElems - 1) >> kChunkShift);
                const unsigned groups = static_cast<unsigned>(nr);
                const unsigned gx = grid_x_for(tiles, 1, cap);
                if (atomic)
                    EMU_K(run_grid_threaded(kBatchThreads, gx, groups, [&] { k_accum_multi_batched<K_, true>(tb, rp, gp, r0); }));
                else
                    EMU_K(run_grid_threaded(kBatchThreads, gx, groups, [&] { k_accum_multi_batched<K_, false>(tb, rp, gp, r0); }));
            }
        }
#undef EMU_K
        std::vector<float> out(arena * static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) std::memcpy(out.data() + arena * r, bufs[r], arena * 4);
        write_file(dir + "/acc.out", out.data(), out.size());
        for (auto *b : bufs) std::free(b);
        for (auto *g : gbufs) std::free(g);
        return 0;
    }

    if (op == "stage") {
        // script: comma-separated steps (see below); the k-th push started reads grad<k>.u16
        std::vector<float> all = read_file<float>(dir + "/acc.f32");
        if (all.size() != arena * static_cast<size_t>(R)) return 4;
        const int64_t slot = (H.arena_elems + kStageSlotAlignElems - 1) / kStageSlotAlignElems * kStageSlotAlignElems;
        std::vector<float *> accs(static_cast<size_t>(R));
        std::vector<uint16_t *> stages(static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) {
            accs[r] = static_cast<float *>(std::malloc(arena * 4));
            std::memcpy(accs[r], all.data() + arena * r, arena * 4);
            stages[r] = static_cast<uint16_t *>(std::malloc(static_cast<size_t>(slot) * R * 2));
            std::memset(stages[r], 0xEE, static_cast<size_t>(slot) * R * 2);
        }
        const size_t nflags = static_cast<size_t>(R) * R + 1, nsnap = static_cast<size_t>(R) * (R + 1);
        int32_t *flags = static_cast<int32_t *>(std::malloc(nflags * 4));
        int32_t *snap = static_cast<int32_t *>(std::malloc(nsnap * 4));
        std::memset(flags, 0x55, nflags * 4);
        run_grid(256, grid_x_for(static_cast<int64_t>(nflags), 256, 1024), 1, [&] { k_stage_zero(flags, static_cast<int64_t>(nflags)); });
        int pushes = 0;
        std::vector<uint16_t *> open_grad(static_cast<size_t>(R), nullptr);  // gradient of each client's push in flight
        auto push_claim = [&](int worker) {
            std::vector<uint16_t> gi = read_file<uint16_t>(dir + "/grad" + std::to_string(pushes++) + ".u16");
            if (gi.size() != full_n) std::exit(4);
            std::free(open_grad[worker]);
            open_grad[worker] = static_cast<uint16_t *>(std::malloc(full_n * 2));
            std::memcpy(open_grad[worker], gi.data(), full_n * 2);
            run_grid(64, (R + 63) / 64, 1, [&] { k_stage_claim(flags, R, worker); });
        };
        auto push_copy = [&](int worker) {
            const uint16_t *g = open_grad[worker];
            if (!g) std::exit(5);
            for (int r0 = 0; r0 < R; r0 += kRanksPerLaunch) {
                const int nr = R - r0 < kRanksPerLaunch ? R - r0 : kRanksPerLaunch;
                RankPtrs rs{};
                for (int k = 0; k < nr; ++k) rs.p[k] = stages[r0 + k];
                if (flat) {
                    EMU_NT(nt, run_grid(64, grid_x_for((S >> 3) + 1, 64, cap), nr, [&] {
                               k_stage_push_flat<NT_>(rs, g, flags, S, N, slot, R, r0, worker);
                           }));
                } else {
                    const int64_t chunks = ((tb.arena_elems + kChunkElems - 1) >> kChunkShift);
                    const int64_t tiles = (chunks + kPushChunks - 1) / kPushChunks;
                    const int prg = rg >= 2 ? 2 : 1;  // owners per workgroup of the push kernel
                    const unsigned groups = static_cast<unsigned>((nr + prg - 1) / prg);
                    if (prg == 2)
                        EMU_NT(nt, run_grid_threaded(kBatchThreads, grid_x_for(tiles, 1, cap), groups, [&] {
                                   k_stage_push_batched<NT_, 2>(tb, rs, g, flags, slot, R, r0, nr, worker);
                               }));
                    else
                        EMU_NT(nt, run_grid_threaded(kBatchThreads, grid_x_for(tiles, 1, cap), groups, [&] {
                                   k_stage_push_batched<NT_, 1>(tb, rs, g, flags, slot, R, r0, nr, worker);
                               }));
                }
            }
        };
        auto push_raise = [&](int worker) { run_grid(64, (R + 63) / 64, 1, [&] { k_stage_raise(flags, R, worker); }); };
        auto drain_snapshot = [&] { run_grid_threaded(64, static_cast<unsigned>(R), 1, [&] { k_stage_snapshot(flags, snap, R); }); };
        auto drain_add = [&] {
            for (int r0 = 0; r0 < R; r0 += kRanksPerLaunch) {
                const int nr = R - r0 < kRanksPerLaunch ? R - r0 : kRanksPerLaunch;
                RankPtrs ra{}, rs{};
                for (int k = 0; k < nr; ++k) {
                    ra.p[k] = accs[r0 + k];
                    rs.p[k] = stages[r0 + k];
                }
                if (flat) {
                    EMU_NT(nt, run_grid(64, grid_x_for((S >> 2) + 1, 64, cap), nr, [&] {
                               k_stage_drain_flat<NT_>(ra, rs, snap, S, N, slot, R, r0);
                           }));
                } else {
                    const int64_t tiles = ((tb.arena_elems + kChunkElems - 1) >> kChunkShift);
                    const unsigned groups = static_cast<unsigned>(nr);
                    EMU_NT(nt, run_grid_threaded(kBatchThreads, grid_x_for(tiles, 1, cap), groups, [&] {
                               k_stage_drain_batched<NT_>(tb, ra, rs, snap, slot, R, r0);
                           }));
                }
            }
        };
        auto drain_clear = [&] { run_grid(64, static_cast<unsigned>(R), 1, [&] { k_stage_clear(flags, snap, R); }); };
        // Steps: "pW" whole push by client W; its three kernels one by one: "cW" claim (takes the
        // next grad<k>.u16), "xW" copy or "xW:k:n" only the copy workgroups congruent to k mod n,
        // "rW" raise; "d" whole drain, or its kernels "s" snapshot, "a" add, "z" clear.
        size_t pos = 0;
        while (pos < script.size()) {
            size_t comma = script.find(',', pos);
            if (comma == std::string::npos) comma = script.size();
            const std::string step = script.substr(pos, comma - pos);
            pos = comma + 1;
            const int worker = step.size() > 1 ? std::atoi(step.c_str() + 1) : 0;
            switch (step[0]) {
                case 'p': push_claim(worker); push_copy(worker); push_raise(worker); break;
                case 'c': push_claim(worker); break;
                case 'x': {
                    const size_t c1 = step.find(':');
                    if (c1 != std::string::npos) {
                        const size_t c2 = step.find(':', c1 + 1);
                        if (c2 == std::string::npos) return 2;
                        part_k = static_cast<unsigned>(std::atoi(step.c_str() + c1 + 1));
                        part_n = static_cast<unsigned>(std::atoi(step.c_str() + c2 + 1));
                    }
                    push_copy(worker);
                    part_k = 0;
                    part_n = 1;
                    break;
                }
                case 'r': push_raise(worker); break;
                case 'd': drain_snapshot(); drain_add(); drain_clear(); break;
                case 's': drain_snapshot(); break;
                case 'a': drain_add(); break;
                case 'z': drain_clear(); break;
                default: std::fprintf(stderr, "unknown step %s\n", step.c_str()); return 2;
            }
        }
        for (auto *g : open_grad) std::free(g);
        std::vector<float> out(arena * static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) std::memcpy(out.data() + arena * r, accs[r], arena * 4);
        write_file(dir + "/acc.out", out.data(), out.size());
        write_file(dir + "/flags.out", flags, nflags);
        for (auto *b : accs) std::free(b);
        for (auto *b : stages) std::free(b);
        std::free(flags);
        std::free(snap);
        return 0;
    }

    if (op == "wide") {
        // acc.f64 [R * arena] in/out; grad<k>.u16 for k < count: reset, count contributions, then both
        // retrievals into out32.f32 / out16.u16 [R * arena] (in/out)
        std::vector<double> all = read_file<double>(dir + "/acc.f64");
        std::vector<float> o32 = read_file<float>(dir + "/out32.f32");
        std::vector<uint16_t> o16 = read_file<uint16_t>(dir + "/out16.u16");
        if (all.size() != arena * static_cast<size_t>(R) || o32.size() != all.size() || o16.size() != all.size()) return 4;
        std::vector<double *> accs(static_cast<size_t>(R));
        std::vector<float *> out32(static_cast<size_t>(R));
        std::vector<uint16_t *> out16(static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) {
            accs[r] = static_cast<double *>(std::malloc(arena * 8));
            std::memcpy(accs[r], all.data() + arena * r, arena * 8);
            out32[r] = static_cast<float *>(std::malloc(arena * 4));
            std::memcpy(out32[r], o32.data() + arena * r, arena * 4);
            out16[r] = static_cast<uint16_t *>(std::malloc(arena * 2));
            std::memcpy(out16[r], o16.data() + arena * r, arena * 2);
        }
        std::vector<uint16_t *> grads;
        for (int k = 0; k < count; ++k) {
            std::vector<uint16_t> gi = read_file<uint16_t>(dir + "/grad" + std::to_string(k) + ".u16");
            if (gi.size() != full_n) return 4;
            grads.push_back(static_cast<uint16_t *>(std::malloc(full_n * 2)));
            std::memcpy(grads.back(), gi.data(), full_n * 2);
        }
        auto run_op = [&](auto op_tag, void *const *outs, const uint16_t *g) {
            constexpr int OP = decltype(op_tag)::value;
            for (int r0 = 0; r0 < R; r0 += kRanksPerLaunch) {
                const int nr = R - r0 < kRanksPerLaunch ? R - r0 : kRanksPerLaunch;
                RankPtrs ra{}, ro{};
                for (int k = 0; k < nr; ++k) {
                    ra.p[k] = accs[r0 + k];
                    ro.p[k] = outs ? outs[r0 + k] : nullptr;
                }
                if (flat)
                    run_grid(kWideThreads, grid_x_for(S + 1, kWideThreads * kWideElems, cap), nr,
                             [&] { k_wide_flat<OP>(ra, ro, g, S, N, r0, scale); });
                else
                    run_grid_threaded(kBatchThreads, grid_x_for((tb.arena_elems + kChunkElems - 1) >> kChunkShift, 1, cap),
                                      static_cast<unsigned>(nr), [&] { k_wide_batched<OP>(tb, ra, ro, g, r0, scale); });
            }
        };
        run_op(std::integral_constant<int, kWideReset>{}, nullptr, nullptr);
        for (auto *g : grads) run_op(std::integral_constant<int, kWideAccumulate>{}, nullptr, g);
        run_op(std::integral_constant<int, kWideRetrieveF32>{}, reinterpret_cast<void *const *>(out32.data()), nullptr);
        run_op(std::integral_constant<int, kWideRetrieveBf16>{}, reinterpret_cast<void *const *>(out16.data()), nullptr);
        for (int r = 0; r < R; ++r) {
            std::memcpy(all.data() + arena * r, accs[r], arena * 8);
            std::memcpy(o32.data() + arena * r, out32[r], arena * 4);
            std::memcpy(o16.data() + arena * r, out16[r], arena * 2);
            std::free(accs[r]);
            std::free(out32[r]);
            std::free(out16[r]);
        }
        for (auto *g : grads) std::free(g);
        write_file(dir + "/acc.out", all.data(), all.size());
        write_file(dir + "/out32.out", o32.data(), o32.size());
        write_file(dir + "/out16.out", o16.data(), o16.size());
        return 0;
    }

    if (op == "reduce") {
        // groups.f32 [count * R * arena] group-major; out.f32 [R * arena] in/out; inplace=1: the
        // output buffers are group 0's (out.f32 is then ignored on input)
        const int K = count;
        std::vector<float> all = read_file<float>(dir + "/groups.f32");
        std::vector<float> out_in = read_file<float>(dir + "/out.f32");
        if (K < 1 || all.size() != arena * static_cast<size_t>(R) * K || out_in.size() != arena * static_cast<size_t>(R)) return 4;
        std::vector<float *> srcs(static_cast<size_t>(R) * K), outs(static_cast<size_t>(R));
        for (size_t q = 0; q < srcs.size(); ++q) {
            srcs[q] = static_cast<float *>(std::malloc(arena * 4));
            std::memcpy(srcs[q], all.data() + arena * q, arena * 4);
        }
        for (int r = 0; r < R; ++r) {
            if (lds_max) outs[r] = srcs[r];  // reuse of the flag: in place into group 0
            else {
                outs[r] = static_cast<float *>(std::malloc(arena * 4));
                std::memcpy(outs[r], out_in.data() + arena * r, arena * 4);
            }
        }
        for (int r0 = 0; r0 < R; r0 += kReduceRanks) {
            const int nr = R - r0 < kReduceRanks ? R - r0 : kReduceRanks;
            for (int k0 = 0; k0 < K; k0 += kReduceSources) {
                const int cnt = K - k0 < kReduceSources ? K - k0 : kReduceSources;
                ReducePtrs p{};
                for (int r = 0; r < nr; ++r) {
                    for (int k = 0; k < cnt; ++k) p.src[r][k] = srcs[static_cast<size_t>(k0 + k) * R + r0 + r];
                    p.out[r] = outs[r0 + r];
                }
#define EMU_REDUCE(K_, INIT_)                                                                                        \
    do {                                                                                                             \
        if (flat) run_grid(64, grid_x_for((S >> 2) + 1, 64, cap), nr, [&] { k_reduce_flat<K_, INIT_>(p, S, N, r0); }); \
        else                                                                                                         \
            run_grid_threaded(kBatchThreads, grid_x_for((tb.arena_elems + kChunkElems - 1) >> kChunkShift, 1, cap),  \
                              static_cast<unsigned>(nr), [&] { k_reduce_batched<K_, INIT_>(tb, p, r0); });           \
    } while (0)
#define EMU_REDUCE_K(INIT_)                          \
    switch (cnt) {                                   \
        case 1: EMU_REDUCE(1, INIT_); break;         \
        case 2: EMU_REDUCE(2, INIT_); break;         \
        case 3: EMU_REDUCE(3, INIT_); break;         \
        case 4: EMU_REDUCE(4, INIT_); break;         \
        case 5: EMU_REDUCE(5, INIT_); break;         \
        case 6: EMU_REDUCE(6, INIT_); break;         \
        case 7: EMU_REDUCE(7, INIT_); break;         \
        default: EMU_REDUCE(8, INIT_); break;        \
    }
                if (k0 == 0) EMU_REDUCE_K(true)
                else EMU_REDUCE_K(false)
#undef EMU_REDUCE_K
#undef EMU_REDUCE
            }
        }
        std::vector<float> out(arena * static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) std::memcpy(out.data() + arena * r, outs[r], arena * 4);
        write_file(dir + "/out.out", out.data(), out.size());
        if (!lds_max)
            for (auto *b : outs) std::free(b);
        for (auto *b : srcs) std::free(b);
        return 0;
    }

    if (op == "retrieve") {
        std::vector<float> all = read_file<float>(dir + "/acc.f32");
        if (all.size() != arena * static_cast<size_t>(R)) return 4;
        const size_t esz = bf16 ? 2 : 4;
        std::vector<char> out_in = read_file<char>(dir + "/out.bin");
        if (out_in.size() != arena * esz * static_cast<size_t>(R)) return 4;
        std::vector<float *> accs(static_cast<size_t>(R));
        std::vector<char *> outs(static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) {
            accs[r] = static_cast<float *>(std::malloc(arena * 4));
            std::memcpy(accs[r], all.data() + arena * r, arena * 4);
            outs[r] = static_cast<char *>(std::malloc(arena * esz));
            std::memcpy(outs[r], out_in.data() + arena * esz * r, arena * esz);
        }
        for (int r0 = 0; r0 < R; r0 += kRanksPerLaunch) {
            const int nr = R - r0 < kRanksPerLaunch ? R - r0 : kRanksPerLaunch;
            RankPtrs ra{}, ro{};
            for (int k = 0; k < nr; ++k) {
                ra.p[k] = accs[r0 + k];
                ro.p[k] = outs[r0 + k];
            }
            if (flat) {
                if (bf16) {
                    EMU_DISPATCH(threads, unroll, nt, run_grid(TPB_, gx_for((S >> 2) + 1, TPB_ * U_, cap, 0), nr, [&] {
                                     k_retrieve_flat<TPB_, U_, NT_, true>(ra, ro, S, N, r0, scale);
                                 }));
                } else {
                    EMU_DISPATCH(threads, unroll, nt, run_grid(TPB_, gx_for((S >> 2) + 1, TPB_ * U_, cap, 0), nr, [&] {
                                     k_retrieve_flat<TPB_, U_, NT_, false>(ra, ro, S, N, r0, scale);
                                 }));
                }
            } else {
                const int64_t tiles = ((tb.arena_elems + kChunkElems - 1) >> kChunkShift);
                const unsigned groups = static_cast<unsigned>((nr + rg - 1) / rg);
                if (bf16) {
                    EMU_RG(rg, nt, run_grid_threaded(kBatchThreads, grid_x_for(tiles, 1, cap), groups, [&] {
                               k_retrieve_batched<RG_, NT_, true>(tb, ra, ro, r0, nr, scale);
                           }));
                } else {
                    EMU_RG(rg, nt, run_grid_threaded(kBatchThreads, grid_x_for(tiles, 1, cap), groups, [&] {
                               k_retrieve_batched<RG_, NT_, false>(tb, ra, ro, r0, nr, scale);
                           }));
                }
            }
        }
        std::vector<char> out(arena * esz * static_cast<size_t>(R));
        std::vector<float> acc_after(arena * static_cast<size_t>(R));
        for (int r = 0; r < R; ++r) {
            std::memcpy(out.data() + arena * esz * r, outs[r], arena * esz);
            std::memcpy(acc_after.data() + arena * r, accs[r], arena * 4);
        }
        write_file(dir + "/out.out", out.data(), out.size());
        write_file(dir + "/acc.out", acc_after.data(), acc_after.size());
        for (auto *b : accs) std::free(b);
        for (auto *b : outs) std::free(b);
        return 0;
    }
#endif  // EMU_GATHER_ONLY

    std::fprintf(stderr, "unknown op %s\n", op.c_str());
    return 2;
}

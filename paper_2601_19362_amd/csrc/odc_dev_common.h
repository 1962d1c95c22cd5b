// Types and memory-access helpers shared by all ODC kernels (gfx950): 16-byte vectors, loads and
// stores with and without the non-temporal hint, byte-unaligned wide loads, the hand-written
// sc1 + nt store, the pointer table that travels in the kernel arguments.
#pragma once

#include <cstdint>

#include "odc_internal.h"

namespace odc {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Wide accesses whose address is only 2-byte aligned.
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef u32x2 u32x2_a2 __attribute__((aligned(2)));

struct RankPtrs {
    void *p[kRanksPerLaunch];
};

// Every data pointer in these kernels points to device (global) memory.  Pointers that reach
// a lane through LDS or a per-lane table lookup lose that information and would be accessed
// with slower generic-address instructions, so every access goes through a pointer that is
// explicitly in the global address space.  (On the host, in the CPU emulation build, the
// qualifier is empty.)
#ifdef __HIP_DEVICE_COMPILE__
#define ODC_GLOBAL __attribute__((address_space(1)))
#else
#define ODC_GLOBAL
#endif

// Register budget of a kernel, as the number of wavefronts per SIMD it must allow (512 vector
// registers per SIMD: 8 wavefronts = 64 registers each).  Used where the compiler lands one
// register above a boundary.  (Empty in the CPU emulation build.)
#ifdef __HIP__
#define ODC_WAVES_PER_EU(n) __attribute__((amdgpu_waves_per_eu(n)))
#else
#define ODC_WAVES_PER_EU(n)
#endif

template <bool NT, typename V>
__device__ __forceinline__ V ld(const V *p)
{
    const ODC_GLOBAL V *q = (const ODC_GLOBAL V *)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

template <bool NT, typename V>
__device__ __forceinline__ void st(V *p, V v)
{
    ODC_GLOBAL V *q = (ODC_GLOBAL V *)p;
    if constexpr (NT) __builtin_nontemporal_store(v, q);
    else *q = v;
}

// Stores with the non-temporal hint and system-scope write-through (sc1 nt).  For streams
// that are only written (gather output, reset, retrieval, staging) this measured about 3 %
// faster than the plain non-temporal store; the compiler has no builtin for the combination,
// so the store is written as one instruction.  It is an ordinary vector store: the only
// thing the compiler does not know is that it bumps the memory-operation counter, which can
// only make a later wait longer, never too short.
template <typename V>
__device__ __forceinline__ void st_sc1_nt(V *p, V v)
{
    static_assert(sizeof(V) == 16 || sizeof(V) == 8, "a 16-byte or an 8-byte vector");
#ifdef __HIP_DEVICE_COMPILE__
    if constexpr (sizeof(V) == 16) asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
    else asm volatile("global_store_dwordx2 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
#else
    *p = v;
#endif
}

// Store of a write-only stream: WT = 2 sc1 + nt, 1 nt, 0 plain.
template <int WT, typename V>
__device__ __forceinline__ void st_stream(V *p, V v)
{
    if constexpr (WT == 2) st_sc1_nt(p, v);
    else st<WT == 1>(p, v);
}

template <bool NT>
__device__ __forceinline__ u32x4 ld_u128_unaligned(const uint16_t *p)
{
    const ODC_GLOBAL u32x4_a2 *q = (const ODC_GLOBAL u32x4_a2 *)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

template <bool NT>
__device__ __forceinline__ u32x2 ld_u64_unaligned(const uint16_t *p)
{
    const ODC_GLOBAL u32x2_a2 *q = (const ODC_GLOBAL u32x2_a2 *)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

// Single elements (heads, tails, ragged ends, pieces of small tensors).
__device__ __forceinline__ uint16_t ld_u16(const uint16_t *p) { return *(const ODC_GLOBAL uint16_t *)p; }
__device__ __forceinline__ void st_u16(uint16_t *p, uint16_t v) { *(ODC_GLOBAL uint16_t *)p = v; }
__device__ __forceinline__ float ld_f32(const float *p) { return *(const ODC_GLOBAL float *)p; }
__device__ __forceinline__ void st_f32(float *p, float v) { *(ODC_GLOBAL float *)p = v; }

// bf16 -> binary32 is exact: the 16 bits are the high half of the word.
__device__ __forceinline__ float widen_lo(uint32_t two) { return __uint_as_float(two << 16); }
__device__ __forceinline__ float widen_hi(uint32_t two) { return __uint_as_float(two & 0xFFFF0000u); }
__device__ __forceinline__ float widen_one(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

template <bool ATOMIC, bool WEIGHTED>
__device__ __forceinline__ void add_one(float *a, float v, float w)
{
    if constexpr (ATOMIC) unsafeAtomicAdd(a, WEIGHTED ? w * v : v);
    else if constexpr (WEIGHTED) st_f32(a, __builtin_fmaf(w, v, ld_f32(a)));
    else st_f32(a, ld_f32(a) + v);
}


// ----------------------------------------------------------------------------------- probe
template <int TPB, int U>
__global__ __launch_bounds__(TPB) void k_probe_copy(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                         int64_t nvec)
{
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * (TPB * U) + threadIdx.x;
    u32x4 reg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = v0 + u * TPB;
        if (v < nvec) reg[u] = __builtin_nontemporal_load(src + v);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t v = v0 + u * TPB;
        if (v < nvec) __builtin_nontemporal_store(reg[u], dst + v);
    }
}

}  // namespace
}  // namespace odc

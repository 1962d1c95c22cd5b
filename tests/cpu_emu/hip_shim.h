// Host stand-ins for the few HIP constructs the ODC kernels use, so that the kernel source
// can be compiled for the CPU (clang++, AddressSanitizer + UBSan) and run there.  Kernels
// without LDS run one thread after the other; kernels that stage data in LDS run each
// workgroup on real host threads with __syncthreads() mapped to a pthread barrier.
// Test infrastructure only.
#pragma once

#include <pthread.h>

#include <cstdint>
#include <cstring>

#define __global__
#define __device__
#define __host__
#define __shared__ static
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(n)

struct dim3 {
    unsigned x = 1, y = 1, z = 1;
};

static thread_local dim3 blockIdx, threadIdx;
static dim3 gridDim, blockDim;

static pthread_barrier_t *emu_block_barrier = nullptr;  // set while a threaded workgroup runs

static inline void __syncthreads()
{
    if (emu_block_barrier) pthread_barrier_wait(emu_block_barrier);
}

static inline float __uint_as_float(uint32_t u)
{
    float f;
    std::memcpy(&f, &u, sizeof f);
    return f;
}

static inline void unsafeAtomicAdd(float *a, float v) { *a = *a + v; }
static inline void unsafeAtomicAdd(double *a, double v) { *a = *a + v; }

static inline int atomicAdd(int32_t *p, int v)
{
    const int old = *p;
    *p = old + v;
    return old;
}

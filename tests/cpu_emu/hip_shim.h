// Host stand-ins for the few HIP constructs the ODC kernels use, so that the kernel source
// can be compiled for the CPU (clang++, AddressSanitizer + UBSan) and run thread by thread.
// The kernels use no LDS and no barrier, so running the threads of a grid one after the
// other is a valid schedule.  Test infrastructure only.
#pragma once

#include <cstdint>
#include <cstring>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(n)

struct dim3 {
    unsigned x = 1, y = 1, z = 1;
};

static dim3 blockIdx, threadIdx, gridDim, blockDim;

static inline float __uint_as_float(uint32_t u)
{
    float f;
    std::memcpy(&f, &u, sizeof f);
    return f;
}

static inline void unsafeAtomicAdd(float *a, float v) { *a = *a + v; }

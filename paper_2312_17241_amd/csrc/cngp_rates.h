// Microbenchmarks of the chip rates that bound the encoding kernels: streaming copy, random
// gathers, global floating-point atomics and LDS fp64 atomics.  They give the benchmark an
// "applicable roofline" measured in the same run, on the same device.
#pragma once
#include "cngp_device.h"

namespace cngp {

__device__ __forceinline__ uint32_t rate_mix(uint32_t a) {
    a ^= a >> 16; a *= 0x7feb352dU; a ^= a >> 15; a *= 0x846ca68bU; a ^= a >> 16;
    return a;
}

__global__ __launch_bounds__(kBlock) void rate_copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst,
                                                          const size_t n)
{
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// GROUP lanes read (ATOMIC = false) or atomically add to (ATOMIC = true) one random row of GROUP floats
// of a table of rows_mask + 1 rows; 8 independent rows per lane and iteration.
template <int GROUP, bool ATOMIC>
__global__ __launch_bounds__(kBlock) void rate_rows_kernel(float *__restrict__ tab, const uint32_t rows_mask,
                                                          const int iters, float *__restrict__ sink)
{
    const uint32_t gid = blockIdx.x * kBlock + threadIdx.x, grp = gid / GROUP, k = gid % GROUP;
    uint32_t r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = rate_mix(grp * 8u + j);
    float acc = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float *q = tab + (size_t)((r[j] + it * 0x9e3779b1u) & rows_mask) * GROUP + k;
            if (ATOMIC) atomic_add(q, 1.0f);
            else acc += *q;
        }
    }
    if (acc == 12345.678f) sink[0] = acc;          // keeps the loads alive
}

// Atomic adds (no return value, workgroup scope) to random rows of 32 consecutive accumulators of type T in a
// 64 KB (4-byte T) or 128 KB (fp64) LDS array: 16384 accumulators either way, 32 adjacent lanes per row, so that
// the three accumulator types are measured on the same access pattern and with the same compiler flags as the
// kernels of the library.
template <typename T>
__global__ __launch_bounds__(1024) void rate_lds_atomic_kernel(const int iters, float *__restrict__ sink)
{
    extern __shared__ __align__(16) unsigned char rate_lds_raw[];
    T *lds = reinterpret_cast<T *>(rate_lds_raw);
    constexpr uint32_t kAccs = 16384, kRows = kAccs / 32;
    for (uint32_t i = threadIdx.x; i < kAccs; i += 1024) lds[i] = T(0);
    __syncthreads();
    const uint32_t gid = blockIdx.x * 1024 + threadIdx.x, grp = gid / 32, k = gid % 32;
    uint32_t r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = rate_mix(grp * 8u + j);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            (void)__hip_atomic_fetch_add(lds + ((r[j] + it * 97u) & (kRows - 1)) * 32 + k, T(1), __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    __syncthreads();
    if (lds[threadIdx.x] == T(3)) sink[0] = 1.0f;    // (every accumulator ends far above 3: keeps the adds alive)
}

// Random 4-byte reads of a 128 KB LDS table, every lane its own address (the lookups of the level-resident forward
// kernel): 8 independent reads per lane and iteration.
__global__ __launch_bounds__(1024) void rate_lds_gather_kernel(const int iters, float *__restrict__ sink)
{
    extern __shared__ __align__(16) unsigned char rate_lds_raw[];
    uint32_t *lds = reinterpret_cast<uint32_t *>(rate_lds_raw);
    constexpr uint32_t kWords = 32768;
    for (uint32_t i = threadIdx.x; i < kWords; i += 1024) lds[i] = i;
    __syncthreads();
    const uint32_t gid = blockIdx.x * 1024 + threadIdx.x;
    uint32_t r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = rate_mix(gid * 8u + j);
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc += lds[(r[j] + it * 0x9e3779b1u) & (kWords - 1)];
    }
    if (acc == 0x12345678u) sink[0] = 1.0f;          // keeps the reads alive
}

}  // namespace cngp

// Optional reordering of a batch of query points by Morton code (the interleaved bits of the quantised
// coordinates), so that points that are close in space are close in the batch.  Not part of the paper's
// method: its hash tables leave no locality between neighbouring vertices, but neighbouring POINTS share
// the vertices of the coarse levels, and a forward pass over points in Morton order finds them in the
// first-level cache (measured: 2x on uniformly random points).  The sort itself is rocPRIM's radix sort
// (a stable least-significant-digit sort on the 20- or 21-bit codes); the code and gather kernels are here.
#include <cstdint>
#include <cstring>

#include <hip/hip_runtime.h>
#include <rocprim/device/device_radix_sort.hpp>

#include "../../include/cngp.h"

namespace cngp { int record_hip_failure(hipError_t e, const char *what); }   // cngp_api.hip

namespace {

constexpr int kSortBlock = 256;

// Bits per axis: more than these change nothing measurable (the finer levels have no reuse to find).
constexpr int morton_bits(int d) { return d == 3 ? 7 : 10; }

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// code = bit b of coordinate j at position b * D + j; coordinates quantised as floor(x * 2^B) clamped to
// [0, 2^B - 1] (the scaling by a power of two is exact; a NaN counts as 0).
template <int D>
__global__ __launch_bounds__(kSortBlock) void morton_keys_kernel(const float *__restrict__ x, const int64_t N,
                                                                 uint32_t *__restrict__ keys, int32_t *__restrict__ index)
{
    constexpr int B = morton_bits(D);
    const int64_t n = (int64_t)blockIdx.x * kSortBlock + threadIdx.x;
    if (n >= N) return;
    uint32_t code = 0;
#pragma unroll
    for (int j = 0; j < D; ++j) {
        const float    v = fminf(fmaxf(x[n * D + j] * (float)(1 << B), 0.0f), (float)((1 << B) - 1));
        const uint32_t q = (uint32_t)v;
#pragma unroll
        for (int b = 0; b < B; ++b) code |= ((q >> b) & 1u) << (b * D + j);
    }
    keys[n] = code;
    index[n] = (int32_t)n;
}

template <int D>
__global__ __launch_bounds__(kSortBlock) void gather_points_kernel(const float *__restrict__ x, const int32_t *__restrict__ perm,
                                                                   const int64_t N, float *__restrict__ x_sorted)
{
    const int64_t n = (int64_t)blockIdx.x * kSortBlock + threadIdx.x;
    if (n >= N) return;
    const int64_t from = perm[n];
#pragma unroll
    for (int j = 0; j < D; ++j) x_sorted[n * D + j] = x[from * D + j];
}

// Scratch of rocPRIM's sort for n pairs (host call, no launch); 0 when it cannot be asked (no device).
size_t sort_temp_bytes(size_t n, unsigned bits) {
    size_t bytes = 0;
    const hipError_t e = rocprim::radix_sort_pairs(nullptr, bytes, (const uint32_t *)nullptr, (uint32_t *)nullptr,
                                                   (const int32_t *)nullptr, (int32_t *)nullptr, n, 0u, bits, (hipStream_t)0);
    if (e != hipSuccess) { (void)hipGetLastError(); return 0; }
    return bytes ? bytes : 1;
}

template <int D>
int morton_sort(const float *x, int64_t N, int32_t *perm, float *x_sorted, char *ws, size_t temp_bytes, hipStream_t s) {
    uint32_t *keys_in = (uint32_t *)ws, *keys_out = (uint32_t *)(ws + align256((size_t)N * 4));
    int32_t  *index = (int32_t *)(ws + 2 * align256((size_t)N * 4));
    void     *temp = ws + 3 * align256((size_t)N * 4);
    const unsigned blocks = (unsigned)((N + kSortBlock - 1) / kSortBlock);
    morton_keys_kernel<D><<<blocks, kSortBlock, 0, s>>>(x, N, keys_in, index);
    if (hipError_t e = hipGetLastError()) return cngp::record_hip_failure(e, "morton_keys_kernel");
    if (hipError_t e = rocprim::radix_sort_pairs(temp, temp_bytes, keys_in, keys_out, index, perm, (size_t)N, 0u,
                                                 (unsigned)(morton_bits(D) * D), s)) {
        (void)hipGetLastError();
        return cngp::record_hip_failure(e, "rocprim::radix_sort_pairs");
    }
    if (x_sorted) {
        gather_points_kernel<D><<<blocks, kSortBlock, 0, s>>>(x, perm, N, x_sorted);
        if (hipError_t e = hipGetLastError()) return cngp::record_hip_failure(e, "gather_points_kernel");
    }
    return CNGP_OK;
}

}  // namespace

extern "C" {

size_t cngp_morton_sort_workspace_bytes(int32_t d, int64_t N) {
    if ((d != 2 && d != 3) || N <= 0 || N > 0x7fffffffLL) return 0;
    const size_t temp = sort_temp_bytes((size_t)N, (unsigned)(morton_bits(d) * d));
    return temp ? 3 * align256((size_t)N * 4) + align256(temp) : 0;
}

int cngp_morton_sort(int32_t d, const float *x, int64_t N, int32_t *perm, float *x_sorted,
                     void *workspace, size_t workspace_bytes, void *stream) {
    if (d != 2 && d != 3) return CNGP_ERR_INVALID;
    if (N < 0 || N > 0x7fffffffLL) return CNGP_ERR_INVALID;
    if (N == 0) return CNGP_OK;
    if (!x || !perm) return CNGP_ERR_NULL;
    const size_t temp = sort_temp_bytes((size_t)N, (unsigned)(morton_bits(d) * d));
    if (!temp) return cngp::record_hip_failure(hipErrorUnknown, "rocprim::radix_sort_pairs (size query)");
    const size_t need = 3 * align256((size_t)N * 4) + align256(temp);
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < need) return CNGP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    return d == 3 ? morton_sort<3>(x, N, perm, x_sorted, (char *)workspace, temp, s)
                  : morton_sort<2>(x, N, perm, x_sorted, (char *)workspace, temp, s);
}

}  // extern "C"

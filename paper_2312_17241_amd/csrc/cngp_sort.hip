// Optional reordering of a batch of query points by Morton code (the interleaved bits of the quantised
// coordinates), so that points that are close in space are close in the batch.  Not part of the paper's
// method: its hash tables leave no locality between neighbouring vertices, but neighbouring POINTS share
// the vertices of the coarse levels.
//
// The sort is a stable least-significant-digit radix sort of (code, index) pairs, 7 bits per pass, three
// passes for the 20- or 21-bit codes (10, 7 and 5 bits per axis for d = 2, 3, 4), written for 64-lane wavefronts:
//   keys     one workgroup per tile of 8192 points: codes from x, and the tile's histogram of the first digit
//   count    (passes 2, 3) the tile histograms of the next digit in the order the previous pass left
//   row scan one workgroup per digit value: exclusive prefix over the tiles, the digit's total beside it
//   scatter  one workgroup per tile.  A wavefront walks its eighth of the tile 64 elements at a time; the lanes
//            that hold the same digit find each other with seven ballots, which gives every element its rank
//            among the equal digits before it without an atomic, so the order of equal digits is the order of
//            the input.  The tile is then laid out by digit in LDS and leaves in runs of consecutive addresses
//            (64 elements of a digit per tile on average: whole cache lines instead of 64 lines per store).
// No kernel waits for another workgroup; every pass is three ordinary launches.
#include <cstdint>
#include <cstring>

#include <hip/hip_runtime.h>

#include "../../include/cngp.h"

namespace cngp { int record_hip_failure(hipError_t e, const char *what); }   // cngp_api.hip

namespace {

constexpr int kSortBlock = 256;          // gather kernel
constexpr int kDigitBits = 7;
constexpr int kDigits = 1 << kDigitBits;
constexpr int kTileBlock = 512;          // 8 wavefronts per tile
constexpr int kTileWaves = kTileBlock / 64;
constexpr int kRounds = 16;              // elements per lane
constexpr int kTile = kTileBlock * kRounds;
constexpr int kScanBlock = 1024;

// Bits per axis: more than these change nothing measurable (the finer levels have no reuse to find).
constexpr int morton_bits(int d) { return d == 3 ? 7 : d == 4 ? 5 : 10; }

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline int64_t tiles_of(int64_t N) { return (N + kTile - 1) / kTile; }

// code = bit b of coordinate j at position b * D + j; coordinates quantised as floor(x * 2^B) clamped to
// [0, 2^B - 1] (the scaling by a power of two is exact; a NaN counts as 0).
template <int D>
__device__ __forceinline__ uint32_t morton_code(const float *__restrict__ x, const int64_t n)
{
    constexpr int B = morton_bits(D);
    uint32_t code = 0;
#pragma unroll
    for (int j = 0; j < D; ++j) {
        const float    v = fminf(fmaxf(x[n * D + j] * (float)(1 << B), 0.0f), (float)((1 << B) - 1));
        const uint32_t q = (uint32_t)v;
#pragma unroll
        for (int b = 0; b < B; ++b) code |= ((q >> b) & 1u) << (b * D + j);
    }
    return code;
}

// Sum of a tile's per-wavefront histograms, written as column `tile` of counts[digit][tiles].
__device__ __forceinline__ void flush_tile_histogram(const uint32_t *hist, uint32_t *__restrict__ counts,
                                                     const int64_t tiles, const int64_t tile, const int t)
{
    if (t < kDigits) {
        uint32_t sum = 0;
#pragma unroll
        for (int w = 0; w < kTileWaves; ++w) sum += hist[w * kDigits + t];
        counts[(size_t)t * (size_t)tiles + (size_t)tile] = sum;
    }
}

template <int D>
__global__ __launch_bounds__(kTileBlock) void morton_keys_kernel(const float *__restrict__ x, const int64_t N,
                                                                 uint32_t *__restrict__ keys, uint32_t *__restrict__ counts,
                                                                 const int64_t tiles)
{
    __shared__ uint32_t hist[kTileWaves * kDigits];
    const int     t = threadIdx.x, w = t >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * kTile;
    for (int i = t; i < kTileWaves * kDigits; i += kTileBlock) hist[i] = 0;
    __syncthreads();
#pragma unroll 4
    for (int r = 0; r < kRounds; ++r) {
        const int64_t n = n0 + (int64_t)r * kTileBlock + t;
        if (n < N) {
            const uint32_t code = morton_code<D>(x, n);
            keys[n] = code;
            atomicAdd(&hist[w * kDigits + (code & (kDigits - 1))], 1u);
        }
    }
    __syncthreads();
    flush_tile_histogram(hist, counts, tiles, blockIdx.x, t);
}

__global__ __launch_bounds__(kTileBlock) void digit_count_kernel(const uint32_t *__restrict__ keys, const int64_t N, const int shift,
                                                                 uint32_t *__restrict__ counts, const int64_t tiles)
{
    __shared__ uint32_t hist[kTileWaves * kDigits];
    const int     t = threadIdx.x, w = t >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * kTile;
    for (int i = t; i < kTileWaves * kDigits; i += kTileBlock) hist[i] = 0;
    __syncthreads();
    uint32_t key[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t n = n0 + (int64_t)r * kTileBlock + t;
        key[r] = n < N ? keys[n] : 0u;
    }
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t n = n0 + (int64_t)r * kTileBlock + t;
        if (n < N) atomicAdd(&hist[w * kDigits + ((key[r] >> shift) & (kDigits - 1))], 1u);
    }
    __syncthreads();
    flush_tile_histogram(hist, counts, tiles, blockIdx.x, t);
}

// Exclusive prefix of v over the 64 lanes of a wavefront; *total = the sum.
__device__ __forceinline__ uint32_t wave_exclusive_scan(const uint32_t v, uint32_t *total)
{
    const int lane = threadIdx.x & 63;
    uint32_t  inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(inc, o, 64);
        if (lane >= o) inc += up;
    }
    *total = __shfl(inc, 63, 64);
    return inc - v;
}

// Row `digit` of counts[digit][tiles] -> its exclusive prefix over the tiles, in place; totals[digit] = the row's sum.
__global__ __launch_bounds__(kScanBlock) void digit_row_scan_kernel(uint32_t *__restrict__ counts, const int64_t tiles,
                                                                    uint32_t *__restrict__ totals)
{
    __shared__ uint32_t wave_sum[kScanBlock / 64];
    uint32_t *row = counts + (size_t)blockIdx.x * (size_t)tiles;
    const int t = threadIdx.x, w = t >> 6, lane = t & 63;
    uint32_t  carry = 0;
    for (int64_t base = 0; base < tiles; base += kScanBlock) {
        const int64_t  i = base + t;
        const uint32_t v = i < tiles ? row[i] : 0u;
        uint32_t       wtotal;
        const uint32_t in_wave = wave_exclusive_scan(v, &wtotal);
        if (lane == 0) wave_sum[w] = wtotal;
        __syncthreads();
        uint32_t before = 0, all = 0;
#pragma unroll
        for (int k = 0; k < kScanBlock / 64; ++k) {
            const uint32_t s = wave_sum[k];
            before += k < w ? s : 0u;
            all += s;
        }
        if (i < tiles) row[i] = carry + before + in_wave;
        carry += all;
        __syncthreads();
    }
    if (t == 0) totals[blockIdx.x] = carry;
}

// One pass of the sort for one tile.  keys_in in the order of the previous pass; index_in NULL = the identity
// (first pass).  keys_out NULL on the last pass (nobody reads them).  Element n of the input goes to
//   sum of totals of smaller digits + counts[digit][tile] (prefix over earlier tiles) + its rank inside the tile.
__global__ __launch_bounds__(kTileBlock) void digit_scatter_kernel(
    const uint32_t *__restrict__ keys_in, const int32_t *__restrict__ index_in, const int64_t N, const int shift,
    const uint32_t *__restrict__ counts, const int64_t tiles, const uint32_t *__restrict__ totals,
    uint32_t *__restrict__ keys_out, int32_t *__restrict__ index_out)
{
    __shared__ uint32_t wave_count[kTileWaves * kDigits];   // per wavefront and digit: running count, then base inside the digit's run
    __shared__ uint32_t tile_start[kDigits];                // first slot of the digit in the sorted tile
    __shared__ uint32_t dest[kDigits];                      // global position of that slot
    __shared__ uint32_t stage[kTile];                       // the tile in sorted order: first its keys, then its indices
    __shared__ uint32_t carry[2];
    const int     t = threadIdx.x, w = t >> 6, lane = t & 63;
    const int64_t tile = blockIdx.x;
    const int64_t n0 = tile * kTile;
    const int     tile_n = (int)((N - n0 < kTile) ? N - n0 : kTile);
    uint32_t     *mine = wave_count + w * kDigits;
    for (int i = t; i < kTileWaves * kDigits; i += kTileBlock) wave_count[i] = 0;
    __syncthreads();

    // rank of every element among the equal digits before it in this wavefront's eighth of the tile
    uint32_t key[kRounds], rank[kRounds];
    int32_t  index[kRounds];
    const int64_t  w0 = n0 + (int64_t)w * (kRounds * 64);
    const uint64_t below = lane ? (~0ull >> (64 - lane)) : 0ull;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t n = w0 + r * 64 + lane;
        key[r] = n < N ? keys_in[n] : 0u;
        index[r] = n < N ? (index_in ? index_in[n] : (int32_t)n) : 0;
    }
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t  n = w0 + r * 64 + lane;
        const bool     valid = n < N;
        const uint32_t digit = (key[r] >> shift) & (kDigits - 1);
        uint64_t       peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kDigitBits; ++b) {
            const bool     bit = (digit >> b) & 1u;
            const uint64_t has = __ballot(bit);
            peers &= bit ? has : ~has;
        }
        rank[r] = 0;
        if (valid) {
            const uint32_t seen = mine[digit];                        // same address for all peers: one broadcast read
            rank[r] = seen + (uint32_t)__popcll(peers & below);
            if ((peers & below) == 0) mine[digit] = seen + (uint32_t)__popcll(peers);   // the first peer moves the count on
        }
        __builtin_amdgcn_wave_barrier();                              // the next round's read stays behind this write
    }
    __syncthreads();

    // per digit: counts of the wavefronts -> bases inside the digit's run; runs laid end to end; global targets
    uint32_t count = 0, total = 0;
    if (t < kDigits) {                                                 // wavefronts 0 and 1 hold the 128 digits
#pragma unroll
        for (int k = 0; k < kTileWaves; ++k) {
            const uint32_t c = wave_count[k * kDigits + t];
            wave_count[k * kDigits + t] = count;
            count += c;
        }
        total = totals[t];
    }
    uint32_t       count_sum, total_sum;
    const uint32_t count_before = wave_exclusive_scan(count, &count_sum);
    const uint32_t total_before = wave_exclusive_scan(total, &total_sum);
    if (t == 0) { carry[0] = count_sum; carry[1] = total_sum; }        // digits 0..63, for wavefront 1
    __syncthreads();
    if (t < kDigits) {
        tile_start[t] = (w ? carry[0] : 0u) + count_before;
        dest[t] = (w ? carry[1] : 0u) + total_before + counts[(size_t)t * (size_t)tiles + (size_t)tile];
    }
    __syncthreads();

    // keys: into LDS in sorted order (rank[] becomes the slot), out in runs of consecutive addresses;
    // slot j of the sorted tile is element (j - tile_start[digit]) of its digit's run
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t  n = w0 + r * 64 + lane;
        const uint32_t digit = (key[r] >> shift) & (kDigits - 1);
        rank[r] = n < N ? tile_start[digit] + mine[digit] + rank[r] : (uint32_t)kTile;
        if (rank[r] < (uint32_t)kTile) stage[rank[r]] = key[r];
    }
    __syncthreads();
    uint32_t to[kRounds];
#pragma unroll
    for (int i = 0; i < kRounds; ++i) {
        const int j = t + i * kTileBlock;
        to[i] = 0xffffffffu;
        if (j < tile_n) {
            const uint32_t k = stage[j];
            const uint32_t digit = (k >> shift) & (kDigits - 1);
            to[i] = dest[digit] + ((uint32_t)j - tile_start[digit]);
            if (keys_out && (int64_t)to[i] < N) keys_out[to[i]] = k;
        }
    }
    __syncthreads();
    // indices: the same way through the same buffer
#pragma unroll
    for (int r = 0; r < kRounds; ++r)
        if (rank[r] < (uint32_t)kTile) stage[rank[r]] = (uint32_t)index[r];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kRounds; ++i) {
        const int j = t + i * kTileBlock;
        if (j < tile_n && (int64_t)to[i] < N) index_out[to[i]] = (int32_t)stage[j];
    }
}

// x_sorted[n] = x[perm[n]].  Every read fetches a whole 128-byte line for 4d bytes of it, and that line traffic (2.1 GB
// for 2^24 points) is what the kernel waits for: more loads in flight per lane, non-temporal loads or doing the reads
// inside the last scatter pass were all slower (measured).
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

struct SortSpace {
    size_t keys_a, keys_b, index, counts, totals, bytes;
};
SortSpace sort_space(int64_t N) {
    SortSpace s{};
    const size_t col = align256((size_t)N * 4);
    s.keys_a = 0;
    s.keys_b = col;
    s.index = 2 * col;
    s.counts = 3 * col;
    s.totals = s.counts + align256((size_t)kDigits * (size_t)tiles_of(N) * 4);
    s.bytes = s.totals + align256((size_t)kDigits * 4);
    return s;
}

template <int D>
int morton_sort(const float *x, int64_t N, int32_t *perm, float *x_sorted, char *ws, hipStream_t s) {
    const SortSpace sp = sort_space(N);
    uint32_t *keys_a = (uint32_t *)(ws + sp.keys_a), *keys_b = (uint32_t *)(ws + sp.keys_b);
    int32_t  *index = (int32_t *)(ws + sp.index);
    uint32_t *counts = (uint32_t *)(ws + sp.counts), *totals = (uint32_t *)(ws + sp.totals);
    const int64_t  tiles = tiles_of(N);
    const unsigned grid = (unsigned)tiles;
    constexpr int  bits = morton_bits(D) * D, passes = (bits + kDigitBits - 1) / kDigitBits;
    static_assert(passes == 3, "the buffers below are laid out for three passes");

    morton_keys_kernel<D><<<grid, kTileBlock, 0, s>>>(x, N, keys_a, counts, tiles);
    if (hipError_t e = hipGetLastError()) return cngp::record_hip_failure(e, "morton_keys_kernel");
    // pass 0: keys_a, identity -> keys_b, perm (as scratch); 1: keys_b, perm -> keys_a, index; 2: keys_a, index -> perm
    const uint32_t *k_in[3] = {keys_a, keys_b, keys_a};
    uint32_t       *k_out[3] = {keys_b, keys_a, nullptr};
    const int32_t  *i_in[3] = {nullptr, perm, index};
    int32_t        *i_out[3] = {perm, index, perm};
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = pass * kDigitBits;
        if (pass) {
            digit_count_kernel<<<grid, kTileBlock, 0, s>>>(k_in[pass], N, shift, counts, tiles);
            if (hipError_t e = hipGetLastError()) return cngp::record_hip_failure(e, "digit_count_kernel");
        }
        digit_row_scan_kernel<<<kDigits, kScanBlock, 0, s>>>(counts, tiles, totals);
        if (hipError_t e = hipGetLastError()) return cngp::record_hip_failure(e, "digit_row_scan_kernel");
        digit_scatter_kernel<<<grid, kTileBlock, 0, s>>>(k_in[pass], i_in[pass], N, shift, counts, tiles, totals, k_out[pass], i_out[pass]);
        if (hipError_t e = hipGetLastError()) return cngp::record_hip_failure(e, "digit_scatter_kernel");
    }
    if (x_sorted) {
        gather_points_kernel<D><<<(unsigned)((N + kSortBlock - 1) / kSortBlock), kSortBlock, 0, s>>>(x, perm, N, x_sorted);
        if (hipError_t e = hipGetLastError()) return cngp::record_hip_failure(e, "gather_points_kernel");
    }
    return CNGP_OK;
}

}  // namespace

extern "C" {

size_t cngp_morton_sort_workspace_bytes(int32_t d, int64_t N) {
    if (d < 2 || d > 4 || N <= 0 || N > 0x7fffffffLL) return 0;
    return sort_space(N).bytes;
}

int cngp_morton_sort(int32_t d, const float *x, int64_t N, int32_t *perm, float *x_sorted,
                     void *workspace, size_t workspace_bytes, void *stream) {
    if (d < 2 || d > 4) return CNGP_ERR_INVALID;
    if (N < 0 || N > 0x7fffffffLL) return CNGP_ERR_INVALID;
    if (N == 0) return CNGP_OK;
    if (!x || !perm) return CNGP_ERR_NULL;
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < sort_space(N).bytes) return CNGP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    return d == 3 ? morton_sort<3>(x, N, perm, x_sorted, (char *)workspace, s)
         : d == 4 ? morton_sort<4>(x, N, perm, x_sorted, (char *)workspace, s)
                  : morton_sort<2>(x, N, perm, x_sorted, (char *)workspace, s);
}

}  // extern "C"

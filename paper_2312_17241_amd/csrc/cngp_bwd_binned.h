// Backward pass of the hashed levels with the corner references BINNED by table slice first.
//
// The LDS-sliced backward pass (cngp_bwd_sliced.h) lets every slice's workgroup scan all points and
// keep the references that fall into its slice: cheap while a level has a few dozen slices, but the
// scan is repeated per slice.  Here the references are partitioned once:
//   1. count    per (level, chunk of points): how many references go to each slice of the feature
//               table (by hash) and of the confidence table (by hash2); histogram in LDS
//   2. offsets  exclusive prefix sums: where every (chunk, slice) writes inside the level's record array
//   3. scatter  the same walk again, every reference written as a 4-byte record  point index * 2^d + corner
//               to its slice's bin, positions handed out by LDS counters that start at the offsets
//   4. drain    a workgroup owns a slice as fp64 accumulators in LDS, as in the sliced variant, but reads
//               only its own bin, coalesced, one record per lane: the lane re-derives the two hashed rows and
//               weight * dL/dy of its record from the point (some thirty instructions per record, against 12
//               more bytes written and read per record if the record carried them: the scatter is bound by
//               its writes); record loads run two batches ahead, the gathers the records ask for (softmax
//               row / feature row) one batch ahead of the LDS atomics that consume them
// Per reference this replaces the replicated hashing and the ring-buffer emission by one 4-byte write
// and one 4-byte read per table, which is the better trade from a few dozen slices per level upwards and the
// only workable one for tables of thousands of slices.
#pragma once
#include "cngp_bwd_sliced.h"

namespace cngp {

// Count and scatter run one workgroup per chunk of points.  With a single wavefront (the default block size)
// the records a chunk adds to a bin follow the order of the points, so the drain's gathers of a batch of
// records (the points and their upstream gradients) fall into a few cache lines instead of one line per
// record; the host launches 256 lanes instead when there are many bins.
constexpr int kBinBlock = 64;

// A binned corner reference: point index * 2^d + corner (the host keeps N * 2^d below 2^31 per pass).
using BinRecord = uint32_t;
constexpr size_t kRecordBytes = sizeof(BinRecord);

struct BinParams {
    int32_t  level0, nlevels;             // the hashed levels
    uint32_t rows_f_log2, slices_f;       // feature-gradient slices per level
    uint32_t rows_c_log2, slices_c;       // logit-gradient slices per level; slices_c = 0 when N_p = 1
    uint32_t chunks, chunk_pts;           // point chunks of count / scatter
    uint32_t cap;                         // records per level and role: N * 2^d
    int32_t  dense_bins;                  // 1: the pre-reduced coarse levels are binned too, by slice of their vertex grid
};
// slices_f = 0: no bins by feature-table slice.  That is the case of a small feature table (the paper's
// N_f = 2^6 .. 2^11), whose whole level sits in LDS beside a slice of the confidence table: the workgroups
// that drain the confidence-table bins then accumulate both gradients in one pass (drain_both).

// Bins of a pre-reduced level: slices of kDenseSliceVerts vertices of its dense grid; every level is given
// kGridBins of them (the largest grid that is pre-reduced has that many).
constexpr uint32_t kGridBins = 32;

// Bin of a vertex; the clamp only matters for coordinates outside [0,1]^d, which are invalid input but must not fault.
__device__ __forceinline__ uint32_t grid_bin(const uint32_t v) {
    const uint32_t s = v / kDenseSliceVerts;
    return s < kGridBins ? s : kGridBins - 1u;
}

// Vertex numbers (dimension 0 fastest) of the 2^d corners of the cell x lies in, on a grid of `side` vertices per axis.
template <int D>
__device__ __forceinline__ void corner_vertices(const float (&xp)[D], const float res, const uint32_t side, uint32_t (&v)[1 << D]) {
    uint32_t base = 0, stride = 1, step[D];
    {
#pragma clang fp contract(off)
#pragma unroll
        for (int i = 0; i < D; ++i) {
            const float pos = xp[i] * res;                  // one rounded fp32 multiply
            base += (uint32_t)floorf(pos) * stride;
            step[i] = stride;
            stride *= side;
        }
    }
#pragma unroll
    for (int c = 0; c < (1 << D); ++c) {
        uint32_t t = base;
#pragma unroll
        for (int i = 0; i < D; ++i) t += ((c >> i) & 1) ? step[i] : 0u;
        v[c] = t;
    }
}

// A corner whose interpolation weight is exactly zero (the point lies on a face of its cell: clipped samples
// do) adds exactly nothing to either gradient, so it is never binned.  The weight is the product the drain
// itself forms (no factor below 2^-24, so the product of up to four cannot underflow to zero).
template <int D>
__device__ __forceinline__ float corner_weight(const float (&xp)[D], const float res, const int c) {
#pragma clang fp contract(off)
    float wt = 1.0f;
#pragma unroll
    for (int j = 0; j < D; ++j) {
        const float pos = xp[j] * res;                      // one rounded fp32 multiply
        const float w = pos - floorf(pos);
        wt *= ((c >> j) & 1) ? w : 1.0f - w;
    }
    return wt;
}

// Slice of the feature table (role 0) / confidence table (role 1) a corner's hashes select.
template <int D>
__device__ __forceinline__ void corner_rows(const Cell<D> &cell, const Params &p, const int c, uint32_t &h1, uint32_t &h2) {
    h1 = cell.hash1(c) & p.row_mask;
    h2 = cell.hash2(c) & p.c_mask;
}

// Workgroups [0, nlevels * chunks) count the hashed levels; with dense_bins the next level0 * chunks ones
// count the pre-reduced levels 0 .. level0 - 1 by slice of their vertex grid.
template <int D>
__device__ __forceinline__ void bin_count_block(
    const Params &p, const BinParams &bp, const DenseLevels &dl, const float *__restrict__ x, const int64_t N,
    uint32_t *__restrict__ cntF, uint32_t *__restrict__ cntC, uint32_t *__restrict__ cntG, const uint32_t hist_replicas,
    const uint32_t block)
{
    extern __shared__ uint32_t hist[];                      // [hist_replicas][max(slices_f + slices_c, kGridBins)]
    const uint32_t li = block / bp.chunks, chunk = block % bp.chunks;
    const int64_t n0 = (int64_t)chunk * bp.chunk_pts;
    const int64_t n1 = (n0 + bp.chunk_pts < N) ? n0 + bp.chunk_pts : N;
    if (li >= (uint32_t)bp.nlevels) {                       // a pre-reduced level
        const uint32_t ld = li - (uint32_t)bp.nlevels;
        uint32_t *own = hist + (threadIdx.x % hist_replicas) * kGridBins;
        for (uint32_t i = threadIdx.x; i < kGridBins * hist_replicas; i += blockDim.x) hist[i] = 0u;
        __syncthreads();
        for (int64_t n = n0 + threadIdx.x; n < n1; n += blockDim.x) {
            float xp[D];
#pragma unroll
            for (int j = 0; j < D; ++j) xp[j] = x[n * D + j];
            uint32_t v[1 << D];
            corner_vertices<D>(xp, (float)p.N_l[ld], dl.side[ld], v);
#pragma unroll
            for (int c = 0; c < (1 << D); ++c)
                if (corner_weight<D>(xp, (float)p.N_l[ld], c) != 0.0f) atomicAdd(&own[grid_bin(v[c])], 1u);
        }
        __syncthreads();
        uint32_t *rowG = cntG + ((size_t)ld * bp.chunks + chunk) * kGridBins;
        for (uint32_t s = threadIdx.x; s < kGridBins; s += blockDim.x) {
            uint32_t total = 0;
            for (uint32_t r = 0; r < hist_replicas; ++r) total += hist[r * kGridBins + s];
            rowG[s] = total;
        }
        return;
    }
    const int      l = bp.level0 + (int)li;
    const uint32_t bins = bp.slices_f + bp.slices_c;
    // `reps` copies of the histogram, picked by lane: 64 lanes adding to a handful of counters would
    // otherwise serialise on the same LDS addresses (the atomics were the whole cost of this kernel)
    const uint32_t reps = hist_replicas;
    uint32_t *mine = hist + (threadIdx.x % reps) * bins;
    for (uint32_t i = threadIdx.x; i < bins * reps; i += blockDim.x) hist[i] = 0u;
    __syncthreads();
    for (int64_t n = n0 + threadIdx.x; n < n1; n += blockDim.x) {
        float xp[D];
#pragma unroll
        for (int j = 0; j < D; ++j) xp[j] = x[n * D + j];
        Cell<D> cell;
        cell.locate(xp, p.N_l[l]);
#pragma unroll
        for (int c = 0; c < (1 << D); ++c) {
            if (cell.weight(c) == 0.0f) continue;
            uint32_t h1, h2;
            corner_rows<D>(cell, p, c, h1, h2);
            if (bp.slices_f) atomicAdd(&mine[h1 >> bp.rows_f_log2], 1u);
            if (bp.slices_c) atomicAdd(&mine[bp.slices_f + (h2 >> bp.rows_c_log2)], 1u);
        }
    }
    __syncthreads();
    uint32_t *rowF = cntF + ((size_t)li * bp.chunks + chunk) * bp.slices_f;
    uint32_t *rowC = cntC + ((size_t)li * bp.chunks + chunk) * bp.slices_c;
    for (uint32_t s = threadIdx.x; s < bins; s += blockDim.x) {
        uint32_t total = 0;
        for (uint32_t r = 0; r < reps; ++r) total += hist[r * bins + s];
        if (s < bp.slices_f) rowF[s] = total;
        else rowC[s - bp.slices_f] = total;
    }
}

// The count shares its launch with the preparation of cngp_bwd_sliced.h (clearing, softmax table, level-major
// dL/dy): neither needs the other's results, one is bound by hashing and LDS atomics, the other by memory.
// Workgroups [0, count_blocks) count, the rest prepare (alternating the two kinds over the grid was slower).
template <int D, int NP, typename PairT>
__global__ __launch_bounds__(kBlock) void bwd_prep_count_kernel(
    const PrepArgs a, const Params p, const BinParams bp, const DenseLevels dl, const float *__restrict__ x,
    uint32_t *__restrict__ cntF, uint32_t *__restrict__ cntC, uint32_t *__restrict__ cntG, const uint32_t hist_replicas,
    const uint32_t count_blocks)
{
    if (blockIdx.x < count_blocks) bin_count_block<D>(p, bp, dl, x, a.N, cntF, cntC, cntG, hist_replicas, blockIdx.x);
    else bwd_prep_block<NP, PairT>(a, blockIdx.x - count_blocks);
}

constexpr int kOffsetsBlock = 256;

// One workgroup per (level, role).  In place: cnt[chunk][slice] becomes the position, inside the level's
// record array, of the first record that chunk writes to that slice; base[slice] = start of the slice's
// bin, base[slices] = number of records of the level.  `lds_words` words of dynamic LDS hold the whole
// matrix when it fits (the scans then run in LDS; through memory they are chains of dependent loads).
// Threads form a [segment][slice] array: a thread owns one slice's counts of a run of chunks.
__global__ __launch_bounds__(kOffsetsBlock) void bin_offsets_kernel(
    const BinParams bp, uint32_t *__restrict__ cntF, uint32_t *__restrict__ cntC, uint32_t *__restrict__ cntG,
    uint32_t *__restrict__ baseF, uint32_t *__restrict__ baseC, uint32_t *__restrict__ baseG, const uint32_t lds_words)
{
    extern __shared__ __align__(16) uint32_t mat[];
    __shared__ uint32_t part[kOffsetsBlock];                // [segment][slice lane]: sum of the thread's run
    __shared__ uint32_t carry;                              // records of the slices handled in earlier rounds
    // workgroups 0 .. 2 nlevels - 1: (hashed level, table); then one per pre-reduced level
    const bool     dense = blockIdx.x >= 2u * (uint32_t)bp.nlevels;
    const uint32_t li = dense ? blockIdx.x - 2u * (uint32_t)bp.nlevels : blockIdx.x >> 1, role = blockIdx.x & 1u;
    const uint32_t slices = dense ? kGridBins : role ? bp.slices_c : bp.slices_f;
    if (slices == 0) return;
    uint32_t *gcnt = (dense ? cntG : role ? cntC : cntF) + (size_t)li * bp.chunks * slices;
    uint32_t *base = (dense ? baseG : role ? baseC : baseF) + (size_t)li * (slices + 1);
    const uint32_t elems = bp.chunks * slices;
    const bool     in_lds = elems <= lds_words;
    uint32_t      *cnt = in_lds ? mat : gcnt;
    // (the copies in and out move 16 bytes per lane and step: word by word they were a chain of memory latencies that
    // took longer than the scans)
    const bool wide = in_lds && elems % 4u == 0 && (reinterpret_cast<uintptr_t>(gcnt) & 15u) == 0;
    if (wide)
        for (uint32_t i = threadIdx.x; i < elems / 4u; i += kOffsetsBlock)
            reinterpret_cast<uint4 *>(mat)[i] = reinterpret_cast<const uint4 *>(gcnt)[i];
    else if (in_lds)
        for (uint32_t i = threadIdx.x; i < elems; i += kOffsetsBlock) mat[i] = gcnt[i];
    if (threadIdx.x == 0) carry = 0u;
    __syncthreads();
    const uint32_t width = slices < (uint32_t)kOffsetsBlock ? slices : (uint32_t)kOffsetsBlock;   // slices per round
    const uint32_t segs = kOffsetsBlock / width;                                                // width is a power of two
    const uint32_t lane_s = threadIdx.x % width, seg = threadIdx.x / width;
    const uint32_t per = (bp.chunks + segs - 1) / segs;
    const uint32_t c0 = seg * per, c1 = (c0 + per < bp.chunks) ? c0 + per : bp.chunks;
    for (uint32_t s_round = 0; s_round < slices; s_round += width) {
        const uint32_t s = s_round + lane_s;                // < slices: both are powers of two
        uint32_t sum = 0;
        for (uint32_t ch = c0; ch < c1; ++ch) sum += cnt[(size_t)ch * slices + s];
        part[threadIdx.x] = sum;
        __syncthreads();
        uint32_t before = 0, total = 0;                     // this slice: records of earlier segments, of all
        for (uint32_t g = 0; g < segs; ++g) {
            const uint32_t v = part[g * width + lane_s];
            before += g < seg ? v : 0u;
            total += v;
        }
        __syncthreads();
        if (seg == 0) part[lane_s] = total;
        __syncthreads();
        uint32_t start = carry;                             // exclusive prefix of the totals over the slices
        for (uint32_t j = 0; j < lane_s; ++j) start += part[j];
        if (seg == 0) base[s] = start;
        uint32_t run = start + before;
        for (uint32_t ch = c0; ch < c1; ++ch) {
            const uint32_t v = cnt[(size_t)ch * slices + s];
            cnt[(size_t)ch * slices + s] = run;
            run += v;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t all = carry;
            for (uint32_t j = 0; j < width; ++j) all += part[j];
            carry = all;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) base[slices] = carry;
    if (in_lds) {
        __syncthreads();
        if (wide)
            for (uint32_t i = threadIdx.x; i < elems / 4u; i += kOffsetsBlock)
                reinterpret_cast<uint4 *>(gcnt)[i] = reinterpret_cast<const uint4 *>(mat)[i];
        else
            for (uint32_t i = threadIdx.x; i < elems; i += kOffsetsBlock) gcnt[i] = mat[i];
    }
}

// Scatter, one workgroup per (level, chunk).
template <int D>
__global__ __launch_bounds__(256) void bin_scatter_kernel(
    const Params p, const BinParams bp, const DenseLevels dl, const float *__restrict__ x, const int64_t N,
    const uint32_t *__restrict__ cntF, const uint32_t *__restrict__ cntC, const uint32_t *__restrict__ cntG,
    BinRecord *__restrict__ recF, BinRecord *__restrict__ recC, BinRecord *__restrict__ recG)
{
    extern __shared__ uint32_t cursor[];                    // [max(slices_f + slices_c, kGridBins)]
    const uint32_t li = blockIdx.x / bp.chunks, chunk = blockIdx.x % bp.chunks;
    if (li >= (uint32_t)bp.nlevels) {                       // a pre-reduced level, binned by slice of its vertex grid
        const uint32_t ld = li - (uint32_t)bp.nlevels;
        const uint32_t *rowG = cntG + ((size_t)ld * bp.chunks + chunk) * kGridBins;
        for (uint32_t s = threadIdx.x; s < kGridBins; s += blockDim.x) cursor[s] = rowG[s];
        __syncthreads();
        BinRecord *outG = recG + (size_t)ld * bp.cap;
        const int64_t m0 = (int64_t)chunk * bp.chunk_pts;
        const int64_t m1 = (m0 + bp.chunk_pts < N) ? m0 + bp.chunk_pts : N;
        for (int64_t n = m0 + threadIdx.x; n < m1; n += blockDim.x) {
            float xp[D];
#pragma unroll
            for (int j = 0; j < D; ++j) xp[j] = x[n * D + j];
            uint32_t v[1 << D];
            corner_vertices<D>(xp, (float)p.N_l[ld], dl.side[ld], v);
#pragma unroll
            for (int c = 0; c < (1 << D); ++c) {
                if (corner_weight<D>(xp, (float)p.N_l[ld], c) == 0.0f) continue;
                const uint32_t pos = atomicAdd(&cursor[grid_bin(v[c])], 1u);
                outG[pos] = ((uint32_t)n << D) | (uint32_t)c;
            }
        }
        return;
    }
    const int      l = bp.level0 + (int)li;
    const uint32_t *rowF = cntF + ((size_t)li * bp.chunks + chunk) * bp.slices_f;
    for (uint32_t s = threadIdx.x; s < bp.slices_f; s += blockDim.x) cursor[s] = rowF[s];
    if (bp.slices_c) {
        const uint32_t *rowC = cntC + ((size_t)li * bp.chunks + chunk) * bp.slices_c;
        for (uint32_t s = threadIdx.x; s < bp.slices_c; s += blockDim.x) cursor[bp.slices_f + s] = rowC[s];
    }
    __syncthreads();
    BinRecord *outF = recF + (size_t)li * bp.cap;
    BinRecord *outC = recC + (size_t)li * bp.cap;
    const int64_t  n0 = (int64_t)chunk * bp.chunk_pts;
    const int64_t  n1 = (n0 + bp.chunk_pts < N) ? n0 + bp.chunk_pts : N;
    for (int64_t n = n0 + threadIdx.x; n < n1; n += blockDim.x) {
        float xp[D];
#pragma unroll
        for (int j = 0; j < D; ++j) xp[j] = x[n * D + j];
        Cell<D> cell;
        cell.locate(xp, p.N_l[l]);
#pragma unroll
        for (int c = 0; c < (1 << D); ++c) {
            if (cell.weight(c) == 0.0f) continue;
            uint32_t h1, h2;
            corner_rows<D>(cell, p, c, h1, h2);
            const uint32_t ref = ((uint32_t)n << D) | (uint32_t)c;
            if (bp.slices_f) {
                const uint32_t posF = atomicAdd(&cursor[h1 >> bp.rows_f_log2], 1u);
                outF[posF] = ref;
            }
            if (bp.slices_c) {
                const uint32_t posC = atomicAdd(&cursor[bp.slices_f + (h2 >> bp.rows_c_log2)], 1u);
                outC[posC] = ref;
            }
        }
    }
}

// ------------------------------------------------------------------ drain
// Value of lane `u` of this lane's group of NP lanes.  Groups of 16 (a DPP row), 4 and 2 (inside a quad): one VALU move;
// groups of 8 (half a row): two, each writing the two banks of four lanes of its half (a cross-lane read through the
// LDS crossbar instead cost the drain a fifth of its time at N_p = 8).
template <int NP, int U>
__device__ __forceinline__ uint32_t group_bcast(const uint32_t v) {
    if constexpr (NP == 16) {                                             // row_newbcast:U
        return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x150 + U, 0xF, 0xF, true);
    } else if constexpr (NP == 8) {                                       // row_newbcast:U into banks 0-1, row_newbcast:8+U into banks 2-3
        const int lo = __builtin_amdgcn_update_dpp(0, (int)v, 0x150 + U, 0xF, 0x3, false);
        return (uint32_t)__builtin_amdgcn_update_dpp(lo, (int)v, 0x150 + 8 + U, 0xF, 0xC, false);
    } else if constexpr (NP == 4) {                                       // quad_perm:[U,U,U,U]
        return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, U * 0x55, 0xF, 0xF, true);
    } else if constexpr (NP == 2) {                                       // quad_perm:[U,U,U+2,U+2]
        return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, U * 0x05 + (U + 2) * 0x50, 0xF, 0xF, true);
    } else if constexpr (NP == 1) {
        return v;
    } else {
        return (uint32_t)__shfl((int)v, (int)((threadIdx.x & 63u & ~(uint32_t)(NP - 1)) + U), 64);
    }
}

__device__ __forceinline__ float2 pair_to_float2(const float2 v) { return v; }
__device__ __forceinline__ float2 pair_to_float2(const uint32_t v) {
    return __half22float2(*reinterpret_cast<const __half2 *>(&v));
}

// Step U of a batch: every group reads the key its lane U holds and issues the gather it asks for ...
template <int NP, int U, typename T, typename Load>
__device__ __forceinline__ void gather_steps(const uint4 &r, T (&g)[NP], Load load) {
    if constexpr (U < NP) {
        g[U] = load(group_bcast<NP, U>(r.x));
        gather_steps<NP, U + 1>(r, g, load);
    }
}
// ... and, a batch later, accumulates it with what the gather brought.  BOTH: the accumulation wants the
// gather's offset as well (it is the second accumulator row).
template <int NP, int U, bool BOTH, typename T, typename Accum>
__device__ __forceinline__ void accum_steps(const uint4 &r, const T (&g)[NP], Accum accum) {
    if constexpr (U < NP) {
        const float2 gy = make_float2(__uint_as_float(group_bcast<NP, U>(r.y)), __uint_as_float(group_bcast<NP, U>(r.z)));
        if constexpr (BOTH) accum(group_bcast<NP, U>(r.w), gy, g[U], group_bcast<NP, U>(r.x));
        else accum(group_bcast<NP, U>(r.w), gy, g[U]);
        accum_steps<NP, U + 1, BOTH>(r, g, accum);
    }
}

// Records [beg, end) of one bin.  A wavefront takes batches of 64 records round-robin with the other
// wavefronts of the workgroup; EVERY LANE LOADS ONE RECORD of a batch (a 16-byte load each: loading a
// record with all NP lanes that work on it costs NP times the return bandwidth of the memory pipeline,
// which then bounds the kernel), and the NP lanes of a group pass their NP records around: in step u the
// group works on the record its lane u holds.
//
// Three-stage pipeline over three register buffers, unrolled so that no buffer is ever copied: in the
// step that accumulates batch i, the gathers of batch i + 1 and the record load of batch i + 2 are issued
// -- the record first, so that waiting for it next step leaves the younger gathers in flight.  Loads
// are never predicated: a position past `end` re-reads the bin's last record and its gather result is
// replaced by zero, so it adds nothing.
// BOTH (records of a confidence-table bin, both gradients accumulated): the gather reads the row INSIDE the
// slice (the softmax row of the record's own confidence row), the accumulator row is the other table's.
// ACC: doubles per candidate of an accumulator row (2 where both features of a row sit side by side).
// BY_FEAT: the bin belongs to a slice of the feature table (rows by hash), else of the confidence table (hash2).
template <int D, int NP, typename T, bool BOTH, int ACC, bool BY_FEAT, typename IoT, typename Load, typename Accum>
__device__ __forceinline__ void drain_records(const Params &p, const BinRecord *__restrict__ rec, const uint32_t beg, const uint32_t end,
                                              const float *__restrict__ x, const IoT *__restrict__ dy_l, const float res,
                                              const uint32_t rows_log2, Load load, Accum accum)
{
    const uint32_t row_lo_mask = (1u << rows_log2) - 1u;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t stride = kSlicedWaves * 64u;
    uint32_t b = beg + wave * 64u;
    if (b >= end) return;
    const uint32_t last = end - 1u;
    using Pair = typename std::conditional<sizeof(IoT) == 2, uint32_t, float2>::type;   // dL/dy of a level as stored
    // Four stages, a batch apart, over four register buffers (unrolled four times, so no buffer is copied):
    //   A  this lane's record of a batch                          (coalesced 4-byte load)
    //   B  the record's point and upstream gradient               (gathers by point index)
    //   C  the record's two table rows and weight * dL/dy from those, and the gathers the rows ask for
    //   D  accumulate
    // Each stage consumes what the stage before it loaded one step earlier; within a step the loads are
    // issued A, B, C, so that a wait for an older stage's data leaves the younger loads in flight.
    BinRecord Q[4];
    float X[4][D];
    Pair  Y[4];
    uint4 R[4];                                              // gather offset, weight * dL/dy (two floats), LDS offset
    T     G[4][NP];
    auto stage_a = [&](const uint32_t base, BinRecord &q) {
        const uint32_t i = base + lane;
        // streamed once: a non-temporal load keeps it out of the way of the rows that are gathered again and again
        q = __builtin_nontemporal_load(rec + (i < last ? i : last));
    };
    auto stage_b = [&](const BinRecord &q, float (&xp)[D], Pair &y) {
        const uint32_t n = q >> D;
#pragma unroll
        for (int j = 0; j < D; ++j) xp[j] = x[(size_t)n * D + j];
        y = reinterpret_cast<const Pair *>(dy_l)[n];
    };
    auto stage_c = [&](const uint32_t base, const BinRecord &q, const float (&xp)[D], const Pair &y, uint4 &r, T (&g)[NP]) {
        const uint32_t c = q & ((1u << D) - 1u);
        float    wt = (base + lane < end) ? 1.0f : 0.0f;     // beyond the bin: contributes nothing
        uint32_t h1 = 0, h2 = 0;                             // Eq. 3 for this corner, as in Cell<D>
        {
#pragma clang fp contract(off)
#pragma unroll
            for (int j = 0; j < D; ++j) {
                const float    pos = xp[j] * res;            // one rounded fp32 multiply
                const float    fl = floorf(pos);
                const float    w = pos - fl;
                const uint32_t up = (c >> j) & 1u;
                wt *= up ? w : 1.0f - w;
                const uint32_t v = (uint32_t)fl + up;
                h1 ^= v * kPi[j];
                h2 ^= v * kPi2[j];
            }
        }
        h1 &= p.row_mask;
        h2 &= p.c_mask;
        const float2 gy = pair_to_float2(y);
        // once per record: byte offset of the row the gather reads (candidate 0), and byte offset of the
        // accumulator row in LDS; the lanes of the group add their candidate's share
        const uint32_t inside = (BY_FEAT ? h1 : h2) & row_lo_mask, other = BY_FEAT ? h2 : h1;
        r = make_uint4((BOTH ? inside : other) * (uint32_t)(NP * sizeof(T)), __float_as_uint(wt * gy.x),
                       __float_as_uint(wt * gy.y), (BOTH ? other : inside) * (uint32_t)(ACC * NP * sizeof(double)));
        gather_steps<NP, 0>(r, g, load);
    };
    // prologue: batches b, b + stride, b + 2 stride enter the pipeline
    stage_a(b, Q[0]);
    stage_a(b + stride, Q[1]);
    stage_a(b + 2 * stride, Q[2]);
    stage_b(Q[0], X[0], Y[0]);
    stage_b(Q[1], X[1], Y[1]);
    stage_c(b, Q[0], X[0], Y[0], R[0], G[0]);
#define CNGP_DRAIN_STEP(P0, P1, P2, P3)                                                  \
        stage_a(b + 3 * stride, Q[P3]);                                                  \
        stage_b(Q[P2], X[P2], Y[P2]);                                                    \
        stage_c(b + stride, Q[P1], X[P1], Y[P1], R[P1], G[P1]);                          \
        accum_steps<NP, 0, BOTH>(R[P0], G[P0], accum);                                         \
        b += stride;                                                                     \
        if (b >= end) break;
    for (;;) {
        CNGP_DRAIN_STEP(0, 1, 2, 3)
        CNGP_DRAIN_STEP(1, 2, 3, 0)
        CNGP_DRAIN_STEP(2, 3, 0, 1)
        CNGP_DRAIN_STEP(3, 0, 1, 2)
    }
#undef CNGP_DRAIN_STEP
}

// The records of (level index li, slice, sub) of one role: sub-range `sub` of `subs` equal parts of the bin.
__device__ __forceinline__ void bin_range(const uint32_t *__restrict__ base, const uint32_t slices, const uint32_t li,
                                          const uint32_t slice, const uint32_t sub, const uint32_t subs,
                                          uint32_t &beg, uint32_t &end) {
    const uint32_t *b = base + (size_t)li * (slices + 1);
    const uint32_t  b0 = b[slice], n = b[slice + 1] - b0;
    beg = b0 + (uint32_t)(((uint64_t)n * sub) / subs);
    end = b0 + (uint32_t)(((uint64_t)n * (sub + 1)) / subs);
}

// ------------------------------------------------------------------ vertex-grid sums from binned references
// G[l][v][f] = sum over the corner references to vertex v of pre-reduced level l of weight * dL/dy (what
// bwd_vertex_grid computes by scanning all points once per slice of the grid).  A workgroup owns the slice
// of one level's grid as fp64 accumulators in LDS and part `sub` of the slice's bin; every lane works on
// a record of its own: no gathers of table rows here, two LDS atomics per reference.
struct GridDrainPlan {
    uint32_t first[kMaxDense + 1];        // first workgroup of each pre-reduced level; [count] = grid size
    uint32_t subs[kMaxDense];             // workgroups per slice of the level's grid
};

template <int D, typename IoT>
__global__ __launch_bounds__(kSlicedBlock) void bin_grid_drain_kernel(
    const Params p, const DenseLevels dl, const GridDrainPlan gp, const float *__restrict__ x,
    const IoT *__restrict__ dyT, const int64_t N, const BinRecord *__restrict__ recG,
    const uint32_t *__restrict__ baseG, const uint32_t cap, float *__restrict__ G)
{
    extern __shared__ __align__(16) unsigned char smem[];
    double *acc = reinterpret_cast<double *>(smem);
    int ld = 0;
    while (ld < dl.count - 1 && blockIdx.x >= gp.first[ld + 1]) ++ld;
    const uint32_t wg = blockIdx.x - gp.first[ld], subs = gp.subs[ld];
    const uint32_t slice = wg / subs, sub = wg % subs;
    const uint32_t first = slice * kDenseSliceVerts;
    const uint32_t count = dl.verts[ld] - first < kDenseSliceVerts ? dl.verts[ld] - first : kDenseSliceVerts;
    for (uint32_t i = threadIdx.x; i < count * 2; i += kSlicedBlock) acc[i] = 0.0;
    __syncthreads();

    uint32_t beg, end;
    bin_range(baseG, kGridBins, (uint32_t)ld, slice, sub, subs, beg, end);
    if (beg < end) {
        using Pair = typename std::conditional<sizeof(IoT) == 2, uint32_t, float2>::type;
        const BinRecord *rec = recG + (size_t)ld * cap;
        const uint32_t side = dl.side[ld];
        const Pair    *dy_l = reinterpret_cast<const Pair *>(dyT + (size_t)ld * N * 2);
        const float    res = (float)p.N_l[ld];
        const uint32_t last = end - 1u;
        struct Point { float xp[D]; Pair y; };
        auto record = [&](const uint32_t i) { return rec[i < last ? i : last]; };
        auto point = [&](const BinRecord q) {
            Point pt;
            const uint32_t n = q >> D;
#pragma unroll
            for (int j = 0; j < D; ++j) pt.xp[j] = x[(size_t)n * D + j];
            pt.y = dy_l[n];
            return pt;
        };
        // record loads run two steps ahead, the point and gradient they name one step ahead
        uint32_t i = beg + threadIdx.x;
        BinRecord q0 = record(i), q1 = record(i + kSlicedBlock);
        Point p0 = point(q0);
        for (; i < end; i += kSlicedBlock) {
            const BinRecord q2 = record(i + 2 * kSlicedBlock);
            const Point p1 = point(q1);
            const uint32_t c = q0 & ((1u << D) - 1u);
            float    wt = 1.0f;
            uint32_t v = 0, stride = 1;                     // the corner's vertex number, as corner_vertices gives it
            {
#pragma clang fp contract(off)
#pragma unroll
                for (int j = 0; j < D; ++j) {
                    const float    pos = p0.xp[j] * res;    // one rounded fp32 multiply
                    const float    fl = floorf(pos);
                    const float    w = pos - fl;
                    const uint32_t up = (c >> j) & 1u;
                    wt *= up ? w : 1.0f - w;
                    v += ((uint32_t)fl + up) * stride;
                    stride *= side;
                }
            }
            const uint32_t at = 2u * (v % kDenseSliceVerts);    // inside the slice whatever the point was
            const float2 g = pair_to_float2(p0.y);
            atomicAdd(acc + at, (double)(wt * g.x));
            atomicAdd(acc + at + 1, (double)(wt * g.y));
            q0 = q1; q1 = q2; p0 = p1;
        }
    }
    __syncthreads();
    float *out = G + ((size_t)dl.g_off[ld] + first) * 2;
    for (uint32_t i = threadIdx.x; i < count * 2; i += kSlicedBlock) {
        const float v = (float)acc[i];
        if (subs == 1) out[i] = v;
        else if (v != 0.0f) atomic_add(out + i, v);
    }
}

// sp: rows_log2, slices, chunks (= drain workgroups per bin), store_direct, level0, nlevels as in the sliced variant.
template <int D, int NP, typename IoT>
__device__ __forceinline__ void drain_feat(const Params &p, const SliceParams &sp, const uint32_t wg, unsigned char *smem,
                                           const float *__restrict__ x, const IoT *__restrict__ dyT, const int64_t N,
                                           const float *__restrict__ sigma, const BinRecord *__restrict__ recF,
                                           const uint32_t *__restrict__ baseF, const uint32_t cap, float *__restrict__ gD_f)
{
    const uint32_t rows = 1u << sp.rows_log2, plane = rows * NP;
    double *acc = reinterpret_cast<double *>(smem);
    const SliceCoord co = slice_coord(sp, wg);
    if (co.index < 0) return;
    for (uint32_t i = threadIdx.x; i < plane * 2; i += kSlicedBlock) acc[i] = 0.0;
    __syncthreads();
    // accumulators [row][f][k]: the NP lanes of a record add to NP consecutive doubles, and feature 1 sits a constant
    // NP doubles behind feature 0 (an immediate offset of the LDS instruction)
    const char    *sig_l = reinterpret_cast<const char *>(sigma + (size_t)co.level * p.N_c * NP);   // uniform: scalar base of the gathers
    const uint32_t k = (threadIdx.x & 63) % NP, k4 = k * (uint32_t)sizeof(float);
    char          *acc_k = reinterpret_cast<char *>(acc + k);
    auto load = [&](const uint32_t off) -> float {           // off: byte offset of the softmax row
        return NP == 1 ? 1.0f : *reinterpret_cast<const float *>(sig_l + (off + k4));
    };
    auto accum = [&](const uint32_t off, const float2 g, const float s) {      // off: byte offset of the accumulator row
        double *a = reinterpret_cast<double *>(acc_k + off);
        atomicAdd(a, (double)(s * g.x));
        atomicAdd(a + NP, (double)(s * g.y));
    };
    uint32_t beg, end;
    bin_range(baseF, sp.slices, (uint32_t)co.index, co.slice, co.chunk, sp.chunks, beg, end);
    drain_records<D, NP, float, false, 2, true>(p, recF + (size_t)co.index * cap, beg, end, x, dyT + (size_t)co.level * N * 2,
                                          (float)p.N_l[co.level], sp.rows_log2, load, accum);
    __syncthreads();
    float *out = gD_f + (size_t)co.level * p.N_f * 2 + (size_t)co.slice * plane * 2;
    for (uint32_t i = threadIdx.x; i < plane * 2; i += kSlicedBlock) {     // i = (row * NP + k) * 2 + f
        const uint32_t e = i >> 1;
        const float v = (float)acc[(e / NP) * (2 * NP) + (i & 1u) * NP + (e % NP)];
        if (sp.store_direct) out[i] = v;
        else if (v != 0.0f) atomic_add(out + i, v);
    }
}

template <int D, int NP, typename FeatT, typename IoT>
__device__ __forceinline__ void drain_logit(const Params &p, const SliceParams &sp, const uint32_t wg, unsigned char *smem,
                                            const float *__restrict__ x, const IoT *__restrict__ dyT, const int64_t N,
                                            const FeatT *__restrict__ D_f, const float *__restrict__ sigma,
                                            const BinRecord *__restrict__ recC, const uint32_t *__restrict__ baseC,
                                            const uint32_t cap, float *__restrict__ gDhat_c)
{
    const uint32_t rows = 1u << sp.rows_log2;
    double *acc = reinterpret_cast<double *>(smem);
    const SliceCoord co = slice_coord(sp, wg);
    if (co.index < 0) return;
    for (uint32_t i = threadIdx.x; i < rows * NP; i += kSlicedBlock) acc[i] = 0.0;
    __syncthreads();
    const FeatT   *F_l = D_f + (size_t)co.level * p.N_f * 2;
    const uint32_t k = (threadIdx.x & 63) % NP;
    using Raw = typename RawPair<FeatT>::type;
    const char    *feat_l = reinterpret_cast<const char *>(F_l);          // uniform: scalar base of the gathers
    const uint32_t kb = k * (uint32_t)sizeof(Raw);                        // this lane's candidate
    char          *acc_k = reinterpret_cast<char *>(acc + k);
    auto load = [&](const uint32_t off) -> Raw { return *reinterpret_cast<const Raw *>(feat_l + (off + kb)); };
    auto accum = [&](const uint32_t off, const float2 g, const Raw raw) {
        const float2 feat = RawPair<FeatT>::to_float2(raw);
        atomicAdd(reinterpret_cast<double *>(acc_k + off), (double)fmaf(feat.x, g.x, feat.y * g.y));
    };
    uint32_t beg, end;
    bin_range(baseC, sp.slices, (uint32_t)co.index, co.slice, co.chunk, sp.chunks, beg, end);
    drain_records<D, NP, Raw, false, 1, false>(p, recC + (size_t)co.index * cap, beg, end, x, dyT + (size_t)co.level * N * 2,
                              (float)p.N_l[co.level], sp.rows_log2, load, accum);
    __syncthreads();
    // softmax Jacobian per row, then out to HBM; NP consecutive lanes hold one row
    const size_t row0 = (size_t)co.level * p.N_c + (size_t)co.slice * rows;
    const float *sig = sigma + row0 * NP;
    float       *out = gDhat_c + row0 * NP;
    for (uint32_t i = threadIdx.x; i < rows * NP; i += kSlicedBlock) {
        const double Q = acc[i];
        const double s = (double)sig[i];
        double dot = s * Q;
#pragma unroll
        for (int o = NP / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, NP);
        const float v = (float)(s * (Q - dot));
        if (sp.store_direct) out[i] = v;
        else if (v != 0.0f) atomic_add(out + i, v);
    }
}

// Small feature table: both gradients from the confidence-table bins in one pass.  LDS holds the slice of
// Q accumulators (as drain_logit), fp64 accumulators for the level's WHOLE feature gradient, and a copy of the
// level's feature codebook, so the only gather left per record is its softmax row -- from the 64 KB or so of
// rows of this slice instead of the whole table.  The feature gradient goes out with atomics (every
// workgroup of the level holds a share of it): the caller has cleared it.
template <int D, int NP, typename FeatT, typename IoT>
__device__ __forceinline__ void drain_both(const Params &p, const SliceParams &sp, const uint32_t wg, unsigned char *smem,
                                           const float *__restrict__ x, const IoT *__restrict__ dyT, const int64_t N,
                                           const FeatT *__restrict__ D_f, const float *__restrict__ sigma,
                                           const BinRecord *__restrict__ recC, const uint32_t *__restrict__ baseC,
                                           const uint32_t cap, float *__restrict__ gD_f, float *__restrict__ gDhat_c)
{
    using Raw = typename RawPair<FeatT>::type;
    const uint32_t rows = 1u << sp.rows_log2, plane = p.N_f;            // plane: feature entries of a level
    double *accQ = reinterpret_cast<double *>(smem);                    // [rows][NP]
    double *accF = accQ + (size_t)rows * NP;                            // [2][N_f]: feature 0 of every entry, then feature 1
    Raw    *feat = reinterpret_cast<Raw *>(accF + 2 * (size_t)plane);   // [N_f]
    const SliceCoord co = slice_coord(sp, wg);
    if (co.index < 0) return;
    const Raw *F_l = reinterpret_cast<const Raw *>(D_f + (size_t)co.level * p.N_f * 2);
    for (uint32_t i = threadIdx.x; i < rows * NP + 2 * plane; i += kSlicedBlock) accQ[i] = 0.0;
    for (uint32_t i = threadIdx.x; i < plane; i += kSlicedBlock) feat[i] = F_l[i];
    __syncthreads();
    const size_t   row0 = (size_t)co.level * p.N_c + (size_t)co.slice * rows;
    const uint32_t k = (threadIdx.x & 63) % NP;
    const char *sig_k = reinterpret_cast<const char *>(sigma + row0 * NP + k);          // this lane's candidate, this slice's rows
    char       *accF_k = reinterpret_cast<char *>(accF + k), *accQ_k = reinterpret_cast<char *>(accQ + k);
    const char *feat_k = reinterpret_cast<const char *>(feat + k);
    auto load = [&](const uint32_t off) -> float { return *reinterpret_cast<const float *>(sig_k + off); };
    // offF: byte offset of the feature row among fp64 accumulators (row * NP * 8); offS: of the confidence row
    // among floats (row * NP * 4)
    auto accum = [&](const uint32_t offF, const float2 g, const float s, const uint32_t offS) {
        const float2 f = RawPair<FeatT>::to_float2(*reinterpret_cast<const Raw *>(feat_k + offF / 8u * sizeof(Raw)));
        double *a = reinterpret_cast<double *>(accF_k + offF);
        atomicAdd(a, (double)(s * g.x));
        atomicAdd(a + plane, (double)(s * g.y));
        atomicAdd(reinterpret_cast<double *>(accQ_k + 2u * offS), (double)fmaf(f.x, g.x, f.y * g.y));
    };
    uint32_t beg, end;
    bin_range(baseC, sp.slices, (uint32_t)co.index, co.slice, co.chunk, sp.chunks, beg, end);
    drain_records<D, NP, float, true, 1, false>(p, recC + (size_t)co.index * cap, beg, end, x, dyT + (size_t)co.level * N * 2,
                                      (float)p.N_l[co.level], sp.rows_log2, load, accum);
    __syncthreads();
    float *outF = gD_f + (size_t)co.level * p.N_f * 2;
    for (uint32_t i = threadIdx.x; i < plane * 2; i += kSlicedBlock) {     // i = entry * 2 + f
        const float v = (float)accF[(i & 1u) * plane + (i >> 1)];
        if (v != 0.0f) atomic_add(outF + i, v);
    }
    const float *sig = sigma + row0 * NP;
    float       *out = gDhat_c + row0 * NP;
    for (uint32_t i = threadIdx.x; i < rows * NP; i += kSlicedBlock) {
        const double Q = accQ[i];
        const double s = (double)sig[i];
        double dot = s * Q;
#pragma unroll
        for (int o = NP / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, NP);
        const float v = (float)(s * (Q - dot));
        if (sp.store_direct) out[i] = v;
        else if (v != 0.0f) atomic_add(out + i, v);
    }
}

// Workgroups [0, first_feat) drain the confidence-table bins, [first_feat, first_vtx) the feature-table
// bins; the rest are the two roles of the pre-reduced coarse levels (cngp_bwd_sliced.h: they scan the
// vertex grids that the launch before this one has completed), sharing the launch so that the CUs stay busy.
template <int D, int NP, typename FeatT, typename IoT>
__global__ __launch_bounds__(kSlicedBlock) void bin_drain_kernel(
    const Params p, const SliceParams sp_c, const SliceParams sp_f, const uint32_t first_feat, const uint32_t first_vtx,
    const float *__restrict__ x, const IoT *__restrict__ dyT, const int64_t N,
    const FeatT *__restrict__ D_f, const float *__restrict__ sigma,
    const BinRecord *__restrict__ recF, const BinRecord *__restrict__ recC,
    const uint32_t *__restrict__ baseF, const uint32_t *__restrict__ baseC, const uint32_t cap,
    const BwdRoles vtx, const DenseLevels dl, const float *__restrict__ G,
    float *__restrict__ gD_f, float *__restrict__ gDhat_c)
{
    extern __shared__ __align__(16) unsigned char smem[];
    if (blockIdx.x < first_feat) {
        if constexpr (NP > 1) {
            if (sp_f.nlevels == 0) drain_both<D, NP, FeatT, IoT>(p, sp_c, blockIdx.x, smem, x, dyT, N, D_f, sigma, recC, baseC, cap, gD_f, gDhat_c);
            else drain_logit<D, NP, FeatT, IoT>(p, sp_c, blockIdx.x, smem, x, dyT, N, D_f, sigma, recC, baseC, cap, gDhat_c);
        }
    } else if (blockIdx.x < first_vtx) {
        drain_feat<D, NP, IoT>(p, sp_f, blockIdx.x - first_feat, smem, x, dyT, N, sigma, recF, baseF, cap, gD_f);
    } else {
        const uint32_t wg = blockIdx.x - first_vtx;
        if (wg < vtx.first[ROLE_FEAT_VTX]) {
            if (NP > 1)
                bwd_logit_sliced<D, NP, true, FeatT, float>(p, vtx.sp[ROLE_LOGIT_VTX], dl, wg - vtx.first[ROLE_LOGIT_VTX], smem,
                                                            x, D_f, sigma, G, gDhat_c, N);
        } else {
            bwd_feat_sliced<D, NP, true, float>(p, vtx.sp[ROLE_FEAT_VTX], dl, wg - vtx.first[ROLE_FEAT_VTX], smem, x, sigma,
                                                G, gD_f, N);
        }
    }
}

}  // namespace cngp

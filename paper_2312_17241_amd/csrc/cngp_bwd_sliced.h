// Backward pass with gradient accumulation in LDS (Sec. 4 "Performance": accumulate the
// gradients of small codebooks in workgroup-local memory before they go to RAM).
//
// On gfx950 a global floating-point atomic costs about one 64-byte memory segment per
// ~50 ps for the whole chip, whatever the table size, which makes the scatter-add of the
// N * L * 2^d * N_p candidate updates the whole cost of training.  Here every workgroup owns
// one SLICE of one level's gradient table in LDS (as fp64 accumulators: ds_add_f64 runs at full
// LDS rate on this chip, ds_add_f32 does not), scans a chunk of the points, keeps the corner
// references that hash into its slice, accumulates them with LDS atomics and writes the slice
// to HBM once.  Scanning is replicated per slice (hashing is cheap, atomics are not).
//
// Two kernels share the structure:
//   feature gradient  grad_D_f[base + k][f] += sigma_k * g[f]              slice = range of hashed rows
//   logit gradient    Q[h2][k] += <D_f[base + k], g>, then per row          slice = range of D^_c rows
//                     grad_Dhat_c[h2][k] += sigma_k * (Q_k - sum_j sigma_j Q_j)
// (the softmax Jacobian is linear in Q, so it is applied once per row when the slice is flushed).
// Both read a softmax table sigma = softmax(D^_c) and a level-major copy of dL/dy that two
// small kernels prepare in the workspace.
#pragma once
#include "cngp_kernels.h"

namespace cngp {

constexpr int kSlicedBlock = 1024;                  // 16 wavefronts share one slice
constexpr int kSlicedWaves = kSlicedBlock / 64;
constexpr int kQueueCap    = 96;                    // pending corner references per wavefront
constexpr int kSliceBytes  = 128 * 1024;            // LDS bytes of fp64 accumulators per workgroup

struct SliceParams {
    int32_t  level0;        // first level of this launch (blockIdx.z counts from it)
    uint32_t rows_log2;     // log2(table rows per slice)
    uint32_t chunk_pts;     // points per blockIdx.x
    int32_t  store_direct;  // 1: every slice is written by exactly one workgroup -> plain stores
};

struct __align__(16) QEntry {
    uint32_t row;           // row inside this workgroup's slice
    uint32_t other;         // index into the table the drain step reads (sigma row / D_f row group)
    float    g0, g1;        // weight * dL/dy of the corner
};

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}
// LDS traffic of one wavefront is ordered by the hardware; this only pins the compiler.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// ------------------------------------------------------------------ preparation kernels
// sigma[r][k] = softmax(D^_c[r][:])_k, one lane per element, NP lanes per row.
template <int NP>
__global__ __launch_bounds__(kBlock) void softmax_table_kernel(const float *__restrict__ Dhat_c,
                                                              float *__restrict__ sigma, const int64_t elems)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= elems) return;                       // elems is a multiple of NP: whole rows leave together
    const float v = Dhat_c[i];
    const float m = group_max<NP>(v);
    const float e = expf(v - m);
    sigma[i] = e / group_sum<NP>(e);
}

// dyT[l][n] = dy[n][l] for the F = 2 pair of each level (PairT: 4 bytes for fp16, 8 for fp32).
template <typename PairT>
__global__ __launch_bounds__(kBlock) void transpose_dy_kernel(const PairT *__restrict__ dy, PairT *__restrict__ dyT,
                                                             const int64_t N, const int L)
{
    const int64_t n = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (n >= N) return;
    for (int l = 0; l < L; ++l) dyT[(size_t)l * N + n] = dy[(size_t)n * L + l];
}

// ------------------------------------------------------------------ shared scan loop
// Walks the chunk of points, 64 per wavefront step; for every corner whose `row_of` falls into this
// workgroup's slice appends an entry to the wavefront's queue and drains the queue when it fills.
template <int D, bool BY_FEATURE_ROW, typename IoT, typename Drain>
__device__ __forceinline__ void scan_chunk(const Params &p, const SliceParams &sp, const int l,
                                           const float *__restrict__ x, const IoT *__restrict__ dy_l,
                                           const int64_t N, QEntry *queue, Drain drain)
{
    const int      lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t slice = blockIdx.y;
    const uint32_t row_lo_mask = (1u << sp.rows_log2) - 1u;
    const int64_t  n0 = (int64_t)blockIdx.x * sp.chunk_pts;
    const int64_t  n1 = (n0 + sp.chunk_pts < N) ? n0 + sp.chunk_pts : N;
    uint32_t       qn = 0;                                    // wavefront-uniform queue length

    for (int64_t nb = n0 + wave * 64; nb < n1; nb += kSlicedBlock) {
        const int64_t n = nb + lane;
        const bool    valid = n < n1;
        float xp[D];
#pragma unroll
        for (int j = 0; j < D; ++j) xp[j] = valid ? x[n * D + j] : 0.0f;
        Cell<D> cell;
        cell.locate(xp, p.N_l[l]);
        float2 g = make_float2(0.f, 0.f);
        if (valid) g = load_pair(dy_l, (size_t)n);
#pragma unroll
        for (int c = 0; c < (1 << D); ++c) {
            const uint32_t r1 = cell.hash1(c) & p.row_mask;    // hashed row group of D_f
            const uint32_t r2 = cell.hash2(c) & p.c_mask;      // row of D^_c
            const uint32_t mine = BY_FEATURE_ROW ? r1 : r2;
            const bool     take = valid && (mine >> sp.rows_log2) == slice;
            const uint64_t m = __ballot(take);
            if (take) {
                const float wt = cell.weight(c);
                QEntry e;
                e.row = mine & row_lo_mask;
                e.other = BY_FEATURE_ROW ? r2 : r1;
                e.g0 = wt * g.x;
                e.g1 = wt * g.y;
                queue[qn + lanes_below(m)] = e;
            }
            qn += (uint32_t)__popcll(m);
            if (qn > (uint32_t)(kQueueCap - 64)) {             // the next corner may add up to 64
                wave_lds_fence();
                drain(qn);
                wave_lds_fence();
                qn = 0;
            }
        }
    }
    wave_lds_fence();
    drain(qn);
}

// ------------------------------------------------------------------ feature gradient
template <int D, int NP, typename IoT>
__global__ __launch_bounds__(kSlicedBlock) void bwd_feat_sliced_kernel(
    const Params p, const SliceParams sp, const float *__restrict__ x, const float *__restrict__ sigma,
    const IoT *__restrict__ dyT, float *__restrict__ gD_f, const int64_t N)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int  RW = NP * 2;                               // accumulators per row group (F = 2)
    constexpr int  EPI = 64 / RW;                             // queue entries per wavefront instruction
    const uint32_t rows = 1u << sp.rows_log2;
    double *acc = reinterpret_cast<double *>(smem);
    QEntry *queue = reinterpret_cast<QEntry *>(smem + (size_t)rows * RW * sizeof(double)) +
                    (threadIdx.x >> 6) * kQueueCap;
    const int l = sp.level0 + (int)blockIdx.z;

    for (uint32_t i = threadIdx.x; i < rows * RW; i += kSlicedBlock) acc[i] = 0.0;
    __syncthreads();

    const float *sig_l = sigma + (size_t)l * p.N_c * NP;
    const int    lane = threadIdx.x & 63;
    const int    sub = lane / RW, j = lane % RW;              // entry slot, accumulator within the row group
    auto drain = [&](const uint32_t qn) {
        constexpr int U = 4;                                  // entries in flight per lane group
        for (uint32_t e0 = 0; e0 < qn; e0 += EPI * U) {
            QEntry q[U];
            float  s[U];
            bool   ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t e = e0 + u * EPI + sub;
                ok[u] = e < qn;
                q[u] = queue[ok[u] ? e : 0];
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                s[u] = (NP == 1 || !ok[u]) ? 1.0f : sig_l[(size_t)q[u].other * NP + (j >> 1)];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ok[u]) atomicAdd(&acc[q[u].row * RW + j], (double)(s[u] * ((j & 1) ? q[u].g1 : q[u].g0)));
        }
    };
    scan_chunk<D, true>(p, sp, l, x, dyT + (size_t)l * N * 2, N, queue, drain);
    __syncthreads();

    float *out = gD_f + (size_t)l * p.N_f * 2 + (size_t)blockIdx.y * rows * RW;
    for (uint32_t i = threadIdx.x; i < rows * RW; i += kSlicedBlock) {
        const float v = (float)acc[i];
        if (sp.store_direct) out[i] = v;
        else if (v != 0.0f) atomic_add(out + i, v);
    }
}

// ------------------------------------------------------------------ logit gradient
template <int D, int NP, typename FeatT, typename IoT>
__global__ __launch_bounds__(kSlicedBlock) void bwd_logit_sliced_kernel(
    const Params p, const SliceParams sp, const float *__restrict__ x, const FeatT *__restrict__ D_f,
    const float *__restrict__ sigma, const IoT *__restrict__ dyT, float *__restrict__ gDhat_c, const int64_t N)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int  EPI = 64 / NP;
    const uint32_t rows = 1u << sp.rows_log2;
    double *acc = reinterpret_cast<double *>(smem);
    QEntry *queue = reinterpret_cast<QEntry *>(smem + (size_t)rows * NP * sizeof(double)) +
                    (threadIdx.x >> 6) * kQueueCap;
    const int l = sp.level0 + (int)blockIdx.z;

    for (uint32_t i = threadIdx.x; i < rows * NP; i += kSlicedBlock) acc[i] = 0.0;
    __syncthreads();

    const FeatT *F_l = D_f + (size_t)l * p.N_f * 2;
    const int    lane = threadIdx.x & 63;
    const int    sub = lane / NP, k = lane % NP;
    auto drain = [&](const uint32_t qn) {
        constexpr int U = 4;
        for (uint32_t e0 = 0; e0 < qn; e0 += EPI * U) {
            QEntry q[U];
            float2 feat[U];
            bool   ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t e = e0 + u * EPI + sub;
                ok[u] = e < qn;
                q[u] = queue[ok[u] ? e : 0];
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                feat[u] = ok[u] ? load_pair(F_l, (size_t)q[u].other * NP + k) : make_float2(0.f, 0.f);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ok[u]) atomicAdd(&acc[q[u].row * NP + k], (double)fmaf(feat[u].x, q[u].g0, feat[u].y * q[u].g1));
        }
    };
    scan_chunk<D, false>(p, sp, l, x, dyT + (size_t)l * N * 2, N, queue, drain);
    __syncthreads();

    // softmax Jacobian per row, then out to HBM; NP consecutive lanes hold one row
    const size_t row0 = (size_t)l * p.N_c + (size_t)blockIdx.y * rows;
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

}  // namespace cngp

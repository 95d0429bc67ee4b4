// Level-resident forward (Eq. 6 + interpolation) for large batches.
//
// The tile kernel takes 256 points through all levels; every one of its feature lookups is a divergent 4- or 8-byte
// load that the texture addresser and the L2 serve one cache line at a time, and that request rate is what bounds it.
// Here a workgroup belongs to ONE level for its whole life: it copies the level's index codebook and as much of the
// level's feature codebook as fits into LDS once, then streams its share of the points.  Lookups below `resident`
// are LDS reads; the rest still go to memory.  A workgroup produces one level's two columns only, so the encodings
// are written level-major (yT[l][n], coalesced) and a second kernel turns them into rows of y.
// Per point and level the arithmetic is that of the tile kernel, in the same order: the results are bit-identical.
#pragma once
#include "cngp_kernels.h"

namespace cngp {

constexpr int kLevelBlock = 1024;        // 16 wavefronts: one workgroup per CU, the LDS is what limits residency
constexpr int kLevelUnroll = 2;          // points per lane in flight

template <int D, typename FeatT, typename IoT, int FMT>
__global__ __launch_bounds__(kLevelBlock) void encode_fwd_level_kernel(
    const Params p, const float *__restrict__ x, const FeatT *__restrict__ D_f, const uint8_t *__restrict__ D_c,
    IoT *__restrict__ yT, const int64_t N, const uint32_t c_stride, const int vec, const uint32_t resident,
    const int64_t per_part)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint8_t       *probes = smem;                                            // D_c of this level: 4-bit packed, or its bit string
    const uint32_t lds_c = (p.N_c + 1u) / 2u;
    FeatT         *feats = reinterpret_cast<FeatT *>(smem + ((lds_c + 15u) & ~15u));   // entries [0, resident) of this level
    const int      t = threadIdx.x;
    const int      l = (int)(blockIdx.x % (uint32_t)p.L_loaded);
    const int64_t  part = blockIdx.x / (uint32_t)p.L_loaded;
    const uint8_t *C_l = D_c + (size_t)l * c_stride;
    const FeatT   *F_l = D_f + (size_t)l * p.N_f * 2;

    stage_probes<FMT, kLevelBlock>(probes, C_l, c_stride, lds_c, vec, t);
    {
        const uint32_t bytes = resident * (uint32_t)(2 * sizeof(FeatT));     // a multiple of 16 (host)
        for (uint32_t i = (uint32_t)t * 16u; i < bytes; i += kLevelBlock * 16u)
            *reinterpret_cast<uint4 *>(reinterpret_cast<unsigned char *>(feats) + i) =
                *reinterpret_cast<const uint4 *>(reinterpret_cast<const unsigned char *>(F_l) + i);
    }
    __syncthreads();

    const int64_t  n_begin = part * per_part;
    const int64_t  n_end = (n_begin + per_part < N) ? n_begin + per_part : N;
    IoT           *out = yT + (size_t)l * (size_t)N * 2;
    const uint32_t N_l = p.N_l[l];

    // the coordinates of the next step's points are loaded while this step's lookups are under way
    constexpr int64_t kStep = (int64_t)kLevelUnroll * kLevelBlock;
    float xnext[kLevelUnroll][D];
    auto fetch = [&](const int64_t first) {
#pragma unroll
        for (int u = 0; u < kLevelUnroll; ++u) {
            const int64_t n = first + (int64_t)u * kLevelBlock;
#pragma unroll
            for (int j = 0; j < D; ++j) xnext[u][j] = n < n_end ? x[n * D + j] : 0.0f;
        }
    };
    fetch(n_begin + t);
    for (int64_t n0 = n_begin + t; n0 < n_end; n0 += kStep) {
        uint32_t idx[kLevelUnroll][1 << D];
        float    wt[kLevelUnroll][1 << D];
        bool     live[kLevelUnroll];
        float    xcur[kLevelUnroll][D];
#pragma unroll
        for (int u = 0; u < kLevelUnroll; ++u)
#pragma unroll
            for (int j = 0; j < D; ++j) xcur[u][j] = xnext[u][j];
        fetch(n0 + kStep);
#pragma unroll
        for (int u = 0; u < kLevelUnroll; ++u) {
            const int64_t n = n0 + (int64_t)u * kLevelBlock;
            live[u] = n < n_end;
            const float (&xp)[D] = xcur[u];
            Cell<D> cell;
            cell.locate(xp, N_l);
#pragma unroll
            for (int c = 0; c < (1 << D); ++c) {
                idx[u][c] = probe_base(cell.hash1(c), p) +
                            (FMT == kFmtBits ? read_probe_bits_lds(probes, cell.hash2(c) & p.c_mask, p.log2_Np)
                                             : read_probe<kFmtPacked4>(probes, cell.hash2(c) & p.c_mask, p.log2_Np));
                wt[u][c] = cell.weight(c);
            }
        }
        float2 feat[kLevelUnroll][1 << D];
#pragma unroll
        for (int u = 0; u < kLevelUnroll; ++u)
#pragma unroll
            for (int c = 0; c < (1 << D); ++c) {
                if (idx[u][c] < resident) feat[u][c] = load_pair(feats, idx[u][c]);
                else feat[u][c] = load_pair(F_l, idx[u][c]);
            }
#pragma unroll
        for (int u = 0; u < kLevelUnroll; ++u) {
            float y0 = 0.0f, y1 = 0.0f;
#pragma unroll
            for (int c = 0; c < (1 << D); ++c) {
                y0 = fmaf(wt[u][c], feat[u][c].x, y0);
                y1 = fmaf(wt[u][c], feat[u][c].y, y1);
            }
            if (live[u]) store_pair(out, (size_t)(n0 + (int64_t)u * kLevelBlock), y0, y1);
        }
    }
}

// yT[l][n] (pairs) -> y[row(n)][l], row(n) = perm ? perm[n] : n; levels from L_loaded on are written as zeros.
// One workgroup per 256 points: coalesced reads per level into a padded LDS tile, then the tile's rows leave as one
// contiguous block (whole rows, piece by piece, under a permutation).
constexpr int kRowsTile = 256;
template <typename IoT>
__global__ __launch_bounds__(kRowsTile) void level_major_to_rows_kernel(
    const IoT *__restrict__ yT, IoT *__restrict__ y, const int64_t N, const int L, const int L_loaded,
    const int32_t *__restrict__ perm)
{
    using Pair = typename std::conditional<sizeof(IoT) == 2, uint32_t, uint2>::type;
    extern __shared__ __align__(16) unsigned char smem[];
    Pair         *tile = reinterpret_cast<Pair *>(smem);                     // [kRowsTile][L + 1]
    const int     t = threadIdx.x;
    const int64_t n0 = (int64_t)blockIdx.x * kRowsTile;
    const int64_t rows = (N - n0 < kRowsTile) ? N - n0 : kRowsTile;
    const Pair   *src = reinterpret_cast<const Pair *>(yT);
    Pair          zero;
    __builtin_memset(&zero, 0, sizeof(zero));
    for (int l0 = 0; l0 < L; l0 += 8) {                     // eight levels' loads in flight, then their LDS writes
        Pair v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            v[j] = (l0 + j < L_loaded && t < rows) ? src[(size_t)(l0 + j) * (size_t)N + (size_t)(n0 + t)] : zero;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (l0 + j < L) tile[t * (L + 1) + l0 + j] = v[j];
    }
    __syncthreads();
    Pair *dst = reinterpret_cast<Pair *>(y);
    for (int i = t; i < (int)rows * L; i += kRowsTile) {
        const int r = i / L, c = i - r * L;
        const size_t row = perm ? (size_t)perm[n0 + r] : (size_t)(n0 + r);
        dst[row * (size_t)L + c] = tile[r * (L + 1) + c];
    }
}

}  // namespace cngp

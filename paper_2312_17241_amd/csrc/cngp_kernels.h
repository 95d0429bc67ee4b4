// gfx950 kernels of the encoding path: forward gather + interpolation, backward
// scatter-add with wavefront-cooperative probe rows, bake, index dump, fill.
#pragma once
#include "cngp_device.h"

namespace cngp {

// ------------------------------------------------------------------ forward (Eq. 6 + interpolation)
// One thread per (point, level) pair, pairs numbered n * L + l, so that the F = 2 outputs
// of consecutive threads are consecutive in y: every wavefront writes one contiguous run.
template <int D, typename FeatT, typename IoT, int FMT>
__global__ __launch_bounds__(kBlock) void encode_fwd_kernel(
    const Params p, const float *__restrict__ x, const FeatT *__restrict__ D_f,
    const uint8_t *__restrict__ D_c, IoT *__restrict__ y, const int64_t pairs, const uint32_t c_stride,
    const int32_t *__restrict__ perm)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= pairs) return;
    const int64_t n = i / p.L;
    const int     l = (int)(i - n * p.L);
    // with a permutation the encoding of point n is row perm[n] of y
    const size_t  o = perm ? (size_t)perm[n] * p.L + l : (size_t)i;
    if (l >= p.L_loaded) {                        // level not loaded
        store_pair(y, o, 0.0f, 0.0f);
        return;
    }

    float xp[D];
#pragma unroll
    for (int j = 0; j < D; ++j) xp[j] = x[n * D + j];
    Cell<D> cell;
    cell.locate(xp, p.N_l[l]);

    const FeatT   *F_l = D_f + (size_t)l * p.N_f * 2;
    const uint8_t *C_l = D_c + (size_t)l * c_stride;

    // issue all probe reads, then all feature reads, so the gathers overlap
    uint32_t idx[1 << D];
#pragma unroll
    for (int c = 0; c < (1 << D); ++c)
        idx[c] = read_probe<FMT>(C_l, cell.hash2(c) & p.c_mask, p.log2_Np);
#pragma unroll
    for (int c = 0; c < (1 << D); ++c) idx[c] += probe_base(cell.hash1(c), p);
    float2 feat[1 << D];
#pragma unroll
    for (int c = 0; c < (1 << D); ++c) feat[c] = load_pair(F_l, idx[c]);
    float y0 = 0.0f, y1 = 0.0f;
#pragma unroll
    for (int c = 0; c < (1 << D); ++c) {
        const float wt = cell.weight(c);
        y0 = fmaf(wt, feat[c].x, y0);
        y1 = fmaf(wt, feat[c].y, y1);
    }
    store_pair(y, o, y0, y1);
}

// Tile variant of the forward pass: a workgroup of TILE lanes takes TILE consecutive points through all levels.
// Per level it copies that level's index codebook D_c into LDS (always as packed 4-bit entries, N_c / 2
// bytes: byte-per-entry input is packed on the way in), so the probe lookups -- half of all random
// reads of the forward pass -- never reach the memory pipeline; only the D_f gathers do.  Outputs are
// collected in LDS and leave as one contiguous, fully coalesced block.
constexpr int kFwdTile = 256;        // default; kFwdTileLarge when staging a level's codebook is the larger cost
constexpr int kFwdTileLarge = 1024;

// One level's index codebook into LDS, by the whole workgroup: the bit string of the exact-width format as it
// is, everything else as packed 4-bit entries (byte-per-entry input is packed on the way in).
template <int FMT, int TILE>
__device__ __forceinline__ void stage_probes(uint8_t *probes, const uint8_t *__restrict__ C_l, const uint32_t c_stride,
                                             const uint32_t lds_c, const int vec, const int t)
{
    if (FMT == kFmtBits) {                                               // the level's bit string as it is
        if (vec) {
            for (uint32_t i = t * 16u; i < c_stride; i += TILE * 16u)
                *reinterpret_cast<uint4 *>(probes + i) = *reinterpret_cast<const uint4 *>(C_l + i);
        } else {
            for (uint32_t i = t * 4u; i < c_stride; i += TILE * 4u)
                *reinterpret_cast<uint32_t *>(probes + i) = *reinterpret_cast<const uint32_t *>(C_l + i);
        }
    } else if (FMT == kFmtPacked4) {
        if (vec) {
            for (uint32_t i = t * 16u; i < c_stride; i += TILE * 16u)
                *reinterpret_cast<uint4 *>(probes + i) = *reinterpret_cast<const uint4 *>(C_l + i);
        } else {
            for (uint32_t i = t; i < c_stride; i += TILE) probes[i] = C_l[i];
        }
    } else if (vec) {                                                    // 16 entries in, 8 bytes out
        for (uint32_t i = t * 16u; i < c_stride; i += TILE * 16u) {
            const uint4 w = *reinterpret_cast<const uint4 *>(C_l + i);
            auto pack = [](uint32_t v) {                                 // 4 entries -> 2 bytes
                v &= 0x0F0F0F0Fu;
                v = (v | (v >> 4)) & 0x00FF00FFu;
                return (v | (v >> 8)) & 0xFFFFu;
            };
            *reinterpret_cast<uint2 *>(probes + i / 2) =
                make_uint2(pack(w.x) | (pack(w.y) << 16), pack(w.z) | (pack(w.w) << 16));
        }
    } else {
        for (uint32_t i = t; i < lds_c; i += TILE) {
            const uint32_t lo = C_l[2 * i] & 0xFu, hi = (2 * i + 1 < c_stride) ? (C_l[2 * i + 1] & 0xFu) : 0u;
            probes[i] = (uint8_t)(lo | (hi << 4));
        }
    }
}

// The same in two halves, for codebooks of at most kPrefetch 16-byte pieces per lane: `fetch` issues the loads of a
// level's codebook into registers, `commit` writes them to LDS.  The kernel fetches level l + 1 before it works
// on level l, so the latency of the copy hides behind the lookups instead of stalling the workgroup between two
// barriers.
constexpr int kPrefetch = 4;
template <int TILE>
__device__ __forceinline__ void fetch_probes(uint4 (&buf)[kPrefetch], const uint8_t *__restrict__ C_l, const uint32_t c_stride, const int t)
{
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) {
        const uint32_t i = ((uint32_t)j * TILE + (uint32_t)t) * 16u;
        if (i < c_stride) buf[j] = *reinterpret_cast<const uint4 *>(C_l + i);
    }
}
template <int FMT, int TILE>
__device__ __forceinline__ void commit_probes(uint8_t *probes, const uint4 (&buf)[kPrefetch], const uint32_t c_stride, const int t)
{
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) {
        const uint32_t i = ((uint32_t)j * TILE + (uint32_t)t) * 16u;
        if (i >= c_stride) continue;
        if (FMT == kFmtU8) {                                             // 16 entries in, 8 bytes out
            auto pack = [](uint32_t v) {                                 // 4 entries -> 2 bytes
                v &= 0x0F0F0F0Fu;
                v = (v | (v >> 4)) & 0x00FF00FFu;
                return (v | (v >> 8)) & 0xFFFFu;
            };
            *reinterpret_cast<uint2 *>(probes + i / 2) =
                make_uint2(pack(buf[j].x) | (pack(buf[j].y) << 16), pack(buf[j].z) | (pack(buf[j].w) << 16));
        } else {
            *reinterpret_cast<uint4 *>(probes + i) = buf[j];
        }
    }
}

template <int D, typename FeatT, typename IoT, int FMT, int TILE>
__global__ __launch_bounds__(TILE) void encode_fwd_tile_kernel(
    const Params p, const float *__restrict__ x, const FeatT *__restrict__ D_f,
    const uint8_t *__restrict__ D_c, IoT *__restrict__ y, const int64_t N, const uint32_t c_stride, const int vec,
    const int32_t *__restrict__ perm, const uint32_t feat_lds)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint8_t *probes = smem;                                  // D_c of the current level: 4-bit packed, or its exact-width bit string
    const uint32_t lds_c = (p.N_c + 1u) / 2u;                                // bytes of it
    IoT     *out = reinterpret_cast<IoT *>(smem + ((lds_c + 15u) & ~15u));   // [TILE][L * 2]
    // feat_lds != 0: a level's feature codebook is small enough to sit in LDS too (the paper's compressed models), after the outputs
    FeatT   *feats = reinterpret_cast<FeatT *>(reinterpret_cast<unsigned char *>(out) + (size_t)TILE * p.L * 2 * sizeof(IoT));
    const int     t = threadIdx.x;
    const int64_t n0 = (int64_t)blockIdx.x * TILE;
    const int64_t n = n0 + t;
    const bool    valid = n < N;
    float xp[D];
#pragma unroll
    for (int j = 0; j < D; ++j) xp[j] = valid ? x[n * D + j] : 0.0f;

    for (int l = p.L_loaded; l < p.L; ++l) store_pair(out, (size_t)t * p.L + l, 0.0f, 0.0f);    // levels that are not loaded
    // the codebook of the next level travels in registers (small tiles only: with 1024-lane tiles it was slower, measured)
    const bool ahead = TILE == kFwdTile && vec && c_stride <= (uint32_t)(kPrefetch * TILE * 16);
    uint4 next[kPrefetch];
    if (ahead && p.L_loaded > 0) fetch_probes<TILE>(next, D_c, c_stride, t);
    for (int l = 0; l < p.L_loaded; ++l) {
        const uint8_t *C_l = D_c + (size_t)l * c_stride;
        __syncthreads();                                                     // previous level's lookups are done
        if (ahead) commit_probes<FMT, TILE>(probes, next, c_stride, t);
        else stage_probes<FMT, TILE>(probes, C_l, c_stride, lds_c, vec, t);
        const FeatT *F_l = D_f + (size_t)l * p.N_f * 2;
        if (feat_lds) {                                                      // N_f pairs: 4 or 8 bytes each, copied as 4-byte words
            const uint32_t words = p.N_f * (uint32_t)(2 * sizeof(FeatT) / 4);
            for (uint32_t i = t; i < words; i += TILE)
                reinterpret_cast<uint32_t *>(feats)[i] = reinterpret_cast<const uint32_t *>(F_l)[i];
        }
        __syncthreads();
        if (ahead && l + 1 < p.L_loaded) fetch_probes<TILE>(next, C_l + c_stride, c_stride, t);

        Cell<D> cell;
        cell.locate(xp, p.N_l[l]);
        uint32_t idx[1 << D];
#pragma unroll
        for (int c = 0; c < (1 << D); ++c)
            idx[c] = probe_base(cell.hash1(c), p) +
                     (FMT == kFmtBits ? read_probe_bits_lds(probes, cell.hash2(c) & p.c_mask, p.log2_Np)
                                      : read_probe<kFmtPacked4>(probes, cell.hash2(c) & p.c_mask, p.log2_Np));
        float2 feat[1 << D];
        const FeatT *table = feat_lds ? feats : F_l;
#pragma unroll
        for (int c = 0; c < (1 << D); ++c) feat[c] = load_pair(table, idx[c]);
        float y0 = 0.0f, y1 = 0.0f;
#pragma unroll
        for (int c = 0; c < (1 << D); ++c) {
            const float wt = cell.weight(c);
            y0 = fmaf(wt, feat[c].x, y0);
            y1 = fmaf(wt, feat[c].y, y1);
        }
        store_pair(out, (size_t)t * p.L + l, y0, y1);
    }
    __syncthreads();

    const int64_t rows = (N - n0 < TILE) ? N - n0 : TILE;
    if (perm) {                                   // row r of the tile is row perm[n0 + r] of y: whole rows, piece by piece
        const size_t row_bytes = (size_t)p.L * 2 * sizeof(IoT);
        unsigned char       *ybytes = reinterpret_cast<unsigned char *>(y);
        const unsigned char *src = reinterpret_cast<const unsigned char *>(out);
        if (row_bytes % 16 == 0 && ((uintptr_t)y & 15u) == 0) {
            const uint32_t pieces = (uint32_t)(row_bytes / 16);
            for (uint32_t i = t; i < (uint32_t)rows * pieces; i += TILE) {
                const uint32_t r = i / pieces, q = i % pieces;
                *reinterpret_cast<uint4 *>(ybytes + (size_t)perm[n0 + r] * row_bytes + (size_t)q * 16) =
                    *reinterpret_cast<const uint4 *>(src + (size_t)i * 16);
            }
        } else {
            const uint32_t pieces = (uint32_t)(row_bytes / sizeof(IoT));
            for (uint32_t i = t; i < (uint32_t)rows * pieces; i += TILE) {
                const uint32_t r = i / pieces, q = i % pieces;
                reinterpret_cast<IoT *>(ybytes + (size_t)perm[n0 + r] * row_bytes)[q] = reinterpret_cast<const IoT *>(src)[i];
            }
        }
        return;
    }
    // the tile's outputs are one contiguous block of y
    const size_t  bytes = (size_t)rows * p.L * 2 * sizeof(IoT);
    unsigned char *dst = reinterpret_cast<unsigned char *>(y + (size_t)n0 * p.L * 2);
    const unsigned char *src = reinterpret_cast<const unsigned char *>(out);
    if (((uintptr_t)dst & 15u) == 0 && bytes % 16 == 0) {
        for (size_t i = (size_t)t * 16; i < bytes; i += (size_t)TILE * 16)
            *reinterpret_cast<uint4 *>(dst + i) = *reinterpret_cast<const uint4 *>(src + i);
    } else {
        for (size_t i = (size_t)t * sizeof(IoT); i < bytes; i += (size_t)TILE * sizeof(IoT))
            *reinterpret_cast<IoT *>(dst + i) = *reinterpret_cast<const IoT *>(src + i);
    }
}

// ------------------------------------------------------------------ gradient with respect to the points
// dL/dx of the forward pass above (the index of Eq. 6 is constant inside a cell, so the derivative acts on
// the d-linear weights):  dL/dx_j = sum_l N_l sum_c (+-1)_j prod_{i != j} w_i(c) <D_f[l][idx_c], dL/dy[n, l]>.
// Same tile structure as the forward pass: the level's index codebook staged in LDS, one lane per point.
template <int D, typename FeatT, typename IoT, int FMT, int TILE, bool STAGED>
__global__ __launch_bounds__(TILE) void encode_bwd_input_kernel(
    const Params p, const float *__restrict__ x, const FeatT *__restrict__ D_f, const uint8_t *__restrict__ D_c,
    const IoT *__restrict__ dy, float *__restrict__ grad_x, const int64_t N, const uint32_t c_stride, const int vec)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint8_t *probes = smem;
    const uint32_t lds_c = (p.N_c + 1u) / 2u;
    const int     t = threadIdx.x;
    const int64_t n = (int64_t)blockIdx.x * TILE + t;
    const bool    valid = n < N;
    float xp[D], gx[D];
#pragma unroll
    for (int j = 0; j < D; ++j) { xp[j] = valid ? x[n * D + j] : 0.0f; gx[j] = 0.0f; }

    for (int l = 0; l < p.L; ++l) {
        const uint8_t *C_l = D_c + (size_t)l * c_stride;
        if (STAGED) {
            __syncthreads();                                                 // previous level's lookups are done
            stage_probes<FMT, TILE>(probes, C_l, c_stride, lds_c, vec, t);
            __syncthreads();
        }
        Cell<D> cell;
        cell.locate(xp, p.N_l[l]);
        const FeatT *F_l = D_f + (size_t)l * p.N_f * 2;
        uint32_t idx[1 << D];
#pragma unroll
        for (int c = 0; c < (1 << D); ++c) {
            const uint32_t r = cell.hash2(c) & p.c_mask;
            const uint32_t probe = !STAGED ? read_probe<FMT>(C_l, r, p.log2_Np)
                                 : FMT == kFmtBits ? read_probe_bits_lds(probes, r, p.log2_Np)
                                                   : read_probe<kFmtPacked4>(probes, r, p.log2_Np);
            idx[c] = probe_base(cell.hash1(c), p) + probe;
        }
        float2 feat[1 << D];
#pragma unroll
        for (int c = 0; c < (1 << D); ++c) feat[c] = load_pair(F_l, idx[c]);
        const float2 g = valid ? load_pair(dy, (size_t)n * p.L + l) : make_float2(0.f, 0.f);
        const float  res = (float)p.N_l[l];
#pragma unroll
        for (int c = 0; c < (1 << D); ++c) {
            const float tc = res * fmaf(feat[c].x, g.x, feat[c].y * g.y);
#pragma unroll
            for (int j = 0; j < D; ++j) {
                float dw = ((c >> j) & 1) ? tc : -tc;
#pragma unroll
                for (int i = 0; i < D; ++i)
                    if (i != j) dw *= ((c >> i) & 1) ? cell.w[i] : 1.0f - cell.w[i];
                gx[j] += dw;
            }
        }
    }
    if (valid) {
#pragma unroll
        for (int j = 0; j < D; ++j) grad_x[n * D + j] = gx[j];
    }
}

// ------------------------------------------------------------------ backward (Sec. 3 "Training")
// Reduction over the NP lanes that share one probe row.
template <int NP>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
    for (int o = NP / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, NP));
    return v;
}
template <int NP>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
    for (int o = NP / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, NP);
    return v;
}

// Sparse variant of the backward: how many candidates of its row are ranked before candidate k, which
// holds confidence value v (larger first; equal values: lowest index first; a NaN after every number).
// The NP lanes of a row call this together.
template <int NP>
__device__ __forceinline__ uint32_t rank_in_row(const float v, const int k) {
    uint32_t ahead = 0;
    const int first = (int)(threadIdx.x & 63u) - k;
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const float o = __shfl(v, first + j, 64);
        const bool  o_num = o == o, v_num = v == v;
        ahead += ((o_num && !v_num) || (o_num == v_num && (o > v || ((o == v || !v_num) && j < k)))) ? 1u : 0u;
    }
    return ahead;
}
// The confidence value as the softmax should see it: itself when it is among the top_k largest of its
// row, minus infinity otherwise, which gives the candidate weight exactly 0.
template <int NP>
__device__ __forceinline__ float keep_top_k(const float v, const int k, const uint32_t top_k) {
    if (NP == 1 || top_k == 0 || top_k >= (uint32_t)NP) return v;
    return rank_in_row<NP>(v, k) < top_k ? v : -INFINITY;
}

// Direct backward: NP adjacent lanes own one (point, level) pair and walk its 2^d corners;
// lane k is candidate k of the probing range, so the NP lanes read and update one contiguous
// row of D^_c / grad D^_c and one contiguous run of D_f / grad D_f per corner.
// blockIdx.y is the level: the whole grid works through one level's tables at a time.
template <int D, int NP, typename FeatT, typename IoT>
__global__ __launch_bounds__(kBlock) void encode_bwd_direct_kernel(
    const Params p, const int level0, const float *__restrict__ x, const FeatT *__restrict__ D_f,
    const float *__restrict__ Dhat_c, const IoT *__restrict__ dy,
    float *__restrict__ gD_f, float *__restrict__ gDhat_c, const int64_t N)
{
    constexpr int PTS = kBlock / NP;
    const int     l = level0 + (int)blockIdx.y;
    const int     k = threadIdx.x % NP;
    const int64_t n = (int64_t)blockIdx.x * PTS + threadIdx.x / NP;
    if (n >= N) return;           // whole lane groups leave together (PTS * NP == kBlock)

    float xp[D];
#pragma unroll
    for (int j = 0; j < D; ++j) xp[j] = x[n * D + j];
    Cell<D> cell;
    cell.locate(xp, p.N_l[l]);
    const float2 g_up = load_pair(dy, (size_t)n * p.L + l);

    const FeatT *F_l  = D_f + (size_t)l * p.N_f * 2;
    const float *C_l  = Dhat_c + (size_t)l * p.N_c * NP;
    float       *gF_l = gD_f + (size_t)l * p.N_f * 2;
    float       *gC_l = gDhat_c + (size_t)l * p.N_c * NP;

#pragma unroll
    for (int c = 0; c < (1 << D); ++c) {
        const uint32_t entry = probe_base(cell.hash1(c), p) + k;
        const uint32_t slot  = (cell.hash2(c) & p.c_mask) * NP + k;
        const float    logit = keep_top_k<NP>(C_l[slot], k, p.top_k);
        const float2   feat  = load_pair(F_l, entry);
        const float    wt = cell.weight(c);
        const float    g0 = wt * g_up.x, g1 = wt * g_up.y;

        const float m     = group_max<NP>(logit);
        const float e     = expf(logit - m);
        const float sigma = e / group_sum<NP>(e);
        const float q     = fmaf(feat.x, g0, feat.y * g1);
        const float qbar  = group_sum<NP>(sigma * q);

        atomic_add(gF_l + 2 * (size_t)entry, sigma * g0);
        atomic_add(gF_l + 2 * (size_t)entry + 1, sigma * g1);
        if (NP > 1) atomic_add(gC_l + slot, sigma * (q - qbar));
    }
}

// ------------------------------------------------------------------ bake (Fig. 3: argmax per row)
// One thread per output byte: one row (u8) or two rows (packed nibbles).
template <int NP>
__device__ __forceinline__ uint32_t argmax_row(const float *__restrict__ row) {
    uint32_t best = 0;
    bool     have = false;
    float    bv = 0.0f;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const float v = row[k];
        const bool  take = (v == v) && (!have || v > bv);   // NaN never wins; first maximum wins
        if (take) { best = k; bv = v; have = true; }
    }
    return best;
}

template <int NP, bool PACKED4>
__global__ __launch_bounds__(kBlock) void bake_probes_kernel(
    const float *__restrict__ Dhat_c, uint8_t *__restrict__ D_c, const int64_t bytes_out)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= bytes_out) return;
    if (PACKED4) {
        const uint32_t lo = argmax_row<NP>(Dhat_c + (size_t)(2 * i) * NP);
        const uint32_t hi = argmax_row<NP>(Dhat_c + (size_t)(2 * i + 1) * NP);
        D_c[i] = (uint8_t)(lo | (hi << 4));
    } else {
        D_c[i] = (uint8_t)argmax_row<NP>(Dhat_c + (size_t)i * NP);
    }
}

// Exact-width output: one thread per 32-bit word of a level's bit string.  An entry that straddles two
// words (3-bit entries only) is evaluated by both threads.
template <int NP>
__global__ __launch_bounds__(kBlock) void bake_probes_bits_kernel(
    const float *__restrict__ Dhat_c, uint32_t *__restrict__ D_c, const uint32_t N_c,
    const uint32_t words_per_level, const int64_t words)
{
    constexpr uint32_t bits = NP == 16 ? 4u : NP == 8 ? 3u : NP == 4 ? 2u : 1u;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= words) return;
    const uint32_t l = (uint32_t)(i / words_per_level), w = (uint32_t)(i % words_per_level);
    const uint32_t first = (32u * w) / bits;
    uint32_t last = (32u * w + 31u) / bits;
    if (last > N_c - 1u) last = N_c - 1u;
    uint32_t out = 0;
    for (uint32_t e = first; e <= last; ++e) {
        const uint32_t v = argmax_row<NP>(Dhat_c + ((size_t)l * N_c + e) * NP);
        const int pos = (int)(e * bits) - (int)(32u * w);
        out |= pos >= 0 ? (v << pos) : (v >> (-pos));
    }
    D_c[i] = out;
}

// ------------------------------------------------------------------ index dump (parity checks)
template <int D, int FMT>
__global__ __launch_bounds__(kBlock) void debug_indices_kernel(
    const Params p, const float *__restrict__ x, const uint8_t *__restrict__ D_c,
    uint32_t *__restrict__ base_out, uint32_t *__restrict__ h2_out, uint8_t *__restrict__ probe_out,
    uint32_t *__restrict__ idx_out, const int64_t pairs, const uint32_t c_stride)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= pairs) return;
    const int64_t n = i / p.L;
    const int     l = (int)(i - n * p.L);
    float xp[D];
#pragma unroll
    for (int j = 0; j < D; ++j) xp[j] = x[n * D + j];
    Cell<D> cell;
    cell.locate(xp, p.N_l[l]);
#pragma unroll
    for (int c = 0; c < (1 << D); ++c) {
        const uint32_t base = probe_base(cell.hash1(c), p);
        const uint32_t r    = cell.hash2(c) & p.c_mask;
        const uint32_t pr   = D_c ? read_probe<FMT>(D_c + (size_t)l * c_stride, r, p.log2_Np) : 0u;
        const size_t   o    = (size_t)i * (1 << D) + c;
        if (base_out)  base_out[o] = base;
        if (h2_out)    h2_out[o] = r;
        if (probe_out) probe_out[o] = (uint8_t)pr;
        if (idx_out)   idx_out[o] = base + pr;
    }
}

// ------------------------------------------------------------------ fill with zeros
// ------------------------------------------------------------------ feature widths other than two
// Every kernel of the library works on codebook entries of two features (the paper's F, Table 1).  F = 1, 4 and 8 are
// taken two features at a time: the interpolation and the feature gradient act on every feature by itself, and the
// logit gradient is a sum over the features, so a codebook of F features per entry is ceil(F / 2) codebooks of two
// that share their indices.  These two kernels move one such pair plane out of and into an array whose rows hold F
// values: rows of D_f ([L * N_f, F]), of y and dL/dy ([N * L, F]), of grad D_f.  A missing second feature (F = 1)
// reads as zero and is not written.
template <typename T>
__global__ __launch_bounds__(kBlock) void plane_take_kernel(const T *__restrict__ src, T *__restrict__ dst, const int64_t rows,
                                                           const int F, const int plane)
{
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r >= rows) return;
    const int f0 = 2 * plane;
    dst[2 * r] = src[r * F + f0];
    dst[2 * r + 1] = (f0 + 1 < F) ? src[r * F + f0 + 1] : T(0.0f);
}

// dst[r][2 plane (+ 1)] = src[r][0 (1)], or += when `accumulate`.
template <typename T>
__global__ __launch_bounds__(kBlock) void plane_put_kernel(const T *__restrict__ src, T *__restrict__ dst, const int64_t rows,
                                                          const int F, const int plane, const int accumulate)
{
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r >= rows) return;
    const int f0 = 2 * plane;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (f0 + j >= F) break;
        T *o = dst + r * F + f0 + j;
        if (accumulate) *o = T((float)*o + (float)src[2 * r + j]);
        else *o = src[2 * r + j];
    }
}

// Clears up to kZeroSegments float arrays in one launch; blockIdx.y selects the array.
constexpr int kZeroSegments = 6;
struct ZeroSegments {
    float  *ptr[kZeroSegments];
    int64_t count[kZeroSegments];
};

// Block `block` of `nblocks` clearing segment `which`.
__device__ __forceinline__ void zero_segment(const ZeroSegments &seg, const int which, const uint32_t block, const uint32_t nblocks)
{
    float        *p = seg.ptr[which];
    const int64_t n = seg.count[which];
    // scalar head up to 16-byte alignment, float4 body, scalar tail
    int64_t head = (int64_t)(((16u - ((uintptr_t)p & 15u)) & 15u) / 4u);
    if (head > n) head = n;
    const int64_t n4 = (n - head) / 4;
    float4       *p4 = reinterpret_cast<float4 *>(p + head);
    const int64_t stride = (int64_t)nblocks * kBlock;
    for (int64_t i = (int64_t)block * kBlock + threadIdx.x; i < n4; i += stride)
        p4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (block == 0) {
        if ((int64_t)threadIdx.x < head) p[threadIdx.x] = 0.0f;
        const int64_t tail0 = head + n4 * 4;
        if (tail0 + threadIdx.x < n) p[tail0 + threadIdx.x] = 0.0f;
    }
}

__global__ __launch_bounds__(kBlock) void zero_kernel(const ZeroSegments seg)
{
    zero_segment(seg, (int)blockIdx.y, blockIdx.x, gridDim.x);
}

}  // namespace cngp

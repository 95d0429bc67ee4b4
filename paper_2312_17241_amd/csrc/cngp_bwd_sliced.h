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
// Two roles of one kernel share the structure:
//   feature gradient  grad_D_f[base + k][f] += sigma_k * g[f]              slice = range of hashed rows
//   logit gradient    Q[h2][k] += <D_f[base + k], g>, then per row          slice = range of D^_c rows
//                     grad_Dhat_c[h2][k] += sigma_k * (Q_k - sum_j sigma_j Q_j)
// (the softmax Jacobian is linear in Q, so it is applied once per row when the slice is flushed).
// Both read a softmax table sigma = softmax(D^_c) and a level-major copy of dL/dy that a
// preparation launch writes into the workspace.
//
// Coarse levels are pre-reduced per grid vertex.  The backward pass is linear in g = weight * dL/dy
// of a corner reference, and both hashes depend on the vertex only, so all references to one vertex
// can be summed first: a further role accumulates G[v] = sum of g over the references to vertex v
// into the level's dense vertex grid (LDS slices again, no hashing), and the two roles above then
// scan the grid's vertices (one "corner" of weight 1 with g = G[v]) instead of the points.  A level
// with few vertices and many points (2M references onto 5832 vertices on the coarsest NeRF level)
// costs almost nothing this way.
#pragma once
#include "cngp_kernels.h"
#include <type_traits>

namespace cngp {

constexpr int kSlicedBlock = 1024;                  // 16 wavefronts share one slice
constexpr int kSlicedWaves = kSlicedBlock / 64;
constexpr int kRing        = 128;                   // pending corner references per wavefront (ring buffer)
constexpr int kRingBytes   = kRing * 12;            // 4-byte key + two floats per reference
constexpr int kSliceBytes  = 128 * 1024;            // LDS bytes of fp64 accumulators per workgroup

struct SliceParams {
    uint32_t rows_log2;     // log2(table rows per slice)
    uint32_t slices;        // slices per level
    uint32_t chunks;        // point chunks per slice
    uint32_t chunk_pts;     // points per chunk
    int32_t  store_direct;  // 1: every slice is written by exactly one workgroup -> plain stores
    int32_t  level0;        // levels [level0, level0 + nlevels) are covered by this launch
    int32_t  nlevels;
};

// Levels whose dense vertex grid is small enough to pre-reduce the upstream gradient per vertex.
// They are the first `count` levels; a grid has side = N_l + 2 vertices per axis (x = 1 reaches
// vertex N_l + 1).
constexpr int      kMaxDense = 16;
constexpr uint32_t kDenseSliceVerts = 8192;          // vertices per LDS slice (2 fp64 accumulators each)
struct DenseLevels {
    int32_t  count;
    uint32_t side[kMaxDense];
    uint32_t verts[kMaxDense];                       // side^d
    uint32_t slices[kMaxDense];                      // ceil(verts / kDenseSliceVerts)
    uint32_t g_off[kMaxDense];                       // offset of the level's grid in G, in vertices
};

// Which (level, slice, chunk) a workgroup works on.  Workgroups are handed to the 8 XCDs round-robin
// by their linear index, and every XCD has an L2 of its own.  The (level, slice, chunk) units of a
// role, numbered level-major, are cut into 8 equal contiguous runs, one per XCD: the workgroups of a
// level then sit on one XCD (two where a run boundary falls inside the level), so the rows a level
// gathers at random (its softmax table, its slice of D_f) stay in that L2 instead of all levels'
// tables competing for every L2, and every XCD gets the same amount of work.  `i` is the workgroup's
// index within its role; every role starts at a multiple of 8 in the grid, so i mod 8 is the XCD.
constexpr int kXcds = 8;
struct SliceCoord { int level, index; uint32_t slice, chunk; };   // index = level - level0; index < 0: no work
__device__ __forceinline__ SliceCoord slice_coord(const SliceParams &sp, const uint32_t i) {
    const uint32_t xcd = i % kXcds, j = i / kXcds;
    const uint32_t per_level = sp.slices * sp.chunks;
    const uint32_t total = per_level * (uint32_t)sp.nlevels;
    const uint32_t per_xcd = (total + kXcds - 1) / kXcds;
    const uint32_t unit = xcd * per_xcd + j;
    SliceCoord c;
    const uint32_t rem = unit % per_level;
    c.index = (j < per_xcd && unit < total) ? (int)(unit / per_level) : -1;
    c.level = sp.level0 + c.index;
    // chunk-major inside a level: the workgroups that run side by side on an XCD take the SAME run of points through
    // neighbouring slices, so the points and their gradients are read from memory once per level, not once per slice
    c.chunk = rem / sp.slices;
    c.slice = rem % sp.slices;
    return c;
}

// A two-feature codebook entry as it sits in memory.
template <typename FeatT> struct RawPair;
template <> struct RawPair<float> {
    using type = float2;
    static __device__ __forceinline__ float2 to_float2(float2 v) { return v; }
};
template <> struct RawPair<__half> {
    using type = __half2;
    static __device__ __forceinline__ float2 to_float2(__half2 v) { return __half22float2(v); }
};

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}
// LDS traffic of one wavefront is ordered by the hardware; this only pins the compiler.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// ------------------------------------------------------------------ preparation
// sigma[r][k] = softmax(D^_c[r][:])_k, one lane per element, NP lanes per row (top_k > 0: over the kept
// candidates only, 0 for the others).
template <int NP>
__device__ __forceinline__ void softmax_rows(const float *__restrict__ Dhat_c, float *__restrict__ sigma,
                                             const int64_t elems, const uint32_t block, const uint32_t top_k)
{
    const int64_t i = (int64_t)block * kBlock + threadIdx.x;
    if (i >= elems) return;                       // elems is a multiple of NP: whole rows leave together
    const float v = keep_top_k<NP>(Dhat_c[i], (int)(threadIdx.x % NP), top_k);
    const float m = group_max<NP>(v);
    const float e = expf(v - m);
    sigma[i] = e / group_sum<NP>(e);
}

// dyT[l][n] = dy[n][l] for the F = 2 pair of each level (PairT: 4 bytes for fp16, 8 for fp32).
template <typename PairT>
__device__ __forceinline__ void transpose_rows(const PairT *__restrict__ dy, PairT *__restrict__ dyT,
                                               const int64_t N, const int L, const uint32_t block)
{
    const int64_t n = (int64_t)block * kBlock + threadIdx.x;
    if (n >= N) return;
    for (int l = 0; l < L; ++l) dyT[(size_t)l * N + n] = dy[(size_t)n * L + l];
}

// Everything the accumulation kernels need first, in one launch: the gradient (and vertex-grid) ranges
// that are accumulated with atomics are cleared, the softmax table and the level-major copy of dL/dy are
// written.  Blocks [0, seg_count * zero_blocks) clear, the next softmax_blocks tabulate, the rest transpose.
struct PrepArgs {
    ZeroSegments seg;
    uint32_t     seg_count, zero_blocks;
    const float *Dhat_c;
    float       *sigma;
    int64_t      elems;
    uint32_t     softmax_blocks;
    const void  *dy;
    void        *dyT;
    int64_t      N;
    int32_t      L;
    uint32_t     top_k;
};

template <int NP, typename PairT>
__device__ __forceinline__ void bwd_prep_block(const PrepArgs &a, uint32_t b)
{
    if (b < a.seg_count * a.zero_blocks) {
        zero_segment(a.seg, (int)(b / a.zero_blocks), b % a.zero_blocks, a.zero_blocks);
        return;
    }
    b -= a.seg_count * a.zero_blocks;
    if (b < a.softmax_blocks) {
        softmax_rows<NP>(a.Dhat_c, a.sigma, a.elems, b, a.top_k);
        return;
    }
    transpose_rows<PairT>(reinterpret_cast<const PairT *>(a.dy), reinterpret_cast<PairT *>(a.dyT), a.N, a.L, b - a.softmax_blocks);
}

template <int NP, typename PairT>
__global__ __launch_bounds__(kBlock) void bwd_prep_kernel(const PrepArgs a)
{
    bwd_prep_block<NP, PairT>(a, blockIdx.x);
}

// ------------------------------------------------------------------ shared scan loop
// One wavefront walks its share of the chunk, 64 points per step:
//   1. locate each point's cell and test its 2^d corners against the workgroup's slice with the
//      slice-selecting hash only (a bit mask per lane);
//   2. in two phases (low and high half of the corners) emit the accepted corners, one per lane and
//      round, into the wavefront's ring buffer in LDS: key = row inside the slice | (row the other
//      table is read at) << rows_log2, and g = weight * dL/dy (weight and second hash are computed
//      for accepted corners only);
//   3. software pipeline over fixed batches of kBatch references: after every phase the batch whose
//      gathers (`load`) were issued one phase ago is accumulated (`accum`: LDS atomics) and the next
//      full batch is issued, so memory latency hides behind the hashing of the phase in between.
// NP lanes cooperate on one reference (lane k = candidate k of the probing range): 64 / NP
// references per wavefront instruction, U = kBatch * NP / 64 instructions per batch.  T is what
// `load` brings per lane.  Batches start at multiples of kBatch in the ring, so a batch never wraps.
constexpr int kBatch = 32;
static_assert(kRing % kBatch == 0 && kRing >= 64 + 2 * kBatch, "ring holds a round, a batch in flight and slack");

//
// VERTEX mode (pre-reduced coarse levels): the "points" are the n_items vertices of the level's dense
// grid, g_l holds their summed gradient G[v], and each has exactly one corner of weight 1: itself.
template <int D, int NP, bool BY_FEATURE_ROW, bool VERTEX, typename T, typename GradT, typename Load, typename Accum>
__device__ __forceinline__ void scan_chunk(const Params &p, const SliceParams &sp, const SliceCoord &co,
                                           const float *__restrict__ x, const GradT *__restrict__ g_l,
                                           const int64_t n_items, const uint32_t side,
                                           unsigned char *ring_mem, Load load, Accum accum)
{
    constexpr int  EPI = (64 / NP < kBatch) ? 64 / NP : kBatch;     // references per wavefront instruction
    constexpr int  U = kBatch / EPI;                                // instructions per batch
    const int      lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t sub = lane / NP;                                 // reference slot of this lane
    const bool     slot_ok = sub < (uint32_t)EPI;                   // N_p = 1: only the first kBatch lanes work
    uint32_t *ring_key = reinterpret_cast<uint32_t *>(ring_mem + (size_t)wave * kRingBytes);
    float2   *ring_g   = reinterpret_cast<float2 *>(ring_key + kRing);
    const uint32_t mine_mask   = BY_FEATURE_ROW ? p.row_mask : p.c_mask;
    const uint32_t other_mask  = BY_FEATURE_ROW ? p.c_mask : p.row_mask;
    const uint32_t row_lo_mask = (1u << sp.rows_log2) - 1u;
    const uint32_t slice_sel   = mine_mask & ~row_lo_mask;          // bits of the hash that name the slice
    const uint32_t slice_val   = co.slice << sp.rows_log2;
    const int64_t  n0 = (int64_t)co.chunk * sp.chunk_pts;
    const int64_t  n1 = (n0 + sp.chunk_pts >= n_items) ? n_items : n0 + sp.chunk_pts;
    const float    res = (float)p.N_l[co.level];

    // wavefront-uniform ring state: [head, mid) in flight, [mid, tail) waiting; head, mid multiples of kBatch
    uint32_t head = 0, mid = 0, tail = 0;
    T        inflight[U];
    auto issue = [&]() {                                            // gathers of the batch at mid
        const uint32_t base = (mid & (kRing - 1)) + sub;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (slot_ok) inflight[u] = load(ring_key[base + u * EPI]);
        mid += kBatch;
    };
    auto complete = [&]() {                                         // accumulate the batch at head
        const uint32_t base = (head & (kRing - 1)) + sub;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (slot_ok) accum(ring_key[base + u * EPI], ring_g[base + u * EPI], inflight[u]);
        head += kBatch;
    };
    auto pump = [&]() {                                             // one pipeline beat
        wave_lds_fence();
        if (mid != head) complete();
        if (tail - mid >= (uint32_t)kBatch) issue();
    };

    // software prefetch of the next step's point (or vertex) and its upstream gradient; items are
    // addressed by a 32-bit index relative to the chunk (a chunk holds fewer than 2^32 items)
    const float   *xc = x + n0 * D;
    const GradT   *gc = g_l + n0 * 2;
    const uint32_t items = (uint32_t)(n1 > n0 ? n1 - n0 : 0);
    auto fetch = [&](const uint32_t i, float (&xo)[D], float2 &go) {
        const bool ok = i < items;
        if (!VERTEX) {
#pragma unroll
            for (int j = 0; j < D; ++j) xo[j] = ok ? xc[i * D + j] : 0.0f;
        }
        go = ok ? load_pair(gc, i) : make_float2(0.f, 0.f);
    };
    float    xn[D] = {};
    float2   gn;
    uint32_t nb = wave * 64;
    fetch(nb + lane, xn, gn);
    for (; nb < items; nb += kSlicedBlock) {
        const bool valid = nb + lane < items;
        float xp[D];
#pragma unroll
        for (int j = 0; j < D; ++j) xp[j] = xn[j];
        const float2 g = gn;
        fetch(nb + kSlicedBlock + lane, xn, gn);

        float    w[D], w1[D];                                       // fraction and 1 - fraction
        uint32_t a[D], b[D], ao[D], bo[D];                          // slice hash, other hash: lower / upper vertex
        uint32_t accepted = 0;                                      // corners of this lane's item in the slice
        if (VERTEX) {
            // grid coordinates of vertex number nb + lane; its only corner is itself, weight 1
            uint32_t rest = (uint32_t)n0 + nb + lane;
#pragma unroll
            for (int i = 0; i < D; ++i) {
                const uint32_t v = (i == D - 1) ? rest : rest % side;
                rest /= side;
                a[i] = b[i] = v * (BY_FEATURE_ROW ? kPi[i] : kPi2[i]);
                ao[i] = bo[i] = v * (BY_FEATURE_ROW ? kPi2[i] : kPi[i]);
                w[i] = 0.0f;
                w1[i] = 1.0f;
            }
            uint32_t h = 0;
#pragma unroll
            for (int i = 0; i < D; ++i) h ^= a[i];
            if (valid && (g.x != 0.0f || g.y != 0.0f) && (h & slice_sel) == slice_val) accepted = 1u;
        } else {
            // cell of the point: fraction and the two hashes' terms per dimension
#pragma clang fp contract(off)
#pragma unroll
            for (int i = 0; i < D; ++i) {
                const float pos = xp[i] * res;                      // one rounded fp32 multiply
                const float fl = floorf(pos);
                w[i] = pos - fl;
                w1[i] = 1.0f - w[i];
                const uint32_t v0 = (uint32_t)fl;
                const uint32_t pi = BY_FEATURE_ROW ? kPi[i] : kPi2[i];
                const uint32_t po = BY_FEATURE_ROW ? kPi2[i] : kPi[i];
                a[i] = v0 * pi;
                b[i] = a[i] + pi;
                ao[i] = v0 * po;
                bo[i] = ao[i] + po;
            }
#pragma unroll
            for (int c = 0; c < (1 << D); ++c) {
                uint32_t h = 0;
#pragma unroll
                for (int i = 0; i < D; ++i) h ^= ((c >> i) & 1) ? b[i] : a[i];
                if ((h & slice_sel) == slice_val) accepted |= 1u << c;
            }
            // a corner with weight exactly zero (the point on a face of its cell) adds nothing: never emitted
#pragma unroll
            for (int i = 0; i < D; ++i) {
                uint32_t upper = 0;                                 // the corners whose bit i is set
#pragma unroll
                for (int c = 0; c < (1 << D); ++c) upper |= (uint32_t)((c >> i) & 1) << c;
                if (w[i] == 0.0f) accepted &= ~upper;
            }
            if (!valid) accepted = 0;
        }

        constexpr uint32_t kHalf = (1u << ((1 << D) / 2)) - 1u;     // low half of the corners
#pragma unroll 1
        for (int phase = 0; phase < (VERTEX ? 1 : 2); ++phase) {
            uint32_t pending = VERTEX ? accepted : phase == 0 ? (accepted & kHalf) : (accepted & ~kHalf);
            for (;;) {
                const bool     take = pending != 0;
                const uint64_t m = __ballot(take);
                if (m == 0) break;
                while (kRing - (tail - head) < 64u) {               // a round may add up to 64 references
                    wave_lds_fence();
                    if (mid == head) issue();                       // (then tail - mid >= kBatch)
                    complete();
                }
                if (take) {
                    const int c = __ffs(pending) - 1;
                    pending &= pending - 1;
                    uint32_t h = 0, ho = 0;
                    float    wt = 1.0f;
#pragma unroll
                    for (int i = 0; i < D; ++i) {
                        const bool up = (c >> i) & 1;
                        h ^= up ? b[i] : a[i];
                        ho ^= up ? bo[i] : ao[i];
                        wt *= up ? w[i] : w1[i];
                    }
                    const uint32_t i = (tail + lanes_below(m)) & (kRing - 1);
                    ring_key[i] = (h & row_lo_mask) | ((ho & other_mask) << sp.rows_log2);
                    ring_g[i] = make_float2(wt * g.x, wt * g.y);
                }
                tail += (uint32_t)__popcll(m);
            }
            pump();
        }
    }
    // drain: pad the last batch with references that add zero to row 0, then empty the pipeline
    {
        const uint32_t pad = (kBatch - (tail & (kBatch - 1))) & (kBatch - 1);
        if ((uint32_t)lane < pad) {
            const uint32_t i = (tail + lane) & (kRing - 1);
            ring_key[i] = 0u;
            ring_g[i] = make_float2(0.f, 0.f);
        }
        tail += pad;
    }
    while (head != tail) pump();
}

// ------------------------------------------------------------------ feature gradient
// Accumulators: two planes (f = 0, 1) of rows * NP doubles, so that the NP lanes of a reference
// add to NP consecutive doubles.
template <int D, int NP, bool VERTEX, typename GradT>
__device__ __forceinline__ void bwd_feat_sliced(
    const Params &p, const SliceParams &sp, const DenseLevels &dl, const uint32_t wg, unsigned char *smem,
    const float *__restrict__ x, const float *__restrict__ sigma, const GradT *__restrict__ grad,
    float *__restrict__ gD_f, const int64_t N)
{
    const uint32_t rows = 1u << sp.rows_log2;
    const uint32_t plane = rows * NP;
    double *acc = reinterpret_cast<double *>(smem);
    unsigned char *ring_mem = smem + (size_t)plane * 2 * sizeof(double);
    const SliceCoord co = slice_coord(sp, wg);
    const int l = co.level;
    if (co.index < 0) return;                                 // padding of the role's grid to 8 equal runs

    for (uint32_t i = threadIdx.x; i < plane * 2; i += kSlicedBlock) acc[i] = 0.0;
    __syncthreads();

    const float   *sig_l = sigma + (size_t)l * p.N_c * NP;
    const uint32_t k = (threadIdx.x & 63) % NP;
    const uint32_t row_lo_mask = rows - 1u, rows_log2 = sp.rows_log2;
    auto load = [&](const uint32_t key) -> float {
        return NP == 1 ? 1.0f : sig_l[(key >> rows_log2) * NP + k];
    };
    auto accum = [&](const uint32_t key, const float2 g, const float s) {
        double *a = acc + (key & row_lo_mask) * NP + k;
        atomicAdd(a, (double)(s * g.x));
        atomicAdd(a + plane, (double)(s * g.y));
    };
    if (VERTEX)   // grad = G: summed gradient per vertex of the dense levels' grids
        scan_chunk<D, NP, true, true, float>(p, sp, co, x, grad + (size_t)dl.g_off[co.index] * 2,
                                             (int64_t)dl.verts[co.index], dl.side[co.index], ring_mem, load, accum);
    else          // grad = level-major dL/dy
        scan_chunk<D, NP, true, false, float>(p, sp, co, x, grad + (size_t)l * N * 2, N, 0u, ring_mem, load, accum);
    __syncthreads();

    float *out = gD_f + (size_t)l * p.N_f * 2 + (size_t)co.slice * plane * 2;
    for (uint32_t i = threadIdx.x; i < plane * 2; i += kSlicedBlock) {     // i = (row * NP + k) * 2 + f
        const float v = (float)acc[(i & 1u) * plane + (i >> 1)];
        if (sp.store_direct) out[i] = v;
        else if (v != 0.0f) atomic_add(out + i, v);
    }
}

// ------------------------------------------------------------------ logit gradient
template <int D, int NP, bool VERTEX, typename FeatT, typename GradT>
__device__ __forceinline__ void bwd_logit_sliced(
    const Params &p, const SliceParams &sp, const DenseLevels &dl, const uint32_t wg, unsigned char *smem,
    const float *__restrict__ x, const FeatT *__restrict__ D_f, const float *__restrict__ sigma,
    const GradT *__restrict__ grad, float *__restrict__ gDhat_c, const int64_t N)
{
    const uint32_t rows = 1u << sp.rows_log2;
    double *acc = reinterpret_cast<double *>(smem);
    unsigned char *ring_mem = smem + (size_t)rows * NP * sizeof(double);
    const SliceCoord co = slice_coord(sp, wg);
    const int l = co.level;
    if (co.index < 0) return;

    for (uint32_t i = threadIdx.x; i < rows * NP; i += kSlicedBlock) acc[i] = 0.0;
    __syncthreads();

    const FeatT   *F_l = D_f + (size_t)l * p.N_f * 2;
    const uint32_t k = (threadIdx.x & 63) % NP;
    const uint32_t row_lo_mask = rows - 1u, rows_log2 = sp.rows_log2;
    using Raw = typename RawPair<FeatT>::type;                // the entry as loaded; converted when it is used
    auto load = [&](const uint32_t key) -> Raw {
        return reinterpret_cast<const Raw *>(F_l)[(key >> rows_log2) * NP + k];
    };
    auto accum = [&](const uint32_t key, const float2 g, const Raw raw) {
        const float2 feat = RawPair<FeatT>::to_float2(raw);
        atomicAdd(acc + (key & row_lo_mask) * NP + k, (double)fmaf(feat.x, g.x, feat.y * g.y));
    };
    if (VERTEX)
        scan_chunk<D, NP, false, true, Raw>(p, sp, co, x, grad + (size_t)dl.g_off[co.index] * 2,
                                            (int64_t)dl.verts[co.index], dl.side[co.index], ring_mem, load, accum);
    else
        scan_chunk<D, NP, false, false, Raw>(p, sp, co, x, grad + (size_t)l * N * 2, N, 0u, ring_mem, load, accum);
    __syncthreads();

    // softmax Jacobian per row, then out to HBM; NP consecutive lanes hold one row
    const size_t row0 = (size_t)l * p.N_c + (size_t)co.slice * rows;
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

// ------------------------------------------------------------------ per-vertex pre-reduction
// G[l][v][f] = sum over the corner references to vertex v of level l of weight * dL/dy[n, l, f], for the
// dense levels.  A workgroup owns kDenseSliceVerts consecutive vertices (row-major: dimension 0 fastest)
// of one level as fp64 accumulators in LDS and scans a chunk of the points; no hashing is involved.
template <int D, typename IoT>
__device__ __forceinline__ void bwd_vertex_grid(
    const Params &p, const DenseLevels &dl, const uint32_t chunks, const uint32_t chunk_pts, const int store_direct,
    uint32_t wg, unsigned char *smem, const float *__restrict__ x, const IoT *__restrict__ dyT,
    float *__restrict__ G, const int64_t N)
{
    double *acc = reinterpret_cast<double *>(smem);
    int l = 0;
    while (l < dl.count - 1 && wg >= dl.slices[l] * chunks) { wg -= dl.slices[l] * chunks; ++l; }
    const uint32_t slice = wg / chunks, chunk = wg % chunks;
    const uint32_t side = dl.side[l];
    const uint32_t first = slice * kDenseSliceVerts;
    const uint32_t count = dl.verts[l] - first < kDenseSliceVerts ? dl.verts[l] - first : kDenseSliceVerts;

    for (uint32_t i = threadIdx.x; i < count * 2; i += kSlicedBlock) acc[i] = 0.0;
    __syncthreads();

    const int64_t n0 = (int64_t)chunk * chunk_pts;
    const int64_t n1 = (n0 + chunk_pts < N) ? n0 + chunk_pts : N;
    const float   res = (float)p.N_l[l];
    const IoT    *dy_l = dyT + (size_t)l * N * 2;
    for (int64_t n = n0 + threadIdx.x; n < n1; n += kSlicedBlock) {
        float    w[D];
        uint32_t base = 0, stride = 1, step[D];
        {
#pragma clang fp contract(off)
#pragma unroll
            for (int i = 0; i < D; ++i) {
                const float pos = x[n * D + i] * res;               // one rounded fp32 multiply
                const float fl = floorf(pos);
                w[i] = pos - fl;
                base += (uint32_t)fl * stride;
                step[i] = stride;
                stride *= side;
            }
        }
        const float2 g = load_pair(dy_l, (size_t)n);
#pragma unroll
        for (int c = 0; c < (1 << D); ++c) {
            uint32_t v = base;
            float    wt = 1.0f;
#pragma unroll
            for (int i = 0; i < D; ++i) {
                const bool up = (c >> i) & 1;
                v += up ? step[i] : 0u;
                wt *= up ? w[i] : 1.0f - w[i];
            }
            const uint32_t rel = v - first;
            if (rel < count) {                                      // unsigned: also rejects v < first
                atomicAdd(acc + 2 * rel, (double)(wt * g.x));
                atomicAdd(acc + 2 * rel + 1, (double)(wt * g.y));
            }
        }
    }
    __syncthreads();

    float *out = G + ((size_t)dl.g_off[l] + first) * 2;
    for (uint32_t i = threadIdx.x; i < count * 2; i += kSlicedBlock) {
        const float v = (float)acc[i];
        if (store_direct) out[i] = v;
        else if (v != 0.0f) atomic_add(out + i, v);
    }
}

// ------------------------------------------------------------------ one kernel, five roles
// The grid lists, in this order, the workgroups of: logit gradient over points, feature gradient over
// points (hashed levels), logit gradient over vertices, feature gradient over vertices (dense levels),
// vertex-grid accumulation.  Sharing a launch keeps all CUs busy across the roles' different run times.
// The host launches it twice: points roles + vertex-grid accumulation (independent of each other), then
// the two vertex roles, which read the finished grid sums G.
enum { ROLE_LOGIT_PTS = 0, ROLE_FEAT_PTS, ROLE_LOGIT_VTX, ROLE_FEAT_VTX, ROLE_GRID, ROLE_COUNT };
struct BwdRoles {
    uint32_t    first[ROLE_COUNT + 1];      // first workgroup of each role (multiples of 8); [ROLE_COUNT] = grid size
    SliceParams sp[ROLE_COUNT];             // for ROLE_GRID only chunks, chunk_pts and store_direct are used
};

template <int D, int NP, typename FeatT, typename IoT>
__global__ __launch_bounds__(kSlicedBlock) void bwd_sliced_kernel(
    const Params p, const BwdRoles roles, const DenseLevels dl, const float *__restrict__ x,
    const FeatT *__restrict__ D_f, const float *__restrict__ sigma, const IoT *__restrict__ dyT,
    float *__restrict__ G, float *__restrict__ gD_f, float *__restrict__ gDhat_c, const int64_t N)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t wg = blockIdx.x;
    if (wg < roles.first[ROLE_FEAT_PTS]) {
        if (NP > 1)
            bwd_logit_sliced<D, NP, false, FeatT, IoT>(p, roles.sp[ROLE_LOGIT_PTS], dl, wg - roles.first[ROLE_LOGIT_PTS],
                                                       smem, x, D_f, sigma, dyT, gDhat_c, N);
    } else if (wg < roles.first[ROLE_LOGIT_VTX]) {
        bwd_feat_sliced<D, NP, false, IoT>(p, roles.sp[ROLE_FEAT_PTS], dl, wg - roles.first[ROLE_FEAT_PTS], smem, x,
                                           sigma, dyT, gD_f, N);
    } else if (wg < roles.first[ROLE_FEAT_VTX]) {
        if (NP > 1)
            bwd_logit_sliced<D, NP, true, FeatT, float>(p, roles.sp[ROLE_LOGIT_VTX], dl, wg - roles.first[ROLE_LOGIT_VTX],
                                                        smem, x, D_f, sigma, G, gDhat_c, N);
    } else if (wg < roles.first[ROLE_GRID]) {
        bwd_feat_sliced<D, NP, true, float>(p, roles.sp[ROLE_FEAT_VTX], dl, wg - roles.first[ROLE_FEAT_VTX], smem, x,
                                            sigma, G, gD_f, N);
    } else {
        const SliceParams &sp = roles.sp[ROLE_GRID];
        bwd_vertex_grid<D, IoT>(p, dl, sp.chunks, sp.chunk_pts, sp.store_direct, wg - roles.first[ROLE_GRID], smem, x,
                                dyT, G, N);
    }
}

}  // namespace cngp

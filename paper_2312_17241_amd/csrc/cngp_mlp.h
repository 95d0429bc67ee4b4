// Decoder after the encoding (Fig. 3: the interpolated features are fed into an MLP; Table 1: 64 hidden
// neurons).  Assumed, because the paper does not say: two hidden layers, ReLU, linear output, no biases.
//
//     h1 = relu(W1 y)   h2 = relu(W2 h1)   out = W3 h2        W1 [64, n_in], W2 [64, 64], W3 [n_out, 64]
//
// The only dense contraction of the method, hence the only user of the matrix cores here.  Everything is
// computed transposed, points along the columns: one wavefront owns 32 points and every layer is
//     (weights as the A operand, 32 x 16 per instruction) x (activations^T as the B operand, 16 x 32)
// with v_mfma_f32_32x32x16_f16.  The accumulator layout (lane = column, four consecutive rows per register
// group, the two halves of the wavefront four rows apart) feeds the next layer straight from registers:
// after ReLU and rounding to fp16, accumulator registers 4j .. 4j+3 of row tile t hold rows
// 32t + 8j + 4h .. + 3 (h = lane / 32), a "quarter step"; two quarter steps 2s', 2s'+1 side by side are
// this lane's eight B values of K-step s'.  That is not the instruction's natural K order (rows
// 16s' + 8h .. + 7) but a permutation of it inside the step, and a contraction does not care about the
// order of its terms as long as both operands use the same one: the weights are staged in LDS in that
// order.  Only the weight gradients, which contract over the points, need a transpose; it goes through a
// per-wavefront tile in LDS.
#pragma once
#include "cngp_bwd_sliced.h"   // wave_lds_fence

namespace cngp {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float    acc16_t __attribute__((ext_vector_type(16)));

constexpr int kMlpHidden = 64;
constexpr int kMlpBlock = 256;                 // 4 wavefronts
constexpr int kMlpMaxIn = 32, kMlpMaxOut = 16;

struct MlpDims {
    int n_in, n_out;
    int ks1;                                   // quarter steps (8 rows) of layer 1: ceil(n_in / 8)
    int ks3;                                   // quarter steps of the transposed output layer: ceil(n_out / 8)
    int vec_in, vec_out;                       // rows of y (and dL/dy) / of dL/dout can be read four values at a time
};

// Slots of the weight operands in LDS, counted in quarter steps (one half4 per lane: rows 8s + 4h .. + 3 of the
// contraction).  Slots 2p and 2p + 1 lie side by side per lane, so that operand p of an instruction is one
// 16-byte read: half8 number p * 64 + lane.
enum : int { kOpW1 = 0, kOpW2 = 8, kOpW3 = 24, kOpW3T = 32, kOpW2T = 36, kOpW1T = 52, kOpFwdSlots = 32, kOpAllSlots = 60 };

__device__ __forceinline__ half8_t cat(const half4_t lo, const half4_t hi) {
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
__device__ __forceinline__ acc16_t mfma(const half8_t a, const half8_t b, const acc16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ acc16_t acc_zero() {
    acc16_t z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.0f;
    return z;
}

// A-operand element (row i, column k) of a matrix stored row-major [rows, cols] (or its transpose).
__device__ __forceinline__ _Float16 w_at(const __half *W, int rows, int cols, bool transposed, int i, int k) {
    const int r = transposed ? k : i, c = transposed ? i : k;
    return (r < rows && c < cols) ? (_Float16)__half2float(W[r * cols + c]) : (_Float16)0.0f;
}

// Fills `slots` operand slots, the work spread over the workgroup.  The weights first come into LDS as
// they are, with wide coalesced loads (`raw`: room for weight_count halves, 16-byte aligned, may be reused
// after the barrier at the end); building the operand layout from global memory element by element is a
// chain of dependent cache round trips that costs more than the whole forward pass of a small batch.
__device__ __forceinline__ void stage_operands(half8_t *ops8, __half *raw, const __half *W, const MlpDims d,
                                               const int slots) {
    half4_t *ops = reinterpret_cast<half4_t *>(ops8);
    const int count = kMlpHidden * d.n_in + kMlpHidden * kMlpHidden + kMlpHidden * d.n_out;
    if ((reinterpret_cast<uintptr_t>(W) & 15u) == 0) {
        for (int i = threadIdx.x * 8; i < count; i += kMlpBlock * 8) {
            if (i + 8 <= count) *reinterpret_cast<uint4 *>(raw + i) = *reinterpret_cast<const uint4 *>(W + i);
            else for (int j = i; j < count; ++j) raw[j] = W[j];
        }
    } else {
        for (int i = threadIdx.x; i < count; i += kMlpBlock) raw[i] = W[i];
    }
    __syncthreads();
    const __half *W1 = raw, *W2 = raw + kMlpHidden * d.n_in, *W3 = W2 + kMlpHidden * kMlpHidden;
    for (int e = threadIdx.x; e < slots * 64; e += kMlpBlock) {
        const int slot = e >> 6, lane = e & 63, row = lane & 31, k4 = 4 * (lane >> 5);
        const __half *M;
        int  rows, cols, t, s;
        bool tr;
        if (slot < kOpW2)       { M = W1; rows = kMlpHidden; cols = d.n_in;      tr = false; t = (slot - kOpW1) >> 2;  s = (slot - kOpW1) & 3; }
        else if (slot < kOpW3)  { M = W2; rows = kMlpHidden; cols = kMlpHidden;  tr = false; t = (slot - kOpW2) >> 3;  s = (slot - kOpW2) & 7; }
        else if (slot < kOpW3T) { M = W3; rows = d.n_out;    cols = kMlpHidden;  tr = false; t = 0;                    s = slot - kOpW3; }
        else if (slot < kOpW2T) { M = W3; rows = d.n_out;    cols = kMlpHidden;  tr = true;  t = (slot - kOpW3T) >> 1; s = (slot - kOpW3T) & 1; }
        else if (slot < kOpW1T) { M = W2; rows = kMlpHidden; cols = kMlpHidden;  tr = true;  t = (slot - kOpW2T) >> 3; s = (slot - kOpW2T) & 7; }
        else                    { M = W1; rows = kMlpHidden; cols = d.n_in;      tr = true;  t = 0;                    s = slot - kOpW1T; }
        half4_t v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = w_at(M, rows, cols, tr, 32 * t + row, 8 * s + k4 + j);
        ops[(((slot >> 1) * 64 + lane) << 1) + (slot & 1)] = v;
    }
    __syncthreads();
}

template <typename T> __device__ __forceinline__ float to_float(T v);
template <> __device__ __forceinline__ float to_float<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_float<__half>(__half v) { return __half2float(v); }
template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ __half from_float<__half>(float v) { return __float2half_rn(v); }

// B operand of K-step s from a row-major [N, cols] array: this lane's point, columns k0 .. k0 + 3.
// `vec`: cols is a multiple of four and the array 16-byte aligned, so the four values are one load.
__device__ __forceinline__ half4_t load_b(const __half *__restrict__ a, const int64_t pt, const int64_t N,
                                          const int cols, const int k0, const bool vec) {
    half4_t v;
    if (vec) {
        if (pt < N && k0 < cols) return *reinterpret_cast<const half4_t *>(a + pt * cols + k0);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (_Float16)0.0f;
        return v;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
        v[j] = (pt < N && k0 + j < cols) ? (_Float16)__half2float(a[pt * cols + k0 + j]) : (_Float16)0.0f;
    return v;
}
__device__ __forceinline__ half4_t load_b(const float *__restrict__ a, const int64_t pt, const int64_t N,
                                          const int cols, const int k0, const bool vec) {
    half4_t v;
    float4  f = make_float4(0.f, 0.f, 0.f, 0.f);
    if (vec) {
        if (pt < N && k0 < cols) f = *reinterpret_cast<const float4 *>(a + pt * cols + k0);
    } else {
        if (pt < N && k0 + 0 < cols) f.x = a[pt * cols + k0 + 0];
        if (pt < N && k0 + 1 < cols) f.y = a[pt * cols + k0 + 1];
        if (pt < N && k0 + 2 < cols) f.z = a[pt * cols + k0 + 2];
        if (pt < N && k0 + 3 < cols) f.w = a[pt * cols + k0 + 3];
    }
    v[0] = (_Float16)f.x; v[1] = (_Float16)f.y; v[2] = (_Float16)f.z; v[3] = (_Float16)f.w;
    return v;
}

__device__ __forceinline__ void store4(float *p, float a, float b, float c, float e) {
    *reinterpret_cast<float4 *>(p) = make_float4(a, b, c, e);
}
__device__ __forceinline__ void store4(__half *p, float a, float b, float c, float e) {
    half4_t v;
    v[0] = (_Float16)a; v[1] = (_Float16)b; v[2] = (_Float16)c; v[3] = (_Float16)e;
    *reinterpret_cast<half4_t *>(p) = v;
}

// ReLU, rounding to fp16, and the re-use of an accumulator tile as B operands of the next layer.
__device__ __forceinline__ void relu_to_b(const acc16_t a, half4_t (&b)[8], const int t) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        half4_t v;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = (_Float16)fmaxf(a[4 * j + q], 0.0f);
        b[4 * t + j] = v;
    }
}

// Same for a gradient tile: entries whose forward pre-activation was not positive are dropped.
__device__ __forceinline__ void mask_to_b(const acc16_t g, const uint32_t mask, half4_t (&b)[8], const int t) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        half4_t v;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = ((mask >> (4 * j + q)) & 1u) ? (_Float16)g[4 * j + q] : (_Float16)0.0f;
        b[4 * t + j] = v;
    }
}

__device__ __forceinline__ uint32_t positive_mask(const acc16_t a) {
    uint32_t m = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) m |= (a[r] > 0.0f ? 1u : 0u) << r;
    return m;
}

// Layers 1 and 2 for this wavefront's 32 points.
struct Hidden {
    half4_t  yb[4], h1[8], h2[8];
    uint32_t m1[2], m2[2];
};

// This lane's part of the inputs of one tile of 32 points (the B operands of layer 1).
template <typename IoT>
__device__ __forceinline__ void load_inputs(const MlpDims d, const IoT *__restrict__ y, const int64_t pt,
                                            const int64_t N, const int lane, half4_t (&yb)[4]) {
    const int k4 = 4 * (lane >> 5);
#pragma unroll
    for (int s = 0; s < 4; ++s) yb[s] = load_b(y, pt, N, d.n_in, 8 * s + k4, d.vec_in != 0);
}

// The same from a level-major array yT[n_in / 2][N] of fp16 pairs (what the level-resident forward of the encoding
// writes before its rows kernel): four halves of a row are two neighbouring planes' pairs, and the 32 lanes of a
// tile read 128 contiguous bytes of each plane.
__device__ __forceinline__ void load_inputs_planes(const MlpDims d, const uint32_t *__restrict__ yT, const int64_t pt,
                                                   const int64_t N, const int lane, half4_t (&yb)[4]) {
    const int k2 = 2 * (lane >> 5);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int l0 = 4 * s + k2;
        uint2 v = make_uint2(0u, 0u);
        if (pt < N) {
            if (2 * l0 < d.n_in) v.x = yT[(size_t)l0 * (size_t)N + (size_t)pt];
            if (2 * l0 + 2 < d.n_in) v.y = yT[(size_t)(l0 + 1) * (size_t)N + (size_t)pt];
        }
        yb[s] = *reinterpret_cast<const half4_t *>(&v);
    }
}

// H.yb holds the inputs on entry.
__device__ __forceinline__ void hidden_layers(const half8_t *ops, const MlpDims d, const int lane, Hidden &H) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        acc16_t a = acc_zero();
#pragma unroll
        for (int s = 0; s < 2; ++s)
            if (2 * s < d.ks1) a = mfma(ops[(kOpW1 / 2 + 2 * t + s) * 64 + lane], cat(H.yb[2 * s], H.yb[2 * s + 1]), a);
        H.m1[t] = positive_mask(a);
        relu_to_b(a, H.h1, t);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        acc16_t a = acc_zero();
#pragma unroll
        for (int s = 0; s < 4; ++s) a = mfma(ops[(kOpW2 / 2 + 4 * t + s) * 64 + lane], cat(H.h1[2 * s], H.h1[2 * s + 1]), a);
        H.m2[t] = positive_mask(a);
        relu_to_b(a, H.h2, t);
    }
}

// Per-wavefront transpose tile: rows = input dimensions / neurons / output channels, 32 points per row,
// rows padded to 36 halves so that the 8-byte operand reads of 32 lanes fall into different banks.
constexpr int kTileStride = 36;
enum : int { kRowY = 0, kRowH1 = 32, kRowH2 = 96, kRowD1 = 160, kRowD2 = 224, kRowDo = 288, kTileRows = 320 };
constexpr size_t kMlpBwdLds = (size_t)kOpAllSlots * 64 * sizeof(half4_t) +
                              (size_t)(kMlpBlock / 64) * kTileRows * kTileStride * sizeof(_Float16);
constexpr size_t kMlpRawBytes = ((size_t)kMlpHidden * (kMlpMaxIn + kMlpHidden + kMlpMaxOut) * 2 + 15) & ~(size_t)15;
constexpr size_t kMlpFwdOps = (size_t)kOpFwdSlots * 64 * sizeof(half4_t);
constexpr size_t kMlpFwdLds = kMlpFwdOps + kMlpRawBytes;
constexpr size_t kMlpAccBytes = (size_t)8 * 16 * 64 * sizeof(float);        // one wavefront's weight-gradient registers
static_assert(kMlpRawBytes <= (size_t)(kMlpBlock / 64) * kTileRows * kTileStride * sizeof(_Float16), "raw weights share the tile region");
static_assert(kMlpAccBytes <= (size_t)(kMlpBlock / 64) * kTileRows * kTileStride * sizeof(_Float16), "the reduction shares the tile region");

// ------------------------------------------------------------------ forward
// PLANES: y is the level-major array of fp16 pairs described at load_inputs_planes (IoT = __half, n_in even).
template <typename IoT, bool PLANES = false>
__global__ __launch_bounds__(kMlpBlock) void mlp_fwd_kernel(
    const MlpDims d, const IoT *__restrict__ y, const int64_t N, const __half *__restrict__ W,
    float *__restrict__ out, const int64_t tiles)
{
    auto fetch = [&](const int64_t pt, const int lane, half4_t (&yb)[4]) {
        if constexpr (PLANES) load_inputs_planes(d, reinterpret_cast<const uint32_t *>(y), pt, N, lane, yb);
        else load_inputs(d, y, pt, N, lane, yb);
    };
    extern __shared__ __align__(16) unsigned char smem[];
    half8_t *ops = reinterpret_cast<half8_t *>(smem);
    stage_operands(ops, reinterpret_cast<__half *>(smem + kMlpFwdOps), W, d, kOpFwdSlots);
    const int lane = threadIdx.x & 63, k4 = 4 * (lane >> 5);
    const int64_t waves = (int64_t)gridDim.x * (kMlpBlock / 64);
    int64_t tile = (int64_t)blockIdx.x * (kMlpBlock / 64) + (threadIdx.x >> 6);
    half4_t next[4];
    fetch(tile * 32 + (lane & 31), lane, next);
    for (; tile < tiles; tile += waves) {
        const int64_t pt = tile * 32 + (lane & 31);
        Hidden H;
#pragma unroll
        for (int s = 0; s < 4; ++s) H.yb[s] = next[s];
        fetch((tile + waves) * 32 + (lane & 31), lane, next);                    // next tile, in flight during this one
        hidden_layers(ops, d, lane, H);
        acc16_t o = acc_zero();
#pragma unroll
        for (int s = 0; s < 4; ++s) o = mfma(ops[(kOpW3 / 2 + s) * 64 + lane], cat(H.h2[2 * s], H.h2[2 * s + 1]), o);
        if (pt < N) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {                       // rows 0 .. 15 of the tile are the outputs
                const int ch = 8 * (r >> 2) + k4 + (r & 3);
                if (ch < d.n_out) out[pt * d.n_out + ch] = o[r];
            }
        }
    }
}

// ------------------------------------------------------------------ encoding + decoder in one kernel (inference)
// The forward tile kernel of the encoding (cngp_kernels.h: 256 points per workgroup through all levels,
// the level's index codebook staged in LDS) with the decoder applied to the tile while it is still in LDS:
// the encoded features never go to memory.  y is kept as fp16, the value the decoder's matrix
// instructions would read from a stored y of either type, so the result equals the two separate calls.
// Row stride of the tile: 36 halves (the operand reads of 32 lanes then fall into different banks);
// columns from 2 L on are zero, which is what the K-steps beyond n_in need.
constexpr int kFusedTile = 256;
constexpr int kFusedStride = 36;

template <int D, typename FeatT, int FMT>
__global__ __launch_bounds__(kFusedTile) void encode_mlp_fwd_kernel(
    const Params p, const MlpDims d, const float *__restrict__ x, const FeatT *__restrict__ D_f,
    const uint8_t *__restrict__ D_c, const __half *__restrict__ W, float *__restrict__ out, const int64_t N,
    const int64_t tiles, const uint32_t c_stride, const int vec)
{
    extern __shared__ __align__(16) unsigned char smem[];
    half8_t  *ops = reinterpret_cast<half8_t *>(smem);
    _Float16 *ytile = reinterpret_cast<_Float16 *>(smem + kMlpFwdOps);                      // [kFusedTile][kFusedStride]
    unsigned char *rest = smem + kMlpFwdOps + (size_t)kFusedTile * kFusedStride * sizeof(_Float16);
    uint8_t  *probes = rest;                                 // the raw weights first, then each level's index codebook
    const uint32_t lds_c = (p.N_c + 1u) / 2u;
    stage_operands(ops, reinterpret_cast<__half *>(rest), W, d, kOpFwdSlots);
    const int t = threadIdx.x;
    for (int i = t; i < kFusedTile * kFusedStride; i += kFusedTile) ytile[i] = (_Float16)0.0f;
    const int lane = t & 63, k4 = 4 * (lane >> 5);

    // persistent: a workgroup stages the decoder's weights once and then walks over tiles of points
    for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int64_t n0 = tile * kFusedTile;
        const int64_t n = n0 + t;
        const bool    valid = n < N;
        float xp[D];
#pragma unroll
        for (int j = 0; j < D; ++j) xp[j] = valid ? x[n * D + j] : 0.0f;

        for (int l = 0; l < p.L; ++l) {
            const uint8_t *C_l = D_c + (size_t)l * c_stride;
            __syncthreads();                                 // previous lookups, previous tile's decoder reads, the clearing above
            stage_probes<FMT, kFusedTile>(probes, C_l, c_stride, lds_c, vec, t);
            __syncthreads();
            Cell<D> cell;
            cell.locate(xp, p.N_l[l]);
            const FeatT *F_l = D_f + (size_t)l * p.N_f * 2;
            uint32_t idx[1 << D];
#pragma unroll
            for (int c = 0; c < (1 << D); ++c)
                idx[c] = probe_base(cell.hash1(c), p) +
                         (FMT == kFmtBits ? read_probe_bits_lds(probes, cell.hash2(c) & p.c_mask, p.log2_Np)
                                          : read_probe<kFmtPacked4>(probes, cell.hash2(c) & p.c_mask, p.log2_Np));
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
            ytile[t * kFusedStride + 2 * l] = (_Float16)y0;
            ytile[t * kFusedStride + 2 * l + 1] = (_Float16)y1;
        }
        wave_lds_fence();                                    // a wavefront decodes the rows it wrote itself

        // decoder: every wavefront takes its own 64 points as two tiles of 32
#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            const int row = (t & ~63) + 32 * half + (lane & 31);
            Hidden H;
#pragma unroll
            for (int s = 0; s < 4; ++s)
                H.yb[s] = *reinterpret_cast<const half4_t *>(ytile + row * kFusedStride + 8 * s + k4);
            hidden_layers(ops, d, lane, H);
            acc16_t o = acc_zero();
#pragma unroll
            for (int s = 0; s < 4; ++s) o = mfma(ops[(kOpW3 / 2 + s) * 64 + lane], cat(H.h2[2 * s], H.h2[2 * s + 1]), o);
            const int64_t pt = n0 + row;
            if (pt < N) {
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const int ch = 8 * (r >> 2) + k4 + (r & 3);
                    if (ch < d.n_out) out[pt * d.n_out + ch] = o[r];
                }
            }
        }
    }
}

// ------------------------------------------------------------------ backward
// B-layout registers (lane = point, K-step s holds rows 8s + 4h .. + 3) written as rows of the tile.
template <int STEPS>
__device__ __forceinline__ void put_rows(_Float16 *tile, const int row0, const half4_t (&b)[STEPS], const int lane) {
    const int p = lane & 31, k4 = 4 * (lane >> 5);
#pragma unroll
    for (int s = 0; s < STEPS; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) tile[(row0 + 8 * s + k4 + j) * kTileStride + p] = b[s][j];
}

// Operand whose K index runs over the 32 points: row 32u + lane % 32, points 16s + 8h .. + 7 (both operands of
// these products come from the tile, so the instruction's natural K order serves).
__device__ __forceinline__ half8_t get_op(const _Float16 *tile, const int row0, const int u, const int s, const int lane) {
    const _Float16 *q = tile + (row0 + 32 * u + (lane & 31)) * kTileStride + 16 * s + 8 * (lane >> 5);
    return cat(*reinterpret_cast<const half4_t *>(q), *reinterpret_cast<const half4_t *>(q + 4));
}

template <typename IoT>
__global__ __launch_bounds__(kMlpBlock) void mlp_bwd_kernel(
    const MlpDims d, const IoT *__restrict__ y, const int64_t N, const __half *__restrict__ W,
    const float *__restrict__ dout, IoT *__restrict__ dy, float *__restrict__ gW, const int64_t tiles)
{
    extern __shared__ __align__(16) unsigned char smem[];
    half8_t  *ops = reinterpret_cast<half8_t *>(smem);
    _Float16 *tile = reinterpret_cast<_Float16 *>(smem + (size_t)kOpAllSlots * 64 * sizeof(half4_t)) +
                     (size_t)(threadIdx.x >> 6) * kTileRows * kTileStride;
    stage_operands(ops, reinterpret_cast<__half *>(smem + (size_t)kOpAllSlots * 64 * sizeof(half4_t)), W, d, kOpAllSlots);
    const int lane = threadIdx.x & 63, k4 = 4 * (lane >> 5);
    for (int i = lane; i < kTileRows * kTileStride; i += 64) tile[i] = (_Float16)0.0f;   // padding rows stay zero
    __syncthreads();

    acc16_t gW1[2], gW2[2][2], gW3[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        gW1[t] = acc_zero(); gW3[t] = acc_zero();
        gW2[t][0] = acc_zero(); gW2[t][1] = acc_zero();
    }

    const int64_t waves = (int64_t)gridDim.x * (kMlpBlock / 64);
    int64_t tl = (int64_t)blockIdx.x * (kMlpBlock / 64) + (threadIdx.x >> 6);
    half4_t next[4], next_db[2];
    load_inputs(d, y, tl * 32 + (lane & 31), N, lane, next);
#pragma unroll
    for (int s = 0; s < 2; ++s) next_db[s] = load_b(dout, tl * 32 + (lane & 31), N, d.n_out, 8 * s + k4, d.vec_out != 0);
    for (; tl < tiles; tl += waves) {
        const int64_t pt = tl * 32 + (lane & 31);
        Hidden H;
        half4_t db[2], dh2[8], dh1[8];
#pragma unroll
        for (int s = 0; s < 4; ++s) H.yb[s] = next[s];
#pragma unroll
        for (int s = 0; s < 2; ++s) db[s] = next_db[s];
        load_inputs(d, y, (tl + waves) * 32 + (lane & 31), N, lane, next);       // next tile, in flight during this one
#pragma unroll
        for (int s = 0; s < 2; ++s)
            next_db[s] = load_b(dout, (tl + waves) * 32 + (lane & 31), N, d.n_out, 8 * s + k4, d.vec_out != 0);
        hidden_layers(ops, d, lane, H);

#pragma unroll
        for (int t = 0; t < 2; ++t) {                           // dL/dh2 = W3^T dout, where h2 was active
            acc16_t g = acc_zero();
            g = mfma(ops[(kOpW3T / 2 + t) * 64 + lane], cat(db[0], db[1]), g);   // rows beyond n_out are zero in both operands
            mask_to_b(g, H.m2[t], dh2, t);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {                           // dL/dh1 = W2^T dL/dh2, where h1 was active
            acc16_t g = acc_zero();
#pragma unroll
            for (int s = 0; s < 4; ++s) g = mfma(ops[(kOpW2T / 2 + 4 * t + s) * 64 + lane], cat(dh2[2 * s], dh2[2 * s + 1]), g);
            mask_to_b(g, H.m1[t], dh1, t);
        }
        {                                                       // dL/dy = W1^T dL/dh1
            acc16_t g = acc_zero();
#pragma unroll
            for (int s = 0; s < 4; ++s) g = mfma(ops[(kOpW1T / 2 + s) * 64 + lane], cat(dh1[2 * s], dh1[2 * s + 1]), g);
            if (pt < N) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {                   // register group q: input dimensions 8q + 4h .. + 3
                    const int i = 8 * q + k4;
                    if (d.vec_in && i < d.n_in) {
                        store4(dy + pt * d.n_in + i, g[4 * q], g[4 * q + 1], g[4 * q + 2], g[4 * q + 3]);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (i + j < d.n_in) dy[pt * d.n_in + i + j] = from_float<IoT>(g[4 * q + j]);
                    }
                }
            }
        }

        // weight gradients contract over the points: transpose through the tile
        wave_lds_fence();                                       // the previous tile's operand reads are done
        put_rows<4>(tile, kRowY, H.yb, lane);
        put_rows<8>(tile, kRowH1, H.h1, lane);
        put_rows<8>(tile, kRowH2, H.h2, lane);
        put_rows<8>(tile, kRowD1, dh1, lane);
        put_rows<8>(tile, kRowD2, dh2, lane);
        put_rows<2>(tile, kRowDo, db, lane);
        wave_lds_fence();
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const half8_t yT = get_op(tile, kRowY, 0, s, lane), doT = get_op(tile, kRowDo, 0, s, lane);
            half8_t h1T[2], h2T[2], d1T[2], d2T[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                h1T[u] = get_op(tile, kRowH1, u, s, lane);
                h2T[u] = get_op(tile, kRowH2, u, s, lane);
                d1T[u] = get_op(tile, kRowD1, u, s, lane);
                d2T[u] = get_op(tile, kRowD2, u, s, lane);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                gW1[t] = mfma(d1T[t], yT, gW1[t]);              // [hidden 32t.., input dim]
                gW3[t] = mfma(doT, h2T[t], gW3[t]);             // [channel, hidden 32t..]
#pragma unroll
                for (int u = 0; u < 2; ++u) gW2[t][u] = mfma(d2T[t], h1T[u], gW2[t][u]);   // [hidden 32t.., hidden 32u..]
            }
        }
    }

    // Sum over the workgroup's wavefronts in LDS (plain read-add-write, one wavefront after the other; the
    // tile region is free now), then one set of global atomics per workgroup.
    // Register r of accumulator a, lane l lives at red[(a * 16 + r) * 64 + l].
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem + (size_t)kOpAllSlots * 64 * sizeof(half4_t));
    const int wave = threadIdx.x >> 6;
    for (int w = 0; w < kMlpBlock / 64 - 1; ++w) {
        if (wave == w) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    float *p1 = red + ((0 + t) * 16 + r) * 64 + lane, *p3 = red + ((2 + t) * 16 + r) * 64 + lane;
                    *p1 = (w == 0 ? 0.0f : *p1) + gW1[t][r];
                    *p3 = (w == 0 ? 0.0f : *p3) + gW3[t][r];
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        float *p2 = red + ((4 + 2 * t + u) * 16 + r) * 64 + lane;
                        *p2 = (w == 0 ? 0.0f : *p2) + gW2[t][u][r];
                    }
                }
            }
        }
        __syncthreads();
    }
    if (wave != kMlpBlock / 64 - 1) return;
    // lane = column, registers = rows 8 (r / 4) + 4 h + r % 4
    float *g1 = gW, *g2 = gW + kMlpHidden * d.n_in, *g3 = g2 + kMlpHidden * kMlpHidden;
    const int col = lane & 31;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + k4 + (r & 3);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const float v1 = gW1[t][r] + red[((0 + t) * 16 + r) * 64 + lane];
            const float v3 = gW3[t][r] + red[((2 + t) * 16 + r) * 64 + lane];
            if (col < d.n_in && v1 != 0.0f) atomic_add(g1 + (32 * t + row) * d.n_in + col, v1);
            if (row < d.n_out && v3 != 0.0f) atomic_add(g3 + row * kMlpHidden + 32 * t + col, v3);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const float v2 = gW2[t][u][r] + red[((4 + 2 * t + u) * 16 + r) * 64 + lane];
                if (v2 != 0.0f) atomic_add(g2 + (32 * t + row) * kMlpHidden + 32 * u + col, v2);
            }
        }
    }
}

}  // namespace cngp

// Optimiser step fused with the bake (Fig. 3: D_c is re-derived from D^_c after every training
// step).  One streaming launch updates the feature codebook and the confidence values with Adam
// (an assumption: the paper names no optimiser) and, while a row of updated confidence values is
// still in registers, takes its argmax and writes D_c -- the separate pass of the bake over D^_c
// disappears.  HBM-bound: every array is read and written exactly once, 16 bytes per lane.
#pragma once
#include "cngp_device.h"

namespace cngp {

constexpr int kOptBlock = 256;

struct AdamCoef {
    float b1, one_minus_b1, b2, one_minus_b2;
    float step;        // lr / (1 - beta1^t)
    float rsqrt_c2;    // 1 / sqrt(1 - beta2^t)
    float eps;
    float grad_scale;  // the gradient is multiplied by this before use
};

struct AdamTable {
    AdamCoef a;
    float   *theta, *m, *v, *grad;
    int64_t  n;        // entries
};

struct Quad { float e[4]; };

// Four consecutive floats starting at entry i (a multiple of 4); entries at or beyond n read as 0.
__device__ __forceinline__ Quad load_quad(const float *__restrict__ p, const int64_t i, const int64_t n) {
    Quad q;
    if (i + 4 <= n) {
        const float4 t = *reinterpret_cast<const float4 *>(p + i);
        q.e[0] = t.x; q.e[1] = t.y; q.e[2] = t.z; q.e[3] = t.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) q.e[k] = (i + k < n) ? p[i + k] : 0.0f;
    }
    return q;
}

__device__ __forceinline__ void store_quad(float *__restrict__ p, const int64_t i, const int64_t n, const Quad &q) {
    if (i + 4 <= n) {
        *reinterpret_cast<float4 *>(p + i) = make_float4(q.e[0], q.e[1], q.e[2], q.e[3]);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + k < n) p[i + k] = q.e[k];
    }
}

// Adam on four entries of one table; returns the updated parameters (also stored).
__device__ __forceinline__ Quad adam_quad(const AdamTable &t, const int64_t i, const bool clear_grad) {
    Quad th = load_quad(t.theta, i, t.n);
    Quad m  = load_quad(t.m, i, t.n);
    Quad v  = load_quad(t.v, i, t.n);
    const Quad g = load_quad(t.grad, i, t.n);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float gk = g.e[k] * t.a.grad_scale;
        m.e[k] = t.a.b1 * m.e[k] + t.a.one_minus_b1 * gk;
        v.e[k] = t.a.b2 * v.e[k] + t.a.one_minus_b2 * (gk * gk);
        th.e[k] -= t.a.step * m.e[k] / (sqrtf(v.e[k]) * t.a.rsqrt_c2 + t.a.eps);
    }
    store_quad(t.theta, i, t.n, th);
    store_quad(t.m, i, t.n, m);
    store_quad(t.v, i, t.n, v);
    if (clear_grad) {
        Quad z; z.e[0] = z.e[1] = z.e[2] = z.e[3] = 0.0f;
        store_quad(t.grad, i, t.n, z);
    }
    return th;
}

// Workgroups [0, blocks_f) update the feature codebook, the rest the confidence values.
// Each lane owns four consecutive entries.  A row of D^_c (N_p values) spans N_p / 4 neighbouring
// lanes (or a lane holds 4 / N_p whole rows): the argmax is taken per lane, then combined over the
// lanes of the row with the rule of the bake (first maximum wins, NaN never wins, no valid value: 0).
template <int NP, bool PACKED4>
__global__ __launch_bounds__(kOptBlock) void adam_step_bake_kernel(
    const AdamTable f, const AdamTable c, __half *__restrict__ D_f_half, uint8_t *__restrict__ D_c,
    const uint32_t blocks_f, const int clear_grad)
{
    if (blockIdx.x < blocks_f) {
        const int64_t i = ((int64_t)blockIdx.x * kOptBlock + threadIdx.x) * 4;
        if (i >= f.n) return;
        const Quad th = adam_quad(f, i, clear_grad != 0);
        if (D_f_half) {
            if (i + 4 <= f.n) {
                __half2 *o = reinterpret_cast<__half2 *>(D_f_half + i);
                o[0] = __floats2half2_rn(th.e[0], th.e[1]);
                o[1] = __floats2half2_rn(th.e[2], th.e[3]);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (i + k < f.n) D_f_half[i + k] = __float2half_rn(th.e[k]);
            }
        }
        return;
    }

    // confidence values; every lane of the wave stays active for the cross-lane steps below
    const int64_t q = (int64_t)(blockIdx.x - blocks_f) * kOptBlock + threadIdx.x;
    const int64_t i = q * 4;
    const bool    live = i < c.n;
    Quad th;
    if (live) th = adam_quad(c, i, clear_grad != 0);
    const int64_t rows = c.n / NP;

    if constexpr (NP >= 4) {
        constexpr int G = NP / 4;                         // lanes per row
        uint32_t best = 0;
        bool     have = false;
        float    bv = 0.0f;
        if (live) {
            const uint32_t k0 = (uint32_t)(q & (G - 1)) * 4u;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float val = th.e[k];
                if ((val == val) && (!have || val > bv)) { best = k0 + k; bv = val; have = true; }
            }
        }
#pragma unroll
        for (int s = 1; s < G; s <<= 1) {
            const float    ov = __shfl_xor(bv, s);
            const uint32_t ob = (uint32_t)__shfl_xor((int)best, s);
            const bool     oh = __shfl_xor((int)have, s) != 0;
            const bool take = oh && (!have || ov > bv || (ov == bv && ob < best));
            if (take) { best = ob; bv = ov; have = true; }
        }
        const int64_t row = q / G;
        if (PACKED4) {
            const uint32_t hi = (uint32_t)__shfl_down((int)best, G);      // the next row's result
            if (live && (q & (2 * G - 1)) == 0) D_c[row >> 1] = (uint8_t)(best | (hi << 4));
        } else {
            if (live && (q & (G - 1)) == 0) D_c[row] = (uint8_t)best;
        }
    } else {
        constexpr int R = 4 / NP;                         // whole rows per lane
        if (!live) return;
        uint32_t res[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            uint32_t best = 0;
            if (NP == 2) {
                const float a = th.e[2 * r], b = th.e[2 * r + 1];
                best = ((b == b) && (!(a == a) || b > a)) ? 1u : 0u;
            }
            res[r] = best;
        }
        const int64_t row0 = q * R;
        if (PACKED4) {
#pragma unroll
            for (int r = 0; r < R; r += 2)
                if (row0 + r < rows) D_c[(row0 + r) >> 1] = (uint8_t)(res[r] | (res[r + 1] << 4));
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (row0 + r < rows) D_c[row0 + r] = (uint8_t)res[r];
        }
    }
}

}  // namespace cngp

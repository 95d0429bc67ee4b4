// Device-side building blocks shared by the gfx950 kernels: grid-cell location,
// the two spatial hashes (Eq. 3) and the probed feature index (Eq. 6).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace cngp {

constexpr int kMaxLevels = 32;
constexpr int kBlock = 256;          // threads per workgroup = 4 wavefronts of 64

// Eq. 3: hash(v) = XOR_i v_i * pi_i in uint32.  pi: the primes of the hash encoding the
// method generalises (pi_0 = 1); pi2: a second, disjoint set for hash2 (Sec. 3).
// The fourth entries serve a fourth input dimension (the paper's experiments stop at three): the next primes
// above 2^32 / sqrt(5) and 2^32 / sqrt(3).
__device__ constexpr uint32_t kPi[4]  = {1u, 2654435761u, 805459861u, 1920767767u};
__device__ constexpr uint32_t kPi2[4] = {1580030173u, 1367130559u, 3037000507u, 2479700537u};

// Everything a kernel needs to know about the encoding, passed by value.
struct Params {
    uint32_t N_l[kMaxLevels];   // grid resolution per level
    int32_t  L;
    int32_t  L_loaded;          // forward only: levels from here on are not loaded and encode to zero (level-of-detail streaming)
    uint32_t N_f, N_c;
    uint32_t row_mask;          // N_f / N_p - 1 : hashed most significant bits of the index
    uint32_t c_mask;            // N_c - 1
    uint32_t log2_Np;
    uint32_t top_k;             // backward only: 0 = every candidate of a row keeps weight, else the top_k largest
};

// The cell of one level that contains a point: lower vertex, fractional position and the
// per-dimension hash terms of the lower (a*) and upper (b*) vertex coordinate.
template <int D>
struct Cell {
    float    w[D];
    uint32_t a1[D], b1[D];      // v0_i * pi_i,  (v0_i + 1) * pi_i
    uint32_t a2[D], b2[D];      // same with pi2

    // x scaled by the level resolution in ONE fp32 multiply (no fused multiply-add), so the
    // integer cell is the same on every implementation that follows this rule.
    // The pragma keeps the compiler from fusing the multiply into pos - floor(pos): the fraction
    // must come from the ROUNDED product, as everywhere else.
    __device__ __forceinline__ void locate(const float *xp, uint32_t N_l) {
#pragma clang fp contract(off)
        const float s = (float)N_l;
#pragma unroll
        for (int i = 0; i < D; ++i) {
            float pos = xp[i] * s;
            float fl  = floorf(pos);
            w[i] = pos - fl;
            uint32_t v0 = (uint32_t)fl;
            a1[i] = v0 * kPi[i];   b1[i] = a1[i] + kPi[i];
            a2[i] = v0 * kPi2[i];  b2[i] = a2[i] + kPi2[i];
        }
    }
    // corner c: offset (c >> i) & 1 along dimension i
    __device__ __forceinline__ uint32_t hash1(int c) const {
        uint32_t h = 0;
#pragma unroll
        for (int i = 0; i < D; ++i) h ^= ((c >> i) & 1) ? b1[i] : a1[i];
        return h;
    }
    __device__ __forceinline__ uint32_t hash2(int c) const {
        uint32_t h = 0;
#pragma unroll
        for (int i = 0; i < D; ++i) h ^= ((c >> i) & 1) ? b2[i] : a2[i];
        return h;
    }
    __device__ __forceinline__ float weight(int c) const {
        float wt = 1.0f;
#pragma unroll
        for (int i = 0; i < D; ++i) wt *= ((c >> i) & 1) ? w[i] : 1.0f - w[i];
        return wt;
    }
};

// Eq. 6: (N_p * hash(v)) mod N_f, i.e. the low log2(N_f / N_p) bits of the hash moved above
// the log2(N_p) learned bits.
__device__ __forceinline__ uint32_t probe_base(uint32_t h1, const Params &p) {
    return (h1 & p.row_mask) << p.log2_Np;
}

// Baked index codebook readers.  FMT: 0 one byte per entry, 1 two entries per byte, 2 exact width
// (entry r = bits [r * bits, (r + 1) * bits) of the level's little-endian bit string, read as 32-bit words).
constexpr int kFmtU8 = 0, kFmtPacked4 = 1, kFmtBits = 2;

template <int FMT>
__device__ __forceinline__ uint32_t read_probe(const uint8_t *D_c_level, uint32_t r, uint32_t bits) {
    if (FMT == kFmtPacked4) {
        uint32_t b = D_c_level[r >> 1];
        return (b >> ((r & 1u) * 4u)) & ((1u << bits) - 1u);
    }
    if (FMT == kFmtBits) {
        if (bits == 0) return 0u;
        const uint32_t *W = reinterpret_cast<const uint32_t *>(D_c_level);
        const uint32_t  pos = r * bits, w = pos >> 5, sh = pos & 31u;
        uint32_t v = W[w] >> sh;
        if (sh + bits > 32u) v |= W[w + 1] << (32u - sh);          // only 3-bit entries ever straddle a word
        return v & ((1u << bits) - 1u);
    }
    return D_c_level[r] & ((1u << bits) - 1u);
}

// Exact-width entry from a copy of the level's bit string in LDS.  Only 3-bit entries can straddle two
// words; they always read the following word as well (the caller keeps 4 readable bytes behind the
// string; when the entry does not straddle, the funnel shift takes nothing from that word).
__device__ __forceinline__ uint32_t read_probe_bits_lds(const uint8_t *lds_level, uint32_t r, uint32_t bits) {
    const uint32_t *W = reinterpret_cast<const uint32_t *>(lds_level);
    const uint32_t  pos = r * bits, w = pos >> 5, sh = pos & 31u;
    const uint32_t  lo = W[w];
    const uint32_t  v = (bits == 3u) ? __funnelshift_r(lo, W[w + 1], sh) : (lo >> sh);
    return v & ((1u << bits) - 1u);
}

// Two-feature codebook entry as a pair of floats.
__device__ __forceinline__ float2 load_pair(const float *base, size_t entry) {
    return *reinterpret_cast<const float2 *>(base + 2 * entry);
}
__device__ __forceinline__ float2 load_pair(const __half *base, size_t entry) {
    return __half22float2(*reinterpret_cast<const __half2 *>(base + 2 * entry));
}
__device__ __forceinline__ void store_pair(float *base, size_t entry, float a, float b) {
    *reinterpret_cast<float2 *>(base + 2 * entry) = make_float2(a, b);
}
__device__ __forceinline__ void store_pair(__half *base, size_t entry, float a, float b) {
    *reinterpret_cast<__half2 *>(base + 2 * entry) = __floats2half2_rn(a, b);
}

// Relaxed device-scope floating-point add without a return value.
__device__ __forceinline__ void atomic_add(float *addr, float v) {
    (void)__hip_atomic_fetch_add(addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace cngp

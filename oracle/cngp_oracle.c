/*
 * CPU oracle for the Compact NGP encoding path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 evaluation of what the multiresolution hash-grid
 * encoding with learned hash probing computes.  It exists to check the GPU
 * library and shares no code with it; only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it.  The product path never does.
 *
 * What is computed, and where the paper defines it:
 *   - level resolutions N_l between N_min and N_max        (Table 1; growth rule: reading R1 below)
 *   - the 2^d grid vertices enclosing a point and their d-linear weights
 *                                                          (Fig. 3 caption; Sec. 2.2 footnote on interpolation)
 *   - hash(v) = XOR_i v_i * pi_i                            (Eq. 3, spatial hashing)
 *   - feature index (N_p * hash(v)) mod N_f + D_c[hash2(v)] (Eq. 6, the learned-probing lookup)
 *   - forward: interpolate the looked-up features per level, concatenate levels
 *                                                          (Fig. 3 caption; Sec. 3 "Training": forward uses D_c)
 *   - backward: gradients go to all N_p features of the probing range, weighted
 *     by the softmax of the row of confidence values, i.e. the exact gradient of
 *     the forward pass with the hard maximum replaced by a softmax
 *                                                          (Fig. 3 caption, straight-through estimator; Sec. 3 "Training")
 *   - bake: D_c[r] = index of the largest confidence value of row r of D^_c
 *                                                          (Fig. 3 caption; Sec. 3, the two index codebooks)
 *
 * Readings of points the paper leaves open (each is also listed in the design notes):
 *   R1  N_l = floor(N_min * b^l + 1e-6), b = exp(ln(N_max/N_min)/(L-1)); L == 1 gives N_0 = N_min.
 *   R2  pos_i = x_i * N_l as ONE fp32 multiply (round to nearest even); v0 = floor(pos); the upper
 *       vertex is v0 + 1; no half-voxel offset.  Zero-weight corners are still looked up.
 *   R3  pi  = (1, 2654435761, 805459861)           (the constants of the cited Instant NGP paper)
 *   R4  pi' = (1580030173, 1367130559, 3037000507) (this build's choice; parity unpinned by the paper)
 *   R16 a fourth input dimension (d = 4; the paper's experiments have d = 2 and 3, Table 1) takes a fourth prime in
 *       each hash: 1920767767 and 2479700537, the next primes above 2^32/sqrt(5) and 2^32/sqrt(3) (this build's
 *       choice; parity unpinned by the paper).  d <= 4.
 *   R5  all hashing in uint32 with wrap-around; hash2 is reduced mod N_c; N_f, N_c, N_p powers of two.
 *   R6  every level owns its codebooks; every level is hashed.
 *   R7  softmax has no temperature; D_f values used in the logit gradient are the current ones.
 *   R8  argmax ties: lowest index wins; NaN never wins; an all-NaN row gives 0.
 *   Corner c of a cell has offset delta_i = (c >> i) & 1 along dimension i.
 *
 * Pins: tests/test_oracle_pins.py (brute force with a resolved dense grid and a library
 * interpolator, the N_p = 1 reduction to the plain hash grid of Eq. 3, adjoint identity and
 * finite differences of the softmax-relaxed forward, row-sum and mass invariants, argmax
 * properties).  The hash2 constants, the 1e-6 of R1 and the tie rule R8 are free choices:
 * parity unpinned for those.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC (see oracle/build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static const uint32_t PRIMES_HASH[4]  = {1u, 2654435761u, 805459861u, 1920767767u};
static const uint32_t PRIMES_HASH2[4] = {1580030173u, 1367130559u, 3037000507u, 2479700537u};

/* Table 1 (N_min, N_max, L) with reading R1. */
int cngp_oracle_level_resolutions(uint32_t N_min, uint32_t N_max, int L, uint32_t *N_l)
{
    if (L < 1 || N_min < 1 || (L > 1 && N_max < N_min)) return -1;
    if (L == 1) { N_l[0] = N_min; return 0; }
    double b = exp(log((double)N_max / (double)N_min) / (double)(L - 1));
    for (int l = 0; l < L; ++l)
        N_l[l] = (uint32_t)floor((double)N_min * pow(b, (double)l) + 1e-6);
    return 0;
}

typedef struct {
    uint32_t base;   /* (N_p * hash(v)) mod N_f        -- Eq. 6, the hashed most significant bits */
    uint32_t h2;     /* hash2(v) mod N_c               -- row of the index codebook               */
    double   weight; /* d-linear interpolation weight of this corner                               */
} corner_t;

/* Fig. 3 caption: enclosing vertex number c of point xp on a level of resolution Nl,
 * its two hashes (Eq. 3 with the two prime sets) and its interpolation weight. */
static corner_t corner_of(const float *xp, int d, uint32_t Nl, int c,
                          uint32_t N_f, uint32_t N_c, uint32_t N_p)
{
    corner_t r;
    uint32_t h = 0, g = 0;
    double wt = 1.0;
    for (int i = 0; i < d; ++i) {
        float pos = xp[i] * (float)Nl;            /* R2: one fp32 multiply */
        float fl  = floorf(pos);
        float w   = pos - fl;                     /* exact in fp32 */
        uint32_t delta = (uint32_t)((c >> i) & 1);
        uint32_t v = (uint32_t)fl + delta;
        wt *= delta ? (double)w : 1.0 - (double)w;
        h ^= v * PRIMES_HASH[i];                  /* uint32 wrap-around, R5 */
        g ^= v * PRIMES_HASH2[i];
    }
    r.base   = (uint32_t)(((uint64_t)N_p * (uint64_t)h) % (uint64_t)N_f);
    r.h2     = g % N_c;
    r.weight = wt;
    return r;
}

/* Index dump: for every (point, level, corner) the four integers of Eq. 6.
 * Arrays are [N, L, 2^d]; any output pointer may be NULL. */
void cngp_oracle_indices(int d, int L, uint32_t N_f, uint32_t N_c, uint32_t N_p,
                         const uint32_t *N_l, const float *x, int64_t N,
                         const uint8_t *D_c /* [L, N_c] */,
                         uint32_t *base_out, uint32_t *h2_out, uint8_t *probe_out,
                         uint32_t *feat_idx_out, double *weight_out)
{
    const int C = 1 << d;
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int l = 0; l < L; ++l)
            for (int c = 0; c < C; ++c) {
                corner_t k = corner_of(x + n * d, d, N_l[l], c, N_f, N_c, N_p);
                int64_t o = (n * L + l) * C + c;
                uint8_t p = D_c ? D_c[(int64_t)l * N_c + k.h2] : 0;
                if (base_out)     base_out[o] = k.base;
                if (h2_out)       h2_out[o] = k.h2;
                if (probe_out)    probe_out[o] = p;
                if (feat_idx_out) feat_idx_out[o] = k.base + p;
                if (weight_out)   weight_out[o] = k.weight;
            }
}

/* Hard forward (Eq. 6 + interpolation; forward uses the baked D_c).
 * D_f is [L, N_f, F] given in fp64 (the stored values, converted exactly).
 * y is [N, L*F] in fp64, unrounded.  ymag (may be NULL) receives, per output,
 * sum_c weight_c * |feature_c|, the scale the comparison tolerance refers to. */
void cngp_oracle_encode_fwd(int d, int L, int F, uint32_t N_f, uint32_t N_c, uint32_t N_p,
                            const uint32_t *N_l, const float *x, int64_t N,
                            const double *D_f, const uint8_t *D_c,
                            double *y, double *ymag)
{
    const int C = 1 << d;
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int l = 0; l < L; ++l) {
            double acc[16], mag[16];
            for (int f = 0; f < F; ++f) { acc[f] = 0.0; mag[f] = 0.0; }
            for (int c = 0; c < C; ++c) {
                corner_t k = corner_of(x + n * d, d, N_l[l], c, N_f, N_c, N_p);
                uint32_t p = D_c[(int64_t)l * N_c + k.h2];
                for (int f = 0; f < F; ++f) {
                    double feat = D_f[((int64_t)l * N_f + k.base + p) * F + f];
                    acc[f] += k.weight * feat;
                    mag[f] += k.weight * fabs(feat);
                }
            }
            for (int f = 0; f < F; ++f) {
                y[n * (int64_t)(L * F) + l * F + f] = acc[f];
                if (ymag) ymag[n * (int64_t)(L * F) + l * F + f] = mag[f];
            }
        }
}

/* softmax of one row of confidence values (footnote of Sec. 2.2), max-subtracted. */
static void softmax_row(const double *row, uint32_t N_p, double *sigma)
{
    double m = row[0], s = 0.0;
    for (uint32_t k = 1; k < N_p; ++k) if (row[k] > m) m = row[k];
    for (uint32_t k = 0; k < N_p; ++k) { sigma[k] = exp(row[k] - m); s += sigma[k]; }
    for (uint32_t k = 0; k < N_p; ++k) sigma[k] /= s;
}

/* Weights of the candidates of one row.  top_k == 0 or >= N_p: the softmax of the paper.  Otherwise
 * the sparse variant (Sec. 5, alternatives to the straight-through softmax; the choice of top-k is this
 * build's, the paper names the direction only): the top_k largest confidence values, equal values by
 * lowest index first, a NaN after every number, keep the softmax among themselves; the others get 0. */
static void candidate_weights(const double *row, uint32_t N_p, uint32_t top_k, double *sigma)
{
    if (top_k == 0 || top_k >= N_p) { softmax_row(row, N_p, sigma); return; }
    int      chosen[64] = {0};
    double   kept[64];
    uint32_t at[64];
    for (uint32_t j = 0; j < top_k; ++j) {
        int best = -1;
        for (uint32_t k = 0; k < N_p; ++k) {
            if (chosen[k]) continue;
            if (best < 0) { best = (int)k; continue; }
            const double a = row[k], b = row[best];
            if ((b != b && a == a) || a > b) best = (int)k;      /* a number beats a NaN; ties keep the lower index */
        }
        chosen[best] = 1;
        kept[j] = row[best];
        at[j] = (uint32_t)best;
    }
    double part[64];
    softmax_row(kept, top_k, part);
    for (uint32_t k = 0; k < N_p; ++k) sigma[k] = 0.0;
    for (uint32_t j = 0; j < top_k; ++j) sigma[at[j]] = part[j];
}

/* Softmax-relaxed forward: the function whose gradient the backward pass is
 * (Fig. 3 caption: gradients propagate as if the index codebook used a softmax).
 * Test helper; the product has no such entry point. */
void cngp_oracle_encode_soft_fwd(int d, int L, int F, uint32_t N_f, uint32_t N_c, uint32_t N_p,
                                 const uint32_t *N_l, const float *x, int64_t N,
                                 const double *D_f, const double *Dhat_c /* [L, N_c, N_p] */,
                                 uint32_t top_k, double *y)
{
    const int C = 1 << d;
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double sigma[64];
        for (int l = 0; l < L; ++l)
            for (int f = 0; f < F; ++f) {
                double acc = 0.0;
                for (int c = 0; c < C; ++c) {
                    corner_t k = corner_of(x + n * d, d, N_l[l], c, N_f, N_c, N_p);
                    candidate_weights(Dhat_c + ((int64_t)l * N_c + k.h2) * N_p, N_p, top_k, sigma);
                    double mix = 0.0;
                    for (uint32_t j = 0; j < N_p; ++j)
                        mix += sigma[j] * D_f[((int64_t)l * N_f + k.base + j) * F + f];
                    acc += k.weight * mix;
                }
                y[n * (int64_t)(L * F) + l * F + f] = acc;
            }
    }
}

/* Backward (Sec. 3 "Training"; Fig. 3 caption).  For every corner reference:
 *   g[f]   = weight * dy[n, l*F + f]
 *   sigma  = softmax(D^_c[l][h2][:])      (top_k > 0: candidate_weights above, the kept set held fixed)
 *   q_k    = <D_f[l][base + k], g>,  qbar = sum_j sigma_j q_j
 *   gD_f[l][base + k][f] += sigma_k * g[f]
 *   gD^_c[l][h2][k]      += sigma_k * (q_k - qbar)
 * Accumulates (+=) into gD_f [L, N_f, F] and gDhat_c [L, N_c, N_p] in fp64.
 * A_f / A_c (may be NULL) accumulate the same sums with every term replaced by
 * its magnitude (|sigma_k g[f]|, resp. sigma_k (sum_f |D_f g| + sum_j sigma_j sum_f |D_f g|)):
 * the scale that rounding errors of any summation order are proportional to. */
void cngp_oracle_encode_bwd(int d, int L, int F, uint32_t N_f, uint32_t N_c, uint32_t N_p,
                            const uint32_t *N_l, const float *x, int64_t N,
                            const double *D_f, const double *Dhat_c, const double *dy, uint32_t top_k,
                            double *gD_f, double *gDhat_c, double *A_f, double *A_c)
{
    const int C = 1 << d;
    #pragma omp parallel for schedule(dynamic, 1)
    for (int l = 0; l < L; ++l) {
        double sigma[64], q[64], qa[64], g[16];
        for (int64_t n = 0; n < N; ++n)
            for (int c = 0; c < C; ++c) {
                corner_t k = corner_of(x + n * d, d, N_l[l], c, N_f, N_c, N_p);
                candidate_weights(Dhat_c + ((int64_t)l * N_c + k.h2) * N_p, N_p, top_k, sigma);
                for (int f = 0; f < F; ++f)
                    g[f] = k.weight * dy[n * (int64_t)(L * F) + l * F + f];
                double qbar = 0.0, qabar = 0.0;
                for (uint32_t j = 0; j < N_p; ++j) {
                    const double *row = D_f + ((int64_t)l * N_f + k.base + j) * F;
                    q[j] = 0.0; qa[j] = 0.0;
                    for (int f = 0; f < F; ++f) { q[j] += row[f] * g[f]; qa[j] += fabs(row[f] * g[f]); }
                    qbar  += sigma[j] * q[j];
                    qabar += sigma[j] * qa[j];
                }
                for (uint32_t j = 0; j < N_p; ++j) {
                    int64_t fo = ((int64_t)l * N_f + k.base + j) * F;
                    int64_t co = ((int64_t)l * N_c + k.h2) * N_p + j;
                    for (int f = 0; f < F; ++f) {
                        gD_f[fo + f] += sigma[j] * g[f];
                        if (A_f) A_f[fo + f] += fabs(sigma[j] * g[f]);
                    }
                    gDhat_c[co] += sigma[j] * (q[j] - qbar);
                    if (A_c) A_c[co] += sigma[j] * (qa[j] + qabar);
                }
            }
    }
}

/* Bake (Fig. 3 caption): per row of D^_c the index of the maximal confidence, R8.
 * D_c is uint8 [rows]; rows = L * N_c. */
void cngp_oracle_bake_probes(const float *Dhat_c, int64_t rows, uint32_t N_p, uint8_t *D_c)
{
    for (int64_t r = 0; r < rows; ++r) {
        const float *row = Dhat_c + r * N_p;
        uint32_t best = 0;
        int have = 0;
        float bv = 0.0f;
        for (uint32_t k = 0; k < N_p; ++k) {
            float v = row[k];
            if (v != v) continue;                 /* NaN never wins */
            if (!have || v > bv) { best = k; bv = v; have = 1; }
        }
        D_c[r] = (uint8_t)best;
    }
}

/* Optimiser step fused with the bake (Fig. 3 caption: the bake follows every training step).
 * The paper does not name its optimiser; this build ASSUMES Adam (Kingma & Ba 2015: exponential
 * moving averages m, v of the gradient and its square, bias-corrected by 1 - beta^t, update
 * theta -= lr * m_hat / (sqrt(v_hat) + eps)), without weight decay, as in the hash-grid encoding the
 * method builds on.  All arrays have n entries; t >= 1 is the step number; everything in fp64. */
void cngp_oracle_adam_step(int64_t n, double lr, double beta1, double beta2, double eps, int t,
                           double *theta, double *m, double *v, const double *grad)
{
    const double c1 = 1.0 - pow(beta1, (double)t), c2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        m[i] = beta1 * m[i] + (1.0 - beta1) * grad[i];
        v[i] = beta2 * v[i] + (1.0 - beta2) * grad[i] * grad[i];
        theta[i] -= lr * (m[i] / c1) / (sqrt(v[i] / c2) + eps);
    }
}

/* Gradient of the hard forward with respect to the query points (the paper does not use it; it is what
 * a caller needs for normals of a signed distance field or other losses on spatial derivatives).
 * Inside a cell the feature index of Eq. 6 does not depend on x, so the derivative acts on the d-linear
 * weights only: with frac_i = x_i N_l - floor(x_i N_l) and the corner offsets delta_i(c),
 *     d weight_c / d x_j = N_l * (delta_j ? +1 : -1) * prod_{i != j} (delta_i ? frac_i : 1 - frac_i)
 *     dL/dx_j[n] = sum_l sum_c  d weight_c / d x_j * < D_f[l][base_c + D_c[l][h2_c]], dL/dy[n, l, :] >
 * (one-sided on a cell face: the cell is the one floor() selects).  gx, gmag are [N, d]; gmag sums the
 * magnitudes of the terms. */
void cngp_oracle_encode_bwd_input(int d, int L, int F, uint32_t N_f, uint32_t N_c, uint32_t N_p,
                                  const uint32_t *N_l, const float *x, int64_t N,
                                  const double *D_f, const uint8_t *D_c, const double *dy,
                                  double *gx, double *gmag)
{
    const int C = 1 << d;
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int j = 0; j < d; ++j) { gx[n * d + j] = 0.0; if (gmag) gmag[n * d + j] = 0.0; }
        for (int l = 0; l < L; ++l) {
            double frac[8];
            for (int i = 0; i < d; ++i) {
                float pos = x[n * d + i] * (float)N_l[l];      /* R2: one fp32 multiply */
                frac[i] = (double)(pos - floorf(pos));
            }
            for (int c = 0; c < C; ++c) {
                corner_t k = corner_of(x + n * d, d, N_l[l], c, N_f, N_c, N_p);
                uint32_t p = D_c[(int64_t)l * N_c + k.h2];
                double t = 0.0, tm = 0.0;
                for (int f = 0; f < F; ++f) {
                    double feat = D_f[((int64_t)l * N_f + k.base + p) * F + f];
                    double g = dy[n * (int64_t)(L * F) + l * F + f];
                    t += feat * g;
                    tm += fabs(feat * g);
                }
                for (int j = 0; j < d; ++j) {
                    double dw = ((c >> j) & 1) ? 1.0 : -1.0;
                    for (int i = 0; i < d; ++i)
                        if (i != j) dw *= ((c >> i) & 1) ? frac[i] : 1.0 - frac[i];
                    gx[n * d + j] += (double)N_l[l] * dw * t;
                    if (gmag) gmag[n * d + j] += (double)N_l[l] * fabs(dw) * tm;
                }
            }
        }
    }
}

/* Threads the parallel loops above use, and a way to change that (timing of the oracle on one core). */
int cngp_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void cngp_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

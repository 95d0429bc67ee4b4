/*
 * Runs every function of the CPU oracle (cngp_oracle.c, compiled into this program) on small seeded inputs under
 * AddressSanitizer and UndefinedBehaviorSanitizer.  TEST INFRASTRUCTURE ONLY: built by `python oracle/build.py
 * --sanitize` (gcc -fsanitize=address,undefined), run by tests/test_oracle_pins.py.  The sanitizers abort on an
 * out-of-bounds access, a signed overflow, a misaligned or invalid conversion; this program itself only checks
 * that results are finite and that baked indices are inside the probing range.  Exit code 0 = clean.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int  cngp_oracle_level_resolutions(uint32_t, uint32_t, int, uint32_t *);
void cngp_oracle_indices(int, int, uint32_t, uint32_t, uint32_t, const uint32_t *, const float *, int64_t, const uint8_t *,
                         uint32_t *, uint32_t *, uint8_t *, uint32_t *, double *);
void cngp_oracle_encode_fwd(int, int, int, uint32_t, uint32_t, uint32_t, const uint32_t *, const float *, int64_t,
                            const double *, const uint8_t *, double *, double *);
void cngp_oracle_encode_soft_fwd(int, int, int, uint32_t, uint32_t, uint32_t, const uint32_t *, const float *, int64_t,
                                 const double *, const double *, uint32_t, double *);
void cngp_oracle_encode_bwd(int, int, int, uint32_t, uint32_t, uint32_t, const uint32_t *, const float *, int64_t,
                            const double *, const double *, const double *, uint32_t, double *, double *, double *, double *);
void cngp_oracle_bake_probes(const float *, int64_t, uint32_t, uint8_t *);
void cngp_oracle_adam_step(int64_t, double, double, double, double, int, double *, double *, double *, const double *);
void cngp_oracle_encode_bwd_input(int, int, int, uint32_t, uint32_t, uint32_t, const uint32_t *, const float *, int64_t,
                                  const double *, const uint8_t *, const double *, double *, double *);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double uniform(void) {                       /* splitmix64 */
    uint64_t z = (state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return (double)((z ^ (z >> 31)) >> 11) / 9007199254740992.0;
}

static int all_finite(const double *a, int64_t n) {
    for (int64_t i = 0; i < n; ++i) if (!isfinite(a[i])) return 0;
    return 1;
}

int main(void)
{
    int bad = 0;
    for (int d = 2; d <= 3; ++d)
        for (uint32_t N_p = 1; N_p <= 16; N_p *= 2)
            for (int F = 1; F <= 4; F *= 2) {
                const int      L = 3, C = 1 << d;
                const uint32_t N_f = 64 > N_p ? 64 : N_p, N_c = 32;
                const int64_t  N = 37;
                uint32_t       res[8];
                if (cngp_oracle_level_resolutions(2, 19, L, res)) return 2;
                float   *x = malloc(sizeof(float) * N * d);
                double  *D_f = malloc(sizeof(double) * L * N_f * F), *Dhat = malloc(sizeof(double) * L * N_c * N_p);
                float   *Dhat32 = malloc(sizeof(float) * L * N_c * N_p);
                double  *dy = malloc(sizeof(double) * N * L * F);
                uint8_t *D_c = malloc(L * N_c);
                for (int64_t i = 0; i < N * d; ++i) x[i] = (float)uniform();
                x[0] = 0.0f; x[1] = 1.0f; x[d] = 1.0f;                       /* the cube's faces and corners */
                for (int64_t i = 0; i < (int64_t)L * N_f * F; ++i) D_f[i] = uniform() - 0.5;
                for (int64_t i = 0; i < (int64_t)L * N_c * N_p; ++i) { Dhat[i] = 4.0 * uniform() - 2.0; Dhat32[i] = (float)Dhat[i]; }
                Dhat32[0] = NAN; Dhat32[N_p] = INFINITY;                     /* the bake's special cases */
                for (int64_t i = 0; i < N * L * F; ++i) dy[i] = uniform() - 0.5;
                cngp_oracle_bake_probes(Dhat32, (int64_t)L * N_c, N_p, D_c);
                for (int64_t i = 0; i < (int64_t)L * N_c; ++i) bad |= D_c[i] >= N_p;

                uint32_t *base = malloc(4 * N * L * C), *h2 = malloc(4 * N * L * C), *fi = malloc(4 * N * L * C);
                uint8_t  *pr = malloc(N * L * C);
                double   *wt = malloc(8 * N * L * C);
                cngp_oracle_indices(d, L, N_f, N_c, N_p, res, x, N, D_c, base, h2, pr, fi, wt);
                for (int64_t i = 0; i < N * L * C; ++i) bad |= fi[i] >= N_f || h2[i] >= N_c;

                double *y = malloc(8 * N * L * F), *ymag = malloc(8 * N * L * F);
                cngp_oracle_encode_fwd(d, L, F, N_f, N_c, N_p, res, x, N, D_f, D_c, y, ymag);
                bad |= !all_finite(y, N * L * F) || !all_finite(ymag, N * L * F);
                for (uint32_t top_k = 0; top_k <= N_p; top_k += (N_p > 2 ? N_p / 2 : 1)) {
                    cngp_oracle_encode_soft_fwd(d, L, F, N_f, N_c, N_p, res, x, N, D_f, Dhat, top_k, y);
                    bad |= !all_finite(y, N * L * F);
                    double *gF = calloc((size_t)L * N_f * F, 8), *gC = calloc((size_t)L * N_c * N_p, 8);
                    double *aF = calloc((size_t)L * N_f * F, 8), *aC = calloc((size_t)L * N_c * N_p, 8);
                    cngp_oracle_encode_bwd(d, L, F, N_f, N_c, N_p, res, x, N, D_f, Dhat, dy, top_k, gF, gC, aF, aC);
                    cngp_oracle_encode_bwd(d, L, F, N_f, N_c, N_p, res, x, N, D_f, Dhat, dy, top_k, gF, gC, NULL, NULL);
                    bad |= !all_finite(gF, (int64_t)L * N_f * F) || !all_finite(gC, (int64_t)L * N_c * N_p);
                    free(gF); free(gC); free(aF); free(aC);
                }
                double *gx = malloc(8 * N * d), *gm = malloc(8 * N * d);
                cngp_oracle_encode_bwd_input(d, L, F, N_f, N_c, N_p, res, x, N, D_f, D_c, dy, gx, gm);
                cngp_oracle_encode_bwd_input(d, L, F, N_f, N_c, N_p, res, x, N, D_f, D_c, dy, gx, NULL);
                bad |= !all_finite(gx, N * d);
                free(x); free(D_f); free(Dhat); free(Dhat32); free(dy); free(D_c); free(base); free(h2); free(fi);
                free(pr); free(wt); free(y); free(ymag); free(gx); free(gm);
            }
    {
        double th[5] = {1, -2, 3, 0, 1e-9}, m[5] = {0}, v[5] = {0}, g[5] = {0.5, -0.25, 0, 1e-30, 7};
        for (int t = 1; t <= 3; ++t) cngp_oracle_adam_step(5, 1e-2, 0.9, 0.99, 1e-15, t, th, m, v, g);
        bad |= !all_finite(th, 5);
    }
    uint32_t r1[1];
    bad |= cngp_oracle_level_resolutions(5, 1, 1, r1) != 0 || r1[0] != 5;
    bad |= cngp_oracle_level_resolutions(0, 4, 2, r1) == 0;                /* rejected */
    if (bad) { fprintf(stderr, "oracle sanitizer run: a result was out of range or not finite\n"); return 1; }
    printf("oracle sanitizer run: clean\n");
    return 0;
}

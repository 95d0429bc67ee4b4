/*
 * cngp.h -- C ABI of the Compact NGP encoding library for AMD MI355X (gfx950).
 *
 * The library implements the data-parallel hot path of "Compact Neural Graphics
 * Primitives with Learned Hash Probing": a multiresolution hash-grid input
 * encoding y = psi(x; theta) whose feature index is
 *
 *     f(v) = D_f[ (N_p * hash(v)) mod N_f + D_c[hash2(v)] ]            (Eq. 6)
 *
 * with hash / hash2 two spatial hashes (Eq. 3) over different primes, D_f the
 * feature codebook, D_c the index codebook of learned probe offsets, and D^_c its
 * training-time version holding N_p confidence values per row (Sec. 3).
 *
 * Conventions shared by every entry point
 *   - Pointers marked "dev" are device (HBM) addresses, "host" are host addresses.
 *     Every buffer is allocated, owned and freed by the caller.  The library keeps no
 *     device state, allocates no device memory and never synchronises the device:
 *     all work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     null stream) and the call returns once it is enqueued.
 *   - Arrays are dense, row-major, with the shapes given below; no strides.
 *   - Return value: 0 (CNGP_OK) or a negative cngp_status.  All argument checks run on
 *     the host before anything is launched, so they need no GPU.  N == 0 is a successful
 *     no-op.  Nothing throws across this boundary.
 *   - Preconditions that are NOT checked on the device: x finite and inside [0, 1]^d;
 *     every entry of D_c smaller than N_p.
 *   - Corner numbering: corner c of a grid cell has offset (c >> i) & 1 along dimension i.
 *   - Level l uses rows [l] of every codebook; output column l*F + f holds feature f of level l.
 */
#ifndef CNGP_H
#define CNGP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CNGP_OK              =  0,
    CNGP_ERR_NULL        = -1,  /* a required pointer is NULL                                  */
    CNGP_ERR_INVALID     = -2,  /* a size is out of range or not a power of two where required  */
    CNGP_ERR_UNSUPPORTED = -3,  /* valid in the paper's terms, not built here (e.g. F = 3)      */
    CNGP_ERR_WORKSPACE   = -4,  /* workspace missing, misaligned or smaller than required       */
    CNGP_ERR_HIP         = -5   /* a HIP call failed; see cngp_last_hip_error()                 */
} cngp_status;

typedef enum { CNGP_F32 = 0, CNGP_F16 = 1 } cngp_dtype;

/* Layout of the baked index codebook D_c.
 *   CNGP_IDX_U8      one byte per entry, [L, N_c]
 *   CNGP_IDX_PACKED4 two entries per byte, [L, N_c / 2]; entry 2i is the low nibble of byte i.
 *                    Needs N_c >= 2 (N_p <= 16 always fits four bits).
 *   CNGP_IDX_BITS    exact width, the storage the model sizes of Tables 3 and 4 imply: with
 *                    b = log2(N_p), entry r of a level is bits [r * b, (r + 1) * b) of that level's
 *                    bit string, least significant bit first within little-endian 32-bit words.
 *                    Every level starts on a 4-byte boundary: consecutive levels are
 *                    4 * ceil(N_c * b / 32) bytes apart, padding bits are zero when the library writes
 *                    them and ignored when it reads; the array must be 4-byte aligned.  N_p = 1
 *                    stores nothing (the pointer may be NULL).  Read by cngp_encode_fwd and
 *                    cngp_debug_indices, written by cngp_bake_probes; the optimiser step does not
 *                    take it (CNGP_ERR_UNSUPPORTED): training keeps one of the two formats above. */
typedef enum { CNGP_IDX_U8 = 0, CNGP_IDX_PACKED4 = 1, CNGP_IDX_BITS = 2 } cngp_index_format;

/* cngp_config.flags */
enum {
    CNGP_ZERO_GRADS = 1u,   /* cngp_encode_bwd clears both gradient arrays before accumulating            */
    CNGP_BWD_DIRECT = 2u,   /* force the backward variant that adds straight into HBM with global atomics  */
    CNGP_BWD_SLICED = 4u,   /* force the variant that accumulates table slices in LDS (needs workspace)   */
                            /* neither of the two: the library picks by table size and N                   */
    CNGP_BWD_NO_PREREDUCE = 8u, /* LDS variant only: do not pre-reduce coarse levels per grid vertex       */
    CNGP_FWD_SIMPLE = 16u,  /* force the forward variant that reads D_c from memory, not from LDS          */
    CNGP_BWD_BINNED = 32u,  /* LDS variant: bin the references of the hashed levels by slice first instead */
                            /* of scanning all points once per slice (more workspace, see plan info)       */
    CNGP_FWD_LEVEL = 64u,   /* force the level-resident forward variant (a workgroup keeps one level's     */
                            /* codebooks in LDS and streams the points; needs cngp_fwd_workspace_bytes);   */
                            /* CNGP_ERR_UNSUPPORTED / CNGP_ERR_WORKSPACE where it cannot run                */
    CNGP_FWD_TILE = 128u    /* never take the level-resident variant                                       */
                            /* none of the three forward flags: the library picks by table size and N; the */
                            /* three variants give bit-identical encodings                                 */
};

/* Hyper-parameters of the encoding (Table 1 of the paper, same symbols). */
typedef struct {
    int32_t  d;            /* dimension of the input domain: 2, 3 or 4                         */
    int32_t  L;            /* number of resolution levels, 1 .. 32                             */
    int32_t  F;            /* features per codebook entry: 1, 2, 4 or 8 (the paper's value is 2, and 2 is the
                              width every kernel works in: the others run as ceil(F / 2) passes over pairs of
                              features, need the workspace also for cngp_encode_fwd, and are refused
                              (CNGP_ERR_UNSUPPORTED) by the entry points that take no workspace)  */
    uint32_t N_f;          /* entries of the feature codebook per level, power of two          */
    uint32_t N_c;          /* rows of the index codebook per level, power of two               */
    uint32_t N_p;          /* probing range, power of two, 1 .. 16, N_p <= N_f                 */
    uint32_t N_min;        /* coarsest grid resolution, >= 1                                   */
    uint32_t N_max;        /* finest grid resolution, >= N_min, <= 2^24 (ignored when L == 1)  */
    int32_t  feat_dtype;   /* cngp_dtype of D_f                                                */
    int32_t  io_dtype;     /* cngp_dtype of y and dL/dy                                        */
    int32_t  index_format; /* cngp_index_format of D_c                                         */
    uint32_t flags;        /* bitwise OR of the CNGP_* flags above                             */
    uint64_t bin_bytes_max; /* most workspace cngp_encode_bwd spends on binned references (4 bytes per
                              corner reference, level and gradient table); 0 = 8 GiB.  A larger batch
                              is taken in several passes inside the one call                      */
    uint32_t top_k;        /* cngp_encode_bwd only.  0 or N_p: the paper's backward (softmax over all N_p
                              candidates of a row).  1 .. N_p - 1: sparse variant (Sec. 5 names sparse
                              alternatives to the dense softmax as future work; top-k is this library's
                              choice): per row of D^_c only the top_k largest confidence values, equal
                              values by lowest index first and any number before a NaN, keep the softmax
                              among themselves; the other candidates get weight 0, hence no gradient    */
    uint32_t reserved;     /* must be 0                                                                 */
} cngp_config;

/* Grid resolution of every level (Table 1: N_min, N_max, L; geometric growth):
 * N_l = floor(N_min * b^l + 1e-6), b = exp(ln(N_max / N_min) / (L - 1)); L == 1 gives N_min.
 * out_N_l: host, L entries.  Runs on the host. */
int cngp_level_resolutions(const cngp_config *cfg, uint32_t *out_N_l);

/* Bytes of the stored model (Tables 3 and 4 count these): D_f in feat_dtype, D_c in index_format
 * (per level, i.e. the distance between consecutive levels, and in total).  Any output may be NULL.  Host only. */
int cngp_storage_bytes(const cngp_config *cfg, size_t *D_f_bytes, size_t *D_c_level_bytes, size_t *D_c_bytes);

/* Bytes of device scratch the calls below use for N points (may be 0): the larger of what cngp_encode_bwd needs
 * (softmax table, level-major dL/dy, bins; CNGP_ERR_WORKSPACE without it) and what the forward calls can use
 * (cngp_fwd_workspace_bytes below; without it they run a slower variant with the same result).  With F != 2 one pair
 * of features at a time is copied out of D_f, y, dL/dy and back, and those planes sit in the workspace too (the
 * forward calls then need it as well).
 * The workspace must be 256-byte aligned; its contents are undefined before and after each call.
 * Returns 0 for an invalid configuration as well (the encode calls then report the error). */
size_t cngp_workspace_bytes(const cngp_config *cfg, int64_t N);

/* The part of it the forward calls use: room for a level-major copy of the encodings (N * L * F values of io_dtype)
 * when the level-resident variant would be taken for this configuration and N, else 0 (F != 2: the pair planes,
 * as above).  A forward call that is given less runs the tile variant instead, with the same result. */
size_t cngp_fwd_workspace_bytes(const cngp_config *cfg, int64_t N);

/* How a forward call with enough workspace would run: info[0] = 1 if the level-resident variant is taken, info[1] =
 * entries of a level's feature codebook it keeps in LDS (of N_f), info[2] = runs of points a level is cut into (the
 * grid has that many workgroups per level), info[3] = bytes of LDS per workgroup.  Host only. */
enum { CNGP_FWD_PLAN_INFO_COUNT = 4 };
int cngp_fwd_plan_info(const cngp_config *cfg, int64_t N, int32_t *info);

/* Forward encoding (Eq. 6; Fig. 3: enclosing vertices, two hashes, probe lookup, feature
 * gather, d-linear interpolation, concatenation over levels; the forward pass uses the baked
 * D_c, Sec. 3 "Training").
 *   x    dev  float32 [N, d], inside [0,1]^d; scaled per level as one fp32 multiply x * N_l
 *   D_f  dev  feat_dtype [L, N_f, F]
 *   D_c  dev  index_format, see above
 *   y    dev  io_dtype [N, L*F], written (not accumulated); fp32 arithmetic, one final rounding
 *   workspace  dev, may be NULL (see above); the variants differ in speed only, their encodings are bit-identical */
int cngp_encode_fwd(const cngp_config *cfg, const float *x, int64_t N,
                    const void *D_f, const void *D_c, void *y,
                    void *workspace, size_t workspace_bytes, void *stream);

/* Forward encoding from a partially loaded model (Sec. 1, Sec. 5: level-of-detail streaming, partial results
 * in bandwidth-constrained settings): only levels 0 .. levels_loaded - 1 of D_f and D_c need to be present
 * (the arrays keep their full layout; the rest is never read); the columns of the other levels are written
 * as zero.  levels_loaded = L is cngp_encode_fwd; 0 writes zeros and reads no table. */
int cngp_encode_fwd_partial(const cngp_config *cfg, int32_t levels_loaded, const float *x, int64_t N,
                            const void *D_f, const void *D_c, void *y,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Optional reordering of the query points (not part of the paper's method: the hash tables have no locality
 * between neighbouring vertices, but neighbouring points share the vertices of the coarse levels, so a batch
 * in Morton order is encoded mostly from the first-level cache: measured 2x on uniformly random points).
 * cngp_morton_sort: code(x) = the interleaved bits (bit b of coordinate j at position b * d + j) of
 * q_j = min(max(floor(x_j * 2^B), 0), 2^B - 1), B = 10, 7, 5 for d = 2, 3, 4; perm = the STABLE ascending order of
 * the codes, i.e. perm[i] is the index of the i-th point in Morton order, and x_sorted[i] = x[perm[i]].
 *   x         dev float32 [N, d]
 *   perm      dev int32 [N], written
 *   x_sorted  dev float32 [N, d], written; may be NULL
 *   workspace dev, 256-byte aligned, cngp_morton_sort_workspace_bytes(d, N) bytes (0 = invalid d or N): two key
 *             columns, one index column, and 128 counters per tile of 8192 points (about 12 bytes per point)
 * N <= 2^31 - 1.  The sort is this library's own: a stable radix sort of (code, index), 7 bits per pass.
 * cngp_encode_fwd_permuted: the forward encoding of x_sorted with row i of the result written to row perm[i] of
 * y, so y is in the order of the caller's original points and equals cngp_encode_fwd on them bit for bit.
 * perm must be a permutation of 0 .. N-1 (not checked: any other content writes outside y or leaves rows unset).
 * workspace as for cngp_encode_fwd (cngp_fwd_workspace_bytes; NULL / 0: the tile variant). */
size_t cngp_morton_sort_workspace_bytes(int32_t d, int64_t N);
int cngp_morton_sort(int32_t d, const float *x, int64_t N, int32_t *perm, float *x_sorted,
                     void *workspace, size_t workspace_bytes, void *stream);
int cngp_encode_fwd_permuted(const cngp_config *cfg, const float *x_sorted, const int32_t *perm, int64_t N,
                             const void *D_f, const void *D_c, void *y,
                             void *workspace, size_t workspace_bytes, void *stream);

/* Backward pass (Sec. 3 "Training"; Fig. 3: straight-through estimator).  The gradient of the
 * forward pass with the hard maximum replaced by a softmax over each row of D^_c: for every
 * enclosing vertex, with g = weight * dL/dy, sigma = softmax(D^_c[l][hash2(v)]) and
 * q_k = <D_f[l][base + k], g>,
 *     grad_D_f[l][base + k][f]       += sigma_k * g[f]                    for all k < N_p
 *     grad_Dhat_c[l][hash2(v)][k]    += sigma_k * (q_k - sum_j sigma_j q_j)
 * With cfg->top_k in 1 .. N_p - 1, sigma is the sparse weight vector described at cngp_config.top_k
 * (the kept set is treated as constant).
 * Uses D^_c only, never D_c.  No gradient with respect to x.
 *   Dhat_c       dev float32 [L, N_c, N_p]
 *   dy           dev io_dtype [N, L*F]
 *   grad_D_f     dev float32 [L, N_f, F]      accumulated (+=), or cleared first with CNGP_ZERO_GRADS
 *   grad_Dhat_c  dev float32 [L, N_c, N_p]    same
 * Sums are formed with floating-point atomics: their order, hence the last bits, vary run to run.
 * A vertex whose interpolation weight is exactly zero (the point lies on a face of its cell) contributes exactly
 * nothing; the variants that accumulate in LDS leave such references out altogether, so a non-finite dL/dy or
 * D_f entry reaches the gradients only through the vertices of non-zero weight (every point has at least one).
 * A batch whose binned references would pass cfg->bin_bytes_max is taken in several passes over runs of
 * points, each adding onto the one before, inside the one call (cngp_bwd_plan_info reports how many). */
int cngp_encode_bwd(const cngp_config *cfg, const float *x, int64_t N,
                    const void *D_f, const float *Dhat_c, const void *dy,
                    float *grad_D_f, float *grad_Dhat_c,
                    void *workspace, size_t workspace_bytes, void *stream);

/* cngp_encode_bwd for callers that cannot allocate device memory or size a workspace: code under HIP graph
 * capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * cngp_encode_bwd without the workspace: the scratch (softmax table, level-major dL/dy, vertex sums, bins) lives in
 * a static device array of cngp_static_scratch_bytes() = 64 MiB inside the library, which every GPU the library
 * runs on holds from load to process end.  A batch whose binned references would not fit is taken in several
 * passes inside the call; if the part that does not shrink with the passes (the softmax table L * N_c * N_p * 4
 * bytes, dL/dy of one pass) still does not fit: CNGP_ERR_WORKSPACE, with the sizes in cngp_last_hip_error().
 * Calls no hipMalloc / hipFree.  All calls on one GPU share that GPU's array: calls that overlap in time on one
 * GPU (two streams, two threads) race; calls on one stream are ordered and safe.  Nothing in the array needs to
 * survive between calls, and nothing in it is assumed to be zero. */
size_t cngp_static_scratch_bytes(void);
int cngp_encode_bwd_static(const cngp_config *cfg, const float *x, int64_t N,
                           const void *D_f, const float *Dhat_c, const void *dy,
                           float *grad_D_f, float *grad_Dhat_c, void *stream);

/* Gradient with respect to the query points (not used by the paper; for losses on spatial derivatives such
 * as the normals of a signed distance field).  Inside a cell the feature index of Eq. 6 is constant, so
 * the derivative of the forward pass acts on the d-linear weights only:
 *     grad_x[n][j] = sum_l N_l sum_c (+1 | -1)_j(c) prod_{i != j} w_i(c) <D_f[l][base_c + D_c[l][h2_c]], dL/dy[n, l, :]>
 * one-sided on a cell face (the cell floor() selects).  Uses the baked D_c like the forward pass.
 *   dy dev io_dtype [N, L*F];  grad_x dev float32 [N, d], written. */
int cngp_encode_bwd_input(const cngp_config *cfg, const float *x, int64_t N, const void *D_f, const void *D_c,
                          const void *dy, float *grad_x, void *stream);

/* How cngp_encode_bwd would run for this configuration and N (host only; for tests, tuning and logs).
 * info (host, CNGP_PLAN_INFO_COUNT entries): [0] 1 = LDS-sliced variant, 0 = global atomics;
 * [1] number of coarse levels pre-reduced per grid vertex; [2], [3] slices per level of the feature and
 * of the logit gradient table; [4], [5] point chunks of the feature / logit role on hashed levels;
 * [6], [7] vertex chunks of the two roles on pre-reduced levels; [8] point chunks and [9] total slices
 * of the vertex-grid accumulation; [10] 1 = the hashed levels' references are binned by slice first, and then
 * [11], [12] workgroups that drain one bin of the feature / logit table and [13] point chunks of the binning;
 * with [2] = 0 when a level's feature table is small enough (N_f <= 4096) to be accumulated whole in LDS by the
 * workgroups that drain the confidence-table bins (one pass for both gradients, no pre-reduced levels);
 * [14] passes over runs of points (1 unless the batch is split to bound the scratch; [0] .. [13] then
 * describe the first pass). */
enum { CNGP_PLAN_INFO_COUNT = 15 };
int cngp_bwd_plan_info(const cngp_config *cfg, int64_t N, int32_t *info);

/* Where cngp_encode_bwd keeps what in its workspace for this configuration and N (one pass of it, when the batch is
 * taken in passes).  Host only; for tests of the plan: region i covers bytes [regions[2i], regions[2i] + regions[2i+1])
 * -- the softmax table, the level-major dL/dy, the per-vertex sums, then for the binned variant the count matrices,
 * bin starts and records of the two tables and of the pre-reduced levels.  No two regions may overlap, every one
 * starts on a 256-byte boundary and ends inside cngp_workspace_bytes(cfg, N).  Returns the number of regions
 * (at most CNGP_PLAN_REGIONS; 0 for the variant that needs no workspace) or a negative status. */
enum { CNGP_PLAN_REGIONS = 12 };
int cngp_bwd_plan_layout(const cngp_config *cfg, int64_t N, uint64_t *regions);

/* Bake (Fig. 3; Sec. 3): D_c[l][r] = index of the largest confidence value in row r of D^_c.
 * Ties: lowest index; NaN never wins; an all-NaN row gives 0.  Result always < N_p.
 *   Dhat_c dev float32 [L, N_c, N_p];  D_c dev, written in cfg->index_format. */
int cngp_bake_probes(const cngp_config *cfg, const float *Dhat_c, void *D_c, void *stream);

/* Optimiser step fused with the bake (Fig. 3: the bake follows every training step).  The paper
 * names no optimiser: this entry point ASSUMES Adam (Kingma & Ba 2015) without weight decay.
 * For every entry of a table, with g = grad * grad_scale and t = step (the number of this step, >= 1):
 *     m = beta1 * m + (1 - beta1) * g            v = beta2 * v + (1 - beta2) * g * g
 *     theta -= lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
 * in fp32.  Then D_c[l][r] = argmax of the UPDATED row r of D^_c, with the rule of cngp_bake_probes.
 * One launch; every array is read once and written once. */
typedef struct cngp_adam {
    float   lr, beta1, beta2;   /* lr >= 0; 0 <= beta < 1                                            */
    float   eps;                /* > 0; with eps >= 1e-15 squares of gradients that underflow fp32
                                   change the step by less than the tolerance of the parity tests   */
    float   grad_scale;         /* e.g. 1 / loss scale; must be finite                               */
    int32_t step;               /* t >= 1                                                            */
} cngp_adam;

/*   opt_f, opt_c   host; either may be NULL: that table is then left alone (with opt_c == NULL
 *                  D_c is not written either) and its pointers are ignored
 *   D_f_master     dev float32 [L, N_f, F]   parameters, updated in place
 *   D_f            dev: with feat_dtype F16, receives the updated parameters rounded to fp16 (the array
 *                  the forward and backward passes read); with F32 pass NULL or D_f_master itself
 *   m_f, v_f       dev float32 [L, N_f, F]   moments, updated in place (zero before the first step)
 *   grad_D_f       dev float32 [L, N_f, F]   read; set to zero afterwards if cfg->flags has CNGP_ZERO_GRADS
 *   Dhat_c, m_c, v_c, grad_Dhat_c   dev float32 [L, N_c, N_p], likewise
 *   D_c            dev, written in cfg->index_format
 * All float arrays must be 16-byte aligned (D_f with F16: 8-byte), else CNGP_ERR_INVALID. */
int cngp_adam_step_bake(const cngp_config *cfg, const cngp_adam *opt_f, const cngp_adam *opt_c,
                        float *D_f_master, void *D_f, float *m_f, float *v_f, float *grad_D_f,
                        float *Dhat_c, float *m_c, float *v_c, float *grad_Dhat_c, void *D_c,
                        void *stream);

/* Decoder after the encoding (Fig. 3: the interpolated features are fed into an MLP; Table 1: 64 hidden
 * neurons).  The paper gives the width only; ASSUMED here: two hidden layers, ReLU after each, a linear
 * output layer, no biases:
 *     h1 = relu(W1 y)    h2 = relu(W2 h1)    out = W3 h2
 * Runs on the matrix cores: fp16 operands (y, the weights, h1, h2 and the hidden-layer gradients are
 * rounded to fp16), fp32 accumulation.
 *   n_in   columns of y, 1 .. 32 (L * F of the encoding)      n_out  1 .. 16
 *   W      dev float16: W1 [64, n_in], W2 [64, 64], W3 [n_out, 64], row-major, one after the other
 *   y      dev io_dtype [N, n_in]          out   dev float32 [N, n_out], written */
typedef struct cngp_mlp_config {
    int32_t  n_in, n_out;
    int32_t  io_dtype;     /* cngp_dtype of y and dL/dy                                            */
    uint32_t flags;        /* CNGP_ZERO_GRADS: cngp_mlp_bwd clears grad_W before accumulating      */
} cngp_mlp_config;
size_t cngp_mlp_weight_count(const cngp_mlp_config *cfg);     /* 64 n_in + 64 * 64 + 64 n_out; 0 if invalid */
int cngp_mlp_fwd(const cngp_mlp_config *cfg, const void *y, int64_t N, const void *W, float *out, void *stream);

/* Encoding and decoder in one call, for inference: out = decoder(encode(x)).  Equal, bit for bit, to
 * cngp_encode_fwd followed by cngp_mlp_fwd (the features pass as fp16 either way).
 *   workspace dev, 256-byte aligned, N * L * F * 2 bytes (= cngp_fwd_workspace_bytes of the same configuration with
 *             fp16 encodings), or NULL / 0.
 * With the workspace (and a configuration the level-resident forward takes): that forward writes its level-major
 * fp16 encodings into the workspace and the decoder reads them as they lie, so the kernel that turns them into
 * rows of y and y itself are saved.  Without: one kernel in which the encoded features never go to memory, which
 * is slower than the two separate calls and needs an index codebook whose level fits in LDS (N_c <= 2^17 entries;
 * otherwise CNGP_ERR_UNSUPPORTED).  Needs mlp->n_in == cfg->L * cfg->F and F = 2; mlp->io_dtype and flags are ignored. */
int cngp_encode_mlp_fwd(const cngp_config *cfg, const cngp_mlp_config *mlp, const float *x, int64_t N,
                        const void *D_f, const void *D_c, const void *W, float *out,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Backward pass of the decoder for L = sum(out * dout): recomputes the hidden layers, then
 *   dy      dev io_dtype [N, n_in]    written: dL/dy, the upstream gradient cngp_encode_bwd takes
 *   grad_W  dev float32, layout of W  accumulated (+=) with floating-point atomics, or cleared first
 * relu'(a) = 1 for a > 0, else 0, decided on the fp32 pre-activation the kernel itself computed. */
int cngp_mlp_bwd(const cngp_mlp_config *cfg, const void *y, int64_t N, const void *W, const float *dout,
                 void *dy, float *grad_W, void *stream);

/* Adam step (see cngp_adam_step_bake) on one plain array of n parameters, e.g. the decoder's weights:
 * master, m, v, grad dev float32 [n], 16-byte aligned; half_copy dev float16 [n] (8-byte aligned) receives
 * the updated parameters rounded to fp16, or NULL; clear_grad != 0 sets grad to zero afterwards. */
int cngp_adam_step(const cngp_adam *opt, int64_t n, float *master, void *half_copy, float *m, float *v,
                   float *grad, int clear_grad, void *stream);

/* Index dump for parity checks: for every (point, level, corner) the integers of Eq. 6.
 * All outputs dev, shape [N, L, 2^d]; any of them may be NULL.
 *   base      (N_p * hash(v)) mod N_f        h2        hash2(v) mod N_c
 *   probe     D_c[l][h2]                     feat_idx  base + probe */
int cngp_debug_indices(const cngp_config *cfg, const float *x, int64_t N, const void *D_c,
                       uint32_t *base, uint32_t *h2, uint8_t *probe, uint32_t *feat_idx,
                       void *stream);

/* Rates of this device that bound the kernels above, measured by short microbenchmarks (about 20 ms):
 * the codebooks of this method are cache resident, so its forward pass is bound by random gathers and
 * its backward pass by scatter-add atomics (Sec. 4 "Performance" of the paper: gradient accumulation
 * must be staged in workgroup-local memory), not by streaming bandwidth.
 *   scratch  dev, at least 64 MiB, 256-byte aligned; contents are overwritten.
 * Unlike the other entry points this one waits for its kernels (it returns host-side numbers). */
typedef struct {
    double copy_GBps;            /* streaming copy of 32 MB to 32 MB, bytes read + written per second / 1e9: a working
                                    set that stays in the 256 MB memory-side cache, as the tables and the batch of
                                    a training step do; a copy from DRAM (1 GiB) runs at about 4.5e3 here         */
    double gather4_Gps;          /* random 4-byte gathers from a 4 MB table, 1e9 per second          */
    double row_gather_Gps;       /* random 64-byte rows read by 16 lanes each, 1e9 rows per second   */
    double global_atomic_Gseg;   /* fp32 atomic adds to random 64-byte rows, 1e9 rows per second     */
    double lds_atomic_f64_Gps;   /* fp64 atomic adds in LDS (rows of 32), 1e9 adds per second, chip  */
    double lds_atomic_f32_Gps;   /* the same access pattern with fp32 accumulators                   */
    double lds_atomic_u32_Gps;   /* ... and with 32-bit integer accumulators                         */
    double row_gather_far_Gps;   /* random 64-byte rows from a 32 MB table (beyond the 4 MB L2 of an XCD) */
    double gather4_far_Gps;      /* random 4-byte gathers from that table                            */
    double lds_gather4_Gps;      /* random 4-byte reads of a 128 KB LDS table, every lane its own address */
} cngp_rates;
int cngp_measure_rates(cngp_rates *out, void *scratch, size_t scratch_bytes, void *stream);

/* Per-kernel timing, off by default.  When enabled every kernel the library launches is bracketed
 * by HIP events on its stream.  cngp_profile_read() waits for those events, adds each kernel's
 * elapsed milliseconds and launch count into the caller's arrays (host, `max_kernels` entries;
 * kernel i is named cngp_profile_kernel_name(i)), clears the record and returns the number of
 * kernel kinds.  Not thread safe; meant for benchmarks. */
int         cngp_profile_enable(int on);
int         cngp_profile_read(double *ms_sum, int64_t *launches, int max_kernels);
const char *cngp_profile_kernel_name(int i);

const char *cngp_error_string(int status);
const char *cngp_last_hip_error(void);   /* text of the last failed HIP call in this thread, or "" */
int         cngp_version(void);          /* major * 10000 + minor * 100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* CNGP_H */

// C ABI of the Compact NGP encoding library: argument checks, level table, kernel
// selection and launches.  See include/cngp.h for the contract of every entry point.
#include "../../include/cngp.h"
#include "cngp_kernels.h"
#include "cngp_fwd_level.h"
#include "cngp_bwd_sliced.h"
#include "cngp_bwd_binned.h"
#include "cngp_rates.h"
#include "cngp_optim.h"
#include "cngp_mlp.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <type_traits>
#include <string>
#include <vector>
#include <algorithm>
#include <utility>

namespace {

using namespace cngp;

thread_local std::string g_hip_error;

bool is_pow2(uint32_t v) { return v != 0 && (v & (v - 1)) == 0; }
uint32_t ilog2(uint32_t v) { uint32_t r = 0; while (v > 1) { v >>= 1; ++r; } return r; }

int hip_fail(hipError_t e, const char *what) {
    g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return CNGP_ERR_HIP;
}
}  // namespace

// for the other translation unit of the library (cngp_sort.hip): same record as cngp_last_hip_error() reads
namespace cngp { int record_hip_failure(hipError_t e, const char *what) { return hip_fail(e, what); } }

namespace {
#define CNGP_HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) return hip_fail(e_, #call); } while (0)

// ---------------------------------------------------------------- static scratch of the allocation-free entry point
// cngp_encode_bwd_static works in this array instead of a caller's workspace.  Every GPU the library runs on
// holds its own copy, at its own address, until the process ends.  In host code the array's NAME is only a
// handle: the device address comes from hipGetSymbolAddress, once per device, and is what every launch gets.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
constexpr int    kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void **out) {
    int dev = -1;
    CNGP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return CNGP_ERR_UNSUPPORTED;
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        CNGP_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return CNGP_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CNGP_OK;
}

// ---------------------------------------------------------------- validation (host only)
int validate(const cngp_config *c) {
    if (!c) return CNGP_ERR_NULL;
    if (c->d < 2 || c->d > 4) return CNGP_ERR_INVALID;
    if (c->L < 1 || c->L > kMaxLevels) return CNGP_ERR_INVALID;
    if (c->F < 1) return CNGP_ERR_INVALID;
    if (!is_pow2(c->N_f) || !is_pow2(c->N_c) || !is_pow2(c->N_p)) return CNGP_ERR_INVALID;
    if (c->N_p > 16 || c->N_p > c->N_f) return CNGP_ERR_INVALID;
    if (c->N_f > (1u << 30) || c->N_c > (1u << 30)) return CNGP_ERR_INVALID;
    if (c->N_min < 1) return CNGP_ERR_INVALID;
    if (c->L > 1 && (c->N_max < c->N_min || c->N_max > (1u << 24))) return CNGP_ERR_INVALID;
    if (c->N_min > (1u << 24)) return CNGP_ERR_INVALID;
    if (c->feat_dtype != CNGP_F32 && c->feat_dtype != CNGP_F16) return CNGP_ERR_INVALID;
    if (c->io_dtype != CNGP_F32 && c->io_dtype != CNGP_F16) return CNGP_ERR_INVALID;
    if (c->index_format != CNGP_IDX_U8 && c->index_format != CNGP_IDX_PACKED4 && c->index_format != CNGP_IDX_BITS) return CNGP_ERR_INVALID;
    if (c->index_format == CNGP_IDX_PACKED4 && c->N_c < 2) return CNGP_ERR_INVALID;
    if (c->flags & ~(uint32_t)(CNGP_ZERO_GRADS | CNGP_BWD_DIRECT | CNGP_BWD_SLICED | CNGP_BWD_NO_PREREDUCE | CNGP_FWD_SIMPLE | CNGP_BWD_BINNED | CNGP_FWD_LEVEL | CNGP_FWD_TILE)) return CNGP_ERR_INVALID;
    if ((c->flags & CNGP_BWD_DIRECT) && (c->flags & (CNGP_BWD_SLICED | CNGP_BWD_BINNED))) return CNGP_ERR_INVALID;
    if ((c->flags & CNGP_FWD_LEVEL) && (c->flags & (CNGP_FWD_SIMPLE | CNGP_FWD_TILE))) return CNGP_ERR_INVALID;
    if (c->top_k > c->N_p || c->reserved != 0) return CNGP_ERR_INVALID;
    if (c->F != 1 && c->F != 2 && c->F != 4 && c->F != 8) return CNGP_ERR_UNSUPPORTED;
    return CNGP_OK;
}

// Table 1 (N_min, N_max, L): geometric growth, floor with a 1e-6 guard so that exact powers
// (in particular N_{L-1} = N_max) survive the rounding of exp / pow.
void level_table(const cngp_config *c, uint32_t *out) {
    if (c->L == 1) { out[0] = c->N_min; return; }
    const double b = std::exp(std::log((double)c->N_max / (double)c->N_min) / (double)(c->L - 1));
    for (int l = 0; l < c->L; ++l)
        out[l] = (uint32_t)std::floor((double)c->N_min * std::pow(b, (double)l) + 1e-6);
}

Params make_params(const cngp_config *c) {
    Params p;
    std::memset(&p, 0, sizeof(p));
    level_table(c, p.N_l);
    p.L = c->L;
    p.L_loaded = c->L;
    p.N_f = c->N_f;
    p.N_c = c->N_c;
    p.row_mask = c->N_f / c->N_p - 1;
    p.c_mask = c->N_c - 1;
    p.log2_Np = ilog2(c->N_p);
    p.top_k = (c->top_k && c->top_k < c->N_p) ? c->top_k : 0;
    return p;
}

// Bytes between the index codebooks of consecutive levels.
size_t index_level_bytes(const cngp_config *c) {
    if (c->index_format == CNGP_IDX_PACKED4) return c->N_c / 2;
    if (c->index_format == CNGP_IDX_BITS) return 4 * (((size_t)c->N_c * ilog2(c->N_p) + 31) / 32);
    return c->N_c;
}
// The exact-width format of a codebook with N_p = 1 has no bytes at all: its pointer may be NULL.
bool index_codebook_is_empty(const cngp_config *c) { return c->index_format == CNGP_IDX_BITS && c->N_p == 1; }

int check_blocks(int64_t blocks) { return (blocks > 0x7fffffffLL) ? CNGP_ERR_INVALID : CNGP_OK; }

// ---------------------------------------------------------------- per-kernel timing
enum KernelId { K_FWD = 0, K_BWD_DIRECT, K_BWD_PREP, K_BWD_SLICED, K_BWD_SLICED_V, K_BWD_GRID_DRAIN,
                K_BAKE, K_ZERO, K_DEBUG, K_ADAM, K_MLP_FWD, K_MLP_BWD,
                K_BWD_BIN_OFFSETS, K_BWD_BIN_SCATTER, K_BWD_BIN_DRAIN, K_BWD_INPUT, K_FUSED_FWD, K_PLANES, K_FWD_ROWS, K_COUNT };
const char *const kKernelNames[K_COUNT] = {"encode_fwd", "encode_bwd_direct", "encode_bwd_prepare",
                                           "encode_bwd_sliced_points_and_grid", "encode_bwd_sliced_vertices",
                                           "encode_bwd_bin_grid_sums", "bake_probes", "zero", "debug_indices",
                                           "adam_step_bake", "mlp_fwd", "mlp_bwd",
                                           "encode_bwd_bin_offsets", "encode_bwd_bin_scatter",
                                           "encode_bwd_bin_drain", "encode_bwd_input", "encode_mlp_fwd", "feature_planes",
                                           "encode_fwd_rows"};

struct TimedLaunch { int id; hipEvent_t t0, t1; };
bool g_profile = false;
std::vector<TimedLaunch> g_timed;

struct LaunchTimer {
    hipStream_t s; int id; hipEvent_t t0 = nullptr, t1 = nullptr; bool on;
    LaunchTimer(hipStream_t s_, int id_) : s(s_), id(id_), on(g_profile) {
        if (on && (hipEventCreate(&t0) != hipSuccess || hipEventCreate(&t1) != hipSuccess)) on = false;
        if (on) (void)hipEventRecord(t0, s);
    }
    ~LaunchTimer() {
        if (on) { (void)hipEventRecord(t1, s); g_timed.push_back({id, t0, t1}); }
    }
};

int launch_status(const char *what) {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? CNGP_OK : hip_fail(e, what);
}

// ---------------------------------------------------------------- launches
// Collects the arrays one call has to clear and clears them with a single launch.
struct ZeroList {
    ZeroSegments seg;
    int          n = 0;
    int64_t      largest = 0;
    void add(float *ptr, int64_t count) {
        if (count <= 0 || n >= kZeroSegments) return;
        seg.ptr[n] = ptr;
        seg.count[n] = count;
        if (count > largest) largest = count;
        ++n;
    }
    int launch(hipStream_t s) {
        if (n == 0) return CNGP_OK;
        int64_t blocks = (largest / 4 + kBlock - 1) / kBlock;
        if (blocks > 2048) blocks = 2048;
        if (blocks < 1) blocks = 1;
        LaunchTimer t(s, K_ZERO);
        zero_kernel<<<dim3((unsigned)blocks, (unsigned)n), kBlock, 0, s>>>(seg);
        n = 0;
        largest = 0;
        return launch_status("zero_kernel");
    }
};

template <typename K>
int allow_big_lds(K kernel, size_t bytes) {
    if (bytes <= 64 * 1024) return CNGP_OK;
    hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    return e == hipSuccess ? CNGP_OK : hip_fail(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)");
}

// Level-resident forward (cngp_fwd_level.h): which calls take it, and its launch shape.  Host arithmetic only.
struct FwdLevelPlan {
    bool     use = false;
    uint32_t resident = 0;       // entries of a level's feature codebook that sit in LDS
    size_t   lds = 0;            // dynamic LDS of the kernel
    int64_t  parts = 0, per_part = 0;
    size_t   yT_bytes = 0;       // the level-major copy of the encodings: the workspace this variant needs
};
constexpr size_t  kLevelLdsBudget = 156 * 1024;
constexpr int64_t kLevelPartPoints = 65536;              // points per workgroup when the batch is large

FwdLevelPlan fwd_level_plan(const cngp_config *c, int levels_loaded, int64_t N) {
    FwdLevelPlan f;
    if (c->F != 2 || levels_loaded < 1 || N <= 0 || (c->flags & (CNGP_FWD_SIMPLE | CNGP_FWD_TILE))) return f;
    const size_t entry = 2 * (c->feat_dtype == CNGP_F16 ? 2 : 4), io = c->io_dtype == CNGP_F16 ? 2 : 4;
    const size_t probes = (((size_t)c->N_c + 1) / 2 + 15) & ~(size_t)15;
    if (((size_t)c->N_f * entry) % 16 != 0 || probes > 64 * 1024) return f;
    size_t resident = (kLevelLdsBudget - probes) / entry;
    if (resident > c->N_f) resident = c->N_f;
    resident &= ~(size_t)3;                                              // whole 16-byte pieces
    // Measured on nerf3d's, image2d's and the compressed model's tables from 2^12 to 2^24 points: never slower than the
    // tile variant (1.2x - 3x faster), also when only a seventh of a level's feature codebook fits (sdf3d, 1.15x: the
    // workgroups of a level run on one XCD, so a level's table is held by one L2 instead of all eight).  So it is taken
    // whenever it can run -- except for a few thousand points, where its second launch costs more than it saves.
    if (!(c->flags & CNGP_FWD_LEVEL) && N * levels_loaded < ((int64_t)1 << 15)) return f;
    f.use = true;
    f.resident = (uint32_t)resident;
    f.lds = probes + resident * entry + 16;
    const int64_t step = (int64_t)kLevelBlock * kLevelUnroll;
    int64_t parts = 256 / levels_loaded;                                 // one workgroup per CU at least ...
    if (parts < N / kLevelPartPoints) parts = N / kLevelPartPoints;       // ... and many short ones for a large batch: the levels differ in cost
    if (parts > (N + step - 1) / step) parts = (N + step - 1) / step;
    if (parts < 1) parts = 1;
    f.per_part = ((N + parts - 1) / parts + step - 1) / step * step;
    f.parts = (N + f.per_part - 1) / f.per_part;
    f.yT_bytes = (size_t)N * c->L * 2 * io;
    return f;
}

template <int D, typename FeatT, typename IoT>
int launch_fwd_level(const cngp_config *c, const FwdLevelPlan &f, const Params &p, const float *x, int64_t N, const void *D_f,
                     const void *D_c, void *y, void *yT, hipStream_t s, const int32_t *perm, bool rows = true) {
    const size_t  c_stride = index_level_bytes(c);
    const int64_t blocks = f.parts * p.L_loaded;
    if (int rc = check_blocks(blocks)) return rc;
    const int vec = (c_stride % 16 == 0 && ((uintptr_t)D_c & 15u) == 0) ? 1 : 0;
#define CNGP_FWD_LEVEL_LAUNCH(FMT)                                                                          \
    do {                                                                                                    \
        auto kernel = encode_fwd_level_kernel<D, FeatT, IoT, FMT>;                                          \
        if (int rc = allow_big_lds(kernel, f.lds)) return rc;                                               \
        LaunchTimer t(s, K_FWD);                                                                            \
        kernel<<<(unsigned)blocks, kLevelBlock, f.lds, s>>>(p, x, (const FeatT *)D_f, (const uint8_t *)D_c, \
                                                            (IoT *)yT, N, (uint32_t)c_stride, vec, f.resident, f.per_part); \
    } while (0)
    if (c->index_format == CNGP_IDX_PACKED4) CNGP_FWD_LEVEL_LAUNCH(kFmtPacked4);
    else if (c->index_format == CNGP_IDX_BITS) CNGP_FWD_LEVEL_LAUNCH(kFmtBits);
    else CNGP_FWD_LEVEL_LAUNCH(kFmtU8);
#undef CNGP_FWD_LEVEL_LAUNCH
    if (int rc = launch_status("encode_fwd_level_kernel")) return rc;
    if (!rows) return CNGP_OK;                               // the caller reads the level-major array itself
    const int64_t tiles = (N + kRowsTile - 1) / kRowsTile;
    if (int rc = check_blocks(tiles)) return rc;
    const size_t lds = (size_t)kRowsTile * (c->L + 1) * 2 * sizeof(IoT);
    {
        LaunchTimer t(s, K_FWD_ROWS);
        level_major_to_rows_kernel<IoT><<<(unsigned)tiles, kRowsTile, lds, s>>>((const IoT *)yT, (IoT *)y, N, c->L, p.L_loaded, perm);
    }
    return launch_status("level_major_to_rows_kernel");
}

template <int D, typename FeatT, typename IoT>
int launch_fwd(const cngp_config *c, const Params &p, const float *x, int64_t N, const void *D_f,
               const void *D_c, void *y, hipStream_t s, const int32_t *perm = nullptr,
               void *workspace = nullptr, size_t workspace_bytes = 0) {
    // level-resident variant: large batches, when the caller lent the room for the level-major copy
    {
        const FwdLevelPlan f = fwd_level_plan(c, p.L_loaded, N);
        const bool room = workspace && workspace_bytes >= f.yT_bytes && ((uintptr_t)workspace & 255u) == 0 &&
                          ((uintptr_t)D_f & 15u) == 0;
        if (f.use && room) return launch_fwd_level<D, FeatT, IoT>(c, f, p, x, N, D_f, D_c, y, workspace, s, perm);
        if ((c->flags & CNGP_FWD_LEVEL) != 0) return f.use ? CNGP_ERR_WORKSPACE : CNGP_ERR_UNSUPPORTED;
    }
    // tile variant: one level's index codebook and the tile's outputs fit in LDS
    const size_t c_stride = index_level_bytes(c);
    const int    fmt = c->index_format;
    const size_t lds_probes = (((size_t)c->N_c + 1) / 2 + 15) & ~(size_t)15;
    const size_t lds = lds_probes + (size_t)kFwdTile * c->L * 2 * sizeof(IoT);
    const size_t lds_large = lds_probes + (size_t)kFwdTileLarge * c->L * 2 * sizeof(IoT);
    if (lds <= 64 * 1024 && N >= kFwdTile && !(c->flags & CNGP_FWD_SIMPLE)) {
        // Staging a level's codebook costs c_stride bytes per workgroup; a tile looks up TILE * 2^d entries.
        // When the staging outweighs the lookups of a small tile and there are points enough to keep every
        // CU busy with large ones, take the large tile.
        const bool large = c_stride >= 8192 && lds_large <= 128 * 1024 && N >= (int64_t)kFwdTileLarge * 1024;
        const int  tile = large ? kFwdTileLarge : kFwdTile;
        // a small feature codebook (the paper's compressed models) goes to LDS with the index codebook
        const size_t   feat_bytes = (size_t)c->N_f * 2 * sizeof(FeatT);
        // (measured: a third faster at N_f = 2^10, even at 2^12, slower from 2^13: the copy then costs more than the gathers it saves)
        const uint32_t feat_lds = (c->N_f <= 4096 && (large ? lds_large : lds) + feat_bytes <= 150 * 1024) ? (uint32_t)feat_bytes : 0u;
        const int64_t blocks = (N + tile - 1) / tile;
        if (int rc = check_blocks(blocks)) return rc;
        const int vec = (c_stride % 16 == 0 && ((uintptr_t)D_c & 15u) == 0) ? 1 : 0;
#define CNGP_FWD_TILE(FMT, TILE, LDS)                                                                   \
        do {                                                                                            \
            auto kernel = encode_fwd_tile_kernel<D, FeatT, IoT, FMT, TILE>;                             \
            if (int rc = allow_big_lds(kernel, LDS + feat_lds)) return rc;                              \
            LaunchTimer t(s, K_FWD);                                                                    \
            kernel<<<(unsigned)blocks, TILE, LDS + feat_lds, s>>>(                                      \
                p, x, (const FeatT *)D_f, (const uint8_t *)D_c, (IoT *)y, N, (uint32_t)c_stride, vec, perm, feat_lds); \
        } while (0)
#define CNGP_FWD_TILE_FMT(FMT)                                                                          \
        if (large) CNGP_FWD_TILE(FMT, kFwdTileLarge, lds_large); else CNGP_FWD_TILE(FMT, kFwdTile, lds)
        if (fmt == CNGP_IDX_PACKED4) { CNGP_FWD_TILE_FMT(kFmtPacked4); }
        else if (fmt == CNGP_IDX_BITS) { CNGP_FWD_TILE_FMT(kFmtBits); }
        else { CNGP_FWD_TILE_FMT(kFmtU8); }
#undef CNGP_FWD_TILE_FMT
#undef CNGP_FWD_TILE
        return launch_status("encode_fwd_tile_kernel");
    }
    const int64_t pairs = N * c->L;
    const int64_t blocks = (pairs + kBlock - 1) / kBlock;
    if (int rc = check_blocks(blocks)) return rc;
    LaunchTimer t(s, K_FWD);
#define CNGP_FWD_SIMPLE_LAUNCH(FMT)                                                                     \
    encode_fwd_kernel<D, FeatT, IoT, FMT><<<(unsigned)blocks, kBlock, 0, s>>>(                          \
        p, x, (const FeatT *)D_f, (const uint8_t *)D_c, (IoT *)y, pairs, (uint32_t)c_stride, perm)
    if (fmt == CNGP_IDX_PACKED4) CNGP_FWD_SIMPLE_LAUNCH(kFmtPacked4);
    else if (fmt == CNGP_IDX_BITS) CNGP_FWD_SIMPLE_LAUNCH(kFmtBits);
    else CNGP_FWD_SIMPLE_LAUNCH(kFmtU8);
#undef CNGP_FWD_SIMPLE_LAUNCH
    return launch_status("encode_fwd_kernel");
}

template <int D, typename FeatT, typename IoT>
int launch_bwd_input(const cngp_config *c, const Params &p, const float *x, int64_t N, const void *D_f,
                     const void *D_c, const void *dy, float *grad_x, hipStream_t s) {
    const size_t c_stride = index_level_bytes(c);
    const int    fmt = c->index_format;
    const size_t lds = (((size_t)c->N_c + 1) / 2 + 15) & ~(size_t)15;
    const bool   staged = lds <= 64 * 1024 && N >= kFwdTile;
    const bool   large = staged && c_stride >= 8192 && N >= (int64_t)kFwdTileLarge * 1024;
    const int    tile = large ? kFwdTileLarge : kFwdTile;
    const int64_t blocks = (N + tile - 1) / tile;
    if (int rc = check_blocks(blocks)) return rc;
    const int vec = (c_stride % 16 == 0 && ((uintptr_t)D_c & 15u) == 0) ? 1 : 0;
    LaunchTimer t(s, K_BWD_INPUT);
#define CNGP_BWD_INPUT(FMT, TILE, STAGED)                                                                   \
    encode_bwd_input_kernel<D, FeatT, IoT, FMT, TILE, STAGED><<<(unsigned)blocks, TILE, STAGED ? lds : 0, s>>>( \
        p, x, (const FeatT *)D_f, (const uint8_t *)D_c, (const IoT *)dy, grad_x, N, (uint32_t)c_stride, vec)
#define CNGP_BWD_INPUT_FMT(FMT)                                                                             \
    if (!staged) CNGP_BWD_INPUT(FMT, kFwdTile, false);                                                      \
    else if (large) CNGP_BWD_INPUT(FMT, kFwdTileLarge, true);                                               \
    else CNGP_BWD_INPUT(FMT, kFwdTile, true)
    if (fmt == CNGP_IDX_PACKED4) { CNGP_BWD_INPUT_FMT(kFmtPacked4); }
    else if (fmt == CNGP_IDX_BITS) { CNGP_BWD_INPUT_FMT(kFmtBits); }
    else { CNGP_BWD_INPUT_FMT(kFmtU8); }
#undef CNGP_BWD_INPUT_FMT
#undef CNGP_BWD_INPUT
    return launch_status("encode_bwd_input_kernel");
}

template <int D, int NP, typename FeatT, typename IoT>
int launch_bwd_direct(const cngp_config *c, const Params &p, int level0, int nlevels, const float *x,
                      int64_t N, const void *D_f, const float *Dhat_c, const void *dy, float *gD_f,
                      float *gDhat_c, hipStream_t s) {
    (void)c;
    if (nlevels <= 0) return CNGP_OK;
    constexpr int PTS = kBlock / NP;
    const int64_t blocks = (N + PTS - 1) / PTS;
    if (int rc = check_blocks(blocks)) return rc;
    LaunchTimer t(s, K_BWD_DIRECT);
    encode_bwd_direct_kernel<D, NP, FeatT, IoT><<<dim3((unsigned)blocks, (unsigned)nlevels), kBlock, 0, s>>>(
        p, level0, x, (const FeatT *)D_f, Dhat_c, (const IoT *)dy, gD_f, gDhat_c, N);
    return launch_status("encode_bwd_direct_kernel");
}


// ---------------------------------------------------------------- backward plan
size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// How one sliced kernel launch splits its items (points or grid vertices) into chunks.
struct Geom { uint32_t chunks, chunk_items; };

struct BwdPlan {
    bool     sliced;
    uint32_t rows_f_log2, slices_f;     // feature-gradient slices per level
    uint32_t rows_c_log2, slices_c;     // logit-gradient slices per level (0 when N_p == 1)
    Geom     feat_pts, logit_pts;       // hashed levels: chunks of points
    Geom     feat_vtx, logit_vtx;       // dense levels: chunks of grid vertices
    Geom     grid;                      // vertex-grid accumulation: chunks of points
    size_t   lds_f, lds_c;              // dynamic LDS bytes of the two kernels
    size_t   sigma_off, dyT_off, G_off, ws_bytes;
    bool     binned;                    // hashed levels: references binned by slice first (cngp_bwd_binned.h)
    bool     fused;                     // ... by slice of the confidence table only: a level's whole feature gradient sits in LDS beside it
    uint32_t bin_chunks, bin_chunk_pts; // point chunks of the count / scatter kernels
    uint32_t subs_f, subs_c;            // drain workgroups per bin
    size_t   cntF_off, cntC_off, baseF_off, baseC_off, recF_off, recC_off;
    size_t   cntG_off, baseG_off, recG_off;          // pre-reduced levels binned by slice of their vertex grid
    GridDrainPlan grid_drain;
    DenseLevels dense;                  // levels pre-reduced per grid vertex (a prefix of the levels)
    uint32_t dense_slices, dense_verts, dense_max_verts;
};

constexpr uint64_t kMaxAutoBinBytes = 8ull << 30;   // workspace the library asks for on its own initiative
constexpr uint32_t kMaxFusedNf = 4096;          // largest feature table per level whose gradient is kept whole in LDS
constexpr size_t   kFusedLdsBytes = 152 * 1024; // LDS of the workgroups that accumulate both gradients
constexpr uint32_t kMinBinnedSlicesPerLevel = 24; // from here on binning the references beats the replicated scan
constexpr uint32_t kMaxSlicesPerLevel = 128;   // beyond this the replicated scan costs more than global atomics
constexpr int64_t  kMinBinnedRefs = 1 << 21;    // corner references from which the library bins by itself (measured: 2^14 points of the headline shape)
constexpr int64_t  kMinSlicedRefs = 1 << 19;    // corner references (N * L * 2^d) below which launch overheads win
constexpr uint64_t kMaxDenseVerts = 32ull * kDenseSliceVerts;   // largest vertex grid that is pre-reduced
constexpr int64_t  kMinRefsPerVertex = 4;      // below this reuse the vertex pass saves nothing
constexpr int64_t  kCus = 256;

// Chunk count that minimises (rounds of workgroups over the CUs) x (items per chunk + fixed cost per
// workgroup, in items: clearing and flushing its LDS slice).  `groups` workgroups exist per chunk.
Geom pick_chunks(int64_t items, int64_t groups, int64_t fixed, int64_t min_chunk) {
    Geom best = {1, (uint32_t)((items + 63) / 64 * 64)};
    int64_t best_cost = -1;
    for (int64_t c = 1; c <= 64; ++c) {
        int64_t chunk = ((items + c - 1) / c + 63) / 64 * 64;
        if (chunk < 64) chunk = 64;
        if (c > 1 && chunk < min_chunk) break;
        const int64_t real = (items + chunk - 1) / chunk;                 // chunks that hold items
        const int64_t rounds = (groups * real + kCus - 1) / kCus;
        const int64_t cost = rounds * (chunk + fixed);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = {(uint32_t)real, (uint32_t)chunk}; }
    }
    if (best.chunks < 1) best.chunks = 1;
    return best;
}

// Chunk counts of the four roles of the sliced kernel, by simulating its launch: workgroups are
// handed out in grid order to the first free of 256 CUs; a workgroup costs a fixed part (clearing and
// flushing its LDS slice, about 12000 scanned points' worth) plus its items times a per-item cost that
// grows with the share of corners it keeps.  Measured on MI355X: fewer, longer workgroups win unless a
// finer split fills the last round.
double simulate_makespan(const std::vector<std::pair<int64_t, double>> &batches /* count, duration */) {
    std::vector<double> cu(kCus, 0.0);                      // min-heap of CU free times
    auto cmp = [](double a, double b) { return a > b; };
    double end = 0.0;
    for (const auto &bt : batches)
        for (int64_t i = 0; i < bt.first; ++i) {
            std::pop_heap(cu.begin(), cu.end(), cmp);
            cu.back() += bt.second;
            if (cu.back() > end) end = cu.back();
            std::push_heap(cu.begin(), cu.end(), cmp);
        }
    return end;
}

Geom chunks_of(int64_t items, int64_t c) {
    int64_t chunk = ((items + c - 1) / c + 63) / 64 * 64;
    if (chunk < 64) chunk = 64;
    return {(uint32_t)((items + chunk - 1) / chunk), (uint32_t)chunk};
}

void choose_geometry(const cngp_config *c, int64_t N, BwdPlan &b) {
    const int    Ld = b.dense.count, Lh = c->L - Ld;
    const double corners = (double)(1 << c->d);
    // fixed cost per workgroup ~ clearing and flushing its slice: 12000 points' worth for a full 128 KB slice
    const double fixed_f = 1500.0 + 10500.0 * (double)(((size_t)1 << b.rows_f_log2) * c->N_p * 16) / kSliceBytes;
    const double fixed_c = 1500.0 + 10500.0 * (double)(((size_t)1 << b.rows_c_log2) * c->N_p * 8) / kSliceBytes;
    const double item_f = 1.0 + 2.0 * corners / b.slices_f;                      // per point, feature role
    const double item_c = b.slices_c ? 1.0 + 1.5 * corners / b.slices_c : 0.0;   // per point, logit role
    const double vtx_f = 0.6 + 2.0 / b.slices_f, vtx_c = b.slices_c ? 0.6 + 1.5 / b.slices_c : 0.0;
    b.feat_vtx = b.logit_vtx = chunks_of(b.dense_max_verts ? b.dense_max_verts : 64, 1);
    if (Ld > 0) {
        b.grid = pick_chunks(N, b.dense_slices, 4096, 8192);
        const int64_t cv = (b.dense_max_verts + 16383) / 16384;                  // vertex chunks of <= 16384
        b.feat_vtx = b.logit_vtx = chunks_of(b.dense_max_verts, cv > 0 ? cv : 1);
    }
    if (b.binned) {                         // the point roles of the hashed levels are not launched
        b.logit_pts = b.feat_pts = chunks_of(N, 1);
        return;
    }
    // small slices are cheap to clear and flush: allow finer chunks there
    const bool    small = fixed_f + fixed_c < 8000.0;
    const int64_t min_chunk = small ? 8192 : 16384, cap = small ? 32 : 12;
    const int64_t cmax = N / min_chunk > 1 ? (N / min_chunk < cap ? N / min_chunk : cap) : 1;
    double best = -1.0;
    for (int64_t cc = 1; cc <= (b.slices_c ? cmax : 1); ++cc)
        for (int64_t cf = 1; cf <= cmax; ++cf) {
            const Geom gc = chunks_of(N, cc), gf = chunks_of(N, cf);
            std::vector<std::pair<int64_t, double>> batches;
            if (Lh > 0 && b.slices_c)
                batches.push_back({(int64_t)Lh * b.slices_c * gc.chunks, fixed_c + gc.chunk_items * item_c});
            if (Lh > 0)
                batches.push_back({(int64_t)Lh * b.slices_f * gf.chunks, fixed_f + gf.chunk_items * item_f});
            if (Ld > 0 && b.slices_c)
                batches.push_back({(int64_t)Ld * b.slices_c * b.logit_vtx.chunks, fixed_c + b.logit_vtx.chunk_items * vtx_c});
            if (Ld > 0)
                batches.push_back({(int64_t)Ld * b.slices_f * b.feat_vtx.chunks, fixed_f + b.feat_vtx.chunk_items * vtx_f});
            const double t = simulate_makespan(batches);
            if (best < 0.0 || t < best) { best = t; b.logit_pts = gc; b.feat_pts = gf; }
        }
}


BwdPlan make_bwd_plan_uncached(const cngp_config *c, int64_t N) {
    BwdPlan b;
    std::memset(&b, 0, sizeof(b));
    const uint32_t groups = c->N_f / c->N_p;                               // hashed rows of D_f
    const uint32_t max_rows_f = (uint32_t)kSliceBytes / (c->N_p * 2 * 8);
    const uint32_t rows_f = groups < max_rows_f ? groups : max_rows_f;
    b.rows_f_log2 = ilog2(rows_f);
    b.slices_f = groups / rows_f;
    if (c->N_p > 1) {
        const uint32_t max_rows_c = (uint32_t)kSliceBytes / (c->N_p * 8);
        const uint32_t rows_c = c->N_c < max_rows_c ? c->N_c : max_rows_c;
        b.rows_c_log2 = ilog2(rows_c);
        b.slices_c = c->N_c / rows_c;
    }
    // A small feature table (the paper's N_f = 2^6 .. 2^12): a level's whole feature gradient (fp64) and a copy of
    // its codebook fit in LDS beside a slice of the confidence table, and one pass over that table's bins gives
    // both gradients.  The confidence slice shrinks until everything fits in kFusedLdsBytes.
    const size_t feat_lds = (size_t)c->N_f * (2 * sizeof(double) + (c->feat_dtype == CNGP_F16 ? 4 : 8));
    bool fused_ok = c->N_p > 1 && c->N_f <= kMaxFusedNf;
    uint32_t fused_rows_c_log2 = b.rows_c_log2;
    while (fused_ok && (((size_t)1 << fused_rows_c_log2) * c->N_p * 8 + feat_lds > kFusedLdsBytes)) {
        if (fused_rows_c_log2 == 0) fused_ok = false;
        else --fused_rows_c_log2;
    }
    if (fused_ok && (c->N_c >> fused_rows_c_log2) > 8192) fused_ok = false;
    const uint32_t per_level = b.slices_f + b.slices_c;
    // a queued reference packs (row inside the slice, row of the other table) into 32 bits
    const bool keys_fit = b.rows_f_log2 + ilog2(c->N_c) <= 32 && b.rows_c_log2 + ilog2(groups) <= 32;
    const bool enough = (N << c->d) * c->L >= kMinSlicedRefs;
    b.sliced = per_level <= kMaxSlicesPerLevel && enough;
    // Binning the references of the hashed levels first (cngp_bwd_binned.h): possible whenever record
    // positions and byte offsets into a level fit 32 bits and a level's bins can be counted in LDS.  It pays
    // from about two dozen slices per level (measured: 24 slices 1.15x, 64 slices 1.6x over the replicated
    // scan; 10 slices 0.75x) and is the only LDS variant for tables of hundreds of slices.
    const bool bin_ok = keys_fit && N > 0 && ((uint64_t)N << c->d) < (1ull << 31) &&
                        b.slices_f <= 8192 && b.slices_c <= 8192 &&
                        (uint64_t)c->N_c * c->N_p <= (1ull << 29) && c->N_f <= (1u << 28);
    // (the bins take 4 bytes per reference, level and table: not chosen unasked beyond kMaxAutoBinBytes)
    const uint64_t bin_bytes = ((uint64_t)N << c->d) * kRecordBytes * (uint64_t)c->L * (c->N_p > 1 ? 2u : 1u);
    const uint64_t bin_bytes_max = c->bin_bytes_max ? c->bin_bytes_max : kMaxAutoBinBytes;
    // (with both gradients in one pass binning pays from four slices per level: below that the replicated scan is as fast)
    const bool plenty = (N << c->d) * c->L >= kMinBinnedRefs;           // below, the three extra launches cost more than they save
    b.binned = bin_ok && plenty && (per_level >= kMinBinnedSlicesPerLevel || (fused_ok && per_level >= 4)) && bin_bytes <= bin_bytes_max;
    if (c->flags & CNGP_BWD_BINNED) b.binned = bin_ok;
    if (c->flags & (CNGP_BWD_DIRECT | CNGP_BWD_SLICED)) b.binned = false;
    b.fused = b.binned && fused_ok;
    if (b.fused) {
        b.rows_c_log2 = fused_rows_c_log2;
        b.slices_c = c->N_c >> fused_rows_c_log2;
    }
    if (b.binned) b.sliced = true;
    if (c->flags & CNGP_BWD_DIRECT) b.sliced = false;
    if ((c->flags & CNGP_BWD_SLICED) && (uint64_t)per_level * 32u * 64u < 0x7fffffffull) b.sliced = true;
    if (!keys_fit) b.sliced = false;
    // coarse levels whose dense vertex grid is small, much smaller than the number of references, and
    // takes clearly fewer slice scans than the level's hashed tables.  With binning a hashed level costs
    // no replicated scan, and pre-reduction only pays for grids of a few slices.
    if (b.sliced && !(c->flags & CNGP_BWD_NO_PREREDUCE)) {
        uint32_t res[kMaxLevels];
        level_table(c, res);
        for (int l = 0; l < c->L && l < kMaxDense; ++l) {
            uint64_t verts = 1;
            for (int i = 0; i < c->d; ++i) verts *= (uint64_t)res[l] + 2;
            const uint64_t slices = (verts + kDenseSliceVerts - 1) / kDenseSliceVerts;
            if (verts > kMaxDenseVerts || (N << c->d) < kMinRefsPerVertex * (int64_t)verts) break;
            if (slices * 2 > per_level && slices > 1) break;
            if (b.fused) break;      // both gradients from one pass over the bins: cheaper than the grid sums and vertex scans (measured)
            if (b.binned && l == c->L - 1) break;                        // (at least one level stays hashed)
            b.dense.side[l] = res[l] + 2;
            b.dense.verts[l] = (uint32_t)verts;
            b.dense.slices[l] = (uint32_t)slices;
            b.dense.g_off[l] = b.dense_verts;
            b.dense_verts += (uint32_t)verts;
            b.dense_slices += (uint32_t)slices;
            if (verts > b.dense_max_verts) b.dense_max_verts = (uint32_t)verts;
            b.dense.count = l + 1;
        }
    }
    const int Lh = c->L - b.dense.count;
    if (b.sliced) choose_geometry(c, N, b);
    if (b.binned) {
        // chunks of at least 1024 points, at most 256 of them
        int64_t cp = ((N + 255) / 256 + 63) / 64 * 64;
        if (cp < 1024) cp = 1024;
        b.bin_chunk_pts = (uint32_t)cp;
        b.bin_chunks = (uint32_t)((N + cp - 1) / cp);
        // drain workgroups per bin: about 2^16 records each, and enough workgroups to fill the chip twice
        const double refs = (double)((uint64_t)N << c->d);
        auto subs = [&](uint32_t slices) -> uint32_t {
            if (!slices) return 1;
            double want = refs / slices / 65536.0;
            const double fill = 512.0 / ((double)Lh * (b.slices_f + b.slices_c));
            if (want < fill) want = fill;
            const double by_size = refs / slices / 8192.0;              // but never less than 8192 records each
            if (want > by_size) want = by_size;
            uint32_t r = (uint32_t)(want + 0.5);
            return r < 1 ? 1 : (r > 64 ? 64 : r);
        };
        b.subs_f = subs(b.slices_f);
        b.subs_c = subs(b.slices_c);
        if (b.fused) b.subs_f = 2;              // never one writer per entry: the feature gradient is cleared first and added to
    }
    const size_t queues = (size_t)kSlicedWaves * kRingBytes;
    b.lds_f = ((size_t)1 << b.rows_f_log2) * c->N_p * 2 * 8 + queues;
    b.lds_c = ((size_t)1 << b.rows_c_log2) * c->N_p * 8 + queues;
    if (b.sliced) {
        const size_t io = c->io_dtype == CNGP_F16 ? 2 : 4;
        b.sigma_off = 0;
        b.dyT_off = align256((size_t)c->L * c->N_c * c->N_p * sizeof(float));
        b.G_off = b.dyT_off + align256((size_t)N * c->L * c->F * io);
        b.ws_bytes = b.G_off + align256((size_t)b.dense_verts * 2 * sizeof(float));
        if (b.binned) {
            const size_t cap = (size_t)N << c->d;
            b.cntF_off = b.ws_bytes;
            b.cntC_off = b.cntF_off + align256((size_t)Lh * b.bin_chunks * b.slices_f * 4);
            b.baseF_off = b.cntC_off + align256((size_t)Lh * b.bin_chunks * b.slices_c * 4);
            b.baseC_off = b.baseF_off + align256((size_t)Lh * (b.slices_f + 1) * 4);
            b.recF_off = b.baseC_off + align256((size_t)Lh * (b.slices_c + 1) * 4);
            b.recC_off = b.recF_off + (b.fused ? 0 : align256((size_t)Lh * cap * kRecordBytes));
            b.cntG_off = b.recC_off + (b.slices_c ? align256((size_t)Lh * cap * kRecordBytes) : 0);
            const size_t Ld = (size_t)b.dense.count;
            b.baseG_off = b.cntG_off + align256(Ld * b.bin_chunks * kGridBins * 4);
            b.recG_off = b.baseG_off + align256(Ld * (kGridBins + 1) * 4);
            b.ws_bytes = b.recG_off + align256(Ld * cap * kRecordBytes);
            // workgroups per slice of a level's grid: about 2^15 references each
            uint32_t next = 0;
            for (int l = 0; l < b.dense.count; ++l) {
                uint64_t subs = (cap / b.dense.slices[l] + 32767) / 32768;
                if (subs < 1) subs = 1;
                if (subs > 256) subs = 256;
                b.grid_drain.first[l] = next;
                b.grid_drain.subs[l] = (uint32_t)subs;
                next += b.dense.slices[l] * (uint32_t)subs;
            }
            b.grid_drain.first[b.dense.count] = next;
        }
    }
    return b;
}

// The plan depends on (configuration, N) only; the last one is kept (host memory, per thread).
BwdPlan make_bwd_plan(const cngp_config *c, int64_t N) {
    thread_local cngp_config last_cfg;
    thread_local int64_t     last_N = -1;
    thread_local BwdPlan     last_plan;
    if (last_N == N && std::memcmp(&last_cfg, c, sizeof(*c)) == 0) return last_plan;
    last_plan = make_bwd_plan_uncached(c, N);
    last_cfg = *c;
    last_N = N;
    return last_plan;
}

// Points per pass of cngp_encode_bwd.  A batch whose bins would pass the configured limit (or whose references
// would not fit the 31-bit record positions) is taken in equal passes, each a complete backward over a run
// of points that accumulates onto the one before, when a pass of that size is binned; otherwise N.
int64_t bwd_pass_points(const cngp_config *c, int64_t N) {
    if (N <= 0 || (c->flags & (CNGP_BWD_DIRECT | CNGP_BWD_SLICED))) return N;
    int64_t most = (((int64_t)1 << 31) - 1) >> c->d;
    if (!(c->flags & CNGP_BWD_BINNED) || c->bin_bytes_max) {
        const int64_t per_point = ((int64_t)kRecordBytes << c->d) * c->L * (c->N_p > 1 ? 2 : 1);
        const int64_t by_bytes = (int64_t)((c->bin_bytes_max ? c->bin_bytes_max : kMaxAutoBinBytes) / (uint64_t)per_point);
        if (by_bytes < most) most = by_bytes;
    }
    most = most >= 65536 ? most / 65536 * 65536 : most / 1024 * 1024;
    if (N <= most || most <= 0) return N;
    const int64_t passes = (N + most - 1) / most;
    const int64_t per = ((N + passes - 1) / passes + 63) / 64 * 64;
    return make_bwd_plan_uncached(c, per).binned ? per : N;
}

template <int NP>
BinParams make_bin_params(const cngp_config *c, const BwdPlan &b, int64_t N) {
    BinParams bp;
    std::memset(&bp, 0, sizeof(bp));
    bp.level0 = b.dense.count;
    bp.nlevels = c->L - b.dense.count;
    bp.rows_f_log2 = b.rows_f_log2; bp.slices_f = b.fused ? 0 : b.slices_f;
    bp.rows_c_log2 = b.rows_c_log2; bp.slices_c = NP > 1 ? b.slices_c : 0;
    bp.chunks = b.bin_chunks; bp.chunk_pts = b.bin_chunk_pts;
    bp.cap = (uint32_t)((uint64_t)N << c->d);
    bp.dense_bins = b.dense.count > 0 ? 1 : 0;
    return bp;
}
// Bins of the level with the most of them, and the copies of the histogram the count keeps in LDS.
uint32_t most_bins_of(const BinParams &bp) { return bp.slices_f + bp.slices_c > kGridBins ? bp.slices_f + bp.slices_c : kGridBins; }
uint32_t hist_replicas_of(uint32_t most_bins) { return most_bins <= 64 ? 16u : most_bins <= 512 ? 4u : 1u; }

// Binned variant: (the count has run with the preparation launch) offsets, scatter (+ vertex-grid accumulation of the dense levels), drain
// (+ the two roles of the dense levels, which scan the finished vertex grids).
template <int D, int NP, typename FeatT, typename IoT>
int launch_bwd_binned(const cngp_config *c, const Params &p, const BwdPlan &b, const float *x, int64_t N,
                      const void *D_f, const float *sigma, const IoT *dyT, float *G, float *gD_f, float *gDhat_c,
                      void *workspace, hipStream_t s) {
    const int Ld = b.dense.count, Lh = c->L - Ld;
    char *ws = (char *)workspace;
    uint32_t *cntF = (uint32_t *)(ws + b.cntF_off), *cntC = (uint32_t *)(ws + b.cntC_off);
    uint32_t *baseF = (uint32_t *)(ws + b.baseF_off), *baseC = (uint32_t *)(ws + b.baseC_off);
    BinRecord *recF = (BinRecord *)(ws + b.recF_off), *recC = (BinRecord *)(ws + b.recC_off);
    uint32_t *cntG = (uint32_t *)(ws + b.cntG_off), *baseG = (uint32_t *)(ws + b.baseG_off);
    BinRecord *recG = (BinRecord *)(ws + b.recG_off);
    const bool zero_first = (c->flags & CNGP_ZERO_GRADS) != 0;
    const BinParams bp = make_bin_params<NP>(c, b, N);
    const int64_t blocks = (int64_t)(Lh + Ld) * bp.chunks;
    if (int rc = check_blocks(blocks)) return rc;
    const size_t lds_bins = (size_t)most_bins_of(bp) * sizeof(uint32_t);
    // One wavefront per chunk keeps a bin's records in the order of the points, which the drain's gathers
    // like (measured: drain 7 % faster); with many bins a lone wavefront fills its cache lines too slowly
    // for the memory system to merge the 4-byte writes, and four wavefronts sharing the cursors write
    // 1.7 times faster (measured at 64 bins per level).
    const unsigned bin_block = bp.slices_f + bp.slices_c >= 48 ? 256u : (unsigned)kBinBlock;
    {
        LaunchTimer t(s, K_BWD_BIN_OFFSETS);
        uint32_t big = bp.slices_f > bp.slices_c ? bp.slices_f : bp.slices_c;
        if (Ld > 0 && big < kGridBins) big = kGridBins;
        const uint32_t words = (uint64_t)bp.chunks * big <= 36864 ? bp.chunks * big : 0u;    // up to 144 KB of LDS
        if (int rc = allow_big_lds(bin_offsets_kernel, (size_t)words * 4)) return rc;
        bin_offsets_kernel<<<(unsigned)(2 * Lh + Ld), kOffsetsBlock, (size_t)words * 4, s>>>(bp, cntF, cntC, cntG, baseF, baseC,
                                                                                            baseG, words);
        if (int rc = launch_status("bin_offsets_kernel")) return rc;
    }
    {
        LaunchTimer t(s, K_BWD_BIN_SCATTER);
        bin_scatter_kernel<D><<<(unsigned)blocks, bin_block, lds_bins, s>>>(p, bp, b.dense, x, N, cntF, cntC, cntG, recF, recC, recG);
        if (int rc = launch_status("bin_scatter_kernel")) return rc;
    }
    if (Ld > 0) {   // vertex-grid sums of the pre-reduced levels from their bins
        auto kernel = bin_grid_drain_kernel<D, IoT>;
        const size_t lds_grid = (size_t)kDenseSliceVerts * 2 * sizeof(double);
        if (int rc = allow_big_lds(kernel, lds_grid)) return rc;
        LaunchTimer t(s, K_BWD_GRID_DRAIN);
        kernel<<<b.grid_drain.first[Ld], kSlicedBlock, lds_grid, s>>>(p, b.dense, b.grid_drain, x, dyT, N, recG, baseG, bp.cap, G);
        if (int rc = launch_status("bin_grid_drain_kernel")) return rc;
    }
    auto role = [&](uint32_t rows_log2, uint32_t slices, const Geom &g, int level0, int nlevels, uint32_t &wgs) {
        SliceParams sp;
        std::memset(&sp, 0, sizeof(sp));
        sp.rows_log2 = rows_log2;
        sp.slices = slices ? slices : 1;
        sp.chunks = g.chunks ? g.chunks : 1;
        sp.chunk_pts = g.chunk_items;
        sp.store_direct = (sp.chunks == 1 && zero_first) ? 1 : 0;       // matches the clearing in cngp_encode_bwd
        sp.level0 = level0;
        sp.nlevels = slices ? nlevels : 0;
        wgs = (slices && nlevels > 0) ? (uint32_t)kXcds * (((uint32_t)nlevels * sp.slices * sp.chunks + kXcds - 1) / kXcds) : 0u;
        return sp;
    };
    uint32_t wgs_c = 0, wgs_f = 0, wgs_cv = 0, wgs_fv = 0;
    const uint32_t slices_c = NP > 1 ? b.slices_c : 0;
    const SliceParams sp_c = role(b.rows_c_log2, slices_c, Geom{b.subs_c, 0}, Ld, Lh, wgs_c);
    const SliceParams sp_f = role(b.rows_f_log2, b.fused ? 0u : b.slices_f, Geom{b.subs_f, 0}, Ld, Lh, wgs_f);
    BwdRoles vtx;
    std::memset(&vtx, 0, sizeof(vtx));
    vtx.sp[ROLE_LOGIT_VTX] = role(b.rows_c_log2, slices_c, b.logit_vtx, 0, Ld, wgs_cv);
    vtx.sp[ROLE_FEAT_VTX] = role(b.rows_f_log2, b.slices_f, b.feat_vtx, 0, Ld, wgs_fv);
    vtx.first[ROLE_LOGIT_VTX] = 0;
    vtx.first[ROLE_FEAT_VTX] = wgs_cv;
    auto kernel = bin_drain_kernel<D, NP, FeatT, IoT>;
    size_t lds = b.lds_f > b.lds_c ? b.lds_f : b.lds_c;                 // slice + the vertex roles' ring buffers
    if (b.fused) {
        const size_t both = ((size_t)1 << b.rows_c_log2) * NP * 8 + (size_t)c->N_f * (2 * sizeof(double) + sizeof(typename RawPair<FeatT>::type));
        if (both > lds) lds = both;
    }
    if (int rc = allow_big_lds(kernel, lds)) return rc;
    const uint32_t total = wgs_c + wgs_f + wgs_cv + wgs_fv;
    if (total == 0) return CNGP_OK;
    LaunchTimer t(s, K_BWD_BIN_DRAIN);
    kernel<<<total, kSlicedBlock, lds, s>>>(p, sp_c, sp_f, wgs_c, wgs_c + wgs_f, x, dyT, N, (const FeatT *)D_f, sigma, recF, recC,
                                            baseF, baseC, bp.cap, vtx, b.dense, G, gD_f, gDhat_c);
    return launch_status("bin_drain_kernel");
}

template <int D, int NP, typename FeatT, typename IoT>
int launch_bwd_sliced(const cngp_config *c, const Params &p, const BwdPlan &b, const float *x, int64_t N,
                      const void *D_f, const float *Dhat_c, const void *dy, float *gD_f, float *gDhat_c,
                      void *workspace, ZeroList &zero, hipStream_t s) {
    float *sigma = reinterpret_cast<float *>((char *)workspace + b.sigma_off);
    IoT   *dyT = reinterpret_cast<IoT *>((char *)workspace + b.dyT_off);
    // per-vertex sums of weight * dL/dy on the dense levels
    float *G = reinterpret_cast<float *>((char *)workspace + b.G_off);
    const int Ld = b.dense.count, Lh = c->L - Ld;
    bool grid_direct = b.grid.chunks == 1;
    if (b.binned) {
        grid_direct = true;
        for (int l = 0; l < Ld; ++l) grid_direct = grid_direct && b.grid_drain.subs[l] == 1;
    }
    if (Ld > 0 && !grid_direct) zero.add(G, (int64_t)b.dense_verts * 2);
    {   // one launch: clear what is accumulated with atomics, softmax table, level-major dL/dy
        using PairT = typename std::conditional<sizeof(IoT) == 2, uint32_t, float2>::type;
        const int64_t elems = NP > 1 ? (int64_t)c->L * c->N_c * NP : 0;
        const int64_t softmax_blocks = (elems + kBlock - 1) / kBlock;
        const int64_t transpose_blocks = (N + kBlock - 1) / kBlock;
        int64_t zero_blocks = (zero.largest / 4 + kBlock - 1) / kBlock;
        if (zero_blocks > 1024) zero_blocks = 1024;
        if (zero_blocks < 1) zero_blocks = 1;
        const int64_t blocks = (int64_t)zero.n * zero_blocks + softmax_blocks + transpose_blocks;
        if (int rc = check_blocks(blocks)) return rc;
        PrepArgs a;
        a.seg = zero.seg; a.seg_count = (uint32_t)zero.n; a.zero_blocks = (uint32_t)zero_blocks;
        a.Dhat_c = Dhat_c; a.sigma = sigma; a.elems = elems; a.softmax_blocks = (uint32_t)softmax_blocks;
        a.dy = dy; a.dyT = dyT; a.N = N; a.L = c->L; a.top_k = p.top_k;
        LaunchTimer t(s, K_BWD_PREP);
        if (b.binned) {          // the count of the binned variant rides along: it needs nothing this launch writes
            const BinParams bp = make_bin_params<NP>(c, b, N);
            const int64_t   count_blocks = (int64_t)c->L * bp.chunks;
            if (int rc = check_blocks(blocks + count_blocks)) return rc;
            const uint32_t most = most_bins_of(bp), reps = hist_replicas_of(most);
            char *ws = (char *)workspace;
            bwd_prep_count_kernel<D, NP, PairT><<<(unsigned)(blocks + count_blocks), kBlock, (size_t)most * reps * sizeof(uint32_t), s>>>(
                a, p, bp, b.dense, x, (uint32_t *)(ws + b.cntF_off), (uint32_t *)(ws + b.cntC_off), (uint32_t *)(ws + b.cntG_off),
                reps, (uint32_t)count_blocks);
        } else {
            bwd_prep_kernel<NP, PairT><<<(unsigned)blocks, kBlock, 0, s>>>(a);
        }
        zero.n = 0;
        zero.largest = 0;
        if (int rc = launch_status("bwd_prep_kernel")) return rc;
    }

    if (b.binned)
        return launch_bwd_binned<D, NP, FeatT, IoT>(c, p, b, x, N, D_f, sigma, dyT, G, gD_f, gDhat_c, workspace, s);

    // Launch 1: feature and logit gradients of the hashed levels (scan the points) together with the
    // vertex-grid accumulation of the dense levels.  Launch 2: the two gradients of the dense levels
    // (scan the vertex grids, which launch 1 has completed).
    const bool zero_first = (c->flags & CNGP_ZERO_GRADS) != 0;
    auto kernel = bwd_sliced_kernel<D, NP, FeatT, IoT>;
    size_t lds = b.lds_f > b.lds_c ? b.lds_f : b.lds_c;
    const size_t lds_grid = (size_t)kDenseSliceVerts * 2 * sizeof(double);
    if (Ld > 0 && lds_grid > lds) lds = lds_grid;
    if (int rc = allow_big_lds(kernel, lds)) return rc;
    for (int launch = 0; launch < 2; ++launch) {
        BwdRoles roles;
        std::memset(&roles, 0, sizeof(roles));
        uint32_t next = 0;
        auto add_role = [&](int role, bool present, const Geom &g, uint32_t rows_log2, uint32_t slices, int level0,
                            int nlevels) {
            SliceParams &sp = roles.sp[role];
            sp.rows_log2 = rows_log2;
            sp.slices = slices ? slices : 1;
            sp.chunks = g.chunks ? g.chunks : 1;
            sp.chunk_pts = g.chunk_items;
            sp.store_direct = (g.chunks == 1 && zero_first) ? 1 : 0;     // matches the clearing in cngp_encode_bwd
            sp.level0 = level0;
            sp.nlevels = present ? nlevels : 0;
            roles.first[role] = next;
            if (present && nlevels > 0)      // 8 equal runs of (level, slice, chunk) units, one per XCD
                next += (uint32_t)kXcds * (((uint32_t)nlevels * sp.slices * sp.chunks + kXcds - 1) / kXcds);
        };
        const bool pts = launch == 0, vtx = launch == 1;
        add_role(ROLE_LOGIT_PTS, pts && NP > 1, b.logit_pts, b.rows_c_log2, b.slices_c, Ld, Lh);
        add_role(ROLE_FEAT_PTS, pts, b.feat_pts, b.rows_f_log2, b.slices_f, Ld, Lh);
        add_role(ROLE_LOGIT_VTX, vtx && NP > 1, b.logit_vtx, b.rows_c_log2, b.slices_c, 0, Ld);
        add_role(ROLE_FEAT_VTX, vtx, b.feat_vtx, b.rows_f_log2, b.slices_f, 0, Ld);
        roles.first[ROLE_GRID] = next;
        roles.sp[ROLE_GRID].chunks = b.grid.chunks ? b.grid.chunks : 1;
        roles.sp[ROLE_GRID].chunk_pts = b.grid.chunk_items;
        roles.sp[ROLE_GRID].store_direct = grid_direct;
        if (pts && Ld > 0) next += b.dense_slices * roles.sp[ROLE_GRID].chunks;
        roles.first[ROLE_COUNT] = next;
        if (next == 0) continue;
        LaunchTimer t(s, pts ? K_BWD_SLICED : K_BWD_SLICED_V);
        kernel<<<next, kSlicedBlock, lds, s>>>(p, roles, b.dense, x, (const FeatT *)D_f, sigma, dyT, G, gD_f, gDhat_c, N);
        if (int rc = launch_status("bwd_sliced_kernel")) return rc;
    }
    return CNGP_OK;
}

template <int D, typename FeatT, typename IoT>
int dispatch_bwd_np(const cngp_config *c, const Params &p, const BwdPlan &b, const float *x, int64_t N,
                    const void *D_f, const float *Dhat_c, const void *dy, float *gD_f, float *gDhat_c,
                    void *workspace, ZeroList &zero, hipStream_t s) {
#define CNGP_BWD_CASE(NP)                                                                                        \
    if (b.sliced) return launch_bwd_sliced<D, NP, FeatT, IoT>(c, p, b, x, N, D_f, Dhat_c, dy, gD_f, gDhat_c, workspace, zero, s); \
    if (int rc = zero.launch(s)) return rc;                                                                         \
    return launch_bwd_direct<D, NP, FeatT, IoT>(c, p, 0, c->L, x, N, D_f, Dhat_c, dy, gD_f, gDhat_c, s)
    switch (c->N_p) {
    case 1:  CNGP_BWD_CASE(1);
    case 2:  CNGP_BWD_CASE(2);
    case 4:  CNGP_BWD_CASE(4);
    case 8:  CNGP_BWD_CASE(8);
    default: CNGP_BWD_CASE(16);
    }
#undef CNGP_BWD_CASE
}

// d x feat_dtype x io_dtype -> template instance
#define CNGP_DISPATCH_TYPES(FN, ...)                                                             \
    do {                                                                                         \
        const bool f16 = cfg->feat_dtype == CNGP_F16, io16 = cfg->io_dtype == CNGP_F16;          \
        if (cfg->d == 2) {                                                                       \
            if (f16) return io16 ? FN<2, __half, __half>(__VA_ARGS__) : FN<2, __half, float>(__VA_ARGS__); \
            return io16 ? FN<2, float, __half>(__VA_ARGS__) : FN<2, float, float>(__VA_ARGS__);  \
        }                                                                                        \
        if (cfg->d == 3) {                                                                       \
            if (f16) return io16 ? FN<3, __half, __half>(__VA_ARGS__) : FN<3, __half, float>(__VA_ARGS__); \
            return io16 ? FN<3, float, __half>(__VA_ARGS__) : FN<3, float, float>(__VA_ARGS__);  \
        }                                                                                        \
        if (f16) return io16 ? FN<4, __half, __half>(__VA_ARGS__) : FN<4, __half, float>(__VA_ARGS__);     \
        return io16 ? FN<4, float, __half>(__VA_ARGS__) : FN<4, float, float>(__VA_ARGS__);      \
    } while (0)

}  // namespace

// ==================================================================== exported C ABI
namespace {
template <int D, typename FeatT, typename IoT>
int launch_fused_fwd(const cngp_config *c, const Params &p, const MlpDims &d, const float *x, int64_t N, const void *D_f,
                     const void *D_c, const void *W, float *out, hipStream_t s) {
    const size_t c_stride = index_level_bytes(c);
    size_t rest = (((size_t)c->N_c + 1) / 2 + 15) & ~(size_t)15;
    if (rest < kMlpRawBytes) rest = kMlpRawBytes;
    const size_t lds = kMlpFwdOps + (size_t)kFusedTile * kFusedStride * sizeof(_Float16) + rest;
    if (lds > 128 * 1024) return CNGP_ERR_UNSUPPORTED;
    const int64_t tiles = (N + kFusedTile - 1) / kFusedTile;
    int64_t per_cu = (int64_t)(160 * 1024 / lds);            // workgroups that fit a CU at once: LDS, and three
    if (per_cu > 3) per_cu = 3;                              // wavefronts per SIMD by registers
    if (per_cu < 1) per_cu = 1;
    const int64_t blocks = tiles < 256 * per_cu ? tiles : 256 * per_cu;
    const int vec = (c_stride % 16 == 0 && ((uintptr_t)D_c & 15u) == 0) ? 1 : 0;
#define CNGP_FUSED(FMT)                                                                                   \
    do {                                                                                                  \
        auto kernel = encode_mlp_fwd_kernel<D, FeatT, FMT>;                                               \
        if (int rc = allow_big_lds(kernel, lds)) return rc;                                               \
        LaunchTimer t(s, K_FUSED_FWD);                                                                    \
        kernel<<<(unsigned)blocks, kFusedTile, lds, s>>>(p, d, x, (const FeatT *)D_f, (const uint8_t *)D_c, \
                                                         (const __half *)W, out, N, tiles, (uint32_t)c_stride, vec); \
    } while (0)
    if (c->index_format == CNGP_IDX_PACKED4) CNGP_FUSED(kFmtPacked4);
    else if (c->index_format == CNGP_IDX_BITS) CNGP_FUSED(kFmtBits);
    else CNGP_FUSED(kFmtU8);
#undef CNGP_FUSED
    return launch_status("encode_mlp_fwd_kernel");
}
}  // namespace

namespace {
// Workspace of the entry points for entries of two features (every kernel's native width).
size_t workspace_bytes_pairs(const cngp_config *cfg, int64_t N) {
    const int64_t per = bwd_pass_points(cfg, N);
    if (per >= N) return make_bwd_plan(cfg, N).ws_bytes;
    const size_t  most = make_bwd_plan_uncached(cfg, per).ws_bytes;          // the last pass is the shorter one
    const size_t  last = make_bwd_plan_uncached(cfg, N - (N - 1) / per * per).ws_bytes;
    return most > last ? most : last;
}

// ---------------------------------------------------------------- feature widths other than two
// F = 1, 4, 8 run as ceil(F / 2) passes over pair planes (cngp_kernels.h, plane_take_kernel): behind the workspace
// of the two-feature problem sit one plane of D_f, one plane of y or dL/dy, and one plane of grad D_f.
struct PlaneSpace { size_t pairs, D_off, io_off, g_off, total; };
cngp_config as_pairs(const cngp_config *c) { cngp_config p = *c; p.F = 2; return p; }
PlaneSpace plane_space(const cngp_config *c, int64_t N) {
    const cngp_config c2 = as_pairs(c);
    PlaneSpace ps;
    const size_t bwd = workspace_bytes_pairs(&c2, N), fwd = fwd_level_plan(&c2, c2.L, N).yT_bytes;
    ps.pairs = align256(bwd > fwd ? bwd : fwd);
    ps.D_off = ps.pairs;
    ps.io_off = ps.D_off + align256((size_t)c->L * c->N_f * 2 * (c->feat_dtype == CNGP_F16 ? 2 : 4));
    ps.g_off = ps.io_off + align256((size_t)N * c->L * 2 * (c->io_dtype == CNGP_F16 ? 2 : 4));
    ps.total = ps.g_off + align256((size_t)c->L * c->N_f * 2 * sizeof(float));
    return ps;
}

template <typename T>
int take_plane(const void *src, void *dst, int64_t rows, int F, int plane, hipStream_t s) {
    if (rows <= 0) return CNGP_OK;
    const int64_t blocks = (rows + kBlock - 1) / kBlock;
    if (int rc = check_blocks(blocks)) return rc;
    LaunchTimer t(s, K_PLANES);
    plane_take_kernel<T><<<(unsigned)blocks, kBlock, 0, s>>>((const T *)src, (T *)dst, rows, F, plane);
    return launch_status("plane_take_kernel");
}
template <typename T>
int put_plane(const void *src, void *dst, int64_t rows, int F, int plane, bool accumulate, hipStream_t s) {
    if (rows <= 0) return CNGP_OK;
    const int64_t blocks = (rows + kBlock - 1) / kBlock;
    if (int rc = check_blocks(blocks)) return rc;
    LaunchTimer t(s, K_PLANES);
    plane_put_kernel<T><<<(unsigned)blocks, kBlock, 0, s>>>((const T *)src, (T *)dst, rows, F, plane, accumulate ? 1 : 0);
    return launch_status("plane_put_kernel");
}
int take_plane_dt(int dtype, const void *src, void *dst, int64_t rows, int F, int plane, hipStream_t s) {
    return dtype == CNGP_F16 ? take_plane<__half>(src, dst, rows, F, plane, s) : take_plane<float>(src, dst, rows, F, plane, s);
}
int put_plane_dt(int dtype, const void *src, void *dst, int64_t rows, int F, int plane, bool acc, hipStream_t s) {
    return dtype == CNGP_F16 ? put_plane<__half>(src, dst, rows, F, plane, acc, s) : put_plane<float>(src, dst, rows, F, plane, acc, s);
}
bool plane_workspace_ok(const void *ws, size_t bytes, const PlaneSpace &ps) {
    return ws && ((uintptr_t)ws & 255u) == 0 && bytes >= ps.total;
}

int fwd_planes(const cngp_config *cfg, int32_t levels_loaded, const float *x, int64_t N, const void *D_f, const void *D_c,
               void *y, void *workspace, size_t workspace_bytes, void *stream) {
    const PlaneSpace ps = plane_space(cfg, N);
    if (!plane_workspace_ok(workspace, workspace_bytes, ps)) return CNGP_ERR_WORKSPACE;
    const cngp_config c2 = as_pairs(cfg);
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    for (int p = 0; p < (cfg->F + 1) / 2; ++p) {
        if (int rc = take_plane_dt(cfg->feat_dtype, D_f, ws + ps.D_off, (int64_t)levels_loaded * cfg->N_f, cfg->F, p, s)) return rc;
        if (int rc = cngp_encode_fwd_partial(&c2, levels_loaded, x, N, ws + ps.D_off, D_c, ws + ps.io_off, workspace, ps.pairs, stream)) return rc;
        if (int rc = put_plane_dt(cfg->io_dtype, ws + ps.io_off, y, N * cfg->L, cfg->F, p, false, s)) return rc;
    }
    return CNGP_OK;
}

int bwd_planes(const cngp_config *cfg, const float *x, int64_t N, const void *D_f, const float *Dhat_c, const void *dy,
               float *grad_D_f, float *grad_Dhat_c, void *workspace, size_t workspace_bytes, void *stream) {
    hipStream_t s = (hipStream_t)stream;
    const bool zero_first = (cfg->flags & CNGP_ZERO_GRADS) != 0;
    if (N == 0) {                                   // nothing to add; clear if asked
        ZeroList z;
        if (zero_first) { z.add(grad_D_f, (int64_t)cfg->L * cfg->N_f * cfg->F); z.add(grad_Dhat_c, (int64_t)cfg->L * cfg->N_c * cfg->N_p); }
        return z.launch(s);
    }
    const PlaneSpace ps = plane_space(cfg, N);
    if (!plane_workspace_ok(workspace, workspace_bytes, ps)) return CNGP_ERR_WORKSPACE;
    cngp_config c2 = as_pairs(cfg);
    c2.flags &= ~(uint32_t)CNGP_ZERO_GRADS;         // the plane of grad D_f is cleared here, grad D^_c once if asked
    char  *ws = (char *)workspace;
    float *gp = (float *)(ws + ps.g_off);
    for (int p = 0; p < (cfg->F + 1) / 2; ++p) {
        ZeroList z;
        z.add(gp, (int64_t)cfg->L * cfg->N_f * 2);
        if (p == 0 && zero_first) z.add(grad_Dhat_c, (int64_t)cfg->L * cfg->N_c * cfg->N_p);
        if (int rc = z.launch(s)) return rc;
        if (int rc = take_plane_dt(cfg->feat_dtype, D_f, ws + ps.D_off, (int64_t)cfg->L * cfg->N_f, cfg->F, p, s)) return rc;
        if (int rc = take_plane_dt(cfg->io_dtype, dy, ws + ps.io_off, N * cfg->L, cfg->F, p, s)) return rc;
        if (int rc = cngp_encode_bwd(&c2, x, N, ws + ps.D_off, Dhat_c, ws + ps.io_off, gp, grad_Dhat_c, workspace, ps.pairs, stream)) return rc;
        if (int rc = put_plane<float>(gp, grad_D_f, (int64_t)cfg->L * cfg->N_f, cfg->F, p, !zero_first, s)) return rc;
    }
    return CNGP_OK;
}

int adam_coefficients(const cngp_adam *o, AdamCoef *a) {
    if (!(o->lr >= 0.0f) || !std::isfinite(o->lr)) return CNGP_ERR_INVALID;
    if (!(o->beta1 >= 0.0f && o->beta1 < 1.0f) || !(o->beta2 >= 0.0f && o->beta2 < 1.0f)) return CNGP_ERR_INVALID;
    if (!(o->eps > 0.0f) || !std::isfinite(o->eps) || !std::isfinite(o->grad_scale) || o->step < 1) return CNGP_ERR_INVALID;
    const double c1 = 1.0 - std::pow((double)o->beta1, (double)o->step);
    const double c2 = 1.0 - std::pow((double)o->beta2, (double)o->step);
    a->b1 = o->beta1;  a->one_minus_b1 = (float)(1.0 - (double)o->beta1);
    a->b2 = o->beta2;  a->one_minus_b2 = (float)(1.0 - (double)o->beta2);
    a->step = (float)((double)o->lr / c1);
    a->rsqrt_c2 = (float)(1.0 / std::sqrt(c2));
    a->eps = o->eps;
    a->grad_scale = o->grad_scale;
    return CNGP_OK;
}
bool aligned(const void *p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }
}  // namespace

extern "C" {

int cngp_version(void) { return 100; }

const char *cngp_error_string(int status) {
    switch (status) {
    case CNGP_OK:              return "success";
    case CNGP_ERR_NULL:        return "a required pointer is NULL";
    case CNGP_ERR_INVALID:     return "invalid argument (size out of range or not a power of two)";
    case CNGP_ERR_UNSUPPORTED: return "valid in the paper's terms, not supported by this entry point (F other than 1, 2, 4, 8; F != 2 where no workspace can hold the pair planes)";
    case CNGP_ERR_WORKSPACE:   return "workspace missing, misaligned or too small";
    case CNGP_ERR_HIP:         return "a HIP call failed (see cngp_last_hip_error)";
    default:                   return "unknown status";
    }
}

const char *cngp_last_hip_error(void) { return g_hip_error.c_str(); }

int cngp_level_resolutions(const cngp_config *cfg, uint32_t *out_N_l) {
    if (!cfg || !out_N_l) return CNGP_ERR_NULL;
    int rc = validate(cfg);
    if (rc != CNGP_OK && rc != CNGP_ERR_UNSUPPORTED) return rc;
    level_table(cfg, out_N_l);
    return CNGP_OK;
}

size_t cngp_workspace_bytes(const cngp_config *cfg, int64_t N) {
    if (validate(cfg) != CNGP_OK || N <= 0) return 0;
    if (cfg->F != 2) return plane_space(cfg, N).total;
    const size_t bwd = workspace_bytes_pairs(cfg, N), fwd = fwd_level_plan(cfg, cfg->L, N).yT_bytes;
    return bwd > fwd ? bwd : fwd;
}

int cngp_fwd_plan_info(const cngp_config *cfg, int64_t N, int32_t *info) {
    if (!info) return CNGP_ERR_NULL;
    if (int rc = validate(cfg)) return rc;
    if (N < 0) return CNGP_ERR_INVALID;
    const cngp_config pairs = as_pairs(cfg);
    const FwdLevelPlan f = fwd_level_plan(&pairs, cfg->L, N);
    info[0] = f.use ? 1 : 0;
    info[1] = (int32_t)f.resident;
    info[2] = (int32_t)(f.parts > 0x7fffffffLL ? 0x7fffffffLL : f.parts);
    info[3] = (int32_t)(f.lds);
    return CNGP_OK;
}

size_t cngp_fwd_workspace_bytes(const cngp_config *cfg, int64_t N) {
    if (validate(cfg) != CNGP_OK || N <= 0) return 0;
    if (cfg->F != 2) return plane_space(cfg, N).total;
    return fwd_level_plan(cfg, cfg->L, N).yT_bytes;
}

int cngp_bwd_plan_info(const cngp_config *cfg, int64_t N, int32_t *info) {
    if (!info) return CNGP_ERR_NULL;
    if (int rc = validate(cfg)) return rc;
    if (N < 0) return CNGP_ERR_INVALID;
    const cngp_config pairs = as_pairs(cfg);                // other widths run as passes over pairs of features
    cfg = &pairs;
    const int64_t per = bwd_pass_points(cfg, N);
    const BwdPlan b = make_bwd_plan(cfg, per < N ? per : N);
    const int32_t v[CNGP_PLAN_INFO_COUNT] = {
        b.sliced ? 1 : 0, b.dense.count, (int32_t)(b.fused ? 0 : b.slices_f), (int32_t)b.slices_c,
        (int32_t)b.feat_pts.chunks, (int32_t)b.logit_pts.chunks, (int32_t)b.feat_vtx.chunks,
        (int32_t)b.logit_vtx.chunks, (int32_t)b.grid.chunks, (int32_t)b.dense_slices,
        b.binned ? 1 : 0, (int32_t)b.subs_f, (int32_t)b.subs_c, (int32_t)b.bin_chunks,
        (int32_t)(N > 0 ? (N + per - 1) / per : 1)};
    for (int i = 0; i < CNGP_PLAN_INFO_COUNT; ++i) info[i] = v[i];
    return CNGP_OK;
}

int cngp_bwd_plan_layout(const cngp_config *cfg, int64_t N, uint64_t *regions) {
    if (!regions) return CNGP_ERR_NULL;
    if (int rc = validate(cfg)) return rc;
    if (N < 0) return CNGP_ERR_INVALID;
    const cngp_config pairs = as_pairs(cfg);
    cfg = &pairs;
    const int64_t per = bwd_pass_points(cfg, N);
    const int64_t n = per < N ? per : N;
    const BwdPlan b = make_bwd_plan(cfg, n);
    if (!b.sliced || n == 0) return 0;
    // what the kernels index, region by region (not the differences of the offsets: those would prove nothing)
    const uint64_t io = cfg->io_dtype == CNGP_F16 ? 2 : 4;
    const uint64_t Ld = (uint64_t)b.dense.count, Lh = (uint64_t)cfg->L - Ld, cap = (uint64_t)n << cfg->d;
    int k = 0;
    auto add = [&](size_t off, uint64_t bytes) { regions[2 * k] = off; regions[2 * k + 1] = bytes; ++k; };
    add(b.sigma_off, (uint64_t)cfg->L * cfg->N_c * cfg->N_p * 4);
    add(b.dyT_off, (uint64_t)n * cfg->L * cfg->F * io);
    add(b.G_off, (uint64_t)b.dense_verts * 2 * 4);
    if (b.binned) {
        const uint64_t sf = b.fused ? 0 : b.slices_f, sc = cfg->N_p > 1 ? b.slices_c : 0;
        add(b.cntF_off, Lh * b.bin_chunks * sf * 4);
        add(b.cntC_off, Lh * b.bin_chunks * sc * 4);
        add(b.baseF_off, sf ? Lh * (sf + 1) * 4 : 0);
        add(b.baseC_off, sc ? Lh * (sc + 1) * 4 : 0);
        add(b.recF_off, sf ? Lh * cap * kRecordBytes : 0);
        add(b.recC_off, sc ? Lh * cap * kRecordBytes : 0);
        add(b.cntG_off, Ld * b.bin_chunks * kGridBins * 4);
        add(b.baseG_off, Ld ? Ld * (kGridBins + 1) * 4 : 0);
        add(b.recG_off, Ld * cap * kRecordBytes);
    }
    return k;
}

int cngp_encode_fwd(const cngp_config *cfg, const float *x, int64_t N, const void *D_f, const void *D_c,
                    void *y, void *workspace, size_t workspace_bytes, void *stream) {
    if (int rc = validate(cfg)) return rc;
    if (N < 0) return CNGP_ERR_INVALID;
    if (N == 0) return CNGP_OK;
    if (!x || !D_f || !y || (!D_c && !index_codebook_is_empty(cfg))) return CNGP_ERR_NULL;
    if (cfg->index_format == CNGP_IDX_BITS && ((uintptr_t)D_c & 3u)) return CNGP_ERR_INVALID;
    if (cfg->F != 2) return fwd_planes(cfg, cfg->L, x, N, D_f, D_c, y, workspace, workspace_bytes, stream);
    const Params p = make_params(cfg);
    hipStream_t s = (hipStream_t)stream;
    CNGP_DISPATCH_TYPES(launch_fwd, cfg, p, x, N, D_f, D_c, y, s, nullptr, workspace, workspace_bytes);
}

int cngp_encode_fwd_partial(const cngp_config *cfg, int32_t levels_loaded, const float *x, int64_t N, const void *D_f,
                            const void *D_c, void *y, void *workspace, size_t workspace_bytes, void *stream) {
    if (int rc = validate(cfg)) return rc;
    if (N < 0 || levels_loaded < 0 || levels_loaded > cfg->L) return CNGP_ERR_INVALID;
    if (N == 0) return CNGP_OK;
    if (!x || !y) return CNGP_ERR_NULL;
    if (levels_loaded > 0 && (!D_f || (!D_c && !index_codebook_is_empty(cfg)))) return CNGP_ERR_NULL;
    if (cfg->index_format == CNGP_IDX_BITS && ((uintptr_t)D_c & 3u)) return CNGP_ERR_INVALID;
    if (cfg->F != 2) return fwd_planes(cfg, levels_loaded, x, N, D_f, D_c, y, workspace, workspace_bytes, stream);
    Params p = make_params(cfg);
    p.L_loaded = levels_loaded;
    hipStream_t s = (hipStream_t)stream;
    CNGP_DISPATCH_TYPES(launch_fwd, cfg, p, x, N, D_f, D_c, y, s, nullptr, workspace, workspace_bytes);
}

int cngp_encode_fwd_permuted(const cngp_config *cfg, const float *x_sorted, const int32_t *perm, int64_t N, const void *D_f,
                             const void *D_c, void *y, void *workspace, size_t workspace_bytes, void *stream) {
    if (int rc = validate(cfg)) return rc;
    if (N < 0 || N > 0x7fffffffLL) return CNGP_ERR_INVALID;
    if (cfg->F != 2) return CNGP_ERR_UNSUPPORTED;
    if (N == 0) return CNGP_OK;
    if (!x_sorted || !perm || !D_f || !y || (!D_c && !index_codebook_is_empty(cfg))) return CNGP_ERR_NULL;
    if (cfg->index_format == CNGP_IDX_BITS && ((uintptr_t)D_c & 3u)) return CNGP_ERR_INVALID;
    const Params p = make_params(cfg);
    hipStream_t s = (hipStream_t)stream;
    CNGP_DISPATCH_TYPES(launch_fwd, cfg, p, x_sorted, N, D_f, D_c, y, s, perm, workspace, workspace_bytes);
}

int cngp_encode_bwd(const cngp_config *cfg, const float *x, int64_t N, const void *D_f,
                    const float *Dhat_c, const void *dy, float *grad_D_f, float *grad_Dhat_c,
                    void *workspace, size_t workspace_bytes, void *stream) {
    if (int rc = validate(cfg)) return rc;
    if (N < 0) return CNGP_ERR_INVALID;
    if (!grad_D_f || !grad_Dhat_c) return CNGP_ERR_NULL;
    if (N > 0 && (!x || !D_f || !Dhat_c || !dy)) return CNGP_ERR_NULL;
    if (cfg->F != 2) return bwd_planes(cfg, x, N, D_f, Dhat_c, dy, grad_D_f, grad_Dhat_c, workspace, workspace_bytes, stream);
    hipStream_t s = (hipStream_t)stream;
    const int64_t per = bwd_pass_points(cfg, N);
    if (per < N) {      // several passes over runs of points; the first one clears if asked, the rest accumulate
        if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < cngp_workspace_bytes(cfg, N))
            return CNGP_ERR_WORKSPACE;
        cngp_config   pass = *cfg;
        const size_t  io = cfg->io_dtype == CNGP_F16 ? 2 : 4;
        for (int64_t first = 0; first < N; first += per) {
            const int64_t n = N - first < per ? N - first : per;
            const int rc = cngp_encode_bwd(&pass, x + first * cfg->d, n, D_f, Dhat_c,
                                           (const char *)dy + (size_t)first * cfg->L * cfg->F * io, grad_D_f, grad_Dhat_c,
                                           workspace, workspace_bytes, stream);
            if (rc) return rc;
            pass.flags &= ~(uint32_t)CNGP_ZERO_GRADS;
        }
        return CNGP_OK;
    }
    const BwdPlan b = make_bwd_plan(cfg, N);
    if (N > 0 && b.sliced) {
        if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < b.ws_bytes) return CNGP_ERR_WORKSPACE;
    }
    // A sliced launch with a single chunk writes every gradient entry of its levels itself; the other
    // level ranges (dense levels 0 .. Ld-1, hashed levels Ld .. L-1) are cleared here.
    ZeroList z;
    if (cfg->flags & CNGP_ZERO_GRADS) {
        const int64_t per_f = (int64_t)cfg->N_f * cfg->F, per_c = (int64_t)cfg->N_c * cfg->N_p;
        const bool    sl = N > 0 && b.sliced;
        const int     Ld = sl ? b.dense.count : 0, Lh = cfg->L - Ld;
        if (!(sl && b.feat_vtx.chunks == 1) && Ld > 0) z.add(grad_D_f, per_f * Ld);
        const uint32_t wg_f = b.binned ? b.subs_f : b.feat_pts.chunks, wg_c = b.binned ? b.subs_c : b.logit_pts.chunks;
        if (!(sl && wg_f == 1) && Lh > 0) z.add(grad_D_f + per_f * Ld, per_f * Lh);
        const bool logit = sl && cfg->N_p > 1;
        if (!(logit && b.logit_vtx.chunks == 1) && Ld > 0) z.add(grad_Dhat_c, per_c * Ld);
        if (!(logit && wg_c == 1) && Lh > 0) z.add(grad_Dhat_c + per_c * Ld, per_c * Lh);
    }
    if (N == 0) return z.launch(s);
    const Params p = make_params(cfg);
    // the LDS variants clear these ranges in their preparation launch, the direct one with a launch of its own
    CNGP_DISPATCH_TYPES(dispatch_bwd_np, cfg, p, b, x, N, D_f, Dhat_c, dy, grad_D_f, grad_Dhat_c, workspace, z, s);
}

size_t cngp_static_scratch_bytes(void) { return kStaticScratchBytes; }

int cngp_encode_bwd_static(const cngp_config *cfg, const float *x, int64_t N, const void *D_f,
                           const float *Dhat_c, const void *dy, float *grad_D_f, float *grad_Dhat_c, void *stream) {
    if (int rc = validate(cfg)) return rc;
    if (N < 0) return CNGP_ERR_INVALID;
    if (!grad_D_f || !grad_Dhat_c) return CNGP_ERR_NULL;
    if (N > 0 && (!x || !D_f || !Dhat_c || !dy)) return CNGP_ERR_NULL;
    // The variant is the one cngp_encode_bwd would pick for (cfg, N).  Only the bins of the binned variant grow
    // with N: they are bounded until everything fits the static array (the batch is then taken in several passes
    // inside the one call, like any batch beyond cfg->bin_bytes_max) -- as long as a pass is still binned: this
    // entry point never falls back to a slower variant behind the caller's back.
    cngp_config c = *cfg;
    size_t need = cngp_workspace_bytes(&c, N);
    if (need > kStaticScratchBytes && N > 0) {
        const int64_t per0 = bwd_pass_points(cfg, N);
        const bool    binned = make_bwd_plan_uncached(cfg, per0 < N ? per0 : N).binned;
        for (uint64_t bins = kStaticScratchBytes / 2; binned && bins >= ((uint64_t)1 << 20); bins /= 2) {
            if (cfg->bin_bytes_max && cfg->bin_bytes_max < bins) continue;      // never beyond the caller's own bound
            cngp_config t = *cfg;
            t.bin_bytes_max = bins;
            const int64_t per = bwd_pass_points(&t, N);
            if (!make_bwd_plan_uncached(&t, per < N ? per : N).binned) break;   // passes too small to bin
            const size_t  n = cngp_workspace_bytes(&t, N);
            if (n <= kStaticScratchBytes) { c = t; need = n; break; }
        }
    }
    if (need > kStaticScratchBytes) {
        g_hip_error = "cngp_encode_bwd_static: this configuration and N need " + std::to_string(need) +
                      " bytes of scratch, the static array holds " + std::to_string(kStaticScratchBytes) +
                      "; use cngp_encode_bwd with a workspace";
        return CNGP_ERR_WORKSPACE;
    }
    void *ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    return cngp_encode_bwd(&c, x, N, D_f, Dhat_c, dy, grad_D_f, grad_Dhat_c, ws, kStaticScratchBytes, stream);
}

int cngp_encode_bwd_input(const cngp_config *cfg, const float *x, int64_t N, const void *D_f, const void *D_c,
                          const void *dy, float *grad_x, void *stream) {
    if (int rc = validate(cfg)) return rc;
    if (cfg->F != 2) return CNGP_ERR_UNSUPPORTED;           // (no workspace argument to hold the pair planes)
    if (N < 0) return CNGP_ERR_INVALID;
    if (N == 0) return CNGP_OK;
    if (!x || !D_f || !dy || !grad_x || (!D_c && !index_codebook_is_empty(cfg))) return CNGP_ERR_NULL;
    if (cfg->index_format == CNGP_IDX_BITS && ((uintptr_t)D_c & 3u)) return CNGP_ERR_INVALID;
    const Params p = make_params(cfg);
    hipStream_t s = (hipStream_t)stream;
    CNGP_DISPATCH_TYPES(launch_bwd_input, cfg, p, x, N, D_f, D_c, dy, grad_x, s);
}

int cngp_storage_bytes(const cngp_config *cfg, size_t *D_f_bytes, size_t *D_c_level_bytes, size_t *D_c_bytes) {
    if (int rc = validate(cfg)) return rc;
    const size_t level = index_level_bytes(cfg);
    if (D_f_bytes) *D_f_bytes = (size_t)cfg->L * cfg->N_f * cfg->F * (cfg->feat_dtype == CNGP_F16 ? 2 : 4);
    if (D_c_level_bytes) *D_c_level_bytes = level;
    if (D_c_bytes) *D_c_bytes = level * cfg->L;
    return CNGP_OK;
}

int cngp_bake_probes(const cngp_config *cfg, const float *Dhat_c, void *D_c, void *stream) {
    if (int rc = validate(cfg)) return rc;
    if (index_codebook_is_empty(cfg)) return Dhat_c ? CNGP_OK : CNGP_ERR_NULL;       // nothing to write
    if (!Dhat_c || !D_c) return CNGP_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (cfg->index_format == CNGP_IDX_BITS) {
        if ((uintptr_t)D_c & 3u) return CNGP_ERR_INVALID;
        const uint32_t wpl = (uint32_t)(index_level_bytes(cfg) / 4);
        const int64_t  words = (int64_t)cfg->L * wpl;
        const int64_t  blocks = (words + kBlock - 1) / kBlock;
        if (int rc = check_blocks(blocks)) return rc;
        LaunchTimer t(s, K_BAKE);
#define CNGP_BAKE_BITS(NP) bake_probes_bits_kernel<NP><<<(unsigned)blocks, kBlock, 0, s>>>(Dhat_c, (uint32_t *)D_c, cfg->N_c, wpl, words)
        switch (cfg->N_p) {
        case 2:  CNGP_BAKE_BITS(2); break;
        case 4:  CNGP_BAKE_BITS(4); break;
        case 8:  CNGP_BAKE_BITS(8); break;
        default: CNGP_BAKE_BITS(16); break;
        }
#undef CNGP_BAKE_BITS
        return launch_status("bake_probes_bits_kernel");
    }
    const bool packed = cfg->index_format == CNGP_IDX_PACKED4;
    const int64_t rows = (int64_t)cfg->L * cfg->N_c;
    const int64_t bytes_out = packed ? rows / 2 : rows;
    const int64_t blocks = (bytes_out + kBlock - 1) / kBlock;
    if (int rc = check_blocks(blocks)) return rc;
    LaunchTimer t(s, K_BAKE);
#define CNGP_BAKE(NP)                                                                                  \
    if (packed) bake_probes_kernel<NP, true><<<(unsigned)blocks, kBlock, 0, s>>>(Dhat_c, (uint8_t *)D_c, bytes_out); \
    else        bake_probes_kernel<NP, false><<<(unsigned)blocks, kBlock, 0, s>>>(Dhat_c, (uint8_t *)D_c, bytes_out)
    switch (cfg->N_p) {
    case 1:  CNGP_BAKE(1); break;
    case 2:  CNGP_BAKE(2); break;
    case 4:  CNGP_BAKE(4); break;
    case 8:  CNGP_BAKE(8); break;
    default: CNGP_BAKE(16); break;
    }
#undef CNGP_BAKE
    return launch_status("bake_probes_kernel");
}

int cngp_adam_step_bake(const cngp_config *cfg, const cngp_adam *opt_f, const cngp_adam *opt_c,
                        float *D_f_master, void *D_f, float *m_f, float *v_f, float *grad_D_f,
                        float *Dhat_c, float *m_c, float *v_c, float *grad_Dhat_c, void *D_c, void *stream) {
    if (int rc = validate(cfg)) return rc;
    if (cfg->index_format == CNGP_IDX_BITS) return CNGP_ERR_UNSUPPORTED;   // training keeps whole-byte or 4-bit entries
    AdamTable f, c;
    std::memset(&f, 0, sizeof(f));
    std::memset(&c, 0, sizeof(c));
    __half *D_f_half = nullptr;
    if (opt_f) {
        if (!D_f_master || !m_f || !v_f || !grad_D_f) return CNGP_ERR_NULL;
        if (int rc = adam_coefficients(opt_f, &f.a)) return rc;
        if (cfg->feat_dtype == CNGP_F16) {
            if (!D_f) return CNGP_ERR_NULL;
            if (!aligned(D_f, 8)) return CNGP_ERR_INVALID;
            D_f_half = (__half *)D_f;
        } else if (D_f && D_f != (void *)D_f_master) {
            return CNGP_ERR_INVALID;
        }
        if (!aligned(D_f_master, 16) || !aligned(m_f, 16) || !aligned(v_f, 16) || !aligned(grad_D_f, 16)) return CNGP_ERR_INVALID;
        f.theta = D_f_master; f.m = m_f; f.v = v_f; f.grad = grad_D_f;
        f.n = (int64_t)cfg->L * cfg->N_f * cfg->F;
    }
    if (opt_c) {
        if (!Dhat_c || !m_c || !v_c || !grad_Dhat_c || !D_c) return CNGP_ERR_NULL;
        if (int rc = adam_coefficients(opt_c, &c.a)) return rc;
        if (!aligned(Dhat_c, 16) || !aligned(m_c, 16) || !aligned(v_c, 16) || !aligned(grad_Dhat_c, 16)) return CNGP_ERR_INVALID;
        c.theta = Dhat_c; c.m = m_c; c.v = v_c; c.grad = grad_Dhat_c;
        c.n = (int64_t)cfg->L * cfg->N_c * cfg->N_p;
    }
    const int64_t per_block = (int64_t)kOptBlock * 4;
    const int64_t blocks_f = (f.n + per_block - 1) / per_block;
    const int64_t blocks_c = (c.n + per_block - 1) / per_block;
    if (blocks_f + blocks_c == 0) return CNGP_OK;
    if (int rc = check_blocks(blocks_f + blocks_c)) return rc;
    const bool packed = cfg->index_format == CNGP_IDX_PACKED4;
    const int  clear = (cfg->flags & CNGP_ZERO_GRADS) ? 1 : 0;
    hipStream_t s = (hipStream_t)stream;
    LaunchTimer t(s, K_ADAM);
#define CNGP_ADAM(NP)                                                                                   \
    if (packed) adam_step_bake_kernel<NP, true><<<(unsigned)(blocks_f + blocks_c), kOptBlock, 0, s>>>(  \
                    f, c, D_f_half, (uint8_t *)D_c, (uint32_t)blocks_f, clear);                         \
    else        adam_step_bake_kernel<NP, false><<<(unsigned)(blocks_f + blocks_c), kOptBlock, 0, s>>>( \
                    f, c, D_f_half, (uint8_t *)D_c, (uint32_t)blocks_f, clear)
    switch (cfg->N_p) {
    case 1:  CNGP_ADAM(1); break;
    case 2:  CNGP_ADAM(2); break;
    case 4:  CNGP_ADAM(4); break;
    case 8:  CNGP_ADAM(8); break;
    default: CNGP_ADAM(16); break;
    }
#undef CNGP_ADAM
    return launch_status("adam_step_bake_kernel");
}

int cngp_adam_step(const cngp_adam *opt, int64_t n, float *master, void *half_copy, float *m, float *v,
                   float *grad, int clear_grad, void *stream) {
    if (!opt || !master || !m || !v || !grad) return CNGP_ERR_NULL;
    if (n < 0) return CNGP_ERR_INVALID;
    AdamTable f, c;
    std::memset(&f, 0, sizeof(f));
    std::memset(&c, 0, sizeof(c));
    if (int rc = adam_coefficients(opt, &f.a)) return rc;
    if (!aligned(master, 16) || !aligned(m, 16) || !aligned(v, 16) || !aligned(grad, 16) || !aligned(half_copy, 8)) return CNGP_ERR_INVALID;
    if (n == 0) return CNGP_OK;
    f.theta = master; f.m = m; f.v = v; f.grad = grad; f.n = n;
    const int64_t per_block = (int64_t)kOptBlock * 4;
    const int64_t blocks = (n + per_block - 1) / per_block;
    if (int rc = check_blocks(blocks)) return rc;
    hipStream_t s = (hipStream_t)stream;
    LaunchTimer t(s, K_ADAM);
    adam_step_bake_kernel<1, false><<<(unsigned)blocks, kOptBlock, 0, s>>>(f, c, (__half *)half_copy, nullptr,
                                                                           (uint32_t)blocks, clear_grad ? 1 : 0);
    return launch_status("adam_step_bake_kernel");
}

namespace {
int mlp_dims(const cngp_mlp_config *cfg, MlpDims *d) {
    if (!cfg) return CNGP_ERR_NULL;
    if (cfg->n_in < 1 || cfg->n_in > kMlpMaxIn || cfg->n_out < 1 || cfg->n_out > kMlpMaxOut) return CNGP_ERR_INVALID;
    if (cfg->io_dtype != CNGP_F32 && cfg->io_dtype != CNGP_F16) return CNGP_ERR_INVALID;
    if (cfg->flags & ~(uint32_t)CNGP_ZERO_GRADS) return CNGP_ERR_INVALID;
    d->n_in = cfg->n_in; d->n_out = cfg->n_out;
    d->ks1 = (cfg->n_in + 7) / 8; d->ks3 = (cfg->n_out + 7) / 8;
    d->vec_in = d->vec_out = 0;            // set by the caller once the pointers are known
    return CNGP_OK;
}
// A persistent grid: every wavefront walks over tiles of 32 points.  At most `per_cu` workgroups per CU
// (what fits at once), and no more than gives each wavefront `min_tiles` tiles, so that the staging of the
// weights, which every workgroup repeats, stays a small part of its work.
unsigned mlp_blocks(int64_t tiles, int per_cu, int min_tiles) {
    const int64_t per_block = (int64_t)(kMlpBlock / 64) * min_tiles;
    const int64_t want = (tiles + per_block - 1) / per_block;
    const int64_t cap = 256 * (int64_t)per_cu;
    return (unsigned)(want < cap ? want : cap);
}
}  // namespace

size_t cngp_mlp_weight_count(const cngp_mlp_config *cfg) {
    MlpDims d;
    if (mlp_dims(cfg, &d)) return 0;
    return (size_t)kMlpHidden * d.n_in + (size_t)kMlpHidden * kMlpHidden + (size_t)kMlpHidden * d.n_out;
}

int cngp_mlp_fwd(const cngp_mlp_config *cfg, const void *y, int64_t N, const void *W, float *out, void *stream) {
    MlpDims d;
    if (int rc = mlp_dims(cfg, &d)) return rc;
    if (N < 0) return CNGP_ERR_INVALID;
    if (N == 0) return CNGP_OK;
    if (!y || !W || !out) return CNGP_ERR_NULL;
    const int64_t tiles = (N + 31) / 32;
    hipStream_t s = (hipStream_t)stream;
    d.vec_in = (cfg->n_in % 4 == 0 && aligned(y, 16)) ? 1 : 0;
    LaunchTimer t(s, K_MLP_FWD);
    if (cfg->io_dtype == CNGP_F16)
        mlp_fwd_kernel<__half><<<mlp_blocks(tiles, 3, 4), kMlpBlock, kMlpFwdLds, s>>>(d, (const __half *)y, N, (const __half *)W, out, tiles);
    else
        mlp_fwd_kernel<float><<<mlp_blocks(tiles, 3, 4), kMlpBlock, kMlpFwdLds, s>>>(d, (const float *)y, N, (const __half *)W, out, tiles);
    return launch_status("mlp_fwd_kernel");
}

int cngp_encode_mlp_fwd(const cngp_config *cfg, const cngp_mlp_config *mlp, const float *x, int64_t N,
                        const void *D_f, const void *D_c, const void *W, float *out,
                        void *workspace, size_t workspace_bytes, void *stream) {
    if (int rc = validate(cfg)) return rc;
    MlpDims d;
    if (int rc = mlp_dims(mlp, &d)) return rc;
    if (cfg->F != 2) return CNGP_ERR_UNSUPPORTED;
    if (d.n_in != cfg->L * cfg->F) return CNGP_ERR_INVALID;
    if (N < 0) return CNGP_ERR_INVALID;
    if (N == 0) return CNGP_OK;
    if (!x || !D_f || !W || !out || (!D_c && !index_codebook_is_empty(cfg))) return CNGP_ERR_NULL;
    if (cfg->index_format == CNGP_IDX_BITS && ((uintptr_t)D_c & 3u)) return CNGP_ERR_INVALID;
    const Params p = make_params(cfg);
    hipStream_t s = (hipStream_t)stream;
    // With room for the level-major fp16 encodings: the level-resident forward without its rows kernel, and the
    // decoder reading the planes as they are.
    {
        cngp_config c16 = *cfg;
        c16.io_dtype = CNGP_F16;
        const FwdLevelPlan f = fwd_level_plan(&c16, cfg->L, N);
        if (f.use && workspace && workspace_bytes >= f.yT_bytes && ((uintptr_t)workspace & 255u) == 0 && ((uintptr_t)D_f & 15u) == 0) {
            int rc;
            const bool f16 = cfg->feat_dtype == CNGP_F16;
            if (cfg->d == 2) rc = f16 ? launch_fwd_level<2, __half, __half>(&c16, f, p, x, N, D_f, D_c, nullptr, workspace, s, nullptr, false)
                                      : launch_fwd_level<2, float, __half>(&c16, f, p, x, N, D_f, D_c, nullptr, workspace, s, nullptr, false);
            else if (cfg->d == 3) rc = f16 ? launch_fwd_level<3, __half, __half>(&c16, f, p, x, N, D_f, D_c, nullptr, workspace, s, nullptr, false)
                                           : launch_fwd_level<3, float, __half>(&c16, f, p, x, N, D_f, D_c, nullptr, workspace, s, nullptr, false);
            else rc = f16 ? launch_fwd_level<4, __half, __half>(&c16, f, p, x, N, D_f, D_c, nullptr, workspace, s, nullptr, false)
                          : launch_fwd_level<4, float, __half>(&c16, f, p, x, N, D_f, D_c, nullptr, workspace, s, nullptr, false);
            if (rc) return rc;
            const int64_t tiles = (N + 31) / 32;
            LaunchTimer t(s, K_MLP_FWD);
            mlp_fwd_kernel<__half, true><<<mlp_blocks(tiles, 3, 4), kMlpBlock, kMlpFwdLds, s>>>(d, (const __half *)workspace, N, (const __half *)W, out, tiles);
            return launch_status("mlp_fwd_kernel");
        }
    }
    CNGP_DISPATCH_TYPES(launch_fused_fwd, cfg, p, d, x, N, D_f, D_c, W, out, s);
}

int cngp_mlp_bwd(const cngp_mlp_config *cfg, const void *y, int64_t N, const void *W, const float *dout,
                 void *dy, float *grad_W, void *stream) {
    MlpDims d;
    if (int rc = mlp_dims(cfg, &d)) return rc;
    if (N < 0) return CNGP_ERR_INVALID;
    if (!grad_W) return CNGP_ERR_NULL;
    if (N > 0 && (!y || !W || !dout || !dy)) return CNGP_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    if (cfg->flags & CNGP_ZERO_GRADS) {
        ZeroList z;
        z.add(grad_W, (int64_t)cngp_mlp_weight_count(cfg));
        if (int rc = z.launch(s)) return rc;
    }
    if (N == 0) return CNGP_OK;
    const int64_t tiles = (N + 31) / 32;
    d.vec_in = (cfg->n_in % 4 == 0 && aligned(y, 16) && aligned(dy, 16)) ? 1 : 0;
    d.vec_out = (cfg->n_out % 4 == 0 && aligned(dout, 16)) ? 1 : 0;
    if (cfg->io_dtype == CNGP_F16) {
        auto kernel = mlp_bwd_kernel<__half>;
        if (int rc = allow_big_lds(kernel, kMlpBwdLds)) return rc;
        LaunchTimer t(s, K_MLP_BWD);
        kernel<<<mlp_blocks(tiles, 1, 4), kMlpBlock, kMlpBwdLds, s>>>(d, (const __half *)y, N, (const __half *)W, dout, (__half *)dy, grad_W, tiles);
    } else {
        auto kernel = mlp_bwd_kernel<float>;
        if (int rc = allow_big_lds(kernel, kMlpBwdLds)) return rc;
        LaunchTimer t(s, K_MLP_BWD);
        kernel<<<mlp_blocks(tiles, 1, 4), kMlpBlock, kMlpBwdLds, s>>>(d, (const float *)y, N, (const __half *)W, dout, (float *)dy, grad_W, tiles);
    }
    return launch_status("mlp_bwd_kernel");
}

int cngp_debug_indices(const cngp_config *cfg, const float *x, int64_t N, const void *D_c, uint32_t *base,
                       uint32_t *h2, uint8_t *probe, uint32_t *feat_idx, void *stream) {
    if (int rc = validate(cfg)) return rc;
    if (N < 0) return CNGP_ERR_INVALID;
    if (N == 0) return CNGP_OK;
    if (!x) return CNGP_ERR_NULL;
    if (!D_c && (probe || feat_idx) && !index_codebook_is_empty(cfg)) return CNGP_ERR_NULL;
    const Params p = make_params(cfg);
    const int64_t pairs = N * cfg->L;
    const int64_t blocks = (pairs + kBlock - 1) / kBlock;
    if (int rc = check_blocks(blocks)) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (cfg->index_format == CNGP_IDX_BITS && ((uintptr_t)D_c & 3u)) return CNGP_ERR_INVALID;
    const uint32_t c_stride = (uint32_t)index_level_bytes(cfg);
    LaunchTimer t(s, K_DEBUG);
#define CNGP_DBG(D, FMT) debug_indices_kernel<D, FMT><<<(unsigned)blocks, kBlock, 0, s>>>(p, x, (const uint8_t *)D_c, base, h2, probe, feat_idx, pairs, c_stride)
#define CNGP_DBG_FMT(D)                                                     \
    if (cfg->index_format == CNGP_IDX_PACKED4) CNGP_DBG(D, kFmtPacked4);   \
    else if (cfg->index_format == CNGP_IDX_BITS) CNGP_DBG(D, kFmtBits);    \
    else CNGP_DBG(D, kFmtU8)
    if (cfg->d == 2) { CNGP_DBG_FMT(2); } else if (cfg->d == 3) { CNGP_DBG_FMT(3); } else { CNGP_DBG_FMT(4); }
#undef CNGP_DBG_FMT
#undef CNGP_DBG
    return launch_status("debug_indices_kernel");
}

int cngp_measure_rates(cngp_rates *out, void *scratch, size_t scratch_bytes, void *stream) {
    if (!out || !scratch) return CNGP_ERR_NULL;
    const size_t need = (size_t)64 << 20;
    if (scratch_bytes < need || ((uintptr_t)scratch & 255u)) return CNGP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t  t0, t1;
    CNGP_HIP(hipEventCreate(&t0));
    CNGP_HIP(hipEventCreate(&t1));
    int rc = CNGP_OK;
    auto timed = [&](auto launch, int reps, double &ms_out) {       // one untimed run, then `reps` timed ones
        launch();
        if (hipEventRecord(t0, s) != hipSuccess) rc = CNGP_ERR_HIP;
        for (int i = 0; i < reps; ++i) launch();
        if (hipEventRecord(t1, s) != hipSuccess || hipEventSynchronize(t1) != hipSuccess) rc = CNGP_ERR_HIP;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, t0, t1) != hipSuccess) rc = CNGP_ERR_HIP;
        ms_out = (double)ms / reps;
    };
    float *tab = (float *)scratch;
    float *sink = tab + (need / 4 - 64);                            // last 256 bytes: never inside a table
    double ms = 0.0;
    const size_t half = need / 2 - 256;
    timed([&] { rate_copy_kernel<<<8192, kBlock, 0, s>>>((const float4 *)scratch, (float4 *)((char *)scratch + need / 2), half / 16); }, 3, ms);
    out->copy_GBps = 2.0 * (double)(half / 16 * 16) / ms / 1e6;
    const int      blocks = 256 * 32, iters = 16;
    const double   lane_ops = (double)blocks * kBlock * iters * 8;
    const uint32_t table_floats = (4u << 20) / 4;                   // 4 MB table: L2 resident
    timed([&] { rate_rows_kernel<1, false><<<blocks, kBlock, 0, s>>>(tab, table_floats - 1, iters, sink); }, 3, ms);
    out->gather4_Gps = lane_ops / ms / 1e6;
    timed([&] { rate_rows_kernel<16, false><<<blocks, kBlock, 0, s>>>(tab, table_floats / 16 - 1, iters, sink); }, 3, ms);
    out->row_gather_Gps = lane_ops / 16 / ms / 1e6;
    timed([&] { rate_rows_kernel<16, true><<<blocks, kBlock, 0, s>>>(tab, table_floats / 16 - 1, iters, sink); }, 3, ms);
    out->global_atomic_Gseg = lane_ops / 16 / ms / 1e6;
    const uint32_t far_floats = (32u << 20) / 4;                    // 32 MB table: beyond every L2, in the memory-side cache
    timed([&] { rate_rows_kernel<16, false><<<blocks, kBlock, 0, s>>>(tab, far_floats / 16 - 1, iters, sink); }, 3, ms);
    out->row_gather_far_Gps = lane_ops / 16 / ms / 1e6;
    timed([&] { rate_rows_kernel<1, false><<<blocks, kBlock, 0, s>>>(tab, far_floats - 1, iters, sink); }, 3, ms);
    out->gather4_far_Gps = lane_ops / ms / 1e6;
    auto lds_rate = [&](auto kernel, size_t lds, double &gps) {
        if (int r2 = allow_big_lds(kernel, lds)) rc = r2;
        const int lblocks = 1024, liters = 64;
        timed([&] { kernel<<<lblocks, 1024, lds, s>>>(liters, sink); }, 3, ms);
        gps = (double)lblocks * 1024 * liters * 8 / ms / 1e6;
    };
    lds_rate(rate_lds_atomic_kernel<double>, 16384 * sizeof(double), out->lds_atomic_f64_Gps);
    lds_rate(rate_lds_atomic_kernel<float>, 16384 * sizeof(float), out->lds_atomic_f32_Gps);
    lds_rate(rate_lds_atomic_kernel<uint32_t>, 16384 * sizeof(uint32_t), out->lds_atomic_u32_Gps);
    lds_rate(rate_lds_gather_kernel, 32768 * sizeof(uint32_t), out->lds_gather4_Gps);
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    if (rc == CNGP_OK) rc = launch_status("cngp_measure_rates");
    return rc;
}

int cngp_profile_enable(int on) {
    const int was = g_profile ? 1 : 0;
    g_profile = on != 0;
    return was;
}

const char *cngp_profile_kernel_name(int i) { return (i >= 0 && i < K_COUNT) ? kKernelNames[i] : ""; }

int cngp_profile_read(double *ms_sum, int64_t *launches, int max_kernels) {
    for (auto &t : g_timed) {
        float ms = 0.0f;
        if (hipEventSynchronize(t.t1) == hipSuccess && hipEventElapsedTime(&ms, t.t0, t.t1) == hipSuccess &&
            t.id < max_kernels) {
            if (ms_sum) ms_sum[t.id] += (double)ms;
            if (launches) launches[t.id] += 1;
        }
        (void)hipEventDestroy(t.t0);
        (void)hipEventDestroy(t.t1);
    }
    g_timed.clear();
    return K_COUNT;
}

}  // extern "C"

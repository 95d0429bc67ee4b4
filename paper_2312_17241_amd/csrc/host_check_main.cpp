// Exerciser of the library's HOST code under AddressSanitizer and UndefinedBehaviorSanitizer: argument
// validation, level table, storage sizes, the backward plan (slices, chunks, bins, passes) and its workspace
// layout, for seeded random configurations.  It is linked with cngp_api.hip and cngp_sort.hip compiled with the
// sanitizers on the host side only (`python paper_2312_17241_amd/build.py --host-sanitizers`) and launches
// nothing: every call below returns before a kernel would be enqueued, so it runs without a GPU.
// Exit code 0 = clean.
#include "../../include/cngp.h"
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <initializer_list>

static uint64_t g_state = 0x243F6A8885A308D3ull;
static uint64_t next_u64() {                       // splitmix64
    uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static uint32_t below(uint32_t n) { return (uint32_t)(next_u64() % n); }

int main() {
    int bad = 0;
    const int64_t sizes[] = {0, 1, 63, 4097, 70001, 1 << 18, (1 << 20) + 5, 1 << 22, (int64_t)1 << 26};
    const uint32_t flag_sets[] = {0, CNGP_BWD_DIRECT, CNGP_BWD_SLICED, CNGP_BWD_BINNED, CNGP_BWD_BINNED | CNGP_BWD_NO_PREREDUCE,
                                  CNGP_BWD_SLICED | CNGP_BWD_NO_PREREDUCE};
    for (int it = 0; it < 300; ++it) {
        cngp_config c;
        std::memset(&c, 0, sizeof(c));
        c.d = 2 + (int)below(2);
        c.L = 1 + (int)below(32);
        c.F = 2;
        c.N_p = 1u << below(5);
        c.N_f = 1u << (below(29) + 2);
        c.N_c = 1u << below(29);
        c.N_min = 1 + below(64);
        c.N_max = c.N_min << below(12);
        c.feat_dtype = (int)below(2);
        c.io_dtype = (int)below(2);
        c.index_format = (int)below(3);
        c.flags = flag_sets[below(6)] | (below(2) ? CNGP_ZERO_GRADS : 0u);
        c.top_k = below(3) ? 0 : below(c.N_p + 1);
        const uint64_t bounds[] = {0, 0, 1ull << 20, 1ull << 27, 1ull << 33};
        c.bin_bytes_max = bounds[below(5)];
        if (it % 7 == 0) c.N_f = below(5000);                               // often invalid: must be rejected, not crash
        if (it % 11 == 0) c.L = (int)below(40);
        const int64_t N = sizes[below(9)];

        uint32_t res[64];
        int32_t  info[CNGP_PLAN_INFO_COUNT];
        uint64_t regions[2 * CNGP_PLAN_REGIONS];
        size_t   a = 0, b = 0, e = 0;
        const int rl = cngp_level_resolutions(&c, res);
        const int rs = cngp_storage_bytes(&c, &a, &b, &e);
        const size_t ws = cngp_workspace_bytes(&c, N);
        const int rp = cngp_bwd_plan_info(&c, N, info);
        const int rr = cngp_bwd_plan_layout(&c, N, regions);
        int32_t finfo[CNGP_FWD_PLAN_INFO_COUNT] = {0, 0, 0, 0};
        const int    rf = cngp_fwd_plan_info(&c, N, finfo);
        const size_t fws = cngp_fwd_workspace_bytes(&c, N);
        if (rf == CNGP_OK) {            // the level-resident forward: resident entries and LDS within their limits, room inside the workspace
            if (finfo[0] && ((uint32_t)finfo[1] > c.N_f || finfo[3] > 160 * 1024 || finfo[2] < 1 || fws > ws)) bad |= 2048;
            if (!finfo[0] && c.F == 2 && fws != 0) bad |= 4096;
        }
        if (rp == CNGP_OK) {
            if (rl != CNGP_OK || rs != CNGP_OK || rr < 0) bad |= 1;
            for (int i = 0; i < rr; ++i)
                if (regions[2 * i + 1] && (regions[2 * i] % 256 || regions[2 * i] + regions[2 * i + 1] > ws)) bad |= 2;
            if (info[14] < 1) bad |= 4;
        } else if (ws != 0 && N > 0) {
            bad |= 8;                                                       // an invalid configuration needs no workspace
        }
        // entry points with a NULL where a buffer is required: rejected on the host, nothing is launched
        if (cngp_encode_fwd(&c, nullptr, 8, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == CNGP_OK) bad |= 16;
        if (cngp_encode_bwd(&c, nullptr, 8, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == CNGP_OK) bad |= 32;
        if (cngp_bake_probes(&c, nullptr, nullptr, nullptr) == CNGP_OK && !(c.index_format == CNGP_IDX_BITS && c.N_p == 1)) bad |= 64;
        if (cngp_encode_bwd_static(&c, nullptr, 8, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == CNGP_OK) bad |= 128;
    }
    cngp_mlp_config m = {32, 3, CNGP_F16, 0};
    if (cngp_mlp_weight_count(&m) != 64 * 32 + 64 * 64 + 64 * 3) bad |= 256;
    m.n_in = 40;
    if (cngp_mlp_weight_count(&m) != 0 || cngp_mlp_fwd(&m, nullptr, 8, nullptr, nullptr, nullptr) == CNGP_OK) bad |= 512;
    for (int s = 1; s >= -7; --s) if (!cngp_error_string(s)[0]) bad |= 1024;
    // the sort's workspace: three columns of N words plus 128 counters per tile of 8192 points and 128 totals
    for (int64_t N : {(int64_t)1, (int64_t)8192, (int64_t)8193, (int64_t)1 << 24, (int64_t)0x7fffffff}) {
        const size_t col = ((size_t)N * 4 + 255) / 256 * 256, tiles = ((size_t)N + 8191) / 8192;
        if (cngp_morton_sort_workspace_bytes(3, N) != 3 * col + (tiles * 512 + 255) / 256 * 256 + 512) bad |= 8192;
    }
    if (cngp_morton_sort_workspace_bytes(5, 100) != 0 || cngp_morton_sort(3, nullptr, 5, nullptr, nullptr, nullptr, 0, nullptr) == CNGP_OK) bad |= 8192;
    if (bad) { std::fprintf(stderr, "host sanitizer run: inconsistent results, mask %d\n", bad); return 1; }
    std::printf("host sanitizer run: clean\n");
    return 0;
}

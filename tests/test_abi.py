"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares,
validates arguments before touching the GPU, and computes the level table.  No GPU needed:
no call here reaches a kernel launch.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2312_17241_amd as cngp
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cngp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cngp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"cngp_encode_fwd", "cngp_encode_bwd", "cngp_bake_probes", "cngp_level_resolutions",
            "cngp_workspace_bytes", "cngp_debug_indices"} <= set(names)
    lib = ctypes.CDLL(cngp.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_error_strings():
    assert cngp.version() >= 100
    seen = {cngp.error_string(s) for s in range(0, -6, -1)}
    assert len(seen) == 6 and all(seen)
    assert "unknown" in cngp.error_string(-99)


def base_cfg(**kw):
    return cngp.Config.from_workload(W.WORKLOADS["nerf3d"], **kw)


@pytest.mark.parametrize("nmin,nmax,L,expect", [
    (int(h.split()[0]), int(h.split()[1]), int(h.split()[2]), list(map(int, t.split())))
    for h, t in (ln.split(":") for ln in open(os.path.join(GOLDEN, "level_tables.txt"))
                 if ln.strip() and not ln.startswith("#"))])
def test_level_table_golden(nmin, nmax, L, expect):
    cfg = base_cfg(N_min=nmin, N_max=nmax, L=L)
    assert cngp.level_resolutions(cfg).tolist() == expect


def test_level_table_edge_cases():
    assert cngp.level_resolutions(base_cfg(L=1, N_min=7, N_max=3)).tolist() == [7]
    assert cngp.level_resolutions(base_cfg(L=11, N_min=1, N_max=1024)).tolist() == [2**i for i in range(11)]
    r = cngp.level_resolutions(base_cfg(L=16, N_min=16, N_max=524288))
    assert r[0] == 16 and r[-1] == 524288 and np.all(np.diff(r.astype(np.int64)) > 0)


BAD = [
    dict(d=1), dict(d=5), dict(L=0), dict(L=33), dict(F=0),
    dict(N_f=0), dict(N_f=3000), dict(N_c=0), dict(N_c=100), dict(N_p=0), dict(N_p=3), dict(N_p=32),
    dict(N_p=16, N_f=8), dict(N_min=0), dict(N_max=8), dict(N_max=2**25),
    dict(feat_dtype=2), dict(io_dtype=-1), dict(index_format=3), dict(flags=256), dict(flags=64 | 128), dict(flags=64 | 16), dict(flags=6), dict(flags=34),
    dict(index_format=cngp.IDX_PACKED4, N_c=1, N_p=1), dict(top_k=17), dict(N_p=4, top_k=5),
]


@pytest.mark.parametrize("over", BAD, ids=[str(b) for b in BAD])
def test_invalid_configs_are_rejected_on_the_host(over):
    c = base_cfg(**over).c()
    one = ctypes.c_void_p(256)          # never dereferenced: validation fails first
    lib = cngp._lib
    assert lib.cngp_encode_fwd(ctypes.byref(c), one, 8, one, one, one, None, 0, None) == cngp.ERR_INVALID
    assert lib.cngp_encode_bwd(ctypes.byref(c), one, 8, one, one, one, one, one, None, 0, None) == cngp.ERR_INVALID
    assert lib.cngp_bake_probes(ctypes.byref(c), one, one, None) == cngp.ERR_INVALID
    assert lib.cngp_debug_indices(ctypes.byref(c), one, 8, one, one, one, one, one, None) == cngp.ERR_INVALID
    assert cngp.workspace_bytes(base_cfg(**over), 8) == 0


def test_reserved_field_must_be_zero_and_top_k_up_to_the_probing_range_is_valid():
    c = base_cfg().c()
    c.reserved = 1
    assert cngp._lib.cngp_bake_probes(ctypes.byref(c), ctypes.c_void_p(256), ctypes.c_void_p(256), None) == cngp.ERR_INVALID
    for k in (0, 1, base_cfg().N_p):
        assert cngp.workspace_bytes(base_cfg(top_k=k, flags=cngp.BWD_SLICED), 1 << 16) > 0


def test_unsupported_feature_width():
    c = base_cfg(F=3).c()                # 1, 2, 4 and 8 are built; the others are valid in the paper's terms only
    one = ctypes.c_void_p(256)
    assert cngp._lib.cngp_encode_fwd(ctypes.byref(c), one, 8, one, one, one, None, 0, None) == cngp.ERR_UNSUPPORTED
    out = np.zeros(16, np.uint32)        # the level table does not depend on F
    assert cngp._lib.cngp_level_resolutions(ctypes.byref(c), out.ctypes.data_as(ctypes.c_void_p)) == cngp.OK


def test_null_pointers_and_negative_counts():
    c = base_cfg().c()
    one = ctypes.c_void_p(256)
    lib = cngp._lib
    assert lib.cngp_encode_fwd(None, one, 8, one, one, one, None, 0, None) == cngp.ERR_NULL
    assert lib.cngp_encode_fwd(ctypes.byref(c), None, 8, one, one, one, None, 0, None) == cngp.ERR_NULL
    assert lib.cngp_encode_fwd(ctypes.byref(c), one, 8, None, one, one, None, 0, None) == cngp.ERR_NULL
    assert lib.cngp_encode_fwd(ctypes.byref(c), one, 8, one, None, one, None, 0, None) == cngp.ERR_NULL
    assert lib.cngp_encode_fwd(ctypes.byref(c), one, 8, one, one, None, None, 0, None) == cngp.ERR_NULL
    assert lib.cngp_encode_fwd(ctypes.byref(c), one, -1, one, one, one, None, 0, None) == cngp.ERR_INVALID
    assert lib.cngp_encode_fwd(ctypes.byref(c), None, 0, None, None, None, None, 0, None) == cngp.OK   # N == 0
    assert lib.cngp_encode_bwd(ctypes.byref(c), one, 8, one, one, one, None, one, None, 0, None) == cngp.ERR_NULL
    assert lib.cngp_encode_bwd(ctypes.byref(c), one, 8, one, None, one, one, one, None, 0, None) == cngp.ERR_NULL
    assert lib.cngp_encode_bwd(ctypes.byref(c), one, -5, one, one, one, one, one, None, 0, None) == cngp.ERR_INVALID
    assert lib.cngp_bake_probes(ctypes.byref(c), None, one, None) == cngp.ERR_NULL
    assert lib.cngp_bake_probes(ctypes.byref(c), one, None, None) == cngp.ERR_NULL
    assert lib.cngp_debug_indices(ctypes.byref(c), None, 8, one, one, one, one, one, None) == cngp.ERR_NULL
    assert lib.cngp_debug_indices(ctypes.byref(c), one, 8, None, one, one, one, None, None) == cngp.ERR_NULL
    assert lib.cngp_level_resolutions(ctypes.byref(c), None) == cngp.ERR_NULL
    # encoding + decoder in one call: checked on the host in the same way, with or without a workspace
    b = base_cfg()
    m, m_bad = cngp.MlpConfig(b.L * b.F, 3).c(), cngp.MlpConfig(b.L * b.F - 2, 3).c()
    mp = lambda v: ctypes.cast(ctypes.byref(v), ctypes.c_void_p)
    assert lib.cngp_encode_mlp_fwd(ctypes.byref(c), mp(m), None, 8, one, one, one, one, None, 0, None) == cngp.ERR_NULL
    assert lib.cngp_encode_mlp_fwd(ctypes.byref(c), mp(m), one, 8, one, one, None, one, one, 1 << 20, None) == cngp.ERR_NULL
    assert lib.cngp_encode_mlp_fwd(ctypes.byref(c), mp(m), one, -1, one, one, one, one, None, 0, None) == cngp.ERR_INVALID
    assert lib.cngp_encode_mlp_fwd(ctypes.byref(c), mp(m_bad), one, 8, one, one, one, one, None, 0, None) == cngp.ERR_INVALID
    assert lib.cngp_encode_mlp_fwd(ctypes.byref(c), mp(m), None, 0, None, None, None, None, None, 0, None) == cngp.OK


def test_adam_step_bake_rejects_bad_arguments():
    """Every check of the optimiser entry point runs on the host before anything is launched."""
    lib = ctypes.CDLL(cngp.LIB_PATH)
    c = base_cfg().c()                                   # nerf3d: fp16 feature storage
    a = ctypes.c_void_p(4096)                            # an aligned, never dereferenced address
    ok = cngp.Adam().c()
    feats = [a, a, a, a, a]
    logits = [a, a, a, a, a]

    def call(cfg, of, oc, f=feats, l=logits):
        ref = lambda o: None if o is None else ctypes.cast(ctypes.byref(o), ctypes.c_void_p)
        return lib.cngp_adam_step_bake(ctypes.byref(cfg), ref(of), ref(oc), *f, *l, None)

    assert call(c, None, None) == cngp.OK                # nothing to do
    for bad in (dict(lr=-1.0), dict(lr=float("nan")), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=0.0),
                dict(step=0), dict(grad_scale=float("inf"))):
        assert call(c, cngp.Adam(**bad).c(), None) == cngp.ERR_INVALID, bad
        assert call(c, None, cngp.Adam(**bad).c()) == cngp.ERR_INVALID, bad
    for i in range(5):
        f = list(feats); f[i] = None
        assert call(c, ok, None, f=f) == cngp.ERR_NULL, i
        l = list(logits); l[i] = None
        assert call(c, None, ok, l=l) == cngp.ERR_NULL, i
    for i in (0, 2, 3, 4):                               # misaligned float arrays
        f = list(feats); f[i] = ctypes.c_void_p(4100)
        assert call(c, ok, None, f=f) == cngp.ERR_INVALID, i
    for i in range(4):
        l = list(logits); l[i] = ctypes.c_void_p(4104)
        assert call(c, None, ok, l=l) == cngp.ERR_INVALID, i
    c32 = base_cfg(feat_dtype=cngp.F32).c()              # fp32 storage: D_f is NULL or the master itself
    assert call(c32, ok, None, f=[a, ctypes.c_void_p(8192), a, a, a]) == cngp.ERR_INVALID
    bad_cfg = base_cfg(N_p=3).c()
    assert call(bad_cfg, ok, ok) == cngp.ERR_INVALID


def test_storage_bytes_match_the_oracle_arithmetic():
    import oracle
    for N_p, N_c, fmt in [(8, 65536, cngp.IDX_BITS), (16, 16384, cngp.IDX_BITS), (2, 4, cngp.IDX_BITS), (1, 64, cngp.IDX_BITS),
                          (4, 8, cngp.IDX_BITS), (8, 1, cngp.IDX_BITS), (16, 16384, cngp.IDX_U8), (16, 16384, cngp.IDX_PACKED4)]:
        w = W.custom(d=3, L=16, N_f=256, N_c=N_c, N_p=N_p, N_min=16, N_max=2048, N=16, feat_dtype="f16")
        got = cngp.storage_bytes(cngp.Config.from_workload(w, index_format=fmt))
        if fmt == cngp.IDX_PACKED4:
            want = {"D_f": 16 * 256 * 2 * 2, "D_c_level": N_c // 2, "D_c": 16 * N_c // 2}
        else:
            want = oracle.storage_bytes(w, index_bits_exact=(fmt == cngp.IDX_BITS))
        assert got == want, (N_p, N_c, fmt)
        assert cngp.Config.from_workload(w, index_format=fmt).index_cols == want["D_c_level"]


def test_backward_plan_is_reported_on_the_host():
    """The plan needs no GPU: benchmark shapes take the LDS-sliced variant with pre-reduced coarse levels,
    a tiny batch takes global atomics, and the flags override the choice."""
    w = W.WORKLOADS["nerf3d"]
    p = cngp.bwd_plan_info(cngp.Config.from_workload(w), w.N)
    assert p["sliced"] == 1 and p["slices_f"] == 8 and p["slices_c"] == 16 and 1 <= p["dense_levels"] <= 6
    assert cngp.workspace_bytes(cngp.Config.from_workload(w), w.N) >= 4 * w.L * w.N_c * w.N_p + 2 * w.N * w.L * w.F
    t = W.WORKLOADS["tiny2d"]
    assert cngp.bwd_plan_info(cngp.Config.from_workload(t), t.N)["sliced"] == 0
    assert cngp.bwd_plan_info(cngp.Config.from_workload(t, flags=cngp.BWD_SLICED), t.N)["sliced"] == 1
    assert cngp.bwd_plan_info(cngp.Config.from_workload(w, flags=cngp.BWD_DIRECT), w.N)["sliced"] == 0
    assert cngp.bwd_plan_info(cngp.Config.from_workload(w, flags=cngp.BWD_NO_PREREDUCE), w.N)["dense_levels"] == 0
    pb = cngp.bwd_plan_info(cngp.Config.from_workload(w, flags=cngp.BWD_BINNED), w.N)
    assert pb["sliced"] == 1 and pb["binned"] == 1 and pb["drain_wgs_feat"] >= 1 and pb["bin_chunks"] == 256
    assert cngp.workspace_bytes(cngp.Config.from_workload(w, flags=cngp.BWD_BINNED), w.N) > 2 * (w.L - pb["dense_levels"]) * w.N * 8 * 4
    assert p["binned"] == 1                               # two dozen slices per level: the library bins by itself
    assert cngp.bwd_plan_info(cngp.Config.from_workload(w, flags=cngp.BWD_SLICED), w.N)["binned"] == 0
    im = W.WORKLOADS["image2d"]
    assert cngp.bwd_plan_info(cngp.Config.from_workload(im), im.N)["binned"] == 0      # ten slices: replicated scan
    huge = cngp.Config.from_workload(w)                   # 2^25 points: the bins would take 32 GiB: 4 passes of 8 GiB
    ph = cngp.bwd_plan_info(huge, 2**25)
    assert ph["binned"] == 1 and ph["passes"] == 4 and cngp.workspace_bytes(huge, 2**25) < 10 << 30
    assert cngp.workspace_bytes(huge, 2**25) == cngp.workspace_bytes(huge, 2**23)
    pf = cngp.bwd_plan_info(cngp.Config.from_workload(w, flags=cngp.BWD_BINNED), 2**25)   # on request: in one pass
    assert pf["binned"] == 1 and pf["passes"] == 1
    assert cngp.bwd_plan_info(cngp.Config.from_workload(w, flags=cngp.BWD_BINNED), 2**29)["passes"] == 3   # 2^31 references at most
    small = cngp.Config.from_workload(w, bin_bytes_max=1 << 30)
    assert cngp.bwd_plan_info(small, w.N)["passes"] == 1 and cngp.bwd_plan_info(small, 2**22)["passes"] == 4
    assert cngp.bwd_plan_info(cngp.Config.from_workload(w, bin_bytes_max=1 << 20), w.N)["binned"] == 0    # too small to bin
    assert p["passes"] == 1 and cngp.bwd_plan_info(cngp.Config.from_workload(w, flags=cngp.BWD_SLICED), 2**25)["passes"] == 1
    # the paper's compressed configurations (small N_f): binned by confidence-table slice only, both gradients in one pass
    for N_f, N_c, N_p, flag in ((2**8, 2**16, 8, 0), (2**12, 2**12, 16, 0), (2**6, 2**10, 4, cngp.BWD_BINNED)):
        small_f = W.custom(d=3, L=16, N_f=N_f, N_c=N_c, N_p=N_p, N_min=16, N_max=2048, N=2**18)
        ps = cngp.bwd_plan_info(cngp.Config.from_workload(small_f, flags=flag), small_f.N)
        assert ps["binned"] == 1 and ps["slices_f"] == 0 and ps["dense_levels"] == 0 and ps["slices_c"] >= 1
    few = W.custom(d=3, L=16, N_f=2**6, N_c=2**10, N_p=4, N_min=16, N_max=2048, N=2**18)      # two slices per level: replicated scan
    assert cngp.bwd_plan_info(cngp.Config.from_workload(few), few.N)["binned"] == 0
    assert cngp.bwd_plan_info(cngp.Config.from_workload(W.custom(d=3, L=16, N_f=2**13, N_c=2**10, N_p=4, N_min=16, N_max=2048, N=2**18)), 2**18)["slices_f"] > 0
    big = W.custom(d=3, L=16, N_f=2**24, N_c=2**24, N_p=2, N_min=16, N_max=2048, N=2**18)
    assert cngp.bwd_plan_info(cngp.Config.from_workload(big), big.N)["sliced"] == 0     # too many slices


def test_binding_rejects_host_tensors_and_wrong_shapes():
    import torch
    cfg = base_cfg()
    x = torch.zeros((4, 3))
    with pytest.raises(TypeError):
        cngp.encode_fwd(cfg, x, x, x, y=x)


def test_product_does_not_import_the_oracle():
    """The product package and its sources never reference the test oracle."""
    pkg = os.path.join(ROOT, "paper_2312_17241_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "cngp_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            assert "paper_2312_17241_amd" not in open(os.path.join(ROOT, "oracle", f)).read(), f


def test_backward_plan_layout_stays_inside_the_workspace():
    """For seeded random configurations and batch sizes, on every backward variant: the regions of the workspace the
    kernels index (cngp_bwd_plan_layout computes them from the kernels' own extents) are 256-byte aligned, do not
    overlap, and end inside cngp_workspace_bytes; the plan's counts are consistent with each other."""
    rng = np.random.default_rng(2024)
    seen = {"direct": 0, "sliced": 0, "binned": 0, "passes": 0, "fused": 0}
    for it in range(400):
        d = int(rng.choice([2, 3]))
        N_p = int(2 ** rng.integers(0, 5))
        N_f = int(2 ** rng.integers(max(2, int(np.log2(N_p))), 21))
        N_c = int(2 ** rng.integers(1, 19))
        L = int(rng.integers(1, 17))
        N_min = int(rng.integers(1, 33))
        N_max = int(N_min * 2 ** rng.integers(0, 9))
        N = int(rng.choice([1, 63, 4097, 70001, 2**18, 2**20 + 5, 2**22]))
        flags = int(rng.choice([0, 0, cngp.BWD_SLICED, cngp.BWD_BINNED, cngp.BWD_BINNED | cngp.BWD_NO_PREREDUCE, cngp.BWD_SLICED | cngp.BWD_NO_PREREDUCE]))
        bound = int(rng.choice([0, 0, 1 << 20, 1 << 26, 1 << 30]))
        w = W.custom(cfg=7, d=d, L=L, N_f=N_f, N_c=N_c, N_p=N_p, N_min=N_min, N_max=N_max, N=N,
                     feat_dtype=str(rng.choice(["f16", "f32"])), io_dtype=str(rng.choice(["f16", "f32"])))
        cfg = cngp.Config.from_workload(w, flags=cngp.ZERO_GRADS | flags, bin_bytes_max=bound)
        total = cngp.workspace_bytes(cfg, N)
        plan = cngp.bwd_plan_info(cfg, N)
        regions = cngp.bwd_plan_layout(cfg, N)
        assert (len(regions) == 0) == (plan["sliced"] == 0), (w, plan)
        spans = sorted((o, o + b) for o, b in regions if b > 0)
        for o, e in spans:
            assert o % 256 == 0 and e <= total, (w, plan, o, e, total)
        for (o0, e0), (o1, e1) in zip(spans, spans[1:]):
            assert e0 <= o1, (w, plan, spans)
        assert plan["passes"] >= 1 and 0 <= plan["dense_levels"] <= L
        if plan["binned"]:
            assert plan["sliced"] == 1 and plan["bin_chunks"] >= 1 and plan["drain_wgs_feat"] >= 1
            assert len(regions) == 12
        seen["binned" if plan["binned"] else "sliced" if plan["sliced"] else "direct"] += 1
        seen["passes"] += plan["passes"] > 1
        seen["fused"] += plan["binned"] == 1 and plan["slices_f"] == 0
    assert min(seen.values()) >= 5, seen          # the sweep reaches every variant


def test_forward_plan_is_within_the_chip_and_the_workspace():
    """The level-resident forward variant for seeded random configurations: the resident part of a level's feature
    codebook is a whole number of 16-byte pieces, at most the codebook; index codebook and resident part fit 160 KB of
    LDS; the level-major copy it needs fits cngp_workspace_bytes; the flags that force a variant are honoured."""
    rng = np.random.default_rng(77)
    taken = 0
    for it in range(300):
        N_p = int(2 ** rng.integers(0, 5))
        N_f = int(2 ** rng.integers(max(2, int(np.log2(N_p))), 22))
        feat, io = str(rng.choice(["f16", "f32"])), str(rng.choice(["f16", "f32"]))
        w = W.custom(cfg=8, d=int(rng.choice([2, 3, 4])), L=int(rng.integers(1, 17)), N_f=N_f, N_c=int(2 ** rng.integers(0, 21)),
                     N_p=N_p, N_min=4, N_max=256, N=int(rng.choice([1, 500, 4097, 2**17, 2**22 + 3])), feat_dtype=feat, io_dtype=io)
        cfg = cngp.Config.from_workload(w, flags=int(rng.choice([0, 0, cngp.FWD_LEVEL])))
        plan = cngp.fwd_plan_info(cfg, w.N)
        need = cngp.fwd_workspace_bytes(cfg, w.N)
        entry = 2 * (2 if feat == "f16" else 4)
        if plan["level_resident"]:
            taken += 1
            assert 0 < plan["resident_entries"] <= N_f and (plan["resident_entries"] * entry) % 16 == 0, (w, plan)
            assert plan["lds_bytes"] <= 160 * 1024 and plan["lds_bytes"] >= plan["resident_entries"] * entry + (w.N_c + 1) // 2
            assert plan["parts"] >= 1
            assert need == w.N * w.L * 2 * (2 if io == "f16" else 4) <= cngp.workspace_bytes(cfg, w.N)
        else:
            assert need == 0, (w, plan)
        tile = cngp.Config.from_workload(w, flags=cngp.FWD_TILE)
        assert cngp.fwd_plan_info(tile, w.N)["level_resident"] == 0 and cngp.fwd_workspace_bytes(tile, w.N) == 0
    assert taken >= 100


def test_morton_sort_workspace_is_host_arithmetic():
    """Two key columns, one index column, 128 counters per tile of 8192 points, 128 totals; no device is asked."""
    a = lambda v: (v + 255) // 256 * 256
    f = cngp._lib.cngp_morton_sort_workspace_bytes
    for N in (1, 8192, 8193, 2**24, 2**31 - 1):
        tiles = (N + 8191) // 8192
        assert f(3, N) == f(2, N) == f(4, N) == 3 * a(4 * N) + a(128 * 4 * tiles) + a(128 * 4)
    assert f(3, 0) == 0 and f(3, -5) == 0 and f(3, 2**31) == 0 and f(5, 100) == 0 and f(1, 100) == 0
    assert cngp._lib.cngp_morton_sort(3, None, 0, None, None, None, 0, None) == cngp.OK
    assert cngp._lib.cngp_morton_sort(3, None, 10, None, None, None, 0, None) == cngp.ERR_NULL
    assert cngp._lib.cngp_morton_sort(5, None, 10, None, None, None, 0, None) == cngp.ERR_INVALID


def test_host_code_runs_clean_under_sanitizers():
    """csrc/host_check_main.cpp drives validation, level table, storage sizes, the backward plan and its workspace
    layout through the C ABI for 300 seeded random configurations (valid and invalid) in a program whose host side
    is built with AddressSanitizer and UndefinedBehaviorSanitizer.  No kernel is launched.  The first run compiles
    the program (about two minutes); later runs reuse it until a source changes."""
    import subprocess
    from paper_2312_17241_amd.build import build_host_sanitized
    exe = build_host_sanitized()
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0 and "clean" in res.stdout, res.stdout + res.stderr

"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integers bit-exact, floating point within the bars of tests/parity.py.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2312_17241_amd as cngp
import workloads as W
import parity
from parity import check_close, check_exact

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def tables(w, n=None):
    x = W.make_points(w, n)
    return x, W.make_feature_codebook(w), W.make_probe_logits(w), W.make_upstream_grad(w, x.shape[0])


def run_fwd(w, x, D_f, D_c, index_format=cngp.IDX_U8, flags=0):
    cfg = cngp.Config.from_workload(w, index_format=index_format, flags=flags)
    D_c_dev = dev(D_c)
    if index_format == cngp.IDX_PACKED4:
        D_c_dev = cngp.pack4(D_c_dev)
    ws = cngp.alloc_workspace(cfg, x.shape[0])
    y = cngp.encode_fwd(cfg, dev(x), dev(D_f), D_c_dev, workspace=ws)
    torch.cuda.synchronize()
    return host(y)


def run_bwd(w, x, D_f, Dhat, dy, flags=cngp.ZERO_GRADS, init=None, **over):
    cfg = cngp.Config.from_workload(w, flags=flags, **over)
    gF = torch.full((w.L, w.N_f, w.F), float("nan") if init is None else init, device=DEV)
    gC = torch.full((w.L, w.N_c, w.N_p), float("nan") if init is None else init, device=DEV)
    ws = cngp.alloc_workspace(cfg, x.shape[0])
    cngp.encode_bwd(cfg, dev(x), dev(D_f), dev(Dhat), dev(dy), gF, gC, workspace=ws)
    torch.cuda.synchronize()
    return host(gF), host(gC)


def check_fwd(w, x, D_f, D_c, index_format=cngp.IDX_U8, name=""):
    """The forward variants (the library's own choice given a workspace: level-resident where it can run; tile: index
    codebook staged in LDS per tile; simple: everything read from memory) against the oracle."""
    y_ref, ymag = oracle.encode_fwd(w, x, D_f, D_c)
    worst = 0.0
    for variant, flags in (("own choice", 0), ("tile", cngp.FWD_TILE), ("simple", cngp.FWD_SIMPLE)):
        y = run_fwd(w, x, D_f, D_c, index_format, flags)
        worst = max(worst, check_close(f"y {name} [{variant}]", y, y_ref, ymag, fp16_out=(w.io_dtype == "f16")))
    return worst


# the ways the library can run the backward pass: its own choice, and each variant forced
BWD_PATHS = {"auto": 0, "direct": cngp.BWD_DIRECT, "sliced": cngp.BWD_SLICED,
             "sliced_nopre": cngp.BWD_SLICED | cngp.BWD_NO_PREREDUCE,
             "binned": cngp.BWD_BINNED, "binned_nopre": cngp.BWD_BINNED | cngp.BWD_NO_PREREDUCE}


def check_bwd(w, x, D_f, Dhat, dy, name="", paths=("auto", "direct", "sliced", "sliced_nopre", "binned", "binned_nopre"),
              top_k=0):
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x, D_f, Dhat, dy, top_k=top_k)
    worst = (0.0, 0.0)
    for path in paths:
        gF, gC = run_bwd(w, x, D_f, Dhat, dy, flags=cngp.ZERO_GRADS | BWD_PATHS[path], top_k=top_k)
        e1 = check_close(f"grad D_f {name} [{path}]", gF, gF_ref, A_f, fp16_out=False)
        e2 = check_close(f"grad Dhat_c {name} [{path}]", gC, gC_ref, A_c, fp16_out=False)
        worst = (max(worst[0], e1), max(worst[1], e2))
    return worst


# ------------------------------------------------------------------ indices, bit-exact

@pytest.mark.parametrize("name", ["tiny2d", "nerf3d", "sdf3d", "image2d"])
@pytest.mark.parametrize("fmt", [cngp.IDX_U8, cngp.IDX_PACKED4])
def test_indices_bit_exact(name, fmt):
    w = W.WORKLOADS[name]
    n = min(w.N, 20000 + 37)
    x = W.make_points(w, n)
    x[:4] = [[0.0] * w.d, [1.0] * w.d, [0.5] * w.d, [1.0] + [0.0] * (w.d - 1)]
    D_c = oracle.bake_probes(W.make_probe_logits(w))
    cfg = cngp.Config.from_workload(w, index_format=fmt)
    D_c_dev = dev(D_c) if fmt == cngp.IDX_U8 else cngp.pack4(dev(D_c))
    got = cngp.debug_indices(cfg, dev(x), D_c_dev)
    torch.cuda.synchronize()
    want = oracle.indices(w, x, D_c)
    for nm, g, r in zip(("base", "h2", "probe", "feat_idx"), got, want):
        check_exact(f"{nm} {name}", host(g).view(r.dtype), r)
    assert int(host(got[3]).max()) < w.N_f


def test_indices_large_resolution_bit_exact():
    """Finest resolution of Table 1's range (N_max = 524288): fp32 scaling must round identically."""
    w = W.custom(d=3, L=16, N_f=2**12, N_c=2**10, N_p=16, N_min=16, N_max=524288, N=5000)
    x = W.make_points(w)
    D_c = np.random.default_rng(3).integers(0, w.N_p, (w.L, w.N_c)).astype(np.uint8)
    got = cngp.debug_indices(cngp.Config.from_workload(w), dev(x), dev(D_c))
    want = oracle.indices(w, x, D_c)
    for nm, g, r in zip(("base", "h2", "probe", "feat_idx"), got, want):
        check_exact(nm, host(g).view(r.dtype), r)


# ------------------------------------------------------------------ bake, bit-exact

@pytest.mark.parametrize("N_p", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("fmt", [cngp.IDX_U8, cngp.IDX_PACKED4])
def test_bake_bit_exact(N_p, fmt):
    w = W.custom(L=3, N_c=2048 + 0, N_p=N_p, N_f=4096)
    rng = np.random.default_rng(N_p)
    Dhat = rng.standard_normal((w.L, w.N_c, w.N_p)).astype(np.float32)
    # degenerate rows: all equal, ties, NaN, infinities
    Dhat[0, 0] = 1.0
    Dhat[0, 1] = np.nan
    Dhat[0, 2] = -np.inf
    if N_p >= 4:
        Dhat[0, 3] = 0.0; Dhat[0, 3, 1] = 2.0; Dhat[0, 3, 2] = 2.0
        Dhat[0, 4] = np.nan; Dhat[0, 4, N_p - 1] = -5.0
        Dhat[0, 5, 0] = np.nan; Dhat[0, 5, 1] = np.inf
    want = oracle.bake_probes(Dhat)
    assert want.max() < N_p
    cfg = cngp.Config.from_workload(w, index_format=fmt)
    got = cngp.bake_probes(cfg, dev(Dhat))
    torch.cuda.synchronize()
    if fmt == cngp.IDX_PACKED4:
        packed = host(got)
        assert packed.shape == (w.L, w.N_c // 2)
        got_u8 = np.empty((w.L, w.N_c), np.uint8)
        got_u8[:, 0::2] = packed & 0xF
        got_u8[:, 1::2] = packed >> 4
    else:
        got_u8 = host(got)
    check_exact("D_c", got_u8, want)


@pytest.mark.parametrize("name", ["tiny2d", "nerf3d"])
def test_bake_workload_tables(name):
    w = W.WORKLOADS[name]
    Dhat = W.make_probe_logits(w)
    got = cngp.bake_probes(cngp.Config.from_workload(w), dev(Dhat))
    check_exact("D_c", host(got), oracle.bake_probes(Dhat))


# ------------------------------------------------------------------ forward / backward, small sweeps

SWEEP = [
    # d, N_p, feat, io
    (2, 1, "f32", "f32"), (2, 4, "f32", "f32"), (2, 8, "f16", "f16"), (2, 16, "f16", "f32"),
    (3, 1, "f16", "f16"), (3, 2, "f32", "f16"), (3, 4, "f32", "f32"), (3, 8, "f16", "f16"),
    (3, 16, "f16", "f16"), (3, 16, "f32", "f32"),
]


def sweep_workload(d, N_p, feat, io, N=3000 + 77):
    return W.custom(cfg=50 + d * 17 + N_p, d=d, L=5, N_f=2**11, N_c=2**9, N_p=N_p, N_min=4, N_max=300,
                    N=N, feat_dtype=feat, io_dtype=io)


@pytest.mark.parametrize("d,N_p,feat,io", SWEEP)
def test_forward_parity_sweep(d, N_p, feat, io):
    w = sweep_workload(d, N_p, feat, io)
    x, D_f, Dhat, _ = tables(w)
    x[:3] = [[0.0] * d, [1.0] * d, [0.5] * d]
    D_c = oracle.bake_probes(Dhat)
    check_fwd(w, x, D_f, D_c, cngp.IDX_U8, "u8")
    if w.N_c >= 2:
        check_fwd(w, x, D_f, D_c, cngp.IDX_PACKED4, "packed4")


@pytest.mark.parametrize("d,N_p,feat,io", SWEEP)
def test_backward_parity_sweep(d, N_p, feat, io):
    w = sweep_workload(d, N_p, feat, io)
    x, D_f, Dhat, dy = tables(w)
    x[:3] = [[0.0] * d, [1.0] * d, [0.5] * d]
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)      # O(1) features: logit gradients well scaled
    check_bwd(w, x, D_f, Dhat, dy)


@pytest.mark.parametrize("path", ["direct", "sliced", "sliced_nopre", "binned", "binned_nopre"])
def test_backward_accumulates_without_zero_flag(path):
    w = sweep_workload(3, 4, "f32", "f32", N=500)
    x, D_f, Dhat, dy = tables(w)
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    gF, gC = run_bwd(w, x, D_f, Dhat, dy, flags=BWD_PATHS[path], init=1.5)
    check_close("grad D_f (+=)", gF, gF_ref + 1.5, A_f + 1.5, fp16_out=False)
    check_close("grad Dhat_c (+=)", gC, gC_ref + 1.5, A_c + 1.5, fp16_out=False)


def test_sliced_backward_many_chunks_and_slices():
    """Tables larger than one LDS slice and enough points for several chunks per slice."""
    w = W.custom(cfg=81, d=3, L=2, N_f=2**15, N_c=2**12, N_p=16, N_min=16, N_max=512, N=70000 + 5,
                 feat_dtype="f16", io_dtype="f16")
    x, D_f, Dhat, dy = tables(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    check_bwd(w, x, D_f, Dhat, dy, paths=("sliced", "sliced_nopre", "auto", "binned", "binned_nopre"))


def test_binned_backward_tables_of_a_thousand_slices():
    """An index codebook of 2^20 rows per level (the upper end of the paper's N_c sweeps) makes 1024 slices of the
    logit gradient: far too many to scan the points once per slice, so the library bins by itself; several point
    chunks, several drain workgroups per bin of the (single-slice) feature table, two pre-reduced levels."""
    w = W.custom(cfg=83, d=2, L=3, N_f=2**10, N_c=2**20, N_p=16, N_min=16, N_max=2048, N=300000 + 19,
                 feat_dtype="f16", io_dtype="f16")
    cfg = cngp.Config.from_workload(w)
    plan = cngp.bwd_plan_info(cfg, w.N)
    assert plan["binned"] == 1 and plan["slices_c"] == 1024 and plan["bin_chunks"] > 1 and plan["drain_wgs_feat"] > 1
    x, D_f, Dhat, dy = tables(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    check_bwd(w, x, D_f, Dhat, dy, paths=("auto", "binned_nopre"))


@pytest.mark.parametrize("d,N_p,top_k", [(3, 16, 1), (3, 16, 2), (3, 16, 4), (3, 16, 5), (3, 16, 8), (3, 16, 16),
                                         (2, 8, 1), (2, 8, 2), (2, 8, 4), (3, 4, 2), (2, 2, 1), (3, 4, 3)])
def test_sparse_backward_parity(d, N_p, top_k):
    """The sparse variant (softmax over the top_k largest confidence values of a row) in every way the library can
    run the backward.  Half of the rows hold values from a coarse lattice, so equal values are common and
    the rule for them (lowest index first) decides the kept set."""
    w = sweep_workload(d, N_p, "f16", "f16")
    x, D_f, Dhat, dy = tables(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    Dhat = Dhat.copy()
    Dhat[:, ::2] = np.round(Dhat[:, ::2] * 2.0) / 2.0             # values k / 2: many ties
    assert np.mean(np.sort(Dhat[:, ::2], axis=-1)[..., 1:] == np.sort(Dhat[:, ::2], axis=-1)[..., :-1]) > 0.05
    check_bwd(w, x, D_f, Dhat, dy, top_k=top_k)


def test_sparse_backward_never_keeps_a_nan_before_a_number():
    w = sweep_workload(3, 8, "f32", "f32", N=2000)
    x, D_f, Dhat, dy = tables(w)
    Dhat = Dhat.copy()
    Dhat[:, :, 3] = np.nan
    Dhat[:, ::3, 6] = np.nan
    check_bwd(w, x, D_f, Dhat, dy, top_k=4)


@pytest.mark.parametrize("N_f,N_c,N_p,feat,io,d", [
    (2**6, 2**10, 4, "f16", "f16", 3), (2**8, 2**16, 8, "f16", "f16", 3), (2**8, 2**12, 16, "f32", "f32", 3),
    (2**12, 2**14, 16, "f16", "f32", 3), (2**12, 2**13, 2, "f32", "f16", 2), (2**10, 2**15, 8, "f16", "f16", 2)])
def test_small_feature_tables_both_gradients_in_one_pass(N_f, N_c, N_p, feat, io, d):
    """The paper's compressed configurations (N_f = 2^6 .. 2^12): the library bins by slice of the confidence table only
    and the workgroups that drain those bins accumulate the level's whole feature gradient in LDS as well.  Enough
    points for several workgroups per bin; with and without clearing first."""
    w = W.custom(cfg=90, d=d, L=6, N_f=N_f, N_c=N_c, N_p=N_p, N_min=8, N_max=512, N=120000 + 11, feat_dtype=feat, io_dtype=io)
    plan = cngp.bwd_plan_info(cngp.Config.from_workload(w, flags=cngp.BWD_BINNED), w.N)
    assert plan["binned"] == 1 and plan["slices_f"] == 0 and plan["dense_levels"] == 0
    x, D_f, Dhat, dy = tables(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    check_bwd(w, x, D_f, Dhat, dy, paths=("auto", "binned", "binned_nopre", "sliced", "direct"))
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    gF, gC = run_bwd(w, x, D_f, Dhat, dy, flags=cngp.BWD_BINNED, init=-0.5)
    check_close("grad D_f (+=)", gF, gF_ref - 0.5, A_f + 0.5, fp16_out=False)
    check_close("grad Dhat_c (+=)", gC, gC_ref - 0.5, A_c + 0.5, fp16_out=False)


def test_small_feature_tables_in_passes_with_the_sparse_variant():
    """The same mode with a bound on the binned references (three passes) and the top-2 sparse variant together."""
    w = W.custom(cfg=91, d=3, L=5, N_f=2**9, N_c=2**13, N_p=8, N_min=8, N_max=400, N=100000 + 3, feat_dtype="f16", io_dtype="f16")
    limit = 40000 * 8 * 4 * w.L * 2
    cfg = cngp.Config.from_workload(w, flags=cngp.ZERO_GRADS | cngp.BWD_BINNED, bin_bytes_max=limit, top_k=2)
    plan = cngp.bwd_plan_info(cfg, w.N)
    assert plan["binned"] == 1 and plan["slices_f"] == 0 and plan["passes"] == 3
    x, D_f, Dhat, dy = tables(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x, D_f, Dhat, dy, top_k=2)
    gF, gC = run_bwd(w, x, D_f, Dhat, dy, flags=cngp.ZERO_GRADS | cngp.BWD_BINNED, bin_bytes_max=limit, top_k=2)
    check_close("grad D_f", gF, gF_ref, A_f, fp16_out=False)
    check_close("grad Dhat_c", gC, gC_ref, A_c, fp16_out=False)


@pytest.mark.parametrize("zero", [True, False])
@pytest.mark.parametrize("forced", [True, False])
def test_binned_backward_in_several_passes(zero, forced):
    """A bound on the bytes of binned references splits the batch into runs of points taken one after the other
    inside the one call: the first pass clears (if asked), the others add; the last run is shorter."""
    w = W.custom(cfg=84, d=3, L=8, N_f=2**16, N_c=2**14, N_p=16, N_min=16, N_max=1024, N=150000 + 7,
                 feat_dtype="f16", io_dtype="f16")
    per_point = 4 * 2**w.d * w.L * 2              # 4-byte records, both tables
    limit = 40000 * per_point                       # 39 * 1024 points per pass
    flags = (cngp.ZERO_GRADS if zero else 0) | (cngp.BWD_BINNED if forced else 0)
    cfg = cngp.Config.from_workload(w, flags=flags, bin_bytes_max=limit)
    plan = cngp.bwd_plan_info(cfg, w.N)
    assert plan["binned"] == 1 and plan["passes"] == 4
    assert cngp.workspace_bytes(cfg, w.N) < cngp.workspace_bytes(cngp.Config.from_workload(w, flags=flags), w.N) / 3
    x, D_f, Dhat, dy = tables(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    init = None if zero else 0.25
    gF, gC = run_bwd(w, x, D_f, Dhat, dy, flags=flags, init=init, bin_bytes_max=limit)
    off = 0.0 if zero else 0.25
    check_close("grad D_f (passes)", gF, gF_ref + off, A_f + off, fp16_out=False)
    check_close("grad Dhat_c (passes)", gC, gC_ref + off, A_c + off, fp16_out=False)


@pytest.mark.parametrize("d", [2, 3])
def test_sliced_backward_vertex_grids_of_several_slices(d):
    """Coarse levels whose dense vertex grid spans several LDS slices, next to hashed fine levels."""
    w = W.custom(cfg=82 + d, d=d, L=6, N_f=2**13, N_c=2**11, N_p=8, N_min=20, N_max=(600 if d == 2 else 90),
                 N=150000 + 11, feat_dtype="f16", io_dtype="f16", points="uniform")
    x, D_f, Dhat, dy = tables(w)
    x[:3] = [[0.0] * d, [1.0] * d, [0.5] * d]
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    check_bwd(w, x, D_f, Dhat, dy, paths=("sliced", "sliced_nopre"))


def test_sliced_backward_needs_workspace():
    w = sweep_workload(3, 4, "f32", "f32", N=5000)
    cfg = cngp.Config.from_workload(w, flags=cngp.BWD_SLICED)
    assert cngp.workspace_bytes(cfg, w.N) > 0
    x, D_f, Dhat, dy = tables(w)
    with pytest.raises(cngp.CngpError) as e:
        cngp.encode_bwd(cfg, dev(x), dev(D_f), dev(Dhat), dev(dy), workspace=None)
    assert e.value.status == cngp.ERR_WORKSPACE
    direct = cngp.Config.from_workload(w, flags=cngp.BWD_DIRECT)              # the backward needs none, the forward may
    assert cngp.workspace_bytes(direct, w.N) == cngp.fwd_workspace_bytes(direct, w.N)
    assert cngp.workspace_bytes(cngp.Config.from_workload(w, flags=cngp.BWD_DIRECT | cngp.FWD_TILE), w.N) == 0


# ------------------------------------------------------------------ edge cases

def test_empty_batch_is_a_noop_and_zeroes_grads():
    w = sweep_workload(3, 4, "f32", "f32", N=0)
    cfg = cngp.Config.from_workload(w, flags=cngp.ZERO_GRADS)
    x = torch.empty((0, 3), device=DEV)
    D_f = dev(W.make_feature_codebook(w)); Dhat = dev(W.make_probe_logits(w))
    y = cngp.encode_fwd(cfg, x, D_f, cngp.bake_probes(cfg, Dhat))
    assert y.shape == (0, w.L * w.F)
    gF = torch.ones((w.L, w.N_f, w.F), device=DEV); gC = torch.ones((w.L, w.N_c, w.N_p), device=DEV)
    cngp.encode_bwd(cfg, x, D_f, Dhat, torch.empty((0, w.L * w.F), device=DEV), gF, gC)
    torch.cuda.synchronize()
    assert float(gF.abs().max()) == 0.0 and float(gC.abs().max()) == 0.0


@pytest.mark.parametrize("N", [1, 63, 64, 65, 255, 257])
def test_ragged_tails(N):
    w = sweep_workload(3, 16, "f16", "f16", N=N)
    x, D_f, Dhat, dy = tables(w)
    check_fwd(w, x, D_f, oracle.bake_probes(Dhat))
    check_bwd(w, x, D_f, Dhat, dy)


@pytest.mark.parametrize("over", [dict(L=1, N_min=9), dict(L=32, N_min=2, N_max=5000), dict(N_c=1), dict(N_c=2),
                                  dict(N_f=16, N_p=16), dict(N_f=2, N_p=2, N_c=4), dict(N_min=1, N_max=1, L=2),
                                  dict(N_f=2**20, N_c=2**18, N_p=2)])
def test_degenerate_configurations(over):
    kw = dict(cfg=77, d=3, L=4, N_f=256, N_c=64, N_p=4, N_min=4, N_max=64, N=700, feat_dtype="f32", io_dtype="f32")
    kw.update(over)
    w = W.custom(**kw)
    x, D_f, Dhat, dy = tables(w)
    x[:2] = [[0.0] * 3, [1.0] * 3]
    D_c = oracle.bake_probes(Dhat)
    check_fwd(w, x, D_f, D_c)
    if w.N_c >= 2:
        check_fwd(w, x, D_f, D_c, cngp.IDX_PACKED4)
    check_bwd(w, x, D_f, Dhat, dy)


def test_points_on_grid_vertices_and_cube_faces():
    """Points on vertices (zero-weight corners still looked up) and on the faces x_i in {0, 1}."""
    w = W.custom(cfg=78, d=3, L=3, N_f=512, N_c=128, N_p=8, N_min=8, N_max=32, N=4096)
    rng = np.random.default_rng(0)
    x = (rng.integers(0, 33, (w.N, 3)) / 32.0).astype(np.float32)
    x[::3, 0] = 1.0; x[1::3, 1] = 0.0
    _, D_f, Dhat, dy = tables(w)
    check_fwd(w, x, D_f, oracle.bake_probes(Dhat))
    check_bwd(w, x, D_f, Dhat, dy)


def test_probe_range_one_matches_unprobed_hash_grid():
    """N_p = 1 (Sec. 3 "Selecting hyperparameters"): the index codebook plays no role."""
    w = W.custom(cfg=79, d=3, L=6, N_f=2**12, N_c=1, N_p=1, N_min=8, N_max=256, N=5000,
                 feat_dtype="f16", io_dtype="f16")
    x, D_f, Dhat, dy = tables(w)
    check_fwd(w, x, D_f, np.zeros((w.L, 1), np.uint8))
    for path in ("direct", "sliced"):
        gF, gC = run_bwd(w, x, D_f, Dhat, dy, flags=cngp.ZERO_GRADS | BWD_PATHS[path])
        assert np.all(gC == 0.0)
    check_bwd(w, x, D_f, Dhat, dy)


# ------------------------------------------------------------------ adversarial point sets

@pytest.mark.parametrize("kind", ["identical", "axis_line", "two_cells", "corner_of_cube"])
def test_backward_hot_spots(kind):
    """Point sets that send every corner reference to a handful of table rows: one workgroup's slice
    takes all the traffic (its queue fills in every round) and its LDS atomics all collide."""
    w = W.custom(cfg=90, d=3, L=5, N_f=2**14, N_c=2**12, N_p=16, N_min=16, N_max=512, N=60000 + 3,
                 feat_dtype="f16", io_dtype="f16")
    rng = np.random.default_rng(11)
    if kind == "identical":
        x = np.tile(np.array([[0.3141, 0.2718, 0.5772]], np.float32), (w.N, 1))
    elif kind == "axis_line":
        x = np.zeros((w.N, 3), np.float32); x[:, 0] = rng.random(w.N); x[:, 1] = 0.5; x[:, 2] = 0.25
    elif kind == "two_cells":
        x = (np.array([[0.1, 0.1, 0.1]]) + (rng.integers(0, 2, (w.N, 1)) * 0.7) + rng.random((w.N, 3)) * 1e-3).astype(np.float32)
    else:
        x = np.ones((w.N, 3), np.float32)
    _, D_f, Dhat, dy = tables(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    check_fwd(w, x, D_f, oracle.bake_probes(Dhat))
    check_bwd(w, x, D_f, Dhat, dy)


def test_backward_is_reproducible_within_tolerance():
    """Two runs of the same backward call: atomics reorder the sums, results stay within the bar of each other."""
    w = W.WORKLOADS["nerf3d"]
    x, D_f, Dhat, dy = tables(w, 50000)
    g1 = run_bwd(w, x, D_f, Dhat, dy)
    g2 = run_bwd(w, x, D_f, Dhat, dy)
    for a, b in zip(g1, g2):
        scale = max(float(np.abs(a).max()), 1e-30)
        assert float(np.abs(a - b).max()) <= 1e-5 * scale


# ------------------------------------------------------------------ randomised configurations

def _random_workloads(count=24, seed=2024):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        d = int(rng.choice([2, 3]))
        N_p = int(rng.choice([1, 2, 4, 8, 16]))
        N_f = int(2 ** rng.integers(max(2, int(np.log2(N_p))), 15))
        N_c = int(2 ** rng.integers(0, 13))
        L = int(rng.integers(1, 9))
        N_min = int(rng.integers(1, 20))
        N_max = int(N_min * 2 ** rng.integers(0, 7)) if L > 1 else N_min
        N = int(rng.choice([1, 17, 300, 2500, 9000, 40000]))
        out.append(W.custom(name=f"rand{i}", cfg=200 + i, d=d, L=L, N_f=max(N_f, N_p), N_c=N_c, N_p=N_p,
                            N_min=N_min, N_max=N_max, N=N, feat_dtype=str(rng.choice(["f32", "f16"])),
                            io_dtype=str(rng.choice(["f32", "f16"])),
                            points=("uniform" if d == 2 else str(rng.choice(["uniform", "nerf_rays", "sdf_shell"])))))
    return out


@pytest.mark.parametrize("w", _random_workloads(), ids=lambda w: f"{w.name}-d{w.d}-L{w.L}-Nf{w.N_f}-Nc{w.N_c}-Np{w.N_p}-N{w.N}")
def test_random_configurations(w):
    """Seeded random hyper-parameters and batch sizes: indices, bake, forward and every backward variant."""
    x, D_f, Dhat, dy = tables(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    D_c = oracle.bake_probes(Dhat)
    cfg = cngp.Config.from_workload(w)
    check_exact("D_c", host(cngp.bake_probes(cfg, dev(Dhat))), D_c)
    got = cngp.debug_indices(cfg, dev(x), dev(D_c))
    for nm, g, r in zip(("base", "h2", "probe", "feat_idx"), got, oracle.indices(w, x, D_c)):
        check_exact(nm, host(g).view(r.dtype), r)
    check_fwd(w, x, D_f, D_c)
    if w.N_c >= 2:
        check_fwd(w, x, D_f, D_c, cngp.IDX_PACKED4)
    check_bwd(w, x, D_f, Dhat, dy)


# ------------------------------------------------------------------ full benchmark sizes

@pytest.mark.parametrize("name", ["tiny2d", "nerf3d", "image2d", "sdf3d"])
def test_full_size_forward_backward(name):
    w = W.WORKLOADS[name]
    x, D_f, Dhat, dy = tables(w)
    D_c = oracle.bake_probes(Dhat)
    e_y = check_fwd(w, x, D_f, D_c, name=name)
    e_f, e_c = check_bwd(w, x, D_f, Dhat, dy, name=name)
    plain = {k.split(" [")[0].replace(f" {name}", ""): v for k, v in parity.PLAIN.items() if name in k}
    print(f"\n{name}: max rel err (relative to the terms' magnitude sum)  y {e_y:.2e}  grad D_f {e_f:.2e}  grad Dhat_c {e_c:.2e}"
          f"\n{name}: plain max|gpu - ref| / max|ref| per tensor  " + "  ".join(f"{k} {v:.2e}" for k, v in plain.items()))
    # the plain figure has its own sanity bar: a tensor's largest error against its largest value
    assert all(v <= (2e-3 if k.startswith("y") and w.io_dtype == "f16" else 1e-5) for k, v in plain.items()), plain


def test_full_size_inference_sampled():
    """2^24-point forward with the 4-bit packed index codebook; the oracle evaluates a random
    sample of the points one by one."""
    w = W.WORKLOADS["infer3d"]
    x = W.make_points(w)
    D_f = W.make_feature_codebook(w)
    D_c = oracle.bake_probes(W.make_probe_logits(w))
    cfg = cngp.Config.from_workload(w, index_format=cngp.IDX_PACKED4)
    # as the benchmark runs it: with the workspace, i.e. the level-resident variant; the tile variant gives the same bits
    assert cngp.fwd_plan_info(cfg, w.N)["level_resident"] == 1
    y = cngp.encode_fwd(cfg, dev(x), dev(D_f), cngp.pack4(dev(D_c)), workspace=cngp.alloc_workspace(cfg, w.N))
    y_tile = cngp.encode_fwd(cfg, dev(x), dev(D_f), cngp.pack4(dev(D_c)))
    torch.cuda.synchronize()
    assert torch.equal(y, y_tile)
    del y_tile
    pick = np.random.default_rng(5).choice(w.N, 1 << 16, replace=False)
    pick[:2] = [0, w.N - 1]
    y_ref, ymag = oracle.encode_fwd(w, x[pick], D_f, D_c)
    check_close("y infer3d sample", host(y[torch.from_numpy(pick).to(DEV)]), y_ref, ymag, fp16_out=True)
    # the unprobed hash grid (N_p = 1) at the same N_f, run alongside
    w1 = W.custom(cfg=w.cfg, d=3, L=16, N_f=w.N_f, N_c=1, N_p=1, N_min=16, N_max=2048, N=w.N,
                  feat_dtype="f16", io_dtype="f16")
    cfg1 = cngp.Config.from_workload(w1)
    zeros = np.zeros((16, 1), np.uint8)
    y1 = cngp.encode_fwd(cfg1, dev(x), dev(D_f), dev(zeros), workspace=cngp.alloc_workspace(cfg1, w.N))
    y1_ref, y1mag = oracle.encode_fwd(w1, x[pick], D_f, zeros)
    check_close("y hash grid sample", host(y1[torch.from_numpy(pick).to(DEV)]), y1_ref, y1mag, fp16_out=True)


def test_probe_entries_beyond_the_probe_range_are_masked():
    """The header requires every D_c entry to be below N_p; the kernels nevertheless mask what they read to the probe
    range, so a corrupt codebook cannot move a lookup out of its feature codebook.  Entries with extra high bits give
    exactly the output of the clean codebook (the last level is left clean: nothing here relies on the mask to stay
    inside the allocation)."""
    w = W.custom(cfg=88, d=3, L=4, N_f=2**10, N_c=2**8, N_p=4, N_min=4, N_max=64, N=3000 + 5)
    x, D_f = W.make_points(w), W.make_feature_codebook(w)
    D_c = oracle.bake_probes(W.make_probe_logits(w))
    rng = np.random.default_rng(11)
    for fmt, top in ((cngp.IDX_U8, 64), (cngp.IDX_PACKED4, 4)):
        bad = D_c.copy()
        bad[:-1] += (w.N_p * rng.integers(0, top, bad[:-1].shape)).astype(np.uint8)
        assert bad.max() >= w.N_p
        pack = (lambda a: dev(a)) if fmt == cngp.IDX_U8 else (lambda a: cngp.pack4(dev(a)))
        for flags in (0, cngp.FWD_SIMPLE):
            cfg = cngp.Config.from_workload(w, index_format=fmt, flags=flags)
            y_clean = cngp.encode_fwd(cfg, dev(x), dev(D_f), pack(D_c))
            y_bad = cngp.encode_fwd(cfg, dev(x), dev(D_f), pack(bad))
            torch.cuda.synchronize()
            assert torch.equal(y_clean, y_bad)


@pytest.mark.parametrize("d", [2, 3])
def test_points_on_cell_faces_and_grid_vertices(d):
    """Corners of weight exactly zero are skipped by the LDS variants of the backward pass (no record, no emission:
    they add exactly nothing); the oracle adds their zeros.  Half of all coordinates sit on multiples of 1/16 here,
    i.e. on cell faces of every level whose resolution is a multiple of 16, a tenth of the points are clipped to the
    faces of the cube, some lie on grid vertices: every variant, both directions."""
    w = W.custom(cfg=86 + d, d=d, L=6, N_f=2**13, N_c=2**11, N_p=8, N_min=16, N_max=512, N=60000 + 3,
                 feat_dtype="f16", io_dtype="f16")
    x, D_f, Dhat, dy = tables(w)
    rng = np.random.default_rng(17)
    snap = rng.random(x.shape) < 0.5
    x[snap] = np.round(x[snap] * 16.0) / 16.0
    edge = rng.random(x.shape[0]) < 0.1
    x[edge] = np.round(x[edge])
    assert np.mean(x == np.round(x * 16) / 16) > 0.5
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    check_fwd(w, x, D_f, oracle.bake_probes(Dhat), name="faces")
    check_bwd(w, x, D_f, Dhat, dy, name="faces")

"""GPU parity of the optional Morton reordering: the permutation bit for bit against the oracle's stable
sort, and the forward pass through the permutation bit for bit against the plain forward pass."""
import numpy as np
import pytest
import torch

import oracle
import paper_2312_17241_amd as cngp
import workloads as W
from parity import check_exact

pytestmark = pytest.mark.gpu
DEV = "cuda"


def points(d, N, seed):
    rng = np.random.default_rng(seed)
    x = rng.random((N, d), dtype=np.float32)
    if N >= 16:
        x[0] = 0.0
        x[1] = 1.0
        x[2] = x[3]                       # equal points: the stable order decides
        x[4] = np.float32(1.0) - np.float32(2.0**-24)
        x[5] = -0.25                      # outside the cube: clamped for the code, still a valid row of the batch
        x[6] = 1.5
        x[7, 0] = 0.5                     # exactly on a cell boundary of every resolution
    return x


@pytest.mark.parametrize("d", [2, 3, 4])
@pytest.mark.parametrize("N", [1, 63, 257, 5000, 8192, 8193, 3 * 8192 - 1, 200003])
def test_morton_sort_matches_the_oracle_bit_for_bit(d, N):
    x = points(d, N, seed=100 + d * 7 + N % 11)
    perm_ref, _ = oracle.morton_order(x)
    perm, xs = cngp.morton_sort(torch.from_numpy(x).to(DEV))
    torch.cuda.synchronize()
    check_exact("perm", perm.cpu().numpy(), perm_ref)
    check_exact("x_sorted", xs.cpu().numpy().view(np.uint32), x[perm_ref].view(np.uint32))


def test_morton_sort_of_two_million_points():
    """244 tiles and a ragged last one; every digit's run crosses many tiles."""
    x = points(3, 2_000_003, seed=9)
    perm_ref, _ = oracle.morton_order(x)
    perm, xs = cngp.morton_sort(torch.from_numpy(x).to(DEV))
    check_exact("perm", perm.cpu().numpy(), perm_ref)
    check_exact("x_sorted", xs.cpu().numpy().view(np.uint32), x[perm_ref].view(np.uint32))


def test_morton_sort_at_the_inference_batch_size():
    """2^24 uniformly random points (the forward-only workload's batch): 2048 full tiles, every count near 2^17."""
    rng = np.random.default_rng(77)
    x = rng.random((2**24, 3), dtype=np.float32)
    perm_ref, _ = oracle.morton_order(x)
    perm, xs = cngp.morton_sort(torch.from_numpy(x).to(DEV))
    check_exact("perm", perm.cpu().numpy(), perm_ref)
    check_exact("x_sorted", xs.cpu().numpy().view(np.uint32), x[perm_ref].view(np.uint32))


def test_morton_sort_twice_in_one_workspace():
    """The second call finds the first call's counters and keys in the workspace and must not depend on them."""
    xa, xb = points(3, 50_000, seed=21), points(3, 20_001, seed=22)
    ws = torch.empty(int(cngp._lib.cngp_morton_sort_workspace_bytes(3, 50_000)), dtype=torch.uint8, device=DEV)
    for x in (xa, xb, xa):
        perm, _ = cngp.morton_sort(torch.from_numpy(x).to(DEV), workspace=ws)
        check_exact("perm", perm.cpu().numpy(), oracle.morton_order(x)[0])


def test_morton_sort_of_a_clustered_batch():
    """Many equal codes (all points in a few cells): the order inside a cell is the order of the batch."""
    rng = np.random.default_rng(3)
    x = (0.5 + 1e-4 * rng.standard_normal((30000, 3))).astype(np.float32)
    perm_ref, codes = oracle.morton_order(x)
    assert len(np.unique(codes)) < 30
    perm, _ = cngp.morton_sort(torch.from_numpy(x).to(DEV))
    check_exact("perm", perm.cpu().numpy(), perm_ref)


@pytest.mark.parametrize("d,N_p,feat,io,fmt,flags", [
    (3, 16, "f16", "f16", cngp.IDX_PACKED4, 0), (3, 8, "f16", "f16", cngp.IDX_BITS, 0), (2, 4, "f32", "f32", cngp.IDX_U8, 0),
    (2, 8, "f16", "f32", cngp.IDX_U8, cngp.FWD_SIMPLE), (3, 1, "f32", "f16", cngp.IDX_U8, 0), (3, 16, "f16", "f16", cngp.IDX_U8, cngp.FWD_SIMPLE)])
def test_forward_through_the_permutation_equals_the_plain_forward(d, N_p, feat, io, fmt, flags):
    w = W.custom(cfg=70 + d, d=d, L=5, N_f=2**11, N_c=2**9, N_p=N_p, N_min=4, N_max=300, N=20000 + 13, feat_dtype=feat, io_dtype=io)
    cfg = cngp.Config.from_workload(w, index_format=fmt, flags=flags)
    x = torch.from_numpy(W.make_points(w)).to(DEV)
    D_f = torch.from_numpy(W.make_feature_codebook(w)).to(DEV)
    D_c = cngp.bake_probes(cfg, torch.from_numpy(W.make_probe_logits(w)).to(DEV))
    y = cngp.encode_fwd(cfg, x, D_f, D_c)
    perm, xs = cngp.morton_sort(x)
    y2 = torch.full_like(y, float("nan"))
    cngp.encode_fwd_permuted(cfg, xs, perm, D_f, D_c, y2)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16 if io == "f16" else torch.int32), y2.view(torch.int16 if io == "f16" else torch.int32))
    if not flags:                                   # with room for the level-major copy: the level-resident variant, same bits
        y3 = torch.full_like(y, float("nan"))
        ws = cngp.alloc_workspace(cfg, w.N)
        assert cngp.fwd_plan_info(cfg, w.N)["level_resident"] == 1 and ws is not None
        cngp.encode_fwd_permuted(cfg, xs, perm, D_f, D_c, y3, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(y2, y3)
    y_ref, ymag = oracle.encode_fwd(w, W.make_points(w), W.make_feature_codebook(w), oracle.bake_probes(W.make_probe_logits(w)))
    from parity import check_close
    check_close("y through the permutation", y2.cpu().numpy(), y_ref, ymag, fp16_out=(io == "f16"))


def test_large_tile_forward_through_the_permutation():
    w = W.custom(cfg=75, d=3, L=4, N_f=2**12, N_c=2**15, N_p=8, N_min=16, N_max=256, N=2**20 + 77, feat_dtype="f16", io_dtype="f16")
    cfg = cngp.Config.from_workload(w, index_format=cngp.IDX_PACKED4)
    x = torch.from_numpy(W.make_points(w)).to(DEV)
    D_f = torch.from_numpy(W.make_feature_codebook(w)).to(DEV)
    D_c = cngp.bake_probes(cfg, torch.from_numpy(W.make_probe_logits(w)).to(DEV))
    y = cngp.encode_fwd(cfg, x, D_f, D_c)
    perm, xs = cngp.morton_sort(x)
    check_exact("perm", perm.cpu().numpy(), oracle.morton_order(W.make_points(w))[0])
    y2 = cngp.encode_fwd_permuted(cfg, xs, perm, D_f, D_c)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))


def test_sort_argument_errors():
    x = torch.rand((100, 3), device=DEV)
    perm = torch.empty(100, dtype=torch.int32, device=DEV)
    lib = cngp._lib
    import ctypes
    assert lib.cngp_morton_sort(5, x.data_ptr(), 100, perm.data_ptr(), None, None, 0, None) == cngp.ERR_INVALID
    assert lib.cngp_morton_sort(3, x.data_ptr(), 100, None, None, None, 0, None) == cngp.ERR_NULL
    assert lib.cngp_morton_sort(3, x.data_ptr(), 100, perm.data_ptr(), None, None, 0, None) == cngp.ERR_WORKSPACE
    assert lib.cngp_morton_sort(3, x.data_ptr(), 0, None, None, None, 0, None) == cngp.OK
    assert lib.cngp_morton_sort_workspace_bytes(3, 100) > 1200 and lib.cngp_morton_sort_workspace_bytes(5, 100) == 0

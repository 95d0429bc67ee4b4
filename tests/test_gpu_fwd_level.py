"""The level-resident forward variant (a workgroup keeps one level's index codebook and the head of its feature
codebook in LDS and streams the points; encodings leave level-major and a second kernel turns them into rows):
against the oracle, and bit for bit against the tile variant, whose arithmetic it repeats (Eq. 6, Fig. 3)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2312_17241_amd as cngp
import workloads as W
from parity import check_close

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def packed(fmt, D_c, N_p):
    return {cngp.IDX_U8: lambda: dev(D_c), cngp.IDX_PACKED4: lambda: cngp.pack4(dev(D_c)),
            cngp.IDX_BITS: lambda: dev(oracle.pack_index_bits(D_c, N_p))}[fmt]()


def case(d, N_p, feat, io, N, **kw):
    base = dict(cfg=30 + d + N_p, d=d, L=6, F=2, N_f=2**16, N_c=2**10, N_p=N_p, N_min=4, N_max=512, N=N,
                feat_dtype=feat, io_dtype=io)
    base.update(kw)
    w = W.custom(**base)
    x = W.make_points(w)
    k = min(3, N)
    x[:k] = [[0.0] * d, [1.0] * d, [0.5] * d][:k]
    D_f = W.make_feature_codebook(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    return w, x, D_f, oracle.bake_probes(W.make_probe_logits(w))


def both_variants(w, x, D_f, D_c, fmt, levels_loaded=None):
    ys = []
    for flags in (cngp.FWD_LEVEL, cngp.FWD_TILE):
        cfg = cngp.Config.from_workload(w, flags=flags, index_format=fmt)
        ws = cngp.alloc_workspace(cngp.Config.from_workload(w, flags=cngp.FWD_LEVEL, index_format=fmt), w.N)
        args = (dev(x), dev(D_f), packed(fmt, D_c, w.N_p))
        y = (cngp.encode_fwd(cfg, *args, workspace=ws) if levels_loaded is None
             else cngp.encode_fwd_partial(cfg, levels_loaded, *args, workspace=ws))
        torch.cuda.synchronize()
        ys.append(y)
    return ys


# the feature codebook of a level (N_f = 2^16): 256 KB in fp16 (more than half resident), 512 KB in fp32 (a quarter)
@pytest.mark.parametrize("d,N_p,feat,io", [(2, 1, "f32", "f32"), (2, 8, "f16", "f16"), (3, 4, "f32", "f16"),
                                           (3, 16, "f16", "f16"), (3, 16, "f16", "f32"), (4, 2, "f16", "f16")])
@pytest.mark.parametrize("fmt", [cngp.IDX_U8, cngp.IDX_PACKED4, cngp.IDX_BITS])
def test_level_resident_forward_sweep(d, N_p, feat, io, fmt):
    w, x, D_f, D_c = case(d, N_p, feat, io, N=5000 + 77)
    cfg = cngp.Config.from_workload(w, flags=cngp.FWD_LEVEL, index_format=fmt)
    assert cngp.fwd_workspace_bytes(cfg, w.N) == w.N * w.L * 2 * (2 if io == "f16" else 4)
    y_level, y_tile = both_variants(w, x, D_f, D_c, fmt)
    y_ref, ymag = oracle.encode_fwd(w, x, D_f, D_c)
    check_close("y [level-resident]", y_level.cpu().numpy(), y_ref, ymag, fp16_out=(io == "f16"))
    assert torch.equal(y_level, y_tile)


@pytest.mark.parametrize("N", [1, 63, 1023, 1024, 2049, 4096 + 1])
def test_ragged_batches(N):
    w, x, D_f, D_c = case(3, 8, "f16", "f16", N=N, L=4)
    y_level, y_tile = both_variants(w, x, D_f, D_c, cngp.IDX_PACKED4)
    y_ref, ymag = oracle.encode_fwd(w, x, D_f, D_c)
    check_close("y [level-resident]", y_level.cpu().numpy(), y_ref, ymag, fp16_out=True)
    assert torch.equal(y_level, y_tile)


def test_whole_feature_codebook_resident_and_levels_not_loaded():
    w, x, D_f, D_c = case(3, 4, "f16", "f16", N=30000 + 9, N_f=2**12, L=7)
    y_ref, ymag = oracle.encode_fwd(w, x, D_f, D_c)
    y_level, y_tile = both_variants(w, x, D_f, D_c, cngp.IDX_U8)
    check_close("y [level-resident]", y_level.cpu().numpy(), y_ref, ymag, fp16_out=True)
    assert torch.equal(y_level, y_tile)
    p_level, p_tile = both_variants(w, x, D_f, D_c, cngp.IDX_U8, levels_loaded=3)
    assert torch.equal(p_level, p_tile)
    assert torch.equal(p_level[:, :6], y_level[:, :6]) and bool((p_level[:, 6:] == 0).all())


def test_library_takes_it_by_itself_for_a_large_batch():
    """2^17 points on 16 levels: the level-resident variant is the library's own choice when the workspace is there,
    the tile variant without it; same encodings."""
    w, x, D_f, D_c = case(3, 16, "f16", "f16", N=2**17 + 5, L=16, N_c=2**14, N_max=2048)
    cfg = cngp.Config.from_workload(w)
    need = cngp.fwd_workspace_bytes(cfg, w.N)
    assert need == w.N * 16 * 2 * 2 and cngp.workspace_bytes(cfg, w.N) >= need
    cngp.profile_enable(True)
    cngp.profile_read()
    y_ws = cngp.encode_fwd(cfg, dev(x), dev(D_f), dev(D_c), workspace=cngp.alloc_workspace(cfg, w.N))
    torch.cuda.synchronize()
    names = cngp.profile_read()
    cngp.profile_enable(False)
    assert "encode_fwd_rows" in names, names
    y_plain = cngp.encode_fwd(cfg, dev(x), dev(D_f), dev(D_c))
    torch.cuda.synchronize()
    assert torch.equal(y_ws, y_plain)
    sample = np.random.default_rng(1).choice(w.N, 4000, replace=False)
    y_ref, ymag = oracle.encode_fwd(w, x[sample], D_f, D_c)
    check_close("y [sample]", y_ws[torch.from_numpy(sample).to(DEV)].cpu().numpy(), y_ref, ymag, fp16_out=True)


def test_wider_features_pass_through_it():
    w, x, D_f, D_c = case(3, 8, "f16", "f16", N=6000 + 1, F=4, L=4)
    cfg = cngp.Config.from_workload(w, flags=cngp.FWD_LEVEL)
    y = cngp.encode_fwd(cfg, dev(x), dev(D_f), dev(D_c), workspace=cngp.alloc_workspace(cfg, w.N))
    torch.cuda.synchronize()
    y_ref, ymag = oracle.encode_fwd(w, x, D_f, D_c)
    check_close("y F=4 [level-resident]", y.cpu().numpy(), y_ref, ymag, fp16_out=True)


def test_forced_where_it_cannot_run_is_an_error():
    w, x, D_f, D_c = case(3, 8, "f16", "f16", N=3000)
    cfg = cngp.Config.from_workload(w, flags=cngp.FWD_LEVEL)
    with pytest.raises(cngp.CngpError) as e:                              # no room for the level-major copy
        cngp.encode_fwd(cfg, dev(x), dev(D_f), dev(D_c))
    assert e.value.status == cngp.ERR_WORKSPACE
    w2, x2, D_f2, D_c2 = case(3, 8, "f16", "f16", N=3000, N_c=2**18, L=2)   # index codebook beyond the LDS share
    cfg2 = cngp.Config.from_workload(w2, flags=cngp.FWD_LEVEL)
    assert cngp.fwd_workspace_bytes(cfg2, w2.N) == 0
    with pytest.raises(cngp.CngpError) as e:
        cngp.encode_fwd(cfg2, dev(x2), dev(D_f2), dev(D_c2), workspace=torch.empty(1 << 20, dtype=torch.uint8, device=DEV))
    assert e.value.status == cngp.ERR_UNSUPPORTED
    bad = cngp.Config.from_workload(w, flags=cngp.FWD_LEVEL | cngp.FWD_TILE)
    with pytest.raises(cngp.CngpError) as e:
        cngp.encode_fwd(bad, dev(x), dev(D_f), dev(D_c))
    assert e.value.status == cngp.ERR_INVALID

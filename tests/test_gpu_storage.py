"""GPU parity of the exact-width index codebook (log2(N_p) bits per entry, the storage the model sizes of
Tables 3 and 4 imply): baked straight into that layout, and read from it by the forward pass and the index
dump.  Everything here is integer or a re-read of the same values, so the bars are bit-exact: the packed
bytes against the oracle's packing of the oracle's bake, and the forward output against the forward output
of the byte-per-entry codebook (which the other parity tests hold against the oracle)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2312_17241_amd as cngp
import workloads as W
from parity import check_close, check_exact

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


@pytest.mark.parametrize("N_p", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("N_c", [1, 2, 4, 8, 16, 32, 2048, 65536])
def test_bake_into_exact_width(N_p, N_c):
    w = W.custom(d=3, L=3, N_f=4096, N_c=N_c, N_p=N_p, N_min=4, N_max=64, N=16)
    rng = np.random.default_rng(N_p * 7 + N_c)
    Dhat = rng.standard_normal((w.L, w.N_c, w.N_p)).astype(np.float32)
    Dhat[0, 0] = np.nan
    cfg = cngp.Config.from_workload(w, index_format=cngp.IDX_BITS)
    want = oracle.pack_index_bits(oracle.bake_probes(Dhat), N_p)
    assert cfg.index_cols == want.shape[1]
    out = torch.full((w.L, cfg.index_cols), 0xEE, dtype=torch.uint8, device=DEV)
    cngp.bake_probes(cfg, dev(Dhat), out)
    torch.cuda.synchronize()
    check_exact("packed D_c", out.cpu().numpy(), want)
    check_exact("torch-side packing", cngp.pack_bits(dev(oracle.bake_probes(Dhat)), N_p).cpu().numpy(), want)


CASES = [dict(d=3, L=4, N_f=2**10, N_c=2**9, N_p=8, N_min=4, N_max=64, N=5000 + 13),
         dict(d=2, L=5, N_f=2**8, N_c=2**12, N_p=2, N_min=8, N_max=300, N=4000 + 1),
         dict(d=3, L=3, N_f=2**6, N_c=4, N_p=8, N_min=4, N_max=32, N=700),
         dict(d=2, L=2, N_f=2**6, N_c=1, N_p=4, N_min=4, N_max=32, N=300),
         dict(d=3, L=3, N_f=2**8, N_c=2**7, N_p=1, N_min=4, N_max=32, N=1000),
         dict(d=3, L=2, N_f=2**12, N_c=2**18, N_p=8, N_min=16, N_max=64, N=3000),      # too large for LDS staging
         dict(d=3, L=16, N_f=2**8, N_c=2**16, N_p=8, N_min=16, N_max=2048, N=20000, feat_dtype="f16", io_dtype="f16")]


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"d{c['d']}_Nc{c['N_c']}_Np{c['N_p']}")
def test_forward_and_indices_from_exact_width(case):
    """The last case is the configuration of the paper's Table 3 row (N_f = 2^8, N_c = 2^16, N_p = 2^3)."""
    w = W.custom(**case)
    x = W.make_points(w)
    D_f = W.make_feature_codebook(w)
    D_c = oracle.bake_probes(W.make_probe_logits(w))
    packed = dev(oracle.pack_index_bits(D_c, w.N_p))
    y_ref, ymag = oracle.encode_fwd(w, x, D_f, D_c)
    for flags in (0, cngp.FWD_SIMPLE):
        cfg_b = cngp.Config.from_workload(w, index_format=cngp.IDX_BITS, flags=flags)
        cfg_u = cngp.Config.from_workload(w, index_format=cngp.IDX_U8, flags=flags)
        y_b = cngp.encode_fwd(cfg_b, dev(x), dev(D_f), packed)
        y_u = cngp.encode_fwd(cfg_u, dev(x), dev(D_f), dev(D_c))
        torch.cuda.synchronize()
        assert torch.equal(y_b, y_u)
        check_close("y", y_b.float().cpu().numpy(), y_ref, ymag, fp16_out=(w.io_dtype == "f16"))
    got = cngp.debug_indices(cngp.Config.from_workload(w, index_format=cngp.IDX_BITS), dev(x), packed)
    want = oracle.indices(w, x, D_c)
    for nm, g, r in zip(("base", "h2", "probe", "feat_idx"), got, want):
        check_exact(nm, g.cpu().numpy().view(r.dtype), r)


def test_exact_width_is_refused_where_it_is_not_supported():
    w = W.custom(d=3, L=2, N_f=256, N_c=64, N_p=8, N_min=4, N_max=32, N=16)
    cfg = cngp.Config.from_workload(w, index_format=cngp.IDX_BITS)
    z = lambda *s: torch.zeros(s, device=DEV)
    with pytest.raises(cngp.CngpError) as e:
        cngp.adam_step_bake(cfg, None, cngp.Adam(), None,
                            (z(2, 64, 8), z(2, 64, 8), z(2, 64, 8), z(2, 64, 8),
                             torch.zeros((2, cfg.index_cols), dtype=torch.uint8, device=DEV)))
    assert e.value.status == cngp.ERR_UNSUPPORTED


@pytest.mark.parametrize("fmt", [cngp.IDX_U8, cngp.IDX_PACKED4, cngp.IDX_BITS])
def test_large_tile_forward(fmt):
    """More than 2^20 points with an index codebook of 2^16 entries per level: the forward pass takes its
    large-tile variant.  Ragged last tile; every output equals the variant that reads D_c from memory, and a
    sample is held against the oracle."""
    w = W.WORKLOADS["compact3d"]
    n = 2**20 + 1024 + 77
    x = W.make_points(w, n)
    D_f = W.make_feature_codebook(w)
    D_c = oracle.bake_probes(W.make_probe_logits(w))
    D_c_dev = {cngp.IDX_U8: dev(D_c), cngp.IDX_PACKED4: cngp.pack4(dev(D_c)),
               cngp.IDX_BITS: dev(oracle.pack_index_bits(D_c, w.N_p))}[fmt]
    y = cngp.encode_fwd(cngp.Config.from_workload(w, index_format=fmt), dev(x), dev(D_f), D_c_dev)
    y_simple = cngp.encode_fwd(cngp.Config.from_workload(w, index_format=fmt, flags=cngp.FWD_SIMPLE), dev(x), dev(D_f), D_c_dev)
    cfg = cngp.Config.from_workload(w, index_format=fmt)
    y_level = cngp.encode_fwd(cfg, dev(x), dev(D_f), D_c_dev, workspace=cngp.alloc_workspace(cfg, n))   # level-resident
    torch.cuda.synchronize()
    assert torch.equal(y, y_simple) and torch.equal(y, y_level)
    assert cngp.fwd_plan_info(cfg, n)["resident_entries"] == w.N_f       # the whole feature codebook of a level in LDS
    pick = np.r_[0:4096, n - 4096:n]
    y_ref, ymag = oracle.encode_fwd(w, x[pick], D_f, D_c)
    check_close("y", y.float().cpu().numpy()[pick], y_ref, ymag, fp16_out=True)


@pytest.mark.parametrize("levels", [0, 1, 5, 11, 12])
@pytest.mark.parametrize("flags", [0, cngp.FWD_SIMPLE])
def test_forward_from_a_partially_loaded_model(levels, flags):
    """Level-of-detail streaming: only the first levels are read (the rest of the arrays is poisoned with
    NaN features and out-of-range indices here), the other columns are zero."""
    w = W.custom(cfg=97, d=3, L=12, N_f=2**11, N_c=2**10, N_p=8, N_min=8, N_max=1024, N=2000 + 9, feat_dtype="f16", io_dtype="f16")
    x = W.make_points(w)
    D_f = W.make_feature_codebook(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    D_c = oracle.bake_probes(W.make_probe_logits(w))
    y_ref, ymag = oracle.encode_fwd_partial(w, levels, x, D_f, D_c)
    if levels == w.L:
        full, _ = oracle.encode_fwd(w, x, D_f, D_c)
        assert np.array_equal(full, y_ref)
    D_f_p, D_c_p = D_f.copy(), D_c.copy()
    D_f_p[levels:] = np.nan
    D_c_p[levels:] = 255
    cfg = cngp.Config.from_workload(w, flags=flags)
    y = cngp.encode_fwd_partial(cfg, levels, dev(x), dev(D_f_p), dev(D_c_p))
    torch.cuda.synchronize()
    got = y.float().cpu().numpy()
    check_close("y", got, y_ref, ymag, fp16_out=True)
    assert not got[:, levels * w.F:].any()

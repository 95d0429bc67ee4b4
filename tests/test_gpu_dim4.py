"""A four-dimensional input domain (e.g. space and time; the paper's experiments have d = 2 and 3, Table 1, and
Sec. 5 expects the method to carry over): every entry point that takes d = 4 against the oracle, whose loops run
over d directly.  16 corners per cell; the fourth prime of each hash is this build's choice."""
import numpy as np
import pytest
import torch

import oracle
import paper_2312_17241_amd as cngp
import workloads as W
from parity import check_close, check_exact

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t if dtype is None else t.to(dtype)


def case(N_p, feat, io, N=3000 + 77, **kw):
    base = dict(cfg=40 + N_p, d=4, L=5, F=2, N_f=2**11, N_c=2**9, N_p=N_p, N_min=4, N_max=96, N=N,
                feat_dtype=feat, io_dtype=io)
    base.update(kw)
    w = W.custom(**base)
    x = W.make_points(w)
    x[:4] = [[0.0] * 4, [1.0] * 4, [0.5] * 4, [1.0, 0.0, 0.0, 1.0]]
    D_f = W.make_feature_codebook(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    return w, x, D_f, W.make_probe_logits(w), W.make_upstream_grad(w)


def packed(fmt, D_c, N_p):
    return {cngp.IDX_U8: lambda: dev(D_c), cngp.IDX_PACKED4: lambda: cngp.pack4(dev(D_c)),
            cngp.IDX_BITS: lambda: dev(oracle.pack_index_bits(D_c, N_p))}[fmt]()


SWEEP = [(1, "f32", "f32"), (2, "f16", "f32"), (4, "f32", "f16"), (8, "f16", "f16"), (16, "f16", "f16"), (16, "f32", "f32")]


@pytest.mark.parametrize("fmt", [cngp.IDX_U8, cngp.IDX_PACKED4, cngp.IDX_BITS])
def test_indices_bit_exact(fmt):
    w, x, _, Dhat, _ = case(8, "f32", "f32", L=8, N_max=4096)
    D_c = oracle.bake_probes(Dhat)
    cfg = cngp.Config.from_workload(w, index_format=fmt)
    got = cngp.debug_indices(cfg, dev(x), packed(fmt, D_c, w.N_p))
    torch.cuda.synchronize()
    want = oracle.indices(w, x, D_c)
    assert want[0].shape == (w.N, w.L, 16)
    for nm, g, r in zip(("base", "h2", "probe", "feat_idx"), got, want):
        check_exact(nm, g.cpu().numpy().view(r.dtype), r)


@pytest.mark.parametrize("N_p,feat,io", SWEEP)
def test_forward(N_p, feat, io):
    w, x, D_f, Dhat, _ = case(N_p, feat, io)
    D_c = oracle.bake_probes(Dhat)
    y_ref, ymag = oracle.encode_fwd(w, x, D_f, D_c)
    for flags in (0, cngp.FWD_SIMPLE):
        for fmt in (cngp.IDX_U8, cngp.IDX_BITS):
            cfg = cngp.Config.from_workload(w, flags=flags, index_format=fmt)
            y = cngp.encode_fwd(cfg, dev(x), dev(D_f), packed(fmt, D_c, N_p))
            torch.cuda.synchronize()
            check_close("y d=4", y.cpu().numpy(), y_ref, ymag, fp16_out=(io == "f16"))
    cfg = cngp.Config.from_workload(w)
    yp = cngp.encode_fwd_partial(cfg, 3, dev(x), dev(D_f), dev(D_c))
    torch.cuda.synchronize()
    yp = yp.cpu().numpy().astype(np.float64)
    assert np.all(yp[:, 6:] == 0.0)
    check_close("y partial d=4", yp[:, :6], y_ref[:, :6], ymag[:, :6], fp16_out=(io == "f16"))


@pytest.mark.parametrize("N_p,feat,io", SWEEP)
def test_backward_every_variant(N_p, feat, io):
    w, x, D_f, Dhat, dy = case(N_p, feat, io)
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    variants = (("auto", 0), ("direct", cngp.BWD_DIRECT), ("sliced", cngp.BWD_SLICED), ("binned", cngp.BWD_BINNED),
                ("sliced, no pre-reduction", cngp.BWD_SLICED | cngp.BWD_NO_PREREDUCE),
                ("binned, no pre-reduction", cngp.BWD_BINNED | cngp.BWD_NO_PREREDUCE))
    for name, flags in variants:
        cfg = cngp.Config.from_workload(w, flags=cngp.ZERO_GRADS | flags)
        gF = torch.full((w.L, w.N_f, 2), float("nan"), device=DEV)
        gC = torch.full((w.L, w.N_c, w.N_p), float("nan"), device=DEV)
        cngp.encode_bwd(cfg, dev(x), dev(D_f), dev(Dhat), dev(dy), gF, gC, workspace=cngp.alloc_workspace(cfg, w.N))
        torch.cuda.synchronize()
        check_close(f"grad D_f d=4 [{name}]", gF.cpu().numpy(), gF_ref, A_f, fp16_out=False)
        check_close(f"grad Dhat_c d=4 [{name}]", gC.cpu().numpy(), gC_ref, A_c, fp16_out=False)


def test_backward_larger_batch_in_passes_and_static_scratch():
    """A batch at which the LDS variants are the library's own choice and the coarse levels are pre-reduced per
    vertex; then in several passes under a bound on the bin memory; then out of the static scratch array."""
    w, x, D_f, Dhat, dy = case(8, "f16", "f16", N=50000 + 5, L=4, N_f=2**13, N_c=2**11, N_max=48)
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    info = cngp.bwd_plan_info(cngp.Config.from_workload(w), w.N)
    assert info["sliced"] == 1 and info["dense_levels"] >= 1, info
    for over in (dict(), dict(flags=cngp.ZERO_GRADS | cngp.BWD_BINNED, bin_bytes_max=8 << 20)):
        cfg = cngp.Config.from_workload(w, **{"flags": cngp.ZERO_GRADS, **over})
        gF = torch.full((w.L, w.N_f, 2), float("nan"), device=DEV)
        gC = torch.full((w.L, w.N_c, w.N_p), float("nan"), device=DEV)
        cngp.encode_bwd(cfg, dev(x), dev(D_f), dev(Dhat), dev(dy), gF, gC, workspace=cngp.alloc_workspace(cfg, w.N))
        torch.cuda.synchronize()
        check_close("grad D_f d=4", gF.cpu().numpy(), gF_ref, A_f, fp16_out=False)
        check_close("grad Dhat_c d=4", gC.cpu().numpy(), gC_ref, A_c, fp16_out=False)
    cfg = cngp.Config.from_workload(w, flags=cngp.ZERO_GRADS)
    gF.fill_(float("nan")); gC.fill_(float("nan"))
    cngp.encode_bwd_static(cfg, dev(x), dev(D_f), dev(Dhat), dev(dy), gF, gC)
    torch.cuda.synchronize()
    check_close("grad D_f d=4 [static]", gF.cpu().numpy(), gF_ref, A_f, fp16_out=False)
    check_close("grad Dhat_c d=4 [static]", gC.cpu().numpy(), gC_ref, A_c, fp16_out=False)


@pytest.mark.parametrize("N_p,feat,io", [(1, "f32", "f32"), (8, "f16", "f16"), (16, "f32", "f16")])
def test_input_gradient(N_p, feat, io):
    w, x, D_f, Dhat, dy = case(N_p, feat, io)
    D_c = oracle.bake_probes(Dhat)
    ref, mag = oracle.encode_bwd_input(w, x, D_f, D_c, dy)
    for fmt in (cngp.IDX_U8, cngp.IDX_PACKED4):
        cfg = cngp.Config.from_workload(w, index_format=fmt)
        gx = torch.full((w.N, 4), float("nan"), device=DEV)
        cngp.encode_bwd_input(cfg, dev(x), dev(D_f), packed(fmt, D_c, N_p), dev(dy), gx)
        torch.cuda.synchronize()
        check_close("dL/dx d=4", gx.cpu().numpy(), ref, mag, fp16_out=False)


def test_fused_encode_and_decoder():
    from test_gpu_mlp import check
    w, x, D_f, Dhat, _ = case(8, "f16", "f16", N=5000 + 9, L=8, N_f=2**12, N_c=2**12, N_max=256)
    D_c = oracle.bake_probes(Dhat)
    rng = np.random.default_rng(5)
    he = lambda rows, cols: (rng.standard_normal((rows, cols)) * np.sqrt(2.0 / cols)).astype(np.float16).astype(np.float64)
    W1, W2, W3 = he(64, 2 * w.L), he(64, 64), he(4, 64)
    Wd = dev(np.concatenate([W1.ravel(), W2.ravel(), W3.ravel()]), torch.float16)
    cfg = cngp.Config.from_workload(w)
    mcfg = cngp.MlpConfig(2 * w.L, 4, cngp.F16)
    fused = cngp.encode_mlp_fwd(cfg, mcfg, dev(x), dev(D_f), dev(D_c), Wd)
    two = cngp.mlp_fwd(mcfg, cngp.encode_fwd(cfg, dev(x), dev(D_f), dev(D_c)), Wd)
    torch.cuda.synchronize()
    assert torch.equal(fused, two)
    y_ref, _ = oracle.encode_fwd(w, x, D_f, D_c)
    ref, mag, _ = oracle.mlp_fwd(y_ref, W1, W2, W3, want_mag=True)
    check("decoder(encode(x)) d=4", fused.cpu().numpy(), ref, mag)


def test_morton_sort_is_for_two_to_four_dimensions():
    x = torch.rand((1000, 5), device=DEV)
    with pytest.raises(cngp.CngpError) as e:
        cngp.morton_sort(x)
    assert e.value.status == cngp.ERR_INVALID

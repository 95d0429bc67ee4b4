"""Feature widths other than the paper's F = 2 (Table 1 fixes F = 2; Sec. 5 expects the method to carry over to other
settings): F = 1, 4, 8 against the oracle, which loops over the features of an entry directly.  The library takes them
two features at a time with the kernels of F = 2 (the interpolation and the feature gradient act per feature, the
logit gradient is a sum over the features)."""
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


def case(F, d, N_p, feat, io, N=3000 + 77, **kw):
    base = dict(cfg=60 + F * 7 + d, d=d, L=5, F=F, N_f=2**11, N_c=2**9, N_p=N_p, N_min=4, N_max=300, N=N,
                feat_dtype=feat, io_dtype=io)
    base.update(kw)
    w = W.custom(**base)
    x = W.make_points(w)
    x[:3] = [[0.0] * d, [1.0] * d, [0.5] * d]
    D_f = W.make_feature_codebook(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    return w, x, D_f, W.make_probe_logits(w), W.make_upstream_grad(w)


SWEEP = [(1, 2, 4, "f32", "f32"), (1, 3, 16, "f16", "f16"), (4, 2, 8, "f16", "f32"), (4, 3, 16, "f16", "f16"),
         (4, 3, 1, "f32", "f32"), (8, 3, 2, "f32", "f16"), (8, 2, 16, "f16", "f16")]


@pytest.mark.parametrize("F,d,N_p,feat,io", SWEEP)
def test_forward(F, d, N_p, feat, io):
    w, x, D_f, Dhat, _ = case(F, d, N_p, feat, io)
    D_c = oracle.bake_probes(Dhat)
    y_ref, ymag = oracle.encode_fwd(w, x, D_f, D_c)
    for flags in (0, cngp.FWD_SIMPLE):
        cfg = cngp.Config.from_workload(w, flags=flags)
        ws = cngp.alloc_workspace(cfg, w.N)
        assert ws is not None                                  # the pair planes live there
        y = cngp.encode_fwd(cfg, dev(x), dev(D_f), dev(D_c), workspace=ws)
        torch.cuda.synchronize()
        assert y.shape == (w.N, w.L * F)
        check_close(f"y F={F}", y.cpu().numpy(), y_ref, ymag, fp16_out=(io == "f16"))
    # partial loading: the columns of the levels that are not loaded are zero, the others unchanged
    cfg = cngp.Config.from_workload(w)
    yp = cngp.encode_fwd_partial(cfg, 2, dev(x), dev(D_f), dev(D_c), workspace=cngp.alloc_workspace(cfg, w.N))
    torch.cuda.synchronize()
    yp = yp.cpu().numpy().astype(np.float64)
    assert np.all(yp[:, 2 * F:] == 0.0)
    check_close("y partial", yp[:, :2 * F], y_ref[:, :2 * F], ymag[:, :2 * F], fp16_out=(io == "f16"))
    # without a workspace the call is refused, not run
    with pytest.raises(cngp.CngpError) as e:
        cngp.encode_fwd(cfg, dev(x), dev(D_f), dev(D_c))
    assert e.value.status == cngp.ERR_WORKSPACE


@pytest.mark.parametrize("F,d,N_p,feat,io", SWEEP)
def test_backward_every_variant(F, d, N_p, feat, io):
    w, x, D_f, Dhat, dy = case(F, d, N_p, feat, io)
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    for name, flags in (("auto", 0), ("direct", cngp.BWD_DIRECT), ("sliced", cngp.BWD_SLICED), ("binned", cngp.BWD_BINNED)):
        cfg = cngp.Config.from_workload(w, flags=cngp.ZERO_GRADS | flags)
        gF = torch.full((w.L, w.N_f, F), float("nan"), device=DEV)
        gC = torch.full((w.L, w.N_c, w.N_p), float("nan"), device=DEV)
        cngp.encode_bwd(cfg, dev(x), dev(D_f), dev(Dhat), dev(dy), gF, gC, workspace=cngp.alloc_workspace(cfg, w.N))
        torch.cuda.synchronize()
        check_close(f"grad D_f F={F} [{name}]", gF.cpu().numpy(), gF_ref, A_f, fp16_out=False)
        check_close(f"grad Dhat_c F={F} [{name}]", gC.cpu().numpy(), gC_ref, A_c, fp16_out=False)
    # without the flag both gradients accumulate onto what is there
    cfg = cngp.Config.from_workload(w)
    gF = torch.full((w.L, w.N_f, F), 1.5, device=DEV)
    gC = torch.full((w.L, w.N_c, w.N_p), -0.5, device=DEV)
    cngp.encode_bwd(cfg, dev(x), dev(D_f), dev(Dhat), dev(dy), gF, gC, workspace=cngp.alloc_workspace(cfg, w.N))
    torch.cuda.synchronize()
    check_close("grad D_f (+=)", gF.cpu().numpy(), gF_ref + 1.5, A_f + 1.5, fp16_out=False)
    check_close("grad Dhat_c (+=)", gC.cpu().numpy(), gC_ref - 0.5, A_c + 0.5, fp16_out=False)


def test_wide_features_on_a_larger_batch_and_the_static_scratch():
    """F = 4 through the LDS variants at a size where they are the library's own choice, in passes, and through the
    allocation-free entry point."""
    w, x, D_f, Dhat, dy = case(4, 3, 8, "f16", "f16", N=60000 + 5, L=4, N_f=2**13, N_c=2**11, N_max=128)
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    for over in (dict(), dict(flags=cngp.ZERO_GRADS | cngp.BWD_BINNED, bin_bytes_max=8 << 20)):
        cfg = cngp.Config.from_workload(w, **{"flags": cngp.ZERO_GRADS, **over})
        gF = torch.full((w.L, w.N_f, 4), float("nan"), device=DEV)
        gC = torch.full((w.L, w.N_c, w.N_p), float("nan"), device=DEV)
        cngp.encode_bwd(cfg, dev(x), dev(D_f), dev(Dhat), dev(dy), gF, gC, workspace=cngp.alloc_workspace(cfg, w.N))
        torch.cuda.synchronize()
        check_close("grad D_f", gF.cpu().numpy(), gF_ref, A_f, fp16_out=False)
        check_close("grad Dhat_c", gC.cpu().numpy(), gC_ref, A_c, fp16_out=False)
    cfg = cngp.Config.from_workload(w, flags=cngp.ZERO_GRADS)
    gF.fill_(float("nan")); gC.fill_(float("nan"))
    cngp.encode_bwd_static(cfg, dev(x), dev(D_f), dev(Dhat), dev(dy), gF, gC)
    torch.cuda.synchronize()
    check_close("grad D_f [static]", gF.cpu().numpy(), gF_ref, A_f, fp16_out=False)
    check_close("grad Dhat_c [static]", gC.cpu().numpy(), gC_ref, A_c, fp16_out=False)


def test_entry_points_without_room_for_the_planes_say_so():
    w, x, D_f, Dhat, dy = case(4, 3, 4, "f32", "f32", N=100)
    cfg = cngp.Config.from_workload(w)
    D_c = oracle.bake_probes(Dhat)
    with pytest.raises(cngp.CngpError) as e:
        cngp.encode_bwd_input(cfg, dev(x), dev(D_f), dev(D_c), dev(dy))
    assert e.value.status == cngp.ERR_UNSUPPORTED
    bad = cngp.Config.from_workload(W.custom(F=3))
    assert cngp.workspace_bytes(bad, 100) == 0

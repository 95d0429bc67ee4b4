"""The allocation-free entry point cngp_encode_bwd_static (static device scratch inside the library) against
cngp_encode_bwd with a caller's workspace, through the C ABI, on two calls in a row -- the second with a smaller
input, so that whatever the first call left in the shared scratch must not matter.  Both are also held to the
oracle.  Collected last (the file name sorts after every other test file)."""
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


def _case(N, seed_cfg, **kw):
    base = dict(cfg=seed_cfg, d=3, L=8, F=2, N_f=2**14, N_c=2**12, N_p=8, N_min=16, N_max=512, N=N,
                feat_dtype="f16", io_dtype="f16")
    base.update(kw)
    w = W.custom(**base)
    x = W.make_points(w)
    D_f = W.make_feature_codebook(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    return w, x, D_f, W.make_probe_logits(w), W.make_upstream_grad(w)


def _both(w, x, D_f, Dhat, dy, flags=cngp.ZERO_GRADS, **over):
    cfg = cngp.Config.from_workload(w, flags=flags, **over)
    xd, Fd, Cd, yd = dev(x), dev(D_f), dev(Dhat), dev(dy)
    gF0 = torch.full((w.L, w.N_f, w.F), float("nan"), device=DEV)
    gC0 = torch.full((w.L, w.N_c, w.N_p), float("nan"), device=DEV)
    gF1, gC1 = gF0.clone(), gC0.clone()
    ws = cngp.alloc_workspace(cfg, x.shape[0])
    cngp.encode_bwd(cfg, xd, Fd, Cd, yd, gF0, gC0, workspace=ws)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    cngp.encode_bwd_static(cfg, xd, Fd, Cd, yd, gF1, gC1)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before            # the binding allocates nothing either
    ref = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    for name, a, b, r, mag in (("grad D_f", gF0, gF1, ref[0], ref[2]), ("grad Dhat_c", gC0, gC1, ref[1], ref[3])):
        a, b = a.cpu().numpy(), b.cpu().numpy()
        check_close(f"{name} [workspace]", a, r, mag, fp16_out=False)
        check_close(f"{name} [static]", b, r, mag, fp16_out=False)
        check_close(f"{name} [static vs workspace]", b, a.astype(np.float64), mag, fp16_out=False)
    return cfg


def test_static_scratch_backward_two_calls_in_a_row():
    assert cngp.static_scratch_bytes() == 64 << 20
    # first call: binned variant whose bins (2^17 points: 67 MB) with the softmax table exceed the scratch, so it runs in passes
    w, x, D_f, Dhat, dy = _case(1 << 17, 41)
    cfg = _both(w, x, D_f, Dhat, dy, flags=cngp.ZERO_GRADS | cngp.BWD_BINNED)
    assert cngp.bwd_plan_info(cfg, w.N)["binned"] == 1
    # second call, smaller input, other table sizes: the replicated-scan variant, leftovers of call one in the scratch
    w, x, D_f, Dhat, dy = _case(20000, 42, L=5, N_f=2**12, N_c=2**11, N_p=16, N_max=200)
    _both(w, x, D_f, Dhat, dy)
    # and a ragged third one through the forced binned variant with a tiny bin bound of the caller's own
    w, x, D_f, Dhat, dy = _case(7777, 43, d=2, L=3, N_p=4, N_max=97, feat_dtype="f32", io_dtype="f32")
    _both(w, x, D_f, Dhat, dy, flags=cngp.ZERO_GRADS | cngp.BWD_BINNED, bin_bytes_max=1 << 20)


def test_static_scratch_rejects_what_does_not_fit():
    """A softmax table alone larger than the static array: a clear error before any launch; the gradient arrays
    are not touched.  (Real buffers all the same: no test hands the library a pointer it could not follow.)"""
    w = W.custom(cfg=44, d=3, L=16, F=2, N_f=2**16, N_c=2**17, N_p=16, N_min=16, N_max=2048, N=1 << 15,
                 feat_dtype="f16", io_dtype="f16")
    cfg = cngp.Config.from_workload(w, flags=cngp.ZERO_GRADS)
    assert cngp.bwd_plan_info(cfg, w.N)["binned"] == 1
    x, dy = dev(W.make_points(w)), dev(W.make_upstream_grad(w))
    D_f = torch.zeros((w.L, w.N_f, w.F), dtype=torch.float16, device=DEV)
    Dhat = torch.zeros((w.L, w.N_c, w.N_p), device=DEV)
    gF = torch.full((w.L, w.N_f, w.F), 7.0, device=DEV)
    gC = torch.full((w.L, w.N_c, w.N_p), 7.0, device=DEV)
    with pytest.raises(cngp.CngpError) as e:
        cngp.encode_bwd_static(cfg, x, D_f, Dhat, dy, gF, gC)
    assert e.value.status == cngp.ERR_WORKSPACE
    assert b"static array holds" in cngp._lib.cngp_last_hip_error()
    torch.cuda.synchronize()
    assert bool((gF == 7.0).all()) and bool((gC == 7.0).all())

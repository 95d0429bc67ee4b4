"""The entry points only enqueue work on the caller's stream (no synchronisation, no allocation, no memset
nodes), so a caller can capture a whole step into a HIP graph.  Captured here through torch.cuda.CUDAGraph
and replayed several times with eager work and synchronisation in between; every replay is held against
the oracle like an eager call."""
import numpy as np
import pytest
import torch

import oracle
import paper_2312_17241_amd as cngp
import workloads as W
from parity import check_close, check_exact

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("flags,n,N_f,passes", [
    (0, 40000 + 3, 2**13, 1), (cngp.BWD_BINNED, 40000 + 3, 2**13, 1), (cngp.BWD_DIRECT, 5000, 2**13, 1),
    (cngp.BWD_BINNED, 40000 + 3, 2**9, 1),          # small feature table: both gradients from one pass over the bins
    (cngp.BWD_BINNED, 40000 + 3, 2**13, 3)])        # bounded bins: three passes inside the one call
def test_graph_replay_matches_the_oracle(flags, n, N_f, passes):
    w = W.custom(cfg=91, d=3, L=6, N_f=N_f, N_c=2**11, N_p=8, N_min=8, N_max=256, N=n, feat_dtype="f16", io_dtype="f16")
    limit = 0 if passes == 1 else 16 * 1024 * 8 * 4 * w.L * 2
    cfg = cngp.Config.from_workload(w, flags=cngp.ZERO_GRADS | flags, bin_bytes_max=limit)
    plan = cngp.bwd_plan_info(cfg, n)
    assert plan["passes"] == passes and (plan["slices_f"] == 0) == (N_f == 2**9 and bool(flags & cngp.BWD_BINNED))
    x_h, D_f_h, Dhat_h, dy_h = W.make_points(w), W.make_feature_codebook(w), W.make_probe_logits(w), W.make_upstream_grad(w)
    D_f_h = (D_f_h.astype(np.float64) * 1e4).astype(D_f_h.dtype)
    x, D_f, Dhat, dy = (torch.from_numpy(a).to(DEV) for a in (x_h, D_f_h, Dhat_h, dy_h))
    D_c = torch.empty((w.L, cfg.index_cols), dtype=torch.uint8, device=DEV)
    y = torch.empty((n, w.L * w.F), dtype=torch.float16, device=DEV)
    gF = torch.empty((w.L, w.N_f, w.F), device=DEV)
    gC = torch.empty((w.L, w.N_c, w.N_p), device=DEV)
    ws = cngp.alloc_workspace(cfg, n, DEV)

    def step():
        cngp.bake_probes(cfg, Dhat, D_c)
        cngp.encode_fwd(cfg, x, D_f, D_c, y, workspace=ws)
        cngp.encode_bwd(cfg, x, D_f, Dhat, dy, gF, gC, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                              # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    D_c_ref = oracle.bake_probes(Dhat_h)
    y_ref, ymag = oracle.encode_fwd(w, x_h, D_f_h, D_c_ref)
    gF_ref, gC_ref, A_f, A_c = oracle.encode_bwd(w, x_h, D_f_h, Dhat_h, dy_h)
    for replay in range(3):
        D_c.fill_(0xEE); y.fill_(float("nan")); gF.fill_(float("nan")); gC.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        check_exact(f"D_c, replay {replay}", D_c.cpu().numpy(), D_c_ref)
        check_close(f"y, replay {replay}", y.float().cpu().numpy(), y_ref, ymag, fp16_out=True)
        check_close(f"grad D_f, replay {replay}", gF.cpu().numpy(), gF_ref, A_f, fp16_out=False)
        check_close(f"grad Dhat_c, replay {replay}", gC.cpu().numpy(), gC_ref, A_c, fp16_out=False)
        step()                                              # eager work between the replays
        (gF.sum() + gC.sum()).item()


def test_graph_replay_of_the_morton_pipeline():
    """cngp_morton_sort and cngp_encode_fwd_permuted captured together: every
    replay gives the oracle's permutation and the plain forward's bits."""
    w = W.custom(cfg=70, d=3, L=5, N_f=2**11, N_c=2**9, N_p=8, N_min=4, N_max=300, N=50000 + 7, feat_dtype="f16", io_dtype="f16")
    cfg = cngp.Config.from_workload(w)
    x_h = W.make_points(w)
    x = torch.from_numpy(x_h).to(DEV)
    D_f = torch.from_numpy(W.make_feature_codebook(w)).to(DEV)
    D_c = cngp.bake_probes(cfg, torch.from_numpy(W.make_probe_logits(w)).to(DEV))
    y_plain = cngp.encode_fwd(cfg, x, D_f, D_c)
    n = x.shape[0]
    ws = torch.empty(int(cngp._lib.cngp_morton_sort_workspace_bytes(w.d, n)), dtype=torch.uint8, device=DEV)
    perm = torch.empty(n, dtype=torch.int32, device=DEV)
    xs, y = torch.empty_like(x), torch.empty_like(y_plain)

    def step():
        cngp._check(cngp._lib.cngp_morton_sort(w.d, x.data_ptr(), n, perm.data_ptr(), xs.data_ptr(), ws.data_ptr(), ws.numel(),
                                               cngp._stream()))
        cngp.encode_fwd_permuted(cfg, xs, perm, D_f, D_c, y)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    perm_ref, _ = oracle.morton_order(x_h)
    for replay in range(4):
        perm.fill_(-1); xs.fill_(float("nan")); y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        check_exact(f"perm, replay {replay}", perm.cpu().numpy(), perm_ref)
        assert torch.equal(y.view(torch.int16), y_plain.view(torch.int16)), f"y, replay {replay}"
        step()                                              # eager work between the replays
        y.float().sum().item()

"""GPU parity of cngp_encode_bwd_input (gradient of the forward pass with respect to the points) against
the oracle: fp32 arithmetic on exactly representable inputs, so the bar is the fp32 one, relative to the
sum of the magnitudes of the terms."""
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


def run(w, fmt, n=None, edge_points=True):
    x = W.make_points(w, n)
    if edge_points:
        x[:4] = [[0.0] * w.d, [1.0] * w.d, [0.5] * w.d, [1.0] + [0.0] * (w.d - 1)]
    D_f = W.make_feature_codebook(w)
    D_f = (D_f.astype(np.float64) * 1e4).astype(D_f.dtype)
    D_c = oracle.bake_probes(W.make_probe_logits(w))
    dy = W.make_upstream_grad(w, x.shape[0])
    D_c_dev = {cngp.IDX_U8: lambda: dev(D_c), cngp.IDX_PACKED4: lambda: cngp.pack4(dev(D_c)),
               cngp.IDX_BITS: lambda: dev(oracle.pack_index_bits(D_c, w.N_p))}[fmt]()
    cfg = cngp.Config.from_workload(w, index_format=fmt)
    gx = torch.full((x.shape[0], w.d), float("nan"), device=DEV)
    cngp.encode_bwd_input(cfg, dev(x), dev(D_f), D_c_dev, dev(dy), gx)
    torch.cuda.synchronize()
    ref, mag = oracle.encode_bwd_input(w, x, D_f, D_c, dy)
    return check_close("dL/dx", gx.cpu().numpy(), ref, mag, fp16_out=False)


@pytest.mark.parametrize("d,N_p,feat,io", [(2, 1, "f32", "f32"), (2, 8, "f16", "f16"), (3, 4, "f32", "f16"),
                                           (3, 16, "f16", "f16"), (3, 16, "f32", "f32"), (3, 2, "f16", "f32")])
@pytest.mark.parametrize("fmt", [cngp.IDX_U8, cngp.IDX_PACKED4, cngp.IDX_BITS])
def test_input_gradient_sweep(d, N_p, feat, io, fmt):
    w = W.custom(cfg=70 + d + N_p, d=d, L=5, N_f=2**11, N_c=2**9, N_p=N_p, N_min=4, N_max=300, N=3000 + 77,
                 feat_dtype=feat, io_dtype=io)
    run(w, fmt)


@pytest.mark.parametrize("N", [1, 63, 255, 256, 257])
def test_input_gradient_small_batches(N):
    """Below one tile the index codebook is read from memory instead of LDS."""
    w = W.custom(cfg=77, d=3, L=4, N_f=2**10, N_c=2**8, N_p=8, N_min=4, N_max=64, N=N)
    run(w, cngp.IDX_U8, edge_points=False)
    run(w, cngp.IDX_BITS, edge_points=False)


def test_input_gradient_index_codebook_too_large_for_lds():
    w = W.custom(cfg=78, d=3, L=2, N_f=2**12, N_c=2**18, N_p=8, N_min=16, N_max=64, N=3000)
    for fmt in (cngp.IDX_U8, cngp.IDX_PACKED4, cngp.IDX_BITS):
        run(w, fmt)


def test_input_gradient_full_size_workloads():
    run(W.WORKLOADS["nerf3d"], cngp.IDX_U8)
    # more than 2^20 points with a 2^16-entry index codebook: the large-tile variant, ragged last tile
    run(W.WORKLOADS["compact3d"], cngp.IDX_BITS, n=2**20 + 1024 + 77)

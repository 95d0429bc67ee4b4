"""End-to-end check on the GPU: the encoding, its straight-through backward (Sec. 3 "Training"), the
optimiser step and the bake, driven through the C ABI, fit a synthetic image together with a small
PyTorch decoder (the decoder is not part of this library: it stands in for the paper's MLP).

Two things are asserted, both consequences the paper claims for the method rather than numbers it prints:
the loss falls by a large factor, and with the same feature codebook size a learned index codebook
(N_p = 16) reaches a lower error than plain hashing (N_p = 1), which is Eq. 6's reason to exist (Sec. 4,
quality vs. size at fixed N_f).  The image is synthetic (random blobs, edges and a high-frequency
pattern); no dataset is involved.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2312_17241_amd as cngp
from paper_2312_17241_amd.module import Encoding
from parity import check_close, check_exact

pytestmark = pytest.mark.gpu
DEV = "cuda"


def synthetic_image(x):
    """A fixed analytic 3-channel 'image' on [0,1]^2: smooth blobs, a hard edge, fine stripes."""
    u, v = x[:, 0], x[:, 1]
    rng = np.random.default_rng(1234)
    out = torch.zeros((x.shape[0], 3), device=x.device)
    for _ in range(12):
        cu, cv, s = rng.random(), rng.random(), 0.03 + 0.1 * rng.random()
        col = torch.tensor(rng.random(3), dtype=torch.float32, device=x.device)
        out += torch.exp(-((u - cu) ** 2 + (v - cv) ** 2) / (2 * s * s))[:, None] * col
    out[:, 0] += (u + 0.5 * v > 0.8).float() * 0.5
    out[:, 1] += 0.25 * torch.sin(2 * math.pi * 40 * u) * torch.sin(2 * math.pi * 37 * v)
    return out


def fit(N_p, N_c, steps=400, N_f=2**8, lr_c=1e-1, seed=0, top_k=0):
    cfg = cngp.Config(d=2, L=8, F=2, N_f=N_f, N_c=N_c, N_p=N_p, N_min=16, N_max=512, top_k=top_k)
    torch.manual_seed(seed)
    enc = Encoding(cfg, DEV, seed=seed)
    mlp = torch.nn.Sequential(torch.nn.Linear(cfg.L * cfg.F, 64), torch.nn.ReLU(),
                              torch.nn.Linear(64, 64), torch.nn.ReLU(), torch.nn.Linear(64, 3)).to(DEV)
    opt = torch.optim.Adam(mlp.parameters(), lr=1e-2, betas=(0.9, 0.99), eps=1e-15)
    gen = torch.Generator(device=DEV).manual_seed(seed + 1)
    losses = []
    for it in range(steps):
        decay = 0.1 ** (it / steps)                    # all learning rates fall tenfold over the run
        for group in opt.param_groups:
            group["lr"] = 1e-2 * decay
        x = torch.rand((2**15, 2), device=DEV, generator=gen)
        loss = ((mlp(enc(x)) - synthetic_image(x)) ** 2).mean()
        opt.zero_grad()
        loss.backward()
        opt.step()
        enc.step(cngp.Adam(lr=1e-2 * decay, beta1=0.9, beta2=0.99, eps=1e-15),
                 cngp.Adam(lr=lr_c * decay, beta1=0.9, beta2=0.99, eps=1e-15))
        losses.append(loss.item())
    # evaluation on a fixed grid of pixel centres
    r = (torch.arange(256, device=DEV) + 0.5) / 256
    grid = torch.stack(torch.meshgrid(r, r, indexing="ij"), dim=-1).reshape(-1, 2).contiguous()
    with torch.no_grad():
        mse = ((mlp(enc(grid)) - synthetic_image(grid)) ** 2).mean().item()
    return losses, mse, enc


def test_training_reduces_the_loss_and_learned_probing_beats_plain_hashing():
    """Feature codebook of 2^8 entries per level: with a learned index codebook of 2^14 rows the fit reaches
    about a third of the error of plain hashing (measured 1.6e-3 vs 5.1e-3 after 400 steps)."""
    losses, mse_learned, enc = fit(N_p=16, N_c=2**14)
    assert np.isfinite(losses).all()
    assert np.mean(losses[-20:]) < 0.1 * np.mean(losses[:5])
    # the index codebook moved away from its initial bake and stays consistent with the confidence values
    D_c = enc.D_c.cpu().numpy()
    check_exact("D_c", D_c, oracle.bake_probes(enc.Dhat_c.cpu().numpy()))
    assert len(np.unique(D_c)) == 16
    assert not enc.grad_D_f.any() and not enc.grad_Dhat_c.any()          # cleared by the last step
    _, mse_plain, _ = fit(N_p=1, N_c=1)
    print(f"MSE learned probing {mse_learned:.3e}  plain hashing {mse_plain:.3e}")
    assert mse_learned < 0.6 * mse_plain


def test_quality_grows_with_the_index_codebook():
    """Fixed N_f and N_p: a larger N_c gives a lower error (Sec. 4: quality vs. N_c at fixed N_f, N_p)."""
    mse = [fit(N_p=16, N_c=n, lr_c=1e-2)[1] for n in (2**12, 2**16)]
    print("MSE at N_c = 2^12, 2^16:", mse)
    assert mse[1] < 0.85 * mse[0]


def test_sparse_backward_still_learns_the_index_codebook():
    """Gradient through the 4 largest confidence values of a row only (the sparse variant): the index codebook
    is still learned -- the fit beats plain hashing clearly -- though the dense softmax of the paper, which lets
    every candidate compete from the first step, ends lower (measured: dense 1.6e-3, top-4 2.4e-3,
    plain hashing 5.0e-3)."""
    _, mse_sparse, enc = fit(N_p=16, N_c=2**14, top_k=4)
    _, mse_plain, _ = fit(N_p=1, N_c=1)
    print(f"MSE top-4 {mse_sparse:.3e}  plain hashing {mse_plain:.3e}")
    assert mse_sparse < 0.8 * mse_plain
    assert len(np.unique(enc.D_c.cpu().numpy())) >= 4


def test_module_gradients_match_the_oracle():
    """The autograd bridge hands the decoder's dL/dy to encode_bwd unchanged and accumulates over calls."""
    import workloads as W
    w = W.custom(d=2, L=4, N_f=256, N_c=128, N_p=8, N_min=8, N_max=64, N=3000)
    cfg = cngp.Config.from_workload(w)
    enc = Encoding(cfg, DEV, seed=3)
    enc.Dhat_c.copy_(torch.from_numpy(W.make_probe_logits(w)).to(DEV))
    cngp.bake_probes(cfg, enc.Dhat_c, enc.D_c)
    x_h = W.make_points(w)
    x = torch.from_numpy(x_h).to(DEV)
    coef = torch.linspace(-1, 1, w.L * w.F, device=DEV)
    for _ in range(2):                                   # two backward calls: gradients add up
        (enc(x) * coef).sum().backward()
    D_f = enc.D_f_master.cpu().numpy().astype(np.float64)
    Dhat = enc.Dhat_c.cpu().numpy()
    dy = np.broadcast_to(coef.cpu().numpy().astype(np.float64), (w.N, w.L * w.F))
    gF, gC, A_f, A_c = oracle.encode_bwd(w, x_h, D_f, Dhat, np.ascontiguousarray(dy))
    check_close("grad D_f", enc.grad_D_f.cpu().numpy(), 2 * gF, 2 * A_f, fp16_out=False)
    check_close("grad Dhat_c", enc.grad_Dhat_c.cpu().numpy(), 2 * gC, 2 * A_c, fp16_out=False)
    # points that require a gradient get dL/dx through the same bridge
    xg = x.clone().requires_grad_(True)
    (enc(xg) * coef).sum().backward()
    gx_ref, gx_mag = oracle.encode_bwd_input(w, x_h, D_f, enc.D_c.cpu().numpy(), np.ascontiguousarray(dy))
    check_close("grad x", xg.grad.cpu().numpy(), gx_ref, gx_mag, fp16_out=False)


def test_training_with_the_library_decoder():
    """The same fit with every trained component inside the library: encoding forward / backward, decoder
    forward / backward on the matrix cores, Adam steps for the codebooks (fused with the bake) and for the
    decoder's weights.  PyTorch only allocates, draws the batch and forms the residual."""
    cfg = cngp.Config(d=2, L=8, F=2, N_f=2**8, N_c=2**14, N_p=16, N_min=16, N_max=512,
                      feat_dtype=cngp.F16, io_dtype=cngp.F16)
    mcfg = cngp.MlpConfig(cfg.L * cfg.F, 3, cngp.F16, flags=cngp.ZERO_GRADS)
    enc = Encoding(cfg, DEV, seed=0)
    g = torch.Generator(device="cpu").manual_seed(5)
    W1, W2, W3 = (torch.randn((r, c), generator=g) * math.sqrt(2.0 / c) for r, c in ((64, 16), (64, 64), (3, 64)))
    master = torch.cat([W1.ravel(), W2.ravel(), W3.ravel()]).to(DEV)
    W = master.half()
    m, v, gW = torch.zeros_like(master), torch.zeros_like(master), torch.zeros_like(master)
    gen = torch.Generator(device=DEV).manual_seed(1)
    steps, scale, losses = 400, 128.0, []
    ws = cngp.alloc_workspace(cfg, 2**15)
    for it in range(steps):
        decay = 0.1 ** (it / steps)
        x = torch.rand((2**15, 2), device=DEV, generator=gen)
        y = cngp.encode_fwd(cfg, x, enc.D_f, enc.D_c, workspace=ws)
        out = cngp.mlp_fwd(mcfg, y, W)
        resid = out - synthetic_image(x)
        losses.append((resid ** 2).mean().item())
        dout = resid * (2.0 * scale / resid.numel())                       # loss scaling keeps fp16 dL/dy in range
        dy, _ = cngp.mlp_bwd(mcfg, y, W, dout, grad_W=gW)
        cngp.encode_bwd(cfg, x, enc.D_f, enc.Dhat_c, dy, enc.grad_D_f, enc.grad_Dhat_c, workspace=ws)
        cngp.adam_step(cngp.Adam(lr=1e-2 * decay, eps=1e-15, grad_scale=1 / scale, step=it + 1), master, W, m, v, gW)
        enc.step(cngp.Adam(lr=1e-2 * decay, eps=1e-15, grad_scale=1 / scale),
                 cngp.Adam(lr=1e-1 * decay, eps=1e-15, grad_scale=1 / scale))
    print(f"loss {np.mean(losses[:5]):.3e} -> {np.mean(losses[-20:]):.3e}")
    assert np.isfinite(losses).all()
    assert np.mean(losses[-20:]) < 0.1 * np.mean(losses[:5])
    assert np.mean(losses[-20:]) < 4e-3          # the PyTorch-decoder run of the same shape ends near 2e-3

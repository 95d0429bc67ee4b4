"""GPU parity of the decoder kernels (matrix cores, fp16 operands, fp32 accumulation) against the fp64
oracle.  Bars: |gpu - ref| <= 2e-3 * M with M the sum of the magnitudes of the terms that form the value
(the oracle returns it): inputs, weights, hidden activations and hidden-layer gradients are each rounded to
fp16 once (relative 2^-11 = 4.9e-4), three of those roundings stack up along the longest path.

The backward pass decides relu'(a) on the sign of a pre-activation.  Both sides take that decision in their own
arithmetic, and it can differ where |a| is within the kernel's rounding error of zero.  EVERY point of the batch
is kept and compared.  Hidden units that close to zero are called ambiguous; for them either decision is accepted,
and what the choice can change is bounded exactly: the magnitude sums of the oracle evaluated with all ambiguous
units on, minus the same with all of them off, is the total magnitude of the terms that pass through such a unit,
hence an upper bound on the difference between any two choices.  That slack is zero for every point without an
ambiguous unit (its dL/dy is held to the plain bar) and a small part of the weight gradients' magnitude."""
import numpy as np
import pytest
import torch

import oracle
import paper_2312_17241_amd as cngp
from parity import TOL_F16

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t if dtype is None else t.to(dtype)


def make_case(seed, N, n_in, n_out, io):
    rng = np.random.default_rng(seed)
    y = rng.standard_normal((N, n_in)) * 0.5
    y = y.astype(np.float16).astype(np.float64) if io == cngp.F16 else y.astype(np.float32).astype(np.float64)
    he = lambda rows, cols: (rng.standard_normal((rows, cols)) * np.sqrt(2.0 / cols)).astype(np.float16).astype(np.float64)
    W1, W2, W3 = he(64, n_in), he(64, 64), he(n_out, 64)
    dout = rng.standard_normal((N, n_out)).astype(np.float32).astype(np.float64)
    return y, W1, W2, W3, dout


def ambiguous_units(y, W1, W2, io):
    """Boolean [N, 64] for each hidden layer: pre-activations closer to zero than the kernel's rounding can move them.
    The weights are fp16 numbers; y is one too when it is stored as fp16, else the kernel rounds it (2^-11
    relative).  The kernel's first pre-activation differs from the oracle's by that rounding and its fp32
    summation (1e-5 of the magnitude sum); the second one also by the rounding of every h1 to fp16."""
    eps = 2.0 ** -11
    # a sum of n independent roundings, each uniform within +-eps of its term: five standard deviations, and never
    # more than the worst case
    spread = lambda terms_sq, terms_abs: np.minimum(5.0 * eps / np.sqrt(3.0) * np.sqrt(terms_sq), eps * terms_abs)
    a1 = y @ W1.T
    m1 = np.abs(y) @ np.abs(W1).T
    d1 = 1e-5 * m1 + (spread((y * y) @ (W1 * W1).T, m1) if io == cngp.F32 else 0.0)
    h1 = np.maximum(a1, 0)
    a2 = h1 @ W2.T
    # (the first layer's 64 errors are independent of each other as well: they add in quadrature)
    d2 = np.sqrt((d1 * d1) @ (W2 * W2).T) + spread((h1 * h1) @ (W2 * W2).T, h1 @ np.abs(W2).T) + 2e-5 * (h1 @ np.abs(W2).T)
    return (np.abs(a1) <= d1, np.abs(a2) <= d2), (a1 > 0, a2 > 0)


def backward_reference(y, W1, W2, W3, dout, io):
    """Oracle gradients, their magnitudes, and per result the slack the ambiguous units allow."""
    (A1, A2), (P1, P2) = ambiguous_units(y, W1, W2, io)
    g, mag, _ = oracle.mlp_bwd(y, W1, W2, W3, dout)
    _, hi, _ = oracle.mlp_bwd(y, W1, W2, W3, dout, masks=(P1 | A1, P2 | A2))
    _, lo, _ = oracle.mlp_bwd(y, W1, W2, W3, dout, masks=(P1 & ~A1, P2 & ~A2))
    slack = {k: hi[k] - lo[k] for k in hi}
    clear = ~(A1.any(axis=1) | A2.any(axis=1))                  # points without an ambiguous unit
    assert np.all(slack["dy"][clear] == 0.0)
    return g, hi, slack, float(clear.mean())


def check(name, got, ref, mag, slack=None):
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), name
    excess = np.abs(got - ref) - (0.0 if slack is None else slack)
    err = excess.clip(min=0.0) / np.maximum(np.maximum(np.abs(ref), mag), 1e-30)
    worst = np.unravel_index(np.argmax(err), err.shape)
    assert err[worst] <= TOL_F16, f"{name}: rel err {err[worst]:.3e} at {worst}: got {got[worst]}, ref {ref[worst]}, mag {mag[worst]}"
    return float(err.max())


CASES = [(32, 3, cngp.F16, 5000), (32, 3, cngp.F32, 777), (16, 3, cngp.F32, 2049), (8, 1, cngp.F32, 300),
         (32, 16, cngp.F16, 1000), (20, 4, cngp.F16, 640), (3, 2, cngp.F32, 31), (32, 4, cngp.F16, 1)]


@pytest.mark.parametrize("n_in,n_out,io,N", CASES)
def test_mlp_forward(n_in, n_out, io, N):
    y, W1, W2, W3, _ = make_case(n_in * 100 + n_out, N, n_in, n_out, io)
    cfg = cngp.MlpConfig(n_in, n_out, io)
    assert cfg.weight_count == 64 * n_in + 64 * 64 + 64 * n_out
    W = dev(np.concatenate([W1.ravel(), W2.ravel(), W3.ravel()]), torch.float16)
    out = cngp.mlp_fwd(cfg, dev(y, torch.float16 if io == cngp.F16 else torch.float32), W)
    torch.cuda.synchronize()
    ref, mag, _ = oracle.mlp_fwd(y, W1, W2, W3, want_mag=True)
    check("out", out.cpu().numpy(), ref, mag)


@pytest.mark.parametrize("n_in,n_out,io,N", CASES)
def test_mlp_backward(n_in, n_out, io, N):
    # (the single-point case takes the next seed: with this one its only point has a unit within rounding of zero)
    y, W1, W2, W3, dout = make_case(n_in * 100 + n_out + 7 + (1 if N == 1 else 0), N, n_in, n_out, io)
    g, mag, slack, clear = backward_reference(y, W1, W2, W3, dout, io)
    assert clear >= 0.7, clear                  # most points have no ambiguous unit: they are held to the plain bar
    for k in ("dW1", "dW2", "dW3"):             # and the slack is a small part of what the weight gradients are made of
        assert N < 40 or slack[k].sum() <= 0.02 * mag[k].sum(), (k, slack[k].sum() / mag[k].sum())
    cfg = cngp.MlpConfig(n_in, n_out, io, flags=cngp.ZERO_GRADS)
    W = dev(np.concatenate([W1.ravel(), W2.ravel(), W3.ravel()]), torch.float16)
    tdt = torch.float16 if io == cngp.F16 else torch.float32
    gW = torch.full((cfg.weight_count,), float("nan"), device=DEV)
    dy, gW = cngp.mlp_bwd(cfg, dev(y, tdt), W, dev(dout, torch.float32), grad_W=gW)
    torch.cuda.synchronize()
    check("dy", dy.float().cpu().numpy(), g["dy"], mag["dy"], slack["dy"])
    g1, g2, g3 = (t.cpu().numpy() for t in cfg.split(gW))
    check("dW1", g1, g["dW1"], mag["dW1"], slack["dW1"])
    check("dW2", g2, g["dW2"], mag["dW2"], slack["dW2"])
    check("dW3", g3, g["dW3"], mag["dW3"], slack["dW3"])
    # without the flag the gradient accumulates
    cfg2 = cngp.MlpConfig(n_in, n_out, io)
    _, gW2 = cngp.mlp_bwd(cfg2, dev(y, tdt), W, dev(dout, torch.float32), grad_W=gW.clone())
    torch.cuda.synchronize()
    check("2 dW2", cfg.split(gW2)[1].cpu().numpy(), 2 * g["dW2"], 2 * mag["dW2"], 2 * slack["dW2"])
    print(f"\nmlp_bwd n_in={n_in} n_out={n_out} N={N}: all {N} points compared, {clear:.1%} of them without an ambiguous unit")


def test_mlp_full_size():
    """The benchmark's batch: 2^18 points, 32 inputs (L * F of the headline workload), RGB output."""
    N, n_in, n_out = 2**18, 32, 3
    y, W1, W2, W3, dout = make_case(99, N, n_in, n_out, cngp.F16)
    cfg = cngp.MlpConfig(n_in, n_out, cngp.F16, flags=cngp.ZERO_GRADS)
    W = dev(np.concatenate([W1.ravel(), W2.ravel(), W3.ravel()]), torch.float16)
    out = cngp.mlp_fwd(cfg, dev(y, torch.float16), W)
    dy, gW = cngp.mlp_bwd(cfg, dev(y, torch.float16), W, dev(dout, torch.float32))
    torch.cuda.synchronize()
    ref, mag, _ = oracle.mlp_fwd(y, W1, W2, W3, want_mag=True)
    check("out", out.cpu().numpy(), ref, mag)
    g, gm, slack, clear = backward_reference(y, W1, W2, W3, dout, cngp.F16)
    assert clear >= 0.7, clear
    check("dy", dy.float().cpu().numpy(), g["dy"], gm["dy"], slack["dy"])
    for name, t in zip(("dW1", "dW2", "dW3"), cfg.split(gW)):
        assert slack[name].sum() <= 0.02 * gm[name].sum()
        check(name, t.cpu().numpy(), g[name], gm[name], slack[name])


def test_adam_step_on_a_plain_array():
    rng = np.random.default_rng(5)
    n = 64 * 32 + 64 * 64 + 64 * 3 + 1                      # not a multiple of four
    theta = rng.standard_normal(n).astype(np.float32)
    m = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    v = (rng.random(n) * 1e-3).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32)
    opt = cngp.Adam(lr=1e-2, beta1=0.9, beta2=0.99, eps=1e-15, step=4)
    t = [dev(a) for a in (theta, m, v, g)]
    half = torch.zeros(n, dtype=torch.float16, device=DEV)
    cngp.adam_step(opt, t[0], half, t[1], t[2], t[3], clear_grad=True)
    torch.cuda.synchronize()
    f = lambda z: float(np.float32(z))
    th, m1, v1 = oracle.adam_step(theta, m, v, g, f(opt.lr), f(opt.beta1), f(opt.beta2), f(opt.eps), opt.step)
    assert np.allclose(t[0].cpu().numpy(), th, rtol=1e-5, atol=1e-7)
    assert np.allclose(t[1].cpu().numpy(), m1, rtol=1e-5, atol=1e-8) and np.allclose(t[2].cpu().numpy(), v1, rtol=1e-5, atol=1e-10)
    assert np.array_equal(half.cpu().numpy().view(np.uint16), t[0].cpu().numpy().astype(np.float16).view(np.uint16))
    assert not t[3].any()


@pytest.mark.parametrize("fmt", [cngp.IDX_U8, cngp.IDX_PACKED4, cngp.IDX_BITS])
@pytest.mark.parametrize("d,L,N_p,N_c,feat,io,n_out,N", [(3, 16, 16, 2**14, "f16", "f16", 3, 5000 + 77),
                                                         (2, 8, 8, 2**12, "f32", "f32", 1, 1000 + 3),
                                                         (3, 5, 4, 2**9, "f16", "f32", 16, 256),
                                                         (3, 16, 8, 2**16, "f16", "f16", 4, 40000)])
def test_fused_encode_and_decoder(fmt, d, L, N_p, N_c, feat, io, n_out, N):
    """cngp_encode_mlp_fwd equals the two separate calls bit for bit (the encoded features pass as fp16 either
    way) and agrees with the oracle chain within the decoder's bar."""
    import workloads as W
    w = W.custom(cfg=95, d=d, L=L, N_f=2**12, N_c=N_c, N_p=N_p, N_min=8, N_max=512, N=N, feat_dtype=feat, io_dtype=io)
    x_h = W.make_points(w)
    D_f_h = W.make_feature_codebook(w)
    D_f_h = (D_f_h.astype(np.float64) * 1e4).astype(D_f_h.dtype)
    D_c_h = oracle.bake_probes(W.make_probe_logits(w))
    rng = np.random.default_rng(3)
    he = lambda rows, cols: (rng.standard_normal((rows, cols)) * np.sqrt(2.0 / cols)).astype(np.float16).astype(np.float64)
    W1, W2, W3 = he(64, 2 * L), he(64, 64), he(n_out, 64)
    Wd = dev(np.concatenate([W1.ravel(), W2.ravel(), W3.ravel()]), torch.float16)
    cfg = cngp.Config.from_workload(w, index_format=fmt)
    mcfg = cngp.MlpConfig(2 * L, n_out, cngp.F16 if io == "f16" else cngp.F32)
    D_c = {cngp.IDX_U8: lambda: dev(D_c_h), cngp.IDX_PACKED4: lambda: cngp.pack4(dev(D_c_h)),
           cngp.IDX_BITS: lambda: dev(oracle.pack_index_bits(D_c_h, N_p))}[fmt]()
    fused = cngp.encode_mlp_fwd(cfg, mcfg, dev(x_h), dev(D_f_h), D_c, Wd)
    y = cngp.encode_fwd(cfg, dev(x_h), dev(D_f_h), D_c)
    two = cngp.mlp_fwd(mcfg, y, Wd)
    torch.cuda.synchronize()
    assert torch.equal(fused, two)
    # with room for the level-major fp16 encodings: level-resident forward + the decoder reading the planes
    need = N * L * 2 * 2
    ws = torch.empty(need + 256, dtype=torch.uint8, device=DEV)
    level = cngp.Config.from_workload(w, index_format=fmt, flags=cngp.FWD_LEVEL)
    planes = cngp.encode_mlp_fwd(level, mcfg, dev(x_h), dev(D_f_h), D_c, Wd, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(planes, two)
    y_ref, _ = oracle.encode_fwd(w, x_h, D_f_h, D_c_h)
    ref, mag, _ = oracle.mlp_fwd(y_ref, W1, W2, W3, want_mag=True)
    check("decoder(encode(x))", fused.cpu().numpy(), ref, mag)
    check("decoder(encode(x)), level-major", planes.cpu().numpy(), ref, mag)


def test_fused_encode_and_decoder_refuses_what_it_cannot_do():
    import workloads as W
    w = W.custom(cfg=96, d=3, L=4, N_f=2**10, N_c=2**19, N_p=2, N_min=8, N_max=64, N=300)     # index codebook too large for LDS
    cfg = cngp.Config.from_workload(w)
    z = lambda shape, dt: torch.zeros(shape, dtype=dt, device=DEV)
    with pytest.raises(cngp.CngpError) as e:
        cngp.encode_mlp_fwd(cfg, cngp.MlpConfig(8, 3), z((300, 3), torch.float32), z((4, 2**10, 2), torch.float32),
                            z((4, 2**19), torch.uint8), z((cngp.MlpConfig(8, 3).weight_count,), torch.float16))
    assert e.value.status == cngp.ERR_UNSUPPORTED
    with pytest.raises(cngp.CngpError) as e:                   # decoder input width must be L * F
        cngp.encode_mlp_fwd(cfg, cngp.MlpConfig(16, 3), z((300, 3), torch.float32), z((4, 2**10, 2), torch.float32),
                            z((4, 2**19), torch.uint8), z((cngp.MlpConfig(16, 3).weight_count,), torch.float16))
    assert e.value.status == cngp.ERR_INVALID

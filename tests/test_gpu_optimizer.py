"""GPU parity of the optimiser step fused with the bake (cngp_adam_step_bake) against the CPU oracle.

The oracle applies Adam in fp64 to the same fp32 inputs, with the hyper-parameters rounded to fp32 as
the library receives them.  Bars:
  * D_c and the fp16 copy of D_f are integer / rounding decisions taken from the fp32 values the kernel
    itself wrote: they are compared bit for bit with the oracle's bake / a round-to-nearest conversion
    of the kernel's updated arrays.  Against the oracle's OWN updated values an argmax may differ only
    where the two largest values of the row lie within the floating-point bar of each other.
  * m' = b1 m + (1-b1) g is a sum of two signed terms: |err| <= 1e-5 * (|b1 m| + |(1-b1) g|).
  * v' is a sum of non-negative terms: relative 1e-5.
  * theta' = theta - u with u = lr_t m' / (sqrt(v'/c2) + eps): a few fp32 roundings on u (whose own error
    is relative to U = lr_t (|b1 m| + |(1-b1) g|) / denominator) and one on the difference:
    |err| <= 1e-5 * (|theta| + U).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2312_17241_amd as cngp
import workloads as W
from parity import check_close, check_exact

pytestmark = pytest.mark.gpu
DEV = "cuda"
f32 = np.float32


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def unpack(cfg, D_c):
    a = host(D_c)
    if cfg.index_format != cngp.IDX_PACKED4:
        return a
    out = np.empty((cfg.L, cfg.N_c), np.uint8)
    out[:, 0::2] = a & 0xF
    out[:, 1::2] = a >> 4
    return out


def sparse_gradient(rng, shape, zero_fraction=0.5):
    """Gradients of a sparse encoding: many exact zeros, magnitudes spread over several decades."""
    g = rng.standard_normal(shape) * 10.0 ** rng.uniform(-6, 0, shape)
    g[rng.random(shape) < zero_fraction] = 0.0
    return g.astype(f32)


def state(rng, shape, step):
    """Moments as some earlier steps would have left them (zero before the first step)."""
    if step == 1:
        return np.zeros(shape, f32), np.zeros(shape, f32)
    m = (rng.standard_normal(shape) * 1e-2).astype(f32)
    v = (rng.random(shape) * 1e-3).astype(f32)
    return m, v


def reference(theta, m, v, g, opt):
    """Oracle step with the hyper-parameters as fp32 numbers, plus the magnitudes the bars refer to."""
    lr, b1, b2, eps, gs = (float(f32(z)) for z in (opt.lr, opt.beta1, opt.beta2, opt.eps, opt.grad_scale))
    g64 = g.astype(np.float64) * gs
    th, m1, v1 = oracle.adam_step(theta, m, v, g64, lr, b1, b2, eps, opt.step)
    mag_m = np.abs(b1 * m.astype(np.float64)) + np.abs((1 - b1) * g64)
    denom = np.sqrt(v1 / (1 - b2 ** opt.step)) + eps
    U = lr / (1 - b1 ** opt.step) * mag_m / denom
    return th, m1, v1, mag_m, np.abs(theta.astype(np.float64)) + U


def check_table(name, got, ref):
    th, m, v = got
    th_ref, m_ref, v_ref, mag_m, mag_th = ref
    e = check_close(f"{name} m", host(m), m_ref, mag_m, fp16_out=False)
    e = max(e, check_close(f"{name} v", host(v), v_ref, v_ref, fp16_out=False))
    return max(e, check_close(f"{name} theta", host(th), th_ref, mag_th, fp16_out=False))


def check_argmax_valid(D_c, logits_ref, mag):
    """Where the kernel's argmax differs from the argmax of the oracle's values, the two candidates
    must be within the floating-point bar of each other in the oracle's values."""
    want = oracle.bake_probes(logits_ref.astype(f32))
    L, R, NP = logits_ref.shape
    diff = np.argwhere(D_c != want)
    for l, r in diff:
        a, b = logits_ref[l, r, D_c[l, r]], logits_ref[l, r, want[l, r]]
        assert abs(a - b) <= 2e-5 * mag[l, r].max(), (l, r, a, b)
    return len(diff)


def run_case(w, fmt, opt_f, opt_c, seed, clear, feat_dtype=None, nan_rows=False):
    rng = np.random.default_rng(seed)
    over = {} if feat_dtype is None else dict(feat_dtype=feat_dtype)
    cfg = cngp.Config.from_workload(w, index_format=fmt, flags=cngp.ZERO_GRADS if clear else 0, **over)
    fs, cs = (w.L, w.N_f, w.F), (w.L, w.N_c, w.N_p)
    D_f = rng.uniform(-1e-1, 1e-1, fs).astype(f32)
    Dhat = (rng.standard_normal(cs) * 0.5).astype(f32)
    g_f, g_c = sparse_gradient(rng, fs), sparse_gradient(rng, cs)
    m_f, v_f = state(rng, fs, opt_f.step)
    m_c, v_c = state(rng, cs, opt_c.step)
    if nan_rows:                                    # a NaN gradient poisons its entry: the bake must skip it
        g_c[0, 0, :] = np.nan
        g_c[0, 1 % w.N_c, 0] = np.nan
        g_c[-1, -1, w.N_p - 1] = np.nan
    half = cfg.feat_dtype == cngp.F16
    t_master, t_mf, t_vf, t_gf = dev(D_f), dev(m_f), dev(v_f), dev(g_f)
    t_half = torch.full(fs, float("nan"), dtype=torch.float16, device=DEV) if half else None
    t_hat, t_mc, t_vc, t_gc = dev(Dhat), dev(m_c), dev(v_c), dev(g_c)
    D_c = torch.full((w.L, cfg.index_cols), 0xEE, dtype=torch.uint8, device=DEV)
    cngp.adam_step_bake(cfg, opt_f, opt_c, (t_master, t_half, t_mf, t_vf, t_gf), (t_hat, t_mc, t_vc, t_gc, D_c))
    torch.cuda.synchronize()

    # decisions taken from the kernel's own fp32 results: bit-exact
    got_c = unpack(cfg, D_c)
    check_exact("D_c from the updated rows", got_c, oracle.bake_probes(host(t_hat)))
    assert got_c.max() < w.N_p
    if half:
        check_exact("fp16 copy of D_f", host(t_half).view(np.uint16), host(t_master).astype(np.float16).view(np.uint16))
    # gradients: consumed and cleared, or left alone
    if clear:
        assert not host(t_gf).any() and not np.nan_to_num(host(t_gc)).any() and not np.isnan(host(t_gc)).any()
    else:
        assert np.array_equal(host(t_gf), g_f) and np.array_equal(host(t_gc), g_c, equal_nan=True)

    ref_f = reference(D_f, m_f, v_f, g_f, opt_f)
    err = check_table("D_f", (t_master, t_mf, t_vf), ref_f)
    if not nan_rows:
        ref_c = reference(Dhat, m_c, v_c, g_c, opt_c)
        err = max(err, check_table("Dhat_c", (t_hat, t_mc, t_vc), ref_c))
        check_argmax_valid(got_c, ref_c[0], ref_c[4])
    else:
        bad = np.isnan(g_c)
        assert np.all(np.isnan(host(t_hat)[bad])) and not np.isnan(host(t_hat)[~bad]).any()
    return err


OPT_A = cngp.Adam(lr=1e-2, beta1=0.9, beta2=0.99, eps=1e-15, grad_scale=1.0, step=1)
OPT_B = cngp.Adam(lr=3e-3, beta1=0.8, beta2=0.999, eps=1e-8, grad_scale=1.0 / 128.0, step=7)


@pytest.mark.parametrize("N_p", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("fmt", [cngp.IDX_U8, cngp.IDX_PACKED4])
def test_adam_step_bake_small(N_p, fmt):
    w = W.custom(d=3, L=3, N_f=4096, N_c=2048, N_p=N_p, N_min=4, N_max=64, N=16)
    run_case(w, fmt, OPT_A, OPT_B, seed=100 + N_p, clear=False)
    run_case(w, fmt, OPT_B, OPT_A, seed=200 + N_p, clear=True, feat_dtype=cngp.F16)


@pytest.mark.parametrize("N_p,N_c,N_f,L", [(1, 1, 1, 1), (1, 1, 2, 3), (2, 1, 2, 1), (2, 2, 4, 3), (1, 2, 8, 5),
                                           (4, 1, 4, 1), (16, 1, 16, 1), (8, 2, 8, 3), (1, 64, 2, 7)])
def test_adam_step_bake_ragged_tables(N_p, N_c, N_f, L):
    """Tables smaller than one lane's four entries, or not a multiple of them."""
    w = W.custom(d=2, L=L, N_f=N_f, N_c=N_c, N_p=N_p, N_min=2, N_max=8, N=16)
    for fmt in (cngp.IDX_U8, cngp.IDX_PACKED4):
        if fmt == cngp.IDX_PACKED4 and N_c < 2:
            continue
        run_case(w, fmt, OPT_A, OPT_A, seed=N_p * 100 + N_c, clear=True)
        run_case(w, fmt, OPT_B, OPT_B, seed=N_p * 100 + N_c + 1, clear=False, feat_dtype=cngp.F16)


@pytest.mark.parametrize("N_p", [2, 4, 16])
def test_adam_step_bake_skips_nan(N_p):
    w = W.custom(d=3, L=2, N_f=1024, N_c=512, N_p=N_p, N_min=4, N_max=64, N=16)
    for fmt in (cngp.IDX_U8, cngp.IDX_PACKED4):
        run_case(w, fmt, OPT_A, OPT_B, seed=7, clear=False, nan_rows=True)


def test_adam_step_bake_ties_take_the_lowest_index():
    """All-equal rows with equal gradients stay all-equal: the bake must return 0 for every row, also
    where the row spans several lanes."""
    for N_p in (4, 8, 16):
        w = W.custom(d=3, L=2, N_f=1024, N_c=256, N_p=N_p, N_min=4, N_max=64, N=16)
        cfg = cngp.Config.from_workload(w)
        cs = (w.L, w.N_c, w.N_p)
        hat = torch.zeros(cs, device=DEV); m = torch.zeros(cs, device=DEV); v = torch.zeros(cs, device=DEV)
        g = torch.ones(cs, device=DEV)
        g[1, :, N_p // 2:] = -1.0                    # second level: the upper half of every row rises
        D_c = torch.full((w.L, w.N_c), 0xEE, dtype=torch.uint8, device=DEV)
        cngp.adam_step_bake(cfg, None, OPT_A, None, (hat, m, v, g, D_c))
        torch.cuda.synchronize()
        assert not host(D_c)[0].any()
        assert np.all(host(D_c)[1] == N_p // 2)


def test_adam_step_bake_one_table_only():
    w = W.custom(d=3, L=2, N_f=1024, N_c=512, N_p=8, N_min=4, N_max=64, N=16)
    cfg = cngp.Config.from_workload(w)
    rng = np.random.default_rng(5)
    fs, cs = (w.L, w.N_f, w.F), (w.L, w.N_c, w.N_p)
    f = [dev(rng.standard_normal(fs).astype(f32)) for _ in range(4)]
    c = [dev(rng.standard_normal(cs).astype(f32)) for _ in range(4)]
    f[2].abs_(); c[2].abs_()                          # second moments are non-negative
    f0 = [t.clone() for t in f]; c0 = [t.clone() for t in c]
    D_c = torch.full((w.L, w.N_c), 0xEE, dtype=torch.uint8, device=DEV)
    cngp.adam_step_bake(cfg, OPT_B, None, (f[0], None, f[1], f[2], f[3]), None)
    torch.cuda.synchronize()
    assert not torch.equal(f[0], f0[0]) and torch.equal(f[3], f0[3])
    assert all(torch.equal(a, b) for a, b in zip(c, c0)) and bool((D_c == 0xEE).all())
    cngp.adam_step_bake(cfg, None, OPT_B, None, (c[0], c[1], c[2], c[3], D_c))
    torch.cuda.synchronize()
    assert not torch.equal(c[0], c0[0])
    check_exact("D_c", host(D_c), oracle.bake_probes(host(c[0])))


def test_adam_step_bake_tiny_gradients():
    """Gradients whose squares underflow fp32 (|g| < 1e-19): with eps = 1e-15 the step stays within the bar."""
    w = W.custom(d=3, L=2, N_f=2048, N_c=512, N_p=4, N_min=4, N_max=64, N=16)
    cfg = cngp.Config.from_workload(w)
    rng = np.random.default_rng(11)
    fs = (w.L, w.N_f, w.F)
    D_f = rng.uniform(-1e-4, 1e-4, fs).astype(f32)
    g = (rng.standard_normal(fs) * 10.0 ** rng.uniform(-26, -17, fs)).astype(f32)
    z = np.zeros(fs, f32)
    t = [dev(D_f), dev(z), dev(z), dev(g)]
    cngp.adam_step_bake(cfg, OPT_A, None, (t[0], None, t[1], t[2], t[3]), None)
    torch.cuda.synchronize()
    ref = reference(D_f, z, z, g, OPT_A)
    check_close("theta", host(t[0]), ref[0], ref[4], fp16_out=False)
    check_close("m", host(t[1]), ref[1], ref[3], fp16_out=False)


@pytest.mark.parametrize("name", ["nerf3d", "image2d"])
def test_adam_step_bake_full_size(name):
    """The benchmark's tables at full size, in the configuration bench.py runs (packed index codebook is
    covered above; the benchmark stores one byte per entry)."""
    w = W.WORKLOADS[name]
    err = run_case(w, cngp.IDX_U8, OPT_A, OPT_A, seed=31, clear=True)
    assert err <= 1e-5
    # several steps in a row, state carried on the device, against the oracle carried in fp64-from-fp32
    cfg = cngp.Config.from_workload(w)
    rng = np.random.default_rng(33)
    cs = (w.L, w.N_c, w.N_p)
    hat = (rng.standard_normal(cs) * 0.1).astype(f32)
    t = [dev(hat), torch.zeros(cs, device=DEV), torch.zeros(cs, device=DEV), None]
    D_c = torch.empty((w.L, w.N_c), dtype=torch.uint8, device=DEV)
    for step in (1, 2, 3):
        g = sparse_gradient(rng, cs)
        before = [host(z) for z in t[:3]]
        t[3] = dev(g)
        opt = cngp.Adam(lr=1e-2, eps=1e-15, step=step)
        cngp.adam_step_bake(cfg, None, opt, None, (t[0], t[1], t[2], t[3], D_c))
        torch.cuda.synchronize()
        check_table(f"step {step}", t[:3], reference(before[0], before[1], before[2], g, opt))
        check_exact("D_c", host(D_c), oracle.bake_probes(host(t[0])))

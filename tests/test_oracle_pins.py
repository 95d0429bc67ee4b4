"""Pins for the CPU oracle: everything here checks oracle/ against something that
is not the oracle -- closed forms, brute force over a resolved dense grid with a
library interpolator, the reduction to the plain hash grid, exact adjoint and
finite-difference identities of the softmax-relaxed forward, and the invariants
the method's definition implies.  CPU only.
"""
import itertools
import os

import numpy as np
import pytest
from scipy.interpolate import RegularGridInterpolator

import oracle
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
M32 = 0xFFFFFFFF

# Constants as the readings fix them (Eq. 3: "large prime numbers, optionally pi_0 = 1").
PI = (1, 2654435761, 805459861, 1920767767)
PI2 = (1580030173, 1367130559, 3037000507, 2479700537)


def py_hash(v, primes):
    """Eq. 3 with Python integers, every product reduced to 32 bits."""
    h = 0
    for vi, p in zip(v, primes):
        h ^= (int(vi) * p) & M32
    return h


def py_feat_index(v, N_f, N_c, N_p, D_c_level):
    """Eq. 6, literally."""
    return (N_p * py_hash(v, PI)) % N_f + int(D_c_level[py_hash(v, PI2) % N_c])


def small(d=2, **kw):
    base = dict(d=d, L=3, F=2, N_f=64, N_c=32, N_p=4, N_min=3, N_max=11, N=160)
    base.update(kw)
    return W.custom(**base)


def random_tables(w, seed=0, scale=1.0):
    rng = np.random.default_rng(seed)
    D_f = rng.uniform(-scale, scale, (w.L, w.N_f, w.F))
    Dhat = rng.standard_normal((w.L, w.N_c, w.N_p)).astype(np.float32)
    x = rng.random((w.N, w.d)).astype(np.float32)
    dy = rng.standard_normal((w.N, w.L * w.F))
    return x, D_f, Dhat, dy


# --------------------------------------------------------------------------- constants

def _is_prime(n):
    if n < 2:
        return False
    if n % 2 == 0:
        return n == 2
    i = 3
    while i * i <= n:
        if n % i == 0:
            return False
        i += 2
    return True


def test_hash_constants_are_distinct_primes():
    for p in PI[1:] + PI2:
        assert _is_prime(p) and p < 2**32
    assert len(set(PI + PI2)) == 8
    assert PI[0] == 1                      # "optionally pi_0 = 1" (Eq. 3)


# --------------------------------------------------------------------------- level table

def _golden_tables():
    rows = []
    for line in open(os.path.join(GOLDEN, "level_tables.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, tail = line.split(":")
        nmin, nmax, L = map(int, head.split())
        rows.append((nmin, nmax, L, list(map(int, tail.split()))))
    return rows


@pytest.mark.parametrize("nmin,nmax,L,expect", _golden_tables())
def test_level_table_golden(nmin, nmax, L, expect):
    assert oracle.level_resolutions(nmin, nmax, L).tolist() == expect


@pytest.mark.parametrize("nmin,nmax,L", [(16, 512, 16), (16, 524288, 16), (16, 2048, 16), (4, 4, 5),
                                         (1, 1024, 11), (16, 2048, 2), (7, 100, 3)])
def test_level_table_closed_forms(nmin, nmax, L):
    """Table 1: coarsest resolution N_min, finest N_max; growth is monotone and geometric."""
    r = oracle.level_resolutions(nmin, nmax, L).astype(np.int64)
    assert r[0] == nmin and r[-1] == nmax
    assert np.all(np.diff(r) >= 0)
    b = (nmax / nmin) ** (1.0 / (L - 1))
    exact = nmin * b ** np.arange(L)
    assert np.all(r <= exact + 1e-5) and np.all(r > exact - 1.0)


def test_level_table_exact_powers():
    # b = 2 exactly: every level must be the exact power (plain floor() would lose some to rounding).
    assert oracle.level_resolutions(1, 1024, 11).tolist() == [2**i for i in range(11)]
    assert oracle.level_resolutions(16, 16, 1).tolist() == [16]
    assert oracle.level_resolutions(5, 99, 1).tolist() == [5]      # L == 1: N_max ignored


# --------------------------------------------------------------------------- hashes and indices

def test_index_closed_forms_at_origin():
    """x = 0: the lower corner is the all-zero vertex (hash = 0), corner 1 is the unit vector e_0
    (hash = pi_0 = 1, so base = N_p), and with d = 1-like inputs hash(v) = v."""
    w = small(d=3, L=1, N_min=8, N_f=256, N_c=64, N_p=8)
    x = np.zeros((1, 3), np.float32)
    base, h2, probe, fidx = oracle.indices(w, x, None)
    assert base[0, 0, 0] == 0 and h2[0, 0, 0] == 0
    assert base[0, 0, 1] == w.N_p                       # N_p * hash(e_0) = N_p
    assert h2[0, 0, 1] == PI2[0] % w.N_c
    assert base[0, 0, 2] == (w.N_p * PI[1]) % w.N_f     # e_1
    assert base[0, 0, 4] == (w.N_p * PI[2]) % w.N_f     # e_2
    assert base[0, 0, 7] == (w.N_p * (1 ^ PI[1] ^ PI[2])) % w.N_f
    # moving along dimension 0 only: hash(v) = v_0 (pi_0 = 1) while v_0 < N_f / N_p
    xs = np.zeros((8, 3), np.float32); xs[:, 0] = np.arange(8) / 8.0
    base, _, _, _ = oracle.indices(w, xs, None)
    assert base[:, 0, 0].tolist() == [(w.N_p * i) % w.N_f for i in range(8)]


@pytest.mark.parametrize("d", [2, 3, 4])
def test_indices_match_bigint_evaluation_and_bit_concatenation(d):
    """Every index of the dump equals an evaluation of Eq. 3 / Eq. 6 with Python integers, and
    Eq. 6's arithmetic form equals the bitwise concatenation described in the Fig. 3 caption:
    hashed most significant bits, learned least significant bits."""
    w = small(d=d, L=4, N_min=5, N_max=1000, N_f=1024, N_c=128, N_p=8, N=300)
    rng = np.random.default_rng(7)
    x = rng.random((w.N, d)).astype(np.float32)
    x[0] = 0.0; x[1] = 1.0; x[2] = 0.5
    D_c = rng.integers(0, w.N_p, (w.L, w.N_c)).astype(np.uint8)
    res = oracle.level_resolutions(w.N_min, w.N_max, w.L)
    base, h2, probe, fidx = oracle.indices(w, x, D_c)
    logp = w.N_p.bit_length() - 1
    for n in range(w.N):
        for l in range(w.L):
            pos = x[n].astype(np.float32) * np.float32(res[l])        # fp32 product
            v0 = np.floor(pos).astype(np.int64)
            for c in range(1 << d):
                v = [int(v0[i]) + ((c >> i) & 1) for i in range(d)]
                h = py_hash(v, PI)
                g = py_hash(v, PI2) % w.N_c
                assert base[n, l, c] == (w.N_p * h) % w.N_f
                assert h2[n, l, c] == g
                assert probe[n, l, c] == D_c[l, g]
                assert fidx[n, l, c] == py_feat_index(v, w.N_f, w.N_c, w.N_p, D_c[l])
                concat = ((h % (w.N_f // w.N_p)) << logp) | int(D_c[l, g])
                assert fidx[n, l, c] == concat
                assert fidx[n, l, c] < w.N_f


def test_weights_partition_unity_and_vertex_positions():
    w = small(d=3, L=2, N_min=4, N_max=16, N=50)
    rng = np.random.default_rng(3)
    x = rng.random((w.N, 3)).astype(np.float32)
    *_, wt = oracle.indices(w, x, None, want_weight=True)
    assert np.allclose(wt.sum(axis=2), 1.0, rtol=0, atol=1e-15)
    assert np.all(wt >= 0)
    # the weighted mean of the corner offsets reproduces the fractional position
    res = oracle.level_resolutions(w.N_min, w.N_max, w.L)
    for l in range(w.L):
        pos = (x * np.float32(res[l])).astype(np.float64)
        frac = pos - np.floor(pos)
        for i in range(3):
            delta = np.array([(c >> i) & 1 for c in range(8)], dtype=np.float64)
            assert np.allclose((wt[:, l, :] * delta).sum(axis=1), frac[:, i], atol=1e-15)


# --------------------------------------------------------------------------- hard forward

def resolved_grid(w, Nl, D_f_level, D_c_level):
    """Dense array T[v] = D_f[f(v)] over every vertex 0..Nl+1 per axis (Eq. 6 evaluated per vertex)."""
    n = Nl + 2
    T = np.zeros((n,) * w.d + (w.F,))
    for v in itertools.product(range(n), repeat=w.d):
        T[v] = D_f_level[py_feat_index(v, w.N_f, w.N_c, w.N_p, D_c_level)]
    return T


@pytest.mark.parametrize("d", [2, 3, 4])
def test_forward_equals_library_interpolation_of_resolved_grid(d):
    w = small(d=d)
    x, D_f, Dhat, _ = random_tables(w, seed=11)
    x[:3] = [[0.0] * d, [1.0] * d, [0.25] * d]
    D_c = np.random.default_rng(5).integers(0, w.N_p, (w.L, w.N_c)).astype(np.uint8)
    y, ymag = oracle.encode_fwd(w, x, D_f, D_c)
    res = oracle.level_resolutions(w.N_min, w.N_max, w.L)
    for l in range(w.L):
        Nl = int(res[l])
        T = resolved_grid(w, Nl, D_f[l], D_c[l])
        axes = [np.arange(Nl + 2, dtype=np.float64)] * d
        pos = (x * np.float32(Nl)).astype(np.float64)            # the fp32 product, widened
        for f in range(w.F):
            interp = RegularGridInterpolator(axes, T[..., f], method="linear")
            assert np.allclose(y[:, l * w.F + f], interp(pos), rtol=0, atol=1e-14)
    assert np.all(ymag >= np.abs(y) - 1e-15)


def test_forward_on_vertices_returns_table_entries():
    """x = v / N_l with N_l a power of two is exact in fp32: y is the looked-up feature itself."""
    w = small(d=3, L=1, N_min=8, N_f=128, N_c=64, N_p=4)
    rng = np.random.default_rng(2)
    D_f = rng.standard_normal((1, w.N_f, w.F))
    D_c = rng.integers(0, w.N_p, (1, w.N_c)).astype(np.uint8)
    vs = rng.integers(0, 9, (64, 3))
    x = (vs / 8.0).astype(np.float32)
    y, _ = oracle.encode_fwd(w, x, D_f, D_c)
    for n, v in enumerate(vs):
        assert np.array_equal(y[n], D_f[0, py_feat_index(v, w.N_f, w.N_c, w.N_p, D_c[0])])


def test_forward_constant_codebook_gives_constant():
    w = small(d=3)
    x, D_f, _, _ = random_tables(w)
    D_f[:] = 0.375
    D_c = np.zeros((w.L, w.N_c), np.uint8)
    y, _ = oracle.encode_fwd(w, x, D_f, D_c)
    assert np.allclose(y, 0.375, rtol=0, atol=1e-15)


def plain_hash_grid(x, res, D_f, primes=PI):
    """Eq. 3: multiresolution hash grid without probing, D_f[hash(v) mod N_f], vectorised numpy."""
    N, d = x.shape
    L, N_f, F = D_f.shape
    y = np.zeros((N, L * F))
    for l in range(L):
        pos = (x * np.float32(res[l])).astype(np.float64)
        v0 = np.floor(pos).astype(np.uint64)
        fr = pos - np.floor(pos)
        for c in range(1 << d):
            h = np.zeros(N, dtype=np.uint64)
            wgt = np.ones(N)
            for i in range(d):
                bit = (c >> i) & 1
                h ^= ((v0[:, i] + np.uint64(bit)) * np.uint64(primes[i])) & np.uint64(M32)
                wgt *= fr[:, i] if bit else 1.0 - fr[:, i]
            y[:, l * F:(l + 1) * F] += wgt[:, None] * D_f[l, (h % np.uint64(N_f)).astype(np.int64)]
    return y


@pytest.mark.parametrize("d,N_c", [(2, 1), (3, 1), (3, 16)])
def test_probe_range_one_is_plain_hash_grid(d, N_c):
    """N_p = 1 turns the method into the unprobed hash grid (Sec. 3 "Selecting hyperparameters")."""
    w = small(d=d, N_p=1, N_c=N_c, N_f=128, L=4, N_min=4, N_max=64)
    x, D_f, _, _ = random_tables(w, seed=21)
    D_c = np.zeros((w.L, w.N_c), np.uint8)
    y, _ = oracle.encode_fwd(w, x, D_f, D_c)
    res = oracle.level_resolutions(w.N_min, w.N_max, w.L)
    assert np.allclose(y, plain_hash_grid(x, res, D_f), rtol=0, atol=1e-14)


def test_single_row_index_codebook_is_global_probe():
    """N_c = 1: one learned probe p for the whole level: a plain hash grid over the N_f / N_p
    entries p, p + N_p, p + 2 N_p, ... of the feature codebook."""
    w = small(d=3, N_c=1, N_p=4, N_f=64, L=3)
    x, D_f, _, _ = random_tables(w, seed=4)
    D_c = np.array([[1], [3], [0]], np.uint8)
    y, _ = oracle.encode_fwd(w, x, D_f, D_c)
    res = oracle.level_resolutions(w.N_min, w.N_max, w.L)
    sub = np.stack([D_f[l, int(D_c[l, 0])::w.N_p] for l in range(w.L)])     # [L, N_f/N_p, F]
    assert np.allclose(y, plain_hash_grid(x, res, sub), rtol=0, atol=1e-14)


# --------------------------------------------------------------------------- soft forward / backward

def loss_soft(w, x, D_f, Dhat, dy):
    return float(np.sum(oracle.encode_soft_fwd(w, x, D_f, Dhat) * dy))


@pytest.mark.parametrize("d", [2, 3, 4])
def test_soft_forward_is_softmax_mix_of_hard_forwards(d):
    """With N_c = 1 the relaxed forward is the softmax-weighted mix of the N_p hard forwards."""
    w = small(d=d, N_c=1, N_p=4, L=2)
    x, D_f, Dhat, _ = random_tables(w, seed=9)
    ys = oracle.encode_soft_fwd(w, x, D_f, Dhat)
    mix = np.zeros_like(ys)
    for l in range(w.L):
        e = np.exp(Dhat[l, 0].astype(np.float64)); s = e / e.sum()
        for k in range(w.N_p):
            D_c = np.zeros((w.L, 1), np.uint8); D_c[l, 0] = k
            yk, _ = oracle.encode_fwd(w, x, D_f, D_c)
            mix[:, l * w.F:(l + 1) * w.F] += s[k] * yk[:, l * w.F:(l + 1) * w.F]
    assert np.allclose(ys, mix, rtol=0, atol=1e-14)


@pytest.mark.parametrize("d", [2, 3, 4])
def test_backward_adjoint_identity(d):
    """The relaxed forward is linear in D_f, so <y~(D_f), dy> = <D_f, gD_f> exactly."""
    w = small(d=d)
    x, D_f, Dhat, dy = random_tables(w, seed=13)
    gDf, gDc, Af, Ac = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    lhs = loss_soft(w, x, D_f, Dhat, dy)
    rhs = float(np.sum(D_f * gDf))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    assert np.all(Af >= np.abs(gDf) - 1e-12) and np.all(Ac >= np.abs(gDc) - 1e-12)


@pytest.mark.parametrize("d", [2, 3, 4])
def test_backward_matches_finite_differences(d):
    w = small(d=d, N=120)
    x, D_f, Dhat, dy = random_tables(w, seed=17)
    gDf, gDc, _, _ = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    rng = np.random.default_rng(1)
    Dh64 = Dhat.astype(np.float64)
    # feature codebook: pick entries with the largest gradients plus random ones
    flat = np.argsort(-np.abs(gDf).ravel())[:6].tolist() + rng.integers(0, gDf.size, 6).tolist()
    for idx in flat:
        i = np.unravel_index(idx, gDf.shape)
        h = 1e-3
        Dp = D_f.copy(); Dp[i] += h
        Dm = D_f.copy(); Dm[i] -= h
        fd = (loss_soft(w, x, Dp, Dh64, dy) - loss_soft(w, x, Dm, Dh64, dy)) / (2 * h)
        assert abs(fd - gDf[i]) <= 1e-8 * max(1.0, abs(gDf[i]))
    # confidence values
    flat = np.argsort(-np.abs(gDc).ravel())[:8].tolist() + rng.integers(0, gDc.size, 6).tolist()
    for idx in flat:
        i = np.unravel_index(idx, gDc.shape)
        h = 1e-5
        Dp = Dh64.copy(); Dp[i] += h
        Dm = Dh64.copy(); Dm[i] -= h
        fd = (loss_soft(w, x, D_f, Dp, dy) - loss_soft(w, x, D_f, Dm, dy)) / (2 * h)
        assert abs(fd - gDc[i]) <= 1e-6 * max(1.0, abs(gDc[i]))


@pytest.mark.parametrize("d", [2, 3, 4])
def test_backward_invariants(d):
    w = small(d=d)
    x, D_f, Dhat, dy = random_tables(w, seed=19)
    gDf, gDc, _, _ = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    # softmax Jacobian annihilates constants: every row of the logit gradient sums to zero
    assert np.allclose(gDc.sum(axis=2), 0.0, rtol=0, atol=1e-12)
    # sigma and the interpolation weights each sum to one: gradient mass is conserved per level/feature
    want = dy.reshape(w.N, w.L, w.F).sum(axis=0)
    assert np.allclose(gDf.sum(axis=1), want, rtol=0, atol=1e-11)
    # a constant added to a row of confidence values changes nothing
    shift = np.random.default_rng(0).standard_normal((w.L, w.N_c, 1))
    g2 = oracle.encode_bwd(w, x, D_f, Dhat.astype(np.float64) + shift, dy)
    assert np.allclose(g2[0], gDf, rtol=0, atol=1e-12) and np.allclose(g2[1], gDc, rtol=0, atol=1e-12)
    # backward accumulates: linear in dy
    g3 = oracle.encode_bwd(w, x, D_f, Dhat, 2.0 * dy)
    assert np.allclose(g3[0], 2 * gDf, atol=1e-12) and np.allclose(g3[1], 2 * gDc, atol=1e-12)


def test_one_hot_confidences_make_soft_equal_hard():
    """Confident rows: softmax -> one-hot, the relaxed forward is the hard forward of the baked
    codebook, the feature gradient is the true gradient of the hard forward and the logit gradient
    vanishes."""
    w = small(d=3)
    x, D_f, _, dy = random_tables(w, seed=23)
    D_c = np.random.default_rng(8).integers(0, w.N_p, (w.L, w.N_c)).astype(np.uint8)
    Dhat = np.zeros((w.L, w.N_c, w.N_p))
    np.put_along_axis(Dhat, D_c[..., None].astype(np.int64), 800.0, axis=2)
    assert np.array_equal(oracle.bake_probes(Dhat), D_c)
    yh, _ = oracle.encode_fwd(w, x, D_f, D_c)
    assert np.allclose(oracle.encode_soft_fwd(w, x, D_f, Dhat), yh, rtol=0, atol=1e-15)
    gDf, gDc, _, _ = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    assert np.allclose(gDc, 0.0, atol=1e-15)
    # gradient of the hard forward <y(D_f), dy> by finite differences (it is linear in D_f)
    for idx in np.argsort(-np.abs(gDf).ravel())[:6]:
        i = np.unravel_index(idx, gDf.shape)
        Dp = D_f.copy(); Dp[i] += 1.0
        fd = float(np.sum((oracle.encode_fwd(w, x, Dp, D_c)[0] - yh) * dy))
        assert abs(fd - gDf[i]) <= 1e-10 * max(1.0, abs(fd))


def test_probe_range_one_backward_is_hash_grid_backward():
    """N_p = 1: sigma = 1, the logit gradient is zero and gD_f is the scatter of weight * dy."""
    w = small(d=2, N_p=1, N_c=8, N_f=32, L=2)
    x, D_f, Dhat, dy = random_tables(w, seed=29)
    gDf, gDc, _, _ = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    assert np.all(gDc == 0.0)
    base, _, _, fidx, wt = oracle.indices(w, x, None, want_weight=True)
    want = np.zeros_like(gDf)
    for n in range(w.N):
        for l in range(w.L):
            for c in range(4):
                want[l, fidx[n, l, c]] += wt[n, l, c] * dy[n, l * w.F:(l + 1) * w.F]
    assert np.allclose(gDf, want, rtol=0, atol=1e-13)


# --------------------------------------------------------------------------- sparse (top-k) variant

def kept_sets(Dhat, k):
    """The k largest entries of each row, equal values by lowest index: numpy's stable sort of the negated row."""
    order = np.argsort(-Dhat.astype(np.float64), axis=-1, kind="stable")[..., :k]
    keep = np.zeros(Dhat.shape, bool)
    np.put_along_axis(keep, order, True, axis=-1)
    return keep


@pytest.mark.parametrize("top_k", [1, 2, 4])
def test_top_k_forward_is_softmax_over_the_kept_set(top_k):
    """With N_c = 1 the relaxed forward is the mix of the hard forwards of the kept candidates, weighted by the
    softmax among them (written out here with numpy); rows with equal values keep the lower indices."""
    w = small(d=2, N_c=1, N_p=8, L=2)
    x, D_f, Dhat, _ = random_tables(w, seed=41)
    Dhat = Dhat.copy()
    Dhat[1, 0, 5] = Dhat[1, 0, 2] = Dhat[1, 0].max() + 1.0          # a tie for the first place on level 1
    keep = kept_sets(Dhat, top_k)
    assert keep[1, 0, 2] and (top_k > 1) == bool(keep[1, 0, 5])
    ys = oracle.encode_soft_fwd(w, x, D_f, Dhat, top_k=top_k)
    mix = np.zeros_like(ys)
    for l in range(w.L):
        e = np.where(keep[l, 0], np.exp(Dhat[l, 0].astype(np.float64)), 0.0); s = e / e.sum()
        for k in range(w.N_p):
            D_c = np.zeros((w.L, 1), np.uint8); D_c[l, 0] = k
            yk, _ = oracle.encode_fwd(w, x, D_f, D_c)
            mix[:, l * w.F:(l + 1) * w.F] += s[k] * yk[:, l * w.F:(l + 1) * w.F]
    assert np.allclose(ys, mix, rtol=0, atol=1e-14)


@pytest.mark.parametrize("d,top_k", [(2, 2), (3, 4), (3, 3)])
def test_top_k_backward_matches_finite_differences_and_invariants(d, top_k):
    """Gradient of the top-k relaxed forward with the kept sets held fixed (small steps do not change them for
    generic values), zero outside the kept sets, and the invariants of the dense variant."""
    w = small(d=d, N=120)
    x, D_f, Dhat, dy = random_tables(w, seed=43)
    Dh64 = Dhat.astype(np.float64)
    gDf, gDc, Af, Ac = oracle.encode_bwd(w, x, D_f, Dhat, dy, top_k=top_k)
    keep = kept_sets(Dhat, top_k)
    assert np.all(gDc[~keep] == 0.0) and np.all(Ac[~keep] == 0.0)
    assert np.count_nonzero(gDc) > 0.5 * np.count_nonzero(oracle.encode_bwd(w, x, D_f, Dhat, dy)[1]) * top_k / w.N_p
    assert np.allclose(gDc.sum(axis=2), 0.0, rtol=0, atol=1e-12)
    assert np.allclose(gDf.sum(axis=1), dy.reshape(w.N, w.L, w.F).sum(axis=0), rtol=0, atol=1e-11)
    lhs = float(np.sum(oracle.encode_soft_fwd(w, x, D_f, Dhat, top_k=top_k) * dy))
    assert abs(lhs - float(np.sum(D_f * gDf))) <= 1e-12 * max(1.0, abs(lhs))

    def loss(Df, Dh):
        return float(np.sum(oracle.encode_soft_fwd(w, x, Df, Dh, top_k=top_k) * dy))
    rng = np.random.default_rng(2)
    for idx in np.argsort(-np.abs(gDf).ravel())[:5].tolist() + rng.integers(0, gDf.size, 4).tolist():
        i = np.unravel_index(idx, gDf.shape)
        Dp = D_f.copy(); Dp[i] += 1e-3
        Dm = D_f.copy(); Dm[i] -= 1e-3
        fd = (loss(Dp, Dh64) - loss(Dm, Dh64)) / 2e-3
        assert abs(fd - gDf[i]) <= 1e-8 * max(1.0, abs(gDf[i]))
    for idx in np.argsort(-np.abs(gDc).ravel())[:8].tolist() + rng.integers(0, gDc.size, 6).tolist():
        i = np.unravel_index(idx, gDc.shape)
        row = np.sort(Dh64[i[0], i[1]])
        if np.min(np.diff(row)) < 1e-3:
            continue                                              # a step could reorder this row
        Dp = Dh64.copy(); Dp[i] += 1e-5
        Dm = Dh64.copy(); Dm[i] -= 1e-5
        fd = (loss(D_f, Dp) - loss(D_f, Dm)) / 2e-5
        assert abs(fd - gDc[i]) <= 1e-6 * max(1.0, abs(gDc[i]))


def test_top_k_limits():
    """top_k = N_p (or 0) is the paper's softmax; top_k = 1 is training of the hard forward: no logit gradient, the
    feature gradient of the baked codebook; a NaN confidence is never kept while a number is left."""
    w = small(d=3)
    x, D_f, Dhat, dy = random_tables(w, seed=47)
    full = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    for k in (0, w.N_p, w.N_p + 3):
        g = oracle.encode_bwd(w, x, D_f, Dhat, dy, top_k=k)
        assert all(np.array_equal(a, b) for a, b in zip(g, full))
    g1 = oracle.encode_bwd(w, x, D_f, Dhat, dy, top_k=1)
    assert np.all(g1[1] == 0.0)
    D_c = oracle.bake_probes(Dhat)
    yh, _ = oracle.encode_fwd(w, x, D_f, D_c)
    assert np.allclose(oracle.encode_soft_fwd(w, x, D_f, Dhat, top_k=1), yh, rtol=0, atol=1e-15)
    for idx in np.argsort(-np.abs(g1[0]).ravel())[:6]:
        i = np.unravel_index(idx, g1[0].shape)
        Dp = D_f.copy(); Dp[i] += 1.0
        fd = float(np.sum((oracle.encode_fwd(w, x, Dp, D_c)[0] - yh) * dy))
        assert abs(fd - g1[0][i]) <= 1e-10 * max(1.0, abs(fd))
    bad = Dhat.astype(np.float64).copy()
    bad[:, :, 0] = np.nan                                         # candidate 0 is never among the kept two
    g2 = oracle.encode_bwd(w, x, D_f, bad, dy, top_k=2)
    assert np.all(np.isfinite(g2[0])) and np.all(g2[1][:, :, 0] == 0.0) and np.all(g2[0].reshape(w.L, -1, w.N_p, w.F)[:, :, 0] == 0.0)


# --------------------------------------------------------------------------- bake

def test_bake_properties():
    rng = np.random.default_rng(31)
    for N_p in (1, 2, 4, 8, 16):
        Dhat = rng.standard_normal((3, 50, N_p)).astype(np.float32)
        D_c = oracle.bake_probes(Dhat)
        assert D_c.dtype == np.uint8 and D_c.shape == (3, 50)
        assert D_c.max() < N_p                                   # D_c in {0..N_p-1} (Sec. 3)
        assert np.array_equal(D_c, np.argmax(Dhat, axis=2))
        assert np.array_equal(oracle.bake_probes(Dhat * 3.0 + 5.0), D_c)      # shift / positive scale
        hot = rng.integers(0, N_p, (3, 50))
        onehot = np.zeros((3, 50, N_p), np.float32)
        np.put_along_axis(onehot, hot[..., None], 1.0, axis=2)
        assert np.array_equal(oracle.bake_probes(onehot), hot)


def test_bake_ties_and_nan():
    rows = np.array([[1, 1, 1, 1], [0, 2, 2, 1], [np.nan, 0, np.nan, 0], [np.nan] * 4,
                     [-np.inf, -np.inf, -np.inf, -np.inf], [np.nan, -np.inf, 3, 3]], np.float32)
    assert oracle.bake_probes(rows).tolist() == [0, 1, 1, 0, 0, 2]


# --------------------------------------------------------------------------- exact-width index storage

@pytest.mark.parametrize("N_p", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("N_c", [1, 2, 8, 16, 32, 128])
def test_index_bit_packing_is_the_little_endian_integer(N_p, N_c):
    """A level's bit string read as one little-endian integer is sum_r D_c[r] * N_p^r (entry r at bit r b)."""
    rng = np.random.default_rng(N_p * 1000 + N_c)
    D_c = rng.integers(0, N_p, (3, N_c)).astype(np.uint8)
    packed = oracle.pack_index_bits(D_c, N_p)
    b = N_p.bit_length() - 1
    assert packed.shape == (3, 4 * ((N_c * b + 31) // 32))
    for l in range(3):
        assert int.from_bytes(packed[l].tobytes(), "little") == sum(int(v) * N_p ** r for r, v in enumerate(D_c[l]))
    assert np.array_equal(oracle.unpack_index_bits(packed, N_c, N_p), D_c)


def test_storage_bytes_against_table_3():
    """The model sizes of Table 3 (which also hold an MLP and, apparently, smaller coarse levels) lie a
    little below the bytes of 16 levels of fp16 features and exact-width indices."""
    for line in open(os.path.join(GOLDEN, "table3_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        _, N_f, N_c, N_p, kB = line.split()
        w = W.custom(d=3, L=16, N_f=int(N_f), N_c=int(N_c), N_p=int(N_p), N_min=16, N_max=2048, N=16, feat_dtype="f16")
        sb = oracle.storage_bytes(w)
        total = (sb["D_f"] + sb["D_c"]) / 1000.0
        assert 0.8 * total <= float(kB) <= total, (line, total)
    # the paper's row: 2^8 features, 2^16 three-bit indices per level
    w = W.custom(d=3, L=16, N_f=256, N_c=65536, N_p=8, N_min=16, N_max=2048, N=16, feat_dtype="f16")
    assert oracle.storage_bytes(w) == {"D_f": 16 * 256 * 2 * 2, "D_c_level": 65536 * 3 // 8, "D_c": 16 * 65536 * 3 // 8}


# --------------------------------------------------------------------------- optimiser step (assumed: Adam)

def test_adam_closed_forms():
    rng = np.random.default_rng(41)
    g = rng.standard_normal(64); theta = rng.standard_normal(64); z = np.zeros(64)
    lr, b1, b2, eps = 1e-2, 0.9, 0.99, 1e-8
    # first step from zero state: m_hat = g, v_hat = g^2, so the step is lr * g / (|g| + eps)
    t1, m1, v1 = oracle.adam_step(theta, z, z, g, lr, b1, b2, eps, 1)
    assert np.allclose(t1, theta - lr * g / (np.abs(g) + eps), rtol=0, atol=1e-15)
    assert np.allclose(m1, (1 - b1) * g) and np.allclose(v1, (1 - b2) * g * g)
    # constant gradient: bias correction makes every step identical
    th, m, v = theta, z, z
    for t in range(1, 8):
        th, m, v = oracle.adam_step(th, m, v, g, lr, b1, b2, eps, t)
    assert np.allclose(th, theta - 7 * lr * g / (np.abs(g) + eps), rtol=0, atol=1e-13)
    # zero gradient, zero state: nothing moves; eps = 0: the step is invariant to the gradient's scale
    t0, m0, v0 = oracle.adam_step(theta, z, z, np.zeros(64), lr, b1, b2, eps, 3)
    assert np.array_equal(t0, theta) and not m0.any() and not v0.any()
    a = oracle.adam_step(theta, z, z, g, lr, b1, b2, 0.0, 1)[0]
    b = oracle.adam_step(theta, z, z, 1000.0 * g, lr, b1, b2, 0.0, 1)[0]
    assert np.allclose(a, b, rtol=0, atol=1e-15)


def test_adam_matches_library_optimiser():
    """Several steps with changing gradients against torch.optim.Adam in fp64."""
    import torch
    rng = np.random.default_rng(43)
    theta0 = rng.standard_normal(200)
    lr, b1, b2, eps = 3e-3, 0.9, 0.99, 1e-15
    par = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.Adam([par], lr=lr, betas=(b1, b2), eps=eps)
    th, m, v = theta0, np.zeros(200), np.zeros(200)
    for t in range(1, 6):
        g = rng.standard_normal(200) * (10.0 ** rng.integers(-4, 2))
        par.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v = oracle.adam_step(th, m, v, g, lr, b1, b2, eps, t)
        assert np.allclose(th, par.detach().numpy(), rtol=1e-12, atol=1e-14)


# --------------------------------------------------------------------------- gradient with respect to the points

@pytest.mark.parametrize("d", [2, 3, 4])
def test_input_gradient_is_the_derivative_of_the_pinned_forward(d):
    """Central differences of the hard forward (pinned above by brute force) at points well inside their
    cells on every level: the forward is d-linear there, so a small step stays exact up to rounding."""
    w = small(d=d, L=3, N_min=3, N_max=19, N=400, N_f=256, N_c=64, N_p=8)
    rng = np.random.default_rng(11)
    x, D_f, Dhat, dy = random_tables(w, seed=5)
    D_c = oracle.bake_probes(Dhat)
    res = oracle.level_resolutions(w.N_min, w.N_max, w.L).astype(np.float64)
    h = 1e-4
    frac = (x[:, None, :].astype(np.float64) * res[None, :, None]) % 1.0
    inside = ((frac > 0.05) & (frac < 0.95)).all(axis=(1, 2))
    assert inside.sum() > 50
    x = x[inside]
    gx, gmag = oracle.encode_bwd_input(w, x, D_f, D_c, dy[inside])
    for j in range(d):
        e = np.zeros(d, np.float64); e[j] = h
        up, _ = oracle.encode_fwd(w, (x.astype(np.float64) + e).astype(np.float32), D_f, D_c)
        dn, _ = oracle.encode_fwd(w, (x.astype(np.float64) - e).astype(np.float32), D_f, D_c)
        step = ((x.astype(np.float64) + e).astype(np.float32).astype(np.float64)
                - (x.astype(np.float64) - e).astype(np.float32).astype(np.float64))[:, j]
        fd = ((up - dn) * dy[inside]).sum(axis=1) / step
        assert np.allclose(fd, gx[:, j], rtol=0, atol=2e-3 * gmag[:, j].max()), j
    assert np.all(gmag >= np.abs(gx) - 1e-9)


def test_input_gradient_closed_forms():
    w = small(d=3, L=2, N_min=4, N_max=16, N=100)
    x, D_f, Dhat, dy = random_tables(w, seed=8)
    D_c = oracle.bake_probes(Dhat)
    # a constant codebook interpolates to a constant: no gradient (the weights' derivatives sum to zero)
    gx, _ = oracle.encode_bwd_input(w, x, np.full_like(D_f, 0.7), D_c, dy)
    assert np.allclose(gx, 0.0, atol=1e-9)
    # linear in dL/dy and in the features
    g1, _ = oracle.encode_bwd_input(w, x, D_f, D_c, dy)
    g2, _ = oracle.encode_bwd_input(w, x, 3.0 * D_f, D_c, -2.0 * dy)
    assert np.allclose(g2, -6.0 * g1, rtol=1e-12, atol=1e-12)
    # one level, d = 2, one output: the x-derivative is N_l * ((1 - fy) (f10 - f00) + fy (f11 - f01))
    w1 = small(d=2, L=1, N_min=8, N_max=8, N=50)
    x, D_f, Dhat, dy = random_tables(w1, seed=9)
    D_c = oracle.bake_probes(Dhat)
    dy[:, 1] = 0.0
    *_, fidx = oracle.indices(w1, x, D_c)
    f = D_f[0, fidx[:, 0, :], 0]                      # [N, 4 corners], corner c = (c & 1) + 2 * (c >> 1 & 1)
    fy = (x[:, 1].astype(np.float32) * np.float32(8)).astype(np.float64) % 1.0
    want = 8.0 * ((1 - fy) * (f[:, 1] - f[:, 0]) + fy * (f[:, 3] - f[:, 2])) * dy[:, 0]
    got, _ = oracle.encode_bwd_input(w1, x, D_f, D_c, dy)
    assert np.allclose(got[:, 0], want, rtol=1e-10, atol=1e-12)


# --------------------------------------------------------------------------- decoder (assumed: 2 hidden ReLU layers)

def _mlp_case(seed, N=50, n_in=16, n_out=3):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((N, n_in)), rng.standard_normal((64, n_in)) * 0.3,
            rng.standard_normal((64, 64)) * 0.2, rng.standard_normal((n_out, 64)) * 0.2,
            rng.standard_normal((N, n_out)))


def test_mlp_matches_library_autograd():
    import torch
    y, W1, W2, W3, dout = _mlp_case(0)
    t = [torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (y, W1, W2, W3)]
    out = torch.relu(torch.relu(t[0] @ t[1].T) @ t[2].T) @ t[3].T
    out.backward(torch.tensor(dout))
    assert np.allclose(oracle.mlp_fwd(y, W1, W2, W3), out.detach().numpy(), rtol=1e-12, atol=1e-13)
    g, mag, _ = oracle.mlp_bwd(y, W1, W2, W3, dout)
    for name, ref in zip(("dy", "dW1", "dW2", "dW3"), t):
        assert np.allclose(g[name], ref.grad.numpy(), rtol=1e-11, atol=1e-12), name
        assert np.all(mag[name] >= np.abs(g[name]) - 1e-12)


def test_mlp_linear_regime_and_finite_differences():
    rng = np.random.default_rng(1)
    # all-positive inputs and weights: no unit is ever clipped, the network is the product of its matrices
    y, W1, W2, W3 = rng.random((20, 8)), rng.random((64, 8)), rng.random((64, 64)), rng.random((3, 64))
    assert np.allclose(oracle.mlp_fwd(y, W1, W2, W3), y @ (W3 @ W2 @ W1).T, rtol=1e-12)
    out, mag, _ = oracle.mlp_fwd(y, W1, W2, W3, want_mag=True)
    assert np.allclose(out, mag)
    # central differences of L = sum(out * dout) in every argument
    y, W1, W2, W3, dout = _mlp_case(2, N=6, n_in=8)
    g, _, _ = oracle.mlp_bwd(y, W1, W2, W3, dout)
    args = {"dy": y, "dW1": W1, "dW2": W2, "dW3": W3}
    loss = lambda: float((oracle.mlp_fwd(y, W1, W2, W3) * dout).sum())
    for name, arr in args.items():
        for idx in [tuple(rng.integers(0, s) for s in arr.shape) for _ in range(12)]:
            old = arr[idx]; h = 1e-6
            arr[idx] = old + h; up = loss()
            arr[idx] = old - h; dn = loss()
            arr[idx] = old
            assert abs((up - dn) / (2 * h) - g[name][idx]) < 1e-6 * max(1.0, abs(g[name][idx])), (name, idx)


# --------------------------------------------------------------------------- storage conventions

def test_model_sizes_consistent_with_table_3():
    """Table 3's file sizes fix the storage conventions by arithmetic: one codebook pair per level,
    F = 2 half-precision features, log2(N_p)-bit probe indices.  The printed sizes (which also hold
    an MLP and, apparently, smaller coarse levels) are a little below L * (2 F N_f + N_c log2 N_p / 8)."""
    for line in open(os.path.join(GOLDEN, "table3_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        _, N_f, N_c, N_p, kB = line.split()
        N_f, N_c, N_p, kB = int(N_f), int(N_c), int(N_p), float(kB)
        bits = N_p.bit_length() - 1
        full = 16 * (N_f * 2 * 2 + N_c * bits / 8) / 1000.0
        assert 0.8 * full <= kB <= full


# --------------------------------------------------------------------------- Morton order (optional reordering)

def test_morton_codes_by_hand_and_by_string_interleaving():
    # 2D, 10 bits per axis: q = (3, 5) -> x bits 011, y bits 101 -> y2 x2 y1 x1 y0 x0 = 1 0 0 1 1 1 = 39
    s = 1.0 / 1024
    pts = np.array([[0, 0], [1.5 * s, 0], [0, 1.5 * s], [3.2 * s, 5.9 * s], [1.0, 1.0], [-0.5, 2.0]], np.float32)
    _, codes = oracle.morton_order(pts)
    assert codes.tolist() == [0, 1, 2, 39, 2**20 - 1, int("10" * 10, 2)]
    # 3D, 7 bits per axis: q = (1, 0, 0), (0, 1, 0), (0, 0, 1), (127, 127, 127)
    t = 1.0 / 128
    pts3 = np.array([[1.1 * t, 0, 0], [0, 1.1 * t, 0], [0, 0, 1.1 * t], [1, 1, 1], [2.5 * t, 0, 3.5 * t]], np.float32)
    _, codes3 = oracle.morton_order(pts3)
    assert codes3.tolist() == [1, 2, 4, 2**21 - 1, int("101100", 2)]               # q = (2, 0, 3): z1 y1 x1 z0 y0 x0 = 1 0 1 1 0 0
    # 4D, 5 bits per axis: single low bits of each axis, the corner of the cube, q = (0, 3, 0, 1): w0 = 8, y0 = 2, y1 = 32
    u = 1.0 / 32
    pts4 = np.array([[1.1 * u, 0, 0, 0], [0, 1.1 * u, 0, 0], [0, 0, 1.1 * u, 0], [0, 0, 0, 1.1 * u], [1, 1, 1, 1], [0, 3.5 * u, 0, 1.5 * u]], np.float32)
    _, codes4 = oracle.morton_order(pts4)
    assert codes4.tolist() == [1, 2, 4, 8, 2**20 - 1, 8 + 2 + 32]
    rng = np.random.default_rng(5)
    for d, B in ((2, 10), (3, 7), (4, 5)):
        x = rng.random((500, d), dtype=np.float32)
        perm, codes = oracle.morton_order(x)
        q = np.minimum((x.astype(np.float64) * (1 << B)).astype(np.int64), (1 << B) - 1)
        for n in range(0, 500, 7):                               # bit strings, most significant first
            bits = "".join(format(int(q[n, j]), f"0{B}b")[B - 1 - b] for b in reversed(range(B)) for j in reversed(range(d)))
            assert int(bits, 2) == int(codes[n])
        assert sorted(perm.tolist()) == list(range(500))
        assert np.all(np.diff(codes[perm].astype(np.int64)) >= 0)
        same = codes[perm][1:] == codes[perm][:-1]
        assert np.all(perm[1:][same] > perm[:-1][same])          # stable: equal codes keep the order of the batch


def test_morton_order_keeps_cells_together():
    """Points of one cell of the 2^k grid form one contiguous run of the order (the prefix property of the curve)."""
    rng = np.random.default_rng(6)
    x = rng.random((4000, 3), dtype=np.float32)
    perm, _ = oracle.morton_order(x)
    for k in (1, 2, 4):
        cell = np.floor(x[perm].astype(np.float64) * (1 << k)).astype(np.int64)
        ident = (cell[:, 0] * 64 + cell[:, 1]) * 64 + cell[:, 2]
        runs = 1 + np.count_nonzero(np.diff(ident))
        assert runs == len(np.unique(ident))


# --------------------------------------------------------------------------- tolerance scales, pinned from above
# The GPU comparisons divide by magnitude sums the oracle returns (ymag, A_f, A_c, gmag, the decoder's
# magnitudes).  The tests above bound them from below (magnitude >= |value|); a magnitude that came out too
# large would loosen every comparison silently, so here each one is fixed exactly: by an identity of the
# definition, by a regime in which no term cancels (magnitude == value), or by a written-out evaluation.

def test_ymag_equals_value_without_cancellation():
    w = small(d=3)
    x, D_f, Dhat, _ = random_tables(w, seed=31)
    D_c = oracle.bake_probes(Dhat)
    y, ymag = oracle.encode_fwd(w, x, np.abs(D_f), D_c)              # non-negative codebook: nothing cancels
    assert np.allclose(ymag, y, rtol=1e-14, atol=0)
    y, ymag = oracle.encode_fwd(w, x, -np.abs(D_f), D_c)
    assert np.allclose(ymag, -y, rtol=1e-14, atol=0)
    y, ymag = oracle.encode_fwd(w, x, np.full_like(D_f, -0.375), D_c)   # constant codebook: the weights sum to one
    assert np.allclose(ymag, 0.375, rtol=0, atol=1e-15)


@pytest.mark.parametrize("d", [2, 3, 4])
def test_feature_gradient_magnitude_mass_and_no_cancellation(d):
    w = small(d=d)
    x, D_f, Dhat, dy = random_tables(w, seed=37)
    _, _, Af, _ = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    # interpolation weights and softmax weights are non-negative and each sum to one
    want = np.abs(dy).reshape(w.N, w.L, w.F).sum(axis=0)
    assert np.allclose(Af.sum(axis=1), want, rtol=1e-11, atol=0)
    gDf, _, Af, _ = oracle.encode_bwd(w, x, D_f, Dhat, np.abs(dy))      # dy >= 0: every term is >= 0
    assert np.allclose(Af, gDf, rtol=1e-13, atol=0)
    for top_k in (1, 2):
        gDf, _, Af, _ = oracle.encode_bwd(w, x, D_f, Dhat, np.abs(dy), top_k=top_k)
        assert np.allclose(Af, gDf, rtol=1e-13, atol=0)
        assert np.allclose(Af.sum(axis=1), want, rtol=1e-11, atol=0)


@pytest.mark.parametrize("d", [2, 3, 4])
def test_logit_gradient_magnitude_written_out(d):
    """dy >= 0 and D_f >= 0: q_k >= 0, so the magnitude of the term sigma_k (q_k - qbar) is sigma_k (q_k + qbar).
    Evaluated here with numpy from the index dump (pinned above) and a library softmax."""
    from scipy.special import softmax
    w = small(d=d)
    x, D_f, Dhat, dy = random_tables(w, seed=41)
    D_f, dy = np.abs(D_f), np.abs(dy)
    gDf, gDc, _, Ac = oracle.encode_bwd(w, x, D_f, Dhat, dy)
    base, h2, _, _, weight = oracle.indices(w, x, None, want_weight=True)
    want = np.zeros_like(Ac)
    sig = softmax(Dhat.astype(np.float64), axis=2)
    for n, l, c in itertools.product(range(w.N), range(w.L), range(1 << d)):
        g = weight[n, l, c] * dy[n, l * w.F:(l + 1) * w.F]
        s = sig[l, h2[n, l, c]]
        q = D_f[l, base[n, l, c]:base[n, l, c] + w.N_p] @ g
        want[l, h2[n, l, c]] += s * (q + s @ q)
    assert np.allclose(Ac, want, rtol=1e-12, atol=0)
    # and in general: the magnitude depends on |D_f|, |dy| only
    x, D_f2, _, dy2 = random_tables(w, seed=43)
    a = oracle.encode_bwd(w, x, D_f2, Dhat, dy2)
    b = oracle.encode_bwd(w, x, np.abs(D_f2), Dhat, np.abs(dy2))
    assert np.allclose(a[2], b[2], rtol=1e-13, atol=0) and np.allclose(a[3], b[3], rtol=1e-13, atol=0)


def test_input_gradient_magnitude_closed_form():
    """One level, d = 2, one output column: gmag_x = N_l ((1 - fy)(|f00 g| + |f10 g|) + fy (|f01 g| + |f11 g|))."""
    w1 = small(d=2, L=1, N_min=8, N_max=8, N=50)
    x, D_f, Dhat, dy = random_tables(w1, seed=9)
    D_c = oracle.bake_probes(Dhat)
    dy[:, 1] = 0.0
    *_, fidx = oracle.indices(w1, x, D_c)
    f = np.abs(D_f[0, fidx[:, 0, :], 0] * dy[:, :1])
    fx = (x[:, 0].astype(np.float32) * np.float32(8)).astype(np.float64) % 1.0
    fy = (x[:, 1].astype(np.float32) * np.float32(8)).astype(np.float64) % 1.0
    _, gmag = oracle.encode_bwd_input(w1, x, D_f, D_c, dy)
    assert np.allclose(gmag[:, 0], 8.0 * ((1 - fy) * (f[:, 0] + f[:, 1]) + fy * (f[:, 2] + f[:, 3])), rtol=1e-12)
    assert np.allclose(gmag[:, 1], 8.0 * ((1 - fx) * (f[:, 0] + f[:, 2]) + fx * (f[:, 1] + f[:, 3])), rtol=1e-12)


def test_mlp_magnitudes_equal_values_without_cancellation():
    rng = np.random.default_rng(3)
    y, W1, W2, W3, dout = rng.random((20, 8)), rng.random((64, 8)), rng.random((64, 64)), rng.random((3, 64)), rng.random((20, 3))
    out, mag, _ = oracle.mlp_fwd(y, W1, W2, W3, want_mag=True)
    assert np.allclose(mag, out, rtol=1e-13, atol=0)
    g, gm, _ = oracle.mlp_bwd(y, W1, W2, W3, dout)
    for name in ("dy", "dW1", "dW2", "dW3"):
        assert np.allclose(gm[name], g[name], rtol=1e-13, atol=0), name
    # signs flipped in the last layer and upstream: magnitudes unchanged, values negated or kept
    g2, gm2, _ = oracle.mlp_bwd(y, W1, W2, W3, -dout)
    for name in ("dy", "dW1", "dW2", "dW3"):
        assert np.allclose(gm2[name], gm[name], rtol=1e-13, atol=0) and np.allclose(g2[name], -g[name], rtol=1e-13, atol=0)


# --------------------------------------------------------------------------- memory safety of the oracle itself

def test_oracle_runs_clean_under_sanitizers():
    """oracle/sanitize_main.c calls every oracle function on small inputs (both dimensions, every probing range,
    F = 1, 2, 4, the sparse variant, NaN and infinite confidences, the cube's corners) in a program built with
    AddressSanitizer and UndefinedBehaviorSanitizer: an out-of-bounds index or an overflowing conversion aborts it."""
    import subprocess
    import sys
    sys.path.insert(0, os.path.join(os.path.dirname(GOLDEN), "..", "oracle"))
    from oracle.build import build_sanitized
    exe = build_sanitized()
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0 and "clean" in res.stdout, res.stdout + res.stderr

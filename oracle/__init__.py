"""CPU oracle of the Compact NGP encoding path.  TEST INFRASTRUCTURE ONLY.

Thin ctypes marshalling around oracle/cngp_oracle.c (plain C, fp64).  Only
tests, the smoke check and the benchmark's CPU-baseline leg import this
package; the product package never does, and this package never imports the
product.  All arithmetic lives in the C file; this file converts arrays and
threads shapes through; the storage convention of the index codebook and the decoder that
follows the encoding (oracle/mlp.py) are a few lines of plain numpy.
"""
import ctypes
import os

import numpy as np

from .build import build as _build
from .mlp import mlp_bwd, mlp_fwd  # noqa: F401

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build())
        _lib.cngp_oracle_level_resolutions.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u32(v):
    return ctypes.c_uint32(int(v))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle use, as the OpenMP runtime reports them."""
    f = lib().cngp_oracle_max_threads
    f.restype = ctypes.c_int
    return int(f())


def set_threads(n: int) -> None:
    """Number of threads for the following oracle calls (the timing of the oracle on one core)."""
    lib().cngp_oracle_set_threads(ctypes.c_int(int(n)))


def level_resolutions(N_min, N_max, L) -> np.ndarray:
    out = np.zeros(L, dtype=np.uint32)
    rc = lib().cngp_oracle_level_resolutions(_u32(N_min), _u32(N_max), ctypes.c_int(L), _p(out))
    if rc != 0:
        raise ValueError("invalid N_min / N_max / L")
    return out


def _res(w, res):
    if res is None:
        res = level_resolutions(w.N_min, w.N_max, w.L)
    res = np.ascontiguousarray(res, dtype=np.uint32)
    assert res.shape == (w.L,)
    return res


def _x(w, x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.ndim == 2 and x.shape[1] == w.d
    return x


def indices(w, x, D_c=None, res=None, want_weight=False):
    """base, h2, probe, feat_idx as [N, L, 2^d] arrays (and the weights if asked)."""
    x = _x(w, x); res = _res(w, res)
    N = x.shape[0]
    shp = (N, w.L, 1 << w.d)
    base = np.zeros(shp, np.uint32); h2 = np.zeros(shp, np.uint32)
    probe = np.zeros(shp, np.uint8); fidx = np.zeros(shp, np.uint32)
    wt = np.zeros(shp, np.float64) if want_weight else None
    if D_c is not None:
        D_c = np.ascontiguousarray(D_c, dtype=np.uint8)
        assert D_c.shape == (w.L, w.N_c)
    lib().cngp_oracle_indices(w.d, w.L, _u32(w.N_f), _u32(w.N_c), _u32(w.N_p), _p(res), _p(x),
                              ctypes.c_int64(N), _p(D_c), _p(base), _p(h2), _p(probe), _p(fidx), _p(wt))
    return (base, h2, probe, fidx, wt) if want_weight else (base, h2, probe, fidx)


def encode_fwd(w, x, D_f, D_c, res=None):
    """Hard forward.  Returns (y, ymag), both float64 [N, L*F]."""
    x = _x(w, x); res = _res(w, res)
    N = x.shape[0]
    D_f = _f64(D_f); assert D_f.shape == (w.L, w.N_f, w.F)
    D_c = np.ascontiguousarray(D_c, dtype=np.uint8); assert D_c.shape == (w.L, w.N_c)
    assert int(D_c.max(initial=0)) < w.N_p
    y = np.zeros((N, w.L * w.F)); ymag = np.zeros((N, w.L * w.F))
    lib().cngp_oracle_encode_fwd(w.d, w.L, w.F, _u32(w.N_f), _u32(w.N_c), _u32(w.N_p), _p(res),
                                 _p(x), ctypes.c_int64(N), _p(D_f), _p(D_c), _p(y), _p(ymag))
    return y, ymag


def encode_fwd_partial(w, levels_loaded, x, D_f, D_c):
    """Forward from a partially loaded model (level-of-detail streaming): the first `levels_loaded` levels
    of the full model's level table are evaluated, the remaining columns are zero."""
    import dataclasses
    res = level_resolutions(w.N_min, w.N_max, w.L)
    N = np.asarray(x).shape[0]
    y = np.zeros((N, w.L * w.F)); ymag = np.zeros((N, w.L * w.F))
    if levels_loaded > 0:
        sub = dataclasses.replace(w, L=levels_loaded)
        ys, ms = encode_fwd(sub, x, np.asarray(D_f)[:levels_loaded], np.asarray(D_c)[:levels_loaded], res=res[:levels_loaded])
        y[:, :levels_loaded * w.F] = ys
        ymag[:, :levels_loaded * w.F] = ms
    return y, ymag


def encode_bwd_input(w, x, D_f, D_c, dy, res=None):
    """Gradient of the hard forward with respect to the points.  Returns (dL/dx, magnitude), float64 [N, d]."""
    x = _x(w, x); res = _res(w, res)
    N = x.shape[0]
    D_f = _f64(D_f); assert D_f.shape == (w.L, w.N_f, w.F)
    D_c = np.ascontiguousarray(D_c, dtype=np.uint8); assert D_c.shape == (w.L, w.N_c)
    dy = _f64(dy); assert dy.shape == (N, w.L * w.F)
    gx = np.zeros((N, w.d)); gmag = np.zeros((N, w.d))
    lib().cngp_oracle_encode_bwd_input(w.d, w.L, w.F, _u32(w.N_f), _u32(w.N_c), _u32(w.N_p), _p(res),
                                       _p(x), ctypes.c_int64(N), _p(D_f), _p(D_c), _p(dy), _p(gx), _p(gmag))
    return gx, gmag


def encode_soft_fwd(w, x, D_f, Dhat_c, res=None, top_k=0):
    """Softmax-relaxed forward (test helper): float64 [N, L*F].  top_k > 0: only the top_k largest confidence
    values of a row keep (softmax) weight."""
    x = _x(w, x); res = _res(w, res)
    N = x.shape[0]
    D_f = _f64(D_f); assert D_f.shape == (w.L, w.N_f, w.F)
    Dhat_c = _f64(Dhat_c); assert Dhat_c.shape == (w.L, w.N_c, w.N_p)
    y = np.zeros((N, w.L * w.F))
    lib().cngp_oracle_encode_soft_fwd(w.d, w.L, w.F, _u32(w.N_f), _u32(w.N_c), _u32(w.N_p), _p(res),
                                      _p(x), ctypes.c_int64(N), _p(D_f), _p(Dhat_c), _u32(top_k), _p(y))
    return y


def encode_bwd(w, x, D_f, Dhat_c, dy, res=None, want_abs=True, top_k=0):
    """Backward.  Returns (gD_f, gDhat_c, A_f, A_c) in float64 (A_* None if not asked).  top_k > 0: the sparse
    variant, gradient through the top_k largest confidence values of a row only."""
    x = _x(w, x); res = _res(w, res)
    N = x.shape[0]
    D_f = _f64(D_f); assert D_f.shape == (w.L, w.N_f, w.F)
    Dhat_c = _f64(Dhat_c); assert Dhat_c.shape == (w.L, w.N_c, w.N_p)
    dy = _f64(dy); assert dy.shape == (N, w.L * w.F)
    gDf = np.zeros_like(D_f); gDc = np.zeros_like(Dhat_c)
    Af = np.zeros_like(D_f) if want_abs else None
    Ac = np.zeros_like(Dhat_c) if want_abs else None
    lib().cngp_oracle_encode_bwd(w.d, w.L, w.F, _u32(w.N_f), _u32(w.N_c), _u32(w.N_p), _p(res),
                                 _p(x), ctypes.c_int64(N), _p(D_f), _p(Dhat_c), _p(dy), _u32(top_k),
                                 _p(gDf), _p(gDc), _p(Af), _p(Ac))
    return gDf, gDc, Af, Ac


def bake_probes(Dhat_c) -> np.ndarray:
    """argmax along the last axis, uint8, same leading shape."""
    Dhat_c = np.ascontiguousarray(Dhat_c, dtype=np.float32)
    N_p = Dhat_c.shape[-1]
    rows = Dhat_c.size // N_p if N_p else 0
    out = np.zeros(Dhat_c.shape[:-1], dtype=np.uint8)
    lib().cngp_oracle_bake_probes(_p(Dhat_c), ctypes.c_int64(rows), _u32(N_p), _p(out))
    return out


def adam_step(theta, m, v, grad, lr, beta1, beta2, eps, t):
    """One Adam step (assumed optimiser) in fp64.  Returns new (theta, m, v); inputs are not modified."""
    theta = _f64(theta).copy(); m = _f64(m).copy(); v = _f64(v).copy(); grad = _f64(grad)
    assert theta.shape == m.shape == v.shape == grad.shape and t >= 1
    lib().cngp_oracle_adam_step(ctypes.c_int64(theta.size), ctypes.c_double(lr), ctypes.c_double(beta1),
                                ctypes.c_double(beta2), ctypes.c_double(eps), ctypes.c_int(t),
                                _p(theta), _p(m), _p(v), _p(grad))
    return theta, m, v


def pack_index_bits(D_c, N_p):
    """Exact-width storage of a baked index codebook [L, N_c] (the storage the model sizes of Tables 3 and 4
    imply: log2(N_p) bits per entry): entry r of a level occupies bits [r b, (r + 1) b) of the level's bit
    string, least significant bit first; each level is padded with zero bits to a whole number of 32-bit
    words.  Returns uint8 [L, 4 * ceil(N_c b / 32)]."""
    D_c = np.asarray(D_c, dtype=np.uint8)
    L, N_c = D_c.shape
    b = int(N_p).bit_length() - 1
    nbytes = 4 * ((N_c * b + 31) // 32)
    full = np.zeros((L, nbytes * 8), np.uint8)
    if b:
        full[:, :N_c * b] = ((D_c[..., None] >> np.arange(b, dtype=np.uint8)) & 1).reshape(L, N_c * b)
    return np.packbits(full, axis=1, bitorder="little") if nbytes else np.zeros((L, 0), np.uint8)


def unpack_index_bits(packed, N_c, N_p):
    """Inverse of pack_index_bits."""
    packed = np.asarray(packed, dtype=np.uint8)
    L = packed.shape[0]
    b = int(N_p).bit_length() - 1
    if b == 0:
        return np.zeros((L, N_c), np.uint8)
    bits = np.unpackbits(packed, axis=1, bitorder="little")[:, :N_c * b].reshape(L, N_c, b)
    return (bits.astype(np.uint32) << np.arange(b, dtype=np.uint32)).sum(axis=-1).astype(np.uint8)


def storage_bytes(w, index_bits_exact=True):
    """Bytes of the stored model: F-wide features per entry in the workload's feature type, index codebook
    at log2(N_p) bits per entry (levels padded to 32-bit words) or one byte per entry."""
    fb = 2 if w.feat_dtype == "f16" else 4
    b = int(w.N_p).bit_length() - 1
    level = 4 * ((w.N_c * b + 31) // 32) if index_bits_exact else w.N_c
    return {"D_f": w.L * w.N_f * w.F * fb, "D_c_level": level, "D_c": w.L * level}



def morton_order(x):
    """Order of a batch of points along the Morton (Z-order) curve: not part of the paper's method, an optional
    reordering of the queries.  code(x) interleaves the bits of q_j = min(max(floor(x_j 2^B), 0), 2^B - 1), B = 10 in
    2D, 7 in 3D and 5 in 4D, with bit b of coordinate j at position b d + j; the order is the stable ascending sort of the
    codes.  Returns (perm int32 [N], codes uint32 [N]); a NaN coordinate counts as 0."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    N, d = x.shape
    B = {2: 10, 3: 7, 4: 5}[d]
    v = np.floor(x.astype(np.float64) * float(1 << B))           # the scaling by a power of two is exact in fp32 too
    v = np.where(np.isnan(v), 0.0, v)
    q = np.clip(v, 0, (1 << B) - 1).astype(np.uint32)
    codes = np.zeros(N, dtype=np.uint32)
    for b in range(B):
        for j in range(d):
            codes |= ((q[:, j] >> np.uint32(b)) & np.uint32(1)) << np.uint32(b * d + j)
    return np.argsort(codes, kind="stable").astype(np.int32), codes

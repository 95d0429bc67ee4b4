"""Seeded synthetic inputs for the Compact NGP encoding path.

This module serves both the CPU oracle and the HIP path, and therefore holds
none of the method's arithmetic: no hashing, no level table, no interpolation,
no softmax, no argmax.  It only names the problem sizes (the hyper-parameters
of Table 1 of the paper: d, L, F, N_f, N_c, N_p, N_min, N_max) and draws
points, codebooks and upstream gradients from numpy's PCG64 generator.

The paper fits images (Kodak, an 8000x8000 Pluto image), NeRF scenes and a
texture set; none of these datasets is used here.  The generators below stand
in for them: they reproduce the shapes, sizes and point distributions only.
"""
from dataclasses import dataclass, asdict

import numpy as np

SEED_BASE = 0xC0FFEE
STREAM_X, STREAM_DF, STREAM_LOGITS, STREAM_DY = 0, 1, 2, 3


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: int            # index used for seeding
    d: int
    L: int
    F: int
    N_f: int
    N_c: int
    N_p: int
    N_min: int
    N_max: int
    N: int              # number of points
    feat_dtype: str     # "f32" | "f16"  (storage type of D_f)
    io_dtype: str       # "f32" | "f16"  (type of y and dL/dy)
    points: str         # "uniform" | "nerf_rays" | "sdf_shell"

    def asdict(self):
        return asdict(self)


WORKLOADS = {
    # Tiny 2D case the oracle finishes in milliseconds; everything fp32.
    "tiny2d": Workload("tiny2d", 1, 2, 4, 2, 2**10, 2**8, 4, 16, 256, 4096,
                       "f32", "f32", "uniform"),
    # 2D image-fitting shape (random pixel batch of a Pluto-scale image).
    "image2d": Workload("image2d", 2, 2, 16, 2, 2**16, 2**12, 8, 16, 8192, 2**20,
                        "f16", "f16", "uniform"),
    # 3D NeRF shape: 4096 rays x 64 stratified samples (headline workload).
    "nerf3d": Workload("nerf3d", 3, 3, 16, 2, 2**16, 2**14, 16, 16, 2048, 2**18,
                       "f16", "f16", "nerf_rays"),
    # 3D SDF shape: points concentrated near a sphere surface.
    "sdf3d": Workload("sdf3d", 4, 3, 16, 2, 2**18, 2**16, 8, 16, 4096, 2**20,
                      "f16", "f16", "sdf_shell"),
    # Inference-only 3D: forward with the baked, 4-bit packed index codebook.
    "infer3d": Workload("infer3d", 5, 3, 16, 2, 2**16, 2**14, 16, 16, 2048, 2**24,
                        "f16", "f16", "uniform"),
    # The same inference with plain hashing at the same feature codebook size (N_p = 1: no index codebook): what the
    # learned probes cost at inference time (Sec. 4 compares against this baseline encoding).
    "infer3d_plain": Workload("infer3d_plain", 5, 3, 16, 2, 2**16, 1, 1, 16, 2048, 2**24,
                              "f16", "f16", "uniform"),
    # Inference from the compressed model of the paper's Table 3 row (N_f = 2^8, N_c = 2^16, N_p = 2^3):
    # forward with the index codebook stored at exactly 3 bits per entry.
    "compact3d": Workload("compact3d", 6, 3, 16, 2, 2**8, 2**16, 8, 16, 2048, 2**22,
                          "f16", "f16", "uniform"),
}


def _rng(cfg: int, stream: int) -> np.random.Generator:
    return np.random.default_rng(SEED_BASE + 1000 * cfg + stream)


def _unit_sphere(rng, n):
    u = rng.standard_normal((n, 3))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    return u


def _points_uniform(rng, n, d):
    return rng.random((n, d), dtype=np.float64)


def _points_nerf_rays(rng, n, d):
    """Rays that start on a sphere of radius 1.5 around the unit cube's centre,
    look at the centre with a jitter of up to 0.3 rad, and carry 64 stratified,
    jittered samples each; samples outside the cube are clipped onto its faces."""
    assert d == 3
    spr = 64
    rays = (n + spr - 1) // spr
    c = np.full(3, 0.5)
    o = c + 1.5 * _unit_sphere(rng, rays)
    fwd = c - o
    fwd /= np.linalg.norm(fwd, axis=1, keepdims=True)
    # orthonormal frame around fwd
    helper = np.where(np.abs(fwd[:, :1]) < 0.9, np.array([[1.0, 0, 0]]), np.array([[0, 1.0, 0]]))
    e1 = np.cross(fwd, helper)
    e1 /= np.linalg.norm(e1, axis=1, keepdims=True)
    e2 = np.cross(fwd, e1)
    theta = rng.uniform(0.0, 0.3, rays)[:, None]
    phi = rng.uniform(0.0, 2 * np.pi, rays)[:, None]
    dirs = np.cos(theta) * fwd + np.sin(theta) * (np.cos(phi) * e1 + np.sin(phi) * e2)
    t_near, t_far = 1.5 - np.sqrt(3) / 2, 1.5 + np.sqrt(3) / 2
    strata = (np.arange(spr)[None, :] + rng.random((rays, spr))) / spr
    t = t_near + strata * (t_far - t_near)
    pts = o[:, None, :] + t[:, :, None] * dirs[:, None, :]
    return np.clip(pts.reshape(-1, 3)[:n], 0.0, 1.0)


def _points_sdf_shell(rng, n, d):
    """80 % of the points within +-0.01 of a sphere of radius 0.35 centred in
    the cube, 20 % uniform; one seeded permutation mixes the two groups."""
    assert d == 3
    n_shell = (n * 4) // 5
    r = 0.35 + rng.uniform(-0.01, 0.01, n_shell)[:, None]
    shell = 0.5 + r * _unit_sphere(rng, n_shell)
    uni = rng.random((n - n_shell, 3))
    pts = np.concatenate([shell, uni], axis=0)
    return np.clip(pts[rng.permutation(n)], 0.0, 1.0)


_POINTS = {"uniform": _points_uniform, "nerf_rays": _points_nerf_rays,
           "sdf_shell": _points_sdf_shell}

_NP_DTYPE = {"f32": np.float32, "f16": np.float16}


def make_points(w: Workload, n: int = None) -> np.ndarray:
    """x: float32 [n, d] in [0, 1]^d (the first n points of the workload)."""
    n = w.N if n is None else n
    x = _POINTS[w.points](_rng(w.cfg, STREAM_X), w.N if w.points != "uniform" else n, w.d)
    return np.ascontiguousarray(x[:n], dtype=np.float32)


def make_feature_codebook(w: Workload) -> np.ndarray:
    """D_f: [L, N_f, F], uniform in (-1e-4, 1e-4), rounded to its storage type."""
    v = _rng(w.cfg, STREAM_DF).uniform(-1e-4, 1e-4, (w.L, w.N_f, w.F))
    return np.ascontiguousarray(v, dtype=_NP_DTYPE[w.feat_dtype])


def make_probe_logits(w: Workload) -> np.ndarray:
    """D^_c: float32 [L, N_c, N_p], standard normal confidence values."""
    v = _rng(w.cfg, STREAM_LOGITS).standard_normal((w.L, w.N_c, w.N_p))
    return np.ascontiguousarray(v, dtype=np.float32)


def make_upstream_grad(w: Workload, n: int = None) -> np.ndarray:
    """dL/dy: [n, L*F], standard normal, rounded to the I/O type."""
    n = w.N if n is None else n
    v = _rng(w.cfg, STREAM_DY).standard_normal((n, w.L * w.F), dtype=np.float32)
    return np.ascontiguousarray(v, dtype=_NP_DTYPE[w.io_dtype])


def custom(name="custom", cfg=99, **kw) -> Workload:
    """A workload with explicit sizes, for edge-case tests."""
    base = dict(d=3, L=2, F=2, N_f=64, N_c=32, N_p=4, N_min=4, N_max=8, N=100,
                feat_dtype="f32", io_dtype="f32", points="uniform")
    base.update(kw)
    return Workload(name, cfg, **base)

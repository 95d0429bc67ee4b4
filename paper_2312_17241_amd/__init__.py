"""Python binding of libcngp.so, the Compact NGP encoding library for MI355X.

Argument marshalling only: every function below checks tensor types and shapes, passes
device pointers and torch's current HIP stream to the C ABI declared in include/cngp.h and
returns.  All arithmetic of the method runs in the library's HIP kernels; there is no CPU
or PyTorch fallback, and importing this package fails if the library has not been built
(run `python paper_2312_17241_amd/build.py` or `__graft_entry__.build()`).

Function names mirror the C entry points: level_resolutions, workspace_bytes, encode_fwd,
encode_bwd, bake_probes, debug_indices.
"""
import ctypes
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcngp.so")

F32, F16 = 0, 1
IDX_U8, IDX_PACKED4, IDX_BITS = 0, 1, 2
ZERO_GRADS, BWD_DIRECT, BWD_SLICED, BWD_NO_PREREDUCE, FWD_SIMPLE, BWD_BINNED, FWD_LEVEL, FWD_TILE = 1, 2, 4, 8, 16, 32, 64, 128

OK, ERR_NULL, ERR_INVALID, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4, -5


class CConfig(ctypes.Structure):
    """Mirror of the C struct cngp_config (Table 1 of the paper: same symbols)."""
    _fields_ = [("d", ctypes.c_int32), ("L", ctypes.c_int32), ("F", ctypes.c_int32),
                ("N_f", ctypes.c_uint32), ("N_c", ctypes.c_uint32), ("N_p", ctypes.c_uint32),
                ("N_min", ctypes.c_uint32), ("N_max", ctypes.c_uint32),
                ("feat_dtype", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
                ("index_format", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("bin_bytes_max", ctypes.c_uint64), ("top_k", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class CngpError(RuntimeError):
    def __init__(self, status, detail=""):
        self.status = status
        msg = _lib.cngp_error_string(status).decode()
        super().__init__(f"cngp status {status}: {msg}{(' -- ' + detail) if detail else ''}")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python paper_2312_17241_amd/build.py` "
            "(hipcc, gfx950).  There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    cfgp = ctypes.POINTER(CConfig)
    lib.cngp_version.restype = ctypes.c_int
    lib.cngp_error_string.restype = ctypes.c_char_p
    lib.cngp_error_string.argtypes = [ctypes.c_int]
    lib.cngp_last_hip_error.restype = ctypes.c_char_p
    lib.cngp_level_resolutions.restype = ctypes.c_int
    lib.cngp_level_resolutions.argtypes = [cfgp, vp]
    lib.cngp_workspace_bytes.restype = sz
    lib.cngp_workspace_bytes.argtypes = [cfgp, i64]
    lib.cngp_fwd_workspace_bytes.restype = sz
    lib.cngp_fwd_workspace_bytes.argtypes = [cfgp, i64]
    lib.cngp_encode_fwd.restype = ctypes.c_int
    lib.cngp_encode_fwd.argtypes = [cfgp, vp, i64, vp, vp, vp, vp, sz, vp]
    lib.cngp_encode_bwd.restype = ctypes.c_int
    lib.cngp_encode_fwd_partial.restype = ctypes.c_int
    lib.cngp_encode_fwd_partial.argtypes = [cfgp, ctypes.c_int32, vp, i64, vp, vp, vp, vp, sz, vp]
    lib.cngp_encode_bwd.argtypes = [cfgp, vp, i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cngp_encode_bwd_static.restype = ctypes.c_int
    lib.cngp_encode_bwd_static.argtypes = [cfgp, vp, i64, vp, vp, vp, vp, vp, vp]
    lib.cngp_static_scratch_bytes.restype = sz
    lib.cngp_static_scratch_bytes.argtypes = []
    lib.cngp_morton_sort_workspace_bytes.restype = sz
    lib.cngp_morton_sort_workspace_bytes.argtypes = [ctypes.c_int32, i64]
    lib.cngp_morton_sort.restype = ctypes.c_int
    lib.cngp_morton_sort.argtypes = [ctypes.c_int32, vp, i64, vp, vp, vp, sz, vp]
    lib.cngp_encode_fwd_permuted.restype = ctypes.c_int
    lib.cngp_encode_fwd_permuted.argtypes = [cfgp, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    lib.cngp_bake_probes.restype = ctypes.c_int
    lib.cngp_bake_probes.argtypes = [cfgp, vp, vp, vp]
    lib.cngp_encode_bwd_input.restype = ctypes.c_int
    lib.cngp_encode_bwd_input.argtypes = [cfgp, vp, i64, vp, vp, vp, vp, vp]
    lib.cngp_mlp_weight_count.restype = ctypes.c_size_t
    lib.cngp_mlp_weight_count.argtypes = [vp]
    lib.cngp_mlp_fwd.restype = ctypes.c_int
    lib.cngp_mlp_fwd.argtypes = [vp, vp, i64, vp, vp, vp]
    lib.cngp_encode_mlp_fwd.restype = ctypes.c_int
    lib.cngp_encode_mlp_fwd.argtypes = [cfgp, vp, vp, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.cngp_mlp_bwd.restype = ctypes.c_int
    lib.cngp_mlp_bwd.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp]
    lib.cngp_adam_step.restype = ctypes.c_int
    lib.cngp_adam_step.argtypes = [vp, i64, vp, vp, vp, vp, vp, ctypes.c_int, vp]
    lib.cngp_storage_bytes.restype = ctypes.c_int
    lib.cngp_storage_bytes.argtypes = [cfgp, vp, vp, vp]
    lib.cngp_adam_step_bake.restype = ctypes.c_int
    lib.cngp_adam_step_bake.argtypes = [cfgp, vp, vp] + [vp] * 10 + [vp]
    lib.cngp_debug_indices.restype = ctypes.c_int
    lib.cngp_debug_indices.argtypes = [cfgp, vp, i64, vp, vp, vp, vp, vp, vp]
    lib.cngp_bwd_plan_info.restype = ctypes.c_int
    lib.cngp_bwd_plan_info.argtypes = [cfgp, i64, vp]
    lib.cngp_fwd_plan_info.restype = ctypes.c_int
    lib.cngp_fwd_plan_info.argtypes = [cfgp, i64, vp]
    lib.cngp_bwd_plan_layout.restype = ctypes.c_int
    lib.cngp_bwd_plan_layout.argtypes = [cfgp, i64, vp]
    lib.cngp_measure_rates.restype = ctypes.c_int
    lib.cngp_measure_rates.argtypes = [vp, vp, sz, vp]
    lib.cngp_profile_enable.restype = ctypes.c_int
    lib.cngp_profile_enable.argtypes = [ctypes.c_int]
    lib.cngp_profile_read.restype = ctypes.c_int
    lib.cngp_profile_read.argtypes = [vp, vp, ctypes.c_int]
    lib.cngp_profile_kernel_name.restype = ctypes.c_char_p
    lib.cngp_profile_kernel_name.argtypes = [ctypes.c_int]
    return lib


_lib = _load()

_DT = {"f32": F32, "f16": F16, F32: F32, F16: F16}
_TORCH_DT = {F32: torch.float32, F16: torch.float16}


@dataclass(frozen=True)
class Config:
    """Hyper-parameters of the encoding; field names follow Table 1 of the paper."""
    d: int
    L: int
    F: int
    N_f: int
    N_c: int
    N_p: int
    N_min: int
    N_max: int
    feat_dtype: int = F32
    io_dtype: int = F32
    index_format: int = IDX_U8
    flags: int = 0
    bin_bytes_max: int = 0      # 0 = the library's 8 GiB
    top_k: int = 0              # backward: 0 = softmax over all N_p candidates; else over the top_k largest only

    @staticmethod
    def from_workload(w, index_format=IDX_U8, flags=0, **over):
        kw = dict(d=w.d, L=w.L, F=w.F, N_f=w.N_f, N_c=w.N_c, N_p=w.N_p, N_min=w.N_min, N_max=w.N_max,
                  feat_dtype=_DT[w.feat_dtype], io_dtype=_DT[w.io_dtype],
                  index_format=index_format, flags=flags)
        kw.update(over)
        return Config(**kw)

    def c(self) -> CConfig:
        return CConfig(self.d, self.L, self.F, self.N_f, self.N_c, self.N_p, self.N_min, self.N_max,
                       self.feat_dtype, self.io_dtype, self.index_format, self.flags, self.bin_bytes_max, self.top_k, 0)

    @property
    def index_cols(self) -> int:
        """Bytes per level of the index codebook in this configuration's format."""
        if self.index_format == IDX_BITS:
            return 4 * ((self.N_c * (self.N_p.bit_length() - 1) + 31) // 32)
        return self.N_c // 2 if self.index_format == IDX_PACKED4 else self.N_c


def _check(status):
    if status != OK:
        detail = _lib.cngp_last_hip_error().decode() if status == ERR_HIP else ""
        raise CngpError(status, detail)


def _dev(t, dtype, shape, name):
    if t is None:
        raise CngpError(ERR_NULL, f"{name} is None")
    if not (isinstance(t, torch.Tensor) and t.is_cuda):
        raise TypeError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(ws):
    if ws is None:
        return ctypes.c_void_p(0), 0
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def version() -> int:
    return _lib.cngp_version()


def error_string(status: int) -> str:
    return _lib.cngp_error_string(status).decode()


def level_resolutions(cfg: Config) -> np.ndarray:
    out = np.zeros(max(cfg.L, 1), dtype=np.uint32)
    c = cfg.c()
    _check(_lib.cngp_level_resolutions(ctypes.byref(c), out.ctypes.data_as(ctypes.c_void_p)))
    return out[:cfg.L]


def storage_bytes(cfg: Config) -> dict:
    """Bytes of the stored model: D_f in feat_dtype, D_c per level and in total in index_format."""
    a, b, t = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    c = cfg.c()
    _check(_lib.cngp_storage_bytes(ctypes.byref(c), ctypes.byref(a), ctypes.byref(b), ctypes.byref(t)))
    return {"D_f": a.value, "D_c_level": b.value, "D_c": t.value}


def workspace_bytes(cfg: Config, N: int) -> int:
    c = cfg.c()
    return int(_lib.cngp_workspace_bytes(ctypes.byref(c), N))


def fwd_workspace_bytes(cfg: Config, N: int) -> int:
    """Bytes the forward calls use of a workspace (0: none; with less they run the tile variant, same result)."""
    c = cfg.c()
    return int(_lib.cngp_fwd_workspace_bytes(ctypes.byref(c), N))


def fwd_plan_info(cfg: Config, N: int) -> dict:
    """How encode_fwd would run for (cfg, N) when it is given its workspace (see cngp_fwd_plan_info)."""
    info = (ctypes.c_int32 * 4)()
    c = cfg.c()
    _check(_lib.cngp_fwd_plan_info(ctypes.byref(c), N, info))
    return dict(zip(("level_resident", "resident_entries", "parts", "lds_bytes"), list(info)))


def bwd_plan_info(cfg: Config, N: int) -> dict:
    """How encode_bwd would run for (cfg, N): variant, pre-reduced levels, slices and chunk counts."""
    info = (ctypes.c_int32 * 15)()
    c = cfg.c()
    _check(_lib.cngp_bwd_plan_info(ctypes.byref(c), N, info))
    names = ("sliced", "dense_levels", "slices_f", "slices_c", "chunks_feat_pts", "chunks_logit_pts",
             "chunks_feat_vtx", "chunks_logit_vtx", "chunks_grid", "grid_slices",
             "binned", "drain_wgs_feat", "drain_wgs_logit", "bin_chunks", "passes")
    return dict(zip(names, list(info)))


def bwd_plan_layout(cfg: Config, N: int):
    """[(offset, bytes)] of the workspace regions encode_bwd would use (see cngp_bwd_plan_layout)."""
    reg = (ctypes.c_uint64 * 24)()
    c = cfg.c()
    k = _lib.cngp_bwd_plan_layout(ctypes.byref(c), N, reg)
    if k < 0:
        _check(k)
    return [(int(reg[2 * i]), int(reg[2 * i + 1])) for i in range(k)]


def alloc_workspace(cfg: Config, N: int, device="cuda"):
    """A device buffer large enough for encode_fwd / encode_bwd on N points (None if none is needed)."""
    nbytes = workspace_bytes(cfg, N)
    if nbytes == 0:
        return None
    return torch.empty((nbytes + 255) // 256 * 256, dtype=torch.uint8, device=device)


def encode_fwd(cfg: Config, x, D_f, D_c, y=None, workspace=None):
    N = x.shape[0]
    if y is None:
        y = torch.empty((N, cfg.L * cfg.F), dtype=_TORCH_DT[cfg.io_dtype], device=x.device)
    c = cfg.c()
    wp, wb = _ws(workspace)
    _check(_lib.cngp_encode_fwd(
        ctypes.byref(c), _dev(x, torch.float32, (N, cfg.d), "x"), N,
        _dev(D_f, _TORCH_DT[cfg.feat_dtype], (cfg.L, cfg.N_f, cfg.F), "D_f"),
        _dc(cfg, D_c),
        _dev(y, _TORCH_DT[cfg.io_dtype], (N, cfg.L * cfg.F), "y"), wp, wb, _stream()))
    return y


def morton_sort(x, workspace=None):
    """cngp_morton_sort: (perm, x_sorted) with x_sorted[i] = x[perm[i]] in Morton order (stable); perm is int32."""
    N, d = x.shape
    perm = torch.empty((N,), dtype=torch.int32, device=x.device)
    x_sorted = torch.empty_like(x)
    if N == 0:
        return perm, x_sorted
    need = int(_lib.cngp_morton_sort_workspace_bytes(d, N))
    if need == 0:
        raise CngpError(ERR_INVALID, "morton_sort: d must be 2, 3 or 4 and N below 2^31")
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    wp, wb = _ws(workspace)
    _check(_lib.cngp_morton_sort(d, _dev(x, torch.float32, (N, d), "x"), N, _dev(perm, torch.int32, (N,), "perm"),
                                 _dev(x_sorted, torch.float32, (N, d), "x_sorted"), wp, wb, _stream()))
    return perm, x_sorted


def encode_fwd_permuted(cfg: Config, x_sorted, perm, D_f, D_c, y=None, workspace=None):
    """cngp_encode_fwd_permuted: row perm[i] of y = encoding of x_sorted[i] (y in the order of the original points)."""
    N = x_sorted.shape[0]
    if y is None:
        y = torch.empty((N, cfg.L * cfg.F), dtype=_TORCH_DT[cfg.io_dtype], device=x_sorted.device)
    c = cfg.c()
    _check(_lib.cngp_encode_fwd_permuted(
        ctypes.byref(c), _dev(x_sorted, torch.float32, (N, cfg.d), "x_sorted"), _dev(perm, torch.int32, (N,), "perm"), N,
        _dev(D_f, _TORCH_DT[cfg.feat_dtype], (cfg.L, cfg.N_f, cfg.F), "D_f"), _dc(cfg, D_c),
        _dev(y, _TORCH_DT[cfg.io_dtype], (N, cfg.L * cfg.F), "y"), *_ws(workspace), _stream()))
    return y


def encode_fwd_partial(cfg: Config, levels_loaded, x, D_f, D_c, y=None, workspace=None):
    """cngp_encode_fwd_partial: only the first `levels_loaded` levels are read, the others encode to zero."""
    N = x.shape[0]
    if y is None:
        y = torch.empty((N, cfg.L * cfg.F), dtype=_TORCH_DT[cfg.io_dtype], device=x.device)
    c = cfg.c()
    _check(_lib.cngp_encode_fwd_partial(
        ctypes.byref(c), int(levels_loaded), _dev(x, torch.float32, (N, cfg.d), "x"), N,
        _dev(D_f, _TORCH_DT[cfg.feat_dtype], (cfg.L, cfg.N_f, cfg.F), "D_f"), _dc(cfg, D_c),
        _dev(y, _TORCH_DT[cfg.io_dtype], (N, cfg.L * cfg.F), "y"), *_ws(workspace), _stream()))
    return y


def encode_bwd(cfg: Config, x, D_f, Dhat_c, dy, grad_D_f=None, grad_Dhat_c=None, workspace=None):
    N = x.shape[0]
    if grad_D_f is None:
        grad_D_f = torch.zeros((cfg.L, cfg.N_f, cfg.F), dtype=torch.float32, device=x.device)
    if grad_Dhat_c is None:
        grad_Dhat_c = torch.zeros((cfg.L, cfg.N_c, cfg.N_p), dtype=torch.float32, device=x.device)
    c = cfg.c()
    wp, wb = _ws(workspace)
    _check(_lib.cngp_encode_bwd(
        ctypes.byref(c), _dev(x, torch.float32, (N, cfg.d), "x"), N,
        _dev(D_f, _TORCH_DT[cfg.feat_dtype], (cfg.L, cfg.N_f, cfg.F), "D_f"),
        _dev(Dhat_c, torch.float32, (cfg.L, cfg.N_c, cfg.N_p), "Dhat_c"),
        _dev(dy, _TORCH_DT[cfg.io_dtype], (N, cfg.L * cfg.F), "dy"),
        _dev(grad_D_f, torch.float32, (cfg.L, cfg.N_f, cfg.F), "grad_D_f"),
        _dev(grad_Dhat_c, torch.float32, (cfg.L, cfg.N_c, cfg.N_p), "grad_Dhat_c"), wp, wb, _stream()))
    return grad_D_f, grad_Dhat_c


def static_scratch_bytes() -> int:
    return int(_lib.cngp_static_scratch_bytes())


def encode_bwd_static(cfg: Config, x, D_f, Dhat_c, dy, grad_D_f, grad_Dhat_c):
    """cngp_encode_bwd_static: the backward pass out of the library's static scratch array.  Allocates nothing,
    here or in the library: both gradient tensors are the caller's."""
    N = x.shape[0]
    c = cfg.c()
    _check(_lib.cngp_encode_bwd_static(
        ctypes.byref(c), _dev(x, torch.float32, (N, cfg.d), "x"), N,
        _dev(D_f, _TORCH_DT[cfg.feat_dtype], (cfg.L, cfg.N_f, cfg.F), "D_f"),
        _dev(Dhat_c, torch.float32, (cfg.L, cfg.N_c, cfg.N_p), "Dhat_c"),
        _dev(dy, _TORCH_DT[cfg.io_dtype], (N, cfg.L * cfg.F), "dy"),
        _dev(grad_D_f, torch.float32, (cfg.L, cfg.N_f, cfg.F), "grad_D_f"),
        _dev(grad_Dhat_c, torch.float32, (cfg.L, cfg.N_c, cfg.N_p), "grad_Dhat_c"), _stream()))
    return grad_D_f, grad_Dhat_c


def encode_bwd_input(cfg: Config, x, D_f, D_c, dy, grad_x=None):
    """dL/dx of the forward pass: float32 [N, d]."""
    N = x.shape[0]
    if grad_x is None:
        grad_x = torch.empty((N, cfg.d), dtype=torch.float32, device=x.device)
    c = cfg.c()
    _check(_lib.cngp_encode_bwd_input(
        ctypes.byref(c), _dev(x, torch.float32, (N, cfg.d), "x"), N,
        _dev(D_f, _TORCH_DT[cfg.feat_dtype], (cfg.L, cfg.N_f, cfg.F), "D_f"), _dc(cfg, D_c),
        _dev(dy, _TORCH_DT[cfg.io_dtype], (N, cfg.L * cfg.F), "dy"),
        _dev(grad_x, torch.float32, (N, cfg.d), "grad_x"), _stream()))
    return grad_x


def bake_probes(cfg: Config, Dhat_c, D_c=None):
    if D_c is None:
        D_c = torch.empty((cfg.L, cfg.index_cols), dtype=torch.uint8, device=Dhat_c.device)
    c = cfg.c()
    _check(_lib.cngp_bake_probes(
        ctypes.byref(c), _dev(Dhat_c, torch.float32, (cfg.L, cfg.N_c, cfg.N_p), "Dhat_c"),
        _dc(cfg, D_c), _stream()))
    return D_c


class CAdam(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("grad_scale", ctypes.c_float), ("step", ctypes.c_int32)]


@dataclass
class Adam:
    """Hyper-parameters of one table's optimiser step (cngp_adam)."""
    lr: float = 1e-2
    beta1: float = 0.9
    beta2: float = 0.99
    eps: float = 1e-15
    grad_scale: float = 1.0
    step: int = 1

    def c(self):
        return CAdam(self.lr, self.beta1, self.beta2, self.eps, self.grad_scale, self.step)


def adam_step_bake(cfg: Config, opt_f, opt_c, features=None, logits=None):
    """cngp_adam_step_bake.  `features` = (D_f_master, D_f, m_f, v_f, grad_D_f) with D_f None when the
    codebook is stored as float32; `logits` = (Dhat_c, m_c, v_c, grad_Dhat_c, D_c).  Updates in place."""
    c = cfg.c()
    null = ctypes.c_void_p(0)
    fa = [null] * 5
    ca = [null] * 5
    of = oc = None
    if opt_f is not None:
        master, D_f, m_f, v_f, g_f = features
        shp = (cfg.L, cfg.N_f, cfg.F)
        fa = [_dev(master, torch.float32, shp, "D_f_master"),
              null if D_f is None else _dev(D_f, _TORCH_DT[cfg.feat_dtype], shp, "D_f"),
              _dev(m_f, torch.float32, shp, "m_f"), _dev(v_f, torch.float32, shp, "v_f"),
              _dev(g_f, torch.float32, shp, "grad_D_f")]
        of = opt_f.c()
    if opt_c is not None:
        Dhat_c, m_c, v_c, g_c, D_c = logits
        shp = (cfg.L, cfg.N_c, cfg.N_p)
        ca = [_dev(Dhat_c, torch.float32, shp, "Dhat_c"), _dev(m_c, torch.float32, shp, "m_c"),
              _dev(v_c, torch.float32, shp, "v_c"), _dev(g_c, torch.float32, shp, "grad_Dhat_c"),
              _dev(D_c, torch.uint8, (cfg.L, cfg.index_cols), "D_c")]
        oc = opt_c.c()
    _check(_lib.cngp_adam_step_bake(
        ctypes.byref(c), None if of is None else ctypes.cast(ctypes.byref(of), ctypes.c_void_p),
        None if oc is None else ctypes.cast(ctypes.byref(oc), ctypes.c_void_p), *fa, *ca, _stream()))


def adam_step(opt: Adam, master, half_copy, m, v, grad, clear_grad=False):
    """cngp_adam_step on one flat float32 parameter array; half_copy (float16, same size) may be None."""
    n = master.numel()
    o = opt.c()
    hc = ctypes.c_void_p(0) if half_copy is None else _dev(half_copy, torch.float16, tuple(master.shape), "half_copy")
    _check(_lib.cngp_adam_step(ctypes.byref(o), n, _dev(master, torch.float32, tuple(master.shape), "master"), hc,
                               _dev(m, torch.float32, tuple(master.shape), "m"),
                               _dev(v, torch.float32, tuple(master.shape), "v"),
                               _dev(grad, torch.float32, tuple(master.shape), "grad"), int(bool(clear_grad)), _stream()))


class CMlpConfig(ctypes.Structure):
    _fields_ = [("n_in", ctypes.c_int32), ("n_out", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]


@dataclass(frozen=True)
class MlpConfig:
    """Decoder after the encoding (cngp_mlp_config): n_in -> 64 -> 64 -> n_out, ReLU, no biases."""
    n_in: int
    n_out: int
    io_dtype: int = F32
    flags: int = 0

    def c(self):
        return CMlpConfig(self.n_in, self.n_out, self.io_dtype, self.flags)

    @property
    def weight_count(self) -> int:
        c = self.c()
        return int(_lib.cngp_mlp_weight_count(ctypes.byref(c)))

    def split(self, W):
        """Views of a flat weight (or gradient) array as W1 [64, n_in], W2 [64, 64], W3 [n_out, 64]."""
        a, b = 64 * self.n_in, 64 * self.n_in + 64 * 64
        return W[:a].view(64, self.n_in), W[a:b].view(64, 64), W[b:].view(self.n_out, 64)


def mlp_fwd(cfg: MlpConfig, y, W, out=None):
    N = y.shape[0]
    if out is None:
        out = torch.empty((N, cfg.n_out), dtype=torch.float32, device=y.device)
    c = cfg.c()
    _check(_lib.cngp_mlp_fwd(ctypes.byref(c), _dev(y, _TORCH_DT[cfg.io_dtype], (N, cfg.n_in), "y"), N,
                             _dev(W, torch.float16, (cfg.weight_count,), "W"),
                             _dev(out, torch.float32, (N, cfg.n_out), "out"), _stream()))
    return out


def encode_mlp_fwd(cfg: Config, mcfg: MlpConfig, x, D_f, D_c, W, out=None, workspace=None):
    """cngp_encode_mlp_fwd: decoder(encode(x)) in one call; float32 [N, n_out].  workspace: N * L * F * 2 bytes (or a
    workspace of alloc_workspace for an fp16-output configuration) lets the level-resident forward feed the decoder."""
    N = x.shape[0]
    if out is None:
        out = torch.empty((N, mcfg.n_out), dtype=torch.float32, device=x.device)
    c, m = cfg.c(), mcfg.c()
    wp, wb = _ws(workspace)
    _check(_lib.cngp_encode_mlp_fwd(
        ctypes.byref(c), ctypes.cast(ctypes.byref(m), ctypes.c_void_p), _dev(x, torch.float32, (N, cfg.d), "x"), N,
        _dev(D_f, _TORCH_DT[cfg.feat_dtype], (cfg.L, cfg.N_f, cfg.F), "D_f"), _dc(cfg, D_c),
        _dev(W, torch.float16, (mcfg.weight_count,), "W"), _dev(out, torch.float32, (N, mcfg.n_out), "out"), wp, wb, _stream()))
    return out


def mlp_bwd(cfg: MlpConfig, y, W, dout, dy=None, grad_W=None):
    N = y.shape[0]
    if dy is None:
        dy = torch.empty((N, cfg.n_in), dtype=_TORCH_DT[cfg.io_dtype], device=y.device)
    if grad_W is None:
        grad_W = torch.zeros((cfg.weight_count,), dtype=torch.float32, device=y.device)
    c = cfg.c()
    _check(_lib.cngp_mlp_bwd(ctypes.byref(c), _dev(y, _TORCH_DT[cfg.io_dtype], (N, cfg.n_in), "y"), N,
                             _dev(W, torch.float16, (cfg.weight_count,), "W"),
                             _dev(dout, torch.float32, (N, cfg.n_out), "dout"),
                             _dev(dy, _TORCH_DT[cfg.io_dtype], (N, cfg.n_in), "dy"),
                             _dev(grad_W, torch.float32, (cfg.weight_count,), "grad_W"), _stream()))
    return dy, grad_W


def debug_indices(cfg: Config, x, D_c):
    """base, h2, probe, feat_idx of every (point, level, corner): tensors of shape [N, L, 2^d]."""
    N = x.shape[0]
    shp = (N, cfg.L, 1 << cfg.d)
    base = torch.empty(shp, dtype=torch.int32, device=x.device)
    h2 = torch.empty(shp, dtype=torch.int32, device=x.device)
    probe = torch.empty(shp, dtype=torch.uint8, device=x.device)
    fidx = torch.empty(shp, dtype=torch.int32, device=x.device)
    c = cfg.c()
    _check(_lib.cngp_debug_indices(
        ctypes.byref(c), _dev(x, torch.float32, (N, cfg.d), "x"), N,
        _dc(cfg, D_c),
        ctypes.c_void_p(base.data_ptr()), ctypes.c_void_p(h2.data_ptr()),
        ctypes.c_void_p(probe.data_ptr()), ctypes.c_void_p(fidx.data_ptr()), _stream()))
    return base, h2, probe, fidx


class CRates(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("copy_GBps", "gather4_Gps", "row_gather_Gps",
                                               "global_atomic_Gseg", "lds_atomic_f64_Gps",
                                               "lds_atomic_f32_Gps", "lds_atomic_u32_Gps", "row_gather_far_Gps", "gather4_far_Gps",
                                               "lds_gather4_Gps")]


def measure_rates(device="cuda") -> dict:
    """Streaming, gather and atomic rates of the device (see cngp_measure_rates); synchronises."""
    scratch = torch.zeros(64 << 20, dtype=torch.uint8, device=device)
    r = CRates()
    _check(_lib.cngp_measure_rates(ctypes.byref(r), ctypes.c_void_p(scratch.data_ptr()), scratch.numel(), _stream()))
    torch.cuda.synchronize()
    return {n: getattr(r, n) for n, _ in CRates._fields_}


def profile_enable(on: bool) -> bool:
    return bool(_lib.cngp_profile_enable(1 if on else 0))


def profile_read() -> dict:
    """{kernel name: (total ms, launches)} since the last read; waits for the recorded events."""
    n = 64                                   # more than the library has kernel kinds
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    k = _lib.cngp_profile_read(ms, cnt, n)
    return {_lib.cngp_profile_kernel_name(i).decode(): (ms[i], cnt[i]) for i in range(min(k, n)) if cnt[i]}


def _dc(cfg, D_c):
    """Device pointer of an index codebook; the exact-width format of N_p = 1 has no bytes (NULL)."""
    if cfg.index_format == IDX_BITS and cfg.N_p == 1:
        return ctypes.c_void_p(0)
    return _dev(D_c, torch.uint8, (cfg.L, cfg.index_cols), "D_c")


def pack_bits(D_c_u8, N_p):
    """Repack a [L, N_c] uint8 index codebook into the exact-width layout (log2(N_p) bits per entry, least
    significant bit first, each level padded to whole 32-bit words).  Pure data movement with torch ops."""
    b = int(N_p).bit_length() - 1
    L, N_c = D_c_u8.shape
    nbytes = 4 * ((N_c * b + 31) // 32)
    if b == 0:
        return torch.empty((L, 0), dtype=torch.uint8, device=D_c_u8.device)
    bits = ((D_c_u8.to(torch.int32).unsqueeze(-1) >> torch.arange(b, device=D_c_u8.device)) & 1).reshape(L, N_c * b)
    pad = torch.zeros((L, nbytes * 8 - N_c * b), dtype=torch.int32, device=D_c_u8.device)
    bits = torch.cat([bits, pad], dim=1).reshape(L, nbytes, 8)
    return (bits << torch.arange(8, device=D_c_u8.device)).sum(dim=-1).to(torch.uint8).contiguous()


def pack4(D_c_u8):
    """Repack a [L, N_c] uint8 index codebook into the two-entries-per-byte layout (entry 2i in
    the low nibble of byte i).  Pure data movement on whatever device the tensor lives on."""
    return (D_c_u8[..., 0::2] | (D_c_u8[..., 1::2] << 4)).contiguous()

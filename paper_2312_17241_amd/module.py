"""torch.nn.Module around the library's entry points, for training loops.

Holds the codebooks of the encoding (Sec. 3: feature codebook D_f, confidence values D^_c, baked index
codebook D_c), their gradient arrays and optimiser moments as device tensors, and wires encode_fwd /
encode_bwd into autograd so that a decoder written in PyTorch can be trained on top of it.  Marshalling
only: every operation on the codebooks runs in the library's kernels (forward, backward, optimiser step
fused with the bake); nothing here computes on them with PyTorch.

Choices the paper leaves open (stated, not claimed): D_f starts uniform in +-1e-4 as in the hash-grid
encoding the method extends; D^_c starts uniform in +-1e-4 (every candidate nearly equally likely, the
first bake picks an arbitrary one); the optimiser is Adam.
"""
import torch

from . import (Adam, Config, ZERO_GRADS, _TORCH_DT, F16, adam_step_bake, alloc_workspace, bake_probes,
               encode_bwd, encode_bwd_input, encode_fwd, workspace_bytes)


class _Encode(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, hook, enc):
        ctx.enc = enc
        ctx.save_for_backward(x)
        return encode_fwd(enc.cfg, x, enc.D_f, enc.D_c, workspace=enc._workspace(x.shape[0]))

    @staticmethod
    def backward(ctx, dy):
        enc = ctx.enc
        (x,) = ctx.saved_tensors
        dy = dy.contiguous().to(_TORCH_DT[enc.cfg.io_dtype])
        encode_bwd(enc.cfg, x, enc.D_f, enc.Dhat_c, dy, enc.grad_D_f, enc.grad_Dhat_c,
                   workspace=enc._workspace(x.shape[0]))          # accumulates (+=)
        grad_x = encode_bwd_input(enc.cfg, x, enc.D_f, enc.D_c, dy) if ctx.needs_input_grad[0] else None
        return grad_x, torch.zeros((), dtype=torch.float32, device=dy.device), None


class Encoding(torch.nn.Module):
    """y = enc(x): x float32 [N, d] in [0,1]^d -> [N, L*F].  Call enc.step(opt_f, opt_c) after backward()."""

    def __init__(self, cfg: Config, device="cuda", seed=0):
        super().__init__()
        if cfg.flags & ZERO_GRADS:
            raise ValueError("the module accumulates gradients across backward calls: pass a Config without ZERO_GRADS")
        self.cfg = cfg
        g = torch.Generator(device="cpu").manual_seed(seed)
        fs, cs = (cfg.L, cfg.N_f, cfg.F), (cfg.L, cfg.N_c, cfg.N_p)
        uni = lambda shape: ((torch.rand(shape, generator=g) * 2 - 1) * 1e-4).to(device)
        self.D_f_master = uni(fs)
        self.D_f = self.D_f_master.half() if cfg.feat_dtype == F16 else self.D_f_master
        self.Dhat_c = uni(cs)
        self.D_c = bake_probes(cfg, self.Dhat_c)
        zeros = lambda shape: torch.zeros(shape, dtype=torch.float32, device=device)
        self.grad_D_f, self.m_f, self.v_f = zeros(fs), zeros(fs), zeros(fs)
        self.grad_Dhat_c, self.m_c, self.v_c = zeros(cs), zeros(cs), zeros(cs)
        self._hook = torch.nn.Parameter(torch.zeros((), device=device))   # lets autograd reach backward()
        self._ws = None
        self._ws_n = -1
        self.steps = 0

    def _workspace(self, n):
        if n != self._ws_n:
            need = workspace_bytes(self.cfg, n)
            if self._ws is None or self._ws.numel() < need:
                self._ws = alloc_workspace(self.cfg, n, self.D_f.device)
            self._ws_n = n
        return self._ws

    def forward(self, x):
        return _Encode.apply(x, self._hook, self)

    def step(self, opt_f: Adam, opt_c: Adam):
        """Optimiser step on both codebooks fused with the bake; clears the gradient arrays."""
        self.steps += 1
        of = Adam(opt_f.lr, opt_f.beta1, opt_f.beta2, opt_f.eps, opt_f.grad_scale, self.steps)
        oc = Adam(opt_c.lr, opt_c.beta1, opt_c.beta2, opt_c.eps, opt_c.grad_scale, self.steps)
        cfg = Config(**{**self.cfg.__dict__, "flags": self.cfg.flags | ZERO_GRADS})
        half = self.D_f if self.cfg.feat_dtype == F16 else None
        adam_step_bake(cfg, of, oc, (self.D_f_master, half, self.m_f, self.v_f, self.grad_D_f),
                       (self.Dhat_c, self.m_c, self.v_c, self.grad_Dhat_c, self.D_c))

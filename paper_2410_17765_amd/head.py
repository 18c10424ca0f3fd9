"""Convenience holders of device buffers for the C-ABI calls.

Only memory management lives here (torch tensors on ``cuda:0`` for inputs,
outputs, ctx and workspace); every computation is a call through ``binding``.

Every method launches on torch's current stream and allocates its buffers there, so the
caching allocator's stream-ordered reuse of a released workspace is safe; to run on a side
stream, call the methods under ``with torch.cuda.stream(side):``.  (The C ABI itself takes
any stream; a caller that passes one to ``binding`` directly owns the lifetime of the buffers.)
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding, synth


def to_device(x: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """Upload a float32 array whose values are exact in `dtype` ("fp32" or "bf16").

    For bf16 the upper 16 bits of each float32 are the bfloat16 pattern; they are copied out in
    bounded chunks (values that are not bf16-exact are rounded to nearest-even first)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype != "bf16":
        return torch.from_numpy(x).to(device)
    flat = x.reshape(-1)
    out = torch.empty(flat.shape[0], dtype=torch.int16, device=device)
    chunk = 1 << 24
    for lo in range(0, flat.shape[0], chunk):
        part = flat[lo:lo + chunk]
        halves = part.view(np.uint16).reshape(-1, 2)        # little-endian: [:, 1] is the upper half
        if halves[:, 0].any():
            bits = synth.bf16_bits(part)
        else:
            bits = np.ascontiguousarray(halves[:, 1])
        out[lo:lo + part.shape[0]] = torch.from_numpy(bits.view(np.int16)).to(device)
    return out.view(torch.bfloat16).reshape(x.shape)


def _scratch(nbytes: int, device) -> torch.Tensor:
    # torch's caching allocator hands out 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class CpHead:
    """Weights of one head on the device plus the scratch the calls need."""

    def __init__(self, W: np.ndarray, U: np.ndarray, G: np.ndarray, dtype: str = "bf16", flags: int = 0,
                 device="cuda:0"):
        self.device = torch.device(device)
        self.dtype = dtype
        self.flags = flags
        self.n, self.r, self.d, _ = W.shape
        self.V = U.shape[0]
        self.W = to_device(W, dtype, self.device)
        self.U = to_device(U, dtype, self.device)
        self.G = to_device(G, dtype, self.device)
        self._ctx: Optional[torch.Tensor] = None
        self._desc = None

    def desc(self, T: int) -> binding.Desc:
        return binding.make_desc(T, self.d, self.V, self.n, self.r,
                                 binding.BF16 if self.dtype == "bf16" else binding.FP32, self.flags)

    # ------------------------------------------------------------------ loss
    def loss_fwd(self, H: torch.Tensor, X: torch.Tensor) -> torch.Tensor:
        """H[T,d] (storage dtype), X[T,n] int32 on the device -> loss[T] fp32 (device).  Keeps ctx for loss_bwd."""
        T = H.shape[0]
        ds = self.desc(T)
        self._ctx = _scratch(binding.cp_head_ctx_bytes(ds), self.device)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_LOSS_FWD), self.device)
        loss = torch.empty(T, dtype=torch.float32, device=self.device)
        binding.cp_head_loss_fwd(ds, H, self.W, self.U, self.G, X, loss, self._ctx, ws)
        self._desc = ds
        return loss

    def loss_bwd(self, H: torch.Tensor, X: torch.Tensor, dloss: Optional[torch.Tensor] = None, scale: float = 1.0,
                 want_dU: bool = True) -> Dict[str, torch.Tensor]:
        assert self._ctx is not None, "call loss_fwd first"
        T = H.shape[0]
        ds = self.desc(T)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_LOSS_BWD), self.device)
        f32 = dict(dtype=torch.float32, device=self.device)
        out = {
            "dH": torch.empty((T, self.d), **f32),
            "dW": torch.empty((self.n, self.r, self.d, self.d), **f32),
            "dU": torch.empty((self.V, self.d), **f32) if want_dU else None,
            "dG": torch.empty((self.r, self.d), **f32),
        }
        binding.cp_head_loss_bwd(ds, H, self.W, self.U, self.G, X, dloss, scale, self._ctx,
                                 out["dH"], out["dW"], out["dU"], out["dG"], ws)
        return {k: v for k, v in out.items() if v is not None}

    def loss_fwd_bwd(self, H: torch.Tensor, X: torch.Tensor, dloss: Optional[torch.Tensor] = None, scale: float = 1.0,
                     want_dU: bool = True):
        """Loss and gradients in one call (the upstream gradient is an input): (loss[T], {dH, dW, dU, dG})."""
        T = H.shape[0]
        ds = self.desc(T)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_LOSS_FWD_BWD), self.device)
        f32 = dict(dtype=torch.float32, device=self.device)
        loss = torch.empty(T, **f32)
        out = {
            "dH": torch.empty((T, self.d), **f32),
            "dW": torch.empty((self.n, self.r, self.d, self.d), **f32),
            "dU": torch.empty((self.V, self.d), **f32) if want_dU else None,
            "dG": torch.empty((self.r, self.d), **f32),
        }
        binding.cp_head_loss_fwd_bwd(ds, H, self.W, self.U, self.G, X, dloss, scale, loss,
                                     out["dH"], out["dW"], out["dU"], out["dG"], ws)
        return loss, {k: v for k, v in out.items() if v is not None}

    # ------------------------------------------------------------------ fine-tuning (distillation) loss
    def distill_loss_fwd(self, H: torch.Tensor, X: torch.Tensor, TZ: torch.Tensor, beta: float = 0.9,
                         discount: float = 1.0) -> torch.Tensor:
        """TZ[T,n,V] teacher logits (storage dtype) -> loss[T] fp32.  Keeps ctx for distill_loss_bwd."""
        T = H.shape[0]
        ds = self.desc(T)
        self._dctx = _scratch(binding.cp_head_distill_ctx_bytes(ds), self.device)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_DISTILL_FWD), self.device)
        loss = torch.empty(T, dtype=torch.float32, device=self.device)
        binding.cp_head_distill_loss_fwd(ds, H, self.W, self.U, self.G, X, TZ, beta, discount, loss, self._dctx, ws)
        return loss

    def distill_loss_bwd(self, H: torch.Tensor, X: torch.Tensor, TZ: torch.Tensor,
                         dloss: Optional[torch.Tensor] = None, scale: float = 1.0, want_dU: bool = False) -> Dict[str, torch.Tensor]:
        T = H.shape[0]
        ds = self.desc(T)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_DISTILL_BWD), self.device)
        f32 = dict(dtype=torch.float32, device=self.device)
        out = {
            "dH": torch.empty((T, self.d), **f32),
            "dW": torch.empty((self.n, self.r, self.d, self.d), **f32),
            "dU": torch.empty((self.V, self.d), **f32) if want_dU else None,
            "dG": torch.empty((self.r, self.d), **f32),
        }
        binding.cp_head_distill_loss_bwd(ds, H, self.W, self.U, self.G, X, TZ, dloss, scale, self._dctx,
                                         out["dH"], out["dW"], out["dU"], out["dG"], ws)
        return {k: v for k, v in out.items() if v is not None}

    # ------------------------------------------------------------------ draft
    def draft_sample(self, H: torch.Tensor, uniforms: torch.Tensor):
        B = H.shape[0]
        ds = self.desc(B)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_DRAFT), self.device)
        alpha = torch.empty(B, dtype=torch.int32, device=self.device)
        tokens = torch.empty((B, self.n), dtype=torch.int32, device=self.device)
        logq = torch.empty(B, dtype=torch.float32, device=self.device)
        binding.cp_head_draft_sample(ds, H, self.W, self.U, self.G, uniforms, alpha, tokens, logq, ws)
        return alpha, tokens, logq

    # ------------------------------------------------------------------ next-token distribution, paper-form sampler
    def first_token_logprob(self, H: torch.Tensor) -> torch.Tensor:
        B = H.shape[0]
        ds = self.desc(B)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_FIRST_TOKEN), self.device)
        logp = torch.empty((B, self.V), dtype=torch.float32, device=self.device)
        binding.cp_head_first_token_logprob(ds, H, self.W, self.U, self.G, logp, ws)
        return logp

    def draft_sample_sequential(self, H: torch.Tensor, uniforms: torch.Tensor):
        B = H.shape[0]
        ds = self.desc(B)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_DRAFT_SEQUENTIAL), self.device)
        tokens = torch.empty((B, self.n), dtype=torch.int32, device=self.device)
        logq = torch.empty(B, dtype=torch.float32, device=self.device)
        binding.cp_head_draft_sample_sequential(ds, H, self.W, self.U, self.G, uniforms, tokens, logq, ws)
        return tokens, logq

    def aux_balance(self, H: torch.Tensor):
        T = H.shape[0]
        ds = self.desc(T)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_AUX_BALANCE), self.device)
        counts = torch.empty(self.r, dtype=torch.int64, device=self.device)
        laux = torch.empty(1, dtype=torch.float32, device=self.device)
        binding.cp_head_aux_balance(ds, H, self.G, counts, laux, ws)
        return counts, laux


class CpFullHead:
    """Full heads F[n,r,V,d] (one V x d matrix per future token and expert) plus the gate, on the device."""

    def __init__(self, F: np.ndarray, G: np.ndarray, dtype: str = "bf16", flags: int = 0, device="cuda:0"):
        self.device = torch.device(device)
        self.dtype = dtype
        self.flags = flags
        self.n, self.r, self.V, self.d = F.shape
        self.F = to_device(F, dtype, self.device)
        self.G = to_device(G, dtype, self.device)
        self._ctx: Optional[torch.Tensor] = None

    def desc(self, T: int) -> binding.Desc:
        return binding.make_desc(T, self.d, self.V, self.n, self.r,
                                 binding.BF16 if self.dtype == "bf16" else binding.FP32, self.flags)

    def loss_fwd(self, H: torch.Tensor, X: torch.Tensor) -> torch.Tensor:
        T = H.shape[0]
        ds = self.desc(T)
        self._ctx = _scratch(binding.cp_head_full_ctx_bytes(ds), self.device)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_FULL_LOSS_FWD), self.device)
        loss = torch.empty(T, dtype=torch.float32, device=self.device)
        binding.cp_head_full_loss_fwd(ds, H, self.F, self.G, X, loss, self._ctx, ws)
        return loss

    def loss_bwd(self, H: torch.Tensor, X: torch.Tensor, dloss: Optional[torch.Tensor] = None, scale: float = 1.0,
                 want_dF: bool = True) -> Dict[str, torch.Tensor]:
        assert self._ctx is not None, "call loss_fwd first"
        T = H.shape[0]
        ds = self.desc(T)
        ws = _scratch(binding.cp_head_workspace_bytes(ds, binding.OP_FULL_LOSS_BWD), self.device)
        f32 = dict(dtype=torch.float32, device=self.device)
        out = {
            "dH": torch.empty((T, self.d), **f32),
            "dF": torch.empty((self.n, self.r, self.V, self.d), **f32) if want_dF else None,
            "dG": torch.empty((self.r, self.d), **f32),
        }
        binding.cp_head_full_loss_bwd(ds, H, self.F, self.G, X, dloss, scale, self._ctx,
                                      out["dH"], out["dF"], out["dG"], ws)
        return {k: v for k, v in out.items() if v is not None}

"""Thin ctypes binding of libcphead.so: argument marshalling only.

Function names mirror the C ABI (``include/cp_head.h``).  Device buffers are
torch tensors (PyTorch supplies device memory and streams, nothing else);
every step of the computation runs in the library's own kernels.  There is no
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

FP32 = 0
BF16 = 1
FORCE_GENERIC = 1
MIN_WORKSPACE = 2
KEEP_LOGITS = 4
OP_LOSS_FWD, OP_LOSS_BWD, OP_DRAFT = 0, 1, 2
OP_FIRST_TOKEN, OP_DRAFT_SEQUENTIAL, OP_AUX_BALANCE = 3, 4, 5
OP_FULL_LOSS_FWD, OP_FULL_LOSS_BWD = 6, 7
OP_DISTILL_FWD, OP_DISTILL_BWD = 8, 9
OP_LOSS_FWD_BWD = 10

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcphead.so")
_lib: Optional[ctypes.CDLL] = None

EXPORTS = ("cp_head_strerror", "cp_head_ctx_bytes", "cp_head_workspace_bytes",
           "cp_head_loss_fwd", "cp_head_loss_bwd", "cp_head_loss_fwd_bwd", "cp_head_draft_sample",
           "cp_head_draft_sample_static",
           "cp_head_first_token_logprob", "cp_head_draft_sample_sequential", "cp_head_aux_balance",
           "cp_head_full_ctx_bytes", "cp_head_full_loss_fwd", "cp_head_full_loss_bwd",
           "cp_head_distill_ctx_bytes", "cp_head_distill_loss_fwd", "cp_head_distill_loss_bwd",
           "cp_head_profile_enable", "cp_head_profile_read")


class CpHeadError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class Desc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("d", ctypes.c_int32), ("V", ctypes.c_int32), ("n", ctypes.c_int32),
                ("r", ctypes.c_int32), ("dtype", ctypes.c_int32), ("flags", ctypes.c_int32)]


class KernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 32), ("launches", ctypes.c_int32), ("total_ms", ctypes.c_double),
                ("total_work", ctypes.c_double)]


def lib() -> ctypes.CDLL:
    """Load libcphead.so (built by ``paper_2410_17765_amd.build``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2410_17765_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.cp_head_strerror.restype = ctypes.c_char_p
        L.cp_head_strerror.argtypes = [ctypes.c_int]
        L.cp_head_ctx_bytes.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(sz)]
        L.cp_head_workspace_bytes.argtypes = [ctypes.POINTER(Desc), ctypes.c_int, ctypes.POINTER(sz)]
        L.cp_head_loss_fwd.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.cp_head_loss_bwd.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, ctypes.c_float, vp,
                                       vp, vp, vp, vp, vp, sz, vp]
        L.cp_head_loss_fwd_bwd.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, ctypes.c_float, vp,
                                           vp, vp, vp, vp, vp, sz, vp]
        L.cp_head_draft_sample.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.cp_head_draft_sample_static.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.cp_head_first_token_logprob.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, sz, vp]
        L.cp_head_draft_sample_sequential.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.cp_head_aux_balance.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, sz, vp]
        L.cp_head_full_ctx_bytes.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(sz)]
        L.cp_head_full_loss_fwd.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.cp_head_full_loss_bwd.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, ctypes.c_float, vp,
                                            vp, vp, vp, vp, sz, vp]
        L.cp_head_distill_ctx_bytes.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(sz)]
        L.cp_head_distill_loss_fwd.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, ctypes.c_float,
                                               ctypes.c_float, vp, vp, vp, sz, vp]
        L.cp_head_distill_loss_bwd.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, vp, ctypes.c_float, vp,
                                               vp, vp, vp, vp, vp, sz, vp]
        L.cp_head_profile_enable.argtypes = [ctypes.c_int]
        L.cp_head_profile_read.argtypes = [ctypes.POINTER(KernelTime), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        for name in EXPORTS[1:]:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().cp_head_strerror(int(code)).decode()


def make_desc(T: int, d: int, V: int, n: int, r: int, dtype: int, flags: int = 0) -> Desc:
    return Desc(T, d, V, n, r, dtype, flags)


def cp_head_ctx_bytes(desc: Desc) -> int:
    out = ctypes.c_size_t(0)
    rc = lib().cp_head_ctx_bytes(ctypes.byref(desc), ctypes.byref(out))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_ctx_bytes")
    return out.value


def cp_head_workspace_bytes(desc: Desc, op: int) -> int:
    out = ctypes.c_size_t(0)
    rc = lib().cp_head_workspace_bytes(ctypes.byref(desc), int(op), ctypes.byref(out))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_workspace_bytes")
    return out.value


def _ptr(t) -> Optional[int]:
    """Device (or raw integer) pointer of a tensor; None passes NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors must be contiguous"
    return t.data_ptr()


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return int(stream)


def cp_head_loss_fwd(desc: Desc, H, W, U, G, X, loss, ctx, workspace, stream=None) -> None:
    rc = lib().cp_head_loss_fwd(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(U), _ptr(G), _ptr(X), _ptr(loss),
                                _ptr(ctx), _ptr(workspace), _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_loss_fwd")


def cp_head_loss_bwd(desc: Desc, H, W, U, G, X, dloss, scale: float, ctx, dH, dW, dU, dG, workspace,
                     stream=None) -> None:
    rc = lib().cp_head_loss_bwd(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(U), _ptr(G), _ptr(X), _ptr(dloss),
                                float(scale), _ptr(ctx), _ptr(dH), _ptr(dW), _ptr(dU), _ptr(dG),
                                _ptr(workspace), _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_loss_bwd")


def cp_head_loss_fwd_bwd(desc: Desc, H, W, U, G, X, dloss, scale, loss, dH, dW, dU, dG, workspace, stream=None) -> None:
    rc = lib().cp_head_loss_fwd_bwd(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(U), _ptr(G), _ptr(X), _ptr(dloss),
                                    float(scale), _ptr(loss), _ptr(dH), _ptr(dW), _ptr(dU), _ptr(dG),
                                    _ptr(workspace), _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_loss_fwd_bwd")


def cp_head_draft_sample(desc: Desc, H, W, U, G, uniforms, alpha, tokens, logq, workspace, stream=None) -> None:
    rc = lib().cp_head_draft_sample(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(U), _ptr(G), _ptr(uniforms),
                                    _ptr(alpha), _ptr(tokens), _ptr(logq), _ptr(workspace), _nbytes(workspace),
                                    _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_draft_sample")


STATIC_SCRATCH_BYTES = 48 << 20
ERR_STATIC_SCRATCH = -5


def cp_head_draft_sample_static(desc: Desc, H, W, U, G, uniforms, alpha, tokens, logq, stream=None) -> None:
    """The draft step on the library's own static scratch array: no workspace argument, no allocation."""
    rc = lib().cp_head_draft_sample_static(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(U), _ptr(G), _ptr(uniforms),
                                           _ptr(alpha), _ptr(tokens), _ptr(logq), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_draft_sample_static")


def cp_head_first_token_logprob(desc: Desc, H, W, U, G, logp, workspace, stream=None) -> None:
    rc = lib().cp_head_first_token_logprob(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(U), _ptr(G), _ptr(logp),
                                           _ptr(workspace), _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_first_token_logprob")


def cp_head_draft_sample_sequential(desc: Desc, H, W, U, G, uniforms, tokens, logq, workspace, stream=None) -> None:
    rc = lib().cp_head_draft_sample_sequential(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(U), _ptr(G),
                                               _ptr(uniforms), _ptr(tokens), _ptr(logq), _ptr(workspace),
                                               _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_draft_sample_sequential")


def cp_head_aux_balance(desc: Desc, H, G, counts, laux, workspace, stream=None) -> None:
    rc = lib().cp_head_aux_balance(ctypes.byref(desc), _ptr(H), _ptr(G), _ptr(counts), _ptr(laux), _ptr(workspace),
                                   _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_aux_balance")


def cp_head_full_ctx_bytes(desc: Desc) -> int:
    out = ctypes.c_size_t(0)
    rc = lib().cp_head_full_ctx_bytes(ctypes.byref(desc), ctypes.byref(out))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_full_ctx_bytes")
    return out.value


def cp_head_full_loss_fwd(desc: Desc, H, F, G, X, loss, ctx, workspace, stream=None) -> None:
    rc = lib().cp_head_full_loss_fwd(ctypes.byref(desc), _ptr(H), _ptr(F), _ptr(G), _ptr(X), _ptr(loss), _ptr(ctx),
                                     _ptr(workspace), _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_full_loss_fwd")


def cp_head_full_loss_bwd(desc: Desc, H, F, G, X, dloss, scale, ctx, dH, dF, dG, workspace, stream=None) -> None:
    rc = lib().cp_head_full_loss_bwd(ctypes.byref(desc), _ptr(H), _ptr(F), _ptr(G), _ptr(X), _ptr(dloss),
                                     ctypes.c_float(scale), _ptr(ctx), _ptr(dH), _ptr(dF), _ptr(dG),
                                     _ptr(workspace), _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_full_loss_bwd")


def cp_head_distill_ctx_bytes(desc: Desc) -> int:
    out = ctypes.c_size_t(0)
    rc = lib().cp_head_distill_ctx_bytes(ctypes.byref(desc), ctypes.byref(out))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_distill_ctx_bytes")
    return out.value


def cp_head_distill_loss_fwd(desc: Desc, H, W, U, G, X, TZ, beta, discount, loss, ctx, workspace, stream=None) -> None:
    rc = lib().cp_head_distill_loss_fwd(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(U), _ptr(G), _ptr(X), _ptr(TZ),
                                        ctypes.c_float(beta), ctypes.c_float(discount), _ptr(loss), _ptr(ctx),
                                        _ptr(workspace), _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_distill_loss_fwd")


def cp_head_distill_loss_bwd(desc: Desc, H, W, U, G, X, TZ, dloss, scale, ctx, dH, dW, dU, dG, workspace,
                             stream=None) -> None:
    rc = lib().cp_head_distill_loss_bwd(ctypes.byref(desc), _ptr(H), _ptr(W), _ptr(U), _ptr(G), _ptr(X), _ptr(TZ),
                                        _ptr(dloss), ctypes.c_float(scale), _ptr(ctx), _ptr(dH), _ptr(dW), _ptr(dU),
                                        _ptr(dG), _ptr(workspace), _nbytes(workspace), _stream(stream))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_distill_loss_bwd")


def cp_head_profile_enable(on: bool) -> None:
    lib().cp_head_profile_enable(1 if on else 0)


def cp_head_profile_read(max_entries: int = 64):
    """[(name, launches, total_ms, total_work)] since profiling was enabled (clears the list)."""
    rows = (KernelTime * max_entries)()
    count = ctypes.c_int(0)
    rc = lib().cp_head_profile_read(rows, max_entries, ctypes.byref(count))
    if rc != 0:
        raise CpHeadError(rc, "cp_head_profile_read")
    return [(rows[i].name.decode(), rows[i].launches, rows[i].total_ms, rows[i].total_work)
            for i in range(min(count.value, max_entries))]

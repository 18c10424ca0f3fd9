"""ctypes front end of the plain fp64 CPU oracle (``cp_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
``cpu_baseline`` leg of the benchmark.  Nothing in the product package may
import this module, and this module imports nothing from the product package.

The C file is compiled twice, once reading ``float`` inputs (values exact in
the storage type, as the GPU sees them) and once reading ``double`` inputs
(for finite-difference tests); the array dtype selects the library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cp_oracle.c")
_LIBS: Dict[str, ctypes.CDLL] = {}


class _Shape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("d", ctypes.c_int32), ("V", ctypes.c_int32),
                ("n", ctypes.c_int32), ("r", ctypes.c_int32), ("round_y", ctypes.c_int32)]


def _lib_path(kind: str) -> str:
    return os.path.join(_HERE, f"libcp_oracle_{kind}.so")


def build(force: bool = False) -> None:
    """Compile the oracle with gcc (-O2, OpenMP) for both input types."""
    for kind, ctype in (("f32", "float"), ("f64", "double")):
        out = _lib_path(kind)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               f"-DCPO_IN_T={ctype}", f"-DCPO_PREFIX=cpo_{kind}_", _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)
        _LIBS.pop(kind, None)


def _lib(kind: str) -> ctypes.CDLL:
    if kind not in _LIBS:
        if not os.path.exists(_lib_path(kind)) or os.path.getmtime(_lib_path(kind)) < os.path.getmtime(_SRC):
            build()
        _LIBS[kind] = ctypes.CDLL(_lib_path(kind))
    return _LIBS[kind]


def _prep(H, W, U, G):
    """Pick the library from the dtype and make the arrays contiguous."""
    kinds = {np.asarray(a).dtype for a in (H, W, U, G)}
    if kinds == {np.dtype(np.float32)}:
        kind, dt = "f32", np.float32
    else:
        kind, dt = "f64", np.float64
    arrs = [np.ascontiguousarray(a, dtype=dt) for a in (H, W, U, G)]
    return kind, arrs


def _shape(H, W, U, round_y: bool) -> _Shape:
    T, d = H.shape
    n, r = W.shape[0], W.shape[1]
    assert W.shape == (n, r, d, d), W.shape
    assert U.shape[1] == d
    return _Shape(T, d, U.shape[0], n, r, 1 if round_y else 0)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    return len(os.sched_getaffinity(0))


def loss_fwd(H, W, U, G, X, round_y: bool = False, details: bool = False):
    """Per-position loss [T] (fp64).  With details: (loss, logw[T,r], C[T,n,r], lse[T,n,r])."""
    kind, (H, W, U, G) = _prep(H, W, U, G)
    sh = _shape(H, W, U, round_y)
    X = np.ascontiguousarray(X, dtype=np.int32)
    assert X.shape == (sh.T, sh.n)
    loss = np.empty(sh.T, dtype=np.float64)
    logw = np.empty((sh.T, sh.r)) if details else None
    C = np.empty((sh.T, sh.n, sh.r)) if details else None
    lse = np.empty((sh.T, sh.n, sh.r)) if details else None
    fn = getattr(_lib(kind), f"cpo_{kind}_loss_fwd")
    fn.restype = ctypes.c_int
    rc = fn(ctypes.byref(sh), _p(H), _p(W), _p(U), _p(G), _p(X), _p(loss), _p(logw), _p(C), _p(lse))
    if rc != 0:
        raise RuntimeError("oracle loss_fwd failed")
    return (loss, logw, C, lse) if details else loss


def joint_prob_naive(H, W, U, G, X):
    """Joint probability per position, straight in probability space (tiny sizes only)."""
    kind, (H, W, U, G) = _prep(H, W, U, G)
    sh = _shape(H, W, U, False)
    X = np.ascontiguousarray(X, dtype=np.int32)
    prob = np.empty(sh.T, dtype=np.float64)
    fn = getattr(_lib(kind), f"cpo_{kind}_joint_prob_naive")
    fn.restype = ctypes.c_int
    if fn(ctypes.byref(sh), _p(H), _p(W), _p(U), _p(G), _p(X), _p(prob)) != 0:
        raise RuntimeError("oracle joint_prob_naive failed")
    return prob


def loss_bwd(H, W, U, G, X, dloss=None, want=("dH", "dW", "dU", "dG")):
    """Gradients of sum_t dloss[t]*loss[t]: dict with dH[T,d], dW[n,r,d,d], dU[V,d], dG[r,d] (fp64)."""
    kind, (H, W, U, G) = _prep(H, W, U, G)
    sh = _shape(H, W, U, False)
    X = np.ascontiguousarray(X, dtype=np.int32)
    dl = None if dloss is None else np.ascontiguousarray(dloss, dtype=np.float64)
    out = {
        "dH": np.empty(H.shape) if "dH" in want else None,
        "dW": np.empty(W.shape) if "dW" in want else None,
        "dU": np.empty(U.shape) if "dU" in want else None,
        "dG": np.empty(G.shape) if "dG" in want else None,
    }
    fn = getattr(_lib(kind), f"cpo_{kind}_loss_bwd")
    fn.restype = ctypes.c_int
    rc = fn(ctypes.byref(sh), _p(H), _p(W), _p(U), _p(G), _p(X), _p(dl),
            _p(out["dH"]), _p(out["dW"]), _p(out["dU"]), _p(out["dG"]))
    if rc != 0:
        raise RuntimeError("oracle loss_bwd failed")
    return {k: v for k, v in out.items() if v is not None}


def draft_sample(H, W, U, G, uniforms, round_y: bool = True, alpha_in=None, want_cdf: bool = False,
                 want_y: bool = False, y_nudge=None):
    """Draw (alpha[B], tokens[B,n], logq[B]); with want_cdf also cdf_w[B,r], cdf_tok[B,n,V]; with want_y
    also the exact y[B,n,r,d] before rounding.  y_nudge[B,n,r,d] is added to y before rounding."""
    kind, (H, W, U, G) = _prep(H, W, U, G)
    sh = _shape(H, W, U, round_y)
    u = np.ascontiguousarray(uniforms, dtype=np.float64)
    assert u.shape == (sh.T, 1 + sh.n)
    a_in = None if alpha_in is None else np.ascontiguousarray(alpha_in, dtype=np.int32)
    alpha = np.empty(sh.T, dtype=np.int32)
    tokens = np.empty((sh.T, sh.n), dtype=np.int32)
    logq = np.empty(sh.T, dtype=np.float64)
    cdf_w = np.empty((sh.T, sh.r)) if want_cdf else None
    cdf_tok = np.empty((sh.T, sh.n, sh.V)) if want_cdf else None
    y_exact = np.empty((sh.T, sh.n, sh.r, sh.d)) if want_y else None
    nudge = None if y_nudge is None else np.ascontiguousarray(y_nudge, dtype=np.float64)
    assert nudge is None or nudge.shape == (sh.T, sh.n, sh.r, sh.d)
    fn = getattr(_lib(kind), f"cpo_{kind}_draft_sample")
    fn.restype = ctypes.c_int
    rc = fn(ctypes.byref(sh), _p(H), _p(W), _p(U), _p(G), _p(u), _p(a_in),
            _p(alpha), _p(tokens), _p(logq), _p(cdf_w), _p(cdf_tok), _p(y_exact), _p(nudge))
    if rc != 0:
        raise RuntimeError("oracle draft_sample failed")
    out = [alpha, tokens, logq]
    if want_cdf:
        out += [cdf_w, cdf_tok]
    if want_y:
        out.append(y_exact)
    return tuple(out)


def sequential_conditional(H, W, U, G, t: int, prefix, round_y: bool = False):
    """P(x_s | prefix) over the vocabulary for position t, s = len(prefix) (paper's sequential scheme)."""
    kind, (H, W, U, G) = _prep(H, W, U, G)
    sh = _shape(H, W, U, round_y)
    prefix = np.ascontiguousarray(prefix, dtype=np.int32)
    prob = np.empty(sh.V, dtype=np.float64)
    fn = getattr(_lib(kind), f"cpo_{kind}_sequential_conditional")
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    rc = fn(ctypes.cast(ctypes.byref(sh), ctypes.c_void_p), _p(H), _p(W), _p(U), _p(G),
            int(t), int(len(prefix)), _p(prefix) if len(prefix) else None, _p(prob))
    if rc != 0:
        raise RuntimeError("oracle sequential_conditional failed")
    return prob


def first_token_logprob(H, W, U, G, round_y: bool = False, y_nudge=None):
    """logp[B,V]: log of the first-token marginal (eq. 11).  y_nudge[B,r,d] is added to y before rounding."""
    kind, (H, W, U, G) = _prep(H, W, U, G)
    sh = _shape(H, W, U, round_y)
    out = np.empty((sh.T, sh.V), dtype=np.float64)
    nudge = None if y_nudge is None else np.ascontiguousarray(y_nudge, dtype=np.float64)
    assert nudge is None or nudge.shape == (sh.T, sh.r, sh.d)
    fn = getattr(_lib(kind), f"cpo_{kind}_first_token_logprob")
    fn.restype = ctypes.c_int
    if fn(ctypes.byref(sh), _p(H), _p(W), _p(U), _p(G), _p(nudge), _p(out)) != 0:
        raise RuntimeError("oracle first_token_logprob failed")
    return out


def draft_sample_sequential(H, W, U, G, uniforms, round_y: bool = True, want_cdf: bool = False, y_nudge=None):
    """The paper's sequential scheme: (tokens[B,n], logq[B]) [+ cdf[B,n,V]] from uniforms[B,n].
    y_nudge[B,n,r,d] is added to y before rounding."""
    kind, (H, W, U, G) = _prep(H, W, U, G)
    sh = _shape(H, W, U, round_y)
    u = np.ascontiguousarray(uniforms, dtype=np.float64)
    assert u.shape == (sh.T, sh.n)
    tokens = np.empty((sh.T, sh.n), dtype=np.int32)
    logq = np.empty(sh.T, dtype=np.float64)
    cdf = np.empty((sh.T, sh.n, sh.V)) if want_cdf else None
    nudge = None if y_nudge is None else np.ascontiguousarray(y_nudge, dtype=np.float64)
    assert nudge is None or nudge.shape == (sh.T, sh.n, sh.r, sh.d)
    fn = getattr(_lib(kind), f"cpo_{kind}_draft_sample_sequential")
    fn.restype = ctypes.c_int
    if fn(ctypes.byref(sh), _p(H), _p(W), _p(U), _p(G), _p(u), _p(nudge), _p(tokens), _p(logq), _p(cdf)) != 0:
        raise RuntimeError("oracle draft_sample_sequential failed")
    return (tokens, logq, cdf) if want_cdf else (tokens, logq)


def aux_balance(H, G):
    """(counts[r] int64, L_aux) of eq. 10 for the positions in H."""
    H = np.asarray(H)
    G = np.asarray(G)
    if H.dtype == np.float32 and G.dtype == np.float32:
        kind, dt = "f32", np.float32
    else:
        kind, dt = "f64", np.float64
    H = np.ascontiguousarray(H, dtype=dt)
    G = np.ascontiguousarray(G, dtype=dt)
    sh = _Shape(H.shape[0], H.shape[1], 1, 1, G.shape[0], 0)
    counts = np.zeros(G.shape[0], dtype=np.int64)
    laux = ctypes.c_double(0.0)
    fn = getattr(_lib(kind), f"cpo_{kind}_aux_balance")
    fn.restype = ctypes.c_int
    if fn(ctypes.byref(sh), _p(H), _p(G), _p(counts), ctypes.byref(laux)) != 0:
        raise RuntimeError("oracle aux_balance failed")
    return counts, laux.value


def _prep_full(H, F, G):
    kinds = {np.asarray(a).dtype for a in (H, F, G)}
    kind, dt = ("f32", np.float32) if kinds == {np.dtype(np.float32)} else ("f64", np.float64)
    H, F, G = (np.ascontiguousarray(a, dtype=dt) for a in (H, F, G))
    n, r, V, d = F.shape
    assert H.shape[1] == d and G.shape == (r, d)
    return kind, H, F, G, _Shape(H.shape[0], d, V, n, r, 0)


def full_loss_fwd(H, F, G, X, details: bool = False):
    """Loss with full heads F[n,r,V,d] (eq. 6 as printed): loss[T] (and logw, C, lse with details)."""
    kind, H, F, G, sh = _prep_full(H, F, G)
    X = np.ascontiguousarray(X, dtype=np.int32)
    assert X.shape == (sh.T, sh.n)
    loss = np.empty(sh.T)
    logw = np.empty((sh.T, sh.r)) if details else None
    C = np.empty((sh.T, sh.n, sh.r)) if details else None
    lse = np.empty((sh.T, sh.n, sh.r)) if details else None
    fn = getattr(_lib(kind), f"cpo_{kind}_full_loss_fwd")
    fn.restype = ctypes.c_int
    if fn(ctypes.byref(sh), _p(H), _p(F), _p(G), _p(X), _p(loss), _p(logw), _p(C), _p(lse)) != 0:
        raise RuntimeError("oracle full_loss_fwd failed")
    return (loss, logw, C, lse) if details else loss


def full_loss_bwd(H, F, G, X, dloss=None, want=("dH", "dF", "dG")):
    """Gradients of sum_t dloss[t] * loss[t] with full heads: dict with dH[T,d], dF[n,r,V,d], dG[r,d]."""
    kind, H, F, G, sh = _prep_full(H, F, G)
    X = np.ascontiguousarray(X, dtype=np.int32)
    dl = None if dloss is None else np.ascontiguousarray(dloss, dtype=np.float64)
    out = {"dH": np.empty(H.shape) if "dH" in want else None,
           "dF": np.empty(F.shape) if "dF" in want else None,
           "dG": np.empty(G.shape) if "dG" in want else None}
    fn = getattr(_lib(kind), f"cpo_{kind}_full_loss_bwd")
    fn.restype = ctypes.c_int
    if fn(ctypes.byref(sh), _p(H), _p(F), _p(G), _p(X), _p(dl), _p(out["dH"]), _p(out["dF"]), _p(out["dG"])) != 0:
        raise RuntimeError("oracle full_loss_bwd failed")
    return {k: v for k, v in out.items() if v is not None}


def _teacher(TZ, kind, sh):
    TZ = np.ascontiguousarray(TZ, dtype=np.float32 if kind == "f32" else np.float64)
    assert TZ.shape == (sh.T, sh.n, sh.V), TZ.shape
    return TZ


def distill_loss_fwd(H, W, U, G, X, TZ, beta: float = 0.9, disc: float = 1.0, details: bool = False):
    """Head-only fine-tuning loss (eq. 14 and the discounted sum after it) against teacher logits TZ[T,n,V]:
    loss[T] (and kl[T,n], ce[T,n] with details)."""
    kinds = {np.asarray(a).dtype for a in (H, W, U, G, TZ)}
    if kinds != {np.dtype(np.float32)}:
        H, W, U, G = (np.asarray(a, dtype=np.float64) for a in (H, W, U, G))
    kind, (H, W, U, G) = _prep(H, W, U, G)
    sh = _shape(H, W, U, False)
    X = np.ascontiguousarray(X, dtype=np.int32)
    TZ = _teacher(TZ, kind, sh)
    loss = np.empty(sh.T)
    kl = np.empty((sh.T, sh.n)) if details else None
    ce = np.empty((sh.T, sh.n)) if details else None
    fn = getattr(_lib(kind), f"cpo_{kind}_distill_loss_fwd")
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p] * 7 + [ctypes.c_double, ctypes.c_double] + [ctypes.c_void_p] * 3
    rc = fn(ctypes.cast(ctypes.byref(sh), ctypes.c_void_p), _p(H), _p(W), _p(U), _p(G), _p(X), _p(TZ),
            float(beta), float(disc), _p(loss), _p(kl), _p(ce))
    if rc != 0:
        raise RuntimeError("oracle distill_loss_fwd failed")
    return (loss, kl, ce) if details else loss


def distill_loss_bwd(H, W, U, G, X, TZ, beta: float = 0.9, disc: float = 1.0, dloss=None,
                     want=("dH", "dW", "dU", "dG")):
    """Gradients of sum_t dloss[t] * distill_loss[t] (teacher logits are constants)."""
    kinds = {np.asarray(a).dtype for a in (H, W, U, G, TZ)}
    if kinds != {np.dtype(np.float32)}:
        H, W, U, G = (np.asarray(a, dtype=np.float64) for a in (H, W, U, G))
    kind, (H, W, U, G) = _prep(H, W, U, G)
    sh = _shape(H, W, U, False)
    X = np.ascontiguousarray(X, dtype=np.int32)
    TZ = _teacher(TZ, kind, sh)
    dl = None if dloss is None else np.ascontiguousarray(dloss, dtype=np.float64)
    out = {"dH": np.empty(H.shape) if "dH" in want else None, "dW": np.empty(W.shape) if "dW" in want else None,
           "dU": np.empty(U.shape) if "dU" in want else None, "dG": np.empty(G.shape) if "dG" in want else None}
    fn = getattr(_lib(kind), f"cpo_{kind}_distill_loss_bwd")
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p] * 7 + [ctypes.c_double, ctypes.c_double] + [ctypes.c_void_p] * 5
    rc = fn(ctypes.cast(ctypes.byref(sh), ctypes.c_void_p), _p(H), _p(W), _p(U), _p(G), _p(X), _p(TZ),
            float(beta), float(disc), _p(dl), _p(out["dH"]), _p(out["dW"]), _p(out["dU"]), _p(out["dG"]))
    if rc != 0:
        raise RuntimeError("oracle distill_loss_bwd failed")
    return {k: v for k, v in out.items() if v is not None}


def round_to_bf16(v: float) -> float:
    fn = _lib("f64").cpo_f64_round_to_bf16
    fn.restype = ctypes.c_double
    fn.argtypes = [ctypes.c_double]
    return fn(float(v))

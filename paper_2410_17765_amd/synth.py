"""Seeded synthetic inputs for the CP multi-token-prediction head.

This module only *draws numbers*: it holds none of the method's arithmetic
(no projections, no softmax, no sampling of the model's distributions).  Both
the CPU oracle's tests and the GPU tests take their inputs from here so that
the two sides read exactly the same bits.

Recipe (every tensor has its own fixed stream, so tensors do not depend on
each other or on the order they are generated in):

* hidden states  H[T,d]      ~ N(0,1)
* head matrices  W[n,r,d,d]  ~ N(0,1/d)   (W[s,a] maps h -> y, row = output feature)
* unembedding    U[V,d]      ~ N(0,1/d)
* gate           G[r,d]      ~ N(0,1/d)
* targets        X[T,n]      uniform over V, or Zipf(1.1) over ranks 1..V mapped
                              through a seeded permutation of the vocabulary
* uniforms       [B,1+n]     float32 in [0,1)

Values are drawn in float32 and, for the bf16 configurations, rounded once to
bfloat16 (round-to-nearest-even).  They are returned as float32 arrays whose
values are exactly representable in the storage type, plus helpers that give
the raw bf16 bit patterns for upload to the device.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional, Sequence

import numpy as np

SEED_H = 1001
SEED_W = 1002
SEED_U = 1003
SEED_G = 1004
SEED_TARGETS = 1005
SEED_UNIFORMS = 1006
SEED_SUBSET = 1007
SEED_PERM = 1008
SEED_F = 1010
SEED_TEACHER = 1011


@dataclasses.dataclass(frozen=True)
class HeadConfig:
    """Shape of one CP-head workload.  T is the number of positions (or the
    draft batch B), d the hidden size, V the vocabulary, n the number of
    future tokens, r the CP rank (number of experts)."""
    name: str
    T: int
    d: int
    V: int
    n: int
    r: int
    dtype: str = "bf16"          # storage type of H, W, U, G: "fp32" or "bf16"
    targets: str = "zipf"        # "uniform" or "zipf"
    u_scale: float = 1.0         # extra factor on U (the peaked draft variant uses 8)

    @property
    def M(self) -> int:
        return self.T * self.n * self.r

    def with_(self, **kw) -> "HeadConfig":
        return dataclasses.replace(self, **kw)


# The five workloads of the build plus the brute-force normalisation case.
CONFIGS: Dict[str, HeadConfig] = {
    "tiny": HeadConfig("tiny", T=64, d=64, V=512, n=2, r=2, dtype="fp32", targets="uniform"),
    "brute": HeadConfig("brute", T=512, d=16, V=8, n=3, r=2, dtype="fp32", targets="uniform"),
    "small_lm": HeadConfig("small_lm", T=8192, d=2048, V=32000, n=4, r=8),
    "head_7b": HeadConfig("head_7b", T=16384, d=4096, V=32000, n=4, r=8),
    "large_vocab": HeadConfig("large_vocab", T=16384, d=4096, V=128256, n=3, r=4),
    "draft": HeadConfig("draft", T=8, d=4096, V=128256, n=4, r=8),
    # full V x d heads per (s, a) (no shared unembedding): the from-scratch parameterisation at a size
    # whose 2.1 GB of head weights the host can still generate in seconds
    "full_heads": HeadConfig("full_heads", T=8192, d=2048, V=32000, n=2, r=4),
}


# ----------------------------------------------------------------------------
# bfloat16 helpers (storage format only)
# ----------------------------------------------------------------------------

def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> uint16 bfloat16 bit patterns, round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 and return them as float32."""
    return bf16_bits_to_f32(bf16_bits(x))


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------

def _normal(seed: int, shape: Sequence[int], scale: float, dtype: str = "fp32") -> np.ndarray:
    """N(0, scale^2) float32 from a Philox stream, scaled in float32 and (for bf16 storage) rounded
    to bfloat16, nearest-even.  Drawn and rounded in bounded chunks with reused buffers."""
    if dtype not in ("fp32", "bf16"):
        raise ValueError(f"unknown storage dtype {dtype!r}")
    rng = np.random.Generator(np.random.Philox(seed))
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.float32)
    chunk = 1 << 22
    buf = np.empty(min(chunk, max(total, 1)), dtype=np.float32)
    tmp = np.empty(buf.shape, dtype=np.uint32)
    for lo in range(0, total, chunk):
        m = min(total, lo + chunk) - lo
        b = buf[:m]
        rng.standard_normal(m, dtype=np.float32, out=b)
        if scale != 1.0:
            b *= np.float32(scale)
        if dtype == "bf16":
            u, t = b.view(np.uint32), tmp[:m]
            np.right_shift(u, np.uint32(16), out=t)
            t &= np.uint32(1)
            t += np.uint32(0x7FFF)
            u += t
            u &= np.uint32(0xFFFF0000)
        out[lo:lo + m] = b
    return out.reshape(shape)


def hidden(cfg: HeadConfig, positions: Optional[np.ndarray] = None) -> np.ndarray:
    """H[T,d] (or the rows listed in `positions`, taken from the full tensor)."""
    H = _normal(SEED_H, (cfg.T, cfg.d), 1.0, cfg.dtype)
    if positions is not None:
        H = np.ascontiguousarray(H[np.asarray(positions)])
    return H


def head_weights(cfg: HeadConfig) -> np.ndarray:
    """W[n,r,d,d]; y = W[s,a] @ h."""
    return _normal(SEED_W, (cfg.n, cfg.r, cfg.d, cfg.d), cfg.d ** -0.5, cfg.dtype)


def unembedding(cfg: HeadConfig) -> np.ndarray:
    """U[V,d]."""
    return _normal(SEED_U, (cfg.V, cfg.d), cfg.u_scale * cfg.d ** -0.5, cfg.dtype)


def full_head_weights(cfg: HeadConfig) -> np.ndarray:
    """F[n,r,V,d]; z = F[s,a] @ h.  N(0, u_scale^2/d), the scale of the shared-unembedding logits."""
    return _normal(SEED_F, (cfg.n, cfg.r, cfg.V, cfg.d), cfg.u_scale * cfg.d ** -0.5, cfg.dtype)


def teacher_logits(cfg: HeadConfig, scale: float = 1.5) -> np.ndarray:
    """TZ[T,n,V]: logits of the original head for the fine-tuning loss, N(0, scale^2) (a moderately peaked
    distribution over the vocabulary), rounded to the storage type like the other tensors."""
    return _normal(SEED_TEACHER, (cfg.T, cfg.n, cfg.V), scale, cfg.dtype)


def gate(cfg: HeadConfig) -> np.ndarray:
    """G[r,d]."""
    return _normal(SEED_G, (cfg.r, cfg.d), cfg.d ** -0.5, cfg.dtype)


def vocabulary_permutation(V: int) -> np.ndarray:
    """Fixed seeded map from frequency rank (0 = most frequent) to token id."""
    rng = np.random.Generator(np.random.Philox(SEED_PERM))
    return rng.permutation(V).astype(np.int32)


def targets(cfg: HeadConfig, positions: Optional[np.ndarray] = None) -> np.ndarray:
    """X[T,n] int32; X[t,s] is the token that follows position t by s+1 steps."""
    rng = np.random.Generator(np.random.Philox(SEED_TARGETS))
    if cfg.targets == "uniform":
        X = rng.integers(0, cfg.V, size=(cfg.T, cfg.n), dtype=np.int64)
    elif cfg.targets == "zipf":
        ranks = np.arange(1, cfg.V + 1, dtype=np.float64)
        cdf = np.cumsum(ranks ** -1.1)
        cdf /= cdf[-1]
        u = rng.random(size=(cfg.T, cfg.n))
        k = np.minimum(np.searchsorted(cdf, u, side="right"), cfg.V - 1)
        X = vocabulary_permutation(cfg.V)[k]
    else:
        raise ValueError(f"unknown target distribution {cfg.targets!r}")
    X = np.ascontiguousarray(X, dtype=np.int32)
    if positions is not None:
        X = np.ascontiguousarray(X[np.asarray(positions)])
    return X


def uniforms(B: int, n: int, seed: int = SEED_UNIFORMS) -> np.ndarray:
    """[B,1+n] float32 in [0,1): column 0 draws the expert, column 1+s token s."""
    rng = np.random.Generator(np.random.Philox(seed))
    u = rng.random(size=(B, 1 + n), dtype=np.float32)
    return np.minimum(u, np.nextafter(np.float32(1.0), np.float32(0.0)))


def position_subset(T: int, count: int, seed: int = SEED_SUBSET) -> np.ndarray:
    """`count` distinct positions of [0,T), sorted."""
    rng = np.random.Generator(np.random.Philox(seed))
    return np.sort(rng.choice(T, size=min(count, T), replace=False)).astype(np.int64)


def upstream_grad(T: int, seed: int = 1009) -> np.ndarray:
    """A non-trivial upstream gradient dloss[T] (float32, around 1/T scale x T)."""
    rng = np.random.Generator(np.random.Philox(seed))
    return (0.5 + rng.random(size=T, dtype=np.float32)).astype(np.float32)


def make_inputs(cfg: HeadConfig, positions: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """All tensors of one workload (float32 holding storage-exact values)."""
    return {
        "H": hidden(cfg, positions),
        "W": head_weights(cfg),
        "U": unembedding(cfg),
        "G": gate(cfg),
        "X": targets(cfg, positions),
    }

"""Shared comparison helpers for the GPU parity tests (no method arithmetic of their own:
the expected values always come from the oracle)."""
import numpy as np

LOSS_ATOL = 2e-3          # per-position loss, max over all checked positions
GRAD_REL_FRO = 1e-2       # relative Frobenius error of each gradient tensor
CDF_BAND = 1e-5           # a draw may differ only if its uniform is this close to a CDF boundary


def rel_fro(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    return float(np.linalg.norm((got - ref).ravel()) / (den if den > 0 else 1.0))


def band_valid(cdf: np.ndarray, idx: int, u: float, band: float = CDF_BAND) -> bool:
    """Index `idx` is an admissible inverse-CDF draw for `u`: cdf[idx-1] - band <= u < cdf[idx] + band
    (the last index also takes everything above the final running sum)."""
    lo = cdf[idx - 1] if idx > 0 else -np.inf
    hi = cdf[idx] if idx < len(cdf) - 1 else np.inf
    return (lo - band <= u) and (u < hi + band)


def check_draft(oracle, H, W, U, G, u, alpha_gpu, tokens_gpu, logq_gpu, round_y, logq_atol=2e-3):
    """Compare one draft call with the oracle.  Returns a dict of match statistics; raises on a
    draw outside the CDF band or a wrong logq."""
    B, n = tokens_gpu.shape
    a_o, tok_o, logq_o, cdf_w, cdf_tok = oracle.draft_sample(H, W, U, G, u, round_y=round_y, want_cdf=True)
    stats = {"alpha_exact": int((a_o == alpha_gpu).sum()), "alpha_total": B,
             "tokens_exact": 0, "tokens_total": B * n}
    for b in range(B):
        assert band_valid(cdf_w[b], int(alpha_gpu[b]), float(u[b, 0])), ("alpha out of band", b)
    if (a_o != alpha_gpu).any():
        # token distributions are conditional on the expert: take the oracle's under the GPU's (valid) expert
        a_o, tok_o, logq_o, _, cdf_tok = oracle.draft_sample(H, W, U, G, u, round_y=round_y,
                                                            alpha_in=alpha_gpu, want_cdf=True)
    for b in range(B):
        for s in range(n):
            v = int(tokens_gpu[b, s])
            assert 0 <= v < cdf_tok.shape[2]
            assert band_valid(cdf_tok[b, s], v, float(u[b, 1 + s])), ("token out of band", b, s, v, int(tok_o[b, s]))
            stats["tokens_exact"] += int(v == tok_o[b, s])
    if logq_gpu is not None:
        # log-probability of the tuple the GPU drew, by the oracle's loss at those tokens
        lq = -oracle.loss_fwd(H, W, U, G, tokens_gpu.astype(np.int32), round_y=round_y)
        err = np.abs(lq - logq_gpu.astype(np.float64)).max()
        assert err <= logq_atol, ("logq", err)
        stats["logq_err"] = float(err)
    return stats

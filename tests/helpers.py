"""Shared comparison helpers for the GPU parity tests (no method arithmetic of their own:
the expected values always come from the oracle)."""
import numpy as np

LOSS_ATOL = 2e-3          # per-position loss, max over all checked positions
GRAD_REL_FRO = 1e-2       # relative Frobenius error of each gradient tensor
CDF_BAND = 1e-5           # a draw may differ only if its uniform is this close to a CDF boundary


def loss_atol_bf16(cfg) -> float:
    """Loss bound for the matrix-core path at shapes beyond the workloads'.  The path's one rounding after the
    inputs is y -> bf16 (an operand of the d -> V contraction); everything below is its consequence.
    * Each log-normaliser moves by dlse = sum_v p_v dz_v = dy . (U^T p).  With rows of U ~ N(0, I/d) the
      softmax-weighted mean row U^T p is y/d to first order, so dlse = sum_k y_k^2 eps_k / d with eps the
      relative rounding errors (rms about 1e-3): rms 1e-3 sqrt(3/d).  That does not average down over the
      vocabulary: 3e-5 at d = 4096, but 2.4e-4 at d = 64, where the largest of a few thousand positions
      (n factors each) reaches 2.5e-3.  The bound of the workloads (d >= 2048) is kept down to d = 256
      and grows as sqrt(256/d) below.
    * The loss sums n factors, each with its own log-normaliser: stated for n <= 4, it grows with n beyond.
    * Under V = 64 entries the softmax weights average nothing: a log-normaliser carries the error of its
      few logits in full (1e-2).
    fp32 storage runs on the plain path, which rounds nothing after the inputs: the workloads' bound as it is."""
    if cfg.dtype == "fp32":
        return LOSS_ATOL
    tol = LOSS_ATOL if cfg.V >= 64 else 1e-2
    return tol * max(1.0, cfg.n / 4) * max(1.0, (256.0 / cfg.d) ** 0.5)


def distill_loss_atol_bf16(cfg) -> float:
    """Loss bound of the fine-tuning loss (eq. 14) on the matrix-core path.  Its KL term weights the error of every
    single logit by the teacher's probability: with dz_v = U_v . dy (dy the bf16 rounding of y, relative rms
    2^-9 / sqrt(3) = 1.1e-3),
        d KL_k = (U^T (p^d - p^c)) . dy,   rms = 1.1e-3 u_scale sqrt(sum_v p^c_v^2 + sum_v p^d_v^2),
    independent of d.  For the synthetic teacher (logits N(0, 1.5^2)) and student (about N(0, 1)) the two sums are
    e^2.25 / V and e / V, together 12 / V: negligible at a language model's vocabulary (1.4e-5 at V = 32000), but
    3e-4 per token at V = 131, where single positions with a peaked teacher row reach five to six times the rms
    of a batch.  The bound is the training loss's, or ten times that rms over the n tokens of a position,
    whichever is larger; it scales with the logits (u_scale)."""
    base = loss_atol_bf16(cfg)
    if cfg.dtype == "fp32":
        return base * cfg.u_scale
    return max(base, 10 * 1.1e-3 * (12.0 * cfg.n / cfg.V) ** 0.5) * cfg.u_scale


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


TIE_ULPS = 1e-3   # |distance to a bf16 rounding midpoint| (in bf16 ulps) below which fp32 accumulation
                  # of y may legitimately round to the other neighbour than the exact value does


def _near_ties(y):
    """Indices of y (exact, fp64) that lie within TIE_ULPS of a bf16 rounding midpoint, and the nudge
    that pushes each across it."""
    y = np.asarray(y, dtype=np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(y), 1e-300))) - 7)
    q = y / ulp
    dist = (q - np.floor(q)) - 0.5
    idx = np.nonzero(np.abs(dist) < TIE_ULPS)[0]
    nudge = -np.where(dist[idx] >= 0, 1.0, -1.0) * (np.abs(dist[idx]) + 1e-4) * ulp[idx]
    return idx, nudge


def tie_variants(y_exact, limit=3):
    """All ways of rounding the elements of y_exact (any shape, exact fp64 values) that sit on a bf16
    rounding tie: yields (flips, nudge) with nudge shaped like y_exact, the unflipped variant first.
    If more than `limit` elements are on a tie, the `limit` closest to their midpoints are tried."""
    import itertools
    y = np.asarray(y_exact, dtype=np.float64)
    idx, nudge = _near_ties(y.reshape(-1))
    yield 0, np.zeros(y.shape)
    if len(idx) == 0:
        return
    if len(idx) > limit:
        keep = np.argsort(np.abs(nudge) / np.abs(y.reshape(-1)[idx]))[:limit]   # ~ distance in ulps
        idx, nudge = idx[keep], nudge[keep]
    for k in range(1, len(idx) + 1):
        for subset in itertools.combinations(range(len(idx)), k):
            nd = np.zeros(y.size)
            for j in subset:
                nd[idx[j]] = nudge[j]
            yield k, nd.reshape(y.shape)


def _valid_under_rounding_ties(oracle, H, W, U, G, u, b, s, a, v, y_exact):
    """The draw v for (b, s) under expert a is admissible if it is band-valid for some way of rounding
    the (at most 3) elements of y that sit on a rounding tie.  Returns the number of flipped elements
    that explains it, or 0 if nothing does."""
    import itertools
    idx, nudge = _near_ties(y_exact[b, s, a])
    if len(idx) == 0 or len(idx) > 3:
        return 0
    n, r, d = y_exact.shape[1:]
    for k in range(1, len(idx) + 1):
        for subset in itertools.combinations(range(len(idx)), k):
            nd = np.zeros((1, n, r, d))
            for j in subset:
                nd[0, s, a, idx[j]] = nudge[j]
            out = oracle.draft_sample(H[b:b + 1], W, U, G, u[b:b + 1], round_y=True, alpha_in=np.array([a], np.int32),
                                      want_cdf=True, y_nudge=nd)
            if band_valid(out[4][0, s], v, float(u[b, 1 + s])):
                return k
    return 0


def check_draft(oracle, H, W, U, G, u, alpha_gpu, tokens_gpu, logq_gpu, round_y, logq_atol=2e-3):
    """Compare one draft call with the oracle.  Returns a dict of match statistics; raises on a
    draw outside the CDF band (unless a rounding tie of y explains it) or a wrong logq."""
    B, n = tokens_gpu.shape
    a_o, tok_o, logq_o, cdf_w, cdf_tok, y_exact = oracle.draft_sample(H, W, U, G, u, round_y=round_y, want_cdf=True,
                                                                      want_y=True)
    stats = {"alpha_exact": int((a_o == alpha_gpu).sum()), "alpha_total": B,
             "tokens_exact": 0, "tokens_total": B * n, "tie_draws": 0, "band_draws": 0, "tie_logq_rows": 0}
    for b in range(B):
        assert band_valid(cdf_w[b], int(alpha_gpu[b]), float(u[b, 0])), ("alpha out of band", b)
    if (a_o != alpha_gpu).any():
        # token distributions are conditional on the expert: take the oracle's under the GPU's (valid) expert
        a_o, tok_o, logq_o, _, cdf_tok = oracle.draft_sample(H, W, U, G, u, round_y=round_y,
                                                            alpha_in=alpha_gpu, want_cdf=True)
    tie_rows = set()
    for b in range(B):
        for s in range(n):
            v = int(tokens_gpu[b, s])
            assert 0 <= v < cdf_tok.shape[2]
            if not band_valid(cdf_tok[b, s], v, float(u[b, 1 + s])):
                flips = _valid_under_rounding_ties(oracle, H, W, U, G, u, b, s, int(alpha_gpu[b]), v, y_exact) \
                    if round_y else 0
                assert flips > 0, ("token out of band", b, s, v, int(tok_o[b, s]))
                stats["tie_draws"] += 1
                tie_rows.add(b)
            elif v != tok_o[b, s]:
                stats["band_draws"] += 1        # another token than the oracle's, inside the band
            stats["tokens_exact"] += int(v == tok_o[b, s])
    if logq_gpu is not None:
        # log-probability of the tuple the GPU drew, by the oracle's loss at those tokens
        lq = -oracle.loss_fwd(H, W, U, G, tokens_gpu.astype(np.int32), round_y=round_y)
        errs = np.abs(lq - logq_gpu.astype(np.float64))
        for b in range(B):
            if b in tie_rows or errs[b] <= logq_atol:
                continue
            # logq reads all n r rows of y: an element of any of them on a bf16 rounding tie moves it; the
            # row must then be the oracle's under another rounding of those elements, draws included
            assert round_y, ("logq", b, errs[b])
            explained = False
            for flips, nd in tie_variants(y_exact[b]):
                if not flips:
                    continue
                out = oracle.draft_sample(H[b:b + 1], W, U, G, u[b:b + 1], round_y=True,
                                          alpha_in=np.array([alpha_gpu[b]], np.int32), want_cdf=True, y_nudge=nd[None])
                if abs(out[2][0] - logq_gpu[b]) <= logq_atol and all(
                        band_valid(out[4][0, s], int(tokens_gpu[b, s]), float(u[b, 1 + s])) for s in range(n)):
                    explained = True
                    break
            assert explained, ("logq off with no rounding tie to explain it", b, errs[b])
            stats["tie_logq_rows"] += 1
            errs[b] = 0.0
        keep = np.array([b not in tie_rows for b in range(B)])
        if keep.any():
            stats["logq_err"] = float(errs[keep].max())
    return stats


def check_sequential(oracle, H, W, U, G, u, tokens_gpu, logq_gpu, logq_atol=1e-3, round_y=True):
    """Compare one call of the sequential sampler (one uniform per token, u[B,n]) with the oracle.
    Every draw must lie inside the CDF band of the oracle's conditional under the prefix the GPU drew,
    and logq must be the oracle's joint log-probability of the drawn tuple; a row that fails either is
    accepted only if it is the oracle's row under another rounding of elements of y on a bf16 tie.
    Returns match statistics."""
    B, n = tokens_gpu.shape
    V = U.shape[0]
    tok_o, _, cdf = oracle.draft_sample_sequential(H, W, U, G, u, round_y=round_y, want_cdf=True)
    lq_err = np.abs(-oracle.loss_fwd(H, W, U, G, tokens_gpu.astype(np.int32), round_y=round_y) - logq_gpu)
    stats = {"tokens_exact": 0, "tokens_total": B * n, "tie_rows": 0}
    for b in range(B):
        ok = lq_err[b] <= logq_atol
        for s in range(n):
            v = int(tokens_gpu[b, s])
            assert 0 <= v < V
            if (tokens_gpu[b, :s] == tok_o[b, :s]).all():
                c = cdf[b, s]
            else:   # an admissible other draw earlier in the row: the oracle's conditional under that prefix
                c = np.cumsum(oracle.sequential_conditional(H, W, U, G, b, list(tokens_gpu[b, :s]), round_y=round_y))
            ok = ok and band_valid(c, v, float(u[b, s]))
            stats["tokens_exact"] += int(v == tok_o[b, s])
        if ok:
            continue
        assert round_y, ("row off", b, tokens_gpu[b], tok_o[b], lq_err[b])
        args = (H[b:b + 1], W, U, G)
        y = oracle.draft_sample(*args, np.zeros((1, 1 + n)), want_y=True)[-1]                     # [1,n,r,d]
        explained = False
        for flips, nd in tie_variants(y):
            if not flips:
                continue
            t2, q2, c2 = oracle.draft_sample_sequential(*args, u[b:b + 1], round_y=True, want_cdf=True, y_nudge=nd)
            if abs(q2[0] - logq_gpu[b]) <= logq_atol and (t2[0] == tokens_gpu[b]).all() and all(
                    band_valid(c2[0, s], int(tokens_gpu[b, s]), float(u[b, s])) for s in range(n)):
                explained = True
                break
        assert explained, ("row off with no rounding tie to explain it", b, tokens_gpu[b], tok_o[b], lq_err[b])
        lq_err[b] = 0.0
        stats["tie_rows"] += 1
    stats["logq_err"] = float(lq_err.max()) if B else 0.0
    return stats

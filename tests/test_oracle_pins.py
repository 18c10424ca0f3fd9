"""Pins for the fp64 CPU oracle: what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each check is chosen so that a
plausible mistake in the oracle (a dropped term, a wrong sign or index, a
transposed operand) fails at least one of them:

* eq. 3 / eq. 5: gate weights and every factor are normalised;
* eq. 2-5: the joint summed by brute force over all V^n tuples is 1;
* eq. 9: probability-space line equals the log-space line;
* eq. 1: r = 1 is a sum of independent softmax cross-entropies (library routine);
* mixture invariants: identical experts, expert permutation, Jensen;
* backward: central finite differences for every input, zero-sum invariants;
* sampling: chain of conditionals (eq. 11-13) multiplies to the joint, tuple
  frequencies follow the joint, boundary cases of the inverse CDF;
* the rounded-y mode that defines the draft calls (y -> bfloat16 before U y): every
  routine that takes it against a library composition with an independently written
  rounding, identity on representable y, and the hooks for rounding ties (exact y,
  zero nudge, a nudge across one midpoint = one ulp of one element).
"""
import itertools

import numpy as np
import pytest
import scipy.special as sps
import scipy.stats

from paper_2410_17765_amd import synth


def small_problem(T=6, d=12, V=9, n=3, r=4, seed=0, dtype=np.float64):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((T, d))
    W = rng.standard_normal((n, r, d, d)) / np.sqrt(d)
    U = rng.standard_normal((V, d)) * (1.5 / np.sqrt(d))
    G = rng.standard_normal((r, d)) / np.sqrt(d)
    X = rng.integers(0, V, size=(T, n)).astype(np.int32)
    return [a.astype(dtype) for a in (H, W, U, G)] + [X]


# ---------------------------------------------------------------------------
# normalisation (eq. 3, eq. 5) and the joint (eq. 2, eq. 4)
# ---------------------------------------------------------------------------

def test_gate_weights_normalised(oracle):
    H, W, U, G, X = small_problem()
    _, logw, _, _ = oracle.loss_fwd(H, W, U, G, X, details=True)
    w = np.exp(logw)
    assert (w >= 0).all()
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-15)


def test_factor_normalised(oracle):
    # With r = 1 the first conditional is the single factor P^(1)(. | a=1): eq. 5.
    H, W, U, G, X = small_problem(r=1)
    for t in range(H.shape[0]):
        p = oracle.sequential_conditional(H, W, U, G, t, [])
        assert (p >= 0).all()
        assert abs(p.sum() - 1.0) < 1e-12


def test_joint_sums_to_one_brute_force(oracle):
    # V = 8, n = 3: all 512 tuples for one hidden state.
    V, n, r, d = 8, 3, 2, 16
    rng = np.random.default_rng(11)
    h = rng.standard_normal(d)
    W = rng.standard_normal((n, r, d, d)) / np.sqrt(d)
    U = rng.standard_normal((V, d))
    G = rng.standard_normal((r, d))
    tuples = np.array(list(itertools.product(range(V), repeat=n)), dtype=np.int32)
    H = np.tile(h, (len(tuples), 1))
    loss = oracle.loss_fwd(H, W, U, G, tuples)
    assert abs(np.exp(-loss).sum() - 1.0) < 1e-12
    # the same on the seeded float32 inputs of the named configuration
    cfg = synth.CONFIGS["brute"]
    inp = synth.make_inputs(cfg)
    Hs = np.tile(inp["H"][3], (len(tuples), 1))
    loss = oracle.loss_fwd(Hs, inp["W"], inp["U"], inp["G"], tuples)
    assert abs(np.exp(-loss).sum() - 1.0) < 1e-12


def test_logspace_equals_probability_space(oracle):
    H, W, U, G, X = small_problem(seed=3)
    loss = oracle.loss_fwd(H, W, U, G, X)
    prob = oracle.joint_prob_naive(H, W, U, G, X)
    np.testing.assert_allclose(np.exp(-loss), prob, rtol=1e-12)


# ---------------------------------------------------------------------------
# reductions to library routines
# ---------------------------------------------------------------------------

def library_loss(H, W, U, G, X):
    """The same quantity composed from numpy/scipy routines (matmul, log_softmax, logsumexp)."""
    Y = np.einsum("sakj,tj->tsak", W, H)
    Z = np.einsum("vk,tsak->tsav", U, Y)
    logp = sps.log_softmax(Z, axis=-1)
    T, n = X.shape
    C = np.take_along_axis(logp, X[:, :, None, None].astype(np.int64), axis=-1)[..., 0]   # [T,n,r]
    logw = sps.log_softmax(H @ G.T, axis=-1)
    return -sps.logsumexp(logw + C.sum(axis=1), axis=-1)


def test_rank_one_is_independent_cross_entropies(oracle):
    # eq. 1: with r = 1 the joint is a product of n independent heads.
    H, W, U, G, X = small_problem(r=1, seed=5)
    loss = oracle.loss_fwd(H, W, U, G, X)
    ce = np.zeros(H.shape[0])
    for s in range(W.shape[0]):
        logits = (H @ W[s, 0].T) @ U.T
        ce -= np.take_along_axis(sps.log_softmax(logits, axis=1), X[:, s:s + 1].astype(np.int64), axis=1)[:, 0]
    np.testing.assert_allclose(loss, ce, rtol=1e-12, atol=1e-12)


def test_matches_library_composition(oracle):
    H, W, U, G, X = small_problem(seed=6)
    np.testing.assert_allclose(oracle.loss_fwd(H, W, U, G, X), library_loss(H, W, U, G, X), rtol=1e-12)


def test_float_and_double_entry_points_agree(oracle):
    H, W, U, G, X = small_problem(seed=8, dtype=np.float32)
    l32 = oracle.loss_fwd(H, W, U, G, X)
    l64 = oracle.loss_fwd(*(a.astype(np.float64) for a in (H, W, U, G)), X)
    np.testing.assert_array_equal(l32, l64)


# ---------------------------------------------------------------------------
# mixture invariants
# ---------------------------------------------------------------------------

def test_identical_experts_collapse_to_rank_one(oracle):
    H, W, U, G, X = small_problem(seed=9)
    Wsame = np.repeat(W[:, :1], W.shape[1], axis=1)
    l_mix = oracle.loss_fwd(H, Wsame, U, G, X)
    l_one = oracle.loss_fwd(H, W[:, :1].copy(), U, G[:1].copy(), X)
    np.testing.assert_allclose(l_mix, l_one, rtol=1e-12)


def test_expert_permutation(oracle):
    H, W, U, G, X = small_problem(seed=10)
    perm = np.array([2, 0, 3, 1])
    l0 = oracle.loss_fwd(H, W, U, G, X)
    l1 = oracle.loss_fwd(H, W[:, perm].copy(), U, G[perm].copy(), X)
    np.testing.assert_allclose(l0, l1, rtol=1e-13)
    g0 = oracle.loss_bwd(H, W, U, G, X)
    g1 = oracle.loss_bwd(H, W[:, perm].copy(), U, G[perm].copy(), X)
    np.testing.assert_allclose(g1["dW"], g0["dW"][:, perm], rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(g1["dG"], g0["dG"][perm], rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(g1["dU"], g0["dU"], rtol=1e-9, atol=1e-13)


def test_jensen_bound(oracle):
    H, W, U, G, X = small_problem(seed=12)
    loss, logw, C, _ = oracle.loss_fwd(H, W, U, G, X, details=True)
    lower = (np.exp(logw) * C.sum(axis=1)).sum(axis=1)
    assert (-loss >= lower - 1e-12).all()
    assert (C <= 1e-15).all()


def test_negative_target_drops_factor(oracle):
    H, W, U, G, X = small_problem(seed=13)
    Xd = X.copy()
    Xd[:, 2] = -1
    l_drop = oracle.loss_fwd(H, W, U, G, Xd)
    l_short = oracle.loss_fwd(H, W[:2].copy(), U, G, X[:, :2].copy())
    np.testing.assert_allclose(l_drop, l_short, rtol=1e-13)
    # the probability-space routine drops the same factors
    np.testing.assert_allclose(oracle.joint_prob_naive(H, W, U, G, Xd), np.exp(-l_short), rtol=1e-12)
    g_drop = oracle.loss_bwd(H, W, U, G, Xd)
    g_short = oracle.loss_bwd(H, W[:2].copy(), U, G, X[:, :2].copy())
    np.testing.assert_allclose(g_drop["dW"][:2], g_short["dW"], rtol=1e-9, atol=1e-14)
    assert np.all(g_drop["dW"][2] == 0)
    np.testing.assert_allclose(g_drop["dH"], g_short["dH"], rtol=1e-9, atol=1e-14)


def test_prescribed_init_statistics(oracle):
    # At the N(0,1/d) init each logit is ~N(0, |y|^2/d) so lse ~ log V + |y|^2/(2d).
    cfg = synth.HeadConfig("stat", T=4, d=256, V=32000, n=1, r=1, dtype="fp32", targets="uniform")
    inp = synth.make_inputs(cfg)
    _, _, _, lse = oracle.loss_fwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"], details=True)
    y = np.einsum("kj,tj->tk", inp["W"][0, 0].astype(np.float64), inp["H"].astype(np.float64))
    expect = np.log(cfg.V) + (y ** 2).sum(axis=1) / (2 * cfg.d)
    np.testing.assert_allclose(lse[:, 0, 0], expect, atol=0.1)


# ---------------------------------------------------------------------------
# backward
# ---------------------------------------------------------------------------

def _objective(oracle, H, W, U, G, X, dloss):
    return float((oracle.loss_fwd(H, W, U, G, X) * dloss).sum())


@pytest.mark.parametrize("which", ["H", "W", "U", "G"])
def test_gradients_match_central_differences(oracle, which):
    H, W, U, G, X = small_problem(T=5, d=10, V=13, n=2, r=3, seed=21)
    rng = np.random.default_rng(22)
    dloss = 0.5 + rng.random(H.shape[0])
    grads = oracle.loss_bwd(H, W, U, G, X, dloss)
    tensors = {"H": H, "W": W, "U": U, "G": G}
    base = tensors[which]
    g = grads["d" + which]
    assert g.shape == base.shape
    eps = 1e-6
    # every coordinate of the small tensors, a random sample of the large one
    flat = np.arange(base.size)
    if base.size > 400:
        flat = rng.choice(base.size, size=400, replace=False)
    for idx in flat:
        pert = base.copy().reshape(-1)
        pert[idx] += eps
        hi = _objective(oracle, *[pert.reshape(base.shape) if k == which else v for k, v in tensors.items()], X, dloss)
        pert[idx] -= 2 * eps
        lo = _objective(oracle, *[pert.reshape(base.shape) if k == which else v for k, v in tensors.items()], X, dloss)
        fd = (hi - lo) / (2 * eps)
        assert abs(fd - g.reshape(-1)[idx]) <= 1e-7 * max(1.0, abs(fd)), (which, idx, fd, g.reshape(-1)[idx])


def test_directional_derivative_tiny_config(oracle):
    # the seeded tiny configuration, all four tensors moved at once
    cfg = synth.CONFIGS["tiny"].with_(T=8)
    inp = {k: v.astype(np.float64) if k != "X" else v for k, v in synth.make_inputs(cfg).items()}
    rng = np.random.default_rng(31)
    dloss = synth.upstream_grad(cfg.T).astype(np.float64)
    grads = oracle.loss_bwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"], dloss)
    dirs = {k: rng.standard_normal(inp[k].shape) for k in "HWUG"}
    analytic = sum((grads["d" + k] * dirs[k]).sum() for k in "HWUG")
    eps = 1e-6
    f = lambda sgn: _objective(oracle, *[inp[k] + sgn * eps * dirs[k] for k in "HWUG"], inp["X"], dloss)
    fd = (f(+1) - f(-1)) / (2 * eps)
    assert abs(fd - analytic) <= 1e-7 * abs(fd)


def test_backward_zero_sum_invariants(oracle):
    H, W, U, G, X = small_problem(seed=23)
    g = oracle.loss_bwd(H, W, U, G, X)
    # sum_a dg_a = 0  =>  columns of dG sum to zero over experts
    np.testing.assert_allclose(g["dG"].sum(axis=0), 0.0, atol=1e-13)
    # sum_v dz_v = 0 for every row  =>  columns of dU sum to zero over the vocabulary
    np.testing.assert_allclose(g["dU"].sum(axis=0), 0.0, atol=1e-12)


def test_backward_linear_in_upstream(oracle):
    H, W, U, G, X = small_problem(seed=24)
    rng = np.random.default_rng(25)
    d1, d2 = rng.random(H.shape[0]), rng.random(H.shape[0])
    g1 = oracle.loss_bwd(H, W, U, G, X, d1)
    g2 = oracle.loss_bwd(H, W, U, G, X, d2)
    g12 = oracle.loss_bwd(H, W, U, G, X, d1 + 2 * d2)
    for k in g1:
        np.testing.assert_allclose(g12[k], g1[k] + 2 * g2[k], rtol=1e-9, atol=1e-13)
    gnone = oracle.loss_bwd(H, W, U, G, X, None)
    gones = oracle.loss_bwd(H, W, U, G, X, np.ones(H.shape[0]))
    for k in gnone:
        np.testing.assert_array_equal(gnone[k], gones[k])


# ---------------------------------------------------------------------------
# sampling
# ---------------------------------------------------------------------------

def test_chain_of_conditionals_is_the_joint(oracle):
    # eq. 11-13 (with the omitted factor and normaliser restored) multiply to eq. 2.
    V, n, r, d = 8, 3, 3, 10
    H, W, U, G, _ = small_problem(T=2, d=d, V=V, n=n, r=r, seed=41)
    tuples = np.array(list(itertools.product(range(V), repeat=n)), dtype=np.int32)
    for t in range(2):
        joint = np.exp(-oracle.loss_fwd(np.tile(H[t], (len(tuples), 1)), W, U, G, tuples))
        cond_cache = {}
        for i, tup in enumerate(tuples):
            p = 1.0
            for s in range(n):
                key = tuple(tup[:s])
                if key not in cond_cache:
                    c = oracle.sequential_conditional(H, W, U, G, t, list(key))
                    assert abs(c.sum() - 1.0) < 1e-12
                    cond_cache[key] = c
                p *= cond_cache[key][tup[s]]
            assert abs(p - joint[i]) <= 1e-12 * max(joint[i], 1e-30) + 1e-15


def test_first_token_marginal(oracle):
    # eq. 11: sum_a w_a P^(1)(x | a)
    H, W, U, G, X = small_problem(seed=42)
    _, logw, _, _ = oracle.loss_fwd(H, W, U, G, X, details=True)
    for t in range(2):
        p = oracle.sequential_conditional(H, W, U, G, t, [])
        ref = np.zeros_like(p)
        for a in range(W.shape[1]):
            ref += np.exp(logw[t, a]) * sps.softmax(U @ (W[0, a] @ H[t]))
        np.testing.assert_allclose(p, ref, rtol=1e-12)


def test_draft_frequencies_follow_the_joint(oracle):
    V, n, r, d = 4, 2, 3, 8
    H, W, U, G, _ = small_problem(T=1, d=d, V=V, n=n, r=r, seed=43)
    U = U * 2.0
    B = 40000
    u = synth.uniforms(B, n, seed=77)
    Hrep = np.tile(H[0], (B, 1))
    alpha, tokens, logq = oracle.draft_sample(Hrep, W, U, G, u, round_y=False)
    tuples = np.array(list(itertools.product(range(V), repeat=n)), dtype=np.int32)
    joint = np.exp(-oracle.loss_fwd(np.tile(H[0], (len(tuples), 1)), W, U, G, tuples))
    counts = np.zeros(len(tuples))
    for tok in tokens:
        counts[tok[0] * V + tok[1]] += 1
    chi2, p = scipy.stats.chisquare(counts, joint * B)
    assert p > 1e-3, (chi2, p)
    # expert frequencies follow w
    _, logw, _, _ = oracle.loss_fwd(H, W, U, G, np.zeros((1, n), np.int32), details=True)
    _, pa = scipy.stats.chisquare(np.bincount(alpha, minlength=r), np.exp(logw[0]) * B)
    assert pa > 1e-3
    # logq is eq. 9 at the drawn tuple
    lq = -oracle.loss_fwd(Hrep[:50], W, U, G, tokens[:50])
    np.testing.assert_allclose(logq[:50], lq, rtol=1e-12)


def test_draft_boundary_cases(oracle):
    H, W, U, G, _ = small_problem(T=3, seed=44)
    n, V, r = W.shape[0], U.shape[0], W.shape[1]
    u0 = np.zeros((3, 1 + n))
    a, tok, _ = oracle.draft_sample(H, W, U, G, u0, round_y=False)
    assert (a == 0).all() and (tok == 0).all()
    u1 = np.full((3, 1 + n), np.nextafter(1.0, 0.0))
    a, tok, _ = oracle.draft_sample(H, W, U, G, u1, round_y=False)
    assert (a == r - 1).all() and (tok == V - 1).all()
    # rank one: the expert is always 0
    a, _, _ = oracle.draft_sample(H, W[:, :1].copy(), U, G[:1].copy(), synth.uniforms(3, n), round_y=False)
    assert (a == 0).all()


def test_draft_cdf_and_forced_expert(oracle):
    H, W, U, G, _ = small_problem(T=4, seed=45)
    n = W.shape[0]
    u = synth.uniforms(4, n, seed=5)
    a, tok, logq, cdf_w, cdf_tok = oracle.draft_sample(H, W, U, G, u, round_y=False, want_cdf=True)
    assert (np.diff(cdf_w, axis=1) >= 0).all() and (np.diff(cdf_tok, axis=2) >= 0).all()
    np.testing.assert_allclose(cdf_w[:, -1], 1.0, atol=1e-14)
    np.testing.assert_allclose(cdf_tok[:, :, -1], 1.0, atol=1e-13)
    for b in range(4):
        assert cdf_w[b, a[b]] > u[b, 0] and (a[b] == 0 or cdf_w[b, a[b] - 1] <= u[b, 0])
        for s in range(n):
            v = tok[b, s]
            assert cdf_tok[b, s, v] > u[b, 1 + s] and (v == 0 or cdf_tok[b, s, v - 1] <= u[b, 1 + s])
            # the token distribution is the factor of the drawn expert (r = 1 conditional of that expert)
            p = oracle.sequential_conditional(H, W[s:s + 1, a[b]:a[b] + 1].copy(), U, G[:1].copy(), b, [])
            np.testing.assert_allclose(np.diff(cdf_tok[b, s], prepend=0.0), p, atol=1e-14)
    forced = (a + 1) % W.shape[1]
    a2, tok2, _ = oracle.draft_sample(H, W, U, G, u, round_y=False, alpha_in=forced)
    assert (a2 == forced).all()


def test_bf16_rounding_helper(oracle):
    rng = np.random.default_rng(46)
    vals = np.concatenate([rng.standard_normal(2000) * 3, [1.00390625, 1.01171875, -1.00390625, 0.0, 257.0, 258.0]])
    vals = vals.astype(np.float32)
    got = np.array([oracle.round_to_bf16(float(v)) for v in vals])
    np.testing.assert_array_equal(got, synth.bf16_round(vals).astype(np.float64))


def test_rounded_y_changes_loss_by_the_expected_amount(oracle):
    cfg = synth.HeadConfig("rnd", T=16, d=128, V=600, n=4, r=2, dtype="bf16", targets="uniform")
    inp = synth.make_inputs(cfg)
    l0 = oracle.loss_fwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"])
    l1 = oracle.loss_fwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"], round_y=True)
    diff = np.abs(l0 - l1)
    # bf16 rounding of y perturbs each target logit by about 2^-9 |z|: visible, but small
    assert 1e-5 < diff.max() < 3e-2


# ---------------------------------------------------------------------------
# the rounded-y mode (y -> bfloat16 before z = U y) and the hooks for rounding ties.
# The draft calls are defined with this rounding, so where it is applied is part of the definition:
# each routine that takes round_y is compared with a numpy/scipy composition that rounds W_sa h, and
# nothing else, with a rounding routine written independently of the oracle's (integer arithmetic on
# the fp64 bit pattern instead of frexp/nearbyint).
# ---------------------------------------------------------------------------

def bf16_nearest_even(x):
    """fp64 -> nearest value with 8 significant bits, ties to even, on the bit pattern: 45 of the 52
    fraction bits are dropped, a carry out of the fraction rightly bumps the exponent."""
    bits = np.ascontiguousarray(x, dtype=np.float64).view(np.uint64)
    drop = np.uint64(45)
    keep_lsb = (bits >> drop) & np.uint64(1)
    bits = ((bits + np.uint64((1 << 44) - 1) + keep_lsb) >> drop) << drop
    return bits.view(np.float64)


def composed_log_factors(H, W, U, G, round_y, y_override=None):
    """(logw[B,r], logP[B,n,r,V], y[B,n,r,d] before rounding) from library routines; the rounding, if any,
    is applied to y = W_sa h only.  y_override replaces the (rounded) y that enters U y."""
    logw = sps.log_softmax(H @ G.T, axis=-1)
    Y = np.einsum("sakj,bj->bsak", W, H)
    Yin = bf16_nearest_even(Y) if round_y else Y
    if y_override is not None:
        Yin = y_override
    Z = np.einsum("vk,bsak->bsav", U, Yin)
    return logw, sps.log_softmax(Z, axis=-1), Y


def rounding_problem(B=5, seed=61, **kw):
    H, W, U, G, _ = small_problem(T=B, seed=seed, **kw)
    return H, W, U * 3.0, G            # peaked enough that one bf16 ulp of y is far above 1e-12


def test_bit_pattern_rounding_agrees_with_the_oracles_helper(oracle):
    rng = np.random.default_rng(60)
    vals = np.concatenate([rng.standard_normal(3000) * np.exp(rng.uniform(-20, 20, 3000)),
                           [1.00390625, 1.01171875, 1.998046875, -1.998046875, 255.5, 0.0]])
    got = np.array([oracle.round_to_bf16(float(v)) for v in vals])
    np.testing.assert_array_equal(got, bf16_nearest_even(vals))
    # every result has 8 significant bits: it survives float32 -> bfloat16 truncation unchanged
    as_f32 = got.astype(np.float32)
    assert (as_f32.astype(np.float64) == got).all()
    assert ((as_f32.view(np.uint32) & 0xFFFF) == 0).all()


def test_rounded_y_loss_is_the_composition_with_y_rounded(oracle):
    H, W, U, G = rounding_problem(B=6)
    X = np.random.default_rng(62).integers(0, U.shape[0], size=(6, W.shape[0])).astype(np.int32)
    logw, logP, _ = composed_log_factors(H, W, U, G, True)
    C = np.take_along_axis(logP, X[:, :, None, None].astype(np.int64).repeat(W.shape[1], axis=2), axis=3)[..., 0]
    ref = -sps.logsumexp(logw + C.sum(axis=1), axis=-1)
    got = oracle.loss_fwd(H, W, U, G, X, round_y=True)
    np.testing.assert_allclose(got, ref, rtol=1e-12)
    # and the rounding matters at this size: the unrounded loss is measurably another number
    assert np.abs(got - oracle.loss_fwd(H, W, U, G, X)).max() > 1e-5
    for t in range(2):
        cond = oracle.sequential_conditional(H, W, U, G, t, [int(X[t, 0])], round_y=True)
        q = sps.softmax(logw[t] + logP[t, 0, :, X[t, 0]])
        np.testing.assert_allclose(cond, q @ np.exp(logP[t, 1]), rtol=1e-11)


def test_rounded_y_draft_is_the_composition_with_y_rounded(oracle):
    H, W, U, G = rounding_problem()
    B, n, r = H.shape[0], W.shape[0], W.shape[1]
    u = synth.uniforms(B, n, seed=63).astype(np.float64)
    logw, logP, Y = composed_log_factors(H, W, U, G, True)
    a, tok, logq, cdf_w, cdf_tok, y_exact = oracle.draft_sample(H, W, U, G, u, round_y=True, want_cdf=True, want_y=True)
    np.testing.assert_allclose(cdf_w, np.cumsum(np.exp(logw), axis=1), rtol=1e-12)
    np.testing.assert_allclose(y_exact, Y, rtol=1e-13, atol=1e-15)            # y before rounding, nothing added
    for b in range(B):
        assert a[b] == min(int(np.searchsorted(cdf_w[b], u[b, 0], side="right")), r - 1)
        for s in range(n):
            ref = np.cumsum(np.exp(logP[b, s, a[b]]))
            np.testing.assert_allclose(cdf_tok[b, s], ref, rtol=1e-12)
            assert tok[b, s] == min(int(np.searchsorted(cdf_tok[b, s], u[b, 1 + s], side="right")), U.shape[0] - 1)
        lq = sps.logsumexp(logw[b] + sum(logP[b, s, :, tok[b, s]] for s in range(n)))
        np.testing.assert_allclose(logq[b], lq, rtol=1e-12)
    # teeth: neither "no rounding" nor "rounding somewhere else" reproduces these running sums
    _, logP_plain, _ = composed_log_factors(H, W, U, G, False)
    assert max(np.abs(np.cumsum(np.exp(logP_plain[b, s, a[b]])) - cdf_tok[b, s]).max()
               for b in range(B) for s in range(n)) > 1e-6
    Zr = bf16_nearest_even(np.einsum("vk,bsak->bsav", U, Y))                   # rounding z instead of y
    logP_z = sps.log_softmax(Zr, axis=-1)
    assert max(np.abs(np.cumsum(np.exp(logP_z[b, s, a[b]])) - cdf_tok[b, s]).max()
               for b in range(B) for s in range(n)) > 1e-6


def test_rounded_y_first_token_and_sequential_are_the_composition(oracle):
    H, W, U, G = rounding_problem(seed=64)
    B, n, V = H.shape[0], W.shape[0], U.shape[0]
    logw, logP, _ = composed_log_factors(H, W, U, G, True)
    lp = oracle.first_token_logprob(H, W, U, G, round_y=True)
    np.testing.assert_allclose(lp, sps.logsumexp(logw[:, :, None] + logP[:, 0], axis=1), rtol=1e-12, atol=1e-13)
    assert np.abs(lp - oracle.first_token_logprob(H, W, U, G, round_y=False)).max() > 1e-6
    u = np.random.default_rng(65).random((B, n))
    tok, logq, cdf = oracle.draft_sample_sequential(H, W, U, G, u, round_y=True, want_cdf=True)
    for b in range(B):
        q = logw[b].copy()
        for s in range(n):
            ref = np.cumsum(sps.softmax(q) @ np.exp(logP[b, s]))
            np.testing.assert_allclose(cdf[b, s], ref, rtol=1e-11)
            assert tok[b, s] == min(int(np.searchsorted(cdf[b, s], u[b, s], side="right")), V - 1)
            q = q + logP[b, s, :, tok[b, s]]
        np.testing.assert_allclose(logq[b], sps.logsumexp(q), rtol=1e-12)


def test_rounding_is_the_identity_on_representable_y(oracle):
    # small integer W and h: every y is an integer below 256, exactly a bfloat16, so the rounded mode must
    # return the unrounded mode's results bit for bit (rounding anything else, e.g. z, would not)
    rng = np.random.default_rng(66)
    B, d, V, n, r = 4, 8, 11, 3, 3
    H = rng.integers(-2, 3, size=(B, d)).astype(np.float64)
    W = rng.integers(-1, 2, size=(n, r, d, d)).astype(np.float64)
    U = rng.standard_normal((V, d)) * 0.2
    G = rng.standard_normal((r, d)) * 0.3
    X = rng.integers(0, V, size=(B, n)).astype(np.int32)
    u = synth.uniforms(B, n, seed=67).astype(np.float64)
    assert np.abs(np.einsum("sakj,bj->bsak", W, H)).max() <= 256
    for x, y in zip(oracle.draft_sample(H, W, U, G, u, round_y=True, want_cdf=True),
                    oracle.draft_sample(H, W, U, G, u, round_y=False, want_cdf=True)):
        np.testing.assert_array_equal(x, y)
    np.testing.assert_array_equal(oracle.first_token_logprob(H, W, U, G, round_y=True),
                                  oracle.first_token_logprob(H, W, U, G, round_y=False))
    for x, y in zip(oracle.draft_sample_sequential(H, W, U, G, u[:, 1:], round_y=True, want_cdf=True),
                    oracle.draft_sample_sequential(H, W, U, G, u[:, 1:], round_y=False, want_cdf=True)):
        np.testing.assert_array_equal(x, y)
    np.testing.assert_array_equal(oracle.loss_fwd(H, W, U, G, X, round_y=True), oracle.loss_fwd(H, W, U, G, X))


def _nudge_across_midpoint(y):
    """For one exact value y: (nudge, other) with y + nudge just across the rounding midpoint on the side of
    the bfloat16 neighbour `other` that y does not round to."""
    near = float(bf16_nearest_even(np.array([y]))[0])
    ulp = 2.0 ** (np.floor(np.log2(abs(y))) - 7)
    other = near + ulp if y > near else near - ulp
    mid = 0.5 * (near + other)
    nudge = (mid - y) + np.sign(other - near) * 1e-3 * ulp
    assert float(bf16_nearest_even(np.array([y + nudge]))[0]) == other and abs(other - near) == ulp
    return nudge, other


def test_tie_hooks_of_the_draft_routines(oracle):
    """y_exact is the value before the nudge and before rounding; a zero nudge is the identity; a nudge that takes one
    element across its rounding midpoint moves exactly that element of the rounded y by one bfloat16 ulp."""
    H, W, U, G = rounding_problem(seed=68)
    B, n, r, d = H.shape[0], W.shape[0], W.shape[1], H.shape[1]
    u = synth.uniforms(B, n, seed=69).astype(np.float64)
    logw, logP, Y = composed_log_factors(H, W, U, G, True)
    forced = np.array([1, 0, 2, 1, 3], dtype=np.int32)[:B] % r
    base = oracle.draft_sample(H, W, U, G, u, round_y=True, alpha_in=forced, want_cdf=True, want_y=True)
    zero = oracle.draft_sample(H, W, U, G, u, round_y=True, alpha_in=forced, want_cdf=True, want_y=True,
                               y_nudge=np.zeros((B, n, r, d)))
    for x, y in zip(base, zero):
        np.testing.assert_array_equal(x, y)
    np.testing.assert_array_equal(oracle.first_token_logprob(H, W, U, G, round_y=True, y_nudge=np.zeros((B, r, d))),
                                  oracle.first_token_logprob(H, W, U, G, round_y=True))
    for x, y in zip(oracle.draft_sample_sequential(H, W, U, G, u[:, 1:], round_y=True, want_cdf=True,
                                                   y_nudge=np.zeros((B, n, r, d))),
                    oracle.draft_sample_sequential(H, W, U, G, u[:, 1:], round_y=True, want_cdf=True)):
        np.testing.assert_array_equal(x, y)

    b, s, k = 2, 1, 5
    a = int(forced[b])
    nudge, other = _nudge_across_midpoint(Y[b, s, a, k])
    nd = np.zeros((B, n, r, d))
    nd[b, s, a, k] = nudge
    Yr = bf16_nearest_even(Y)
    ulp = abs(other - Yr[b, s, a, k])
    Yr[b, s, a, k] = other
    _, logP2, _ = composed_log_factors(H, W, U, G, True, y_override=Yr)
    got = oracle.draft_sample(H, W, U, G, u, round_y=True, alpha_in=forced, want_cdf=True, want_y=True, y_nudge=nd)
    np.testing.assert_array_equal(got[5], base[5])                      # y_exact does not see the nudge
    np.testing.assert_allclose(got[5], Y, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(got[4][b, s], np.cumsum(np.exp(logP2[b, s, a])), rtol=1e-12)
    moved = np.abs(got[4][b, s] - base[4][b, s]).max()
    assert moved > 1e-9, "one ulp of one element must be visible in the running sums"
    # one ulp exactly: the running sums are those of the other neighbour, not of any value in between
    Yhalf = bf16_nearest_even(Y)
    Yhalf[b, s, a, k] += 0.5 * np.sign(other - Yhalf[b, s, a, k]) * ulp
    _, logPh, _ = composed_log_factors(H, W, U, G, True, y_override=Yhalf)
    assert np.abs(got[4][b, s] - np.cumsum(np.exp(logPh[b, s, a]))).max() > 0.2 * moved
    # nothing else moved: every other row's running sums are bit-identical
    mask = np.ones((B, n), bool)
    mask[b, s] = False
    np.testing.assert_array_equal(got[4][mask], base[4][mask])
    keep = np.arange(B) != b
    np.testing.assert_array_equal(got[2][keep], base[2][keep])
    lq = sps.logsumexp(logw[b] + sum(logP2[b, t, :, got[1][b, t]] for t in range(n)))
    np.testing.assert_allclose(got[2][b], lq, rtol=1e-12)

    # the same nudge through the other two routines
    tok, logq, cdf = oracle.draft_sample_sequential(H, W, U, G, u[:, 1:], round_y=True, want_cdf=True, y_nudge=nd)
    q = logw[b].copy()
    for t in range(n):
        np.testing.assert_allclose(cdf[b, t], np.cumsum(sps.softmax(q) @ np.exp(logP2[b, t])), rtol=1e-11)
        q = q + logP2[b, t, :, tok[b, t]]
    np.testing.assert_allclose(logq[b], sps.logsumexp(q), rtol=1e-12)
    nudge0, other0 = _nudge_across_midpoint(Y[b, 0, a, k])
    nd0 = np.zeros((B, r, d))
    nd0[b, a, k] = nudge0
    Yr0 = bf16_nearest_even(Y)
    Yr0[b, 0, a, k] = other0
    _, logP0, _ = composed_log_factors(H, W, U, G, True, y_override=Yr0)
    lp = oracle.first_token_logprob(H, W, U, G, round_y=True, y_nudge=nd0)
    np.testing.assert_allclose(lp, sps.logsumexp(logw[:, :, None] + logP0[:, 0], axis=1), rtol=1e-12, atol=1e-13)
    assert np.abs(lp[b] - oracle.first_token_logprob(H, W, U, G, round_y=True)[b]).max() > 1e-9


# ---------------------------------------------------------------------------
# next rows: first-token marginal, the paper's sequential scheme, eq. 10
# ---------------------------------------------------------------------------

def test_first_token_logprob(oracle):
    # eq. 11 in log space: a distribution over V, equal to the s = 0 conditional and to the library composition
    H, W, U, G, X = small_problem(seed=51)
    lp = oracle.first_token_logprob(H, W, U, G)
    np.testing.assert_allclose(np.exp(lp).sum(axis=1), 1.0, atol=1e-12)
    for t in range(H.shape[0]):
        np.testing.assert_allclose(np.exp(lp[t]), oracle.sequential_conditional(H, W, U, G, t, []), rtol=1e-12)
    logw = sps.log_softmax(H @ G.T, axis=-1)
    Z = np.einsum("vk,tak->tav", U, np.einsum("akj,tj->tak", W[0], H))
    ref = sps.logsumexp(logw[:, :, None] + sps.log_softmax(Z, axis=-1), axis=1)
    np.testing.assert_allclose(lp, ref, rtol=1e-12, atol=1e-12)


def test_sequential_scheme_uses_the_pinned_conditionals(oracle):
    H, W, U, G, _ = small_problem(T=3, seed=52)
    n = W.shape[0]
    rng = np.random.default_rng(53)
    u = rng.random((3, n))
    tokens, logq, cdf = oracle.draft_sample_sequential(H, W, U, G, u, round_y=False, want_cdf=True)
    for t in range(3):
        for s in range(n):
            cond = oracle.sequential_conditional(H, W, U, G, t, list(tokens[t, :s]))
            np.testing.assert_allclose(np.diff(cdf[t, s], prepend=0.0), cond, atol=1e-13)
            v = tokens[t, s]
            assert cdf[t, s, v] > u[t, s] and (v == 0 or cdf[t, s, v - 1] <= u[t, s])
    # the accumulated expert log-weights end as the joint log-probability of the drawn tuple (eq. 9)
    np.testing.assert_allclose(logq, -oracle.loss_fwd(H, W, U, G, tokens), rtol=1e-12)


def test_sequential_scheme_samples_the_joint(oracle):
    V, n, r, d = 4, 2, 3, 8
    H, W, U, G, _ = small_problem(T=1, d=d, V=V, n=n, r=r, seed=43)
    U = U * 2.0
    B = 40000
    rng = np.random.Generator(np.random.Philox(78))
    u = rng.random((B, n))
    tokens, _ = oracle.draft_sample_sequential(np.tile(H[0], (B, 1)), W, U, G, u, round_y=False)
    tuples = np.array(list(itertools.product(range(V), repeat=n)), dtype=np.int32)
    joint = np.exp(-oracle.loss_fwd(np.tile(H[0], (len(tuples), 1)), W, U, G, tuples))
    counts = np.bincount(tokens[:, 0] * V + tokens[:, 1], minlength=V * V)
    _, p = scipy.stats.chisquare(counts, joint * B)
    assert p > 1e-3
    # boundaries of the inverse CDF
    t0, _ = oracle.draft_sample_sequential(H, W, U, G, np.zeros((1, n)), round_y=False)
    t1, _ = oracle.draft_sample_sequential(H, W, U, G, np.full((1, n), np.nextafter(1.0, 0.0)), round_y=False)
    assert (t0 == 0).all() and (t1 == V - 1).all()


def test_aux_balance(oracle):
    # eq. 10 on hand-built gates: G = 5 I picks the largest coordinate of h
    r, d = 4, 4
    G = 5.0 * np.eye(r, d)
    H = np.array([[3, 0, 0, 0], [0, 2, 0, 0], [0, 0, 1, 0], [0, 0, 0, 4], [9, 1, 0, 0], [1, 1, 0, 0]], dtype=np.float64)
    counts, laux = oracle.aux_balance(H, G)
    assert counts.tolist() == [3, 1, 1, 1]          # the tie in the last row goes to the first index
    np.testing.assert_allclose(laux, (3 / 6 - 0.25) ** 2 + 3 * (1 / 6 - 0.25) ** 2, rtol=1e-14)
    # perfectly balanced use gives zero, a single expert gives (1 - 1/r)^2 + (r - 1)/r^2
    counts, laux = oracle.aux_balance(np.eye(4), G)
    assert counts.tolist() == [1, 1, 1, 1] and laux == 0.0
    counts, laux = oracle.aux_balance(np.tile([1.0, 0, 0, 0], (7, 1)), G)
    assert counts.tolist() == [7, 0, 0, 0]
    np.testing.assert_allclose(laux, (1 - 1 / r) ** 2 + (r - 1) / r ** 2, rtol=1e-14)
    # against the gate weights of the forward pass
    Hs, W, U, Gs, X = small_problem(T=40, seed=54)
    counts, _ = oracle.aux_balance(Hs, Gs)
    _, logw, _, _ = oracle.loss_fwd(Hs, W, U, Gs, X, details=True)
    assert counts.tolist() == np.bincount(np.argmax(logw, axis=1), minlength=Gs.shape[0]).tolist()


# ---------------------------------------------------------------------------
# full heads (eq. 6 as printed): one V x d matrix per (s, a)
# ---------------------------------------------------------------------------

def full_problem(T=5, d=7, V=6, n=2, r=3, seed=5):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((T, d))
    F = rng.standard_normal((n, r, V, d)) * (1.2 / np.sqrt(d))
    G = rng.standard_normal((r, d)) / np.sqrt(d)
    X = rng.integers(0, V, size=(T, n)).astype(np.int32)
    return H, F, G, X


def test_full_heads_reduce_to_the_shared_unembedding_head(oracle):
    # F_sa = U W_sa is the reduced head of "Fine tuning": both routines must agree, and the chain rule
    # ties the gradients together: dW_sa = U^T dF_sa, dU = sum_sa dF_sa W_sa^T.
    H, W, U, G, X = small_problem()
    F = np.einsum("vk,sakj->savj", U, W)
    X[1, 2] = -1
    np.testing.assert_allclose(oracle.full_loss_fwd(H, F, G, X), oracle.loss_fwd(H, W, U, G, X), rtol=1e-12)
    dl = np.random.default_rng(2).standard_normal(H.shape[0])
    gf = oracle.full_loss_bwd(H, F, G, X, dl)
    gr = oracle.loss_bwd(H, W, U, G, X, dl)
    np.testing.assert_allclose(gf["dH"], gr["dH"], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(gf["dG"], gr["dG"], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(np.einsum("vk,savj->sakj", U, gf["dF"]), gr["dW"], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(np.einsum("savj,sakj->vk", gf["dF"], W), gr["dU"], rtol=1e-10, atol=1e-13)


def test_full_heads_rank_one_single_token_is_softmax_cross_entropy(oracle):
    H, F, G, X = full_problem(n=1, r=1)
    ref = -np.array([sps.log_softmax(F[0, 0] @ H[t])[X[t, 0]] for t in range(H.shape[0])])
    np.testing.assert_allclose(oracle.full_loss_fwd(H, F, G, X), ref, rtol=1e-12)


def test_full_heads_joint_sums_to_one(oracle):
    H, F, G, _ = full_problem(T=1, V=5, n=3, r=2)
    tuples = np.array(list(itertools.product(range(5), repeat=3)), dtype=np.int32)
    loss = oracle.full_loss_fwd(np.tile(H, (len(tuples), 1)), F, G, tuples)
    assert abs(np.exp(-loss).sum() - 1.0) < 1e-12


@pytest.mark.parametrize("which", ["H", "F", "G"])
def test_full_heads_gradients_match_central_differences(oracle, which):
    H, F, G, X = full_problem()
    X[0, 1] = -1
    dl = np.random.default_rng(3).standard_normal(H.shape[0])
    grads = oracle.full_loss_bwd(H, F, G, X, dl)
    args = {"H": H, "F": F, "G": G}
    rng = np.random.default_rng(4)
    eps = 1e-6
    for _ in range(12):
        idx = tuple(rng.integers(0, s) for s in args[which].shape)
        vals = []
        for sign in (+1, -1):
            pert = {k: v.copy() for k, v in args.items()}
            pert[which][idx] += sign * eps
            vals.append(float(dl @ oracle.full_loss_fwd(pert["H"], pert["F"], pert["G"], X)))
        fd = (vals[0] - vals[1]) / (2 * eps)
        np.testing.assert_allclose(grads["d" + which][idx], fd, rtol=2e-6, atol=2e-9)


def test_full_heads_invariants(oracle):
    H, F, G, X = full_problem()
    X[:, 1] = -1                                     # the second factor is dropped everywhere
    g = oracle.full_loss_bwd(H, F, G, X)
    assert np.abs(g["dF"][1]).max() == 0.0
    np.testing.assert_allclose(g["dF"][0].sum(axis=1), 0.0, atol=1e-13)      # sum_v dz_v = 0
    np.testing.assert_allclose(g["dG"].sum(axis=0), 0.0, atol=1e-13)         # sum_a dg_a = 0


# ---------------------------------------------------------------------------
# head-only fine-tuning loss ("Fine tuning", eq. 14): beta * KL + (1 - beta) * CE per token, discounted
# ---------------------------------------------------------------------------

def distill_problem(T=4, d=6, V=7, n=3, r=3, seed=21):
    H, W, U, G, X = small_problem(T=T, d=d, V=V, n=n, r=r, seed=seed)
    TZ = np.random.default_rng(seed + 1).standard_normal((T, n, V)) * 1.5
    return H, W, U, G, X, TZ


def test_distill_without_teacher_term_is_the_joint_likelihood(oracle):
    # beta = 0, no discount: the per-token cross-entropies are the chain of conditionals of the joint
    H, W, U, G, X, TZ = distill_problem()
    np.testing.assert_allclose(oracle.distill_loss_fwd(H, W, U, G, X, TZ, beta=0.0, disc=1.0),
                               oracle.loss_fwd(H, W, U, G, X), rtol=1e-12)
    dl = np.random.default_rng(5).standard_normal(H.shape[0])
    gd = oracle.distill_loss_bwd(H, W, U, G, X, TZ, beta=0.0, disc=1.0, dloss=dl)
    gr = oracle.loss_bwd(H, W, U, G, X, dl)
    for k in gr:
        np.testing.assert_allclose(gd[k], gr[k], rtol=1e-9, atol=1e-12, err_msg=k)


def test_distill_terms_against_library_routines(oracle):
    # each token's terms from the pinned conditional P(x_k | x_<k) and scipy's relative entropy
    H, W, U, G, X, TZ = distill_problem()
    beta, disc = 0.9, 0.7
    loss, kl, ce = oracle.distill_loss_fwd(H, W, U, G, X, TZ, beta=beta, disc=disc, details=True)
    for t in range(H.shape[0]):
        tot = 0.0
        for k in range(X.shape[1]):
            cond = oracle.sequential_conditional(H, W, U, G, t, list(X[t, :k]))
            pc = sps.softmax(TZ[t, k])
            np.testing.assert_allclose(kl[t, k], sps.rel_entr(pc, cond).sum(), rtol=1e-10)
            np.testing.assert_allclose(ce[t, k], -np.log(cond[X[t, k]]), rtol=1e-10)
            tot += disc ** k * (beta * kl[t, k] + (1 - beta) * ce[t, k])
        np.testing.assert_allclose(loss[t], tot, rtol=1e-12)
    assert (kl >= -1e-14).all()                                  # Gibbs


def test_distill_teacher_equal_to_student_has_zero_divergence(oracle):
    H, W, U, G, X, TZ = distill_problem(T=2)
    for t in range(2):
        for k in range(X.shape[1]):
            TZ[t, k] = np.log(oracle.sequential_conditional(H, W, U, G, t, list(X[t, :k]))) + 3.0   # any shift
    _, kl, _ = oracle.distill_loss_fwd(H, W, U, G, X, TZ, details=True)
    assert np.abs(kl).max() < 1e-13
    # ... and there the divergence is stationary: the gradient is that of the cross-entropy part alone
    g1 = oracle.distill_loss_bwd(H, W, U, G, X, TZ, beta=0.9, disc=1.0)
    g0 = oracle.distill_loss_bwd(H, W, U, G, X, TZ, beta=0.0, disc=1.0)
    for k in g0:
        np.testing.assert_allclose(g1[k], 0.1 * g0[k], rtol=1e-8, atol=1e-12, err_msg=k)


def test_distill_rank_one_single_token_is_textbook_distillation(oracle):
    H, W, U, G, X, TZ = distill_problem(n=1, r=1)
    beta = 0.6
    ref = []
    for t in range(H.shape[0]):
        logp = sps.log_softmax(U @ (W[0, 0] @ H[t]))
        pc = sps.softmax(TZ[t, 0])
        ref.append(beta * sps.rel_entr(pc, np.exp(logp)).sum() - (1 - beta) * logp[X[t, 0]])
    np.testing.assert_allclose(oracle.distill_loss_fwd(H, W, U, G, X, TZ, beta=beta), ref, rtol=1e-12)


@pytest.mark.parametrize("which", ["H", "W", "U", "G"])
def test_distill_gradients_match_central_differences(oracle, which):
    H, W, U, G, X, TZ = distill_problem()
    X[1, 1] = -1                                                 # a dropped token in the middle of a row
    beta, disc = 0.9, 0.8
    dl = np.random.default_rng(8).standard_normal(H.shape[0])
    grads = oracle.distill_loss_bwd(H, W, U, G, X, TZ, beta=beta, disc=disc, dloss=dl)
    args = {"H": H, "W": W, "U": U, "G": G}
    rng = np.random.default_rng(9)
    eps = 1e-6
    for _ in range(14):
        idx = tuple(rng.integers(0, s) for s in args[which].shape)
        vals = []
        for sign in (+1, -1):
            pert = {k: v.copy() for k, v in args.items()}
            pert[which][idx] += sign * eps
            vals.append(float(dl @ oracle.distill_loss_fwd(pert["H"], pert["W"], pert["U"], pert["G"], X, TZ,
                                                           beta=beta, disc=disc)))
        fd = (vals[0] - vals[1]) / (2 * eps)
        np.testing.assert_allclose(grads["d" + which][idx], fd, rtol=5e-6, atol=5e-9)


def test_distill_dropped_token(oracle):
    H, W, U, G, X, TZ = distill_problem()
    X[:, 2] = -1
    loss, kl, ce = oracle.distill_loss_fwd(H, W, U, G, X, TZ, details=True)
    assert np.abs(kl[:, 2]).max() == 0.0 and np.abs(ce[:, 2]).max() == 0.0
    g = oracle.distill_loss_bwd(H, W, U, G, X, TZ)
    assert np.abs(g["dW"][2]).max() == 0.0                        # the third head never enters
    # same as a two-token head
    np.testing.assert_allclose(loss, oracle.distill_loss_fwd(H, W[:2].copy(), U, G, X[:, :2].copy(), TZ[:, :2].copy()),
                               rtol=1e-12)


# ---------------------------------------------------------------------------
# stored reference values (written by tests/golden/make_golden.py from the oracle alone)
# ---------------------------------------------------------------------------

def read_golden():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_reference.txt")
    vals = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        vals[" ".join(parts[:-1])] = float(parts[-1])
    return vals


def test_oracle_reproduces_the_stored_tiny_workload(oracle):
    vals = read_golden()
    cfg = synth.CONFIGS["tiny"]
    inp = synth.make_inputs(cfg)
    args = (inp["H"], inp["W"], inp["U"], inp["G"], inp["X"])
    loss = oracle.loss_fwd(*args)
    for t in range(8):
        np.testing.assert_allclose(loss[t], vals[f"loss {t}"], rtol=1e-13)
    np.testing.assert_allclose(loss.mean(), vals["mean_loss"], rtol=1e-13)
    # at the prescribed initialisation the loss sits near n log V (checked as a closed form elsewhere)
    assert abs(vals["mean_loss"] - cfg.n * np.log(cfg.V)) < 0.6
    g = oracle.loss_bwd(*args, np.full(cfg.T, 1.0 / cfg.T))
    for k in ("dH", "dW", "dU", "dG"):
        np.testing.assert_allclose(np.linalg.norm(g[k].ravel()), vals[f"norm_{k}"], rtol=1e-11)


def test_zero_weights_closed_form(oracle):
    # all logits zero: every factor is uniform, every expert equal, so loss = n log V exactly
    H, W, U, G, X = small_problem()
    loss = oracle.loss_fwd(H, np.zeros_like(W), U, G, X)
    np.testing.assert_allclose(loss, X.shape[1] * np.log(U.shape[0]), rtol=1e-14)
    loss = oracle.loss_fwd(H, W, np.zeros_like(U), G, X)
    np.testing.assert_allclose(loss, X.shape[1] * np.log(U.shape[0]), rtol=1e-14)

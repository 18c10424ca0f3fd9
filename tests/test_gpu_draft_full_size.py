"""The draft step at its full benchmark size (d=4096, V=128256, n=4, r=8; B in {1, 8, 64}) against
the fp64 oracle.  The draw of a row depends on that row only, so for B = 64 the oracle is run on a
sample of rows.  At the prescribed near-uniform init the CDF steps (about 8e-6) are as narrow as the
1e-5 band the specification grants, so every draw is checked for band validity (none exempt) and the
exact-match rate is reported; the peaked variant (U scaled by 8) has steps far wider than the band."""
import numpy as np
import pytest

from paper_2410_17765_amd import synth
from tests.helpers import LOSS_ATOL, check_draft, check_sequential

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", params=[1.0, 8.0], ids=["prescribed_init", "peaked"])
def setup(request):
    import torch
    from paper_2410_17765_amd import head
    cfg = synth.CONFIGS["draft"].with_(T=64, u_scale=request.param)
    print(f"[draft] generating {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    h = head.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype)
    yield cfg, inp, h, head, torch
    del h
    torch.cuda.empty_cache()


@pytest.mark.parametrize("B,rows", [(1, 1), (8, 4), (64, 4)])
def test_draft_step(oracle, setup, B, rows):
    cfg, inp, h, head, torch = setup
    H = inp["H"][:B]
    u = synth.uniforms(B, cfg.n, seed=synth.SEED_UNIFORMS + B)
    print(f"[draft] GPU step B={B} u_scale={cfg.u_scale}", flush=True)
    alpha, tokens, logq = h.draft_sample(head.to_device(H, cfg.dtype), torch.from_numpy(u).cuda())
    torch.cuda.synchronize()
    alpha, tokens, logq = alpha.cpu().numpy(), tokens.cpu().numpy(), logq.cpu().numpy()
    assert ((0 <= alpha) & (alpha < cfg.r)).all() and ((0 <= tokens) & (tokens < cfg.V)).all()
    sel = np.sort(np.random.default_rng(B).choice(B, size=rows, replace=False))
    print(f"[draft] oracle on rows {sel.tolist()}", flush=True)
    stats = check_draft(oracle, H[sel], inp["W"], inp["U"], inp["G"], u[sel], alpha[sel], tokens[sel], logq[sel],
                        round_y=True, logq_atol=2e-3)
    print(f"  {stats}", flush=True)
    if cfg.u_scale > 1.0:
        assert stats["tokens_exact"] == stats["tokens_total"] and stats["alpha_exact"] == stats["alpha_total"]
    else:
        assert stats["alpha_exact"] == stats["alpha_total"]
        assert stats["tokens_exact"] >= 0.75 * stats["tokens_total"]


@pytest.mark.parametrize("B,rows", [(1, 1), (64, 2)])
def test_sequential_step(oracle, setup, B, rows):
    """The paper-form sampler (eq. 11-13) at the same size: one uniform per token."""
    cfg, inp, h, head, torch = setup
    H = inp["H"][:B]
    u = np.ascontiguousarray(synth.uniforms(B, cfg.n, seed=synth.SEED_UNIFORMS + 100 + B)[:, 1:])
    print(f"[draft] sequential GPU step B={B} u_scale={cfg.u_scale}", flush=True)
    tokens, logq = h.draft_sample_sequential(head.to_device(H, cfg.dtype), torch.from_numpy(u).cuda())
    torch.cuda.synchronize()
    tokens, logq = tokens.cpu().numpy(), logq.cpu().numpy()
    assert ((0 <= tokens) & (tokens < cfg.V)).all()
    sel = np.sort(np.random.default_rng(B).choice(B, size=rows, replace=False))
    print(f"[draft] oracle on rows {sel.tolist()}", flush=True)
    stats = check_sequential(oracle, H[sel], inp["W"], inp["U"], inp["G"], u[sel], tokens[sel], logq[sel],
                             logq_atol=2e-3)
    print(f"  {stats}", flush=True)
    if cfg.u_scale > 1.0:
        assert stats["tokens_exact"] >= stats["tokens_total"] - cfg.n * stats["tie_rows"]


def test_first_token_marginal(oracle, setup):
    """log of eq. 11 over the whole vocabulary for B = 8 rows, two of them against the oracle."""
    cfg, inp, h, head, torch = setup
    B = 8
    logp = h.first_token_logprob(head.to_device(inp["H"][:B], cfg.dtype))
    torch.cuda.synchronize()
    assert float(torch.logsumexp(logp.double(), dim=1).abs().max()) <= 1e-4
    sel = [2, 7]
    print(f"[draft] oracle first-token marginal on rows {sel}", flush=True)
    ref = oracle.first_token_logprob(inp["H"][sel], inp["W"], inp["U"], inp["G"], round_y=True)
    diff = np.abs(logp.cpu().numpy()[sel].astype(np.float64) - ref)
    err, mean_err = diff.max(), (np.exp(ref) * diff).sum(axis=1).max()
    print(f"  max |dlogp| {err:.3e}, expected |dlogp| under the marginal itself {mean_err:.3e}", flush=True)
    # Prescribed initialisation: every one of the V entries within the loss tolerance.  In the peaked
    # variant every logit, and with it every absolute error, is 8 times larger (fp32 accumulation makes
    # a few of the 32768 elements of y round to the other bf16 neighbour than the exact value does, and each
    # such element moves a logit by one ulp of y times an entry of U): the far tail (log p near -60) is
    # held to the scaled bound, the error a token drawn from the marginal sees to the unscaled one.
    assert err <= LOSS_ATOL * cfg.u_scale
    assert mean_err <= LOSS_ATOL

"""The draft step at its full benchmark size (d=4096, V=128256, n=4, r=8; B in {1, 8, 64}) against
the fp64 oracle.  The draw of a row depends on that row only, so for B = 64 the oracle is run on a
sample of rows.  At the prescribed near-uniform init the CDF steps (about 8e-6) are as narrow as the
1e-5 band the specification grants, so every draw is checked for band validity (none exempt) and the
exact-match rate is reported; the peaked variant (U scaled by 8) has steps far wider than the band."""
import numpy as np
import pytest

from paper_2410_17765_amd import synth
from tests.helpers import check_draft

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

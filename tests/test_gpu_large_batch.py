"""Beyond the benchmark sizes: four times the headline batch (T = 65536, 2.1 M head rows, 6.7e10 logits per
pass), where row offsets, statistics buffers and operand sizes all pass 2^32 bytes.  The oracle checks
sampled positions (the last one among them); the weight gradients are tied to the headline-size calls, which
the oracle checks elsewhere, by summing the gradients of the four quarters of the batch."""
import numpy as np
import pytest

from paper_2410_17765_amd import synth
from tests.helpers import GRAD_REL_FRO, LOSS_ATOL, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def big():
    import gc
    import torch
    from paper_2410_17765_amd import head
    cfg = synth.CONFIGS["head_7b"].with_(name="head_7b_x4", T=4 * synth.CONFIGS["head_7b"].T)
    print(f"[large batch] generating {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    h = head.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype)
    H = head.to_device(inp["H"], cfg.dtype)
    X = torch.from_numpy(inp["X"]).cuda()
    scale = 1.0 / cfg.T
    print("[large batch] running on the GPU", flush=True)
    loss = h.loss_fwd(H, X)
    grads = h.loss_bwd(H, X, None, scale=scale)
    torch.cuda.synchronize()
    yield dict(cfg=cfg, inp=inp, h=h, H=H, X=X, scale=scale, loss=loss, grads=grads, torch=torch)
    del h, H, X, loss, grads
    gc.collect()
    torch.cuda.empty_cache()


def test_sampled_positions(oracle, big):
    cfg, inp, torch = big["cfg"], big["inp"], big["torch"]
    sel = np.array([0, cfg.T // 2 + 12345, cfg.T - 257, cfg.T - 1])
    print(f"[large batch] oracle forward on positions {sel.tolist()}", flush=True)
    ref = oracle.loss_fwd(inp["H"][sel], inp["W"], inp["U"], inp["G"], inp["X"][sel])
    err = np.abs(big["loss"].cpu().numpy()[sel] - ref).max()
    print(f"  loss max abs err {err:.3e} (mean loss {ref.mean():.3f})", flush=True)
    assert bool(torch.isfinite(big["loss"]).all()) and err <= LOSS_ATOL
    two = sel[[1, 3]]
    print(f"[large batch] oracle backward on positions {two.tolist()}", flush=True)
    rg = oracle.loss_bwd(inp["H"][two], inp["W"], inp["U"], inp["G"], inp["X"][two], np.full(2, big["scale"]))
    got = big["grads"]["dH"][torch.from_numpy(two).cuda()].cpu().numpy()
    e = rel_fro(got, rg["dH"])
    print(f"  dH rows rel fro {e:.3e}", flush=True)
    assert e <= GRAD_REL_FRO


def test_batch_gradients_are_the_sum_over_quarters(big):
    cfg, torch, h, g = big["cfg"], big["torch"], big["h"], big["grads"]
    q = cfg.T // 4
    tot = None
    for i in range(4):
        Hq, Xq = big["H"][i * q:(i + 1) * q].contiguous(), big["X"][i * q:(i + 1) * q].contiguous()
        lq = h.loss_fwd(Hq, Xq)
        gq = h.loss_bwd(Hq, Xq, None, scale=big["scale"])
        torch.cuda.synchronize()
        assert float((lq - big["loss"][i * q:(i + 1) * q]).abs().max()) <= 1e-4
        rel = float((gq["dH"] - g["dH"][i * q:(i + 1) * q]).double().norm() / gq["dH"].double().norm())
        assert rel <= 2e-3, ("dH", i, rel)
        if tot is None:
            tot = {k: gq[k].clone() for k in ("dW", "dU", "dG")}
        else:
            for k in tot:
                tot[k] += gq[k]
    for k in tot:
        rel = float((tot[k] - g[k]).double().norm() / g[k].double().norm())
        print(f"  {k}: |full - sum of quarters| / |full| = {rel:.3e}", flush=True)
        assert rel <= 2e-3, k

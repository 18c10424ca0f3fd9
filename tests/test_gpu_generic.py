"""GPU parity of the plain fp32 path (any shape, fp32 or bf16 storage) against the fp64 oracle,
element by element on the same seeded inputs.  All calls go through the C ABI."""
import itertools

import numpy as np
import pytest

from paper_2410_17765_amd import synth
from tests.helpers import GRAD_REL_FRO, LOSS_ATOL, check_draft, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2410_17765_amd import binding, head
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    return head


def run_loss(head, cfg, inp, dloss=None, flags=0, want_bwd=True):
    import torch
    h = head.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype, flags=flags)
    H = head.to_device(inp["H"], cfg.dtype)
    X = torch.from_numpy(inp["X"]).cuda()
    loss = h.loss_fwd(H, X)
    grads = None
    if want_bwd:
        dl = None if dloss is None else torch.from_numpy(dloss).cuda()
        grads = {k: v.cpu().numpy() for k, v in h.loss_bwd(H, X, dl).items()}
    torch.cuda.synchronize()
    return loss.cpu().numpy(), grads


CASES = [
    synth.CONFIGS["tiny"],
    synth.HeadConfig("ragged_fp32", T=37, d=50, V=301, n=3, r=3, dtype="fp32", targets="zipf"),
    synth.HeadConfig("ragged_bf16", T=45, d=72, V=515, n=2, r=5, dtype="bf16", targets="zipf"),
    synth.HeadConfig("rank_one", T=16, d=32, V=100, n=4, r=1, dtype="fp32", targets="uniform"),
    synth.HeadConfig("one_of_each", T=1, d=1, V=1, n=1, r=1, dtype="fp32", targets="uniform"),
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_loss_and_gradients(gpu, oracle, cfg):
    print(f"case {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    dloss = synth.upstream_grad(cfg.T)
    loss, grads = run_loss(gpu, cfg, inp, dloss, flags=1)
    ref = oracle.loss_fwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"])
    assert np.abs(loss - ref).max() <= LOSS_ATOL
    assert np.abs(loss - ref).max() <= 1e-4 * max(1.0, np.abs(ref).max())     # fp32 path: far inside the bound
    gref = oracle.loss_bwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"], dloss)
    for k, v in gref.items():
        if np.linalg.norm(v) == 0:
            assert np.abs(grads[k]).max() <= 1e-6, k
        else:
            assert rel_fro(grads[k], v) <= min(GRAD_REL_FRO, 1e-4), (k, rel_fro(grads[k], v))


def test_joint_sums_to_one_on_gpu(gpu, oracle):
    cfg = synth.CONFIGS["brute"]
    inp = synth.make_inputs(cfg)
    tuples = np.array(list(itertools.product(range(cfg.V), repeat=cfg.n)), dtype=np.int32)
    inp["H"] = np.tile(inp["H"][3], (len(tuples), 1))
    inp["X"] = tuples
    loss, _ = run_loss(gpu, cfg, inp, want_bwd=False)
    assert abs(np.exp(-loss.astype(np.float64)).sum() - 1.0) < 1e-5
    ref = oracle.loss_fwd(inp["H"], inp["W"], inp["U"], inp["G"], tuples)
    assert np.abs(loss - ref).max() <= 1e-5


def test_negative_targets_and_default_upstream(gpu, oracle):
    cfg = synth.HeadConfig("drop", T=20, d=24, V=64, n=3, r=2, dtype="fp32", targets="uniform")
    inp = synth.make_inputs(cfg)
    inp["X"][::3, 1] = -1
    loss, grads = run_loss(gpu, cfg, inp, None)
    ref = oracle.loss_fwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"])
    assert np.abs(loss - ref).max() <= 1e-5
    gref = oracle.loss_bwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"], None)
    for k, v in gref.items():
        assert rel_fro(grads[k], v) <= 1e-4, k


def test_empty_batch(gpu):
    import torch
    cfg = synth.HeadConfig("empty", T=0, d=8, V=16, n=2, r=2, dtype="fp32", targets="uniform")
    full = synth.make_inputs(cfg.with_(T=1))
    h = gpu.CpHead(full["W"], full["U"], full["G"], dtype="fp32")
    H = torch.empty((0, cfg.d), device="cuda")
    X = torch.empty((0, cfg.n), dtype=torch.int32, device="cuda")
    loss = h.loss_fwd(H, X)
    g = h.loss_bwd(H, X)
    torch.cuda.synchronize()
    assert loss.numel() == 0
    for k in ("dW", "dU", "dG"):
        assert float(g[k].abs().max()) == 0.0


@pytest.mark.parametrize("cfg", [
    synth.HeadConfig("draft_fp32", T=9, d=40, V=333, n=3, r=4, dtype="fp32", targets="uniform", u_scale=3.0),
    synth.HeadConfig("draft_bf16", T=7, d=64, V=700, n=4, r=8, dtype="bf16", targets="uniform", u_scale=4.0),
    synth.HeadConfig("draft_r1", T=3, d=16, V=5, n=2, r=1, dtype="fp32", targets="uniform"),
], ids=lambda c: c.name)
def test_draft_sampling(gpu, oracle, cfg):
    import torch
    print(f"case {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    u = synth.uniforms(cfg.T, cfg.n)
    h = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype, flags=1)
    alpha, tokens, logq = h.draft_sample(gpu.to_device(inp["H"], cfg.dtype), torch.from_numpy(u).cuda())
    torch.cuda.synchronize()
    stats = check_draft(oracle, inp["H"], inp["W"], inp["U"], inp["G"], u, alpha.cpu().numpy(),
                        tokens.cpu().numpy(), logq.cpu().numpy(), round_y=(cfg.dtype == "bf16"), logq_atol=1e-4)
    # at these sizes the CDF steps are far wider than the band: everything must match exactly
    assert stats["alpha_exact"] == stats["alpha_total"]
    assert stats["tokens_exact"] == stats["tokens_total"]


def test_draft_boundaries(gpu):
    import torch
    cfg = synth.HeadConfig("draft_edge", T=4, d=16, V=37, n=2, r=3, dtype="fp32", targets="uniform")
    inp = synth.make_inputs(cfg)
    h = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype="fp32")
    H = gpu.to_device(inp["H"], "fp32")
    a, tok, _ = h.draft_sample(H, torch.zeros((4, 3), device="cuda"))
    assert (a.cpu().numpy() == 0).all() and (tok.cpu().numpy() == 0).all()
    top = float(np.nextafter(np.float32(1.0), np.float32(0.0)))
    a, tok, _ = h.draft_sample(H, torch.full((4, 3), top, device="cuda"))
    assert (a.cpu().numpy() == cfg.r - 1).all() and (tok.cpu().numpy() == cfg.V - 1).all()


def test_tiny_workload_against_stored_reference(gpu):
    """The same numbers the oracle wrote to tests/golden/tiny_reference.txt (see make_golden.py there)."""
    from tests.test_oracle_pins import read_golden
    vals = read_golden()
    cfg = synth.CONFIGS["tiny"]
    inp = synth.make_inputs(cfg)
    loss, grads = run_loss(gpu, cfg, inp, dloss=np.full(cfg.T, 1.0 / cfg.T, dtype=np.float32))
    for t in range(8):
        assert abs(loss[t] - vals[f"loss {t}"]) <= LOSS_ATOL
    assert abs(loss.mean() - vals["mean_loss"]) <= LOSS_ATOL
    for k in ("dH", "dW", "dU", "dG"):
        assert abs(np.linalg.norm(grads[k].ravel()) / vals[f"norm_{k}"] - 1.0) <= GRAD_REL_FRO

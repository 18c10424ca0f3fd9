"""GPU parity of the calls beyond the loss/draft hot path: the first-token marginal (eq. 11), the
paper's sequential sampling scheme (eq. 11-13) and the balancing statistic (eq. 10), each through
the C ABI against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest

from paper_2410_17765_amd import synth
from tests.helpers import LOSS_ATOL, check_sequential, tie_variants

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2410_17765_amd import binding, head
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    return head


def seq_uniforms(B, n):
    """[B,n] float32 in [0,1): one per token (the token columns of the seeded draft uniforms)."""
    return np.ascontiguousarray(synth.uniforms(B, n)[:, 1:])


# ---------------------------------------------------------------------------- first-token marginal
FIRST_CASES = [
    # (config, flags): n > 1 on purpose, only the first head may be read
    (synth.HeadConfig("first_mfma", T=9, d=128, V=1000, n=3, r=4, targets="uniform", u_scale=4.0), 0),
    (synth.HeadConfig("first_mfma_ragged", T=70, d=192, V=777, n=2, r=3, targets="uniform", u_scale=6.0), 0),
    (synth.HeadConfig("first_mfma_one", T=1, d=64, V=130, n=1, r=1, targets="uniform"), 0),
    (synth.HeadConfig("first_mfma_wide_rank", T=3, d=64, V=261, n=2, r=33, targets="uniform", u_scale=3.0), 0),
    (synth.HeadConfig("first_plain_bf16", T=6, d=64, V=300, n=2, r=3, targets="uniform", u_scale=4.0), 1),
    (synth.HeadConfig("first_plain_fp32", T=5, d=50, V=203, n=2, r=3, dtype="fp32", targets="uniform", u_scale=4.0), 0),
]


@pytest.mark.parametrize("cfg,flags", FIRST_CASES, ids=lambda c: c.name if hasattr(c, "name") else str(c))
def test_first_token_logprob(gpu, oracle, cfg, flags):
    import torch
    print(f"case {cfg} flags={flags}", flush=True)
    inp = synth.make_inputs(cfg)
    h = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype, flags=flags)
    logp = h.first_token_logprob(gpu.to_device(inp["H"], cfg.dtype))
    torch.cuda.synchronize()
    got = logp.cpu().numpy().astype(np.float64)
    ref = oracle.first_token_logprob(inp["H"], inp["W"], inp["U"], inp["G"], round_y=(cfg.dtype == "bf16"))
    assert got.shape == ref.shape == (cfg.T, cfg.V)
    row_err = np.abs(got - ref).max(axis=1)
    tie_rows = 0
    for b in np.nonzero(row_err > LOSS_ATOL)[0]:
        # an element of y on a bf16 rounding tie may round either way: the row must match one of them
        assert cfg.dtype == "bf16", ("row off", b, row_err[b])
        args = (inp["H"][b:b + 1], inp["W"], inp["U"], inp["G"])
        y = oracle.draft_sample(*args, np.zeros((1, 1 + cfg.n)), want_y=True)[-1][:, 0]          # [1,r,d]
        errs = [np.abs(got[b] - oracle.first_token_logprob(*args, round_y=True, y_nudge=nd)[0]).max()
                for flips, nd in tie_variants(y) if flips]
        assert errs and min(errs) <= LOSS_ATOL, ("row off with no rounding tie to explain it", b, row_err[b], errs)
        row_err[b] = min(errs)
        tie_rows += 1
    norm = np.abs(np.log(np.exp(got).sum(axis=1))).max()
    print(f"  max |dlogp| {row_err.max():.3e}, max |log sum p| {norm:.3e}, min logp {ref.min():.2f}, "
          f"rows on a rounding tie {tie_rows}", flush=True)
    assert tie_rows <= 1
    assert norm <= 1e-4


def random_shapes(prefix, count, seed, max_T=40):
    """Seeded random shapes over both paths (bf16 with d a multiple of 64, bf16 forced onto the plain path,
    fp32 with any d), peaked and flat heads."""
    rng = np.random.Generator(np.random.Philox(seed))
    out = []
    for i in range(count):
        kind = int(rng.integers(0, 4))                 # 0, 1: matrix-core path; 2: plain bf16; 3: plain fp32
        d = int(rng.integers(20, 200)) if kind == 3 else 64 * int(rng.integers(1, 5))
        cfg = synth.HeadConfig(f"{prefix}_random_{i}", T=int(rng.integers(1, max_T)), d=d,
                               V=int(rng.integers(70, 2500)), n=int(rng.integers(1, 5)), r=int(rng.integers(1, 10)),
                               dtype="fp32" if kind == 3 else "bf16", targets="uniform",
                               u_scale=float(rng.choice([1.0, 3.0, 6.0])))
        out.append((cfg, 1 if kind == 2 else 0))
    return out


@pytest.mark.parametrize("cfg,flags", random_shapes("first", 10, 20241020),
                         ids=lambda c: c.name if hasattr(c, "name") else str(c))
def test_first_token_logprob_random_shapes(gpu, oracle, cfg, flags):
    test_first_token_logprob(gpu, oracle, cfg, flags)


def test_first_token_matches_between_paths(gpu):
    import torch
    cfg = synth.HeadConfig("first_both", T=20, d=128, V=515, n=2, r=5, targets="uniform", u_scale=4.0)
    inp = synth.make_inputs(cfg)
    H = gpu.to_device(inp["H"], "bf16")
    a = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype="bf16").first_token_logprob(H)
    b = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype="bf16", flags=1).first_token_logprob(H)
    torch.cuda.synchronize()
    assert float((a - b).abs().max()) <= 1e-3


# ---------------------------------------------------------------------------- sequential scheme
SEQ_CASES = [
    synth.HeadConfig("seq_peaked", T=9, d=128, V=1000, n=3, r=4, targets="uniform", u_scale=4.0),
    synth.HeadConfig("seq_flat", T=5, d=64, V=2000, n=2, r=8, targets="uniform"),
    synth.HeadConfig("seq_ragged", T=70, d=192, V=777, n=4, r=3, targets="uniform", u_scale=6.0),
    synth.HeadConfig("seq_r1", T=3, d=64, V=130, n=2, r=1, targets="uniform", u_scale=3.0),
    # r*d beyond the staging buffer for y: the kernel reads y from memory
    synth.HeadConfig("seq_wide", T=2, d=1024, V=300, n=1, r=33, targets="uniform", u_scale=6.0),
]


SEQ_CASES += [
    # the plain path: fp32 storage with odd sizes, and bf16 storage forced onto it (flag 1)
    synth.HeadConfig("seq_plain_fp32", T=7, d=50, V=203, n=3, r=3, dtype="fp32", targets="uniform", u_scale=4.0),
    synth.HeadConfig("seq_plain_bf16", T=6, d=64, V=300, n=2, r=5, targets="uniform", u_scale=4.0),
]


@pytest.mark.parametrize("cfg", SEQ_CASES, ids=lambda c: c.name)
def test_sequential_sampling(gpu, oracle, cfg):
    run_sequential(gpu, oracle, cfg, 1 if cfg.name.startswith("seq_plain") else 0)


@pytest.mark.parametrize("cfg,flags", random_shapes("seq", 10, 20241021, max_T=20),
                         ids=lambda c: c.name if hasattr(c, "name") else str(c))
def test_sequential_sampling_random_shapes(gpu, oracle, cfg, flags):
    run_sequential(gpu, oracle, cfg, flags)


def run_sequential(gpu, oracle, cfg, flags):
    import torch
    print(f"case {cfg} flags={flags}", flush=True)
    inp = synth.make_inputs(cfg)
    H, W, U, G = inp["H"], inp["W"], inp["U"], inp["G"]
    u = seq_uniforms(cfg.T, cfg.n)
    h = gpu.CpHead(W, U, G, dtype=cfg.dtype, flags=flags)
    tokens, logq = h.draft_sample_sequential(gpu.to_device(H, cfg.dtype), torch.from_numpy(u).cuda())
    torch.cuda.synchronize()
    tokens, logq = tokens.cpu().numpy(), logq.cpu().numpy()
    stats = check_sequential(oracle, H, W, U, G, u, tokens, logq, round_y=(cfg.dtype == "bf16"))
    print(f"  {stats}", flush=True)
    # check_sequential has verified every draw (inside the band of the oracle's conditional under the drawn
    # prefix, or explained by a rounding tie of y); the CDF steps at these sizes are far wider than the band,
    # so all but a few draws are the oracle's own
    assert stats["tie_rows"] <= 1
    assert stats["tokens_exact"] >= (cfg.T - stats["tie_rows"]) * cfg.n - max(1, cfg.T * cfg.n // 20)


def test_sequential_boundaries(gpu):
    import torch
    cfg = synth.HeadConfig("seq_edge", T=4, d=64, V=300, n=2, r=3, targets="uniform")
    inp = synth.make_inputs(cfg)
    h = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype="bf16")
    H = gpu.to_device(inp["H"], "bf16")
    tok, _ = h.draft_sample_sequential(H, torch.zeros((4, 2), device="cuda"))
    assert (tok.cpu().numpy() == 0).all()
    top = float(np.nextafter(np.float32(1.0), np.float32(0.0)))
    tok, _ = h.draft_sample_sequential(H, torch.full((4, 2), top, device="cuda"))
    assert (tok.cpu().numpy() == cfg.V - 1).all()
    hp = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype="bf16", flags=1)       # the plain path
    tok, _ = hp.draft_sample_sequential(H, torch.zeros((4, 2), device="cuda"))
    assert (tok.cpu().numpy() == 0).all()
    tok, _ = hp.draft_sample_sequential(H, torch.full((4, 2), top, device="cuda"))
    assert (tok.cpu().numpy() == cfg.V - 1).all()


def test_sequential_and_expert_first_draw_agree_for_one_expert(gpu):
    """With r = 1 both samplers draw every token from the same distribution with the same uniform."""
    import torch
    cfg = synth.HeadConfig("seq_vs_expert", T=11, d=128, V=999, n=3, r=1, targets="uniform", u_scale=5.0)
    inp = synth.make_inputs(cfg)
    u = synth.uniforms(cfg.T, cfg.n)
    h = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype="bf16")
    H = gpu.to_device(inp["H"], "bf16")
    _, tok_a, lq_a = h.draft_sample(H, torch.from_numpy(u).cuda())
    tok_b, lq_b = h.draft_sample_sequential(H, torch.from_numpy(np.ascontiguousarray(u[:, 1:])).cuda())
    torch.cuda.synchronize()
    assert torch.equal(tok_a, tok_b)
    assert float((lq_a - lq_b).abs().max()) <= 1e-4


# ---------------------------------------------------------------------------- balancing statistic
AUX_CASES = [
    synth.HeadConfig("aux_bf16", T=5000, d=128, V=8, n=1, r=8),
    synth.HeadConfig("aux_fp32_odd", T=777, d=50, V=8, n=1, r=5, dtype="fp32"),
    synth.HeadConfig("aux_wide", T=100000, d=64, V=8, n=1, r=64),
    synth.HeadConfig("aux_one", T=1, d=64, V=8, n=1, r=3),
]


@pytest.mark.parametrize("cfg", AUX_CASES, ids=lambda c: c.name)
def test_aux_balance(gpu, oracle, cfg):
    import torch
    print(f"case {cfg}", flush=True)
    Hn, Gn = synth.hidden(cfg), synth.gate(cfg)
    h = gpu.CpHead(synth.head_weights(cfg), synth.unembedding(cfg), Gn, dtype=cfg.dtype)
    counts, laux = h.aux_balance(gpu.to_device(Hn, cfg.dtype))
    torch.cuda.synchronize()
    counts, laux = counts.cpu().numpy(), float(laux.cpu().numpy()[0])
    c_o, l_o = oracle.aux_balance(Hn.astype(np.float64), Gn.astype(np.float64))
    print(f"  counts {counts.tolist()[:8]} laux {laux:.6e} (oracle {l_o:.6e})", flush=True)
    assert counts.sum() == cfg.T
    # the arg-max is decided in fp32 on the GPU and in fp64 by the oracle: a position may move between
    # two experts only when their gate pre-activations agree to fp32 accumulation error, which at these
    # sizes is rarer than one position in a million
    np.testing.assert_array_equal(counts, c_o)
    assert abs(laux - l_o) <= 1e-6 * max(1.0, l_o)


def test_aux_balance_empty(gpu):
    import torch
    cfg = synth.HeadConfig("aux_empty", T=0, d=64, V=8, n=1, r=4)
    h = gpu.CpHead(synth.head_weights(cfg), synth.unembedding(cfg), synth.gate(cfg), dtype="bf16")
    counts, laux = h.aux_balance(torch.empty((0, 64), dtype=torch.bfloat16, device="cuda"))
    torch.cuda.synchronize()
    assert counts.cpu().numpy().tolist() == [0, 0, 0, 0]
    assert abs(float(laux.cpu().numpy()[0]) - 0.25) < 1e-7

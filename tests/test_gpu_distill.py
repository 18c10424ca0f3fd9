"""GPU parity of the head-only fine-tuning loss (eq. 14 and the discounted sum after it) against the fp64
oracle, element by element: the ranks the matrix-core path serves, the plain path for every other shape and
for fp32 storage, ragged tiles, several chunks, dropped tokens."""
import numpy as np
import pytest

from paper_2410_17765_amd import synth
from tests.helpers import distill_loss_atol_bf16, GRAD_REL_FRO, LOSS_ATOL, loss_atol_bf16, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2410_17765_amd import binding, head
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    return head


def run(head, cfg, inp, TZ, beta, disc, dloss=None, flags=0, want_dU=True):
    import torch
    h = head.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype, flags=flags)
    H = head.to_device(inp["H"], cfg.dtype)
    X = torch.from_numpy(inp["X"]).cuda()
    tz = head.to_device(TZ, cfg.dtype)
    loss = h.distill_loss_fwd(H, X, tz, beta, disc)
    dl = None if dloss is None else torch.from_numpy(dloss).cuda()
    grads = {k: v.cpu().numpy() for k, v in h.distill_loss_bwd(H, X, tz, dl, want_dU=want_dU).items()}
    torch.cuda.synchronize()
    return loss.cpu().numpy(), grads


_ORACLE_RESULTS = {}

CASES = [
    # (config, flags, beta, discount); the prescribed initialisation (u_scale = 1) except for one peaked case
    (synth.HeadConfig("distill_r8", T=150, d=128, V=1000, n=2, r=8), 0, 0.9, 0.8),
    (synth.HeadConfig("distill_r4_ragged", T=523, d=192, V=777, n=3, r=4), 0, 0.9, 1.0),
    (synth.HeadConfig("distill_r2_chunked", T=300, d=64, V=515, n=2, r=2), 2, 0.5, 0.7),
    (synth.HeadConfig("distill_r1", T=70, d=64, V=300, n=3, r=1), 0, 0.9, 0.9),
    (synth.HeadConfig("distill_one_position", T=1, d=64, V=260, n=1, r=8), 0, 0.9, 1.0),
    (synth.HeadConfig("distill_no_teacher_weight", T=64, d=64, V=300, n=2, r=4), 0, 0.0, 1.0),
    (synth.HeadConfig("distill_r8_peaked", T=150, d=128, V=1000, n=2, r=8, u_scale=3.0), 0, 0.9, 0.8),
    # the plain path: ranks that do not align with the tile rows, fp32 storage with odd sizes, bf16 forced onto
    # it (flag 1), several chunks of 256 rows (flag 2), more experts than a token group of the tile holds
    (synth.HeadConfig("distill_plain_bf16_r3", T=130, d=64, V=300, n=2, r=3), 0, 0.9, 0.9),
    (synth.HeadConfig("distill_plain_fp32_r5", T=37, d=50, V=301, n=3, r=5, dtype="fp32"), 0, 0.9, 0.8),
    (synth.HeadConfig("distill_plain_forced_r4", T=60, d=64, V=515, n=2, r=4), 1, 0.5, 1.0),
    (synth.HeadConfig("distill_plain_chunked_r6", T=200, d=96, V=333, n=2, r=6, dtype="fp32"), 2, 0.9, 0.7),
    (synth.HeadConfig("distill_plain_r33", T=20, d=64, V=260, n=2, r=33), 0, 0.9, 1.0),
]


@pytest.mark.parametrize("cfg,flags,beta,disc", CASES, ids=lambda c: c.name if hasattr(c, "name") else None)
def test_loss_and_gradients(gpu, oracle, cfg, flags, beta, disc):
    print(f"case {cfg} flags={flags} beta={beta} discount={disc}", flush=True)
    inp = synth.make_inputs(cfg)
    TZ = synth.teacher_logits(cfg)
    if cfg.T > 8:
        inp["X"][3, 0] = -1                       # a dropped first token
        inp["X"][4, cfg.n - 1] = -1               # a dropped last token
        inp["X"][5, :] = -1                       # a position with no targets at all
    dloss = synth.upstream_grad(cfg.T).astype(np.float32)
    loss, g = run(gpu, cfg, inp, TZ, beta, disc, dloss, flags)
    if cfg.name not in _ORACLE_RESULTS:       # the cases with kept logits use the same inputs again
        _ORACLE_RESULTS[cfg.name] = (
            oracle.distill_loss_fwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"], TZ, beta=beta, disc=disc),
            oracle.distill_loss_bwd(inp["H"], inp["W"], inp["U"], inp["G"], inp["X"], TZ, beta=beta, disc=disc,
                                    dloss=dloss.astype(np.float64)))
    ref, rg = _ORACLE_RESULTS[cfg.name]
    err = np.abs(loss - ref).max()
    print(f"  loss max abs err {err:.3e} (mean loss {ref.mean():.3f})", flush=True)
    # The logits behind the log-normalisers and the mixture come from y rounded to bf16 (the matrix-core
    # operand): each carries an error of about |U_v| rms(y) 2^-9 / sqrt(3) = 1.1e-3 u_scale, which the
    # probability-weighted sums average down.  The bound is the loss tolerance at the prescribed
    # initialisation, scales with the logits otherwise, and grows where a small vocabulary leaves the teacher's
    # probabilities little to average over (see the helper).
    assert err <= distill_loss_atol_bf16(cfg)
    for k in ("dH", "dW", "dU", "dG"):
        if k == "dG" and cfg.r == 1:
            # one expert: the gate weight is the constant 1 and its gradient vanishes identically
            # (on the GPU: a sum over positions of fp32 rounding noise of size 1e-6 each)
            assert np.abs(rg[k]).max() <= 1e-12 and np.abs(g[k]).max() <= 2e-6 * max(cfg.T, 8)
            continue
        e = rel_fro(g[k], rg[k])
        print(f"  {k} rel fro {e:.3e}", flush=True)
        assert e <= GRAD_REL_FRO, k


def random_shapes(count=12, seed=20241019, budget=6e8):
    """Seeded random shapes over both paths: any rank up to 9, d a multiple of 64 or not, bf16 or fp32."""
    rng = np.random.Generator(np.random.Philox(seed))
    out = []
    for i in range(count):
        fp32 = bool(rng.integers(0, 3) == 0)
        d = int(rng.integers(20, 200)) if fp32 else 64 * int(rng.integers(1, 4))
        V = int(rng.integers(64, 1200))
        n = int(rng.integers(1, 5))
        r = int(rng.integers(1, 10))
        T = int(rng.integers(1, 600))
        if float(T) * n * r * V * d > budget:
            T = max(1, int(budget / (float(n) * r * V * d)))
        flags = 2 if rng.integers(0, 3) == 0 else 0
        cfg = synth.HeadConfig(f"distill_random_{i}", T=T, d=d, V=V, n=n, r=r, dtype="fp32" if fp32 else "bf16")
        out.append((cfg, flags, float(rng.choice([0.3, 0.9, 1.0])), float(rng.choice([0.6, 1.0]))))
    return out


@pytest.mark.parametrize("cfg,flags,beta,disc", random_shapes(), ids=lambda c: c.name if hasattr(c, "name") else None)
def test_loss_and_gradients_random_shapes(gpu, oracle, cfg, flags, beta, disc):
    test_loss_and_gradients(gpu, oracle, cfg, flags, beta, disc)


def test_matches_training_loss_without_teacher_term(gpu):
    """beta = 0, no discount: the loss and its gradients are those of cp_head_loss_fwd/bwd."""
    import torch
    cfg = synth.HeadConfig("distill_vs_loss", T=200, d=128, V=600, n=3, r=8)
    inp = synth.make_inputs(cfg)
    TZ = synth.teacher_logits(cfg)
    l1, g1 = run(gpu, cfg, inp, TZ, 0.0, 1.0)
    h = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype="bf16")
    H = gpu.to_device(inp["H"], "bf16")
    X = torch.from_numpy(inp["X"]).cuda()
    l2 = h.loss_fwd(H, X).cpu().numpy()
    g2 = {k: v.cpu().numpy() for k, v in h.loss_bwd(H, X).items()}
    assert np.abs(l1 - l2).max() <= 1e-4
    for k in g2:
        assert rel_fro(g1[k], g2[k]) <= 5e-3, k


KEEP_LOGITS = 4      # CP_HEAD_KEEP_LOGITS: the two later passes read the first product's logits instead of recomputing them


def kept_shapes(count=8, seed=20241023, budget=6e8):
    """Seeded random shapes on the matrix-core path (bf16, d a multiple of 64, r in {1, 2, 4, 8}), where the flag
    for kept logits is honoured; V is rarely a multiple of 8, so the teacher rows are mostly read unaligned."""
    rng = np.random.Generator(np.random.Philox(seed))
    out = []
    for i in range(count):
        d = 64 * int(rng.integers(1, 4))
        V = int(rng.integers(64, 1200)) if i % 3 else 8 * int(rng.integers(8, 150))
        n = int(rng.integers(1, 5))
        r = int(rng.choice([1, 2, 4, 8]))
        T = int(rng.integers(1, 600))
        if float(T) * n * r * V * d > budget:
            T = max(1, int(budget / (float(n) * r * V * d)))
        flags = KEEP_LOGITS | (2 if rng.integers(0, 3) == 0 else 0)
        cfg = synth.HeadConfig(f"distill_kept_{i}", T=T, d=d, V=V, n=n, r=r)
        out.append((cfg, flags, float(rng.choice([0.3, 0.9, 1.0])), float(rng.choice([0.6, 1.0]))))
    return out


@pytest.mark.parametrize("cfg,flags,beta,disc",
                         [(c, f | KEEP_LOGITS, b, d) for c, f, b, d in CASES + random_shapes()[:3]] + kept_shapes()[:4],
                         ids=lambda c: c.name if hasattr(c, "name") else None)
def test_loss_and_gradients_with_kept_logits(gpu, oracle, cfg, flags, beta, disc):
    """On the plain path the flag is ignored; on the matrix-core path the second and third products become
    passes over the kept logits."""
    test_loss_and_gradients(gpu, oracle, cfg, flags, beta, disc)


def test_kept_logits_against_recomputed_ones(gpu):
    cfg = synth.HeadConfig("distill_keep_vs_recompute", T=300, d=128, V=1000, n=3, r=4)
    inp = synth.make_inputs(cfg)
    TZ = synth.teacher_logits(cfg)
    inp["X"][::5, 1] = -1
    l0, g0 = run(gpu, cfg, inp, TZ, 0.9, 0.8)
    for flags in (KEEP_LOGITS, KEEP_LOGITS | 2):
        l1, g1 = run(gpu, cfg, inp, TZ, 0.9, 0.8, flags=flags)
        print(f"  flags={flags} loss: kept vs recomputed max abs {np.abs(l0 - l1).max():.3e}", flush=True)
        assert np.abs(l0 - l1).max() <= 2e-4
        for k in g0:
            e = rel_fro(g1[k], g0[k])
            print(f"  flags={flags} {k}: kept vs recomputed rel fro {e:.3e}", flush=True)
            assert e <= 3e-3, (k, e)
    # the plain path ignores the flag
    la, ga = run(gpu, cfg, inp, TZ, 0.9, 0.8, flags=1)
    lb, gb = run(gpu, cfg, inp, TZ, 0.9, 0.8, flags=1 | KEEP_LOGITS)
    np.testing.assert_array_equal(la, lb)
    for k in ga:
        np.testing.assert_array_equal(ga[k], gb[k])


def test_frozen_unembedding_and_empty_batch(gpu):
    import torch
    cfg = synth.HeadConfig("distill_opts", T=130, d=64, V=300, n=2, r=2)
    inp = synth.make_inputs(cfg)
    TZ = synth.teacher_logits(cfg)
    _, g1 = run(gpu, cfg, inp, TZ, 0.9, 0.9)
    _, g2 = run(gpu, cfg, inp, TZ, 0.9, 0.9, want_dU=False)
    assert "dU" not in g2
    for k in g2:
        np.testing.assert_array_equal(g1[k], g2[k])
    # empty batch
    h = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype="bf16")
    H0 = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    X0 = torch.empty((0, 2), dtype=torch.int32, device="cuda")
    T0 = torch.empty((0, 2, 300), dtype=torch.bfloat16, device="cuda")
    assert h.distill_loss_fwd(H0, X0, T0).shape == (0,)
    g = h.distill_loss_bwd(H0, X0, T0, want_dU=True)
    torch.cuda.synchronize()
    assert float(g["dW"].abs().max()) == 0.0 and float(g["dU"].abs().max()) == 0.0


def test_headline_shape_on_sampled_positions(gpu, oracle):
    """d, V, n, r of the headline workload (two chunks of head rows, 125 vocabulary tiles, K = 4096) on its
    first 2048 positions; loss and gradients against the oracle on 8 sampled positions, as in the
    full-size tests of the training loss (the unembedding is frozen: dU is not asked for)."""
    import torch
    full = synth.CONFIGS["head_7b"]
    cfg = full.with_(T=2048)
    print(f"[distill] generating {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    TZ = synth.teacher_logits(cfg)
    h = gpu.CpHead(inp["W"], inp["U"], inp["G"], dtype=cfg.dtype)
    H = gpu.to_device(inp["H"], cfg.dtype)
    X = torch.from_numpy(inp["X"]).cuda()
    tz = gpu.to_device(TZ, cfg.dtype)
    beta, disc, scale = 0.9, 0.8, 1.0 / cfg.T
    print("[distill] running on the GPU", flush=True)
    loss = h.distill_loss_fwd(H, X, tz, beta, disc)
    grads = h.distill_loss_bwd(H, X, tz, None, scale=scale)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(loss).all())
    sel = synth.position_subset(cfg.T, 8)
    print(f"[distill] oracle on positions {sel.tolist()}", flush=True)
    args = (inp["H"][sel], inp["W"], inp["U"], inp["G"], inp["X"][sel], TZ[sel])
    ref = oracle.distill_loss_fwd(*args, beta=beta, disc=disc)
    err = np.abs(loss.cpu().numpy()[sel] - ref).max()
    print(f"  loss max abs err {err:.3e} (mean loss {ref.mean():.3f})", flush=True)
    assert err <= LOSS_ATOL
    rg = oracle.distill_loss_bwd(*args, beta=beta, disc=disc, dloss=np.full(len(sel), scale), want=("dH", "dW", "dG"))
    e = rel_fro(grads["dH"][torch.from_numpy(sel).cuda()].cpu().numpy(), rg["dH"])
    print(f"  dH rows rel fro {e:.3e}", flush=True)
    assert e <= GRAD_REL_FRO
    # weight gradients: a GPU call on exactly these positions
    Hs, Xs, tzs = gpu.to_device(inp["H"][sel], cfg.dtype), torch.from_numpy(inp["X"][sel]).cuda(), gpu.to_device(TZ[sel], cfg.dtype)
    h.distill_loss_fwd(Hs, Xs, tzs, beta, disc)
    g = h.distill_loss_bwd(Hs, Xs, tzs, None, scale=scale)
    torch.cuda.synchronize()
    for k in ("dW", "dG", "dH"):
        e = rel_fro(g[k].cpu().numpy(), rg[k])
        print(f"  subset {k} rel fro {e:.3e}", flush=True)
        assert e <= GRAD_REL_FRO, k
    # the batch gradient is the sum of the gradients of its halves
    half = cfg.T // 2
    tot = None
    for lo, hi in ((0, half), (half, cfg.T)):
        h.distill_loss_fwd(H[lo:hi].contiguous(), X[lo:hi].contiguous(), tz[lo:hi].contiguous(), beta, disc)
        gh = h.distill_loss_bwd(H[lo:hi].contiguous(), X[lo:hi].contiguous(), tz[lo:hi].contiguous(), None, scale=scale)
        torch.cuda.synchronize()
        tot = gh["dW"].clone() if tot is None else tot + gh["dW"]
    rel = float((tot - grads["dW"]).double().norm() / grads["dW"].double().norm())
    print(f"  dW: |full - (first half + second half)| / |full| = {rel:.3e}", flush=True)
    assert rel <= 2e-3

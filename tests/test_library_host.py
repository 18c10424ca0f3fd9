"""Host-side checks of libcphead.so that need no GPU: the library loads, exports every symbol the
header declares, answers the size queries and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

from paper_2410_17765_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2410_17765_amd import build
        build.build(verbose=False)
    return binding.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cp_head.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cp_head_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_strerror(lib):
    assert binding.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert binding.strerror(code)


def test_size_queries(lib):
    ds = binding.make_desc(64, 64, 512, 2, 2, binding.FP32)
    ctx = binding.cp_head_ctx_bytes(ds)
    M = 64 * 2 * 2
    assert ctx >= M * 4 + 2 * 64 * 2 * 4 + M * 64 * 4
    for op in (binding.OP_LOSS_FWD, binding.OP_LOSS_BWD, binding.OP_DRAFT):
        assert binding.cp_head_workspace_bytes(ds, op) > 0
    # the backward workspace does not keep logit-sized buffers for all rows: it stops growing with T
    big = binding.make_desc(1 << 20, 64, 512, 2, 2, binding.FP32)
    huge = binding.make_desc(1 << 21, 64, 512, 2, 2, binding.FP32)
    per_row_big = binding.cp_head_workspace_bytes(big, binding.OP_LOSS_BWD) / (1 << 20)
    per_row_huge = binding.cp_head_workspace_bytes(huge, binding.OP_LOSS_BWD) / (1 << 21)
    assert per_row_huge < 2 * 2 * 512 * 2      # far below one row of logits per head row
    assert per_row_huge <= per_row_big + 1


def test_headline_shape_sizes(lib):
    ds = binding.make_desc(16384, 4096, 32000, 4, 8, binding.BF16)
    logits_bytes = 16384 * 32 * 32000 * 2
    assert binding.cp_head_ctx_bytes(ds) < logits_bytes // 4
    assert binding.cp_head_workspace_bytes(ds, binding.OP_LOSS_FWD) < logits_bytes // 4


@pytest.mark.parametrize("kw", [dict(T=-1), dict(d=0), dict(V=0), dict(n=0), dict(r=0)])
def test_bad_dimensions(lib, kw):
    base = dict(T=4, d=8, V=16, n=2, r=2)
    base.update(kw)
    ds = binding.make_desc(base["T"], base["d"], base["V"], base["n"], base["r"], binding.FP32)
    out = ctypes.c_size_t()
    assert lib.cp_head_ctx_bytes(ctypes.byref(ds), ctypes.byref(out)) == -1


def test_unsupported(lib):
    out = ctypes.c_size_t()
    assert lib.cp_head_ctx_bytes(ctypes.byref(binding.make_desc(4, 8, 16, 2, 65, binding.FP32)),
                                 ctypes.byref(out)) == -2
    assert lib.cp_head_ctx_bytes(ctypes.byref(binding.make_desc(4, 8, 16, 2, 2, 7)), ctypes.byref(out)) == -2
    assert lib.cp_head_ctx_bytes(None, ctypes.byref(out)) == -1
    assert lib.cp_head_workspace_bytes(ctypes.byref(binding.make_desc(4, 8, 16, 2, 2, 0)), 99,
                                       ctypes.byref(out)) == -1


def test_null_and_small_workspace_rejected_before_launch(lib):
    # fake, aligned, never dereferenced "device pointers": every call must fail in validation
    ds = binding.make_desc(4, 8, 16, 2, 2, binding.FP32)
    p = 0x10000
    need = binding.cp_head_workspace_bytes(ds, binding.OP_LOSS_FWD)
    args = [ctypes.byref(ds), p, p, p, p, p, p, p, p, need, None]
    bad = list(args); bad[2] = None
    assert lib.cp_head_loss_fwd(*bad) == -1
    bad = list(args); bad[8] = p + 8            # misaligned workspace
    assert lib.cp_head_loss_fwd(*bad) == -1
    bad = list(args); bad[9] = need - 1
    assert lib.cp_head_loss_fwd(*bad) == -3
    needb = binding.cp_head_workspace_bytes(ds, binding.OP_LOSS_BWD)
    argsb = [ctypes.byref(ds), p, p, p, p, p, None, 1.0, p, p, p, p, p, p, needb - 1, None]
    assert lib.cp_head_loss_bwd(*argsb) == -3
    argsb[14] = needb; argsb[9] = None          # dH is required
    assert lib.cp_head_loss_bwd(*argsb) == -1
    needd = binding.cp_head_workspace_bytes(ds, binding.OP_DRAFT)
    argsd = [ctypes.byref(ds), p, p, p, p, p, None, p, p, p, needd, None]
    assert lib.cp_head_draft_sample(*argsd) == -1
    argsd[6] = p; argsd[10] = 0
    assert lib.cp_head_draft_sample(*argsd) == -3


def test_new_calls_reject_bad_arguments_before_launch(lib):
    p = 0x10000
    bf = binding.make_desc(4, 64, 300, 2, 2, binding.BF16)
    fp = binding.make_desc(4, 8, 16, 2, 2, binding.FP32)
    # first-token marginal: both paths are served; null input, short workspace
    for ds in (bf, fp):
        need = binding.cp_head_workspace_bytes(ds, binding.OP_FIRST_TOKEN)
        assert need > 4 * 2 * ds.V * 4                       # it holds the r rows of logits per row of the batch
        args = [ctypes.byref(ds), p, p, p, p, p, p, need, None]
        bad = list(args); bad[5] = None
        assert lib.cp_head_first_token_logprob(*bad) == -1
        bad = list(args); bad[7] = need - 1
        assert lib.cp_head_first_token_logprob(*bad) == -3
    # sequential sampler and full heads: both paths
    args = [ctypes.byref(fp), p, p, p, p, p, p, p, p, 0, None]
    assert lib.cp_head_draft_sample_sequential(*args) == -3
    args[0] = ctypes.byref(bf)
    assert lib.cp_head_draft_sample_sequential(*args) == -3
    args[5] = None                                           # uniforms
    assert lib.cp_head_draft_sample_sequential(*args) == -1
    out = ctypes.c_size_t()
    assert lib.cp_head_full_ctx_bytes(ctypes.byref(bf), ctypes.byref(out)) == 0 and out.value >= 4 * 2 * 2 * 4
    for ds in (fp, bf):
        argsf = [ctypes.byref(ds), p, p, p, p, p, p, p, 0, None]
        assert lib.cp_head_full_loss_fwd(*argsf) == -3
    argsb = [ctypes.byref(bf), p, p, p, p, None, 1.0, p, None, p, p, p, 1 << 30, None]
    assert lib.cp_head_full_loss_bwd(*argsb) == -1           # dH is required
    # fine-tuning loss: both paths, beta in [0, 1], teacher logits required
    r3 = binding.make_desc(4, 64, 300, 2, 3, binding.BF16)
    assert lib.cp_head_distill_ctx_bytes(ctypes.byref(r3), ctypes.byref(out)) == 0
    assert lib.cp_head_distill_ctx_bytes(ctypes.byref(bf), ctypes.byref(out)) == 0
    assert out.value > binding.cp_head_ctx_bytes(bf)
    argsd = [ctypes.byref(bf), p, p, p, p, p, p, 0.9, 1.0, p, p, p, 1 << 30, None]
    bad = list(argsd); bad[7] = 1.5
    assert lib.cp_head_distill_loss_fwd(*bad) == -1
    bad = list(argsd); bad[6] = None
    assert lib.cp_head_distill_loss_fwd(*bad) == -1
    bad = list(argsd); bad[12] = 0
    assert lib.cp_head_distill_loss_fwd(*bad) == -3
    bad = list(argsd); bad[0] = ctypes.byref(r3); bad[12] = 0
    assert lib.cp_head_distill_loss_fwd(*bad) == -3
    # balancing statistic: outputs required
    assert lib.cp_head_aux_balance(ctypes.byref(bf), p, p, None, p, p, 256, None) == -1


def test_binding_constants_match_the_header():
    """The Python binding restates the header's enumerators: flags, storage types, error codes, operations."""
    text = open(os.path.join(ROOT, "include", "cp_head.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    values = {name: int(val) for name, val in re.findall(r"\b(CP_HEAD_[A-Z0-9_]+)\s*=\s*(-?\d+)", text)}
    assert values["CP_HEAD_FORCE_GENERIC"] == binding.FORCE_GENERIC
    assert values["CP_HEAD_MIN_WORKSPACE"] == binding.MIN_WORKSPACE
    assert values["CP_HEAD_KEEP_LOGITS"] == binding.KEEP_LOGITS
    assert values["CP_HEAD_FP32"] == binding.FP32 and values["CP_HEAD_BF16"] == binding.BF16
    for name in ("LOSS_FWD", "LOSS_BWD", "DRAFT", "FIRST_TOKEN", "DRAFT_SEQUENTIAL", "AUX_BALANCE", "FULL_LOSS_FWD",
                 "FULL_LOSS_BWD", "DISTILL_FWD", "DISTILL_BWD"):
        assert values["CP_HEAD_OP_" + name] == getattr(binding, "OP_" + name), name


def test_kept_logits_are_sized_into_ctx_on_the_matrix_core_path_only(lib):
    T, d, V, n, r = 1000, 128, 1000, 2, 3
    plain = binding.make_desc(T, d, V, n, r, binding.BF16, 0)
    keep = binding.make_desc(T, d, V, n, r, binding.BF16, binding.KEEP_LOGITS)
    rows, Vp, blocks = T * n * r, 1024, 8                    # V rounded up to 64; blocks of 128 columns
    extra = binding.cp_head_ctx_bytes(keep) - binding.cp_head_ctx_bytes(plain)
    assert rows * (Vp * 2 + blocks * 8) <= extra <= rows * (Vp * 2 + blocks * 8) + 512
    # the statistics move from the forward workspace into ctx; the backward workspace is the same
    assert (binding.cp_head_workspace_bytes(plain, binding.OP_LOSS_FWD)
            - binding.cp_head_workspace_bytes(keep, binding.OP_LOSS_FWD)) >= rows * blocks * 8
    assert (binding.cp_head_workspace_bytes(plain, binding.OP_LOSS_BWD)
            == binding.cp_head_workspace_bytes(keep, binding.OP_LOSS_BWD))
    # ignored on the plain path and by the fine-tuning loss
    for dtype, flags in ((binding.FP32, 0), (binding.BF16, binding.FORCE_GENERIC)):
        a = binding.make_desc(T, d, V, n, r, dtype, flags)
        b = binding.make_desc(T, d, V, n, r, dtype, flags | binding.KEEP_LOGITS)
        assert binding.cp_head_ctx_bytes(a) == binding.cp_head_ctx_bytes(b)
    # the fine-tuning loss: ignored at r = 3 (its plain path), honoured at r = 4
    out_a, out_b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    assert lib.cp_head_distill_ctx_bytes(ctypes.byref(plain), ctypes.byref(out_a)) == 0
    assert lib.cp_head_distill_ctx_bytes(ctypes.byref(keep), ctypes.byref(out_b)) == 0
    assert out_a.value == out_b.value
    for op in (binding.OP_DISTILL_FWD, binding.OP_DISTILL_BWD):
        assert binding.cp_head_workspace_bytes(plain, op) == binding.cp_head_workspace_bytes(keep, op)
    plain4 = binding.make_desc(T, d, V, n, 4, binding.BF16, 0)
    keep4 = binding.make_desc(T, d, V, n, 4, binding.BF16, binding.KEEP_LOGITS)
    assert lib.cp_head_distill_ctx_bytes(ctypes.byref(plain4), ctypes.byref(out_a)) == 0
    assert lib.cp_head_distill_ctx_bytes(ctypes.byref(keep4), ctypes.byref(out_b)) == 0
    assert out_b.value - out_a.value >= T * n * 4 * Vp * 2
    assert (binding.cp_head_workspace_bytes(keep4, binding.OP_DISTILL_FWD)
            < binding.cp_head_workspace_bytes(plain4, binding.OP_DISTILL_FWD))


def test_full_head_workspace_is_bounded_in_positions(lib):
    a = binding.make_desc(1 << 16, 4096, 32000, 4, 8, binding.BF16)
    b = binding.make_desc(1 << 17, 4096, 32000, 4, 8, binding.BF16)
    wa = binding.cp_head_workspace_bytes(a, binding.OP_FULL_LOSS_BWD)
    wb = binding.cp_head_workspace_bytes(b, binding.OP_FULL_LOSS_BWD)
    # doubling T adds per-position bookkeeping only (row info, transposed H), never logit-sized rows
    assert (wb - wa) / (1 << 16) < 4 * 8 * 16 + 4096 * 2 + 8 * 4 + 4096


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: any other count ends with a message and a non-zero status, before
    anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0 and "one GPU" in res.stderr and res.stdout.strip() == ""


def test_bench_defaults_and_roofline_constants():
    import importlib.util
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    argv, sys.argv = sys.argv, ["bench.py"]
    try:
        args = bench.parse()
    finally:
        sys.argv = argv
    assert args.gpus == 1 and args.steps >= 10 and args.warmup >= 3 and args.workload == "head_7b"
    assert bench.PEAK_BF16_TFLOPS == 2500.0                      # dense bf16 matrix peak of the MI355X


def test_fine_tuning_loss_applies_the_plain_paths_limit_by_its_own_path_choice(lib):
    """Ranks other than 1, 2, 4, 8 send the fine-tuning loss to the plain path even at shapes where the training
    loss runs on the matrix cores, so a hidden size beyond the plain path's limit must be refused up front
    (size queries and calls alike), not after some kernels have been enqueued."""
    wide = binding.make_desc(64, 16384, 1000, 2, 3, binding.BF16)
    assert binding.cp_head_workspace_bytes(wide, binding.OP_LOSS_FWD) > 0          # training loss: matrix cores
    for query in (lambda: binding.cp_head_distill_ctx_bytes(wide),
                  lambda: binding.cp_head_workspace_bytes(wide, binding.OP_DISTILL_FWD),
                  lambda: binding.cp_head_workspace_bytes(wide, binding.OP_DISTILL_BWD)):
        with pytest.raises(binding.CpHeadError) as err:
            query()
        assert err.value.code == -2
    fine = binding.make_desc(64, 16384, 1000, 2, 4, binding.BF16)                  # rank 4: matrix cores
    assert binding.cp_head_distill_ctx_bytes(fine) > 0
    assert binding.cp_head_workspace_bytes(fine, binding.OP_DISTILL_BWD) > 0
    # the calls themselves refuse before looking at any pointer that would be dereferenced
    rc = lib.cp_head_distill_loss_fwd(ctypes.byref(wide), 256, 256, 256, 256, 256, 256, 0.5, 1.0, 256, 256, 256,
                                      1 << 40, None)
    assert rc == -2


def _profile_rows(name):
    """Rows of the markdown tables of one rocprofv3 summary under profiles/: {first cell: [other cells as float or str]}."""
    rows = {}
    for line in open(os.path.join(ROOT, "profiles", name)):
        if not line.startswith("|") or line.startswith("|---"):
            continue
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        vals = []
        for c in cells[1:]:
            try:
                vals.append(float(c))
            except ValueError:
                vals.append(c)
        rows.setdefault(cells[0], []).append(vals)
    return rows


def test_bench_traffic_constants_match_the_profile_summaries():
    """bench.py reports `roofline.traffic` from constants copied out of the counter runs summarised under profiles/:
    every constant must be what the table it names says (fetch + write GiB per dispatch)."""
    import sys
    sys.path.insert(0, ROOT)
    import bench
    gib = float(1 << 30)

    def fetch_write(table, kernel, dispatches):
        hit = [v for v in table[kernel] if len(v) == 3 and v[0] == dispatches]
        assert len(hit) == 1, (kernel, dispatches, table.get(kernel))
        return (hit[0][1] + hit[0][2]) * gib

    head = _profile_rows("loss_head_7b_kernel_stats.md")
    kept = _profile_rows("loss_head_7b_kept_logits_kernel_stats.md")
    single = _profile_rows("loss_head_7b_single_call_kernel_stats.md")
    want = {
        ("head_7b", "gemm_z_stats", 1): fetch_write(head, "k_gemm_nt<256x256x64,EpiRowStats>", 1),
        ("head_7b", "gemm_z_dz", 8): fetch_write(head, "k_gemm_nt<256x256x64,EpiDz>", 8),
        ("head_7b", "gemm_z_stats_keep", 1): fetch_write(kept, "k_gemm_nt<256x256x64,EpiRowStatsKeep>", 1),
        ("head_7b", "gemm_z_stats_keep", 8): fetch_write(single, "k_gemm_nt<256x256x64,EpiRowStatsKeep>", 8),
    }
    draft = _profile_rows("draft_b8_kernel_stats.md")
    per_dispatch = [row[1] for k, v in draft.items() if k.startswith("k_")
                    for row in v if len(row) == 2 and isinstance(row[1], float)
                    and row[0] >= 1 and row[0] == int(row[0])]           # the table of fills at B = 8: dispatches, GiB
    want[("draft", 8)] = sum(per_dispatch) * gib
    step = [v for v in draft["step"] if len(v) == 2][0]
    want[("draft", 1)], want[("draft", 64)] = step[0] * gib, step[1] * gib
    assert set(want) == set(bench.TRAFFIC_BYTES), set(want) ^ set(bench.TRAFFIC_BYTES)
    for key, value in want.items():
        assert abs(bench.TRAFFIC_BYTES[key] - value) <= 2e-3 * value, (key, bench.TRAFFIC_BYTES[key] / gib, value / gib)

"""GPU parity of the level-scan family (the level-by-level formulation of Section 3.2, Eqs. 6-10) through the C ABI.

Expected values come from the fp64 fold oracle (the definition, Section 3.1) and, on small cases, also from the
level-by-level oracle written in the paper's own order; the gate is the same per-level relative error as for the
other families.
"""
import numpy as np
import pytest

from paper_2501_08455_amd import workloads
from test_gpu_parity import TOL, assert_parity, check, gpu, level_errors, run_gpu, say  # noqa: F401  (gpu is a fixture)

pytestmark = pytest.mark.gpu


def plan_for(gpu, chunks=0):
    return gpu.make_plan(gpu.SIG_VARIANT_LEVEL_SCAN, chunks=chunks)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_configs(gpu, oracle, name):
    cfg = workloads.CONFIGS[name]
    x = workloads.make_paths(cfg)
    check(gpu, oracle, x, cfg.depth, cfg.stream, plan=plan_for(gpu), label=name + " level-scan")


@pytest.mark.parametrize("name", ["C1", "C2", "C4"])
def test_configs_other_mode(gpu, oracle, name):
    cfg = workloads.CONFIGS[name]
    x = workloads.make_paths(cfg)[:16]
    check(gpu, oracle, x, cfg.depth, not cfg.stream, plan=plan_for(gpu), label=name + " level-scan, other mode")


# shapes that span several workgroups along the parents, ragged last blocks, one and many chunks, several tiles per
# chunk, chunk counts that do not divide the path, more chunks than steps, one channel, depth 1, the deepest level
SHAPES = [
    (4, 16, 2, 3), (3, 9, 3, 5), (2, 40, 5, 4), (5, 7, 1, 6), (2, 12, 7, 2), (2, 12, 6, 1), (1, 130, 2, 8),
    (2, 70, 4, 4), (1, 20, 10, 5), (3, 2, 3, 4), (7, 3, 3, 3), (130, 5, 3, 4), (2, 1000, 5, 4), (1, 2100, 3, 3),
    (9, 33, 9, 3), (300, 11, 4, 4), (1, 50, 8, 4),
    # more than 10 channels: d is a run-time value and a lane owns a block of four children
    (3, 20, 11, 3), (2, 9, 12, 4), (5, 33, 13, 2), (2, 7, 20, 3), (3, 12, 64, 2), (1, 5, 256, 2), (40, 6, 17, 2), (2, 300, 11, 2),
]


@pytest.mark.parametrize("B,L,d,depth", SHAPES)
@pytest.mark.parametrize("stream", [False, True])
@pytest.mark.parametrize("chunks", [0, 1, 3, 16, 256])
def test_shapes(gpu, oracle, B, L, d, depth, stream, chunks):
    rng = np.random.default_rng(1000 * B + 10 * L + d + depth)
    x = np.cumsum(rng.normal(0, 1.0 / np.sqrt(L), size=(B, L, d)), axis=1).astype(np.float32)
    check(gpu, oracle, x, depth, stream, plan=plan_for(gpu, chunks), label="level-scan", arithmetic_bound=d > 1)


def test_against_the_level_by_level_oracle(gpu, oracle):
    rng = np.random.default_rng(77)
    x = np.cumsum(rng.normal(0, 0.2, size=(6, 45, 3)), axis=1).astype(np.float32)
    for stream in (False, True):
        got = run_gpu(gpu, x, 4, stream, plan_for(gpu, 4))
        want = oracle.signature_levelwise(x, 4, stream=stream)
        say("  level-by-level oracle, stream=%s" % stream)
        assert_parity(got, want, x, 4, stream)


def test_same_result_as_the_fused_family(gpu, oracle):
    x = workloads.make_paths("C2")
    a = run_gpu(gpu, x, 4, False, None)
    b = run_gpu(gpu, x, 4, False, plan_for(gpu))
    errs = level_errors(a, b.astype(np.float64), 5, 4)
    assert max(errs) <= 2e-5, errs


def test_reproducible_and_scratch_reuse(gpu, oracle):
    """Two calls on one context give the same bits; a smaller call after a larger one reuses the scratch tensor."""
    x = workloads.make_paths("C2")
    a = run_gpu(gpu, x, 4, False, plan_for(gpu))
    b = run_gpu(gpu, x, 4, False, plan_for(gpu))
    assert np.array_equal(a, b)
    small = x[:5, :31]
    check(gpu, oracle, small, 4, False, plan=plan_for(gpu), label="level-scan after a larger call")


def test_repeated_points(gpu, oracle):
    x = workloads.make_paths("C1").copy()
    x[:, 5] = x[:, 4]
    x[:, 9] = x[:, 8]
    check(gpu, oracle, x, 3, True, plan=plan_for(gpu, 2), label="level-scan, repeated points")


def test_rejected_plans(gpu):
    import torch
    x = torch.zeros(2, 8, 300, device="cuda")
    with pytest.raises(RuntimeError):
        gpu.signature(x, 2, plan=plan_for(gpu))           # d > 256
    x = torch.zeros(2, 8, 2, device="cuda")
    with pytest.raises(RuntimeError):
        gpu.signature(x, 9, plan=plan_for(gpu))           # depth > 8
    assert gpu.sig_plan_validate(2, 8, 2, 3, 0, plan_for(gpu, -1)) == gpu.SIG_ERR_INVALID
    assert gpu.sig_plan_validate(2, 8, 2, 3, 0, plan_for(gpu, 5)) == gpu.SIG_OK


@pytest.mark.parametrize("name,B", [("C4", 4096), ("C2", 65536)])
def test_saturated_variants_sampled(gpu, oracle, name, B):
    """The batch-saturated stream and final shapes in the launch configuration the benchmark times, checked on
    sampled paths (and every row of the batch for having been written)."""
    import torch
    cfg = workloads.CONFIGS[name]
    x = workloads.make_paths(cfg, B=B)
    say("level-scan case %s-sat B=%d" % (name, B))
    D = gpu.sig_size(cfg.d, cfg.depth)
    out = torch.full((B, cfg.L - 1, D) if cfg.stream else (B, D), float("nan"), dtype=torch.float32, device="cuda")
    gpu.signature(torch.from_numpy(x).cuda(), cfg.depth, stream=cfg.stream, plan=plan_for(gpu), out=out)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    pick = np.sort(np.random.default_rng(5).choice(B, size=32, replace=False))
    pick[0], pick[-1] = 0, B - 1
    got = out[torch.from_numpy(pick).cuda()].cpu().numpy()
    want = oracle.signature(x[pick], cfg.depth, stream=cfg.stream)
    assert_parity(got, want, x[pick], cfg.depth, cfg.stream)


@pytest.mark.parametrize("B,L,d,depth,stream", [(65536, 30, 3, 8, False), (24576, 30, 3, 8, True)])
def test_batches_whose_lower_levels_exceed_the_scratch_limit_go_in_slices(gpu, oracle, B, L, d, depth, stream):
    """The lower levels of every prefix of these batches would take 25 and 9.3 GB: the planner's own choice for
    them (no on-chip kernel) runs the family on equal slices of the batch that share 8 GiB or less.  Sampled
    paths on both sides of every slice boundary against the oracle; every row checked for having been written."""
    import torch
    rc, pl = gpu.sig_plan(None, B, L, d, depth, int(stream))
    assert rc == gpu.SIG_OK and pl.variant == gpu.SIG_VARIANT_LEVEL_SCAN
    rc, _, _, scratch = gpu.sig_plan_footprint(B, L, d, depth, int(stream), pl)
    D = gpu.sig_size(d, depth)
    per_path = (L - 1) * (D - d ** depth) * 4
    assert rc == gpu.SIG_OK and scratch <= 8 << 30 and scratch % per_path == 0
    S = scratch // per_path
    assert S < B
    rng = np.random.default_rng(B + L)
    x = np.cumsum(rng.normal(0, 1.0 / np.sqrt(L), size=(B, L, d)), axis=1).astype(np.float32)
    say("level-scan sliced batch B=%d L=%d d=%d depth=%d stream=%s slice=%d" % (B, L, d, depth, stream, S))
    out = torch.full((B, L - 1, D) if stream else (B, D), float("nan"), dtype=torch.float32, device="cuda")
    gpu.signature(torch.from_numpy(x).cuda(), depth, stream=stream, out=out)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    edges = [b for s in range(S, B, S) for b in (s - 1, s)]
    pick = np.unique(np.concatenate([[0, B - 1], edges, rng.choice(B, size=8, replace=False)]))
    got = out[torch.from_numpy(pick).cuda()].cpu().numpy()
    want = oracle.signature(x[pick], depth, stream=stream)
    assert_parity(got, want, x[pick], depth, stream)

"""GPU parity of sig_backward (through the C ABI binding) against the fp64 gradient oracle.

Gates, all at 1e-4 (the tolerance of the forward transform, applied to the gradient: the kernel's extra error
source, undoing one increment at a time in fp32, stays far below it for these path lengths):
  ||gpu - oracle||_F / ||oracle||_F over the whole gradient of a call, over every channel of it, and over the
  gradient of every single path (so that one wrong path cannot hide in a large batch);
  |gpu - oracle| <= 1e-4 x max|oracle| for every entry, at depths up to 8 (all compiled kernels; beyond that the
  sweep's reconstruction of early prefixes in fp32, S_{k-1} = S_k (x) exp(-dX_k), loses the tiny top levels of the
  first few prefixes -- relative errors above 1 at level 9 of a 22-increment path -- which the norm gates absorb but
  single entries of the gradient at the first points of a path do not: measured 1.35e-4 on (d, depth) = (2, 10)).
grad_path is poisoned with NaN before every call.
"""
import sys

import numpy as np
import pytest

from paper_2501_08455_amd import workloads

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2501_08455_amd import binding
    binding.load()
    return binding


def say(msg):
    print(msg)
    sys.stdout.flush()


def upstream(rng, B, rows, d, depth):
    """A loss gradient of moderate size on every level: level n scaled by n! so that no level drowns."""
    parts = [rng.normal(size=(B, rows, d ** n)) * float(np.prod(np.arange(1, n + 1))) for n in range(1, depth + 1)]
    return np.concatenate(parts, axis=2).astype(np.float32)


def run_backward(gpu, x, depth, stream, g):
    import torch
    ctx = gpu.default_ctx()
    xt = torch.from_numpy(x).cuda()
    out = gpu.signature(xt, depth, stream=stream)
    gt = torch.from_numpy(g).cuda()
    gx = torch.full(x.shape, float("nan"), dtype=torch.float32, device="cuda")
    rc = gpu.sig_backward(ctx, xt, depth, int(stream), out, gt, gx)
    torch.cuda.synchronize()
    return rc, gx.cpu().numpy()


def check(gpu, oracle, x, depth, stream, seed, label="", entry_gate=True):
    B, L, d = x.shape
    say("backward case %s shape=%s depth=%d stream=%s" % (label, x.shape, depth, stream))
    rng = np.random.default_rng(seed)
    g = upstream(rng, B, L - 1 if stream else 1, d, depth)
    if not stream:
        g = g[:, 0]
    rc, got = run_backward(gpu, x, depth, stream, g)
    assert rc == gpu.SIG_OK, rc
    want = oracle.signature_backward(x, depth, g, stream=stream)
    assert_gradient_parity(got, want, entry_gate)
    return got


def assert_gradient_parity(got, want, entry_gate=True):
    """The gates of the module docstring on gradients of shape [paths][points][channels]."""
    assert got.shape == want.shape and np.all(np.isfinite(got))
    d = want.shape[-1]
    got = np.asarray(got, dtype=np.float64)
    err = np.linalg.norm(got - want) / np.linalg.norm(want)
    per_channel = [np.linalg.norm(got[..., a] - want[..., a]) / np.linalg.norm(want[..., a]) for a in range(d)]
    num = np.sqrt(((got - want) ** 2).sum(axis=(1, 2)))
    den = np.sqrt((want ** 2).sum(axis=(1, 2)))
    per_path = np.where(den > 1e-30, num / np.maximum(den, 1e-30), num)
    elem = np.max(np.abs(got - want)) / np.max(np.abs(want))
    say("  rel err %.2e, worst channel %.2e, worst path %.2e (path %d), worst entry / max %.2e"
        % (err, max(per_channel), per_path.max(), int(per_path.argmax()), elem))
    assert err <= TOL and max(per_channel) <= TOL and per_path.max() <= TOL and (elem <= TOL or not entry_gate)


CASES = [
    # d, depth, B, L, stream
    (2, 3, 4, 16, False), (2, 3, 4, 16, True), (2, 3, 1000, 9, False), (2, 3, 77, 2, True),
    (4, 4, 3, 37, False), (4, 4, 64, 256, True), (4, 4, 33, 20, False), (4, 4, 5, 2, True),
    (5, 4, 128, 100, False), (5, 4, 11, 100, True), (5, 4, 7, 2, False), (5, 4, 23, 41, False),
    (5, 4, 2, 2000, False), (5, 4, 3, 333, True), (5, 4, 2600, 12, False),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(str(v) for v in c))
def test_backward_matches_oracle(gpu, oracle, case):
    d, depth, B, L, stream = case
    x = workloads.brownian_paths(B, L, d, seed=4000 + 7 * B + L)
    check(gpu, oracle, x, depth, stream, seed=B + L, label="on-chip")


BACKWARD_GRID = [(2, 2), (3, 2), (4, 2), (5, 2), (6, 2), (8, 2), (10, 2), (2, 3), (3, 3), (4, 3), (5, 3), (6, 3), (7, 3),
                 (8, 3), (10, 3), (2, 4), (3, 4), (4, 4), (5, 4), (6, 4), (7, 4), (2, 5), (3, 5), (4, 5), (5, 5),
                 (2, 6), (3, 6), (7, 2), (9, 2), (9, 3)]


@pytest.mark.parametrize("shape", BACKWARD_GRID, ids=lambda c: "-".join(str(v) for v in c))
def test_backward_shape_grid(gpu, oracle, shape):
    """Every (d, depth) with a gradient kernel: a few long paths (sweep cut in time), many short ones, stream mode."""
    d, depth = shape
    assert gpu.sig_backward_available(d, depth) == 1
    for B, L, stream in [(3, 41, False), (300, 7, False), (4, 19, True)]:
        x = workloads.brownian_paths(B, L, d, seed=8000 + 13 * d + depth + B)
        check(gpu, oracle, x, depth, stream, seed=d + depth + L, label="grid")


# shapes whose lanes per path exceed one workgroup (or whose parked sums would not fit): the sliced sweep
SLICED_GRID = [(8, 4), (10, 4), (6, 5), (4, 6), (5, 6), (10, 6), (9, 4), (7, 5), (8, 5), (9, 5), (10, 5)]


@pytest.mark.parametrize("shape", SLICED_GRID, ids=lambda c: "-".join(str(v) for v in c))
def test_backward_sliced_shapes(gpu, oracle, shape):
    d, depth = shape
    assert gpu.sig_backward_available(d, depth) == 1
    big = workloads.sig_size(d, depth) > 100000
    cases = [(2, 9, False), (3, 4, False), (2, 6, True), (1, 2, False)] if big else \
            [(3, 41, False), (40, 7, False), (4, 19, True), (2, 2, True)]
    for B, L, stream in cases:
        x = workloads.brownian_paths(B, L, d, seed=8100 + 13 * d + depth + B)
        check(gpu, oracle, x, depth, stream, seed=d + depth + L, label="sliced")


def test_backward_sliced_long_paths(gpu, oracle):
    """Long paths leave the sliced sweep less LDS for its parked sums: it parks fewer steps (down to one) before it
    hands the shape to the general sweep."""
    for d, depth, B, L in [(10, 4, 2, 1000), (8, 4, 1, 1600), (10, 4, 1, 1300)]:
        x = workloads.brownian_paths(B, L, d, seed=8400 + L)
        check(gpu, oracle, x, depth, False, seed=L, label="sliced, long path")


SEGMENTED_CASES = [
    # d, depth, B, L: few long paths in final mode, which the library cuts in time across workgroups (segment
    # signatures, their running products and pulled-back gradients, then one sweep per segment); lengths that leave
    # a ragged last segment, both kernel families, one and several paths
    (5, 4, 1, 1000), (5, 4, 3, 777), (2, 3, 2, 4001), (4, 4, 5, 500), (3, 5, 2, 600), (5, 5, 1, 300), (9, 3, 2, 450),
    (6, 4, 1, 130), (7, 4, 2, 513), (8, 4, 1, 400), (10, 4, 3, 333), (6, 5, 1, 200), (4, 6, 2, 260), (9, 4, 1, 129),
    (10, 5, 1, 150), (2, 6, 4, 2000),
]


@pytest.mark.parametrize("case", SEGMENTED_CASES, ids=lambda c: "-".join(str(v) for v in c))
def test_backward_few_long_paths_cut_in_time(gpu, oracle, case):
    d, depth, B, L = case
    x = workloads.brownian_paths(B, L, d, seed=8500 + 3 * L + d)
    check(gpu, oracle, x, depth, False, seed=L + depth, label="cut in time")


def test_backward_cut_in_time_reproducible_and_next_to_uncut_calls(gpu, oracle):
    """The segment rows live in context scratch: the same bits twice, with an uncut call and a stream call between."""
    x = workloads.brownian_paths(2, 900, 5, seed=78)
    a = check(gpu, oracle, x, 4, False, seed=5, label="cut in time, first")
    check(gpu, oracle, x[:, :40], 4, False, seed=6, label="uncut call")
    check(gpu, oracle, x[:1, :300], 4, True, seed=7, label="stream call")
    b = check(gpu, oracle, x, 4, False, seed=5, label="cut in time, again")
    np.testing.assert_array_equal(a, b)


def test_backward_sliced_reproducible_and_after_a_larger_call(gpu, oracle):
    """The per-slice sums live in context scratch: a smaller call after a larger one, and the same bits twice."""
    x = workloads.brownian_paths(6, 30, 10, seed=77)
    a = check(gpu, oracle, x, 4, False, seed=3, label="sliced, first")
    check(gpu, oracle, x[:2, :9], 4, True, seed=4, label="sliced, smaller call")
    b = check(gpu, oracle, x, 4, False, seed=3, label="sliced, again")
    np.testing.assert_array_equal(a, b)


# shapes without a compiled register kernel: the general sweep (state of a path in LDS, or in device scratch for the
# last three), one channel, depth 1, more channels than coefficients per level allow to vectorise, deep and narrow
GENERAL_SHAPES = [(11, 2), (11, 3), (7, 6), (1, 5), (12, 1), (12, 3), (3, 8), (2, 10), (20, 2), (64, 2), (3, 7), (6, 6),
                  (12, 4)]


@pytest.mark.parametrize("shape", GENERAL_SHAPES, ids=lambda c: "-".join(str(v) for v in c))
def test_backward_general_sweep(gpu, oracle, shape):
    d, depth = shape
    assert gpu.sig_backward_available(d, depth) == 0
    for B, L, stream in [(3, 23, False), (17, 5, False), (2, 11, True), (2, 2, False), (1, 2, True)]:
        x = workloads.brownian_paths(B, L, d, seed=8200 + 13 * d + depth + B)
        check(gpu, oracle, x, depth, stream, seed=d + depth + L, label="general sweep", entry_gate=depth <= 8)


def test_backward_paths_too_long_for_one_workgroup(gpu, oracle):
    """Paths whose increments exceed the LDS staging of the register kernels (here 3,500 to 20,000 points in five
    channels): final mode cuts them into time segments (also when the batch alone would fill the chip: 300 paths),
    stream mode walks them in tiles within one workgroup.  The sweep undoes one increment at a time in fp32, so its
    error grows with the length: measured against the same 1e-4 gate."""
    for B, L, stream in [(2, 5000, False), (1, 20000, False), (300, 3500, False), (1, 4000, True)]:
        x = workloads.brownian_paths(B, L, 5, seed=8300 + L)
        check(gpu, oracle, x, 4, stream, seed=L, label="long path")


@pytest.mark.parametrize("case", [(10, 4, 300, 1500, True), (8, 4, 600, 2100, True), (10, 2, 2, 60000, True),
                                  (10, 2, 2, 60000, False), (10, 3, 3, 40001, True), (5, 2, 600, 3500, True)], ids=lambda c: "-".join(str(v) for v in c))
def test_backward_walks_long_paths_in_tiles(gpu, oracle, case):
    """Paths too long for LDS where the sweep is not cut across workgroups — stream mode of the sliced shapes at a
    batch that fills the chip (checked on its first paths), and paths too long even for 32 segments in either mode:
    one workgroup walks tiles of 256 increments (ragged last tile, several paths per workgroup)."""
    d, depth, B, L, stream = case
    assert gpu.sig_backward_segments(None, B, L, d, depth, int(stream)) == 1
    if B <= 8:
        x = workloads.brownian_paths(B, L, d, seed=8600 + L)
        check(gpu, oracle, x, depth, stream, seed=L, label="tiled sweep")
        return
    # a large batch: the device sees all of it (zero upstream gradient beyond the first paths), the oracle only
    # the paths whose gradient is not trivially zero, plus one more
    import torch
    keep = 3
    x = workloads.brownian_paths(B, L, d, seed=8600 + L)
    g = np.zeros((B, L - 1, gpu.sig_size(d, depth)), dtype=np.float32)
    g[:keep] = upstream(np.random.default_rng(L), keep, L - 1, d, depth)
    rc, got = run_backward(gpu, x, depth, True, g)
    assert rc == gpu.SIG_OK and np.all(np.isfinite(got))
    want = oracle.signature_backward(x[:keep], depth, g[:keep], stream=True)
    say("  tiled sweep, %d paths, the first %d:" % (B, keep))
    assert_gradient_parity(got[:keep], want)
    assert not np.any(got[keep:])


STREAM_SEGMENTED_CASES = [
    # d, depth, B, L: stream mode, few long paths of shapes whose lanes fit a workgroup at least twice: two sweeps per
    # segment with a scan over the segments between them; lengths with ragged last segments, one and several paths,
    # paths too long for the LDS of the uncut sweep at a batch that fills the chip
    (5, 4, 1, 600), (5, 4, 3, 777), (2, 3, 2, 30001), (4, 4, 2, 1000), (3, 5, 1, 700), (5, 5, 1, 300), (6, 4, 2, 400),
    (8, 3, 1, 900), (7, 3, 2, 2500), (2, 6, 1, 1200), (10, 2, 70, 1700), (9, 3, 2, 350), (5, 4, 3, 3300),
    # the sliced shapes (lanes of a path in several workgroups: the prefix words' partial adjoints are added across slices)
    (10, 4, 1, 600), (8, 4, 2, 777), (9, 4, 1, 400), (6, 5, 1, 300), (4, 6, 2, 500), (7, 5, 1, 200), (10, 4, 3, 1500),
    (10, 5, 1, 150),
]


@pytest.mark.parametrize("case", STREAM_SEGMENTED_CASES, ids=lambda c: "-".join(str(v) for v in c))
def test_backward_stream_mode_cut_in_time(gpu, oracle, case):
    d, depth, B, L = case
    assert gpu.sig_backward_segments(None, B, L, d, depth, 1) > 1
    x = workloads.brownian_paths(B, L, d, seed=8700 + 3 * L + d)
    check(gpu, oracle, x, depth, True, seed=L + depth, label="stream, cut in time")


def test_backward_on_the_configurations(gpu, oracle):
    for name in ["C1", "C2", "C4"]:
        cfg = workloads.CONFIGS[name]
        x = workloads.make_paths(cfg)
        check(gpu, oracle, x, cfg.depth, cfg.stream, seed=31, label=name)
    # the large-signature configuration: its first path (the fp64 oracle keeps every prefix signature of a path,
    # 2 GB each, and takes most of a minute for three)
    cfg = workloads.CONFIGS["C5"]
    x = workloads.make_paths(cfg)[:1]
    check(gpu, oracle, x, cfg.depth, cfg.stream, seed=32, label="C5, first path")


def sampled_backward(gpu, oracle, x, depth, stream, pick, seed):
    """sig_backward on the whole batch `x` (upstream gradient drawn on the device), the oracle on the paths `pick`."""
    import torch
    xt = torch.from_numpy(x).cuda()
    out = gpu.signature(xt, depth, stream=stream)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    gt = torch.randn(out.shape, dtype=torch.float32, device="cuda", generator=gen)
    gx = torch.full(x.shape, float("nan"), dtype=torch.float32, device="cuda")
    assert gpu.sig_backward(gpu.default_ctx(), xt, depth, int(stream), out, gt, gx) == gpu.SIG_OK
    torch.cuda.synchronize()
    assert bool(torch.isfinite(gx).all())       # the gradient of every path of the batch was written
    idx = torch.from_numpy(np.asarray(pick)).cuda()
    want = oracle.signature_backward(x[pick], depth, gt[idx].cpu().numpy(), stream=stream)
    assert_gradient_parity(gx[idx].cpu().numpy(), want)


def test_backward_large_signature_at_the_benchmark_batch(gpu, oracle):
    """The large-signature configuration at its full batch of 16 (what bench.py times), the oracle on the first and
    the last path."""
    cfg = workloads.CONFIGS["C5"]
    x = workloads.make_paths(cfg)
    say("backward case C5, B=%d, oracle on paths 0 and %d" % (x.shape[0], x.shape[0] - 1))
    sampled_backward(gpu, oracle, x, cfg.depth, cfg.stream, [0, x.shape[0] - 1], seed=33)


def test_backward_length_scaling_configuration_at_the_benchmark_batch(gpu, oracle):
    """128 paths of 2,000 points (the sweep is cut into time segments across workgroups), the oracle on eight paths."""
    cfg = workloads.CONFIGS["C3"]
    x = workloads.make_paths(cfg)
    pick = [0, 1, 17, 63, 64, 100, 126, 127]
    say("backward case C3 literal, B=%d, oracle on paths %s" % (x.shape[0], pick))
    sampled_backward(gpu, oracle, x, cfg.depth, cfg.stream, pick, seed=34)


def test_backward_repeated_points_and_reproducible(gpu, oracle):
    x = workloads.brownian_paths(9, 30, 5, seed=12)
    x[:, 7] = x[:, 6]
    x[:, 20:23] = x[:, 19:20]
    a = check(gpu, oracle, x, 4, False, seed=5, label="repeated points")
    b = check(gpu, oracle, x, 4, False, seed=5, label="again")
    np.testing.assert_array_equal(a, b)


def test_backward_status_codes(gpu):
    import torch
    ctx = gpu.default_ctx()
    assert gpu.sig_backward_available(5, 4) == 1 and gpu.sig_backward_available(11, 2) == 0
    x = torch.zeros((2, 5, 300), device="cuda")
    out = torch.zeros((2, gpu.sig_size(300, 1)), device="cuda")
    gx = torch.zeros_like(x)
    assert gpu.sig_backward(ctx, x, 1, 0, out, out, gx) == gpu.SIG_ERR_UNSUPPORTED  # more channels than a workgroup has threads
    x5 = torch.zeros((1, 50, 5), device="cuda")
    o5 = torch.zeros((1, gpu.sig_size(5, 4)), device="cuda")
    assert gpu.sig_backward(ctx, x5[:, :1].contiguous(), 4, 0, o5, o5, torch.zeros_like(x5)) == gpu.SIG_ERR_INVALID
    assert gpu.sig_backward(None, x5, 4, 0, o5, o5, torch.zeros_like(x5)) == gpu.SIG_ERR_INVALID
    empty = torch.zeros((0, 10, 5), device="cuda")
    assert gpu.sig_backward(ctx, empty, 4, 0, o5, o5, empty) == gpu.SIG_OK
    torch.cuda.synchronize()


def test_autograd_wrapper(gpu, oracle):
    """torch.autograd through the layer alone: signature -> weighted sum, the gradient with respect to the path
    against the oracle (the full Dense -> signature -> Dense step is tests/test_gpu_training_step.py)."""
    import torch
    from paper_2501_08455_amd import autograd
    rng = np.random.default_rng(41)
    for stream in (False, True):
        x = workloads.brownian_paths(6, 30, 5, seed=90)
        xt = torch.from_numpy(x).cuda().requires_grad_(True)
        sig = autograd.signature(xt, 4, stream=stream)
        w = rng.normal(size=tuple(sig.shape)).astype(np.float32)
        (sig * torch.from_numpy(w).cuda()).sum().backward()
        torch.cuda.synchronize()
        want = oracle.signature_backward(x, 4, w, stream=stream)
        assert_gradient_parity(xt.grad.cpu().numpy(), want)


@pytest.mark.parametrize("name,B", [("C2", 65536), ("C4", 4096)])
def test_backward_saturated_variants_sampled(gpu, oracle, name, B):
    """The batch sizes bench.py times (not cut in time), checked on a sample of paths."""
    import torch
    cfg = workloads.CONFIGS[name]
    x = workloads.make_paths(cfg, B=B, seed=98)
    say("backward case %s-sat B=%d" % (name, B))
    rng = np.random.default_rng(6)
    pick = np.sort(rng.choice(B, size=64, replace=False))
    pick[0], pick[-1] = 0, B - 1
    sampled_backward(gpu, oracle, x, cfg.depth, cfg.stream, pick, seed=3)


@pytest.mark.parametrize("d,depth,L,B,stream", [
    (5, 4, 700, 5400, False),     # 25 lanes per path, four paths' increments per workgroup: walked in tiles
    (4, 4, 1200, 8300, False),    # 16 lanes per path: walked in tiles
    (4, 3, 500, 33000, False),    # four lanes per path: cut in time inside the workgroup
    (10, 2, 500, 1700, True),     # ten lanes per path, stream mode: cut in time inside the workgroup
    (5, 4, 700, 700, True),       # stream mode, 25 lanes per path: walked in tiles
    # the same kind of shape with paths short enough for the plain sweep to keep enough lanes on a CU: not cut
    (2, 6, 128, 8200, True),      # two lanes per path, stream mode (pipelined fetch would not apply: the chip is full)
    (3, 4, 256, 8200, True),      # three lanes per path, stream mode
    (5, 3, 128, 33000, False),    # five lanes per path, final mode
    (3, 3, 500, 8200, True),      # stream mode, depth 3 with too few lanes left: still cut in time
    # few-lane kernels whose LDS holds fewer paths than a workgroup has lanes for, on batches that need the plain sweep's
    # resident workgroups several times over: walked in short tiles
    (5, 3, 100, 66000, False),
    (10, 2, 100, 17000, True),
    (5, 3, 256, 16500, True),
    (6, 3, 100, 33000, False),
])
def test_backward_of_long_paths_in_a_batch_that_fills_the_chip(gpu, oracle, d, depth, L, B, stream):
    """Paths whose increments fit the staging only a few at a time, in a batch large enough to fill the chip: the
    sweep that keeps the lanes busy is taken instead of the plain one (tiles, or chunks side by side in a workgroup);
    the oracle on six paths spread over the batch."""
    x = workloads.brownian_paths(B, L, d, seed=900 + d + depth)
    pick = [0, 1, B // 3, B // 2, B - 2, B - 1]
    say("backward case d=%d depth=%d L=%d B=%d stream=%s, oracle on paths %s" % (d, depth, L, B, stream, pick))
    sampled_backward(gpu, oracle, x, depth, stream, pick, seed=70 + d)


def _random_backward_cases():
    """Seeded draws over the compiled shapes: batches from one path to a few thousand (so that workgroups end ragged,
    a CU's share of paths is split over several rounds, and both the pipelined and the plain fetch of the upstream rows
    are taken), lengths from 2 points up, both modes."""
    rng = np.random.default_rng(20250108)
    shapes = [(2, 2), (2, 3), (2, 4), (2, 5), (2, 6), (3, 2), (3, 3), (3, 4), (3, 5), (3, 6), (4, 2), (4, 3), (4, 4),
              (4, 5), (5, 2), (5, 3), (5, 4), (5, 5), (6, 2), (6, 3), (6, 4), (7, 2), (7, 3), (7, 4), (8, 2), (8, 3),
              (9, 2), (9, 3), (10, 2), (10, 3)]
    cases = []
    for i in range(60):
        d, depth = shapes[int(rng.integers(len(shapes)))]
        D = workloads.sig_size(d, depth)
        stream = bool(rng.integers(2))
        L = int(rng.choice([2, 3, 5, 9, 17, 33, 64, 100, 131, 257, 300]))
        B = int(rng.choice([1, 2, 7, 31, 100, 257, 700, 1500, 2900, 4500]))
        while B > 1 and B * (L - 1 if stream else 1) * D * 4 > 3e8:
            B //= 2
        cases.append((d, depth, L, B, stream, i))
    return cases


@pytest.mark.parametrize("d,depth,L,B,stream,seed", _random_backward_cases())
def test_backward_random_shapes(gpu, oracle, d, depth, L, B, stream, seed):
    x = workloads.brownian_paths(B, L, d, seed=4000 + seed)
    rng = np.random.default_rng(seed)
    pick = sorted(set([0, B - 1] + [int(v) for v in rng.integers(0, B, size=10)]))
    say("backward random case d=%d depth=%d L=%d B=%d stream=%s, oracle on %d paths" % (d, depth, L, B, stream, len(pick)))
    sampled_backward(gpu, oracle, x, depth, stream, pick, seed=500 + seed)

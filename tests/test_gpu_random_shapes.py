"""Seeded random shapes through the automatic plan: whatever family sig_plan picks (register kernels with any time
cutting, level-scan, HBM streaming) and whatever gradient path sig_backward takes (register, sliced, general sweep)
must meet the same gate against the fp64 oracles.  The shapes are drawn once from a fixed seed."""
import numpy as np
import pytest

from paper_2501_08455_amd import workloads
from test_gpu_parity import TOL, assert_parity, gpu, level_errors, run_gpu, say  # noqa: F401  (gpu is a fixture)
from test_gpu_backward import assert_gradient_parity, run_backward, upstream

pytestmark = pytest.mark.gpu


def draw_shapes(count, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        d = int(rng.integers(1, 13))
        depth = int(rng.integers(1, 7))
        D = workloads.sig_size(d, depth)
        if D > 30000:
            continue
        L = int(rng.choice([2, 3, 5, 8, 17, 33, 64, 100, 257, 400]))
        B = int(rng.choice([1, 2, 3, 7, 16, 65, 130, 300]))
        if B * L * D > 3e7:      # keeps the fp64 oracles (the gradient one stores every prefix) in seconds
            continue
        shapes.append((B, L, d, depth, bool(rng.integers(0, 2))))
    return shapes


SHAPES = draw_shapes(60, seed=20250108455)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda c: "-".join(str(int(v)) for v in c))
def test_random_shape(gpu, oracle, shape):
    B, L, d, depth, stream = shape
    rc, pl = gpu.sig_plan(None, B, L, d, depth, int(stream))
    assert rc == gpu.SIG_OK
    say("random shape B=%d L=%d d=%d depth=%d stream=%s plan=%s" % (B, L, d, depth, stream, pl.as_dict()))
    x = workloads.brownian_paths(B, L, d, seed=B * 1000 + L * 10 + d)
    got = run_gpu(gpu, x, depth, stream, None)
    want = oracle.signature(x, depth, stream=stream)
    assert_parity(got, want, x, depth, stream)
    g = upstream(np.random.default_rng(L + d), B, L - 1 if stream else 1, d, depth)
    if not stream:
        g = g[:, 0]
    rc, gx = run_backward(gpu, x, depth, stream, g)
    assert rc == gpu.SIG_OK
    want_g = oracle.signature_backward(x, depth, g, stream=stream)
    say("  gradient (%s):" % ("register kernel" if gpu.sig_backward_available(d, depth) else "general sweep"))
    assert_gradient_parity(gx, want_g)


def draw_long_paths(count, seed):
    """Few long paths in final mode: the shapes where the forward pass is cut into tree-joined segments and the
    reverse sweep into time segments across workgroups (lengths that leave ragged last pieces)."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        d = int(rng.integers(2, 11))
        depth = int(rng.integers(2, 7))
        D = workloads.sig_size(d, depth)
        if D > 30000:
            continue
        L = int(rng.integers(130, 3000))
        B = int(rng.choice([1, 1, 2, 3, 5, 9, 20, 40]))
        if B * L * D > 3e7:
            continue
        shapes.append((B, L, d, depth))
    return shapes


LONG_PATHS = draw_long_paths(40, seed=20250108456)


@pytest.mark.parametrize("shape", LONG_PATHS, ids=lambda c: "-".join(str(int(v)) for v in c))
def test_random_long_paths(gpu, oracle, shape):
    B, L, d, depth = shape
    rc, pl = gpu.sig_plan(None, B, L, d, depth, 0)
    assert rc == gpu.SIG_OK
    segs = gpu.sig_backward_segments(None, B, L, d, depth, 0)
    say("long paths B=%d L=%d d=%d depth=%d plan=%s gradient segments=%d" % (B, L, d, depth, pl.as_dict(), segs))
    x = workloads.brownian_paths(B, L, d, seed=B * 1000 + L * 10 + d)
    got = run_gpu(gpu, x, depth, False, None)
    assert_parity(got, oracle.signature(x, depth), x, depth, False)
    g = upstream(np.random.default_rng(L + d), B, 1, d, depth)[:, 0]
    rc, gx = run_backward(gpu, x, depth, False, g)
    assert rc == gpu.SIG_OK
    want_g = oracle.signature_backward(x, depth, g)
    assert_gradient_parity(gx, want_g)

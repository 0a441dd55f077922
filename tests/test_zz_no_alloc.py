"""sig_compute_noalloc (the entry point with the fixed scratch array, for callers that cannot allocate) against
sig_compute through the C ABI: same mapping and kernels, so the two outputs agree bit for bit.  Two calls in a row
on shapes whose mapping needs scratch, the second smaller than the first, then the level-scan family (whose final
mode keeps its lower levels in scratch), a shape that needs no scratch, and a shape that is refused."""
import sys

import numpy as np
import pytest

from paper_2501_08455_amd import workloads

pytestmark = pytest.mark.gpu


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


def both(gpu, x, depth, stream):
    """(status, noalloc output, sig_compute output) on the same input; the noalloc call comes first and its output
    buffer is poisoned, so nothing it returns can come from the other call."""
    import torch
    xt = torch.from_numpy(x).cuda()
    B, L, d = x.shape
    D = gpu.sig_size(d, depth)
    shape = (B, L - 1, D) if stream else (B, D)
    ctx = gpu.default_ctx()
    out_fixed = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    rc = gpu.sig_compute_noalloc(ctx, xt, depth, int(stream), out_fixed)
    if rc != gpu.SIG_OK:
        return rc, None, None
    out_ref = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    assert gpu.sig_compute(ctx, xt, depth, int(stream), out_ref) == gpu.SIG_OK
    torch.cuda.synchronize()
    return rc, out_fixed.cpu().numpy(), out_ref.cpu().numpy()


def test_noalloc_matches_sig_compute_twice_in_a_row(gpu, oracle):
    # 128 paths of 2,000 points, (5,4): four time segments joined by a second launch (1.6 MB of partial rows);
    # then 16 paths of 1,000 points of the same kernel, which reuses the front of the same array
    for (B, L, d, depth, seed) in [(128, 2000, 5, 4, 11), (16, 1000, 5, 4, 12)]:
        rc, pl = gpu.sig_plan(gpu.default_ctx(), B, L, d, depth, 0)
        assert rc == gpu.SIG_OK and pl.segments > 1, pl.as_dict()   # the shape does use scratch
        say("noalloc case B=%d L=%d d=%d depth=%d plan=%s" % (B, L, d, depth, pl.as_dict()))
        x = workloads.brownian_paths(B, L, d, seed=seed)
        rc, got, ref = both(gpu, x, depth, False)
        assert rc == gpu.SIG_OK
        assert np.all(np.isfinite(got))
        assert np.array_equal(got, ref)
        # and against the oracle, to the tolerance of the parity tests, on a few paths
        pick = [0, B // 2, B - 1]
        want = oracle.signature(x[pick], depth, stream=False)
        start = 0
        for n in range(1, depth + 1):
            sl = slice(start, start + d ** n)
            err = np.linalg.norm(got[pick][:, sl] - want[:, sl]) / np.linalg.norm(want[:, sl])
            assert err <= 1e-4, (n, err)
            start += d ** n


def test_noalloc_level_scan_and_no_scratch_shapes(gpu):
    # (7,6) has no register kernel: level-scan family, final mode keeps levels 1..5 of every prefix in scratch
    # (4 * 29 * 19,607 floats = 9.1 MB); then a smaller batch of it; then shapes that need no scratch at all
    for (B, L, d, depth, stream, seed) in [(4, 30, 7, 6, False, 21), (3, 17, 7, 6, False, 22), (64, 100, 5, 4, False, 23),
                                           (16, 64, 4, 4, True, 24), (5, 9, 7, 6, True, 25)]:
        say("noalloc case B=%d L=%d d=%d depth=%d stream=%s" % (B, L, d, depth, stream))
        x = workloads.brownian_paths(B, L, d, seed=seed)
        rc, got, ref = both(gpu, x, depth, stream)
        assert rc == gpu.SIG_OK
        assert np.all(np.isfinite(got))
        assert np.array_equal(got, ref)


def test_noalloc_refuses_what_does_not_fit(gpu):
    # level-scan family, final mode: 64 * 199 * 19,607 floats = 1 GB of scratch, beyond the fixed 16 MiB
    import torch
    B, L, d, depth = 64, 200, 7, 6
    rc, pl = gpu.sig_plan(gpu.default_ctx(), B, L, d, depth, 0)
    assert rc == gpu.SIG_OK and pl.variant == gpu.SIG_VARIANT_LEVEL_SCAN
    xt = torch.zeros((B, L, d), dtype=torch.float32, device="cuda")
    out = torch.zeros((B, gpu.sig_size(d, depth)), dtype=torch.float32, device="cuda")
    assert gpu.sig_compute_noalloc(gpu.default_ctx(), xt, depth, 0, out) == gpu.SIG_ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0   # nothing was launched
    assert gpu.sig_compute_noalloc(None, xt, depth, 0, out) == gpu.SIG_ERR_INVALID

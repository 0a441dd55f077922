"""sig_autotune: measures candidate mappings of a shape on the device and the context remembers the fastest.
Whatever it picks must give the oracle's result, be what sig_plan then reports, and not be slower than the
planner's own choice measured the same way."""
import numpy as np
import pytest

from paper_2501_08455_amd import workloads
from test_gpu_parity import TOL, gpu, level_errors, say  # noqa: F401  (gpu is a fixture)

pytestmark = pytest.mark.gpu


def time_calls(gpu, ctx, xt, depth, stream, out, plan=None, reps=30, rounds=5):
    """Microseconds per call: the fastest of several rounds of back-to-back calls (a round now and then takes a
    multiple of the others on a box that has just freed or mapped memory; the comparison is about the kernels)."""
    import torch
    call = gpu.bind_compute(ctx, xt, depth, int(stream), out, plan=plan)
    for _ in range(10):
        assert call() == gpu.SIG_OK
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(rounds):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / reps * 1e3)
    return best


@pytest.mark.parametrize("B,L,d,depth,stream", [(128, 100, 5, 4, False), (16, 256, 2, 4, True), (128, 500, 10, 2, True),
                                                 (4, 300, 9, 3, False), (3, 40, 11, 2, False), (64, 256, 4, 4, True)])
def test_autotune_picks_a_correct_and_not_slower_plan(gpu, oracle, B, L, d, depth, stream):
    import torch
    ctx = gpu.sig_create()
    try:
        rc, before = gpu.sig_plan(ctx, B, L, d, depth, int(stream))
        assert rc == gpu.SIG_OK
        x = workloads.brownian_paths(B, L, d, seed=300 + B + L)
        xt = torch.from_numpy(x).cuda()
        D = gpu.sig_size(d, depth)
        out = torch.full((B, L - 1, D) if stream else (B, D), float("nan"), device="cuda")
        t_before = time_calls(gpu, ctx, xt, depth, stream, out, plan=before)
        rc, chosen, us = gpu.sig_autotune(ctx, B, L, d, depth, int(stream))
        assert rc == gpu.SIG_OK and us > 0
        rc, after = gpu.sig_plan(ctx, B, L, d, depth, int(stream))
        assert rc == gpu.SIG_OK and after.as_dict() == chosen.as_dict()
        assert gpu.sig_plan_validate(B, L, d, depth, int(stream), chosen) == gpu.SIG_OK
        # another shape is not affected
        rc, other = gpu.sig_plan(ctx, B + 1, L, d, depth, int(stream))
        rc2, other_ref = gpu.sig_plan(None, B + 1, L, d, depth, int(stream))
        assert other.as_dict() == other_ref.as_dict()
        out.fill_(float("nan"))
        assert gpu.sig_compute(ctx, xt, depth, int(stream), out) == gpu.SIG_OK   # uses the remembered mapping
        torch.cuda.synchronize()
        errs = level_errors(out.cpu().numpy(), oracle.signature(x, depth, stream=stream), d, depth)
        assert max(errs) <= TOL
        t_after = time_calls(gpu, ctx, xt, depth, stream, out)
        say("  autotune B=%d L=%d (%d,%d) stream=%s: planner %s %.1f us -> tuned %s %.1f us (reported %.1f)"
            % (B, L, d, depth, stream, before.as_dict(), t_before, chosen.as_dict(), t_after, us))
        assert t_after <= 1.15 * t_before + 1.0
    finally:
        torch.cuda.synchronize()
        gpu.sig_destroy(ctx)


def test_autotune_status_codes(gpu):
    ctx = gpu.sig_create()
    try:
        assert gpu.sig_autotune(None, 4, 16, 2, 3, 0)[0] == gpu.SIG_ERR_INVALID
        assert gpu.sig_autotune(ctx, 0, 16, 2, 3, 0)[0] == gpu.SIG_ERR_INVALID
        assert gpu.sig_autotune(ctx, 4, 1, 2, 3, 0)[0] == gpu.SIG_ERR_INVALID
        assert gpu.sig_autotune(ctx, 4, 16, 2, 3, 2)[0] == gpu.SIG_ERR_INVALID
        # more shapes than the context remembers: the oldest is replaced, every call still succeeds
        for B in range(1, 70):
            assert gpu.sig_autotune(ctx, B, 9, 2, 2, 0)[0] == gpu.SIG_OK
    finally:
        gpu.sig_destroy(ctx)

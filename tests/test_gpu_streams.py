"""Stream semantics of the C ABI on the GPU: every entry point enqueues on the stream it is given and returns
without synchronising, multi-launch plans stay ordered on that stream, and a call whose scratch is already
sized can be captured into a HIP graph and replayed (results compared with eager calls and with the oracle).
"""
import numpy as np
import pytest

from paper_2501_08455_amd import workloads
from test_gpu_parity import TOL, gpu, level_errors, say  # noqa: F401  (gpu is a fixture)

pytestmark = pytest.mark.gpu


def plans(gpu):
    return {
        "auto": None,
        "two segments (fold + join launches)": gpu.make_plan(gpu.SIG_VARIANT_ON_CHIP, prefix_depth=2, chunks=4, segments=2),
        "level-scan (one launch per level)": gpu.make_plan(gpu.SIG_VARIANT_LEVEL_SCAN, chunks=0),
        "HBM streaming": gpu.make_plan(gpu.SIG_VARIANT_HBM_STREAMING, prefix_depth=1),
    }


def test_calls_on_a_side_stream(gpu, oracle):
    import torch
    x = workloads.brownian_paths(40, 400, 5, seed=91)
    want = oracle.signature(x, 4)
    side = torch.cuda.Stream()           # default priority
    ctx = gpu.sig_create()
    try:
        xt = torch.from_numpy(x).cuda()
        torch.cuda.synchronize()
        for label, plan in plans(gpu).items():
            out = torch.full((40, gpu.sig_size(5, 4)), float("nan"), device="cuda")
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                assert gpu.sig_compute(ctx, xt, 4, 0, out, stream=side, plan=plan) == gpu.SIG_OK
                # a consumer on the same stream sees the finished result without any host synchronisation
                total = out.sum()
            side.synchronize()
            errs = level_errors(out.cpu().numpy(), want, 5, 4)
            say("  side stream, %s: %s" % (label, " ".join("%.2e" % e for e in errs)))
            assert max(errs) <= TOL and bool(torch.isfinite(total))
    finally:
        torch.cuda.synchronize()
        gpu.sig_destroy(ctx)


def test_backward_on_a_side_stream(gpu, oracle):
    import torch
    side = torch.cuda.Stream()
    ctx = gpu.sig_create()
    try:
        # the second shape takes the two-launch sliced sweep, the third the sweep cut into time segments (nine launches)
        for d, depth, B, L in [(5, 4, 9, 60), (10, 4, 3, 20), (8, 4, 2, 300)]:
            x = workloads.brownian_paths(B, L, d, seed=92 + d)
            g = np.random.default_rng(d).normal(size=(B, gpu.sig_size(d, depth))).astype(np.float32)
            want = oracle.signature_backward(x, depth, g)
            xt, gt = torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda()
            out = torch.empty((B, gpu.sig_size(d, depth)), device="cuda")
            gx = torch.full(x.shape, float("nan"), device="cuda")
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                assert gpu.sig_compute(ctx, xt, depth, 0, out, stream=side) == gpu.SIG_OK
                assert gpu.sig_backward(ctx, xt, depth, 0, out, gt, gx, stream=side) == gpu.SIG_OK
            side.synchronize()
            got = gx.cpu().numpy()
            err = np.linalg.norm(got - want) / np.linalg.norm(want)
            say("  backward on a side stream (%d, %d): %.2e" % (d, depth, err))
            assert err <= TOL
    finally:
        torch.cuda.synchronize()
        gpu.sig_destroy(ctx)


def test_graph_capture_and_replay(gpu, oracle):
    """The calls allocate nothing once the context's scratch is sized, so they can be captured.  Every replay is
    checked against the eager result, with new input values and eager work between the replays."""
    import torch
    B, L, d, depth = 24, 300, 5, 4
    ctx = gpu.sig_create()
    try:
        xs = [workloads.brownian_paths(B, L, d, seed=93 + i) for i in range(3)]
        xt = torch.from_numpy(xs[0]).cuda()
        for label, plan in plans(gpu).items():
            out = torch.zeros((B, gpu.sig_size(d, depth)), device="cuda")
            # eager call first: sizes the scratch (no allocation may happen under capture)
            assert gpu.sig_compute(ctx, xt, depth, 0, out, plan=plan) == gpu.SIG_OK
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                rc = gpu.sig_compute(ctx, xt, depth, 0, out, plan=plan)
            assert rc == gpu.SIG_OK
            for i, x in enumerate(xs):
                xt.copy_(torch.from_numpy(x).cuda())
                out.fill_(float("nan"))
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                replayed = out.clone()
                assert gpu.sig_compute(ctx, xt, depth, 0, out, plan=plan) == gpu.SIG_OK
                torch.cuda.synchronize()
                assert torch.equal(replayed, out), (label, i)
                errs = level_errors(replayed.cpu().numpy(), oracle.signature(x, depth), d, depth)
                assert max(errs) <= TOL
            say("  graph replay, %s: three replays equal the eager calls bit for bit" % label)
            xt.copy_(torch.from_numpy(xs[0]).cuda())
    finally:
        torch.cuda.synchronize()
        gpu.sig_destroy(ctx)


def test_graph_capture_of_the_paths_cut_in_time(gpu, oracle):
    """The multi-launch paths for few long paths — forward segments joined in device memory (six launches here) and
    the gradient cut into time segments (nine) — captured together and replayed with new inputs."""
    import torch
    B, L, d, depth = 2, 900, 10, 4
    D = gpu.sig_size(d, depth)
    ctx = gpu.sig_create()
    try:
        rc, pl = gpu.sig_plan(ctx, B, L, d, depth, 0)
        assert rc == gpu.SIG_OK and pl.variant == gpu.SIG_VARIANT_ON_CHIP and pl.segments >= 4
        assert gpu.sig_backward_segments(ctx, B, L, d, depth, 0) > 1
        xs = [workloads.brownian_paths(B, L, d, seed=96 + i) for i in range(3)]
        g = np.random.default_rng(5).normal(size=(B, D)).astype(np.float32)
        xt, gt = torch.from_numpy(xs[0]).cuda(), torch.from_numpy(g).cuda()
        out, gx = torch.zeros((B, D), device="cuda"), torch.zeros(xs[0].shape, device="cuda")

        def both():
            assert gpu.sig_compute(ctx, xt, depth, 0, out) == gpu.SIG_OK
            assert gpu.sig_backward(ctx, xt, depth, 0, out, gt, gx) == gpu.SIG_OK

        both()   # sizes the scratch
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            both()
        for i, x in enumerate(xs):
            xt.copy_(torch.from_numpy(x).cuda())
            out.fill_(float("nan"))
            gx.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            r_out, r_gx = out.clone(), gx.clone()
            both()
            torch.cuda.synchronize()
            assert torch.equal(r_out, out) and torch.equal(r_gx, gx), i
            assert max(level_errors(r_out.cpu().numpy(), oracle.signature(x, depth), d, depth)) <= TOL
            want = oracle.signature_backward(x, depth, g)
            assert np.linalg.norm(r_gx.cpu().numpy() - want) / np.linalg.norm(want) <= TOL
        say("  graph replay, paths cut in time: three replays equal the eager calls bit for bit")
    finally:
        torch.cuda.synchronize()
        gpu.sig_destroy(ctx)


def test_pointers_that_are_only_float_aligned(gpu, oracle):
    """The ABI asks for float32 arrays, not for 16-byte alignment: every family, and the gradient, with path, output and
    gradient buffers that start 4 bytes past a 16-byte boundary."""
    import torch

    def shifted(shape, fill=None):
        n = int(np.prod(shape))
        raw = torch.empty(n + 1, dtype=torch.float32, device="cuda")
        view = raw[1:].view(*shape)
        assert view.data_ptr() % 16 == 4
        if fill is not None:
            view.copy_(torch.from_numpy(fill))
        return view

    ctx = gpu.default_ctx()
    cases = [("C1", None), ("C2", None), ("C4", None),
             ("C2", gpu.make_plan(gpu.SIG_VARIANT_LEVEL_SCAN, chunks=0)), ("C4", gpu.make_plan(gpu.SIG_VARIANT_LEVEL_SCAN, chunks=0)),
             ("C4", gpu.make_plan(gpu.SIG_VARIANT_HBM_STREAMING, prefix_depth=1)),
             ("C2", gpu.make_plan(gpu.SIG_VARIANT_ON_CHIP, prefix_depth=2, chunks=4, segments=2))]
    for name, plan in cases:
        cfg = workloads.CONFIGS[name]
        x = workloads.make_paths(cfg)[:16]
        B, L, d = x.shape
        D = gpu.sig_size(d, cfg.depth)
        xt = shifted(x.shape, x)
        out = shifted((B, L - 1, D) if cfg.stream else (B, D))
        out.fill_(float("nan"))
        assert gpu.sig_compute(ctx, xt, cfg.depth, int(cfg.stream), out, plan=plan) == gpu.SIG_OK
        torch.cuda.synchronize()
        errs = level_errors(out.cpu().numpy(), oracle.signature(x, cfg.depth, stream=cfg.stream), d, cfg.depth)
        say("  shifted pointers, %s, %s: %s" % (name, "auto" if plan is None else "variant %d" % plan.variant,
                                                " ".join("%.2e" % e for e in errs)))
        assert max(errs) <= TOL
    # gradient: register kernel (5, 4), sliced sweep (10, 4), general sweep (11, 2), sweep cut into time segments
    for d, depth, B, L, stream in [(5, 4, 9, 60, False), (4, 4, 5, 40, True), (10, 4, 3, 20, False), (11, 2, 4, 15, True),
                                   (10, 4, 1, 200, False), (6, 4, 2, 301, False)]:
        x = workloads.brownian_paths(B, L, d, seed=95 + d)
        D = gpu.sig_size(d, depth)
        rows = (B, L - 1, D) if stream else (B, D)
        g = np.random.default_rng(d).normal(size=rows).astype(np.float32)
        xt, gt, out, gx = shifted(x.shape, x), shifted(rows, g), shifted(rows), shifted(x.shape)
        gx.fill_(float("nan"))
        assert gpu.sig_compute(ctx, xt, depth, int(stream), out) == gpu.SIG_OK
        assert gpu.sig_backward(ctx, xt, depth, int(stream), out, gt, gx) == gpu.SIG_OK
        torch.cuda.synchronize()
        want = oracle.signature_backward(x, depth, g, stream=stream)
        err = np.linalg.norm(gx.cpu().numpy() - want) / np.linalg.norm(want)
        say("  shifted pointers, gradient (%d, %d): %.2e" % (d, depth, err))
        assert err <= TOL

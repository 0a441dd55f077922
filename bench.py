"""Benchmark of the signature transform on one MI355X.

One "step" is one sig_compute call over one batch that already sits in HBM.  The headline
workload is the second benchmark configuration (128 paths, 100 points, 5 channels, depth 4,
final signature); the other configurations and their batch-saturated variants are reported in
`all_configs` of the same JSON line.  The fp64 CPU oracle is timed beside it as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3   # MI355X vector fp32, published
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E, published

PROFILES = os.path.join(ROOT, "profiles")


def measured_traffic(workload, plan):
    """HBM bytes per launch of the call's dominant kernel as the counters read them (rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE, scaled by the copy kernel of the same run), from profiles/hbm_traffic.md -- but only if that profile
    was taken with the plan this run uses; otherwise None (the figure would describe another launch)."""
    path = os.path.join(PROFILES, "hbm_traffic.md")
    if not os.path.exists(path) or plan is None:
        return None
    want = json.dumps(plan, sort_keys=True)
    best = None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) < 6 or cells[0] != workload:
            continue
        if cells[2].strip("`") != want:
            continue
        try:
            rd, wr = (float(v) for v in cells[5].split(" + "))
        except ValueError:
            continue
        if best is None or rd + wr > best:
            best = rd + wr
    return best


def time_calls(binding, ctx, xt, depth, stream_flag, out, steps, warmup, plan=None):
    """Mean milliseconds per sig_compute call over `steps` back-to-back calls, from HIP events on the
    stream the kernels are launched on (torch's current stream) and from the host clock."""
    import torch
    call = binding.bind_compute(ctx, xt, depth, stream_flag, out, plan=plan)  # arguments marshalled once
    for _ in range(warmup):
        rc = call()
        assert rc == 0, rc
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        rc = call()
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert rc == 0, rc
    return e0.elapsed_time(e1) / steps, (t1 - t0) * 1e3 / steps


def algorithmic_work(cfg, B, workloads):
    """(flops, bytes) of one call: fused Horner steps, and path read once + output written once."""
    K = cfg.L - 1
    D = workloads.sig_size(cfg.d, cfg.depth)
    flops = 2.0 * workloads.fused_fma_per_step(cfg.d, cfg.depth) * B * K
    rows = K if cfg.stream else 1
    nbytes = 4.0 * (B * cfg.L * cfg.d + B * rows * D)
    return flops, nbytes, D, rows


def roofline(flops, nbytes, ms, traffic=None):
    """Roofline entry for a call lasting `ms`: the bound is the one whose ideal time is larger."""
    t_alu = flops / (PEAK_FP32_TFLOPS * 1e12)
    t_hbm = nbytes / (PEAK_HBM_GBS * 1e9)
    if t_alu >= t_hbm:
        ach = flops / (ms * 1e-3) / 1e12
        return {"bound": "alu", "achieved": ach, "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_FP32_TFLOPS, "traffic": traffic}
    ach = nbytes / (ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": ach / PEAK_HBM_GBS, "traffic": traffic}


def bench_config(binding, workloads, ctx, cfg, B, steps, warmup, plan=None, label=""):
    import torch
    x = workloads.make_paths(cfg, B=B)
    xt = torch.from_numpy(x).cuda()
    flops, nbytes, D, rows = algorithmic_work(cfg, B, workloads)
    out = torch.empty((B, rows, D) if cfg.stream else (B, D), dtype=torch.float32, device="cuda")
    ms_ev, ms_wall = time_calls(binding, ctx, xt, cfg.depth, int(cfg.stream), out, steps, warmup, plan=plan)
    if plan is None:
        rc, pl = binding.sig_plan(ctx, B, cfg.L, cfg.d, cfg.depth, int(cfg.stream))
    else:
        pl = plan
    res = {"workload": "%s B=%d L=%d d=%d depth=%d %s%s" % (cfg.name, B, cfg.L, cfg.d, cfg.depth,
                                                            "stream" if cfg.stream else "final", label),
           "ms_per_step": ms_ev, "ms_per_step_host_clock": ms_wall, "steps": steps,
           "paths_per_s": B / (ms_ev * 1e-3), "terms_per_s": B * rows * D / (ms_ev * 1e-3),
           "roofline": roofline(flops, nbytes, ms_ev, None),
           "algorithmic": {"flops": flops, "bytes": nbytes}, "plan": pl.as_dict()}
    res["roofline"]["traffic"] = measured_traffic(res["workload"], res["plan"])
    if plan is not None and plan.variant == binding.SIG_VARIANT_HBM_STREAMING:
        # the state-in-HBM design reads and writes every coefficient once per increment: its own byte count
        design_bytes = 8.0 * D * B * (cfg.L - 1)
        ach = design_bytes / (ms_ev * 1e-3) / 1e9
        res["roofline"] = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": ach / PEAK_HBM_GBS, "traffic": None,
                           "note": "bytes of the state-in-HBM design (8 B per coefficient and increment); the HBM "
                                   "counters read the same amount (profiles/sig_hbm_streaming_C5.md)"}
    if plan is not None and plan.variant == binding.SIG_VARIANT_LEVEL_SCAN:
        # the level-by-level design keeps the lower levels of every prefix in memory: per path and step it writes
        # level n once (all levels in stream mode, all but the top one in final mode) and level n's launch reads
        # the distinct coefficients of levels 1 .. n-1 once.  (The kernels of the stream mode write the lower levels
        # twice, into dense tensors and into the rows, and read them twice where a level is cut in time; those
        # bytes are the kernels' own and are not counted here.)
        d, N, K = cfg.d, cfg.depth, cfg.L - 1
        reads = sum(d ** m for n in range(2, N + 1) for m in range(1, n))
        writes = D if cfg.stream else D - d ** N
        design_bytes = 4.0 * B * (K * (reads + writes) + cfg.L * d + (0 if cfg.stream else D))
        ach = design_bytes / (ms_ev * 1e-3) / 1e9
        res["roofline"] = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": ach / PEAK_HBM_GBS, "traffic": None,
                           "note": "bytes of the level-by-level design of Section 3.2 (lower levels of every prefix "
                                   "written once and read once per level above); what the HBM counters read is in "
                                   "profiles/sig_level_scan_*.md"}
    del xt, out
    return res


def backward_work(cfg, B, workloads):
    """(flops, bytes) of one sig_backward call.  Per increment and path: undoing the increment is one fused
    step (2 F flops); the transposed step spends 2 FMAs per top-of-chain coefficient (sum_n d^n of them) and
    3 FMAs + 1 add per inner chain coefficient (F - sum_n d^n of them).  Bytes: path, final signature and
    upstream gradient read once, gradient written once."""
    K = cfg.L - 1
    d, N = cfg.d, cfg.depth
    D = workloads.sig_size(d, N)
    F = workloads.fused_fma_per_step(d, N)
    flops = (2.0 * F + 4.0 * D + 7.0 * (F - D)) * B * K
    rows = K if cfg.stream else 1
    nbytes = 4.0 * (2 * B * cfg.L * d + B * D + B * rows * D)
    return flops, nbytes


def bench_backward(binding, workloads, ctx, cfg, B, steps, warmup, seed=None):
    """Time sig_backward on the named configuration (forward result and upstream gradient resident in HBM)."""
    import torch
    x = workloads.make_paths(cfg, B=B, seed=seed)
    xt = torch.from_numpy(x).cuda()
    D = workloads.sig_size(cfg.d, cfg.depth)
    rows = cfg.L - 1 if cfg.stream else 1
    out = torch.empty((B, rows, D) if cfg.stream else (B, D), dtype=torch.float32, device="cuda")
    assert binding.sig_compute(ctx, xt, cfg.depth, int(cfg.stream), out) == binding.SIG_OK
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    gout = torch.randn(out.shape, dtype=torch.float32, device="cuda", generator=gen)
    gx = torch.empty_like(xt)
    call = binding.bind_backward(ctx, xt, cfg.depth, int(cfg.stream), out, gout, gx)
    for _ in range(warmup):
        rc = call()
        if rc != binding.SIG_OK:
            raise binding.SigError(rc, "sig_backward")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        call()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    flops, nbytes = backward_work(cfg, B, workloads)
    res = {"workload": "%s B=%d L=%d d=%d depth=%d %s, gradient with respect to the path" % (
               cfg.name, B, cfg.L, cfg.d, cfg.depth, "stream" if cfg.stream else "final"),
           "ms_per_step": ms, "steps": steps, "paths_per_s": B / (ms * 1e-3),
           "roofline": roofline(flops, nbytes, ms), "algorithmic": {"flops": flops, "bytes": nbytes}}
    del xt, out, gout, gx
    return res


# The rows of the paper's Table 1 (direct signature computation on GPU): batch, length, depth and the paper's own
# "KS GPU" time in milliseconds on an RTX 4090.  The paper does not state the channel count of that table; d = 5
# (the channel count of the headline configuration) is used here, so the two columns are context, not a comparison.
TABLE1_ROWS = [(32, 100, 4, 0.1312), (64, 100, 4, 0.1424), (128, 100, 4, 0.1785), (256, 100, 4, 0.1833),
               (512, 100, 4, 0.2621), (128, 50, 4, 0.1399), (128, 200, 4, 0.1798), (128, 500, 4, 0.5718),
               (128, 1000, 4, 0.5417), (128, 100, 2, 0.1689), (128, 100, 3, 0.1712), (128, 100, 5, 0.1585),
               (128, 100, 6, 0.2903)]


def table1(binding, workloads, ctx, d=5):
    """Time sig_compute (final signature) on the shapes of the paper's Table 1."""
    import torch
    rows = []
    tuned_ctx = binding.sig_create()
    for B, L, depth, paper_ms in TABLE1_ROWS:
        x = torch.from_numpy(workloads.brownian_paths(B, L, d, seed=1000 + B + L + depth)).cuda()
        out = torch.empty((B, workloads.sig_size(d, depth)), dtype=torch.float32, device="cuda")
        ms, _ = time_calls(binding, ctx, x, depth, 0, out, 500, 300)
        rc, pl = binding.sig_plan(ctx, B, L, d, depth, 0)
        # the same shape after sig_autotune (a context of its own, so that the planner's figure above stays the planner's)
        rc_t, tuned, _ = binding.sig_autotune(tuned_ctx, B, L, d, depth, 0)
        ms_tuned, _ = time_calls(binding, tuned_ctx, x, depth, 0, out, 500, 300) if rc_t == binding.SIG_OK else (None, None)
        rows.append({"batch": B, "length": L, "depth": depth, "channels": d, "ms": ms,
                     "paper_ks_gpu_ms_rtx4090": paper_ms, "plan": pl.as_dict(),
                     "ms_autotuned": ms_tuned, "plan_autotuned": tuned.as_dict() if rc_t == binding.SIG_OK else None})
        del x, out
    binding.sig_destroy(tuned_ctx)
    return rows


def memory_wall_shape(binding, workloads, ctx):
    """The shape the paper names as the memory wall of its level-by-level formulation (Section 3.5, limitations:
    batch 128, length 500, 10 channels, depth 4, more than 700 million intermediate values): forward and gradient
    here, with the device scratch each call needs."""
    import torch
    B, L, d, depth = 128, 500, 10, 4
    x = torch.from_numpy(workloads.brownian_paths(B, L, d, seed=1500)).cuda()
    out = torch.empty((B, workloads.sig_size(d, depth)), dtype=torch.float32, device="cuda")
    ms, _ = time_calls(binding, ctx, x, depth, 0, out, 200, 100)
    rc, pl = binding.sig_plan(ctx, B, L, d, depth, 0)
    cfg = workloads.Config("memory wall", B, L, d, depth, False, "normal")
    grad = bench_backward(binding, workloads, ctx, cfg, B, 50, 20, seed=1500)
    partial = B * pl.segments * workloads.sig_size(d, depth) * 4 if pl.segments > 1 else 0
    return {"batch": B, "length": L, "channels": d, "depth": depth, "ms_forward": ms, "plan": pl.as_dict(),
            "forward_scratch_bytes": partial, "ms_gradient": grad["ms_per_step"],
            "paper_intermediate_values": "more than 700 million (2.8 GB in fp32)"}


STREAM_GRID_SHAPES = [(2, 3), (2, 4), (2, 6), (3, 3), (3, 4), (3, 5), (4, 3), (4, 4), (4, 5), (5, 2), (5, 3), (5, 4),
                      (5, 5), (6, 3), (6, 4), (7, 3), (8, 3), (8, 4), (9, 3), (10, 2), (10, 3), (10, 4)]


def stream_families(binding, workloads, ctx):
    """Stream mode at small and medium batch: the planner's choice next to the level-scan family forced by plan,
    on a grid of shapes (the measurements behind the planner's rule for few paths)."""
    import torch
    rows = []
    ls_plan = binding.make_plan(binding.SIG_VARIANT_LEVEL_SCAN, chunks=0)
    for d, depth in STREAM_GRID_SHAPES:
        D = workloads.sig_size(d, depth)
        for L in (100, 256, 500):
            for B in (1, 16, 128, 1024):
                if B * (L - 1) * D * 4 > 1.5e9:
                    continue
                x = torch.from_numpy(workloads.brownian_paths(B, L, d, seed=1)).cuda()
                out = torch.empty((B, L - 1, D), dtype=torch.float32, device="cuda")
                steps, warm = (10, 3) if B * L * D > 2e8 else (60, 20)
                rc, pl = binding.sig_plan(ctx, B, L, d, depth, 1)
                ms_auto, _ = time_calls(binding, ctx, x, depth, 1, out, steps, warm)
                ms_ls, _ = time_calls(binding, ctx, x, depth, 1, out, steps, warm, plan=ls_plan)
                rows.append({"channels": d, "depth": depth, "length": L, "batch": B,
                             "planner": "level-scan" if pl.variant == binding.SIG_VARIANT_LEVEL_SCAN else "on-chip",
                             "us_auto": ms_auto * 1e3, "us_level_scan": ms_ls * 1e3})
                del x, out
    return rows


TRAIN_SAMPLES = 12765   # size of the training set of the paper's Section 4.2
TRAIN_BATCH = 128


def training_step(workloads, L, d, depth, steps, warmup):
    """The paper's model (Section 4.2, Eq. 11): Dense(20 -> d) with tanh, signature of depth `depth`, Dense(D -> 10), mean
    squared error, plain gradient descent; synthetic inputs of the stated shape (12,765 samples of L points in 20
    channels, batches of 128 -- so the last batch of an epoch is ragged: 12,765 = 99 x 128 + 93).  The two Dense layers are
    torch (rocBLAS / hipBLASLt GEMMs); the signature layer and its gradient are libsig's kernels.  The paper does not name
    the activation; tanh is used here.  Reports one step at batch 128 and one whole epoch (100 steps over the set)."""
    import torch
    from paper_2501_08455_amd import autograd
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    D = workloads.sig_size(d, depth)
    X = torch.randn((TRAIN_SAMPLES, L, 20), device="cuda", generator=gen).cumsum(1) * (1.0 / L) ** 0.5
    Y = torch.randn((TRAIN_SAMPLES, 10), device="cuda", generator=gen)
    W1 = (torch.randn((20, d), device="cuda", generator=gen) * 0.2).requires_grad_(True)
    b1 = torch.zeros(d, device="cuda", requires_grad=True)
    W2 = (torch.randn((D, 10), device="cuda", generator=gen) * 0.05).requires_grad_(True)
    b2 = torch.zeros(10, device="cuda", requires_grad=True)
    params = [W1, b1, W2, b2]

    def one_step(lo, hi):
        Z = torch.tanh(X[lo:hi] @ W1 + b1)
        S = autograd.signature(Z, depth)
        loss = ((S @ W2 + b2 - Y[lo:hi]) ** 2).mean()
        grads = torch.autograd.grad(loss, params)
        with torch.no_grad():
            for p_, g_ in zip(params, grads):
                p_ -= 1e-3 * g_
        # (detached: a loss that is kept would keep the step's autograd graph, and with it the parameters' gradient
        # nodes and the stream they were made on, alive into the capture below, which torch warns can break it)
        return loss.detach()

    def one_epoch():
        loss = None
        for lo in range(0, TRAIN_SAMPLES, TRAIN_BATCH):
            loss = one_step(lo, min(lo + TRAIN_BATCH, TRAIN_SAMPLES))
        return loss

    for _ in range(warmup):
        one_step(0, TRAIN_BATCH)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        one_step(0, TRAIN_BATCH)
    e1.record()
    torch.cuda.synchronize()
    ms_step = e0.elapsed_time(e1) / steps
    one_epoch()                     # the ragged last batch plans and allocates once before it is timed
    torch.cuda.synchronize()
    e0.record()
    loss = one_epoch()
    e1.record()
    torch.cuda.synchronize()
    ms_epoch = e0.elapsed_time(e1)
    final_loss = float(loss)

    # The same step as a HIP graph (one launch per step): one graph for the full batch, one for the ragged last batch;
    # a batch is copied into the graph's input tensors before every replay, inside the timed region.
    last = TRAIN_SAMPLES % TRAIN_BATCH
    del loss
    gparams = [p_.detach().clone().requires_grad_(True) for p_ in params]   # parameters of their own, no history
    graphs = {}
    for nb in sorted({TRAIN_BATCH, last} - {0}):
        xb, yb = X[:nb].clone(), Y[:nb].clone()

        def graph_step(xb=xb, yb=yb):
            Z = torch.tanh(xb @ gparams[0] + gparams[1])
            S = autograd.signature(Z, depth)
            loss_ = ((S @ gparams[2] + gparams[3] - yb) ** 2).mean()
            grads = torch.autograd.grad(loss_, gparams)
            with torch.no_grad():
                for p_, g_ in zip(gparams, grads):
                    p_ -= 1e-3 * g_
            return loss_.detach()
        graphs[nb] = (xb, yb) + autograd.capture(graph_step)

    def graph_replay(lo, hi):
        xb, yb, graph, loss_ = graphs[hi - lo]
        xb.copy_(X[lo:hi])
        yb.copy_(Y[lo:hi])
        graph.replay()
        return loss_

    for _ in range(warmup):
        graph_replay(0, TRAIN_BATCH)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        graph_replay(0, TRAIN_BATCH)
    e1.record()
    torch.cuda.synchronize()
    ms_step_graph = e0.elapsed_time(e1) / steps
    e0.record()
    for lo in range(0, TRAIN_SAMPLES, TRAIN_BATCH):
        loss_g = graph_replay(lo, min(lo + TRAIN_BATCH, TRAIN_SAMPLES))
    e1.record()
    torch.cuda.synchronize()
    return {"model": "Dense(20->%d, tanh) -> signature depth %d -> Dense(%d->10), MSE, SGD" % (d, depth, D),
            "batch": TRAIN_BATCH, "length": L, "ms_per_step": ms_step, "samples": TRAIN_SAMPLES,
            "steps_per_epoch": (TRAIN_SAMPLES + TRAIN_BATCH - 1) // TRAIN_BATCH, "last_batch": last,
            "ms_per_epoch": ms_epoch, "final_loss": final_loss,
            "ms_per_step_graph": ms_step_graph, "ms_per_epoch_graph": e0.elapsed_time(e1),
            "final_loss_graph": float(loss_g)}


def anchors(binding):
    """Achievable rates on this GPU: a plain copy, a plain fill and the stream kernels' write pattern (HBM), an fp32 FMA
    loop without packed instructions, and the FMA form of the fused kernels (acc[a][b] += g[a] * v[b], three vector
    registers per instruction) at three and at eight wavefronts per SIMD."""
    import torch
    n = 1 << 28  # 1 GiB each way
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    out = torch.empty(8192 * 64, dtype=torch.float32, device="cuda")
    res = {}
    for name, fn, work in [("copy_GBps", lambda: binding.sig_probe_copy(dst, src), 8.0 * n / 1e9),
                           ("fill_GBps", lambda: binding.sig_probe_write(dst, 1), 4.0 * n / 1e9),
                           ("write_4096_streams_GBps", lambda: binding.sig_probe_write(dst, 4096), 4.0 * n / 1e9),
                           ("write_1024_streams_GBps", lambda: binding.sig_probe_write(dst, 1024), 4.0 * n / 1e9),
                           ("fma_TFLOPs", lambda: binding.sig_probe_fma(out, 8192, 20000),
                            2.0 * 16 * 20000 * 8192 * 64 / 1e12),
                           # one round of workgroups: 3 (LDS-limited) or 8 wavefronts on every SIMD of 256 compute units
                           ("fma_outer_3_waves_per_simd_TFLOPs", lambda: binding.sig_probe_fma_outer(out, 3072, 4000, 53000),
                            2.0 * 100 * 4000 * 3072 * 64 / 1e12),
                           ("fma_outer_8_waves_per_simd_TFLOPs", lambda: binding.sig_probe_fma_outer(out, 8192, 4000, 0),
                            2.0 * 100 * 4000 * 8192 * 64 / 1e12)]:
        for _ in range(3):
            assert fn() == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[name] = work / (e0.elapsed_time(e1) / 10 * 1e-3)
    # The same FMA loop after a third of a second of it: what the chip sustains once its power management has
    # settled (the figures above are taken within its first 40 ms).  Boxes of this pool differ here by up to 15 %,
    # and the saturated rows of this file, which run for tens of milliseconds each, differ with it.
    fn = lambda: binding.sig_probe_fma_outer(out, 8192, 4000, 0)
    for _ in range(100):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(30):
        fn()
    e1.record()
    torch.cuda.synchronize()
    res["fma_outer_8_waves_per_simd_sustained_TFLOPs"] = 2.0 * 100 * 4000 * 8192 * 64 / 1e12 / (e0.elapsed_time(e1) / 30 * 1e-3)
    return res


def cpu_baseline(workloads, cfg, max_paths, budget_s=20.0):
    """The fp64 oracle on the host cores, on (a sample of) the same workload."""
    import numpy as np
    import oracle
    oracle.build()
    n = max_paths
    x = workloads.make_paths(cfg, B=n)
    xs = x[:n]
    oracle.signature(xs[:1], cfg.depth, stream=cfg.stream)  # load the library
    times = []
    t_start = time.perf_counter()
    while len(times) < 5 and (time.perf_counter() - t_start < budget_s or not times):
        t0 = time.perf_counter()
        oracle.signature(xs, cfg.depth, stream=cfg.stream)
        times.append(time.perf_counter() - t0)
    t = float(np.median(times))
    return {"value": n / t, "unit": "paths/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d paths of the workload's shape, median of %d runs, %.4f s per run" % (n, len(times), t)}


def compact(entry):
    """The figures of one all_configs entry that fit a line: workload, time, throughput, bound and fraction."""
    rf = entry["roofline"]
    return {"workload": entry["workload"], "ms_per_step": round(entry["ms_per_step"], 6),
            "paths_per_s": round(entry["paths_per_s"], 1), "bound": rf["bound"], "achieved": round(rf["achieved"], 2),
            "unit": rf["unit"], "frac": round(rf["frac"], 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--no-extras", action="store_true", help="time the headline workload only")
    ap.add_argument("--full", action="store_true",
                    help="keep every field of the extra entries (plans, algorithmic work, host-clock times) instead of the compact rows")
    ap.add_argument("--anchors", action="store_true", help="also measure the copy and FMA-loop anchors")
    ap.add_argument("--workload", default="C2", help="configuration to time as the headline (C1..C5)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch size (batch-saturated variants)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--backward", action="store_true", help="time sig_backward on the named workload instead")
    ap.add_argument("--stream-families", action="store_true",
                    help="also time stream mode on a grid of small and medium batches: planner's choice vs level-scan")
    ap.add_argument("--level-scan", action="store_true",
                    help="time the level-by-level kernel family (the paper's Section 3.2) instead of the planner's choice")
    ap.add_argument("--hbm-streaming", type=int, default=-1, metavar="P",
                    help="time the HBM-streaming kernel family with prefix depth P instead of the planner's choice")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (a box has one MI355X); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2501_08455_amd import binding, workloads
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    binding.load()
    ctx = binding.default_ctx()

    cfg = workloads.CONFIGS[args.workload]
    B = args.batch or cfg.B
    forced = None
    forced_label = ""
    if args.hbm_streaming >= 0:
        forced = binding.make_plan(binding.SIG_VARIANT_HBM_STREAMING, prefix_depth=args.hbm_streaming)
        forced_label = " (HBM-streaming family)"
    if args.level_scan:
        forced = binding.make_plan(binding.SIG_VARIANT_LEVEL_SCAN, chunks=0)
        forced_label = " (level-scan family)"
    if args.backward:
        head = bench_backward(binding, workloads, ctx, cfg, B, args.steps, args.warmup)
        head["terms_per_s"] = None
        head["plan"] = None
    else:
        head = bench_config(binding, workloads, ctx, cfg, B, args.steps, args.warmup, plan=forced,
                            label=forced_label)
    line = {
        "metric": "signatures/sec at (B=%d, L=%d, d=%d, N=%d), %s" % (
            B, cfg.L, cfg.d, cfg.depth, "every prefix (stream)" if cfg.stream else "final signature"),
        "value": head["paths_per_s"], "unit": "paths/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": head["workload"], "terms_per_s": head["terms_per_s"], "plan": head["plan"],
                   "input": "Brownian paths, increments N(0, 1/L), seeded, resident in HBM"},
        "roofline": head["roofline"],
    }
    keep = (lambda e: e) if args.full else compact
    if not args.no_extras:
        # The literal configurations are bound by launch latency (their ideal times are below one kernel launch); the
        # fractions that say something about the kernels are those of the batch-saturated variants with the same
        # (L, d, N, mode, distribution), and of the large-signature configuration, which fills the chip as it is.  They
        # sit inside the roofline object of the headline so that they travel with it.
        # (configuration, batch, timed steps, warm-up steps); warm-ups are long enough (tens of ms) for the shader clock
        # to ramp up after idle
        saturated = {}
        # (and for its power management to settle: per-launch times of a saturated kernel start at their best, rise by
        # 15-25 % after about eight launches and come back over the next 40-60 ms -- seen alike on every saturated
        # workload in the kernel traces -- so the warm-ups here run for about 70 ms)
        for key, name, Bs, steps, warm in [("C1-sat", "C1", 1 << 20, 400, 2000), ("C2-sat", "C2", 65536, 150, 400),
                                           ("C3-sat", "C3", 4096, 80, 300), ("C4-sat", "C4", 4096, 60, 250),
                                           ("C5", "C5", None, 300, 900), ("C5-sat", "C5", 64, 60, 300)]:
            c = workloads.CONFIGS[name]
            e = bench_config(binding, workloads, ctx, c, Bs or c.B, steps, warm)
            row = compact(e)
            row["traffic"] = e["roofline"]["traffic"]
            saturated[key] = row
        line["roofline"]["saturated"] = saturated
        line["roofline"]["note"] = ("the headline workload is bound by launch latency at its literal size; `saturated` holds "
                                    "the same kernels on batches that fill the chip")
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(workloads, cfg, max_paths=min(B, 128))
    if not args.no_extras:
        extras = []
        for name, steps, warm in [("C1", 3000, 3000), ("C3", 1000, 500), ("C4", 1000, 500)]:
            c = workloads.CONFIGS[name]
            extras.append(bench_config(binding, workloads, ctx, c, c.B, steps, warm))
        # the HBM-streaming family (the fallback for shapes that neither of the other families takes) on C5
        c5 = workloads.CONFIGS["C5"]
        hbm_plan = binding.make_plan(binding.SIG_VARIANT_HBM_STREAMING, prefix_depth=2)
        extras.append(bench_config(binding, workloads, ctx, c5, c5.B, 20, 5, plan=hbm_plan,
                                   label=" (HBM-streaming family)"))
        # the paper's own level-by-level formulation (Section 3.2) as a kernel family, next to the fused fold above
        ls_plan = binding.make_plan(binding.SIG_VARIANT_LEVEL_SCAN, chunks=0)
        for name, Bs, steps, warm in [("C2", None, 500, 200), ("C4", None, 500, 200), ("C5", None, 50, 20),
                                      ("C2", 65536, 10, 3), ("C4", 4096, 20, 5)]:
            c = workloads.CONFIGS[name]
            extras.append(bench_config(binding, workloads, ctx, c, Bs or c.B, steps, warm, plan=ls_plan,
                                       label=" (level-scan family)"))
        # the gradient with respect to the path (reverse sweep) on the shapes it is compiled for
        for name, Bs, steps, warm in [("C2", None, 1000, 500), ("C4", None, 300, 200), ("C5", None, 30, 10),
                                      ("C2", 65536, 30, 20), ("C4", 4096, 20, 10)]:
            c = workloads.CONFIGS[name]
            extras.append(bench_backward(binding, workloads, ctx, c, Bs or c.B, steps, warm))
        # ... and on long paths, where the sweep is cut into time segments across workgroups: C3 (2,000 points), and
        # single paths of 1,000 points in the shapes of C2 and of a ten-channel depth-4 layer (final and stream mode)
        extras.append(bench_backward(binding, workloads, ctx, workloads.CONFIGS["C3"], 128, 100, 50))
        for d, depth, stream in [(5, 4, False), (10, 4, False), (5, 4, True), (10, 4, True)]:
            one = workloads.Config("one path", 1, 1000, d, depth, stream, "normal")
            extras.append(bench_backward(binding, workloads, ctx, one, 1, 200, 100, seed=workloads.BASE_SEED + 11))
        line["all_configs"] = [keep(e) for e in extras]
        t1 = table1(binding, workloads, ctx)
        line["table1_shapes"] = t1 if args.full else [
            {"batch": r["batch"], "length": r["length"], "depth": r["depth"], "channels": r["channels"],
             "ms": round(r["ms"], 5), "ms_autotuned": None if r["ms_autotuned"] is None else round(r["ms_autotuned"], 5),
             "paper_ks_gpu_ms_rtx4090": r["paper_ks_gpu_ms_rtx4090"]} for r in t1]
        line["memory_wall_shape"] = memory_wall_shape(binding, workloads, ctx)
        # the paper's model with the signature layer in the middle (Section 4.2): one step and one epoch of 12,765 samples
        line["training_step"] = [training_step(workloads, L, d, depth, 100, 30)
                                 for (L, d, depth) in [(100, 5, 4), (200, 6, 3), (500, 4, 4)]]
    if args.stream_families:
        line["stream_families"] = stream_families(binding, workloads, ctx)
    if args.anchors or not args.no_extras:
        line["anchors"] = anchors(binding)
    print(json.dumps(line))


if __name__ == "__main__":
    main()

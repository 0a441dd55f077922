"""CPU-only checks of the C-ABI library: it loads, exports what include/sig.h declares, and its
host-only entry points (sizes, planner, error strings) behave."""
import os
import re

import pytest

from paper_2501_08455_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(sig_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = declared_functions()
    assert {"sig_create", "sig_compute", "sig_destroy", "sig_size", "sig_plan", "sig_compute_planned",
            "sig_combine", "sig_strerror", "sig_on_chip_available", "sig_plan_validate", "sig_autotune",
            "sig_probe_copy", "sig_probe_fma", "sig_compute_noalloc"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("d,depth,D", [(2, 3, 14), (5, 4, 780), (4, 4, 340), (10, 6, 1111110), (10, 4, 11110),
                                       (1, 7, 7), (3, 1, 3)])
def test_sig_size(d, depth, D):
    assert binding.sig_size(d, depth) == D == workloads.sig_size(d, depth)


def test_sig_size_rejects_bad_or_overflowing_shapes():
    assert binding.sig_size(0, 3) == -1
    assert binding.sig_size(3, 0) == -1
    assert binding.sig_size(10, 30) == -1


def test_error_strings():
    seen = {binding.sig_strerror(c) for c in range(6)}
    assert len(seen) == 6 and all(seen)
    assert binding.sig_strerror(99) == "unknown status"


def test_plan_rejects_what_compute_rejects():
    for args in [(-1, 5, 2, 3, 0), (4, 1, 2, 3, 0), (4, 5, 0, 3, 0), (4, 5, 2, 0, 0), (4, 5, 2, 3, 2)]:
        rc, _ = binding.sig_plan(None, *args)
        assert rc == binding.SIG_ERR_INVALID, args
    rc, _ = binding.sig_plan(None, 4, 5, 10, 12, 0)
    assert rc == binding.SIG_ERR_TOO_LARGE


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_plan_of_the_five_configs_is_on_chip_and_consistent(name):
    cfg = workloads.CONFIGS[name]
    rc, pl = binding.sig_plan(None, cfg.B, cfg.L, cfg.d, cfg.depth, int(cfg.stream))
    assert rc == binding.SIG_OK
    assert pl.variant == binding.SIG_VARIANT_ON_CHIP
    assert binding.sig_on_chip_available(cfg.d, cfg.depth, pl.prefix_depth)
    K = cfg.L - 1
    assert 1 <= pl.chunks * pl.segments <= K
    assert pl.threads % 64 == 0 and 64 <= pl.threads <= 512
    lanes = cfg.d ** pl.prefix_depth
    assert lanes > pl.threads or pl.chunks * lanes <= pl.threads
    if cfg.stream:
        assert pl.segments == 1


def test_plan_falls_back_for_uncompiled_shapes():
    """Without an on-chip kernel: the level-by-level family where it applies (d <= 256, depth <= 8, levels short
    enough for 32-bit offsets), else the HBM-streaming family."""
    for stream in (0, 1):
        rc, pl = binding.sig_plan(None, 7, 30, 9, 6, stream)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_LEVEL_SCAN
        assert binding.sig_plan_validate(7, 30, 9, 6, stream, pl) == binding.SIG_OK
        rc, pl = binding.sig_plan(None, 7, 30, 12, 3, stream)      # more than 10 channels: run-time d
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_LEVEL_SCAN
        rc, pl = binding.sig_plan(None, 7, 30, 300, 2, stream)     # more channels than a workgroup has threads
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_HBM_STREAMING
        assert 0 <= pl.prefix_depth <= 1
        rc, pl = binding.sig_plan(None, 7, 30, 2, 9, stream)       # deeper than 8
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_HBM_STREAMING
    # lower levels of every prefix: 136 GB for the batch, which is therefore taken in slices that need 8 GiB at most
    rc, pl = binding.sig_plan(None, 512, 1000, 9, 6, 0)
    assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_LEVEL_SCAN
    rc, _, _, scratch = binding.sig_plan_footprint(512, 1000, 9, 6, 0, pl)
    assert rc == binding.SIG_OK and 4 << 30 < scratch <= 8 << 30
    per_path = 999 * (binding.sig_size(9, 6) - 9 ** 6) * 4
    assert scratch % per_path == 0 and 512 % (scratch // per_path) == 0      # 16 equal slices of 32 paths
    # one path of a level too long for the family's 32-bit offsets
    rc, pl = binding.sig_plan(None, 2, 500, 9, 8, 0)
    assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_HBM_STREAMING


def test_large_batches_are_not_cut_in_time():
    rc, pl = binding.sig_plan(None, 65536, 100, 5, 4, 0)
    assert rc == binding.SIG_OK and pl.chunks == 1 and pl.segments == 1


def test_create_without_a_gpu_reports_no_device():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(binding.SigError) as err:
        binding.sig_create()
    assert err.value.status == binding.SIG_ERR_NO_DEVICE


def test_every_forced_plan_of_the_gpu_tests_is_accepted_by_the_host_checks():
    import importlib
    mod = importlib.import_module("test_gpu_parity")
    for case in mod.ON_CHIP_CASES:
        d, depth, p, B, L, chunks, segments, tile, stream, threads = mod.split_case(case)
        plan = binding.make_plan(binding.SIG_VARIANT_ON_CHIP, prefix_depth=p, chunks=chunks, segments=segments,
                                 tile_steps=tile, threads=threads)
        assert binding.sig_plan_validate(B, L, d, depth, int(stream), plan) == binding.SIG_OK, case


def test_plan_validate_rejects_plans_the_kernels_cannot_run():
    mk = binding.make_plan
    on = binding.SIG_VARIANT_ON_CHIP
    assert binding.sig_plan_validate(4, 16, 9, 6, 0, mk(on, prefix_depth=1)) == binding.SIG_ERR_INVALID  # not compiled
    assert binding.sig_plan_validate(4, 16, 5, 4, 0, mk(on, prefix_depth=2, chunks=11)) == binding.SIG_ERR_INVALID
    assert binding.sig_plan_validate(4, 16, 5, 4, 1, mk(on, prefix_depth=2, segments=2)) == binding.SIG_ERR_INVALID
    assert binding.sig_plan_validate(4, 6, 5, 4, 0, mk(on, prefix_depth=2, chunks=3, segments=2)) == binding.SIG_ERR_INVALID
    assert binding.sig_plan_validate(4, 16, 5, 4, 0, mk(on, prefix_depth=2, threads=100)) == binding.SIG_ERR_INVALID
    assert binding.sig_plan_validate(4, 16, 5, 4, 0, mk(binding.SIG_VARIANT_HBM_STREAMING, prefix_depth=4)) \
        == binding.SIG_ERR_INVALID
    assert binding.sig_plan_validate(4, 16, 5, 4, 0, mk(binding.SIG_VARIANT_HBM_STREAMING, prefix_depth=3)) \
        == binding.SIG_OK


def test_join_in_lds_is_checked_with_the_join_the_kernels_take():
    """(8,4) with 512 lanes per path has a small lane state, but its lanes span several workgroups, so its segments
    are joined by the LDS tree (one and a half times the rows), not by the register join: three rows of 18.7 KB would
    fit, the tree's five do not, and three is no power of two for the join in device memory."""
    three = binding.make_plan(binding.SIG_VARIANT_ON_CHIP, prefix_depth=3, chunks=1, segments=3)
    assert binding.sig_plan_validate(4, 100, 8, 4, 0, three) == binding.SIG_ERR_INVALID
    two = binding.make_plan(binding.SIG_VARIANT_ON_CHIP, prefix_depth=3, chunks=1, segments=2)
    assert binding.sig_plan_validate(4, 100, 8, 4, 0, two) == binding.SIG_OK


def test_planner_keeps_the_shape_grid_on_chip():
    """Every compiled (d, depth) gets an on-chip plan that validates, over the batch sizes and lengths of the
    paper's direct-computation tables (Section 4.1) and beyond; host only."""
    grid = [(2, 3), (4, 4), (5, 4), (10, 6), (2, 2), (3, 2), (4, 2), (5, 2), (6, 2), (8, 2), (10, 2), (3, 3), (4, 3),
            (5, 3), (6, 3), (7, 3), (8, 3), (10, 3), (2, 4), (3, 4), (6, 4), (7, 4), (8, 4), (10, 4), (2, 5), (3, 5),
            (4, 5), (5, 5), (6, 5), (2, 6), (3, 6), (4, 6), (5, 6), (7, 2), (9, 2), (9, 3), (9, 4), (7, 5), (8, 5),
            (9, 5), (10, 5)]
    for d, depth in grid:
        for B in (1, 7, 32, 128, 512, 4096, 65536):
            for L in (2, 9, 50, 200, 1000):
                for stream in (0, 1):
                    rc, pl = binding.sig_plan(None, B, L, d, depth, stream)
                    assert rc == binding.SIG_OK, (d, depth, B, L, stream)
                    # few paths may take the level-by-level family (parallel in time): stream mode, or final mode
                    # when the register plan could not be cut in time; from 4096 paths on the register kernels
                    allowed = [binding.SIG_VARIANT_ON_CHIP]
                    if B < 4096 and (stream or pl.chunks == 0):
                        allowed.append(binding.SIG_VARIANT_LEVEL_SCAN)
                    assert pl.variant in allowed, (d, depth, B, L, stream, pl.as_dict())
                    assert binding.sig_plan_validate(B, L, d, depth, stream, pl) == binding.SIG_OK


def test_stream_plans_of_few_long_paths_are_parallel_in_time():
    """One path of 500 points in 8 channels at depth 4: 499 dependent steps in the register kernel against one
    launch per level (measured 737 against 49 us); the configurations keep their register kernels."""
    rc, pl = binding.sig_plan(None, 1, 500, 8, 4, 1)
    assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_LEVEL_SCAN
    rc, pl = binding.sig_plan(None, 1, 500, 8, 4, 0)
    assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP
    # final mode: rows too long for the LDS of a join (10 channels at depth 4) are cut into a power of two of
    # segments that are joined in device memory (one path of 2,000 points: 64 us against 206 us level by level and
    # 573 us uncut); shorter paths stay uncut, and of those only few-path plans lose to the level-by-level family
    rc, pl = binding.sig_plan(None, 1, 2000, 10, 4, 0)
    assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP and pl.segments == 32
    rc, pl = binding.sig_plan(None, 1, 200, 10, 4, 0)
    assert rc == binding.SIG_OK and (pl.variant == binding.SIG_VARIANT_LEVEL_SCAN or pl.segments == 1)
    rc, pl = binding.sig_plan(None, 128, 2000, 10, 4, 0)
    assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP
    for name in ("C4",):
        cfg = workloads.CONFIGS[name]
        for B in (cfg.B, 4096):
            rc, pl = binding.sig_plan(None, B, cfg.L, cfg.d, cfg.depth, 1)
            assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP


def test_level_scan_plans_are_checked_on_the_host():
    """The level-by-level family (Section 3.2) takes d <= 256, depth <= 8, chunks >= 0 and rows that 32-bit lane
    offsets can address; the planner chooses it only for shapes without an on-chip kernel."""
    ls = binding.SIG_VARIANT_LEVEL_SCAN
    mk = binding.make_plan
    for stream in (0, 1):
        assert binding.sig_plan_validate(128, 100, 5, 4, stream, mk(ls, chunks=0)) == binding.SIG_OK
        assert binding.sig_plan_validate(16, 128, 10, 6, stream, mk(ls, chunks=7)) == binding.SIG_OK
        assert binding.sig_plan_validate(4, 16, 1, 8, stream, mk(ls, chunks=1000)) == binding.SIG_OK
        assert binding.sig_plan_validate(4, 16, 11, 2, stream, mk(ls, chunks=0)) == binding.SIG_OK
        assert binding.sig_plan_validate(4, 16, 300, 2, stream, mk(ls, chunks=0)) == binding.SIG_ERR_INVALID
        assert binding.sig_plan_validate(4, 16, 2, 9, stream, mk(ls, chunks=0)) == binding.SIG_ERR_INVALID
        assert binding.sig_plan_validate(4, 16, 2, 3, stream, mk(ls, chunks=-1)) == binding.SIG_ERR_INVALID
    # one path's rows beyond 2^30 floats
    assert binding.sig_plan_validate(1, 2000, 10, 6, 1, mk(ls, chunks=0)) == binding.SIG_ERR_TOO_LARGE
    assert binding.sig_plan_validate(1, 20000, 10, 6, 0, mk(ls, chunks=0)) == binding.SIG_ERR_TOO_LARGE
    for name in ("C1", "C2", "C3", "C4", "C5"):
        cfg = workloads.CONFIGS[name]
        rc, pl = binding.sig_plan(None, cfg.B, cfg.L, cfg.d, cfg.depth, int(cfg.stream))
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP


def test_every_compiled_forward_shape_has_a_gradient_kernel():
    """sig_backward covers the (d, depth) grid of the on-chip forward kernels, the five configurations included."""
    shapes = set()
    for d in range(1, 11):
        for depth in range(1, 7):
            if any(binding.sig_on_chip_available(d, depth, p) for p in range(0, depth)):
                shapes.add((d, depth))
    assert len(shapes) >= 30
    for name in ("C1", "C2", "C3", "C4", "C5"):
        cfg = workloads.CONFIGS[name]
        assert (cfg.d, cfg.depth) in shapes
    missing = sorted(s for s in shapes if not binding.sig_backward_available(*s))
    assert not missing, missing


def test_backward_segment_rule():
    """Host rule for cutting the reverse sweep in time: few long paths in final mode, never in stream mode, paths too
    long for one workgroup's LDS at any batch size, and the general sweep for shapes without a register kernel."""
    seg = lambda B, L, d, depth, stream=0: binding.sig_backward_segments(None, B, L, d, depth, stream)
    # short paths and full batches stay uncut
    assert seg(128, 100, 5, 4) == 1 and seg(65536, 100, 5, 4) == 1 and seg(1, 100, 10, 4) == 1
    assert seg(1024, 1000, 10, 4) == 1 and seg(128, 500, 10, 4) == 1
    # between one and two workgroups per compute unit a few segments still pay
    assert 2 <= seg(128, 500, 8, 4) <= 4 and 2 <= seg(256, 500, 5, 5) <= 4
    # few long paths are cut, at most 32 times, and a segment keeps at least two dozen increments
    for B, L, d, depth in [(1, 1000, 5, 4), (1, 1000, 10, 4), (16, 500, 8, 4), (3, 300, 5, 5), (2, 4001, 2, 3)]:
        W = seg(B, L, d, depth)
        assert 2 <= W <= 32 and (L - 1) // W >= 24, (B, L, d, depth, W)
    # shapes whose plain sweep holds many chunks in a workgroup: only from 512 increments on and up to 32 paths ...
    assert seg(1, 400, 5, 4) == 1 and seg(1, 600, 5, 4) > 1 and seg(64, 600, 5, 4) == 1
    # ... unless the path is so long that the chunks no longer fit (the gradient of the third configuration)
    assert seg(128, 2000, 5, 4) > 1
    # stream mode is cut as well (two sweeps and a scan between them), at smaller batches than final mode; rows of a
    # few dozen floats keep the plain sweep with its chunks
    assert seg(1, 1000, 5, 4, 1) > 1 and seg(1, 1000, 10, 4, 1) > 1 and seg(4, 1000, 2, 3, 1) == 1
    assert seg(64, 300, 10, 4, 1) == 1 and seg(8, 300, 10, 4, 1) > 1
    # paths too long for the LDS of one workgroup: cut across workgroups in final mode at any batch size ...
    assert seg(300, 3500, 5, 4) >= 2 and seg(1, 20000, 5, 4) >= 2
    # ... and walked in tiles by one workgroup where that is not possible (stream mode; final mode beyond 32 segments)
    assert seg(300, 1500, 10, 4, 1) == 1 and seg(2, 60000, 10, 2) == 1 and seg(2, 60000, 10, 2, 1) == 1
    assert seg(100000, 5000, 5, 4) == 1
    # no register kernel: the general sweep; beyond its limits and bad arguments: minus the status
    assert seg(4, 50, 11, 2) == 0 and seg(4, 50, 300, 2) == -binding.SIG_ERR_UNSUPPORTED
    assert seg(4, 1, 5, 4) == -binding.SIG_ERR_INVALID and seg(-1, 10, 5, 4) == -binding.SIG_ERR_INVALID
    # rows of (10, 6) are too large for the scan over segments
    assert seg(16, 128, 10, 6) == 1 and seg(1, 1000, 10, 6) == 1


def test_prefix_depth_follows_the_batch_for_ten_channels_at_depth_four():
    """d = 8 and 10 at depth 4 have two compiled prefix depths: the deeper one (a thousand lanes per path) only while
    the batch is too small to give every compute unit a wavefront with the shallower one; stream mode keeps lanes
    that fit a workgroup."""
    for d, small, large in [(10, 128, 256), (8, 128, 1024), (9, 128, 256)]:
        rc, pl = binding.sig_plan(None, small, 100, d, 4, 0)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP and pl.prefix_depth == 3
        rc, pl = binding.sig_plan(None, large, 100, d, 4, 0)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP and pl.prefix_depth == 2
        rc, pl = binding.sig_plan(None, 4096, 100, d, 4, 1)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP and pl.prefix_depth == 2


def test_small_batches_of_short_paths_take_the_deeper_prefix_for_five_channels_at_depth_four():
    """d = 5 at depth 4: p = 3 with four chunks in a workgroup of 512 threads while the batch leaves the chip mostly
    idle and the path is short; otherwise p = 2 in 256 threads.  Stream mode takes p = 3 (256 threads) on short paths
    of a batch that leaves p = 2 at most half a wavefront per SIMD, and p = 2 otherwise."""
    for B, L in [(128, 100), (1, 100), (32, 50), (256, 200)]:
        rc, pl = binding.sig_plan(None, B, L, 5, 4, 0)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP
        assert (pl.prefix_depth, pl.chunks, pl.threads) == (3, 4, 512), (B, L)
        assert binding.sig_plan_validate(B, L, 5, 4, 0, pl) == binding.SIG_OK
    for B, L, stream in [(512, 100, 0), (128, 300, 0), (128, 2000, 0), (128, 300, 1), (2048, 100, 1)]:
        rc, pl = binding.sig_plan(None, B, L, 5, 4, stream)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP
        assert pl.prefix_depth == 2 and pl.threads <= 256, (B, L, stream)
    for B, L in [(128, 100), (4, 50), (1024, 129)]:
        rc, pl = binding.sig_plan(None, B, L, 5, 4, 1)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP
        assert pl.prefix_depth == 3 and pl.threads <= 256, (B, L)
        assert binding.sig_plan_validate(B, L, 5, 4, 1, pl) == binding.SIG_OK


def test_small_batches_take_wide_workgroups_for_small_states_with_many_lanes():
    """Final mode, lane state of at most 64 floats, more than 64 (and fewer than 256) lanes per path: 512 threads with
    twice the chunks while 256 threads would leave the chip at or below a wavefront per SIMD."""
    for d, depth, chunks in [(5, 5, 4), (6, 5, 2), (9, 3, 6), (10, 3, 4)]:
        rc, pl = binding.sig_plan(None, 128, 100, d, depth, 0)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP
        assert (pl.chunks, pl.threads) == (chunks, 512), (d, depth)
        assert binding.sig_plan_validate(128, 100, d, depth, 0, pl) == binding.SIG_OK
        rc, pl = binding.sig_plan(None, 512, 100, d, depth, 0)
        assert rc == binding.SIG_OK and pl.threads == 256, (d, depth)
        rc, pl = binding.sig_plan(None, 128, 100, d, depth, 1)
        assert rc == binding.SIG_OK and pl.threads <= 256, (d, depth)
    for d, depth in [(4, 6), (3, 5), (4, 5), (7, 4), (10, 4)]:
        rc, pl = binding.sig_plan(None, 128, 100, d, depth, 0)
        assert rc == binding.SIG_OK and pl.threads <= 256, (d, depth)


def test_few_long_paths_with_small_states_are_cut_into_more_segments():
    """Final mode, chunked register kernels: while the chip is at most half a wavefront per SIMD full, the segment count
    follows the cost model (steps of a chunk against a join over W rows) instead of 48 steps per chunk."""
    for d, depth, B, L, segments in [(4, 4, 1, 1000, 3), (4, 4, 8, 2000, 4), (5, 4, 32, 1000, 3), (3, 5, 8, 2000, 4),
                                     (5, 3, 8, 2000, 4), (6, 4, 1, 1000, 3)]:
        rc, pl = binding.sig_plan(None, B, L, d, depth, 0)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP
        assert pl.segments == segments, (d, depth, B, L, pl.segments)
        assert (L - 1) // (pl.chunks * pl.segments) >= 8
    # a busier chip keeps the longer chunks; two segments are not taken on the model's word alone
    for d, depth, B, L in [(4, 4, 512, 1000), (3, 5, 512, 1000), (4, 4, 128, 500), (3, 5, 128, 500)]:
        rc, pl = binding.sig_plan(None, B, L, d, depth, 0)
        assert rc == binding.SIG_OK and pl.segments == 1, (d, depth, B, L)
    # the busier the chip, the fewer segments; the longer the path, the more
    got = [binding.sig_plan(None, B, L, 5, 4, 0)[1].segments for B, L in [(128, 2000), (384, 2000), (1024, 2000), (512, 1000), (256, 4000)]]
    assert got == [4, 2, 1, 1, 4], got
    # the third config is unchanged
    rc, pl = binding.sig_plan(None, 128, 2000, 5, 4, 0)
    assert rc == binding.SIG_OK and (pl.prefix_depth, pl.chunks, pl.segments) == (2, 10, 4)


def test_deeper_prefix_entries_behind_the_first_small_state():
    """(4,4), (5,3), (6,3), (4,3), (7,3), (3,4), (3,5), (2,6) and (3,6) have a prefix depth behind the first one with a small lane state: taken in final mode for
    small batches of short paths only; with 512 threads once the path is long enough for twice the chunks."""
    for d, depth, p in [(4, 4, 3), (5, 3, 2), (6, 3, 2), (4, 3, 2), (7, 3, 2), (3, 4, 3), (3, 5, 3), (2, 6, 3), (3, 6, 4), (3, 3, 2), (2, 4, 2), (2, 5, 2)]:
        assert binding.sig_on_chip_available(d, depth, p)
        for B, L in [(16, 100), (128, 50), (128, 257), (256, 100)]:
            rc, pl = binding.sig_plan(None, B, L, d, depth, 0)
            assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP and pl.prefix_depth == p, (d, depth, B, L)
            assert binding.sig_plan_validate(B, L, d, depth, 0, pl) == binding.SIG_OK
        rc, pl = binding.sig_plan(None, 128, 257, d, depth, 0)
        assert pl.threads == (256 if d == 2 or (d, depth) == (3, 3) else 512), (d, depth)
        # longer paths: up to 768 increments where the shallower entry has few lanes or a large state, else 256
        rc, pl = binding.sig_plan(None, 128, 500, d, depth, 0)
        assert rc == binding.SIG_OK and (pl.prefix_depth == p) == ((d, depth) != (4, 4)), (d, depth)
        # larger batches: four times as many paths where the shallower entry has fewer than 16 lanes per path
        rc, pl = binding.sig_plan(None, 1000, 100, d, depth, 0)
        assert rc == binding.SIG_OK and (pl.prefix_depth == p) == ((d, depth) not in [(4, 4), (3, 6)]), (d, depth)
        # (behind an entry with two lanes per path -- two channels, p = 1 -- the second entry is taken at every batch
        # and length)
        behind_two_lanes = d == 2 and p == 2
        for B, L, stream in [(2000, 100, 0), (128, 1000, 0), (4096, 100, 0)]:
            rc, pl = binding.sig_plan(None, B, L, d, depth, stream)
            assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP, (d, depth, B, L)
            assert (pl.prefix_depth == p) if behind_two_lanes else (pl.prefix_depth < p), (d, depth, B, L)
        # stream mode takes them behind an entry with fewer than 16 lanes per path, at every batch; behind the others
        # ((4,4): 16 lanes, (3,6): 27) on short paths of batches that leave the chip at most half a wavefront per SIMD
        for B, L in [(128, 100), (4, 50), (4096, 256)]:
            rc, pl = binding.sig_plan(None, B, L, d, depth, 1)
            assert rc == binding.SIG_OK
            if pl.variant != binding.SIG_VARIANT_ON_CHIP:
                continue
            if (d, depth) in [(4, 4), (3, 6)] and B == 4096:
                assert pl.prefix_depth < p, (d, depth, B, L)
            else:
                assert pl.prefix_depth == p, (d, depth, B, L)


def test_six_channels_at_depth_four_take_the_deeper_prefix_only_up_to_128_increments():
    """(6,4,3) has 216 lanes per path: two chunks in 512 threads, which pays for short paths only."""
    for B, L, p in [(128, 100, 3), (64, 20, 3), (256, 129, 3), (128, 200, 2), (128, 257, 2), (512, 100, 2)]:
        rc, pl = binding.sig_plan(None, B, L, 6, 4, 0)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP and pl.prefix_depth == p, (B, L)
    # stream mode: p = 3 at any length while p = 2 (36 lanes of 43 floats) would leave the chip at most half a wavefront
    # per SIMD, p = 2 beyond
    for B, L, p in [(128, 100, 3), (256, 1000, 3), (900, 50, 3), (1024, 100, 2), (4096, 50, 2)]:
        rc, pl = binding.sig_plan(None, B, L, 6, 4, 1)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP and pl.prefix_depth == p, (B, L)


def test_no_kernel_uses_private_memory():
    """The build records what the compiler reports for every kernel (registers, LDS, private memory).  A kernel whose
    per-lane arrays end up in private memory (an array the optimiser could not turn into registers, or spilled
    vector registers) still computes the right thing, several times slower, and no parity test would notice."""
    import json
    import os
    from paper_2501_08455_amd import build
    if not os.path.exists(build.RESOURCES):
        pytest.skip("no resource report beside the library (built by another build step)")
    report = json.load(open(build.RESOURCES))
    kernels = [(src, name, use) for src, ks in report.items() for name, use in ks.items()]
    assert len(kernels) > 1000                      # every translation unit reported
    bad = [(src, name) for src, name, use in kernels if use.get("ScratchSize", 0) or use.get("VGPRs Spill", 0)]
    assert not bad, bad[:5]


def test_time_cut_fills_the_chip_on_long_paths():
    """Final mode, paths of 200 increments or more: the planner does not trade the chunks that fill the chip for a
    count that merely packs its workgroups better ((5,4) at 8,192 paths of 2,000 points once got one chunk: three
    wavefronts per SIMD, 1.4 times slower than five chunks)."""
    lanes_for_a_full_chip = 256 * 4 * 64 * 8
    for d, depth, B, L in [(5, 4, 8192, 2000), (5, 4, 8192, 500), (5, 4, 6144, 2000), (3, 5, 8192, 1000), (9, 3, 4096, 2000)]:
        rc, pl = binding.sig_plan(None, B, L, d, depth, 0)
        assert rc == binding.SIG_OK and pl.variant == binding.SIG_VARIANT_ON_CHIP
        lanes = B * d ** pl.prefix_depth * pl.chunks * pl.segments
        assert lanes * 10 >= lanes_for_a_full_chip * 8, (d, depth, B, L, pl.as_dict())
    # short paths keep the count that packs the workgroup (measured faster there)
    rc, pl = binding.sig_plan(None, 8192, 100, 5, 4, 0)
    assert rc == binding.SIG_OK and pl.chunks == 1

"""Python binding of libsig.so: the same entry points as include/sig.h, argument marshalling only.

torch is used for device memory and streams; every arithmetic step runs in the
HIP kernels behind the C ABI.  There is no CPU fallback: if the library is not
built, loading raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsig.so")

SIG_OK = 0
SIG_ERR_INVALID = 1
SIG_ERR_TOO_LARGE = 2
SIG_ERR_ALLOC = 3
SIG_ERR_HIP = 4
SIG_ERR_NO_DEVICE = 5

SIG_ERR_UNSUPPORTED = 6
SIG_NOALLOC_SCRATCH_BYTES = 16 * 1024 * 1024
SIG_VARIANT_AUTO = 0
SIG_VARIANT_HBM_STREAMING = 1
SIG_VARIANT_ON_CHIP = 2
SIG_VARIANT_LEVEL_SCAN = 3


class sig_plan_t(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("prefix_depth", ctypes.c_int32),
                ("chunks", ctypes.c_int32), ("segments", ctypes.c_int32),
                ("threads", ctypes.c_int32), ("tile_steps", ctypes.c_int32),
                ("independent_waves", ctypes.c_int32), ("stagger_ticks", ctypes.c_int32),
                ("tile_loader", ctypes.c_int32), ("shared_chain", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 2)]

    def as_dict(self):
        skip = ("reserved", "independent_waves", "stagger_ticks", "tile_loader", "shared_chain")
        return {k: int(getattr(self, k)) for k, _ in self._fields_ if k not in skip}


class SigError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, sig_strerror(status)))


_lib = None


def load():
    """dlopen libsig.so (building it first only if it does not exist) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    # torch brings its own copy of the HIP runtime; loading it first keeps one runtime in charge of the device
    # (libsig loaded before torch has been seen to end in "no usable HIP device" at sig_create)
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.sig_size.restype = i64
    lib.sig_size.argtypes = [i32, i32]
    lib.sig_create.restype = i32
    lib.sig_create.argtypes = [ctypes.POINTER(vp)]
    lib.sig_destroy.restype = None
    lib.sig_destroy.argtypes = [vp]
    lib.sig_compute.restype = i32
    lib.sig_compute.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, vp]
    lib.sig_compute_noalloc.restype = i32
    lib.sig_compute_noalloc.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, vp]
    lib.sig_plan.restype = i32
    lib.sig_plan.argtypes = [vp, i64, i64, i32, i32, i32, ctypes.POINTER(sig_plan_t)]
    lib.sig_autotune.restype = i32
    lib.sig_autotune.argtypes = [vp, i64, i64, i32, i32, i32, ctypes.POINTER(sig_plan_t),
                                 ctypes.POINTER(ctypes.c_float), vp]
    lib.sig_plan_validate.restype = i32
    lib.sig_plan_validate.argtypes = [i64, i64, i32, i32, i32, ctypes.POINTER(sig_plan_t)]
    lib.sig_plan_footprint.restype = i32
    lib.sig_plan_footprint.argtypes = [i64, i64, i32, i32, i32, ctypes.POINTER(sig_plan_t), ctypes.POINTER(i64),
                                       ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.sig_compute_planned.restype = i32
    lib.sig_compute_planned.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, ctypes.POINTER(sig_plan_t), vp]
    lib.sig_combine.restype = i32
    lib.sig_combine.argtypes = [vp, vp, vp, i64, i32, i32, vp, vp]
    lib.sig_on_chip_available.restype = i32
    lib.sig_on_chip_available.argtypes = [i32, i32, i32]
    lib.sig_backward.restype = i32
    lib.sig_backward.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
    lib.sig_backward_available.restype = i32
    lib.sig_backward_available.argtypes = [i32, i32]
    lib.sig_backward_segments.restype = i32
    lib.sig_backward_segments.argtypes = [ctypes.c_void_p, i64, i64, i32, i32, i32]
    lib.sig_probe_copy.restype = i32
    lib.sig_probe_copy.argtypes = [vp, vp, i64, vp]
    lib.sig_probe_write.restype = i32
    lib.sig_probe_write.argtypes = [vp, i64, i64, vp]
    lib.sig_probe_fma.restype = i32
    lib.sig_probe_fma.argtypes = [vp, i64, i64, i32, i32, vp]
    lib.sig_probe_fma_outer.restype = i32
    lib.sig_probe_fma_outer.argtypes = [vp, i64, i64, i32, vp]
    lib.sig_strerror.restype = ctypes.c_char_p
    lib.sig_strerror.argtypes = [i32]
    _lib = lib
    return lib


# ---------------------------------------------------------------- thin wrappers, one per C entry point
def sig_size(d, depth):
    return int(load().sig_size(int(d), int(depth)))


def sig_strerror(status):
    return load().sig_strerror(int(status)).decode()


def sig_create():
    h = ctypes.c_void_p()
    rc = load().sig_create(ctypes.byref(h))
    if rc != SIG_OK:
        raise SigError(rc, "sig_create")
    return h


def sig_destroy(ctx):
    load().sig_destroy(ctx)


def sig_on_chip_available(d, depth, prefix_depth):
    return bool(load().sig_on_chip_available(int(d), int(depth), int(prefix_depth)))


def sig_plan(ctx, B, L, d, depth, stream_flag):
    """Returns (status, sig_plan_t).  `ctx` may be None."""
    pl = sig_plan_t()
    rc = load().sig_plan(ctx, int(B), int(L), int(d), int(depth), int(stream_flag), ctypes.byref(pl))
    return rc, pl


def sig_autotune(ctx, B, L, d, depth, stream_flag, stream=None):
    """Measure candidate mappings of this shape on the device and remember the fastest in `ctx`.
    Returns (status, plan, microseconds per call)."""
    pl = sig_plan_t()
    us = ctypes.c_float(0.0)
    rc = load().sig_autotune(ctx, int(B), int(L), int(d), int(depth), int(stream_flag), ctypes.byref(pl),
                             ctypes.byref(us), _stream_handle(stream))
    return int(rc), pl, float(us.value)


def sig_plan_validate(B, L, d, depth, stream_flag, plan):
    return int(load().sig_plan_validate(int(B), int(L), int(d), int(depth), int(stream_flag), ctypes.byref(plan)))


def sig_plan_footprint(B, L, d, depth, stream_flag, plan):
    """(status, LDS bytes per workgroup, workgroups, scratch bytes) of a plan, worked out on the host."""
    lds, wgs, scr = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_int64(0)
    rc = load().sig_plan_footprint(int(B), int(L), int(d), int(depth), int(stream_flag), ctypes.byref(plan),
                                   ctypes.byref(lds), ctypes.byref(wgs), ctypes.byref(scr))
    return int(rc), int(lds.value), int(wgs.value), int(scr.value)


def make_plan(variant, prefix_depth=0, chunks=1, segments=1, threads=256, tile_steps=0, independent_waves=0,
              stagger_ticks=0, tile_loader=0, shared_chain=0):
    pl = sig_plan_t()
    pl.independent_waves = int(independent_waves)
    pl.stagger_ticks = int(stagger_ticks)
    pl.tile_loader = int(tile_loader)
    pl.shared_chain = int(shared_chain)
    pl.variant, pl.prefix_depth, pl.chunks = int(variant), int(prefix_depth), int(chunks)
    pl.segments, pl.threads, pl.tile_steps = int(segments), int(threads), int(tile_steps)
    return pl


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def sig_compute(ctx, path, depth, stream_flag, out, stream=None, plan=None):
    """Raw call: `path` [B, L, d] and `out` are contiguous float32 torch tensors on the GPU.  Returns the status."""
    B, L, d = path.shape
    args = [ctx, ctypes.c_void_p(path.data_ptr()), B, L, d, int(depth), int(stream_flag),
            ctypes.c_void_p(out.data_ptr())]
    if plan is None:
        return load().sig_compute(*args, _stream_handle(stream))
    return load().sig_compute_planned(*args, ctypes.byref(plan), _stream_handle(stream))


def sig_compute_noalloc(ctx, path, depth, stream_flag, out, stream=None):
    """Raw call of the entry point that allocates nothing (fixed scratch inside the library).  Returns the status."""
    B, L, d = path.shape
    return load().sig_compute_noalloc(ctx, ctypes.c_void_p(path.data_ptr()), B, L, d, int(depth), int(stream_flag),
                                      ctypes.c_void_p(out.data_ptr()), _stream_handle(stream))


def bind_compute(ctx, path, depth, stream_flag, out, stream=None, plan=None):
    """Marshal the arguments of one sig_compute / sig_compute_planned call once and return a
    zero-argument callable that issues it (for tight loops: no per-call tensor introspection)."""
    lib = load()
    B, L, d = path.shape
    args = [ctx, ctypes.c_void_p(path.data_ptr()), ctypes.c_int64(B), ctypes.c_int64(L), ctypes.c_int(d),
            ctypes.c_int(int(depth)), ctypes.c_int(int(stream_flag)), ctypes.c_void_p(out.data_ptr())]
    if plan is None:
        fn = lib.sig_compute
    else:
        fn = lib.sig_compute_planned
        args.append(ctypes.byref(plan))
    args.append(_stream_handle(stream))
    args = tuple(args)
    keep = (path, out, plan)

    def call(_fn=fn, _args=args, _keep=keep):
        return _fn(*_args)
    return call


def sig_combine(ctx, a, b, d, depth, out, stream=None):
    return load().sig_combine(ctx, ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(b.data_ptr()),
                              a.shape[0], int(d), int(depth), ctypes.c_void_p(out.data_ptr()),
                              _stream_handle(stream))


def sig_backward(ctx, path, depth, stream_flag, out, grad_out, grad_path, stream=None):
    """Raw call: gradient with respect to `path` given the forward result `out` and d(loss)/d(out)."""
    B, L, d = path.shape
    return load().sig_backward(ctx, ctypes.c_void_p(path.data_ptr()), B, L, d, int(depth), int(stream_flag),
                               ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(grad_out.data_ptr()),
                               ctypes.c_void_p(grad_path.data_ptr()), _stream_handle(stream))


def bind_backward(ctx, path, depth, stream_flag, out, grad_out, grad_path, stream=None):
    """sig_backward with the arguments marshalled once (see bind_compute)."""
    lib = load()
    B, L, d = path.shape
    args = (ctx, ctypes.c_void_p(path.data_ptr()), ctypes.c_int64(B), ctypes.c_int64(L), ctypes.c_int(d),
            ctypes.c_int(int(depth)), ctypes.c_int(int(stream_flag)), ctypes.c_void_p(out.data_ptr()),
            ctypes.c_void_p(grad_out.data_ptr()), ctypes.c_void_p(grad_path.data_ptr()), _stream_handle(stream))
    keep = (path, out, grad_out, grad_path)

    def call(_fn=lib.sig_backward, _args=args, _keep=keep):
        return _fn(*_args)
    return call


def sig_backward_available(d, depth):
    return int(load().sig_backward_available(int(d), int(depth)))


def sig_backward_segments(ctx, B, L, d, depth, stream_flag):
    """Time segments sig_backward cuts this shape into (1: uncut, 0: general sweep, < 0: a status); ctx may be None."""
    return int(load().sig_backward_segments(ctx, int(B), int(L), int(d), int(depth), int(stream_flag)))


def sig_probe_copy(dst, src, stream=None):
    """Copy kernel of include/sig_probe.h on two equally sized float32 CUDA tensors."""
    return load().sig_probe_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()),
                                 src.numel(), _stream_handle(stream))


def sig_probe_write(dst, streams=1, stream=None):
    """Write-only kernel of include/sig_probe.h over the float32 CUDA tensor `dst` (plain fill, or `streams`
    sequential write cursors)."""
    return load().sig_probe_write(ctypes.c_void_p(dst.data_ptr()), dst.numel(), int(streams), _stream_handle(stream))


def sig_probe_fma(out, waves, iters, ilp=16, lds_bytes=0, stream=None):
    """FMA loop of include/sig_probe.h; `out` holds waves * 64 floats."""
    return load().sig_probe_fma(ctypes.c_void_p(out.data_ptr()), int(waves), int(iters), int(ilp), int(lds_bytes),
                                _stream_handle(stream))


def sig_probe_fma_outer(out, waves, iters, lds_bytes=0, stream=None):
    """The fused kernels' FMA form (acc[a][b] += g[a] * v[b]) of include/sig_probe.h; `out` holds waves * 64 floats."""
    return load().sig_probe_fma_outer(ctypes.c_void_p(out.data_ptr()), int(waves), int(iters), int(lds_bytes),
                                      _stream_handle(stream))


# ---------------------------------------------------------------- convenience on top of the raw calls
_default_ctx = None


def default_ctx():
    global _default_ctx
    if _default_ctx is None:
        _default_ctx = sig_create()
    return _default_ctx


def signature(path, depth, stream=False, plan=None, ctx=None, out=None):
    """Depth-`depth` signatures of `path` (float32 CUDA tensor [B, L, d]); allocates the output with torch."""
    import torch
    if not path.is_cuda or path.dtype != torch.float32:
        raise ValueError("path must be a float32 tensor on the GPU")
    path = path.contiguous()
    B, L, d = path.shape
    D = sig_size(d, depth)
    if D < 0:
        raise SigError(SIG_ERR_TOO_LARGE, "sig_size")
    shape = (B, L - 1, D) if stream else (B, D)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=path.device)
    rc = sig_compute(ctx or default_ctx(), path, depth, 1 if stream else 0, out, plan=plan)
    if rc != SIG_OK:
        raise SigError(rc, "sig_compute")
    return out

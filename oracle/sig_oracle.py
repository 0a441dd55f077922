"""ctypes binding of oracle/sig_oracle.c (test infrastructure only, see that file's header).

Argument marshalling only; all arithmetic is in the C file.  Inputs are widened
to float64 here (exact for float32 inputs), so the oracle and the GPU see the
same path values.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sig_oracle.c")
_SRC_GRAD = os.path.join(_HERE, "sig_grad_oracle.c")
_LIB = os.path.join(_HERE, "libsig_oracle.so")
_lib = None


def build(force=False):
    """Compile sig_oracle.c and sig_grad_oracle.c with gcc (OpenMP over the batch only)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_GRAD))
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= newest:
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", _LIB, _SRC, _SRC_GRAD]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.oracle_sig_size.restype = ctypes.c_int64
        lib.oracle_sig_size.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.oracle_exp.restype = None
        lib.oracle_exp.argtypes = [dp, ctypes.c_int, ctypes.c_int, dp]
        lib.oracle_mul.restype = None
        lib.oracle_mul.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, dp]
        lib.oracle_signature.restype = ctypes.c_int
        lib.oracle_signature.argtypes = [dp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_int, dp]
        lib.oracle_signature_backward.restype = ctypes.c_int
        lib.oracle_signature_backward.argtypes = [dp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                                  ctypes.c_int, ctypes.c_int, dp, dp]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def sig_size(d, depth):
    """Row length of Eq. 10: d + d^2 + ... + d^depth."""
    return int(_load().oracle_sig_size(int(d), int(depth)))


def num_threads():
    return int(_load().oracle_num_threads())


def level_slices(d, depth):
    """[slice of level 1, ..., slice of level depth] inside an output row."""
    out, start = [], 0
    for n in range(1, depth + 1):
        out.append(slice(start, start + d ** n))
        start += d ** n
    return out


def tensor_exp(v, depth):
    """Eq. 2 of one increment; returns the 1 + D element including level 0."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    d = v.shape[0]
    E = np.empty(1 + sig_size(d, depth), dtype=np.float64)
    _load().oracle_exp(_dptr(v), d, depth, _dptr(E))
    return E


def tensor_mul(a, b, d, depth):
    """Eq. 4 of two 1 + D elements (level 0 in slot 0)."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    n = 1 + sig_size(d, depth)
    assert a.shape == (n,) and b.shape == (n,)
    c = np.empty(n, dtype=np.float64)
    _load().oracle_mul(_dptr(a), _dptr(b), d, depth, _dptr(c))
    return c


def signature(path, depth, stream=False):
    """Depth-`depth` signature of every path in `path` ([B, L, d]), Eq. 3/5/10.

    Returns float64 [B, D] (final) or [B, L-1, D] (stream).
    """
    x = np.ascontiguousarray(path, dtype=np.float64)
    if x.ndim != 3:
        raise ValueError("path must be [B, L, d]")
    B, L, d = x.shape
    D = sig_size(d, depth)
    if D < 0 or L < 2:
        raise ValueError("bad shape")
    shape = (B, L - 1, D) if stream else (B, D)
    out = np.empty(shape, dtype=np.float64)
    if B == 0:
        return out
    rc = _load().oracle_signature(_dptr(x), B, L, d, depth, 1 if stream else 0, _dptr(out))
    if rc != 0:
        raise RuntimeError("oracle_signature failed with code %d" % rc)
    return out


def signature_backward(path, depth, grad_out, stream=False):
    """Gradient of a scalar loss with respect to `path` ([B, L, d]) given `grad_out`, the gradient with
    respect to the output of signature(path, depth, stream) (same shape as that output).  float64 [B, L, d].
    """
    x = np.ascontiguousarray(path, dtype=np.float64)
    g = np.ascontiguousarray(grad_out, dtype=np.float64)
    if x.ndim != 3:
        raise ValueError("path must be [B, L, d]")
    B, L, d = x.shape
    D = sig_size(d, depth)
    if D < 0 or L < 2:
        raise ValueError("bad shape")
    want = (B, L - 1, D) if stream else (B, D)
    if g.shape != want:
        raise ValueError("grad_out must have shape %r" % (want,))
    out = np.empty((B, L, d), dtype=np.float64)
    if B == 0:
        return out
    rc = _load().oracle_signature_backward(_dptr(x), B, L, d, depth, 1 if stream else 0, _dptr(g), _dptr(out))
    if rc != 0:
        raise RuntimeError("oracle_signature_backward failed with code %d" % rc)
    return out

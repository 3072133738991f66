"""CPU fp64 oracle for the transpose convolution of arxiv 2209.03704.

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the CPU-baseline
leg of the benchmark may import this package; the product never does.  The
arithmetic lives in ``kst_oracle.c`` (plain C, literal zero-embedding of
Section 1 followed by the correlation of Eq. 1); this module only compiles it
with gcc, loads it with ctypes and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kst_oracle.c")
_LIB = os.path.join(_HERE, "libkst_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitize_check(exe_path: str, sanitize: bool = True) -> str:
    """Compile sanitize_check.c together with the oracle into an executable: with the address and
    undefined-behaviour sanitizers (the test-suite runs that one), or plainly (the build check)."""
    flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
    subprocess.run(["gcc", "-std=c11", "-fopenmp", "-Wall", "-Wextra"] + flags +
                   ["-o", exe_path, os.path.join(_HERE, "sanitize_check.c"), _SRC, "-lm"], check=True)
    return exe_path


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            dp = ctypes.POINTER(ctypes.c_double)
            ip = ctypes.POINTER(ctypes.c_int32)
            lib.kst_oracle_out_size.argtypes = [ctypes.c_int] * 3
            lib.kst_oracle_out_size.restype = ctypes.c_int
            lib.kst_oracle_threads.argtypes = []
            lib.kst_oracle_threads.restype = ctypes.c_int
            lib.kst_oracle_forward.argtypes = [dp, dp, dp] + [ctypes.c_int] * 6
            lib.kst_oracle_forward.restype = ctypes.c_int
            for fn in (lib.kst_oracle_backward_input, lib.kst_oracle_backward_weight):
                fn.argtypes = [dp, dp, dp] + [ctypes.c_int] * 6
                fn.restype = ctypes.c_int
            lib.kst_oracle_forward_epilogue.argtypes = [dp, dp, dp, dp] + [ctypes.c_int] * 7
            lib.kst_oracle_forward_epilogue.restype = ctypes.c_int
            lib.kst_oracle_forward_planes.argtypes = (
                [dp, dp, dp, ip, ip, ctypes.c_int] + [ctypes.c_int] * 6)
            lib.kst_oracle_forward_planes.restype = ctypes.c_int
            lib.kst_oracle_conventional_ops.argtypes = (
                [ctypes.c_int] * 5 + [ctypes.POINTER(ctypes.c_int64)] * 2)
            lib.kst_oracle_conventional_ops.restype = None
            _lib = lib
    return _lib


def _f64(a, shape_len):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if a.ndim != shape_len:
        raise ValueError("expected %d dimensions, got %r" % (shape_len, a.shape))
    return a


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def out_size(N: int, n: int, P: int = 0) -> int:
    """Output edge (2N-1) + 2P - n + 1 (Section 1: 2N-n without padding)."""
    return _load().kst_oracle_out_size(N, n, P)


def threads() -> int:
    return _load().kst_oracle_threads()


def _dims(x, w):
    B, Cin, N, N2 = x.shape
    Cout, Cin2, n, n2 = w.shape
    if N != N2 or n != n2 or Cin != Cin2:
        raise ValueError("need square maps/kernels with matching Cin: %r %r" % (x.shape, w.shape))
    return B, Cin, Cout, N, n


def forward(x, w, P: int = 0) -> np.ndarray:
    """out[B][Cout][M][M] in fp64 for x[B][Cin][N][N], w[Cout][Cin][n][n]."""
    x = _f64(x, 4)
    w = _f64(w, 4)
    B, Cin, Cout, N, n = _dims(x, w)
    lib = _load()
    M = lib.kst_oracle_out_size(N, n, P)
    if M < 1:
        raise ValueError("kernel larger than the up-sampled map")
    out = np.empty((B, Cout, M, M), dtype=np.float64)
    rc = lib.kst_oracle_forward(_dptr(x), _dptr(w), _dptr(out), B, Cin, Cout, N, n, P)
    if rc != 0:
        raise RuntimeError("kst_oracle_forward failed (%d)" % rc)
    return out


ACT_NONE, ACT_RELU, ACT_TANH = 0, 1, 2


def forward_epilogue(x, w, bias=None, act: int = ACT_NONE, P: int = 0) -> np.ndarray:
    """act(forward(x, w, P) + bias[co]) in fp64; bias: Cout values or None."""
    x = _f64(x, 4)
    w = _f64(w, 4)
    B, Cin, Cout, N, n = _dims(x, w)
    lib = _load()
    M = lib.kst_oracle_out_size(N, n, P)
    if M < 1:
        raise ValueError("kernel larger than the up-sampled map")
    bp = None
    if bias is not None:
        bias = _f64(bias, 1)
        if bias.shape != (Cout,):
            raise ValueError("bias must hold Cout values")
        bp = _dptr(bias)
    out = np.empty((B, Cout, M, M), dtype=np.float64)
    rc = lib.kst_oracle_forward_epilogue(_dptr(x), _dptr(w), bp, _dptr(out), B, Cin, Cout, N, n, P, int(act))
    if rc != 0:
        raise RuntimeError("kst_oracle_forward_epilogue failed (%d)" % rc)
    return out


def forward_planes(x, w, b_idx, co_idx, P: int = 0) -> np.ndarray:
    """Complete output planes (b_idx[k], co_idx[k]) -> [K][M][M], same definition."""
    x = _f64(x, 4)
    w = _f64(w, 4)
    B, Cin, Cout, N, n = _dims(x, w)
    b_idx = np.ascontiguousarray(np.asarray(b_idx, dtype=np.int32))
    co_idx = np.ascontiguousarray(np.asarray(co_idx, dtype=np.int32))
    if b_idx.shape != co_idx.shape or b_idx.ndim != 1:
        raise ValueError("b_idx and co_idx must be equal-length vectors")
    lib = _load()
    M = lib.kst_oracle_out_size(N, n, P)
    if M < 1:
        raise ValueError("kernel larger than the up-sampled map")
    out = np.empty((b_idx.size, M, M), dtype=np.float64)
    ip = ctypes.POINTER(ctypes.c_int32)
    rc = lib.kst_oracle_forward_planes(
        _dptr(x), _dptr(w), _dptr(out), b_idx.ctypes.data_as(ip), co_idx.ctypes.data_as(ip),
        int(b_idx.size), B, Cin, Cout, N, n, P)
    if rc != 0:
        raise RuntimeError("kst_oracle_forward_planes failed (%d)" % rc)
    return out


def conventional_ops(Cin: int, Cout: int, N: int, n: int, P: int = 0):
    """(multiplications, additions) of the conventional method, as Table 4 counts them."""
    m = ctypes.c_int64()
    a = ctypes.c_int64()
    _load().kst_oracle_conventional_ops(Cin, Cout, N, n, P, ctypes.byref(m), ctypes.byref(a))
    return m.value, a.value


def backward_input(g, w, N: int, P: int = 0) -> np.ndarray:
    """d(loss)/d(in) [B][Cin][N][N] in fp64 from g = d(loss)/d(out) [B][Cout][M][M] and w."""
    g = _f64(g, 4)
    w = _f64(w, 4)
    B, Cout, M, M2 = g.shape
    Cout2, Cin, n, n2 = w.shape
    lib = _load()
    if M != M2 or n != n2 or Cout != Cout2 or M != lib.kst_oracle_out_size(N, n, P):
        raise ValueError("shapes of g %r and w %r do not fit N=%d, P=%d" % (g.shape, w.shape, N, P))
    din = np.empty((B, Cin, N, N), dtype=np.float64)
    rc = lib.kst_oracle_backward_input(_dptr(g), _dptr(w), _dptr(din), B, Cin, Cout, N, n, P)
    if rc != 0:
        raise RuntimeError("kst_oracle_backward_input failed (%d)" % rc)
    return din


def backward_weight(x, g, n: int, P: int = 0) -> np.ndarray:
    """d(loss)/d(w) [Cout][Cin][n][n] in fp64 from x [B][Cin][N][N] and g [B][Cout][M][M]."""
    x = _f64(x, 4)
    g = _f64(g, 4)
    B, Cin, N, N2 = x.shape
    B2, Cout, M, M2 = g.shape
    lib = _load()
    if N != N2 or M != M2 or B != B2 or M != lib.kst_oracle_out_size(N, n, P):
        raise ValueError("shapes of x %r and g %r do not fit n=%d, P=%d" % (x.shape, g.shape, n, P))
    dw = np.empty((Cout, Cin, n, n), dtype=np.float64)
    rc = lib.kst_oracle_backward_weight(_dptr(x), _dptr(g), _dptr(dw), B, Cin, Cout, N, n, P)
    if rc != 0:
        raise RuntimeError("kst_oracle_backward_weight failed (%d)" % rc)
    return dw

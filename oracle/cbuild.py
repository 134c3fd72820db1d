"""Build and call the C oracle (test infrastructure; see ``wkv6_oracle.c``)."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wkv6_oracle.c")
_SRC_C2 = os.path.join(_HERE, "finch_c2_oracle.c")
_SRC_KC = os.path.join(_HERE, "key_compress_oracle.c")
_LIB = os.path.join(_HERE, "libwkv6_oracle.so")
_handle = None


def build_oracle(force=False):
    """Compile the oracle's C sources with the host C compiler (no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(_SRC_C2), os.path.getmtime(_SRC_KC))
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-pthread",
               "-ffp-contract=off", "-o", _LIB, _SRC, _SRC_C2, _SRC_KC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def _lib():
    global _handle
    if _handle is None:
        lib = ctypes.CDLL(build_oracle())
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.wkv6_oracle_f64.restype = ctypes.c_int
        lib.wkv6_oracle_f64.argtypes = [ctypes.c_int] * 4 + [fp] * 6 + [dp, dp, ctypes.c_int]
        lib.finch_c2_oracle_f64.restype = ctypes.c_int
        lib.finch_c2_oracle_f64.argtypes = [ctypes.c_int] * 4 + [fp] * 6 + [dp, dp, ctypes.c_int]
        lib.key_compress_oracle_f64.restype = ctypes.c_int
        lib.key_compress_oracle_f64.argtypes = [ctypes.c_longlong, ctypes.c_int, ctypes.c_int, fp, fp, dp,
                                                ctypes.c_int]
        _handle = lib
    return _handle


def _f32(a, shape, name):
    a = np.ascontiguousarray(np.asarray(a), dtype=np.float32)
    if a.shape != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {a.shape}")
    return a


def wkv6_oracle(r, k, v, x, u, state_in=None, nthreads=None):
    """Sequential fp64 WKV6 recurrence (Finch-C2 Time Mixing equations).

    r, k, v, x : [B, T, H, N] arrays whose values are exactly representable in
    float32 (bf16 or fp32 test tensors); u : [H, N]; state_in : [B, H, N, N]
    or None (zero state).  Returns (out [B,T,H,N] float64,
    state_out [B,H,N,N] float64).
    """
    r = np.asarray(r)
    B, T, H, N = r.shape
    r = _f32(r, (B, T, H, N), "r")
    k = _f32(k, (B, T, H, N), "k")
    v = _f32(v, (B, T, H, N), "v")
    x = _f32(x, (B, T, H, N), "x")
    u = _f32(u, (H, N), "u")
    s0 = None if state_in is None else _f32(state_in, (B, H, N, N), "state_in")
    out = np.empty((B, T, H, N), dtype=np.float64)
    sout = np.empty((B, H, N, N), dtype=np.float64)
    if nthreads is None:
        nthreads = os.cpu_count() or 1
    fp = ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _lib().wkv6_oracle_f64(
        B, T, H, N,
        r.ctypes.data_as(fp), k.ctypes.data_as(fp), v.ctypes.data_as(fp),
        x.ctypes.data_as(fp), u.ctypes.data_as(fp),
        s0.ctypes.data_as(fp) if s0 is not None else None,
        out.ctypes.data_as(dp), sout.ctypes.data_as(dp), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"wkv6_oracle_f64 failed with status {rc}")
    return out, sout


def finch_c2_oracle(r, kbar, v, x, uprime, state_in=None, nthreads=None):
    """Sequential fp64 Finch-C2 time mix per head (Finch-C2 Time Mixing equations).

    k_t = kbar_t (1 - w_t);  o_t = r_t . S_{t-1} + u'_t;  S_t = diag(w_t) S_{t-1} + k_t^T v_t.
    r, kbar, v, x, uprime : [B, T, H, N]; state_in : [B, H, N, N] or None.
    Returns (out [B,T,H,N] float64, state_out [B,H,N,N] float64).
    """
    r = np.asarray(r)
    B, T, H, N = r.shape
    r = _f32(r, (B, T, H, N), "r")
    kbar = _f32(kbar, (B, T, H, N), "kbar")
    v = _f32(v, (B, T, H, N), "v")
    x = _f32(x, (B, T, H, N), "x")
    uprime = _f32(uprime, (B, T, H, N), "uprime")
    s0 = None if state_in is None else _f32(state_in, (B, H, N, N), "state_in")
    out = np.empty((B, T, H, N), dtype=np.float64)
    sout = np.empty((B, H, N, N), dtype=np.float64)
    if nthreads is None:
        nthreads = os.cpu_count() or 1
    fp = ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _lib().finch_c2_oracle_f64(
        B, T, H, N,
        r.ctypes.data_as(fp), kbar.ctypes.data_as(fp), v.ctypes.data_as(fp),
        x.ctypes.data_as(fp), uprime.ctypes.data_as(fp),
        s0.ctypes.data_as(fp) if s0 is not None else None,
        out.ctypes.data_as(dp), sout.ctypes.data_as(dp), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"finch_c2_oracle_f64 failed with status {rc}")
    return out, sout


def key_compress_oracle(x, w, nthreads=None):
    """c = x W in fp64 (GOLD Key Compression): x [M, D] (or [..., D]), w [D, C].  Returns [M, C]
    (leading axes of x kept) float64."""
    x = np.asarray(x)
    w = np.asarray(w)
    lead = x.shape[:-1]
    D = x.shape[-1]
    if w.ndim != 2 or w.shape[0] != D:
        raise ValueError(f"w: expected shape ({D}, C), got {w.shape}")
    C = w.shape[1]
    x2 = np.ascontiguousarray(x.reshape(-1, D), dtype=np.float32)
    w2 = np.ascontiguousarray(w, dtype=np.float32)
    M = x2.shape[0]
    c = np.empty((M, C), dtype=np.float64)
    if nthreads is None:
        nthreads = os.cpu_count() or 1
    fp = ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _lib().key_compress_oracle_f64(M, D, C, x2.ctypes.data_as(fp), w2.ctypes.data_as(fp),
                                        c.ctypes.data_as(dp), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"key_compress_oracle_f64 failed with status {rc}")
    return c.reshape(*lead, C)

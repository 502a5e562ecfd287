"""ctypes front end of the plain-C oracle (slide_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It marshals numpy float64 arrays into the C functions; all of the
method's arithmetic lives in slide_oracle.c.  The shared object is compiled with
gcc on first use if it is not there (building the checker is not using it).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slide_oracle.c")
_LIB = os.path.join(_HERE, "libslide_oracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int)


def build(force=False):
    """Compile slide_oracle.c into libslide_oracle.so with gcc (-O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_dp)


def num_threads():
    return int(_load().oracle_num_threads())


def set_num_threads(n):
    _load().oracle_set_num_threads(ctypes.c_int(int(n)))


def reparam(w_learned, ksize):
    """Merged kernel = one-hot shift kernel + learned kernel (Sec. 4.3, Fig. 4)."""
    w, wp = _d(w_learned)
    C = w.shape[0]
    out = np.empty_like(w)
    _load().oracle_reparam(wp, out.ctypes.data_as(_dp), C, int(ksize))
    return out


def deformed_shift(x, w, ksize, two_branch):
    """Materialised deformed shift [B, C, S, H, W] (small inputs only)."""
    x, xp = _d(x)
    w, wp = _d(w)
    B, C, H, W = x.shape
    S = ksize * ksize
    out = np.empty((B, C, S, H, W), dtype=np.float64)
    _load().oracle_deformed_shift(xp, wp, out.ctypes.data_as(_dp), B, H, W, C, int(ksize),
                                  int(bool(two_branch)))
    return out


def fwd(q, k, v, wk, wv, bias, heads, ksize, two_branch=False, return_attn=False, return_lse=False):
    """Forward.  wk/wv are merged kernels, or learned ones when two_branch.

    Returns out, then attn [B, heads, S, H, W] if return_attn, then lse [B, heads, H, W]
    (log of the softmax denominator of Eq. 2) if return_lse."""
    q, qp = _d(q); k, kp = _d(k); v, vp = _d(v)
    wk, wkp = _d(wk); wv, wvp = _d(wv)
    B, C, H, W = q.shape
    S = ksize * ksize
    bp = None
    if bias is not None:
        bias, bp = _d(bias)
    out = np.empty_like(q)
    attn = np.empty((B, heads, S, H, W), dtype=np.float64) if return_attn else None
    lse = np.empty((B, heads, H, W), dtype=np.float64) if return_lse else None
    _load().oracle_fwd(qp, kp, vp, wkp, wvp, bp, out.ctypes.data_as(_dp),
                       attn.ctypes.data_as(_dp) if return_attn else None,
                       lse.ctypes.data_as(_dp) if return_lse else None,
                       B, H, W, C, int(heads), int(ksize), int(bool(two_branch)))
    res = (out,) + ((attn,) if return_attn else ()) + ((lse,) if return_lse else ())
    return res if len(res) > 1 else out


def fwd_samples(q, k, v, wk, wv, bias, heads, ksize, positions, two_branch=False):
    """Forward at sampled (b, head, i, j) rows of `positions`; returns [n, d]."""
    q, qp = _d(q); k, kp = _d(k); v, vp = _d(v)
    wk, wkp = _d(wk); wv, wvp = _d(wv)
    B, C, H, W = q.shape
    bp = None
    if bias is not None:
        bias, bp = _d(bias)
    pos = np.ascontiguousarray(positions, dtype=np.int32).reshape(-1, 4)
    d = C // heads
    out = np.empty((pos.shape[0], d), dtype=np.float64)
    _load().oracle_fwd_samples(qp, kp, vp, wkp, wvp, bp, pos.ctypes.data_as(_ip),
                               int(pos.shape[0]), out.ctypes.data_as(_dp),
                               B, H, W, C, int(heads), int(ksize), int(bool(two_branch)))
    return out


def bwd(dout, q, k, v, wk, wv, bias, heads, ksize):
    """Backward of the merged form: returns dq, dk, dv, dwk, dwv, dbias."""
    do, dop = _d(dout)
    q, qp = _d(q); k, kp = _d(k); v, vp = _d(v)
    wk, wkp = _d(wk); wv, wvp = _d(wv)
    B, C, H, W = q.shape
    S = ksize * ksize
    bp = None
    if bias is not None:
        bias, bp = _d(bias)
    dq = np.empty_like(q); dk = np.empty_like(q); dv = np.empty_like(q)
    dwk = np.empty_like(wk); dwv = np.empty_like(wv)
    dbias = np.empty((heads, S), dtype=np.float64)
    _load().oracle_bwd(dop, qp, kp, vp, wkp, wvp, bp,
                       dq.ctypes.data_as(_dp), dk.ctypes.data_as(_dp), dv.ctypes.data_as(_dp),
                       dwk.ctypes.data_as(_dp), dwv.ctypes.data_as(_dp),
                       dbias.ctypes.data_as(_dp),
                       B, H, W, C, int(heads), int(ksize))
    return dq, dk, dv, dwk, dwv, dbias

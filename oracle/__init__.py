"""CPU oracle for bucketed approximate top-k (arxiv 2412.04358).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never imports or calls it, and this
package imports nothing from the GPU package.

`approx_topk` / `exact_topk` wrap the plain C definition in topk_oracle.c (Section 2,
Stage 1 / Stage 2; Appendix A.1 interleaved buckets).  `recall` holds the expected
recall formulas of Appendix C.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "topk_oracle.c")
_LIB = os.path.join(_HERE, "libtopk_oracle.so")

F32 = 0
BF16 = 1
INTERLEAVED = 0  # bucket of element i is i mod b (Appendix A.1; the paper's experiments)
CONTIGUOUS = 1   # bucket of element i is floor(b*i/n) (Appendix A.1)

_lib = None


def build(force: bool = False) -> str:
    """Compile topk_oracle.c with gcc into a shared object next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, vp, i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.orc_approx_topk.argtypes = [vp, i64, i64, i64, i64, i64, i32, vp, vp, vp, vp, i32]
        lib.orc_approx_topk.restype = i32
        lib.orc_approx_topk_assign.argtypes = [vp, i64, i64, i64, i64, i64, i32, i32, vp, vp, vp, vp, i32]
        lib.orc_approx_topk_assign.restype = i32
        lib.orc_exact_topk.argtypes = [vp, i64, i64, i64, i32, vp, vp, i32]
        lib.orc_exact_topk.restype = i32
        _lib = lib
    return _lib


def _prep(x):
    """x: 2-D numpy array, float32 (f32 data) or uint16 (bf16 bit patterns)."""
    x = np.ascontiguousarray(x)
    if x.ndim != 2:
        raise ValueError("x must be 2-D (m, n)")
    if x.dtype == np.float32:
        return x, F32
    if x.dtype == np.uint16:
        return x, BF16
    raise TypeError("x must be float32, or uint16 holding bf16 bit patterns")


def approx_topk(x, k, b, k_b, threads=1, return_candidates=False, assignment=INTERLEAVED):
    """Bucketed approximate top-k of every row of x.

    assignment: INTERLEAVED (i mod b) or CONTIGUOUS (floor(b*i/n)), Appendix A.1.

    Returns (vals, idx), each (m, k); vals has x's dtype and carries the original
    bits, idx is int32.  With return_candidates also returns the Stage-1 output
    (cand_vals, cand_idx), each (m, b*k_b), bucket-major.
    """
    x, dt = _prep(x)
    m, n = x.shape
    vals = np.empty((m, k), dtype=x.dtype)
    idx = np.empty((m, k), dtype=np.int32)
    cv = ci = None
    cvp = cip = None
    if return_candidates:
        cv = np.empty((m, b * k_b), dtype=x.dtype)
        ci = np.empty((m, b * k_b), dtype=np.int32)
        cvp, cip = cv.ctypes.data, ci.ctypes.data
    rc = _load().orc_approx_topk_assign(x.ctypes.data, m, n, k, b, k_b, dt, int(assignment), vals.ctypes.data,
                                        idx.ctypes.data, cvp, cip, int(threads))
    if rc != 0:
        raise ValueError("oracle approx_topk rejected its arguments (code %d)" % rc)
    if return_candidates:
        return vals, idx, cv, ci
    return vals, idx


def exact_topk(x, k, threads=1):
    """Exact top-k of every row: full sort by (value descending, index ascending)."""
    x, dt = _prep(x)
    m, n = x.shape
    vals = np.empty((m, k), dtype=x.dtype)
    idx = np.empty((m, k), dtype=np.int32)
    rc = _load().orc_exact_topk(x.ctypes.data, m, n, k, dt, vals.ctypes.data, idx.ctypes.data, int(threads))
    if rc != 0:
        raise ValueError("oracle exact_topk rejected its arguments (code %d)" % rc)
    return vals, idx

"""ctypes binding of the C ABI declared in include/approx_topk.h.

Argument marshalling only: every step of the method runs in the HIP library.  The
library is looked up inside the package (paper_2412_04358_amd/lib/libapprox_topk.so,
built by __graft_entry__.build()); if it is missing the first call raises - there is
no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "lib", "libapprox_topk.so")

ATK_F32 = 0
ATK_BF16 = 1
ATK_INTERLEAVED = 0
ATK_CONTIGUOUS = 1

_lib = None


class ApproxTopkError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("approx_topk library error %d: %s" % (code, message))
        self.code = code


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load (once) and return the ctypes handle of the HIP library."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            "HIP library %s is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "at the repository root. There is no CPU fallback." % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.approx_topk.argtypes = [vp, i64, i64, i64, i64, i64, ci, vp, vp, vp]
    lib.approx_topk.restype = ci
    lib.approx_topk_noalloc.argtypes = [vp, i64, i64, i64, i64, i64, ci, vp, vp, vp]
    lib.approx_topk_noalloc.restype = ci
    lib.approx_topk_assign.argtypes = [vp, i64, i64, i64, i64, i64, ci, ci, vp, vp, vp]
    lib.approx_topk_assign.restype = ci
    lib.atk_plan_describe_assign.argtypes = [i64, i64, i64, i64, i64, ci, ci, ctypes.c_char_p, i64]
    lib.atk_plan_describe_assign.restype = ci
    lib.exact_topk.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp]
    lib.exact_topk.restype = ci
    lib.atk_strerror.argtypes = [ci]
    lib.atk_strerror.restype = ctypes.c_char_p
    lib.atk_last_hip_error.argtypes = []
    lib.atk_last_hip_error.restype = ci
    lib.atk_check_approx.argtypes = [i64, i64, i64, i64, i64, ci]
    lib.atk_check_approx.restype = ci
    lib.atk_check_exact.argtypes = [i64, i64, i64, ci]
    lib.atk_check_exact.restype = ci
    lib.atk_stage2_max_candidates.argtypes = []
    lib.atk_stage2_max_candidates.restype = i64
    lib.atk_workspace_bytes.argtypes = [i64, i64, i64, i64, i64, ci]
    lib.atk_workspace_bytes.restype = i64
    lib.atk_workspace_bytes_assign.argtypes = [i64, i64, i64, i64, i64, ci, ci]
    lib.atk_workspace_bytes_assign.restype = i64
    lib.atk_exact_workspace_bytes.argtypes = [i64, i64, i64, ci]
    lib.atk_exact_workspace_bytes.restype = i64
    lib.atk_exact_workspace_parts.argtypes = [i64, i64, i64, ci, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.atk_exact_workspace_parts.restype = ci
    lib.atk_plan_describe.argtypes = [i64, i64, i64, i64, i64, ci, ctypes.c_char_p, i64]
    lib.atk_plan_describe.restype = ci
    lib.atk_set_plan_override.argtypes = [ctypes.c_char_p]
    lib.atk_set_plan_override.restype = ci
    dbl = ctypes.c_double
    lib.atk_expected_recall.argtypes = [i64, i64, i64]
    lib.atk_expected_recall.restype = dbl
    lib.atk_worst_case_recall.argtypes = [i64, i64, i64, i64]
    lib.atk_worst_case_recall.restype = dbl
    lib.atk_estimate_us.argtypes = [i64, i64, i64, i64, i64, ci]
    lib.atk_estimate_us.restype = dbl
    lib.atk_advise.argtypes = [i64, i64, i64, ci, dbl, ctypes.POINTER(i64), ctypes.POINTER(i64),
                               ctypes.POINTER(dbl), ctypes.POINTER(dbl)]
    lib.atk_advise.restype = ci
    lib.atk_trace_bytes.argtypes = [i64, i64, i64, i64, i64, ci]
    lib.atk_trace_bytes.restype = i64
    lib.atk_trace_approx.argtypes = [vp, i64, i64, i64, i64, i64, ci, vp, vp, vp, i64, vp]
    lib.atk_trace_approx.restype = ci
    lib.atk_read_ceiling.argtypes = [vp, i64, vp, vp]
    lib.atk_read_ceiling.restype = ci
    lib.atk_copy.argtypes = [vp, vp, i64, vp]
    lib.atk_copy.restype = ci
    lib.atk_sleep.argtypes = [i64, vp]
    lib.atk_sleep.restype = ci
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().atk_strerror(code).decode()


def _check(code: int):
    if code != 0:
        lib = load_library()
        msg = lib.atk_strerror(code).decode()
        if code == -6:
            msg += " (hipError_t %d)" % lib.atk_last_hip_error()
        raise ApproxTopkError(code, msg)


def approx_topk_raw(x_ptr, m, n, k, b, k_b, dtype, out_vals_ptr, out_idx_ptr, stream_ptr=0) -> int:
    """The C call itself on raw device addresses; returns the library's status code."""
    return load_library().approx_topk(x_ptr, m, n, k, b, k_b, dtype, out_vals_ptr, out_idx_ptr, stream_ptr)


def approx_topk_noalloc_raw(x_ptr, m, n, k, b, k_b, dtype, out_vals_ptr, out_idx_ptr, stream_ptr=0) -> int:
    """approx_topk_noalloc on raw device addresses: the caller brings the outputs, the library allocates nothing."""
    return load_library().approx_topk_noalloc(x_ptr, m, n, k, b, k_b, dtype, out_vals_ptr, out_idx_ptr, stream_ptr)


def approx_topk_assign_raw(x_ptr, m, n, k, b, k_b, dtype, assignment, out_vals_ptr, out_idx_ptr, stream_ptr=0) -> int:
    return load_library().approx_topk_assign(x_ptr, m, n, k, b, k_b, dtype, assignment, out_vals_ptr, out_idx_ptr,
                                             stream_ptr)


def exact_topk_raw(x_ptr, m, n, k, dtype, out_vals_ptr, out_idx_ptr, stream_ptr=0) -> int:
    return load_library().exact_topk(x_ptr, m, n, k, dtype, out_vals_ptr, out_idx_ptr, stream_ptr)


def _dtype_code(t):
    import torch

    if t.dtype == torch.float32:
        return ATK_F32
    if t.dtype == torch.bfloat16:
        return ATK_BF16
    raise TypeError("x must be float32 or bfloat16")


def _tensor_args(x):
    import torch

    if not x.is_cuda:
        raise ValueError("x must live on the GPU")
    if x.dim() != 2 or not x.is_contiguous():
        raise ValueError("x must be a contiguous (m, n) tensor")
    return torch, x.shape[0], x.shape[1], _dtype_code(x)


def approx_topk(x, k, b, k_b, out=None, assignment=None):
    """Bucketed approximate top-k of every row of a GPU tensor x (m, n), f32 or bf16.

    Returns (vals, idx): vals (m, k) of x's dtype, idx (m, k) int32.  Runs on torch's
    current stream of x's device.  assignment: None calls approx_topk (interleaved buckets);
    ATK_INTERLEAVED / ATK_CONTIGUOUS call approx_topk_assign.
    """
    torch, m, n, dt = _tensor_args(x)
    with torch.cuda.device(x.device):
        if out is None:
            vals = torch.empty((m, k), dtype=x.dtype, device=x.device)
            idx = torch.empty((m, k), dtype=torch.int32, device=x.device)
        else:
            vals, idx = out
        stream = torch.cuda.current_stream(x.device).cuda_stream
        if assignment is None:
            _check(approx_topk_raw(x.data_ptr(), m, n, k, b, k_b, dt, vals.data_ptr(), idx.data_ptr(), stream))
        else:
            _check(approx_topk_assign_raw(x.data_ptr(), m, n, k, b, k_b, dt, int(assignment), vals.data_ptr(),
                                          idx.data_ptr(), stream))
    return vals, idx


def exact_topk(x, k, out=None):
    """Exact top-k (largest first) of every row of a GPU tensor x (m, n)."""
    torch, m, n, dt = _tensor_args(x)
    with torch.cuda.device(x.device):
        if out is None:
            vals = torch.empty((m, k), dtype=x.dtype, device=x.device)
            idx = torch.empty((m, k), dtype=torch.int32, device=x.device)
        else:
            vals, idx = out
        stream = torch.cuda.current_stream(x.device).cuda_stream
        _check(exact_topk_raw(x.data_ptr(), m, n, k, dt, vals.data_ptr(), idx.data_ptr(), stream))
    return vals, idx


def plan_describe(m, n, k, b, k_b, dtype=ATK_F32, assignment=ATK_INTERLEAVED) -> str:
    buf = ctypes.create_string_buffer(512)
    _check(load_library().atk_plan_describe_assign(m, n, k, b, k_b, dtype, assignment, buf, 512))
    return buf.value.decode()


def set_plan_override(spec=None) -> None:
    """Launch-plan override in the syntax of ATK_PLAN ("T=256,S=2"); None removes it.  For sweeps and tests."""
    _check(load_library().atk_set_plan_override(spec.encode() if spec else None))


def expected_recall(k, b, k_b) -> float:
    """Eq. 1 of Appendix C as the library computes it (host only)."""
    return load_library().atk_expected_recall(k, b, k_b)


def worst_case_recall(n, k, b, k_b) -> float:
    """Eq. 2 of Appendix C as the library computes it (host only); -1 for arguments it is not stated for."""
    return load_library().atk_worst_case_recall(n, k, b, k_b)


def estimate_us(m, n, k, b, k_b, dtype=ATK_F32) -> float:
    return load_library().atk_estimate_us(m, n, k, b, k_b, dtype)


def advise(m, n, k, dtype=ATK_F32, min_recall=0.9):
    """(b, k_b, expected recall, estimated microseconds, reached) for a recall target."""
    b, kb = ctypes.c_int64(0), ctypes.c_int64(0)
    rec, us = ctypes.c_double(0.0), ctypes.c_double(0.0)
    rc = load_library().atk_advise(m, n, k, dtype, float(min_recall), ctypes.byref(b), ctypes.byref(kb),
                                   ctypes.byref(rec), ctypes.byref(us))
    if rc < 0:
        _check(rc)
    return b.value, kb.value, rec.value, us.value, rc == 0

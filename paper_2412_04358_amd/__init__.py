"""MI355X (gfx950) bucketed approximate top-k, after arxiv 2412.04358.

`approx_topk` / `exact_topk` call the hand-written HIP library through its C ABI; the
library is loaded on first use and a missing build raises, there is no CPU fallback.
"""
from .binding import (  # noqa: F401
    ATK_BF16,
    ATK_CONTIGUOUS,
    ATK_F32,
    ATK_INTERLEAVED,
    ApproxTopkError,
    advise,
    approx_topk,
    approx_topk_assign_raw,
    approx_topk_noalloc_raw,
    approx_topk_raw,
    estimate_us,
    exact_topk,
    exact_topk_raw,
    expected_recall,
    lib_path,
    load_library,
    plan_describe,
    set_plan_override,
    strerror,
    worst_case_recall,
)

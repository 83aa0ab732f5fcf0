"""approx_topk_noalloc (the entry point for callers that cannot allocate: its scratch is a fixed array inside
the library) against approx_topk, through the C ABI, bit for bit, on plans whose workgroups hand partial
lists over through that scratch; two calls in a row, the second with a smaller input, and the first again."""
import numpy as np
import pytest
import torch

import paper_2412_04358_amd as atk
from paper_2412_04358_amd import workloads

pytestmark = pytest.mark.gpu


def _both(lib, x, k, b, k_b):
    """(vals, idx) of approx_topk and of approx_topk_noalloc on the same device tensor, as numpy bit patterns."""
    m, n = x.shape
    dt = atk.ATK_F32 if x.dtype == torch.float32 else atk.ATK_BF16
    stream = torch.cuda.current_stream().cuda_stream
    res = []
    for fn in (lib.approx_topk, lib.approx_topk_noalloc):
        vals = torch.full((m, k), -7.0, dtype=x.dtype, device=x.device)
        idx = torch.full((m, k), -7, dtype=torch.int32, device=x.device)
        rc = fn(x.data_ptr(), m, n, k, b, k_b, dt, vals.data_ptr(), idx.data_ptr(), stream)
        assert rc == 0, atk.strerror(rc)
        torch.cuda.synchronize()
        v = vals.cpu()
        res.append((v.numpy().view(np.uint32) if v.dtype == torch.float32 else v.view(torch.int16).numpy(), idx.cpu().numpy()))
    return res


def test_noalloc_matches_approx_topk_on_two_calls_in_a_row():
    assert torch.cuda.is_available(), "this test needs the MI355X"
    lib = atk.load_library()
    # (rows, row length, dtype, k, b, k_b): first the larger input, then a smaller one, then the first again;
    # every plan uses scratch (row splits and a ticket, the second and third with Stage 2 in the last workgroup)
    calls = [
        (8, 1 << 20, "f32", 64, 64, 1),
        (3, 1 << 17, "f32", 64, 512, 1),
        (5, 1 << 18, "bf16", 100, 64, 4),
        (8, 1 << 20, "f32", 64, 64, 1),
        (16, 1 << 16, "f32", 64, 64, 1),
    ]
    for i, (m, n, dtype, k, b, k_b) in enumerate(calls):
        dt = atk.ATK_F32 if dtype == "f32" else atk.ATK_BF16
        # (the plan of the entry point under test: it takes no plans with mailboxes, which have to be zero between
        # calls - what "HF=0" says; approx_topk beside it runs the library's own choice)
        atk.set_plan_override("HF=0")
        plan = atk.plan_describe(m, n, k, b, k_b, dt)
        atk.set_plan_override("")
        print("noalloc call %d: %s plan=[%s]" % (i, (m, n, dtype, k, b, k_b), plan), flush=True)
        assert " scratch=1 " in plan, plan
        ws = lib.atk_workspace_bytes(m, n, k, b, k_b, dt)
        assert 0 < ws <= 16 << 20
        x = workloads.normal_rows(m, n, seed=900 + i, dtype=dtype).cuda()
        (rv, ri), (nv, ni) = _both(lib, x, k, b, k_b)
        assert np.array_equal(ni, ri), "call %d: indices differ from approx_topk" % i
        assert np.array_equal(nv, rv), "call %d: values differ from approx_topk" % i
        assert (ri >= 0).all() and (ri < n).all()
    # a plan without scratch goes through as well (nothing of the array is touched)
    x = workloads.normal_rows(128, 65536, seed=910).cuda()
    (rv, ri), (nv, ni) = _both(lib, x, 16384, 16384, 1)
    assert np.array_equal(ni, ri) and np.array_equal(nv, rv)

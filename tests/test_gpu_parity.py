"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, bit for bit.

Values are compared as raw bits and indices as int32; both are unique under the tie rule
(equal values -> lower index), so a plain array comparison is the whole test.
"""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2412_04358_amd as atk
from paper_2412_04358_amd import workloads

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    atk.load_library()  # raises if the HIP library is not built: no fallback


def as_bits(t):
    a = t.detach().cpu().contiguous()
    if a.dtype == torch.float32:
        return a.numpy().view(np.uint32)
    return a.view(torch.int16).numpy().view(np.uint16)


def to_gpu(x_cpu, shift=0):
    """x on the GPU; shift > 0: in a buffer whose first element lies that many elements past a 256-byte boundary."""
    if not shift:
        return x_cpu.cuda()
    buf = torch.empty(x_cpu.numel() + shift, dtype=x_cpu.dtype, device="cuda")
    view = buf[shift:].view(x_cpu.shape)
    view.copy_(x_cpu)
    assert view.is_contiguous() and view.data_ptr() == buf.data_ptr() + shift * x_cpu.element_size()
    return view


def run_case(x_cpu, k, b, k_b, rows=None, tag="", assignment=None, shift=0):
    print("case %s shape=%s dtype=%s k=%d b=%d k_b=%d plan=[%s]" % (
        tag, tuple(x_cpu.shape), x_cpu.dtype, k, b, k_b,
        atk.plan_describe(x_cpu.shape[0], x_cpu.shape[1], k, b, k_b,
                          atk.ATK_F32 if x_cpu.dtype == torch.float32 else atk.ATK_BF16,
                          assignment or atk.ATK_INTERLEAVED)), flush=True)
    xg = to_gpu(x_cpu, shift)
    vals, idx = atk.approx_topk(xg, k, b, k_b, assignment=assignment)
    torch.cuda.synchronize()
    gv, gi = as_bits(vals), idx.cpu().numpy()
    xo = workloads.as_numpy_bits(x_cpu)
    if rows is not None:
        xo, gv, gi = xo[rows], gv[rows], gi[rows]
    ov, oi = oracle.approx_topk(xo, k, b, k_b, threads=THREADS,
                                assignment=oracle.CONTIGUOUS if assignment == atk.ATK_CONTIGUOUS else oracle.INTERLEAVED)
    ovb = ov.view(np.uint32) if ov.dtype == np.float32 else ov
    if not np.array_equal(gi, oi):
        bad = np.argwhere(gi != oi)
        same_set = all(sorted(gi[r].tolist()) == sorted(oi[r].tolist()) for r in np.unique(bad[:, 0])[:8])
        raise AssertionError("indices differ at %d places, first %s: gpu %d oracle %d (same set per row: %s)" % (
            len(bad), bad[0], gi[tuple(bad[0])], oi[tuple(bad[0])], same_set))
    assert np.array_equal(gv, ovb), "values differ"


def run_exact(x_cpu, k, rows=None, shift=0):
    print("exact shape=%s dtype=%s k=%d shift=%d" % (tuple(x_cpu.shape), x_cpu.dtype, k, shift), flush=True)
    xg = to_gpu(x_cpu, shift)
    vals, idx = atk.exact_topk(xg, k)
    torch.cuda.synchronize()
    gv, gi = as_bits(vals), idx.cpu().numpy()
    xo = workloads.as_numpy_bits(x_cpu)
    if rows is not None:
        xo, gv, gi = xo[rows], gv[rows], gi[rows]
    ov, oi = oracle.exact_topk(xo, k, threads=THREADS)
    ovb = ov.view(np.uint32) if ov.dtype == np.float32 else ov
    assert np.array_equal(gi, oi), "exact_topk indices differ"
    assert np.array_equal(gv, ovb), "exact_topk values differ"


# ------------------------------------------------------------------------------- the five configurations
def test_cfg1():
    x = workloads.config_input("cfg1")
    for k, b, k_b in workloads.CONFIGS["cfg1"]["cases"]:
        run_case(x, k, b, k_b, tag="cfg1")


def test_cfg2_small_k_sweep_b():
    x = workloads.config_input("cfg2")
    for k, b, k_b in workloads.CONFIGS["cfg2"]["cases"]:
        run_case(x, k, b, k_b, tag="cfg2")


def test_cfg3_large_k_sweep_kb():
    x = workloads.config_input("cfg3")
    for k, b, k_b in workloads.CONFIGS["cfg3"]["cases"]:
        run_case(x, k, b, k_b, tag="cfg3")


def test_cfg4_long_rows():
    """Every row of every case: these are the plans whose workgroups hand lists over through scratch and a ticket,
    and a fault in the hand-over would hit any row."""
    x = workloads.config_input("cfg4")
    for k, b, k_b in workloads.CONFIGS["cfg4"]["cases"]:
        run_case(x, k, b, k_b, tag="cfg4")


def test_cfg5_attention_scores_bf16():
    x = workloads.config_input("cfg5")
    for k, b, k_b in workloads.CONFIGS["cfg5"]["cases"]:
        run_case(x, k, b, k_b, tag="cfg5")


def test_vocab_shape_bf16():
    x = workloads.config_input("vocab")
    for k, b, k_b in workloads.CONFIGS["vocab"]["cases"]:
        run_case(x, k, b, k_b, tag="vocab")


def test_kg_shape_bf16():
    x = workloads.config_input("kg")
    for k, b, k_b in workloads.CONFIGS["kg"]["cases"]:
        run_case(x, k, b, k_b, tag="kg")


# ------------------------------------------------------------------------------- shapes spanning tiles and tails
SHAPES = [
    # (m, n, k, b, k_b)
    (3, 12288, 96, 96, 1),        # b not a power of two, vector columns (96 % 4 == 0)
    (3, 12288, 48, 96, 1),        # ... with Stage 2
    (2, 4098, 6, 6, 1),           # scalar columns, lanes idle in the last phase
    (2, 4098, 683, 683, 1),       # scalar columns, b > threads, ragged last column block
    (5, 8192, 8, 8, 1),           # two column groups, 128 phases
    (5, 8192, 4, 4, 1),           # one column group
    (5, 8192, 2, 2, 1),
    (5, 8192, 1, 1, 1),           # arg-max of the row
    (2, 8192, 16, 1, 16),         # b = 1: exact top-16 through one bucket
    (3, 20480, 320, 160, 2),
    (3, 20480, 100, 160, 2),      # Stage 2 with k not a power of two
    (3, 20480, 15, 5, 3),         # k_b not a power of two
    (3, 20480, 33, 20, 3),
    (4, 16384, 1024, 256, 4),
    (4, 16384, 700, 256, 4),
    (4, 16384, 512, 64, 8),
    (4, 16384, 2048, 128, 16),
    (4, 16384, 100, 128, 16),
    (5, 1677, 371, 371, 2),       # Stage 2 asks for 384 lanes, few rows ask for smaller workgroups: whole wavefronts
    (4, 16384, 16384, 16384, 1),  # bucket length 1: identity
    (4, 16384, 8192, 8192, 1),
    (4, 16384, 4096, 1024, 4),    # bucket length 16, keep 4
    (4, 16384, 16384, 1024, 16),  # k_b = n/b: every element, each bucket sorted
    (130, 4096, 64, 128, 1),
    (1, 1 << 18, 64, 64, 1),      # one long row: many row splits
    (1, 1 << 18, 64, 512, 1),
    (1, 1 << 18, 256, 32, 8),
    # n not a multiple of b: short buckets (Figure 2), vector and scalar columns
    (3, 4100, 64, 64, 1),         # remainder 4: one whole vector of the ragged row
    (3, 4102, 64, 64, 1),         # n % 4 != 0: scalar columns
    (3, 4136, 48, 64, 1),         # remainder 40, n % 8 == 0, Stage 2
    (2, 20000, 192, 96, 2),       # remainder 32
    (2, 20004, 100, 96, 3),       # remainder 36 with Stage 2, k_b not a power of two
    (5, 1000, 30, 30, 1),         # small odd shapes
    (5, 1001, 45, 15, 3),
    (2, 70001, 250, 250, 1),      # b > 64 column groups, scalar
    (2, 66000, 512, 128, 4),      # remainder 80 of 128 columns: partial vectors
    (1, 128256, 256, 512, 1),     # vocabulary-sized row, b*k_b/k = 2
    (1, 128256, 256, 1000, 2),    # b does not divide n
    # rows that start off a vector boundary (n % V != 0, b % V == 0): read from the aligned address before
    (5, 4099, 1024, 1024, 1),     # every lane owns whole buckets, outputs rotated
    (5, 8197, 2048, 1024, 2),
    (7, 4101, 64, 64, 1),         # lanes share columns
    (7, 4103, 48, 64, 1),         # ... with Stage 2
    (6, 12289, 512, 512, 1),
    (9, 5003, 96, 32, 3),
    (4, 66001, 512, 128, 4),
    (3, 65535, 16380, 16380, 1),  # the ragged last matrix row wraps into one more full row
    (3, 40003, 16000, 8000, 2),
    (7, 4159, 64, 64, 1),         # n % b = b - 1: with the rotation the last matrix row fills up
    (5, 4159, 128, 64, 2),
    (5, 5119, 1024, 1024, 1),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_shapes(dtype):
    for i, (m, n, k, b, k_b) in enumerate(SHAPES):
        x = workloads.normal_rows(m, n, seed=100 + i, dtype=dtype)
        run_case(x, k, b, k_b, tag="shape%d" % i)


@pytest.mark.parametrize("plan", ["T=64,S=1", "T=64,S=7", "T=128,S=3", "T=256,S=2", "T=256,S=64", "T=512,S=1", "T=1024,S=2", "T=1024,S=5",
                                  "P=2", "P=4", "T=128,P=2,S=3"])
def test_forced_plans(plan, plan_override):
    """The same results whatever the launch geometry (threads per workgroup, row splits)."""
    plan_override(plan)
    for i, (m, n, k, b, k_b) in enumerate([(3, 32768, 64, 64, 1), (3, 32768, 64, 256, 1), (3, 32768, 2048, 2048, 1),
                                           (3, 32768, 128, 64, 2), (3, 32768, 100, 32, 4), (2, 32768, 64, 8, 8),
                                           (2, 32768, 200, 16, 16), (3, 32771, 2048, 2048, 1), (3, 32770, 128, 64, 2),
                                           (3, 32773, 4096, 1024, 4), (2, 32768, 4096, 512, 8), (2, 32772, 8192, 512, 16),
                                           (2, 32768, 100, 512, 8)]):
        for dtype in ["f32", "bf16"]:
            x = workloads.normal_rows(m, n, seed=200 + i, dtype=dtype)
            run_case(x, k, b, k_b, tag=plan)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_column_split_plans(dtype):
    """k_b = 1 without Stage 2 on rows that start on 128-byte lines: the workgroups of a row take 128-byte
    pieces of the matrix rows - whole buckets each, no hand-over - alone (enough rows) or with row splits
    on top (few rows); ragged last matrix rows, ties and special values included.  Also with P forced."""
    es = 4 if dtype == "f32" else 2
    dt = atk.ATK_F32 if dtype == "f32" else atk.ATK_BF16
    cases = [(128, 65536, 64, 64, 1), (128, 65536, 128, 128, 1), (128, 65536, 512, 512, 1), (5, 1000000, 64, 64, 1),
             (3, 65600, 128, 128, 1), (33, 16384, 96, 96, 1), (1, 1 << 20, 64, 64, 1), (8, 1 << 18, 256, 256, 1)]
    split = 0
    for i, (m, n, k, b, k_b) in enumerate(cases):
        assert (n * es) % 128 == 0
        plan = atk.plan_describe(m, n, k, b, k_b, dt)
        split += " colblocks=1 " not in plan and " direct=0" in plan
        run_case(workloads.normal_rows(m, n, seed=700 + i, dtype=dtype), k, b, k_b, tag="colsplit")
    assert split >= 4  # the plans this test is about are the ones the library picks
    run_case(workloads.few_levels(6, 65536, levels=3, seed=720, dtype=dtype), 64, 64, 1, tag="colsplit ties")
    run_case(workloads.special_values(6, 65536, seed=721, dtype=dtype), 128, 128, 1, tag="colsplit specials")


@pytest.mark.parametrize("plan", ["P=8", "P=16,T=256", "P=32,T=512,S=3", "P=64,T=512", "P=64,T=256,S=2"])
def test_forced_column_blocks(plan, plan_override):
    """Narrow column blocks forced on shapes with and without Stage 2, several slots per bucket, ragged rows."""
    plan_override(plan)
    for i, (m, n, k, b, k_b) in enumerate([(3, 32768, 64, 64, 1), (3, 32768, 64, 256, 1), (3, 32768, 128, 64, 2),
                                           (2, 32768, 256, 128, 4), (3, 32771, 64, 64, 1), (2, 32776, 128, 128, 1)]):
        for dtype in ["f32", "bf16"]:
            run_case(workloads.normal_rows(m, n, seed=740 + i, dtype=dtype), k, b, k_b, tag=plan)


@pytest.mark.parametrize("lanes", ["V=1", "V=2", "V=4", "V=8"])
def test_forced_lane_widths(lanes, plan_override):
    """Every compiled (type, columns per lane, slots) instance gives the same results."""
    plan_override(lanes)
    for i, (m, n, k, b, k_b) in enumerate([(3, 16384, 2048, 2048, 1), (3, 16384, 64, 64, 1), (3, 16384, 100, 256, 1),
                                           (3, 16384, 2048, 1024, 2), (3, 16384, 128, 64, 2), (3, 16384, 2048, 512, 4),
                                           (3, 16384, 96, 32, 4), (3, 16384, 2048, 256, 8), (2, 16384, 64, 8, 8),
                                           (2, 16384, 2048, 128, 16), (2, 16384, 200, 16, 16), (2, 16392, 64, 64, 3)]):
        for dtype in ["f32", "bf16"]:
            x = workloads.normal_rows(m, n, seed=300 + i, dtype=dtype)
            run_case(x, k, b, k_b, tag=lanes)


def random_cases(seed, count):
    """Seeded random legal (m, n, k, b, k_b) with b*k_b within what Stage 2 accepts."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        m = int(rng.integers(1, 9))
        n = int(rng.choice([rng.integers(1, 200), rng.integers(200, 5000), rng.integers(5000, 70000)]))
        k_b = int(rng.choice([1, 1, 1, 2, 3, 4, 5, 8, 11, 16]))
        if k_b > n:
            continue
        b_max = n // k_b
        b = int(rng.choice([rng.integers(1, min(b_max, 64) + 1), rng.integers(1, b_max + 1)]))
        lo = max(k_b, 1)
        hi = b * k_b
        k = int(rng.choice([hi, rng.integers(lo, hi + 1)]))
        out.append((m, n, k, b, k_b))
    return out


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_shapes(dtype):
    for i, (m, n, k, b, k_b) in enumerate(random_cases(20241127, 60)):
        x = workloads.normal_rows(m, n, seed=600 + i, dtype=dtype)
        run_case(x, k, b, k_b, tag="random%d" % i)
        run_case(x, k, b, k_b, tag="random%d contiguous" % i, assignment=atk.ATK_CONTIGUOUS)


def wide_cases(seed, count):
    """Seeded cases over a wider range than random_cases: up to 300 rows, row lengths up to 300000 that are
    multiples of 1, 8, 32, 64 or 256 elements, power-of-two and odd bucket counts, tie-heavy and special-valued inputs."""
    rng = np.random.default_rng(seed)
    lib = atk.load_library()
    out = []
    while len(out) < count:
        m = int(rng.choice([1, 2, 3, 5, 8, 17, 33, 64, 130, 300]))
        align = int(rng.choice([1, 8, 32, 64, 256]))
        n = int(rng.choice([rng.integers(64, 2000), rng.integers(2000, 40000), rng.integers(40000, 300000)]))
        n = max(align, n // align * align)
        if m * n > 6_000_000:
            m = max(1, 6_000_000 // n)
        k_b = int(rng.choice([1, 1, 1, 1, 2, 2, 3, 4, 8, 16]))
        if k_b > n:
            continue
        b_max = n // k_b
        b = int(rng.choice([2 ** int(rng.integers(0, 13)), rng.integers(1, min(b_max, 64) + 1), rng.integers(1, b_max + 1),
                            4 * int(rng.integers(1, 600))]))
        b = max(1, min(b, b_max))
        hi = b * k_b
        if hi > 8192 and rng.random() < 0.7:
            k = hi
        else:
            k = int(rng.choice([hi, rng.integers(k_b, hi + 1), max(k_b, hi // 2), max(k_b, hi // 16)]))
        dtype = str(rng.choice(["f32", "bf16"]))
        kind = int(rng.integers(0, 10))
        if lib.atk_check_approx(m, n, k, b, k_b, atk.ATK_F32 if dtype == "f32" else atk.ATK_BF16) != 0:
            continue
        out.append((m, n, k, b, k_b, dtype, kind, int(rng.integers(1 << 30)), float(rng.random()), float(rng.random()),
                    int(rng.integers(1, min(n, 5000) + 1))))
    return out


def test_wide_random_shapes():
    for (m, n, k, b, k_b, dtype, kind, seed, r_contig, r_exact, k_exact) in wide_cases(20241128, 1000):
        if kind == 0:
            x = workloads.few_levels(m, n, levels=1 + seed % 4, seed=seed, dtype=dtype)
        elif kind == 1:
            x = workloads.special_values(m, n, seed=seed, dtype=dtype)
        else:
            x = workloads.normal_rows(m, n, seed=seed, dtype=dtype)
        run_case(x, k, b, k_b, tag="wide")
        if r_contig < 0.3:
            run_case(x, k, b, k_b, tag="wide contiguous", assignment=atk.ATK_CONTIGUOUS)
        if r_exact < 0.3:
            run_exact(x, k_exact)


def test_many_short_rows():
    """More rows than a grid dimension holds, each a few matrix rows long."""
    x = workloads.normal_rows(70000, 64, seed=9)
    run_case(x, 8, 8, 1, tag="many rows")
    run_case(x, 6, 16, 1, tag="many rows, Stage 2")
    run_case(x, 16, 8, 2, tag="many rows", assignment=atk.ATK_CONTIGUOUS)


def test_stage2_over_many_candidates():
    """b*k_b above what one workgroup holds: Stage 1 leaves the candidates in scratch and the long-row
    selection finishes; ties are still decided by the original column index."""
    cases = [(3, 65536, 4096, 8192, 1), (3, 65536, 1000, 4096, 2), (2, 100000, 5000, 10000, 3), (2, 40000, 4097, 4100, 1),
             (2, 1 << 18, 20000, 1 << 15, 1), (130, 20000, 100, 5000, 1)]
    for dtype in ["f32", "bf16"]:
        for i, (m, n, k, b, k_b) in enumerate(cases):
            run_case(workloads.normal_rows(m, n, seed=800 + i, dtype=dtype), k, b, k_b, tag="big stage 2")
        run_case(workloads.few_levels(3, 65536, levels=3, seed=5, dtype=dtype), 3000, 8192, 1, tag="big stage 2, 3 levels")
        run_case(workloads.special_values(2, 65536, seed=6, dtype=dtype), 5000, 4096, 2, tag="big stage 2, specials")
        run_case(workloads.normal_rows(3, 65536, seed=810, dtype=dtype), 4096, 8192, 1, tag="big stage 2 contiguous",
                 assignment=atk.ATK_CONTIGUOUS)


# ------------------------------------------------------------------------------- contiguous assignment
CONTIG_SHAPES = [
    # (m, n, k, b, k_b)
    (4, 4096, 64, 64, 1),          # a wavefront's worth of vector chunks per bucket
    (4, 4096, 48, 64, 1),          # ... with Stage 2
    (128, 65536, 64, 64, 1),       # cfg2's shape
    (128, 65536, 64, 1024, 1),
    (64, 65536, 16384, 16384, 1),  # bucket = one 16-byte load
    (64, 65536, 16384, 4096, 4),
    (8, 65536, 16384, 1024, 16),
    (3, 12288, 96, 96, 1),         # b not a power of two
    (2, 4098, 6, 6, 1),            # n % b != 0: runs of unequal length, scalar loads
    (2, 4098, 683, 683, 1),
    (5, 1001, 45, 15, 3),
    (2, 70001, 250, 250, 1),
    (2, 20004, 100, 96, 3),
    (5, 8192, 1, 1, 1),            # one bucket: the whole workgroup on it
    (2, 8192, 16, 1, 16),
    (1, 1 << 20, 64, 8, 8),        # long buckets, split over workgroups
    (1, 1 << 20, 64, 64, 1),
    (1, 1 << 20, 50, 64, 2),
    (3, 1 << 18, 256, 32, 8),
    (2, 16384, 16384, 1024, 16),   # k_b = n/b: every bucket fully sorted
    (2, 16384, 16384, 16384, 1),   # identity
    (1, 128256, 256, 512, 1),      # vocabulary-sized row
    (1, 128256, 256, 1000, 2),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_contiguous_assignment(dtype):
    for i, (m, n, k, b, k_b) in enumerate(CONTIG_SHAPES):
        x = workloads.normal_rows(m, n, seed=400 + i, dtype=dtype)
        run_case(x, k, b, k_b, tag="contig%d" % i, assignment=atk.ATK_CONTIGUOUS)
    # ties: the lowest index wins inside a run and in Stage 2
    for k, b, k_b in [(64, 64, 1), (40, 64, 2), (128, 8, 16)]:
        run_case(workloads.few_levels(3, 8192, levels=3, seed=1, dtype=dtype), k, b, k_b, tag="contig 3 levels",
                 assignment=atk.ATK_CONTIGUOUS)
        run_case(workloads.special_values(3, 8192, seed=3, dtype=dtype), k, b, k_b, tag="contig specials",
                 assignment=atk.ATK_CONTIGUOUS)


@pytest.mark.parametrize("plan", ["T=64", "T=128,S=3", "T=256,S=16", "T=1024,S=2", "V=1"])
def test_contiguous_forced_plans(plan, plan_override):
    plan_override(plan)
    for i, (m, n, k, b, k_b) in enumerate([(3, 32768, 64, 64, 1), (3, 32768, 64, 256, 1), (2, 1 << 17, 16, 4, 4),
                                           (2, 1 << 17, 10, 2, 8), (3, 32768, 2048, 2048, 1)]):
        for dtype in ["f32", "bf16"]:
            x = workloads.normal_rows(m, n, seed=500 + i, dtype=dtype)
            run_case(x, k, b, k_b, tag="contig " + plan, assignment=atk.ATK_CONTIGUOUS)


def test_correlated_sequence_simulation_on_the_gpu():
    """Appendix A.1's simulation (n = 2048, k = 256, Sigma_ij = rho^|i-j|) through the library:
    recall against the library's exact_topk, equal to what the oracle gives on the same rows."""
    n, k, rows, rho = 2048, 256, 64, 0.99
    x = workloads.correlated_rows(rows, n, rho, seed=23)
    xg = x.cuda()
    ex = atk.exact_topk(xg, k)[1].cpu().numpy()
    ex_o = oracle.exact_topk(x.numpy(), k, threads=THREADS)[1]
    assert np.array_equal(ex, ex_o)

    def rec(idx):
        return float(np.mean([len(set(a.tolist()) & set(e.tolist())) / k for a, e in zip(idx, ex)]))

    for k_b in (1, 2, 4):
        b = k // k_b
        inter = atk.approx_topk(xg, k, b, k_b)[1].cpu().numpy()
        contig = atk.approx_topk(xg, k, b, k_b, assignment=atk.ATK_CONTIGUOUS)[1].cpu().numpy()
        assert np.array_equal(contig, oracle.approx_topk(x.numpy(), k, b, k_b, assignment=oracle.CONTIGUOUS)[1])
        print("rho=%.2f k_b=%d recall interleaved %.3f contiguous %.3f" % (rho, k_b, rec(inter), rec(contig)), flush=True)
        assert rec(contig) < rec(inter) - 0.3


def test_interleaved_flag_is_approx_topk():
    x = workloads.config_input("cfg1").cuda()
    a = atk.approx_topk(x, 64, 64, 1)
    c = atk.approx_topk(x, 64, 64, 1, assignment=atk.ATK_INTERLEAVED)
    assert torch.equal(a[0], c[0]) and torch.equal(a[1], c[1])


@pytest.mark.parametrize("plan", ["", "PK=0", "T=64,S=1"])
def test_bf16_packed_queues(plan, plan_override):
    """bf16 with k_b >= 3 keeps (key, row) in one 32-bit word per slot when a lane's share of the row
    is short enough; the results are the same with that path switched off, and on rows whose
    single split is too long for it."""
    if plan:
        plan_override(plan)
    cases = [(3, 16384, 2048, 1024, 2), (3, 16384, 96, 32, 4), (2, 16384, 64, 8, 8), (2, 16392, 64, 64, 3),
             (4, 65536, 16384, 1024, 16), (2, 300000, 16, 4, 4), (2, 300001, 10, 2, 5), (1, 1 << 20, 64, 16, 4)]
    for i, (m, n, k, b, k_b) in enumerate(cases):
        run_case(workloads.normal_rows(m, n, seed=700 + i, dtype="bf16"), k, b, k_b, tag="packed " + plan)
    for k, b, k_b in [(96, 32, 4), (40, 64, 2), (128, 8, 16)]:
        run_case(workloads.few_levels(3, 8192, levels=3, seed=1, dtype="bf16"), k, b, k_b, tag="packed 3 levels " + plan)
        run_case(workloads.special_values(3, 8192, seed=3, dtype="bf16"), k, b, k_b, tag="packed specials " + plan)
    z = torch.zeros((2, 4096))
    z[:, ::3] = -0.0
    run_case(z.to(torch.bfloat16), 50, 64, 2, tag="packed zeros " + plan)


# ------------------------------------------------------------------------------- ties and special values
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ties_and_specials(dtype):
    params = [(64, 64, 1), (64, 256, 1), (96, 32, 4), (40, 64, 2), (128, 8, 16), (2048, 2048, 1)]
    for k, b, k_b in params:
        run_case(workloads.few_levels(3, 8192, levels=3, seed=1, dtype=dtype), k, b, k_b, tag="3 levels")
        run_case(workloads.few_levels(3, 8192, levels=1, seed=2, dtype=dtype), k, b, k_b, tag="constant")
        run_case(workloads.special_values(3, 8192, seed=3, dtype=dtype), k, b, k_b, tag="specials")
    # rows of -inf only, and of -0 / +0 only
    x = torch.full((2, 4096), float("-inf"))
    z = torch.zeros((2, 4096))
    z[:, ::3] = -0.0
    for t in (x, z):
        t = t if dtype == "f32" else t.to(torch.bfloat16)
        run_case(t, 64, 64, 1, tag="-inf/zeros")
        run_case(t, 50, 64, 2, tag="-inf/zeros")


def test_repeatable():
    x = workloads.config_input("cfg2").cuda()
    ref = None
    for _ in range(5):
        vals, idx = atk.approx_topk(x, 64, 256, 1)
        torch.cuda.synchronize()
        cur = (as_bits(vals).copy(), idx.cpu().numpy().copy())
        if ref is None:
            ref = cur
        assert np.array_equal(cur[0], ref[0]) and np.array_equal(cur[1], ref[1])


def _repeat_against_oracle(x_cpu, call, oracle_result, runs, tag, between):
    """`runs` calls of call(xg) -> (vals, idx), other launches in between, each run compared with the oracle
    on every row; stops at the first mismatch."""
    ov, oi = oracle_result
    ovb = ov.view(np.uint32) if ov.dtype == np.float32 else ov
    xg = x_cpu.cuda()
    for run in range(runs):
        vals, idx = call(xg)
        between(run)
        torch.cuda.synchronize()
        gi, gv = idx.cpu().numpy(), as_bits(vals)
        if not (np.array_equal(gi, oi) and np.array_equal(gv, ovb)):
            bad = np.argwhere(gi != oi)
            raise AssertionError("%s: run %d of %d differs from the oracle in %d places (rows %s)" % (
                tag, run, runs, len(bad), np.unique(bad[:, 0])[:16].tolist()))
    del xg


HAND_OVER_CASES = [
    # (tag, input, (k, b, k_b), plan override, what the plan must say)
    ("cfg4 b=1024 Stage 2", ("cfg4",), (64, 1024, 1), None, "pair_rows=512 "),
    ("cfg4 b=1024 Stage 2 in two halves", ("cfg4",), (64, 1024, 1), "HF=0", "scratch=1"),
    ("cfg4 b=128 k_b=8 Stage 2", ("cfg4",), (64, 128, 8), None, "scratch=1"),
    ("8 x 2^20 b=64 row splits through scratch", (8, 1 << 20, 51, "f32"), (64, 64, 1), "MH=0", "scratch=1"),
    ("8 x 2^20 b=64 helpers + finisher", (8, 1 << 20, 51, "f32"), (64, 64, 1), None, "helpers=15 "),
    ("16 x 2^17 b=256 helpers + finisher", (16, 1 << 17, 57, "f32"), (64, 256, 1), None, "helpers=15 "),
    ("5 x 65536 bf16 b=128 helpers + finisher", (5, 65536, 58, "bf16"), (64, 128, 1), None, "helpers=3 "),
    ("3 x 2^18 b=256 S=64", (3, 1 << 18, 52, "f32"), (64, 256, 1), "S=64", "S=64 "),
    ("5 x 2^18 bf16 b=64 k_b=4 S=16 P=4", (5, 1 << 18, 53, "bf16"), (100, 64, 4), "S=16,P=4", "S=16 "),
    ("cfg2 b=512 two workgroups per row", ("cfg2",), (64, 512, 1), "S=2", "scratch=1"),
    ("cfg2 b=256 helper + finisher", ("cfg2",), (64, 256, 1), None, "pair_rows=128"),
    ("cfg2 b=512 helper + finisher", ("cfg2",), (64, 512, 1), None, "pair_rows=64"),
]


@pytest.mark.parametrize("case", HAND_OVER_CASES, ids=[c[0] for c in HAND_OVER_CASES])
def test_repeat_runs_on_hand_over_plans(case, plan_override):
    """Plans whose workgroups hand partial lists over through global scratch and a ticket (Appendix A:
    the per-thread queues are merged once, here also across workgroups): 20 runs each with other
    launches in between, every run compared with the oracle on every row."""
    tag, inp, (k, b, k_b), plan, must = case
    x = workloads.config_input(inp[0]) if len(inp) == 1 else workloads.normal_rows(inp[0], inp[1], seed=inp[2], dtype=inp[3])
    dt = atk.ATK_F32 if x.dtype == torch.float32 else atk.ATK_BF16
    other = workloads.normal_rows(16, 32768, seed=54).cuda()
    expect = oracle.approx_topk(workloads.as_numpy_bits(x), k, b, k_b, threads=THREADS)

    def between(run):  # other shapes on the same scratch pool and tickets; the override is for the case alone
        plan_override(None)
        atk.approx_topk(other, 64, 64 << (run % 3), 1)
        atk.exact_topk(other, 64)
        plan_override(plan)

    plan_override(plan)
    described = atk.plan_describe(x.shape[0], x.shape[1], k, b, k_b, dt)
    print("repeat %s plan=[%s]" % (tag, described), flush=True)
    assert must in described + " ", described
    _repeat_against_oracle(x, lambda xg: atk.approx_topk(xg, k, b, k_b), expect, 20, tag, between)


@pytest.mark.parametrize("shape", [(128, 65536, 64), (1, 1 << 20, 1000), (128, 65536, 16384)])
def test_repeat_runs_of_exact_topk(shape):
    """exact_topk's sweeps whose last workgroup per row decides the digit (a ticket after the counts are
    acknowledged): 20 runs with other launches in between, every run compared with the oracle."""
    m, n, k = shape
    x = workloads.normal_rows(m, n, seed=55)
    other = workloads.normal_rows(16, 32768, seed=56).cuda()
    expect = oracle.exact_topk(workloads.as_numpy_bits(x), k, threads=THREADS)

    def between(run):
        atk.approx_topk(other, 64, 64 << (run % 3), 1)

    _repeat_against_oracle(x, lambda xg: atk.exact_topk(xg, k), expect, 20, "exact %s" % (shape,), between)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_helper_finisher_pairs(dtype, plan_override):
    """Stage 2 with two workgroups per row (the helper leaves its maxima in a mailbox in memory, the finisher
    picks them up): the plans the library chooses on its own, ties and special values included, and forced on
    shapes it would not choose them for - every split of the matrix rows, workgroup sizes, streaming lane counts."""
    dt = atk.ATK_F32 if dtype == "f32" else atk.ATK_BF16
    for (m, n) in [(6, 65536), (128, 65536), (40, 1 << 17)]:
        for (k, b) in [(64, 128), (100, 256), (64, 512), (17, 64 * 5)]:
            plan = atk.plan_describe(m, n if n % b == 0 else n // b * b, k, b, 1, dt)
            nn = n if n % b == 0 else n // b * b
            if m == 128 and nn == n:  # (fewer rows are split over more than two workgroups, with tickets)
                assert " lean=1 " in plan and " pair_rows=0" not in plan, plan
            run_case(workloads.normal_rows(m, nn, seed=950 + b, dtype=dtype), k, b, 1, tag="pair")
        run_case(workloads.few_levels(m, n, levels=3, seed=960, dtype=dtype), 64, 256, 1, tag="pair ties")
        run_case(workloads.few_levels(m, n, levels=1, seed=961, dtype=dtype), 64, 128, 1, tag="pair constant")
        run_case(workloads.special_values(m, n, seed=962, dtype=dtype), 100, 512, 1, tag="pair specials")
    # no Stage 2 (b = k) on rows whose 128-byte matrix rows cannot be shared out between two workgroups: the
    # finisher writes the row of maxima
    bo = 32 if dtype == "f32" else 64
    for (m, n) in [(128, 65536), (40, 1 << 17), (3, 1 << 18)]:
        plan = atk.plan_describe(m, n, bo, bo, 1, dt)
        if m == 128 and dtype == "bf16" and n <= 65536:  # (one workgroup of 512 streaming lanes per row is faster there)
            assert " lean=1 " in plan and " pair_rows=0 " in plan and " S=1 " in plan and " stage2=0 " in plan, plan
        elif m == 128:  # (fewer rows take more than one helper)
            assert " lean=1 " in plan and " pair_rows=%d" % (n // bo // 2) in plan and " stage2=0 " in plan, plan
        run_case(workloads.normal_rows(m, n, seed=985, dtype=dtype), bo, bo, 1, tag="pair, no Stage 2")
        run_case(workloads.few_levels(m, n, levels=2, seed=986, dtype=dtype), bo, bo, 1, tag="pair, no Stage 2, ties")
        run_case(workloads.special_values(m, n, seed=987, dtype=dtype), bo // 2, bo // 2, 1, tag="pair, no Stage 2, specials")
    # long rows: pairs also at 1024 buckets, half the matrix rows each, all 512 lanes streaming in bf16
    for (m, n, k, b) in [(128, 1 << 18, 64, 1024), (100, 1 << 19, 50, 256), (128, 1 << 17, 200, 1024)]:
        plan = atk.plan_describe(m, n, k, b, 1, dt)
        assert " lean=1 " in plan and " pair_rows=%d" % (n // b // 2) in plan and " S=1 " in plan, plan
        if dtype == "bf16" and n >= 1 << 18:
            assert " T=512 " in plan, plan
        run_case(workloads.normal_rows(m, n, seed=990 + b, dtype=dtype), k, b, 1, tag="pair long")
    for spec in ["HF=1", "HF=1,HQ=1", "HF=1,HQ=63", "HF=1,HT=64", "HF=1,HT=128,HQ=40", "HF=1,HT=512,SL=512", "HF=1,HT=512,SL=128,HQ=9"]:
        plan_override(spec)
        for (m, n, k, b) in [(3, 8192, 64, 128), (300, 4096, 16, 64), (5, 36864, 100, 256), (2, 65536, 64, 1024),
                             (2, 1 << 16, 1000, 2048)]:
            x = workloads.normal_rows(m, n, seed=970 + b, dtype=dtype)
            print(spec, atk.plan_describe(m, n, k, b, 1, dt), flush=True)
            run_case(x, k, b, 1, tag=spec)
        run_case(workloads.few_levels(4, 16384, levels=2, seed=980, dtype=dtype), 30, 128, 1, tag=spec + " ties")
        run_case(workloads.special_values(4, 16384, seed=981, dtype=dtype), 64, 256, 1, tag=spec + " specials")
    plan_override(None)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_helpers_and_finisher(dtype, plan_override):
    """Few long rows with one slot per bucket: the splits of a row run as helpers and a finisher (one mailbox per
    helper).  The plans the library chooses on its own - with and without Stage 2, column blocks, ties and special
    values - and forced helper counts on shapes it would not choose them for: bucket counts that are no power of
    two, finishers with a short share, more helpers than a lane of the finisher fetches words for (those stay on
    the row splits through scratch)."""
    dt = atk.ATK_F32 if dtype == "f32" else atk.ATK_BF16
    chosen = 0
    for (m, n) in [(1, 1 << 20), (7, 1 << 18), (16, 1 << 17), (33, 1 << 19), (3, 65536)]:
        for (k, b) in [(64, 64), (32, 32), (64, 128), (100, 256), (64, 512), (300, 1024)]:
            plan = atk.plan_describe(m, n, k, b, 1, dt)
            chosen += " helpers=0" not in plan
            run_case(workloads.normal_rows(m, n, seed=1200 + b, dtype=dtype), k, b, 1, tag="helpers")
        run_case(workloads.few_levels(m, n, levels=3, seed=1210, dtype=dtype), 64, 256, 1, tag="helpers ties")
        run_case(workloads.few_levels(m, n, levels=1, seed=1211, dtype=dtype), 64, 64, 1, tag="helpers constant")
        run_case(workloads.special_values(m, n, seed=1212, dtype=dtype), 100, 128, 1, tag="helpers specials")
        # rows with a trend: the first helper's share lies far from the finisher's (the two lower bounds on Stage 2's bins)
        xs = workloads.normal_rows(m, n, seed=1213, dtype=dtype)
        asc = torch.sort(xs.float(), dim=1).values.to(xs.dtype)
        run_case(asc, 64, 256, 1, tag="helpers ascending")
        run_case(torch.flip(asc, dims=[1]).contiguous(), 64, 256, 1, tag="helpers descending")
    assert chosen >= 15, chosen
    for spec in ["MH=1", "MH=2", "MH=5", "MH=15", "MH=40", "MH=3,T=128", "MH=7,T=64"]:
        plan_override(spec)
        for (m, n, k, b) in [(3, 8192, 64, 128), (70, 4096, 16, 16), (5, 36864, 100, 288), (2, 65536, 64, 1024),
                             (9, 96 * 512, 96, 96), (2, 1 << 16, 1000, 2048), (4, 24 * 1024, 20, 24)]:
            x = workloads.normal_rows(m, n, seed=1220 + b, dtype=dtype)
            print(spec, atk.plan_describe(m, n, k, b, 1, dt), flush=True)
            run_case(x, k, b, 1, tag=spec)
        run_case(workloads.few_levels(4, 16384, levels=2, seed=1230, dtype=dtype), 30, 128, 1, tag=spec + " ties")
        run_case(workloads.special_values(4, 16384, seed=1231, dtype=dtype), 64, 256, 1, tag=spec + " specials")
    plan_override(None)


PLAN_FAMILIES = [
    # (dtype, m, n, k, b, k_b, what the plan must say, rows compared or None for all)
    ("f32", 4, 1 << 20, 64, 4096, 1, " stage2=1 ", None),          # few rows with Stage 2: column blocks, not row splits
    ("f32", 1, 1 << 22, 64, 128, 1, " stage2=1 ", None),
    ("f32", 8, 151936, 256, 512, 2, " stage2=1 ", None),
    ("bf16", 32, 128256, 256, 2048, 1, " stage2=1 ", None),
    ("f32", 128, 65536, 4096, 1024, 4, " S=1 ", list(range(0, 128, 8))),   # queues without Stage 2: lanes share column groups
    ("f32", 128, 65536, 4096, 256, 16, " stage2=0 ", list(range(0, 128, 8))),
    ("f32", 1, 1 << 20, 4096, 256, 16, " stage2=0 ", None),
    ("bf16", 128, 1 << 18, 4096, 2048, 2, " stage2=0 ", list(range(0, 128, 16))),
    ("f32", 128, 65536, 1024, 128, 16, " stage2=1 ", list(range(0, 128, 8))),  # ... and in front of Stage 2 from 2048 candidates
    ("bf16", 2048, 16384, 256, 64, 4, " S=1 ", list(range(0, 2048, 128))),   # many rows: bigger workgroups, no row splits
    ("bf16", 256, 32000, 64, 501, 1, " colblocks=1 ", list(range(0, 256, 16))),  # narrow lanes: a lane per column group
    ("f32", 32, 1 << 18, 1024, 256, 4, " stage2=0 ", None),          # splits capped by the last workgroup's merge
    ("f32", 8, 16384, 64, 8, 8, " stage2=0 ", None),                 # long queues on few short rows keep their splits
    ("f32", 128, 65536, 256, 32, 16, " stage2=1 ", list(range(0, 128, 8))),
    ("bf16", 128, 32768, 64, 256, 1, " lean=1 ", None),             # short rows: the bins' range comes from the merged candidates
    ("f32", 1024, 4096, 64, 128, 1, " lean=1 ", list(range(0, 1024, 32))),
]


@pytest.mark.parametrize("case", PLAN_FAMILIES, ids=["%s %dx%d k=%d b=%d k_b=%d" % c[:6] for c in PLAN_FAMILIES])
def test_plan_families(case):
    """One shape from every family of launch plans that the planner's rules tell apart (Section 2's two stages on very
    different launch geometries): results must not depend on the plan."""
    dtype, m, n, k, b, k_b, must, rows = case
    dt = atk.ATK_F32 if dtype == "f32" else atk.ATK_BF16
    plan = atk.plan_describe(m, n, k, b, k_b, dt)
    assert must in plan + " ", plan
    run_case(workloads.normal_rows(m, n, seed=1300 + b + k_b, dtype=dtype), k, b, k_b, rows=rows, tag="family")
    if m * n <= 1 << 23:
        run_case(workloads.few_levels(m, n, levels=3, seed=1310 + b, dtype=dtype), k, b, k_b, rows=rows, tag="family ties")


def test_calls_on_two_streams_share_the_scratch_pools():
    """The scratch pools are per device; calls that alternate between two streams must not see each other's tickets,
    lists or mailboxes (a call on another stream than the one before it waits for that stream first)."""
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    xa = workloads.normal_rows(8, 1 << 20, seed=1300)   # row splits through scratch and tickets
    xb = workloads.normal_rows(128, 65536, seed=1301)   # helper + finisher mailboxes
    ea = oracle.approx_topk(workloads.as_numpy_bits(xa), 64, 64, 1, threads=THREADS)
    eb = oracle.approx_topk(workloads.as_numpy_bits(xb), 64, 256, 1, threads=THREADS)
    ec = oracle.exact_topk(workloads.as_numpy_bits(xb), 100, threads=THREADS)
    ga, gb = xa.cuda(), xb.cuda()
    torch.cuda.synchronize()
    outs = []
    for rep in range(6):
        with torch.cuda.stream(s1):
            outs.append(("a", atk.approx_topk(ga, 64, 64, 1)))
        with torch.cuda.stream(s2):
            outs.append(("b", atk.approx_topk(gb, 64, 256, 1)))
        with torch.cuda.stream(s1):
            outs.append(("c", atk.exact_topk(gb, 100)))
    torch.cuda.synchronize()
    for name, (v, i) in outs:
        ev, ei = {"a": ea, "b": eb, "c": ec}[name]
        assert np.array_equal(i.cpu().numpy(), ei), name
        assert np.array_equal(as_bits(v), np.asarray(ev).view(as_bits(v).dtype)), name


def test_pooled_queue_floors(plan_override):
    """Eight-slot queues whose lanes pool what they have seen and raise their floors mid-scan (Appendix A's per-thread
    queues, shared between the threads of a bucket before the final merge): the plans that do it on their own, on
    normal, tie-heavy, constant, special-valued and sorted rows (ascending rows make every element enter, descending
    rows none after the first), and forced onto small shapes from the first load batch on."""
    def inputs(m, n, seed):
        x = workloads.normal_rows(m, n, seed=seed)
        yield "normal", x
        yield "three levels", workloads.few_levels(m, n, levels=3, seed=seed + 1)
        yield "constant", workloads.few_levels(m, n, levels=1, seed=seed + 2)
        yield "specials", workloads.special_values(m, n, seed=seed + 3)
        yield "ascending", torch.sort(x, dim=1).values.contiguous()
        yield "descending", torch.sort(x, dim=1, descending=True).values.contiguous()
    for (m, n, k, b) in [(128, 1 << 20, 64, 8), (128, 1 << 20, 40, 16), (128, 1 << 20, 64, 128)]:
        plan = atk.plan_describe(m, n, k, b, 8, atk.ATK_F32)
        assert " refresh=8" in plan, plan
        run_case(workloads.normal_rows(m, n, seed=1200 + b), k, b, 8, tag="pooled floors")
    for (m, n, k, b) in [(3, 1 << 20, 64, 8), (2, 1 << 19, 100, 32)]:
        plan_override("RF=8")
        assert " refresh=8" in atk.plan_describe(m, n, k, b, 8, atk.ATK_F32)
        for name, x in inputs(m, n, 1210 + b):
            run_case(x, k, b, 8, tag="pooled floors, " + name)
    for spec in ["RF=1", "RF=2", "RF=3,P=4", "RF=1,T=64", "RF=1,S=3"]:
        plan_override(spec)
        for (m, n, k, b) in [(5, 8192, 16, 8), (3, 40000, 64, 16), (2, 1 << 16, 64, 128), (7, 30000, 24, 24)]:
            plan = atk.plan_describe(m, n, k, b, 8, atk.ATK_F32)
            print(spec, plan, flush=True)
            for name, x in inputs(m, n, 1230 + b):
                run_case(x, k, b, 8, tag=spec + ", " + name)
    plan_override(None)


@pytest.mark.parametrize("spec", ["LN=0", "LN=0,LM=0", "HF=0", "HF=0,SL=64"])
def test_headline_shapes_on_every_kernel(spec, plan_override):
    """The configurations of the headline sweep and of the attention-score shape through the general kernel (LN=0:
    no lean kernels; LM=0: lanes merge through the LDS exchange instead of LDS atomics) and without pairs."""
    plan_override(spec)
    x = workloads.config_input("cfg2")
    for k, b, k_b in workloads.CONFIGS["cfg2"]["cases"]:
        run_case(x, k, b, k_b, tag=spec)
    xb = workloads.normal_rows(64, 65536, seed=77, dtype="bf16")
    for k, b, k_b in workloads.CONFIGS["cfg2"]["cases"]:
        run_case(xb, k, b, k_b, tag=spec + " bf16")
    run_case(workloads.few_levels(6, 65536, levels=3, seed=78), 64, 256, 1, tag=spec + " ties")
    run_case(workloads.special_values(6, 65536, seed=79), 64, 1024, 1, tag=spec + " specials")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stage2_with_few_rows_per_lane(dtype):
    """Stage 2 whose bins cannot take their lower end from the merge (lanes that saw only a few rows may hold values
    far below the candidates): the selection then finds the range itself.  Also rows of small and negative values, on
    which a loose bound would crowd the bins, and buckets that beat every bound (all-negative columns)."""
    for (m, n, k, b) in [(8, 16384, 64, 1024), (8, 8192, 100, 2048), (128, 16384, 64, 512), (16, 32768, 64, 1024),
                         (128, 8192, 30, 256)]:
        run_case(workloads.normal_rows(m, n, seed=990 + b, dtype=dtype), k, b, 1, tag="few rows per lane")
    x = workloads.normal_rows(16, 65536, seed=995) * 1e-3 - 5.0
    x[:, ::7] = 3.0
    run_case(x if dtype == "f32" else x.to(torch.bfloat16), 64, 256, 1, tag="negative bulk")
    x = -torch.abs(workloads.normal_rows(16, 65536, seed=996)) - 1.0
    run_case(x if dtype == "f32" else x.to(torch.bfloat16), 64, 512, 1, tag="all negative")
    x = workloads.normal_rows(16, 65536, seed=997)
    x[:, 5::64] = -1e30  # one column whose maximum lies far below every other candidate
    run_case(x if dtype == "f32" else x.to(torch.bfloat16), 64, 64 * 4, 1, tag="one tiny column")
    run_case(x if dtype == "f32" else x.to(torch.bfloat16), 250, 64 * 4, 1, tag="one tiny column, k near b")


def test_trace_build_matches_and_stamps():
    """atk_trace_approx (the measurement build of the lean kernels) returns what approx_topk returns and leaves a
    start and an end stamp for every wavefront; shapes without that build are refused before anything is launched."""
    lib = atk.load_library()
    x = workloads.normal_rows(128, 65536, seed=71).cuda()
    st = torch.cuda.current_stream().cuda_stream
    for (k, b) in [(64, 64), (64, 256), (64, 1024)]:
        ref_v, ref_i = atk.approx_topk(x, k, b, 1)
        nbytes = lib.atk_trace_bytes(128, 65536, k, b, 1, atk.ATK_F32)
        assert nbytes > 0
        tr = torch.zeros(nbytes // 8, dtype=torch.int64, device="cuda")
        v = torch.empty_like(ref_v)
        i = torch.empty_like(ref_i)
        rc = lib.atk_trace_approx(x.data_ptr(), 128, 65536, k, b, 1, atk.ATK_F32, v.data_ptr(), i.data_ptr(), tr.data_ptr(), nbytes, st)
        assert rc == 0, atk.strerror(rc)
        torch.cuda.synchronize()
        assert torch.equal(i, ref_i) and torch.equal(v, ref_v)
        t = tr.cpu().numpy().reshape(-1, 16)
        ran = t[t[:, 0] != 0]
        assert len(ran) > 0 and (ran[:, 9] >= ran[:, 0]).all() and (ran[:, 1] >= ran[:, 0]).all()
        assert lib.atk_trace_approx(x.data_ptr(), 128, 65536, k, b, 1, atk.ATK_F32, v.data_ptr(), i.data_ptr(), tr.data_ptr(), 64, st) == -2
    assert lib.atk_trace_bytes(128, 65536, 128, 64, 2, atk.ATK_F32) > 0
    tr = torch.zeros(1 << 20, dtype=torch.int64, device="cuda")
    v = torch.empty((128, 128), dtype=torch.float32, device="cuda")
    i = torch.empty((128, 128), dtype=torch.int32, device="cuda")
    assert lib.atk_trace_approx(x.data_ptr(), 128, 65536, 128, 64, 2, atk.ATK_F32, v.data_ptr(), i.data_ptr(), tr.data_ptr(), 8 << 20, st) == -4
    assert lib.atk_trace_approx(x.data_ptr(), 128, 65536, 128, 64, 2, atk.ATK_F32, v.data_ptr(), i.data_ptr(), None, 8 << 20, st) == -1


def test_cfg2_cfg3_bf16_and_small_batches():
    """The bf16 versions of the two 128 x 65536 sweeps (Appendix B.1's bfloat16 figure), Stage 2 included, and
    the same parameters on batches of 1, 8 and 32 rows (Section 5 leaves the batch size open)."""
    xb = workloads.normal_rows(128, 65536, seed=0, dtype="bf16")
    for k, b, k_b in workloads.CONFIGS["cfg2"]["cases"] + workloads.CONFIGS["cfg3"]["cases"]:
        run_case(xb, k, b, k_b, tag="bf16 cfg2/cfg3")
    for m in (1, 8, 32):
        for dtype in ("f32", "bf16"):
            x = workloads.normal_rows(m, 65536, seed=60 + m, dtype=dtype)
            for k, b, k_b in workloads.CONFIGS["cfg2"]["cases"] + workloads.CONFIGS["cfg3"]["cases"]:
                run_case(x, k, b, k_b, tag="m=%d" % m)


# ------------------------------------------------------------------------------- exact_topk
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_exact_small_rows(dtype):
    # (few rows of up to about 18000 elements take one workgroup each, with up to 160 KB of LDS)
    for m, n, k in [(4, 4096, 64), (3, 1000, 1), (3, 1000, 1000), (2, 3000, 777), (5, 2048, 2048), (7, 33, 5),
                    (3, 8192, 512), (2, 12000, 12000), (3, 18000, 64), (300, 16384, 100)]:
        run_exact(workloads.normal_rows(m, n, seed=300 + n, dtype=dtype), k)
        run_exact(workloads.few_levels(m, n, levels=2, seed=301 + n, dtype=dtype), k)
        run_exact(workloads.special_values(m, n, seed=302 + n, dtype=dtype), k)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_exact_sampled_threshold(dtype, plan_override):
    """Very small k on big inputs: the threshold is first guessed from a sample of the row (every 16th
    run of 4096 elements) and everything that reaches it is copied out in one sweep.  Rows where too
    much reaches it (ties, few levels, an ascending row whose sample misses the large values) start
    over digit by digit; finished and restarted rows share one call.  XS=1 takes that path on inputs
    below the size from which the library would choose it."""
    plan_override("XS=1")
    n = (1 << 19) + 333
    for k in (1, 64, 128):
        run_exact(workloads.normal_rows(3, n, seed=600 + k, dtype=dtype), k)
    run_exact(workloads.normal_rows(2, 1 << 20, seed=610, dtype=dtype), 100)
    asc = torch.sort(workloads.normal_rows(1, n, seed=611, dtype="f32"), dim=1).values
    desc = torch.flip(asc, dims=[1])
    if dtype == "bf16":
        asc, desc = asc.to(torch.bfloat16), desc.to(torch.bfloat16)
    mixed = torch.cat([workloads.normal_rows(2, n, seed=612, dtype=dtype), asc, desc,
                       workloads.few_levels(1, n, levels=2, seed=613, dtype=dtype),
                       workloads.few_levels(1, n, levels=1, seed=614, dtype=dtype),
                       workloads.special_values(1, n, seed=615, dtype=dtype)])
    run_exact(mixed, 64)
    run_exact(mixed, 128)
    run_exact(mixed, 200)  # every 8th run of 4096 elements sampled
    run_exact(mixed, 512)  # every 4th


def test_bf16_long_queues_one_column_per_lane():
    """bf16 with k_b >= 8 over b >= 1024 buckets: the planner gives a lane one column instead of two when
    that leaves the chip one to two (k_b = 16) or four (k_b = 8) wavefronts per SIMD; shapes on both sides
    of those bounds, with the plan checked so that the case keeps meaning what it says."""
    for m, n, b, k_b, v in [(128, 65536, 1024, 16, 1), (128, 65536, 2048, 8, 1), (64, 32768, 1024, 16, 1),
                            (100, 31775, 1025, 16, 1), (256, 32768, 1024, 16, 2), (32, 32768, 1024, 8, 2),
                            (128, 65536, 4096, 4, 2)]:
        plan = atk.plan_describe(m, n, b * k_b, b, k_b, atk.ATK_BF16)
        assert plan.startswith("V=%d " % v), plan
        run_case(workloads.normal_rows(m, n, seed=900 + m + k_b, dtype="bf16"), b * k_b, b, k_b, tag="bf16 queues")
    run_case(workloads.few_levels(64, 32768, levels=3, seed=910, dtype="bf16"), 16384, 1024, 16, tag="bf16 queues, ties")
    run_case(workloads.normal_rows(128, 65536, seed=911, dtype="bf16"), 500, 1024, 16, tag="bf16 queues, Stage 2")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_input_off_a_vector_boundary(dtype):
    """x may start at any multiple of its element size: the 16-byte loads of both entry points are only
    taken from a 16-byte aligned base (rows of a whole number of vectors), everything else goes the
    element-wise way."""
    for shift in (1, 2, 3, 5):
        run_case(workloads.normal_rows(3, 8192, seed=800 + shift, dtype=dtype), 64, 64, 1, shift=shift, tag="shifted")
        run_case(workloads.normal_rows(2, 65536, seed=810 + shift, dtype=dtype), 64, 256, 1, shift=shift, tag="shifted")
        run_case(workloads.normal_rows(2, 16384, seed=820 + shift, dtype=dtype), 128, 64, 4, shift=shift, tag="shifted")
        run_case(workloads.normal_rows(2, 16384, seed=830 + shift, dtype=dtype), 128, 32, 4, shift=shift, tag="shifted",
                 assignment=atk.ATK_CONTIGUOUS)
        run_exact(workloads.normal_rows(2, 4096, seed=840 + shift, dtype=dtype), 100, shift=shift)
        run_exact(workloads.normal_rows(2, 65536, seed=850 + shift, dtype=dtype), 64, shift=shift)
        run_exact(workloads.normal_rows(2, 65536, seed=860 + shift, dtype=dtype), 9000, shift=shift)
    # bf16 rows of a multiple of 4 but not of 8 elements: whole vectors only every other row
    run_exact(workloads.normal_rows(3, 65540, seed=870, dtype=dtype), 64)
    run_exact(workloads.normal_rows(3, 65540, seed=871, dtype=dtype), 64, shift=4)


@pytest.mark.parametrize("chunk", [1024, 4096, 8192, 16384])
def test_exact_sweep_chunks(chunk, plan_override):
    """The sweeps of the long-row path take 4096 to 16384 elements of a row per workgroup, by the size of
    the input; XC=<elements> fixes it.  Every size gives the same results: rows with a ragged last chunk,
    the copy-out path, the digit descent, and many survivors per chunk (the second sweep of the collect step)."""
    plan_override("XC=%d" % chunk)
    for dtype in ("f32", "bf16"):
        run_exact(workloads.normal_rows(3, 70001, seed=700 + chunk % 7, dtype=dtype), 64)
        run_exact(workloads.normal_rows(2, 50000, seed=701, dtype=dtype), 3000)
        run_exact(workloads.normal_rows(2, 50000, seed=702, dtype=dtype), 30000)
        run_exact(workloads.few_levels(2, 40000, levels=2, seed=703, dtype=dtype), 500)
        run_exact(workloads.special_values(2, 40000, seed=704, dtype=dtype), 6000)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_exact_long_rows(dtype):
    """Rows that do not fit one workgroup: global radix select, then LDS or global ordering."""
    for m, n, k in [(3, 20000, 64), (2, 50000, 1), (2, 50000, 3000), (2, 100000, 5000), (1, 70001, 70001),
                    (2, 300000, 40000)]:
        run_exact(workloads.normal_rows(m, n, seed=400 + n % 97, dtype=dtype), k)
    # ties at the threshold: the index decides (index digits of the radix select)
    run_exact(workloads.few_levels(3, 30000, levels=2, seed=5, dtype=dtype), 777)
    run_exact(workloads.few_levels(2, 30000, levels=1, seed=6, dtype=dtype), 9000)
    run_exact(workloads.special_values(2, 40000, seed=7, dtype=dtype), 6000)
    # small k on long rows: after the first digit the elements still in play are copied out and finished
    # in LDS; rows with too many of them (ties, few levels) stay on the digit-by-digit path, both in one call
    for m, n, k in [(5, 200000, 64), (3, 200000, 1000), (4, 65536, 1), (2, 1 << 20, 256)]:
        run_exact(workloads.normal_rows(m, n, seed=500 + k, dtype=dtype), k)
    mixed = torch.cat([workloads.normal_rows(2, 60000, seed=11, dtype=dtype),
                       workloads.few_levels(2, 60000, levels=2, seed=12, dtype=dtype),
                       workloads.special_values(1, 60000, seed=13, dtype=dtype)])
    run_exact(mixed, 100)
    run_exact(mixed, 1024)
    run_exact(mixed, 3000)  # few rows: the copy-out path up to k = 4096, with 8192 elements per row
    run_exact(mixed, 4096)
    # many survivors: partition sort (one wavefront per bin), its bitonic path for crowded bins (k of a
    # million: more than 512 per bin), and rows whose values pile up on a few levels, which fall back to
    # the digit-by-digit sort - all three kinds of row in one call as well
    run_exact(workloads.normal_rows(1, 1 << 21, seed=21, dtype=dtype), 1 << 20)
    run_exact(workloads.few_levels(2, 200000, levels=3, seed=22, dtype=dtype), 50000)
    run_exact(workloads.few_levels(2, 200000, levels=3, seed=23, dtype=dtype), 150000)
    big_mixed = torch.cat([workloads.normal_rows(2, 150000, seed=24, dtype=dtype),
                           workloads.few_levels(1, 150000, levels=2, seed=25, dtype=dtype),
                           workloads.special_values(1, 150000, seed=26, dtype=dtype)])
    run_exact(big_mixed, 30000)
    # values on a grid (about a thousand levels among the survivors, tens of ties each): bins of the partition
    # sort that hold a few levels; the ties of a level land in one sub-bin, and such bins go to the bitonic sort
    grid = torch.round(workloads.normal_rows(3, 100000, seed=27, dtype="f32") * 256) / 256
    run_exact(grid if dtype == "f32" else grid.to(torch.bfloat16), 20000)
    run_exact(grid if dtype == "f32" else grid.to(torch.bfloat16), 6000)


def test_exact_many_long_rows():
    """More long rows than a grid dimension holds: they go through in blocks of rows.  The last block (465 rows)
    is planned on its own and takes the copy-out buffer, which the scratch of the call has to cover."""
    x = workloads.normal_rows(66000, 9000, seed=41)  # 9000 f32 per row do not fit 64 KB of LDS
    assert atk.load_library().atk_exact_workspace_bytes(66000, 9000, 10, atk.ATK_F32) >= \
        atk.load_library().atk_exact_workspace_bytes(465, 9000, 10, atk.ATK_F32)
    run_exact(x, 10, rows=list(range(0, 65535, 4099)) + [65534] + list(range(65535, 66000)))


def test_exact_copy_out_more_rows_than_cus():
    """k up to 4096 with more rows than CUs: the copy-out path is taken when the input is big enough to pay
    for the rounds of one-row-per-CU selections (here 300 rows of 2^18: two rounds)."""
    x = workloads.normal_rows(300, 1 << 18, seed=43)
    run_exact(x, 3000)


def test_exact_cfg4():
    x = workloads.config_input("cfg4")
    run_exact(x, 64)
    run_exact(x, 1 << 18)


def test_b1_equals_exact():
    x = workloads.normal_rows(3, 4096, seed=9)
    xg = x.cuda()
    av, ai = atk.approx_topk(xg, 16, 1, 16)
    ev, ei = atk.exact_topk(xg, 16)
    torch.cuda.synchronize()
    assert torch.equal(ai, ei) and torch.equal(av, ev)


# ------------------------------------------------------------------------------- recall (Appendix C, Eq. 1)
def test_recall_matches_model_cfg2():
    from oracle import recall

    x = workloads.config_input("cfg2")
    xg = x.cuda()
    _, ei = oracle.exact_topk(workloads.as_numpy_bits(x), 64, threads=THREADS)
    m = x.shape[0]
    for k, b, k_b in workloads.CONFIGS["cfg2"]["cases"]:
        _, ai = atk.approx_topk(xg, k, b, k_b)
        ai = ai.cpu().numpy()
        rec = np.array([len(set(ei[r].tolist()) & set(ai[r].tolist())) / k for r in range(m)])
        se = rec.std(ddof=1) / np.sqrt(m)
        assert abs(rec.mean() - recall.expected_recall_iid_exact(x.shape[1], k, b, k_b)) < 4.5 * se + 1e-9


def test_alternating_sizes_share_the_scratch_pool():
    """Calls of different shapes reuse one scratch pool; tickets must read zero for each of them."""
    small = workloads.normal_rows(3, 32768, seed=41)
    big = workloads.normal_rows(128, 65536, seed=42)
    for _ in range(3):
        run_case(small, 64, 64, 1, tag="small")
        run_case(big, 64, 256, 1, tag="big")
        run_case(small, 128, 64, 2, tag="small")
        run_case(big, 64, 64, 1, tag="big")


def test_hip_graph_replay_matches_eager():
    """The calls can be captured in a HIP graph once the scratch pool has its size: replays, with
    eager work and synchronisations between them, give the eager results every time."""
    x1 = workloads.normal_rows(16, 32768, seed=31).cuda()
    x2 = workloads.normal_rows(16, 32768, seed=32).cuda()
    cases = [(64, 64, 1), (64, 512, 1), (128, 32, 4), (4096, 4096, 1)]
    eager = {}
    for xi, x in enumerate((x1, x2)):
        for c in cases:
            v, i = atk.approx_topk(x, *c)
            eager[(xi, c)] = (v.clone(), i.clone())
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    xin = x1.clone()
    outs = {c: (torch.empty((16, c[0]), dtype=torch.float32, device="cuda"),
                torch.empty((16, c[0]), dtype=torch.int32, device="cuda")) for c in cases}
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for c in cases:  # warm-up on the capture stream
            atk.approx_topk(xin, *c, out=outs[c])
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            for c in cases:
                atk.approx_topk(xin, *c, out=outs[c])
    for rep in range(4):
        xi = rep % 2
        xin.copy_((x1, x2)[xi])
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for c in cases:
            assert torch.equal(outs[c][0], eager[(xi, c)][0]) and torch.equal(outs[c][1], eager[(xi, c)][1]), (rep, c)
        # eager work between the replays, on the same pool
        v, i = atk.approx_topk(x2, 64, 256, 1)
        assert torch.equal(i, atk.approx_topk(x2, 64, 256, 1)[1])


# ------------------------------------------------------------------------------- choosing (b, k_b): estimate against the clock
def _time_call_us(x, k, b, k_b, reps=60):
    dt = atk.ATK_F32 if x[0].dtype == torch.float32 else atk.ATK_BF16
    m, n = x[0].shape
    ov = torch.empty((m, k), dtype=x[0].dtype, device="cuda")
    oi = torch.empty((m, k), dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream

    def go(i):
        rc = atk.approx_topk_raw(x[i % len(x)].data_ptr(), m, n, k, b, k_b, dt, ov.data_ptr(), oi.data_ptr(), st)
        assert rc == 0, atk.strerror(rc)

    for i in range(8):
        go(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        go(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def test_runtime_estimate_and_advice_against_the_clock():
    """atk_estimate_us (Appendix D's composition, Stage 1 + [b*k_b > k] Stage 2, with this library's measured terms)
    within a factor 1.6 of event timings on ten shapes, and atk_advise's choice for a recall target not slower, by
    more than that band, than the other ways of reaching the target (Appendix E: more buckets or more slots)."""
    band = 1.6
    shapes = [("f32", 128, 65536, [(64, 64, 1), (64, 256, 1), (64, 1024, 1), (16384, 16384, 1), (16384, 4096, 4), (16384, 1024, 16)]),
              ("bf16", 2048, 8192, [(512, 512, 1), (512, 1024, 1)]),
              ("f32", 8, 1 << 20, [(64, 64, 1)]),
              ("f32", 128, 1 << 18, [(64, 512, 1)])]
    for dtype, m, n, cases in shapes:
        cnt = max(2, min(12, (420 << 20) // (m * n * (4 if dtype == "f32" else 2))))
        xs = [workloads.normal_rows(m, n, seed=40 + s, dtype=dtype).cuda() for s in range(cnt)]
        dt = atk.ATK_F32 if dtype == "f32" else atk.ATK_BF16
        for (k, b, k_b) in cases:
            us, est = _time_call_us(xs, k, b, k_b), atk.estimate_us(m, n, k, b, k_b, dt)
            print("estimate %s %dx%d k=%d b=%d k_b=%d: measured %.2f us, estimated %.2f us" % (dtype, m, n, k, b, k_b, us, est), flush=True)
            assert us / band <= est <= us * band, (dtype, m, n, k, b, k_b, us, est)
        if (dtype, m, n) == ("f32", 128, 65536):
            for k, target in [(64, 0.9), (16384, 0.8)]:
                b, k_b, rec, est, reached = atk.advise(m, n, k, dt, target)
                assert reached and rec >= target
                t_pick = _time_call_us(xs, k, b, k_b)
                others = []
                for kb2 in (1, 2, 4, 8, 16):  # the cheapest b that reaches the target with kb2 slots
                    for ratio in (1, 2, 4, 8, 16, 32, 64):
                        b2 = -(-ratio * k // kb2)
                        b2 += (-b2) % 4
                        if (b2, kb2) != (b, k_b) and atk.load_library().atk_check_approx(m, n, k, b2, kb2, dt) == 0 and \
                                atk.expected_recall(k, b2, kb2) >= target:
                            others.append((_time_call_us(xs, k, b2, kb2), b2, kb2))
                            break
                print("advice k=%d target %.2f: picked b=%d k_b=%d %.2f us; others %s" % (k, target, b, k_b, t_pick, others), flush=True)
                assert others and t_pick <= band * min(o[0] for o in others)
        del xs
        torch.cuda.empty_cache()

"""Pins for the CPU oracle: everything here runs without a GPU.

Each test ties the oracle to something other than itself: the paper's worked example,
a brute-force rank count that shares nothing with the sort-based oracle, special cases
that reduce to a library sort, invariants, and the recall formulas of Appendix C.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import recall
from paper_2412_04358_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def brute_force(row, k, b, k_b, bucket=None):
    """O(n^2) definition by rank counting; returns the selected index list in output order.
    bucket(i): the bucket of element i (default: i mod b).

    rank_in_bucket(i) = #{j in bucket(i) : x_j ranks before x_i}; i is a candidate iff
    that rank is below k_b.  Without Stage 2 the output slot of candidate i is
    bucket*k_b + rank; with Stage 2 it is its rank among all candidates (kept if < k).
    """
    n = len(row)
    row = [float(v) for v in row]
    if bucket is None:
        bucket = lambda i: i % b
    members = {}
    for i in range(n):
        members.setdefault(bucket(i), []).append(i)
    assert sorted(members) == list(range(b))

    def before(j, i):  # does element j rank before element i ?
        return row[j] > row[i] or (row[j] == row[i] and j < i)

    cand = {}
    for i in range(n):
        r = sum(1 for j in members[bucket(i)] if before(j, i))
        if r < k_b:
            cand[i] = r
    assert len(cand) == b * k_b
    out = [None] * k
    if b * k_b == k:
        for i, r in cand.items():
            out[bucket(i) * k_b + r] = i
    else:
        for i in cand:
            r = sum(1 for j in cand if before(j, i))
            if r < k:
                out[r] = i
    assert all(o is not None for o in out)
    return out


def legal_params(n, divisible_only=False):
    for b in range(1, n + 1):
        if divisible_only and n % b:
            continue
        for k_b in range(1, n // b + 1):
            for k in sorted({k_b, b * k_b, max(k_b, (b * k_b) // 2), max(k_b, b * k_b - 1)}):
                if k_b <= k <= b * k_b:
                    yield k, b, k_b


def bits(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16)


def numpy_exact(x, k):
    """Library special case: stable argsort of the negated row = value desc, index asc."""
    xf = x.astype(np.float32) if x.dtype == np.float32 else (x.astype(np.uint32) << 16).view(np.float32)
    order = np.argsort(-xf, axis=1, kind="stable")[:, :k]
    return np.take_along_axis(x, order, axis=1), order.astype(np.int32)


# ----------------------------------------------------------------------------- Figure 2
def read_golden():
    d = {}
    with open(os.path.join(GOLDEN, "fig2_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            d[key] = [int(v) for v in vals]
    return d


def test_fig2_worked_example():
    g = read_golden()
    n, k, b, k_b = g["n"][0], g["k"][0], g["b"][0], g["k_b"][0]
    row = np.array([g["row"]], dtype=np.float32)
    assert row.shape == (1, n)
    vals, idx, cv, ci = oracle.approx_topk(row, k, b, k_b, return_candidates=True)
    # bucket membership printed in the figure
    for j in range(b):
        assert [int(v) for v in row[0, j::b]] == g["bucket%d" % j]
        got = sorted(int(v) for v in cv[0, j * k_b:(j + 1) * k_b])
        assert got == sorted(g["stage1_bucket%d" % j])
    assert sorted(int(v) for v in vals[0]) == sorted(g["final"])
    assert [int(row[0, i]) for i in idx[0]] == [int(v) for v in vals[0]]
    # this build's order convention: largest first after Stage 2
    assert [int(v) for v in vals[0]] == sorted(g["final"], reverse=True)


# ----------------------------------------------------------------------------- brute force
@pytest.mark.parametrize("kind", ["normal", "constant", "two_valued", "special"])
def test_brute_force_small(kind):
    rng = np.random.default_rng(7)
    checked = 0
    for n in list(range(1, 21)) + [24, 32, 33, 48, 64]:
        if kind == "normal":
            row = rng.standard_normal(n).astype(np.float32)
        elif kind == "constant":
            row = np.full(n, 1.5, dtype=np.float32)
        elif kind == "two_valued":
            row = rng.integers(0, 2, n).astype(np.float32)
        else:
            pool = np.array([0.0, -0.0, np.inf, -np.inf, 1e-45, -1e-45, 1.0, -1.0], dtype=np.float32)
            row = pool[rng.integers(0, len(pool), n)]
        params = list(legal_params(n))
        if n > 20:
            sel = rng.choice(len(params), size=min(40, len(params)), replace=False)
            params = [params[i] for i in sel]
        for k, b, k_b in params:
            vals, idx = oracle.approx_topk(row[None, :], k, b, k_b)
            want = brute_force(row, k, b, k_b)
            assert idx[0].tolist() == want, (n, k, b, k_b)
            assert np.array_equal(bits(vals[0]), bits(row[want])), (n, k, b, k_b)
            checked += 1
    assert checked > 500


@pytest.mark.parametrize("kind", ["normal", "two_valued"])
def test_brute_force_contiguous(kind):
    """Contiguous assignment (Appendix A.1): bucket of i is floor(b*i/n), any n and b."""
    rng = np.random.default_rng(11)
    checked = 0
    for n in list(range(1, 19)) + [24, 30, 33, 48, 64]:
        row = rng.standard_normal(n).astype(np.float32) if kind == "normal" else rng.integers(0, 2, n).astype(np.float32)
        params = list(legal_params(n))
        if n > 18:
            sel = rng.choice(len(params), size=min(40, len(params)), replace=False)
            params = [params[i] for i in sel]
        for k, b, k_b in params:
            vals, idx = oracle.approx_topk(row[None, :], k, b, k_b, assignment=oracle.CONTIGUOUS)
            want = brute_force(row, k, b, k_b, bucket=lambda i: (b * i) // n)
            assert idx[0].tolist() == want, (n, k, b, k_b)
            assert np.array_equal(bits(vals[0]), bits(row[want])), (n, k, b, k_b)
            checked += 1
    assert checked > 400


def test_contiguous_is_interleaved_of_the_transposed_row():
    """With b | n the row is a b x L matrix whose rows are the contiguous buckets; read column by
    column (transposed) the same buckets are interleaved.  Tie-free rows, so that Stage 2 does not
    depend on how indices are numbered."""
    for (n, k, b, k_b) in [(4096, 64, 64, 1), (4096, 48, 64, 1), (4096, 256, 64, 4), (6000, 100, 40, 3), (512, 512, 64, 8)]:
        L = n // b
        x = workloads.normal_rows(3, n, seed=n + k).numpy()
        xt = np.ascontiguousarray(x.reshape(3, b, L).transpose(0, 2, 1)).reshape(3, n)
        v1, i1 = oracle.approx_topk(x, k, b, k_b, assignment=oracle.CONTIGUOUS)
        v2, i2 = oracle.approx_topk(xt, k, b, k_b)
        # transposed index l*b + j  <->  original index j*L + l
        back = (i2 % b) * L + i2 // b
        assert np.array_equal(i1, back.astype(np.int32))
        assert np.array_equal(bits(v1), bits(v2))


def test_b1_and_b_equal_n_do_not_depend_on_the_assignment():
    x = workloads.normal_rows(2, 1000, seed=5).numpy()
    for (k, b, k_b) in [(10, 1, 10), (1000, 1000, 1), (300, 1000, 1)]:
        a = oracle.approx_topk(x, k, b, k_b)
        c = oracle.approx_topk(x, k, b, k_b, assignment=oracle.CONTIGUOUS)
        assert np.array_equal(a[1], c[1]) and np.array_equal(bits(a[0]), bits(c[0]))


def _recall(idx, exact_idx):
    return np.mean([len(set(a.tolist()) & set(e.tolist())) / len(e) for a, e in zip(idx, exact_idx)])


def test_correlated_sequences_hurt_contiguous_not_interleaved():
    """Appendix A.1's simulation: n = 2048, k = 256, x ~ N(0, Sigma), Sigma_ij = rho^|i-j|.  As rho
    grows the contiguous assignment loses recall (also for larger k_b), the interleaved one keeps
    it, and shuffling the row first brings the contiguous one back to the interleaved level."""
    n, k, rows = 2048, 256, 96
    for k_b in (1, 2, 4):
        b = k // k_b
        iid = recall.expected_recall_iid_exact(n, k, b, k_b)
        got = {}
        for rho in (0.0, 0.9, 0.99):
            x = workloads.correlated_rows(rows, n, rho, seed=17).numpy()
            xs = workloads.correlated_rows(rows, n, rho, seed=17, shuffle=True).numpy()
            ex = oracle.exact_topk(x, k)[1]
            exs = oracle.exact_topk(xs, k)[1]
            got[rho] = (
                _recall(oracle.approx_topk(x, k, b, k_b)[1], ex),
                _recall(oracle.approx_topk(x, k, b, k_b, assignment=oracle.CONTIGUOUS)[1], ex),
                _recall(oracle.approx_topk(xs, k, b, k_b, assignment=oracle.CONTIGUOUS)[1], exs),
            )
        inter0, contig0, shuf0 = got[0.0]
        assert abs(inter0 - iid) < 0.02 and abs(contig0 - iid) < 0.02 and abs(shuf0 - iid) < 0.02
        for rho in (0.9, 0.99):
            inter, contig, shuf = got[rho]
            assert inter > iid - 0.02          # interleaving keeps (or improves on) the i.i.d. recall
            assert abs(shuf - iid) < 0.02      # a shuffled row is exchangeable: the i.i.d. value again
            assert contig < inter - 0.05       # contiguous buckets share the runs of large values
        assert got[0.99][1] < got[0.9][1] < got[0.0][1] + 0.02


def test_brute_force_bf16_ties():
    rng = np.random.default_rng(3)
    for n in [16, 40, 64]:
        x = (rng.standard_normal(n) * 0.5).astype(np.float32)
        xb = (x.view(np.uint32) >> 16).astype(np.uint16)  # truncation: just need bf16 patterns with ties
        xb[rng.integers(0, n, n // 3)] = xb[0]
        xf = (xb.astype(np.uint32) << 16).view(np.float32)
        for k, b, k_b in list(legal_params(n, divisible_only=True))[::3]:
            vals, idx = oracle.approx_topk(xb[None, :], k, b, k_b)
            want = brute_force(xf, k, b, k_b)
            assert idx[0].tolist() == want
            assert np.array_equal(vals[0], xb[want])


def test_exact_brute_force_and_numpy():
    rng = np.random.default_rng(11)
    for n in [1, 2, 7, 33, 64]:
        row = rng.integers(-3, 4, n).astype(np.float32)  # ties on purpose
        for k in sorted({1, n, (n + 1) // 2}):
            vals, idx = oracle.exact_topk(row[None, :], k)
            want = brute_force(row, k, 1, k)  # b = 1: one bucket holding the row
            assert idx[0].tolist() == want
            nv, ni = numpy_exact(row[None, :], k)
            assert np.array_equal(idx, ni) and np.array_equal(bits(vals), bits(nv))


# ----------------------------------------------------------------------------- special cases
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_b1_is_exact_topk(dtype):
    x = workloads.as_numpy_bits(workloads.normal_rows(3, 1000, seed=1, dtype=dtype))
    for k in [1, 10, 1000]:
        v, i = oracle.approx_topk(x, k, 1, k)
        nv, ni = numpy_exact(x, k)
        assert np.array_equal(i, ni) and np.array_equal(bits(v), bits(nv))
        ev, ei = oracle.exact_topk(x, k)
        assert np.array_equal(i, ei) and np.array_equal(bits(v), bits(ev))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_full_buckets_return_everything(dtype):
    """k_b = n/b makes every element a candidate, so Stage 2 is an exact top-k."""
    x = workloads.as_numpy_bits(workloads.few_levels(2, 96, levels=5, seed=2, dtype=dtype))
    n = x.shape[1]
    for b in [2, 8, 32]:
        k_b = n // b
        for k in [k_b, 50, n]:
            v, i = oracle.approx_topk(x, k, b, k_b)
            if k < n:
                nv, ni = numpy_exact(x, k)
                assert np.array_equal(i, ni) and np.array_equal(bits(v), bits(nv))
            else:
                # no Stage 2: bucket-major, each bucket fully sorted
                assert sorted(i[0].tolist()) == list(range(n))
                for j in range(b):
                    nv, ni = numpy_exact(x[:, j::b], k_b)
                    assert np.array_equal(i[:, j * k_b:(j + 1) * k_b], ni * b + j)


def test_invariants_random():
    x = workloads.as_numpy_bits(workloads.normal_rows(8, 4096, seed=5))
    m, n = x.shape
    ev, ei = oracle.exact_topk(x, n)
    for k, b, k_b in [(64, 64, 1), (64, 256, 1), (256, 64, 4), (100, 128, 2), (1024, 256, 4)]:
        v, i = oracle.approx_topk(x, k, b, k_b)
        assert np.array_equal(bits(np.take_along_axis(x, i.astype(np.int64), axis=1)), bits(v))
        for r in range(m):
            assert len(set(i[r].tolist())) == k
            # the k_b globally largest elements are always returned (Appendix C: E[Z(k_b,b,k_b)] = k_b)
            assert set(ei[r, :k_b].tolist()) <= set(i[r].tolist())
        if b * k_b == k:
            assert np.array_equal(i % b, np.repeat(np.arange(b), k_b)[None, :].repeat(m, 0))
            vv = v.reshape(m, b, k_b)
            assert np.all(vv[:, :, :-1] >= vv[:, :, 1:])
        else:
            assert np.all(v[:, :-1] >= v[:, 1:])


def test_kb1_recall_equals_distinct_buckets():
    """Appendix C: Z(k, b, 1) is the number of distinct buckets that hold a true top-k value."""
    x = workloads.as_numpy_bits(workloads.normal_rows(16, 4096, seed=6))
    for k, b in [(64, 64), (64, 256), (32, 512)]:
        _, ei = oracle.exact_topk(x, k)
        _, ai = oracle.approx_topk(x, k, b, 1)
        for r in range(x.shape[0]):
            z = len(set(ei[r].tolist()) & set(ai[r].tolist()))
            assert z == len(set((ei[r] % b).tolist()))


def test_nesting_in_b():
    """Doubling b splits every bucket in two, so k_b=1 candidates (and recall) only grow."""
    x = workloads.as_numpy_bits(workloads.normal_rows(8, 4096, seed=8))
    k = 64
    _, ei = oracle.exact_topk(x, k)
    prev_c, prev_rec = None, None
    for b in [64, 128, 256, 512, 1024]:
        _, ai, _, ci = oracle.approx_topk(x, k, b, 1, return_candidates=True)
        rec = [len(set(ei[r].tolist()) & set(ai[r].tolist())) for r in range(x.shape[0])]
        if prev_c is not None:
            for r in range(x.shape[0]):
                assert set(prev_c[r].tolist()) <= set(ci[r].tolist())
                assert rec[r] >= prev_rec[r]
        prev_c, prev_rec = ci, rec


def test_worst_case_eq2():
    """Appendix C, Eq. 2: true top-k packed into the fewest buckets."""
    rng = np.random.default_rng(0)
    for n, k, b, k_b in [(64, 8, 8, 1), (64, 12, 8, 2), (256, 40, 16, 4), (128, 16, 16, 1), (64, 20, 16, 2)]:
        length = n // b
        row = rng.standard_normal(n).astype(np.float32) - 100.0
        # fill buckets 0, 1, ... completely with the largest values until k are placed
        placed = 0
        for j in range(b):
            for t in range(length):
                if placed < k:
                    row[t * b + j] = 100.0 + placed
                    placed += 1
        _, ei = oracle.exact_topk(row[None, :], k)
        _, ai = oracle.approx_topk(row[None, :], k, b, k_b)
        got = len(set(ei[0].tolist()) & set(ai[0].tolist())) / k
        assert got == pytest.approx(recall.worst_case_recall(n, k, b, k_b), abs=1e-12), (n, k, b, k_b)


# ----------------------------------------------------------------------------- recall model
def test_eq1_kb1_closed_form():
    for k, b in [(64, 64), (64, 1024), (512, 512), (100, 1000), (16384, 16384)]:
        assert recall.expected_recall_eq1(k, b, 1) == pytest.approx(recall.expected_recall_kb1(k, b), rel=1e-9)
    # values quoted for the benchmark configurations
    assert recall.expected_recall_kb1(64, 64) == pytest.approx(0.6350, abs=5e-4)
    assert recall.expected_recall_kb1(64, 1024) == pytest.approx(0.9699, abs=5e-4)


def test_eq1_is_large_n_limit_of_exact_form():
    for k, b, k_b in [(64, 64, 1), (64, 32, 2), (64, 32, 4)]:
        big = recall.expected_recall_iid_exact(b * 100000, k, b, k_b)
        assert big == pytest.approx(recall.expected_recall_eq1(k, b, k_b), abs=2e-4)
    # dropping k_b << n/b: Eq. 1 bounds the error from above, i.e. the recall from below
    for n, k, b, k_b in [(4096, 1024, 1024, 1), (4096, 1024, 256, 4), (65536, 16384, 1024, 16)]:
        assert recall.expected_recall_iid_exact(n, k, b, k_b) >= recall.expected_recall_eq1(k, b, k_b)


@pytest.mark.parametrize("n,k,b,k_b,rows", [
    (4096, 64, 64, 1, 256),
    (4096, 64, 256, 1, 256),
    (4096, 1024, 1024, 1, 64),
    (4096, 1024, 256, 4, 64),
    (4096, 1024, 64, 16, 64),
    (4096, 64, 32, 2, 256),
    (1000, 50, 30, 2, 256),      # n not a multiple of b
])
def test_measured_recall_matches_model(n, k, b, k_b, rows):
    """Monte-Carlo recall of the oracle on i.i.d. rows vs the closed forms (Appendix C, Eq. 1)."""
    x = workloads.as_numpy_bits(workloads.normal_rows(rows, n, seed=123))
    _, ei = oracle.exact_topk(x, k)
    _, ai = oracle.approx_topk(x, k, b, k_b)
    rec = np.array([len(set(ei[r].tolist()) & set(ai[r].tolist())) / k for r in range(rows)])
    se = rec.std(ddof=1) / np.sqrt(rows)
    exact = recall.expected_recall_iid_exact(n, k, b, k_b)
    assert abs(rec.mean() - exact) < 4.5 * se + 1e-9, (rec.mean(), exact, se)
    assert rec.mean() >= recall.expected_recall_eq1(k, b, k_b) - 4.5 * se


def test_argument_checks():
    x = np.zeros((1, 16), dtype=np.float32)
    for k, b, k_b in [(4, 2, 1), (4, 4, 5), (4, 17, 1), (0, 1, 1), (17, 1, 17), (8, 4, 5), (1, 4, 2)]:
        with pytest.raises(ValueError):
            oracle.approx_topk(x, k, b, k_b)
    with pytest.raises(ValueError):
        oracle.exact_topk(x, 17)

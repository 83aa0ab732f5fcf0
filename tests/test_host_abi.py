"""Host-side checks of the C-ABI library that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest

import paper_2412_04358_amd as atk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(atk.lib_path()):
        import __graft_entry__

        __graft_entry__.build()
    return atk.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "approx_topk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", text)
    return sorted(set(n for n in names if n.startswith("atk_") or n in ("approx_topk", "approx_topk_assign", "exact_topk")))


def test_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert "approx_topk" in names and "exact_topk" in names and "approx_topk_assign" in names and len(names) >= 12
    for n in names:
        assert hasattr(lib, n), "library does not export %s" % n


OK, NULLP, SHAPE, PARAMS, UNSUP, DTYPE = 0, -1, -2, -3, -4, -5


@pytest.mark.parametrize("args,code", [
    ((4, 4096, 64, 64, 1, 0), OK),
    ((128, 65536, 64, 1024, 1, 0), OK),
    ((128, 65536, 16384, 1024, 16, 0), OK),
    ((2048, 8192, 512, 512, 1, 1), OK),
    ((1, 16, 16, 1, 16, 0), OK),            # b = 1: exact top-k by one bucket
    ((0, 4096, 64, 64, 1, 0), SHAPE),
    ((4, 0, 64, 64, 1, 0), SHAPE),
    ((4, 4096, 0, 64, 1, 0), SHAPE),
    ((4, 4096, 4097, 64, 1, 0), SHAPE),
    ((1, 1 << 31, 64, 64, 1, 0), SHAPE),
    ((4, 4096, 64, 0, 1, 0), PARAMS),
    ((4, 4096, 64, 8192, 1, 0), PARAMS),    # b > n
    ((4, 4096, 64, 64, 0, 0), PARAMS),
    ((4, 4096, 64, 32, 1, 0), PARAMS),      # b*k_b < k
    ((4, 4096, 8, 8, 16, 0), PARAMS),       # k_b > k
    ((4, 4096, 4096, 2048, 4, 0), PARAMS),  # k_b > n/b
    ((4, 4096, 64, 64, 1, 2), DTYPE),
    ((4, 4096, 64, 64, 1, -1), DTYPE),
    ((4, 4095, 64, 64, 1, 0), OK),          # n not a multiple of b: short buckets
    ((4, 4095, 64, 64, 64, 0), PARAMS),     # k_b above floor(n/b)
    ((4, 4096, 64, 2, 32, 0), UNSUP),       # k_b above the register-queue cap
    ((4, 1 << 16, 64, 1 << 13, 1, 0), OK),     # Stage 2 over more candidates than fit on chip: further launches
])
def test_check_approx(lib, args, code):
    assert lib.atk_check_approx(*args) == code


def test_calls_reject_before_hip(lib):
    """No GPU here: these must return their code from the host-side checks alone."""
    fake = 0x1000  # never dereferenced: checks fail first
    assert lib.approx_topk(None, 4, 4096, 64, 64, 1, 0, fake, fake, None) == NULLP
    assert lib.approx_topk(fake, 4, 4096, 64, 64, 1, 0, None, fake, None) == NULLP
    assert lib.approx_topk(fake, 4, 4096, 64, 64, 1, 0, fake, None, None) == NULLP
    assert lib.approx_topk(fake, 4, 4096, 64, 32, 1, 0, fake, fake, None) == PARAMS
    assert lib.approx_topk(fake, 4, 4096, 64, 64, 1, 7, fake, fake, None) == DTYPE
    assert lib.approx_topk(fake + 2, 4, 4096, 64, 64, 1, 0, fake, fake, None) == -7
    assert lib.exact_topk(None, 4, 4096, 64, 0, fake, fake, None) == NULLP
    assert lib.exact_topk(fake, 4, 4096, 5000, 0, fake, fake, None) == SHAPE
    assert lib.exact_topk(fake, 4, 4096, 64, 3, fake, fake, None) == DTYPE
    assert lib.atk_read_ceiling(None, 1024, fake, None) == NULLP
    assert lib.atk_sleep(-1, None) == SHAPE


def test_noalloc_rejects_what_does_not_fit(lib):
    """Checked on the host before anything is launched: the pointers are never touched."""
    fake = 0x1000
    # 128 rows of 2^22 elements, 1024 buckets of 16 slots, rows split over workgroups: 67 MB of partial lists
    m, n, k, b, k_b = 128, 1 << 22, 16384, 1024, 16
    need = lib.atk_workspace_bytes(m, n, k, b, k_b, 0)
    assert need > (16 << 20), need
    assert lib.approx_topk_noalloc(fake, m, n, k, b, k_b, 0, fake, fake, None) == -8
    assert b"scratch" in lib.atk_strerror(-8)
    # Stage 2 over more candidates than one workgroup holds takes further launches and their buffers
    assert lib.approx_topk_noalloc(fake, 4, 1 << 16, 64, 1 << 13, 1, 0, fake, fake, None) == UNSUP
    # the argument checks of approx_topk
    assert lib.approx_topk_noalloc(None, 4, 4096, 64, 64, 1, 0, fake, fake, None) == -1
    assert lib.approx_topk_noalloc(fake, 4, 4096, 64, 32, 1, 0, fake, fake, None) == -3
    assert lib.approx_topk_noalloc(fake + 2, 4, 4096, 64, 64, 1, 0, fake, fake, None) == -7


def test_strerror(lib):
    seen = set()
    for code in range(0, -9, -1):
        s = atk.strerror(code)
        assert s and s != "unknown error code"
        seen.add(s)
    assert len(seen) == 9
    assert atk.strerror(-99) == "unknown error code"


def parse_plan(s):
    return {k: int(v) for k, v in (kv.split("=") for kv in s.split())}


def test_plan_shapes(lib):
    # every lane owns whole buckets: straight from registers, one workgroup column block per 1024 columns
    p = parse_plan(atk.plan_describe(128, 65536, 16384, 16384, 1))
    assert p["direct"] == 1 and p["P"] == 1 and p["S"] == 1 and p["colblocks"] == 16 and p["stage2"] == 0
    # few buckets: lanes share columns (P > 1, merged inside the wavefront).  Without Stage 2 the
    # workgroups of a row take 128-byte pieces of the matrix rows (whole buckets each) rather than
    # splitting the rows, so no scratch
    p = parse_plan(atk.plan_describe(128, 65536, 64, 64, 1))
    assert p["V"] == 4 and p["Gw"] == 8 and p["colblocks"] == 2 and p["P"] * p["Gw"] == p["T"] and p["wave_merge"] == 1
    assert p["S"] == 1 and p["scratch"] == 0 and p["direct"] == 0 and p["nparts"] == p["T"] // 64
    assert p["grid"] == 256
    # fewer rows than that fills the chip with: rows are split on top; the splits of a row and column block run as
    # helpers and a finisher (one mailbox per helper, the finisher takes what the helpers' equal shares leave)
    p = parse_plan(atk.plan_describe(32, 65536, 64, 64, 1))
    assert p["Gw"] == 8 and p["colblocks"] == 2 and p["S"] == 1 and p["scratch"] == 0 and p["lean"] == 1
    assert p["helpers"] >= 1 and p["grid"] == 32 * 2 * (p["helpers"] + 1)
    assert p["pair_rows"] % p["P"] == 0 and 0 < 1024 - p["helpers"] * p["pair_rows"] <= 2 * p["pair_rows"]
    assert p["scratch_bytes"] == 32 * 2 * p["helpers"] * p["Gw"] * p["V"] * 8
    # ... or, with queues of several slots, meet through scratch and a ticket
    p = parse_plan(atk.plan_describe(32, 65536, 128, 64, 2))
    assert p["S"] > 1 and p["scratch"] == 1 and p["helpers"] == 0
    assert p["S"] * p["rows_per_split"] >= 1024 and (p["S"] - 1) * p["rows_per_split"] < 1024
    assert p["rows_per_split"] % p["P"] == 0
    # with Stage 2 one workgroup must see every candidate of the row: the columns stay together; few rows of 2^17
    # elements go to helpers and a finisher, up to 32 rows of 65536 to three helpers and a finisher, more to a pair
    p = parse_plan(atk.plan_describe(32, 1 << 17, 64, 128, 1))
    assert p["Gw"] == 32 and p["colblocks"] == 1 and p["S"] == 1 and p["scratch"] == 0 and p["helpers"] > 1
    assert p["helpers"] * p["Gw"] * p["V"] <= 8 * p["T"]  # (the finisher fetches at most eight words per lane)
    p = parse_plan(atk.plan_describe(32, 65536, 64, 128, 1))
    assert p["colblocks"] == 1 and p["S"] == 1 and p["scratch"] == 0 and p["lean"] == 1 and p["helpers"] == 3 and p["pair_rows"] == 128
    p = parse_plan(atk.plan_describe(64, 65536, 64, 128, 1))
    assert p["Gw"] == 32 and p["colblocks"] == 1 and p["S"] == 1 and p["scratch"] == 0 and p["lean"] == 1
    assert p["helpers"] == 0 and p["pair_rows"] == 256 and p["grid"] == 128
    # more helpers' words than that: the row splits stay, through scratch and a ticket
    p = parse_plan(atk.plan_describe(1, 1 << 20, 64, 1024, 1))
    assert p["S"] > 1 and p["scratch"] == 1 and p["helpers"] == 0
    # Stage 2 fused
    p = parse_plan(atk.plan_describe(128, 65536, 64, 1024, 1))
    assert p["stage2"] == 1 and p["lds"] >= (1024 + 64) * 8
    # bf16 uses 8 columns per lane
    p = parse_plan(atk.plan_describe(2048, 8192, 512, 512, 1, atk.ATK_BF16))
    assert p["V"] == 8 and p["Gw"] == 64 and p["wave_merge"] == 0
    # b not a multiple of the vector width: the widest lanes that still divide b and n, else scalar columns
    p = parse_plan(atk.plan_describe(2, 4098, 6, 6, 1))
    assert p["V"] == 2 and p["wave_merge"] == 0
    p = parse_plan(atk.plan_describe(2, 4095, 7, 7, 1))
    assert p["V"] == 1 and p["wave_merge"] == 0
    # several slots per bucket: narrower lanes than for k_b = 1
    p = parse_plan(atk.plan_describe(128, 65536, 16384, 4096, 4))
    assert p["V"] == 2 and p["KB"] == 4 and p["direct"] == 1
    # big register queues keep to 256 lanes
    p = parse_plan(atk.plan_describe(128, 1 << 20, 64, 8, 8))
    assert p["KB"] == 8 and p["T"] <= 256
    # the grid always covers every matrix row and column exactly once, LDS stays within 64 KB
    for (m, n, k, b, kb) in [(1, 4096, 64, 64, 1), (3, 12288, 96, 96, 1), (7, 1 << 20, 64, 8, 8),
                             (128, 1 << 20, 1 << 18, 1 << 15, 8), (5, 8192, 1, 1, 1), (4, 16384, 100, 128, 16),
                             (1, 1 << 18, 64, 512, 1), (130, 4096, 64, 128, 1), (5, 1677, 371, 371, 2), (3, 3000, 700, 350, 2),
                             # few rows with Stage 2 (column blocks instead of row splits), queues on launches of few lanes
                             # (lanes share column groups), many short rows, vocabulary-sized rows with odd bucket counts
                             (4, 1 << 22, 64, 4096, 1), (8, 151936, 256, 512, 2), (1, 1 << 24, 64, 128, 1), (128, 65536, 4096, 1024, 4),
                             (128, 65536, 1024, 128, 16), (1, 1 << 20, 4096, 256, 16), (2048, 16384, 256, 64, 4), (256, 32000, 64, 501, 1),
                             (32, 1 << 18, 1024, 256, 4), (128, 1 << 18, 16384, 2048, 8), (512, 50000, 1024, 256, 4)]:
        p = parse_plan(atk.plan_describe(m, n, k, b, kb))
        assert p["grid"] == m * p["S"] * p["colblocks"]
        assert p["colblocks"] * p["Gw"] * p["V"] >= b
        assert p["S"] * p["rows_per_split"] >= n // b and (p["S"] - 1) * p["rows_per_split"] < n // b
        assert p["T"] % 64 == 0 and p["P"] * p["Gw"] <= p["T"] and p["lds"] <= 65536


def test_helper_and_pair_plans_fit_what_the_kernels_index(lib):
    """Plans that hand maxima over through mailboxes (a helper + finisher pair; several helpers per finisher): the grid,
    the helpers' shares of the matrix rows, the finisher's share and the mailbox bytes must be what the kernels' index
    arithmetic assumes - a pair knows no column blocks, helpers take whole numbers of row phases and leave the finisher at
    least one row per phase, and the finisher fetches at most eight mailbox words per lane."""
    n_multi = n_pair = 0
    for dt, es in ((atk.ATK_F32, 4), (atk.ATK_BF16, 2)):
        for n in (1 << 16, 1 << 17, 1 << 18, 1 << 19, 1 << 20, 1 << 22, 96 * 4096, 3 * (1 << 17)):
            for m in (1, 2, 3, 4, 8, 16, 32, 64, 100, 128):
                for b in (32, 64, 96, 128, 256, 512, 1024, 2048):
                    if n % b:
                        continue
                    for k in (64, b):
                        if k > b:
                            continue
                        d = atk.plan_describe(m, n, k, b, 1, dt)
                        p = parse_plan(d)
                        L = n // b
                        if p["helpers"] == 0:
                            if p["pair_rows"] > 0:
                                n_pair += 1
                                assert p["grid"] == 2 * m and p["colblocks"] == 1 and p["lean"] == 1 and p["S"] == 1, d
                                assert 0 < p["pair_rows"] < L and p["pair_rows"] % p["P"] == 0 and L - p["pair_rows"] >= p["P"], d
                                assert p["scratch_bytes"] >= m * b * 8, d
                            continue
                        n_multi += 1
                        H, Lh = p["helpers"], p["pair_rows"]
                        stride = p["Gw"] * p["V"]
                        assert p["lean"] == 1 and p["S"] == 1 and p["V"] == 16 // es, d
                        assert p["grid"] == m * p["colblocks"] * (H + 1), d
                        assert Lh >= p["P"] and Lh % p["P"] == 0 and H * Lh < L and L - H * Lh >= p["P"], d
                        assert p["scratch_bytes"] >= m * p["colblocks"] * H * stride * 8, d
                        assert H * stride <= 8 * p["T"] and p["Gw"] * p["P"] <= p["T"], d
                        assert p["stage2"] == 0 or p["colblocks"] == 1, d
    assert n_multi > 500 and n_pair > 100, (n_multi, n_pair)


def parse_contig_plan(s):
    assert s.startswith("contiguous ")
    return parse_plan(s[len("contiguous "):])


def test_contiguous_plan_shapes(lib):
    """Launch geometry of the contiguous-assignment kernel covers every bucket and every chunk."""
    C = atk.ATK_CONTIGUOUS
    shapes = [(4, 4096, 64, 64, 1), (128, 65536, 64, 64, 1), (128, 65536, 64, 1024, 1), (128, 65536, 16384, 16384, 1),
              (128, 65536, 16384, 1024, 16), (2, 4098, 6, 6, 1), (2, 4098, 683, 683, 1), (5, 8192, 1, 1, 1),
              (1, 1 << 20, 64, 8, 8), (1, 1 << 20, 64, 64, 1), (3, 1 << 18, 256, 32, 8), (1, 128256, 256, 1000, 2),
              (128, 1 << 20, 64, 64, 1), (2048, 8192, 512, 512, 1), (7, 1000, 30, 30, 1), (1, 2653751, 100, 128, 2)]
    for dt, vfull in ((atk.ATK_F32, 4), (atk.ATK_BF16, 8)):
        for (m, n, k, b, kb) in shapes:
            p = parse_contig_plan(atk.plan_describe(m, n, k, b, kb, dt, C))
            T, Gs = p["T"], p["Gs"]
            assert T % 64 == 0 and 64 <= T <= 1024 and Gs >= 1 and (Gs & (Gs - 1)) == 0
            assert Gs <= 64 or Gs == T
            assert p["V"] in (1, vfull)
            if p["V"] > 1:
                assert n % b == 0 and (n // b) % p["V"] == 0
            chunks = -(-n // b) // p["V"]
            assert p["bblocks"] * (T // Gs) * max(1, p["NB"]) >= b
            if p["NB"] > 0:
                assert chunks <= Gs <= 64 and p["S"] == 1
            assert p["S"] * p["chunks_per_split"] >= chunks and (p["S"] - 1) * p["chunks_per_split"] < chunks
            assert p["S"] == 1 or Gs == T
            assert p["grid"] == m * p["S"] * p["bblocks"]
            assert p["lds"] <= 65536
            assert p["scratch"] == int(p["S"] > 1 or (p["stage2"] == 1 and p["bblocks"] > 1))
    # a short run per bucket: one lane each, written straight out
    p = parse_contig_plan(atk.plan_describe(128, 65536, 16384, 16384, 1, atk.ATK_F32, C))
    assert p["Gs"] == 1 and p["V"] == 4 and p["scratch"] == 0 and p["NB"] >= 1
    # one long row, few buckets: whole workgroups per bucket and row splits
    p = parse_contig_plan(atk.plan_describe(1, 1 << 20, 64, 8, 8, atk.ATK_F32, C))
    assert p["Gs"] == p["T"] and p["S"] > 1 and p["scratch"] == 1


def test_assign_argument_checks(lib):
    fake = ctypes.c_void_p(0x1000)
    assert lib.approx_topk_assign(fake, 4, 4096, 64, 64, 1, 0, 2, fake, fake, None) == PARAMS
    assert lib.approx_topk_assign(fake, 4, 4096, 64, 64, 1, 0, -1, fake, fake, None) == PARAMS
    assert lib.approx_topk_assign(None, 4, 4096, 64, 64, 1, 0, 1, fake, fake, None) == NULLP
    assert lib.approx_topk_assign(fake, 4, 4096, 64, 32, 1, 0, 1, fake, fake, None) == PARAMS
    buf = ctypes.create_string_buffer(256)
    assert lib.atk_plan_describe_assign(4, 4096, 64, 64, 1, 0, 3, buf, 256) == PARAMS
    assert lib.atk_plan_describe_assign(4, 4096, 64, 64, 1, 0, 0, buf, 256) == OK and buf.value.startswith(b"V=")


def test_plan_override(lib, plan_override):
    plan_override("T=64,S=3")
    p = parse_plan(atk.plan_describe(4, 1 << 16, 64, 64, 1))
    assert p["T"] == 64 and p["S"] == 3
    plan_override("T=1024")
    p = parse_plan(atk.plan_describe(4, 1 << 16, 64, 64, 1))
    assert p["T"] == 1024
    plan_override("V=1")
    p = parse_plan(atk.plan_describe(4, 1 << 16, 64, 64, 1))
    assert p["V"] == 1
    plan_override("V=4")
    p = parse_plan(atk.plan_describe(4, 1 << 16, 64, 64, 4))
    assert p["V"] == 4
    plan_override(None)
    q = parse_plan(atk.plan_describe(4, 1 << 16, 64, 64, 1))
    assert q["T"] in (256, 512)


def test_long_queue_lane_widths(lib):
    """f32 queues of 16 slots take one column per lane while two would leave one wavefront per SIMD, two beyond."""
    assert atk.plan_describe(128, 65536, 16384, 1024, 16).startswith("V=1 KB=16 ")
    assert atk.plan_describe(128, 1 << 20, 1 << 18, 1 << 14, 16).startswith("V=2 KB=16 ")
    assert atk.plan_describe(128, 65536, 16384, 2048, 8).startswith("V=2 KB=8 ")


def test_workspace_bytes(lib):
    assert lib.atk_workspace_bytes(128, 65536, 16384, 16384, 1, 0) == 0
    assert lib.atk_workspace_bytes(128, 65536, 64, 64, 1, 0) == 0  # whole buckets per workgroup: no hand-over
    p = parse_plan(atk.plan_describe(32, 65536, 64, 64, 1))
    assert lib.atk_workspace_bytes(32, 65536, 64, 64, 1, 0) == p["scratch_bytes"] > 0
    assert lib.atk_workspace_bytes(128, 65536, 64, 32, 1, 0) == PARAMS
    assert lib.atk_stage2_max_candidates() >= 1024
    # more candidates than one workgroup holds: Stage 1 writes them to scratch (values + indices) for the second step
    p2 = parse_plan(atk.plan_describe(4, 1 << 16, 64, 1 << 13, 1))
    assert p2["stage2"] == 2 and p2["scratch_bytes"] >= 4 * (1 << 13) * 8
    assert lib.atk_workspace_bytes(4, 1 << 16, 64, 1 << 13, 1, 0) == p2["scratch_bytes"]
    assert lib.atk_workspace_bytes_assign(128, 65536, 64, 64, 1, 0, 0) == lib.atk_workspace_bytes(128, 65536, 64, 64, 1, 0)
    pc = parse_contig_plan(atk.plan_describe(1, 1 << 20, 64, 8, 8, atk.ATK_F32, atk.ATK_CONTIGUOUS))
    assert lib.atk_workspace_bytes_assign(1, 1 << 20, 64, 8, 8, 0, 1) == pc["scratch_bytes"] > 0
    assert lib.atk_workspace_bytes_assign(128, 65536, 16384, 16384, 1, 0, 1) == 0
    assert lib.atk_workspace_bytes_assign(128, 65536, 64, 64, 1, 0, 5) == PARAMS


def test_scratch_covers_every_block_of_rows(lib):
    """More long rows than a grid dimension holds go through in blocks of 65535 rows, and the last, smaller block
    is planned on its own: with fewer rows it may switch on buffers the full blocks do not use (the copy-out
    buffer of small k).  The scratch of the whole call must cover every block's plan."""
    block = 65535

    def parts(m, n, k, dt):
        st, da = ctypes.c_int64(0), ctypes.c_int64(0)
        assert lib.atk_exact_workspace_parts(m, n, k, dt, ctypes.byref(st), ctypes.byref(da)) == OK
        assert st.value + da.value == lib.atk_exact_workspace_bytes(m, n, k, dt)
        return st.value, da.value

    for dt in (0, 1):
        for (n, k) in [(9000, 10), (9000, 700), (20000, 64), (20000, 3000), (9000, 4096), (40000, 1), (9000, 9000)]:
            full = parts(block, n, k, dt)
            assert full[0] > 0 and full[1] > 0
            for rem in (1, 255, 256, 257, 465, 4000, 30000, 65534):
                last = parts(rem, n, k, dt)
                for blocks in (1, 2):
                    total = parts(blocks * block + rem, n, k, dt)
                    for pool in (0, 1):  # state and data live in separate pools: each must cover every block
                        assert total[pool] >= full[pool] and total[pool] >= last[pool], (dt, n, k, rem, blocks, total, full, last)
    # the case that showed it: 66000 x 9000 f32, k = 10 - the data of the 465-row last block (with the copy-out
    # buffer) is twice the first block's
    assert parts(465, 9000, 10, 0)[1] > parts(block, 9000, 10, 0)[1]
    assert parts(66000, 9000, 10, 0)[1] >= parts(465, 9000, 10, 0)[1]
    # Stage 2 over more candidates than one workgroup holds runs the same selection over the candidates
    for (m, n, k, b, k_b) in [(block + 465, 20000, 10, 9000, 1), (block + 300, 30000, 100, 5000, 2)]:
        ws = lib.atk_workspace_bytes(m, n, k, b, k_b, 0)
        assert ws >= lib.atk_exact_workspace_bytes(m - block, b * k_b, k, 0) + m * b * k_b * 8
        assert ws >= lib.atk_exact_workspace_bytes(block, b * k_b, k, 0) + m * b * k_b * 8


def test_plan_override_is_read_from_the_environment_once():
    """ATK_PLAN is parsed when the library is loaded, not on every call: a fresh process sees it,
    a change of the variable afterwards does nothing, atk_set_plan_override() replaces it."""
    import subprocess
    import sys

    code = ("import os, paper_2412_04358_amd as atk\n"
            "a = atk.plan_describe(4, 65536, 64, 64, 1)\n"
            "os.environ['ATK_PLAN'] = 'T=1024'\n"
            "b = atk.plan_describe(4, 65536, 64, 64, 1)\n"
            "atk.set_plan_override('T=128')\n"
            "c = atk.plan_describe(4, 65536, 64, 64, 1)\n"
            "atk.set_plan_override(None)\n"
            "d = atk.plan_describe(4, 65536, 64, 64, 1)\n"
            "print(' T=64 ' in a, a == b, ' T=128 ' in c, ' T=64 ' in d or ' T=128 ' in d)\n")
    env = dict(os.environ, ATK_PLAN="T=64,S=2", PYTHONPATH=ROOT)
    out = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, cwd=ROOT)
    assert out.returncode == 0, out.stderr
    assert out.stdout.split() == ["True", "True", "True", "False"], out.stdout


# ----------------------------------------------------------------------------- choosing (b, k_b)
def test_expected_recall_is_eq1(lib):
    """The library's Eq. 1 (per-bucket form, k_b terms) against the oracle's (sum of binomial CDFs):
    two independent writings of the same formula."""
    from oracle import recall

    for (k, b, k_b) in [(64, 64, 1), (64, 1024, 1), (16384, 4096, 4), (16384, 1024, 16), (256, 256, 1), (100, 128, 2),
                        (64, 8, 8), (512, 512, 1), (7, 3, 3), (1, 1, 1), (100, 1, 100), (300, 77, 5)]:
        assert abs(atk.expected_recall(k, b, k_b) - recall.expected_recall_eq1(k, b, k_b)) < 1e-9
    assert abs(atk.expected_recall(64, 64, 1) - recall.expected_recall_kb1(64, 64)) < 1e-12
    assert atk.expected_recall(64, 32, 1) == -1.0 and atk.expected_recall(4, 64, 8) == -1.0


def test_worst_case_recall_is_eq2(lib):
    """The library's Eq. 2 against the oracle's writing of it, on every legal (k, b, k_b) of small rows and on the
    benchmark configurations; and against a row built to be the worst case, run through the oracle itself."""
    import numpy as np

    import oracle
    from oracle import recall

    for n in (12, 16, 60, 64):
        for b in [d for d in range(1, n + 1) if n % d == 0]:
            for k_b in range(1, n // b + 1):
                for k in range(k_b, b * k_b + 1):
                    assert abs(atk.worst_case_recall(n, k, b, k_b) - min(1.0, recall.worst_case_recall(n, k, b, k_b))) < 1e-12
    for (n, k, b, k_b) in [(65536, 64, 64, 1), (65536, 64, 1024, 1), (65536, 16384, 2048, 8), (1 << 20, 1 << 18, 1 << 15, 8),
                           (8192, 512, 512, 1)]:
        assert abs(atk.worst_case_recall(n, k, b, k_b) - recall.worst_case_recall(n, k, b, k_b)) < 1e-12
    # the adversarial row: the k largest values at the indices of as few (interleaved) buckets as possible
    n, b, k_b, k = 64, 8, 2, 12
    x = np.zeros((1, n), dtype=np.float32)
    order = [j + t * b for j in range(b) for t in range(n // b)]  # bucket 0's indices, then bucket 1's, ...
    for rank, i in enumerate(order[:k]):
        x[0, i] = 100.0 - rank
    got = set(oracle.approx_topk(x, k, b, k_b)[1][0].tolist())
    true = set(oracle.exact_topk(x, k)[1][0].tolist())
    assert abs(len(got & true) / k - atk.worst_case_recall(n, k, b, k_b)) < 1e-12
    # not stated for b that does not divide n, nor for arguments the method does not allow
    assert atk.worst_case_recall(65, 8, 8, 1) == -1.0 and atk.worst_case_recall(64, 8, 4, 1) == -1.0
    assert atk.worst_case_recall(64, 8, 8, 9) == -1.0 and atk.worst_case_recall(64, 0, 8, 1) == -1.0


def test_advise(lib):
    for (m, n, k, dt) in [(128, 65536, 64, atk.ATK_F32), (128, 65536, 16384, atk.ATK_F32), (64, 128256, 256, atk.ATK_BF16),
                          (128, 2653751, 100, atk.ATK_BF16), (1, 40000, 5000, atk.ATK_BF16), (4, 4096, 64, atk.ATK_F32)]:
        last_us = 0.0
        for target in (0.3, 0.6, 0.8, 0.9, 0.95, 0.99):
            b, k_b, rec, us, reached = atk.advise(m, n, k, dt, target)
            assert lib.atk_check_approx(m, n, k, b, k_b, dt) == 0
            assert abs(rec - atk.expected_recall(k, b, k_b)) < 1e-12
            assert abs(us - atk.estimate_us(m, n, k, b, k_b, dt)) < 1e-9 and us > 0
            if reached:
                assert rec >= target
                assert us >= last_us - 1e-9  # a higher target never gets cheaper
                last_us = us
    # the cheapest setting: one bucket per output, no Stage 2
    b, k_b, rec, us, reached = atk.advise(128, 65536, 64, atk.ATK_F32, 0.5)
    assert (b, k_b, reached) == (64, 1, True)
    # k = n/4: within b*k_b = k only larger k_b raises recall, and 0.99 is out of its reach; more candidates than a
    # workgroup holds (Stage 1 into scratch, then the exact selection over the pairs) get there
    b, k_b, rec, us, reached = atk.advise(128, 65536, 16384, atk.ATK_F32, 0.99)
    assert reached and rec >= 0.99 and b * k_b > lib.atk_stage2_max_candidates()
    b, k_b, rec, us, reached = atk.advise(128, 65536, 16384, atk.ATK_F32, 0.9)
    assert reached and b * k_b == 16384 and k_b == 16
    i64 = ctypes.c_int64
    bb, kk = i64(0), i64(0)
    assert lib.atk_advise(128, 65536, 64, 0, 1.5, ctypes.byref(bb), ctypes.byref(kk), None, None) == PARAMS
    assert lib.atk_advise(128, 65536, 64, 0, 0.9, None, ctypes.byref(kk), None, None) == NULLP
    assert lib.atk_advise(128, 65536, 0, 0, 0.9, ctypes.byref(bb), ctypes.byref(kk), None, None) == SHAPE


def test_missing_library_fails_loudly(monkeypatch):
    """No CPU fallback: without the built library the binding raises on first use."""
    from paper_2412_04358_amd import binding

    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", os.path.join(ROOT, "paper_2412_04358_amd", "lib", "no_such_library.so"))
    with pytest.raises(RuntimeError, match="not built"):
        binding.load_library()
    with pytest.raises(RuntimeError, match="not built"):
        binding.plan_describe(4, 4096, 64, 64, 1)

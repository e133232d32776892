"""GPU parity of the replay loop (r3_record, r3_eval_candidate) with real candidate kernels:
Jacobi variants (the Jacobi workload), CSR SpMV launch configurations (the SpMV workload), the small
replay (the small-replay workload) and the large snapshot (the large-snapshot workload).  For kernels the GPU ran, the
oracle validates the bytes the candidate actually wrote (downloaded live memory)."""
import ctypes

import numpy as np
import pytest

import r3_inputs as ri

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2604_11109_amd import binding as r3
    from paper_2604_11109_amd import workloads as wl
    assert torch.cuda.is_available(), "these tests need the GPU"
    r3.lib()
    wl.lib()
    ctx = r3.Context(0)
    yield r3, wl, ctx, torch
    ctx.close()


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.cpu().numpy()


def assert_results_equal(got, exp, what=""):
    for name in exp.dtype.names:
        g = got[name].view(np.uint64) if got[name].dtype.kind == "f" else got[name]
        e = exp[name].view(np.uint64) if exp[name].dtype.kind == "f" else exp[name]
        bad = np.flatnonzero(g != e)
        assert bad.size == 0, "%s field %s differs at %s: got %s expected %s" % (
            what, name, bad[:5], got[name][bad[:5]], exp[name][bad[:5]])


def check_eval_against_oracle(r3, oracle, out, d_regions, check_rows, live_host, epi_host, what):
    exp_res, exp_sum = oracle.compare(oracle.make_table(check_rows), live_host, epi_host)
    got = r3.results_to_numpy(d_regions, len(check_rows))
    assert_results_equal(got, exp_res, what)
    s = exp_sum[0]
    assert out.total_mismatch == int(s["total_mismatch"]), what
    assert out.first_region == int(s["first_region"]) and out.first_index == int(s["first_index"]), what
    assert out.passed == int(s["pass"]), what
    assert np.float64(out.max_abs_err).tobytes() == s["max_abs_err"].tobytes(), what
    assert np.float64(out.max_rel_err).tobytes() == s["max_rel_err"].tobytes(), what
    return got


# ----------------------------------------------------------------------------------------
# the Jacobi workload: Jacobi variants
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("n", [40, 256])
def test_jacobi_record_and_eval(env, oracle, n):
    r3, wl, ctx, torch = env
    c = ri.jacobi(n)
    print("case jacobi", n, c["arena_bytes"], flush=True)
    A = c["arena_bytes"]
    tbl = r3.Table(ctx, c["restore_rows"], A)
    d_live = dev(torch, c["prologue"])
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    nw = r3.bitmap_words(A, 4096)
    d_bm = torch.zeros(nw, dtype=torch.int64, device="cuda:0")
    d_cnt = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    d_pcs = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    d_ecs = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    base = wl.jacobi_args(c, 64, 1, 0)
    r3.r3_record(ctx, tbl, d_live, wl.jacobi_launch(), base, d_pro, d_epi, 4096, d_bm, d_cnt, d_pcs, d_ecs)

    # the recorded states: prologue is the input state, epilogue is one sweep of it
    assert (host(d_pro) == c["prologue"]).all()
    epi = host(d_epi)
    grid = c["prologue"][c["in_off"]:c["in_off"] + c["grid_bytes"]].view("<f8").reshape(n, n, n)
    ref = ri.jacobi_reference(grid)
    got_out = epi[c["out_off"]:c["out_off"] + c["grid_bytes"]].view("<f8").reshape(n, n, n)
    assert np.allclose(got_out, ref, rtol=1e-12, atol=0)
    assert (epi[:c["grid_bytes"]] == c["prologue"][:c["grid_bytes"]]).all()
    # the oracle's record of the same two states
    otbl = oracle.make_table(c["restore_rows"])
    exp_bm, exp_cnt = oracle.dirty_diff(c["prologue"], epi, 4096)
    assert (host(d_bm).view(np.uint64) == exp_bm).all() and int(host(d_cnt)[0]) == exp_cnt
    assert (host(d_pcs).view(np.uint64) == oracle.checksum(otbl, c["prologue"])).all()
    assert (host(d_ecs).view(np.uint64) == oracle.checksum(otbl, epi)).all()
    # the write-set is the pages of `out` that hold an interior point
    pages = np.flatnonzero(np.unpackbits(exp_bm.view(np.uint8), bitorder="little"))
    assert pages.min() >= c["out_off"] // 4096 and exp_cnt > 0

    d_regions = torch.zeros(40 * 2, dtype=torch.uint8, device="cuda:0")
    for block, unroll, bug in ri.JACOBI_VARIANTS:
        args = wl.jacobi_args(c, block, unroll, bug)
        d_live.fill_(0x5A)     # the replay must not depend on what the last candidate left
        rc, out = r3.r3_eval_candidate(ctx, tbl, d_pro, tbl, d_epi, d_live, wl.jacobi_launch(), args,
                                       1, 2, r3.EVERY, d_regions)
        what = "variant block=%d unroll=%d bug=%d" % (block, unroll, bug)
        print(what, "ms", out.ms_median, "mismatch", out.total_mismatch, flush=True)
        assert rc == r3.OK and out.candidate_status == 0
        got = check_eval_against_oracle(r3, oracle, out, d_regions, c["check_rows"], host(d_live), epi, what)
        assert out.ms_min > 0 and out.ms_min <= out.ms_median <= out.ms_max
        if not bug:
            assert out.passed == 1
        else:
            # closed form: the column x = n-2 of every interior (y, z) is stale
            assert out.passed == 0 and out.total_mismatch == (n - 2) ** 2
            assert out.first_region == 1 and out.first_index == (1 * n + 1) * n + (n - 2)
            assert out.max_rel_err == 1.0
            assert int(got[0]["mismatch_count"]) == 0


# ----------------------------------------------------------------------------------------
# the SpMV workload: CSR SpMV launch configurations, write-set from the dirty-diff
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("rows", [1 << 15, 1 << 21])
def test_spmv_record_and_sweep(env, oracle, rows):
    r3, wl, ctx, torch = env
    c = ri.spmv(rows)
    print("case spmv", rows, c["arena_bytes"], flush=True)
    A = c["arena_bytes"]
    full = r3.Table(ctx, c["table_rows"], A)
    ytbl = r3.Table(ctx, c["y_rows"], A)
    d_live = dev(torch, c["prologue"])
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    nw = r3.bitmap_words(A, 4096)
    d_bm = torch.zeros(nw, dtype=torch.int64, device="cuda:0")
    d_cnt = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    d_pcs = torch.zeros(5, dtype=torch.int64, device="cuda:0")
    d_ecs = torch.zeros(5, dtype=torch.int64, device="cuda:0")
    r3.r3_record(ctx, full, d_live, wl.spmv_launch(), wl.spmv_args(c, 64, 256), d_pro, d_epi, 4096,
                 d_bm, d_cnt, d_pcs, d_ecs)
    y_off, y_bytes = c["offsets"]["y"], c["sizes"]["y"]
    epi_y = host(d_epi[y_off:y_off + y_bytes])
    # sanity of the recorded product against a host CSR product (not a parity claim)
    row_ptr, col, vals, x = c["csr"]
    ref = (vals.reshape(rows, 27) * x[col]).sum(axis=1)
    bound = 1e-12 * (np.abs(vals.reshape(rows, 27)) * np.abs(x[col])).sum(axis=1)
    assert (np.abs(epi_y.view("<f8") - ref) <= bound).all()
    # write-set: exactly the pages of y
    bm = host(d_bm).view(np.uint64)
    pages = np.flatnonzero(np.unpackbits(bm.view(np.uint8), bitorder="little"))
    assert (pages == np.arange(y_off // 4096, (y_off + y_bytes + 4095) // 4096)).all()
    assert int(host(d_cnt)[0]) == pages.size == (4096 if rows == 1 << 21 else pages.size)
    # prologue checksums: recorded state equals the generated state, region by region
    assert (host(d_pcs).view(np.uint64) == oracle.checksum(oracle.make_table(c["table_rows"]), c["prologue"])).all()
    ecs = host(d_ecs).view(np.uint64)
    assert (ecs[:4] == host(d_pcs).view(np.uint64)[:4]).all() and ecs[4] != host(d_pcs).view(np.uint64)[4]

    d_regions = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    epi_arena = np.zeros(A, dtype=np.uint8)
    epi_arena[y_off:y_off + y_bytes] = epi_y
    live_arena = np.zeros(A, dtype=np.uint8)
    variants = ri.SPMV_VARIANTS if rows == 1 << 21 else ri.SPMV_VARIANTS[::3]
    flagged = 0
    for i, (rpw, block) in enumerate(variants):
        args = wl.spmv_args(c, rpw, block)
        # alternate between restoring the whole arena and only the recorded write-set
        rtbl = full if i % 2 == 0 else ytbl
        rc, out = r3.r3_eval_candidate(ctx, rtbl, d_pro, ytbl, d_epi, d_live, wl.spmv_launch(), args,
                                       0, 2, r3.LAST, d_regions)
        what = "spmv rows_per_wave=%d block=%d" % (rpw, block)
        assert rc == r3.OK, what
        live_arena[y_off:y_off + y_bytes] = host(d_live[y_off:y_off + y_bytes])
        check_eval_against_oracle(r3, oracle, out, d_regions, c["y_rows"], live_arena, epi_arena, what)
        if rpw >= 64:
            assert out.passed == 1, what           # same summation order as the recording
        flagged += int(out.total_mismatch > 0)
        if i % 16 == 0:
            print(what, "ms", out.ms_median, "mismatch", out.total_mismatch, flush=True)
    print("configurations flagged under rtol 1e-12, atol 0:", flagged, "of", len(variants), flush=True)


# ----------------------------------------------------------------------------------------
# the small-replay workload: ten pure restore -> validate replays
# ----------------------------------------------------------------------------------------
def test_replay_small_ten_replays(env, oracle):
    r3, wl, ctx, torch = env
    c = ri.replay_small()
    A = c["arena_bytes"]
    rt, ct = r3.Table(ctx, c["restore_rows"], A), r3.Table(ctx, c["check_rows"], A)
    d_pro, d_epi, d_live = dev(torch, c["prologue"]), dev(torch, c["epilogue"]), dev(torch, c["live"])
    d_regions = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    rc, out = r3.r3_eval_candidate(ctx, rt, d_pro, ct, d_epi, d_live, None, None, 0, 10, r3.EVERY, d_regions)
    assert rc == r3.OK
    live = c["live"].copy()
    exp = oracle.eval_candidate(oracle.make_table(c["restore_rows"]), c["prologue"],
                                oracle.make_table(c["check_rows"]), c["epilogue"], live, None, 0, 10)
    assert_results_equal(r3.results_to_numpy(d_regions, 1), exp["regions"])
    assert out.total_mismatch == exp["total_mismatch"] == 1049
    assert out.first_index == exp["first_index"] == int(c["planted"][0]) and out.passed == 0
    assert (host(d_live) == live).all()
    # the restored inputs carry the recorded checksums
    d_cs = torch.zeros(3, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, rt, d_live, d_cs)
    torch.cuda.synchronize()
    assert (host(d_cs).view(np.uint64) == oracle.checksum(oracle.make_table(c["restore_rows"]), c["prologue"])).all()


# ----------------------------------------------------------------------------------------
# the replay loop itself: policies, flaky and failing candidates
# ----------------------------------------------------------------------------------------
def test_eval_policies_and_failures(env, oracle):
    r3, wl, ctx, torch = env
    rng = np.random.default_rng(51)
    n = 1 << 16
    pro = rng.integers(0, 256, size=n, dtype=np.uint8)
    half = n // 2
    epi = pro.copy()
    epi[half:] = pro[:half] + 1
    rrows = [(0, n, ri.U8, ri.BITWISE, 0, 0)]
    crows = [(0, half, ri.U8, ri.BITWISE, 0, 0), (half, half, ri.U8, ri.BITWISE, 0, 0)]
    rt, ct = r3.Table(ctx, rrows, n), r3.Table(ctx, crows, n)
    d_pro, d_epi = dev(torch, pro), dev(torch, epi)
    d_live = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    d_regions = torch.zeros(80, dtype=torch.uint8, device="cuda:0")
    state = {"k": 0, "bad_at": None, "where": [40000, 50000]}

    def gpu_candidate(live_ptr, stream):
        d_live[half:] = d_live[:half] + 1
        if state["k"] == state["bad_at"]:
            for w in state["where"]:
                d_live[w] ^= 1
        state["k"] += 1
        return 0

    def cpu_candidate(live):
        live[half:] = live[:half] + 1
        if state["k"] == state["bad_at"]:
            for w in state["where"]:
                live[w] ^= 1
        state["k"] += 1
        return 0

    for policy in (r3.EVERY, r3.FIRST, r3.LAST):
        for bad_at in (None, 0, 1, 3):
            for warmup, reps in ((0, 4), (2, 2)):
                state.update(k=0, bad_at=bad_at)
                rc, out = r3.r3_eval_candidate(ctx, rt, d_pro, ct, d_epi, d_live, gpu_candidate, None,
                                               warmup, reps, policy, d_regions)
                state.update(k=0)
                live = np.zeros(n, np.uint8)
                exp = oracle.eval_candidate(oracle.make_table(rrows), pro, oracle.make_table(crows), epi,
                                            live, cpu_candidate, warmup, reps, policy)
                what = "policy %d bad_at %s warmup %d" % (policy, bad_at, warmup)
                assert rc == r3.OK, what
                assert_results_equal(r3.results_to_numpy(d_regions, 2), exp["regions"], what)
                assert (out.total_mismatch, out.passed) == (exp["total_mismatch"], exp["pass"]), what
                assert (out.first_region, out.first_index) == (exp["first_region"], exp["first_index"]), what
                assert (host(d_live) == live).all(), what

    # a candidate that cannot be launched is rejected, whatever ran before
    code = ctypes.c_int(5)
    rc, out = r3.r3_eval_candidate(ctx, rt, d_pro, ct, d_epi, d_live, wl.failing_launch(),
                                   ctypes.addressof(code), 0, 3, r3.EVERY, d_regions)
    assert rc == r3.ECANDIDATE and out.passed == 0 and out.candidate_status == 5
    exp = oracle.eval_candidate(oracle.make_table(rrows), pro, oracle.make_table(crows), epi,
                                np.zeros(n, np.uint8), lambda l: 5, 0, 3)
    assert exp["pass"] == 0 and exp["candidate_status"] == 5
    with pytest.raises(r3.R3Error):
        r3.r3_eval_candidate(ctx, rt, d_pro, ct, d_epi, d_live, wl.failing_launch(), None, 0, 3, r3.EVERY,
                             d_regions, raise_on_candidate=True)
    # argument checks
    for warmup, reps, policy, status in ((0, 0, 0, r3.EINVAL), (1000, 100, 0, r3.ENOSPC), (0, 1, 9, r3.EINVAL)):
        with pytest.raises(r3.R3Error) as e:
            r3.r3_eval_candidate(ctx, rt, d_pro, ct, d_epi, d_live, None, None, warmup, reps, policy, d_regions)
        assert e.value.status == status
    # the library still works after the rejections
    rc, out = r3.r3_eval_candidate(ctx, rt, d_pro, rt, d_pro, d_live, None, None, 0, 1, r3.EVERY, d_regions)
    assert rc == r3.OK and out.passed == 1


# ----------------------------------------------------------------------------------------
# the large-snapshot workload: 16 x 2 GiB, full size
# ----------------------------------------------------------------------------------------
@pytest.mark.timeout(900)
def test_large_snapshot_full_size(env, oracle):
    r3, wl, ctx, torch = env
    free, total = torch.cuda.mem_get_info()
    if free < 110 * (1 << 30):
        pytest.skip("needs 96 GiB of device memory for snapshot, live and golden arenas")
    c = ri.large_snapshot_device()
    A = c["arena_bytes"]
    print("case large_snapshot", A, flush=True)
    tbl = r3.Table(ctx, c["rows"], A)
    d_live = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_regions = torch.zeros(40 * 16, dtype=torch.uint8, device="cuda:0")
    rc, out = r3.r3_eval_candidate(ctx, tbl, c["snapshot"], tbl, c["golden"], d_live, None, None, 0, 1,
                                   r3.EVERY, d_regions)
    assert rc == r3.OK
    got = r3.results_to_numpy(d_regions, 16)
    d_cs = torch.zeros(16, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, tbl, c["snapshot"], d_cs)
    torch.cuda.synchronize()
    # properties that hold for every region: planted counts and first indices, and the
    # checksum of the restored bytes equals the checksum of the snapshot
    for r, idx in enumerate(c["planted"]):
        assert int(got[r]["mismatch_count"]) == len(idx), r
        assert int(got[r]["first_mismatch"]) == int(idx[0]), r
    assert (got["checksum"] == host(d_cs).view(np.uint64)).all()
    assert out.total_mismatch == sum(len(i) for i in c["planted"]) == 8 * 537 + 8 * 1074
    assert out.first_region == 0 and out.passed == 0
    # element by element: the oracle on every one of the 16 regions (2 GiB each, downloaded one at a
    # time; a few host threads work on different regions, each running the plain single-thread oracle)
    import concurrent.futures as cf

    def one_region(r):
        off, nb = c["rows"][r][0], c["rows"][r][1]
        live_h = host(d_live[off:off + nb])
        gold_h = host(c["golden"][off:off + nb])
        row = [(0, nb) + tuple(c["rows"][r][2:])]
        exp, _ = oracle.compare(oracle.make_table(row), live_h, gold_h)
        return r, exp
    exp_all = np.zeros(16, dtype=oracle.RESULT_DTYPE)
    with cf.ThreadPoolExecutor(max_workers=4) as pool:
        for r, exp in pool.map(one_region, range(16)):
            assert_results_equal(got[r:r + 1], exp, "region %d" % r)
            exp_all[r] = exp[0]
            print("region", r, "oracle parity ok", flush=True)
    s = oracle.summarize(exp_all)[0]
    assert out.total_mismatch == int(s["total_mismatch"])
    assert out.first_region == int(s["first_region"]) and out.first_index == int(s["first_index"])
    assert out.passed == int(s["pass"]) == 0
    assert np.float64(out.max_abs_err).tobytes() == s["max_abs_err"].tobytes()
    assert np.float64(out.max_rel_err).tobytes() == s["max_rel_err"].tobytes()


def test_most_replays_one_evaluation_takes(env, oracle):
    """R3_MAX_REPLAYS replays in one evaluation, validated after each: the verdict is the worst
    replay's count, the region results are the last replay's."""
    r3, wl, ctx, torch = env
    rng = np.random.default_rng(99)
    n = 1 << 14
    pro = rng.integers(0, 256, size=n, dtype=np.uint8)
    epi = (pro + 1).astype(np.uint8)
    rows = [(0, n, ri.U8, ri.BITWISE, 0, 0)]
    t = r3.Table(ctx, rows, n)
    d_pro, d_epi = dev(torch, pro), dev(torch, epi)
    d_live = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    d_regions = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    total = 1024
    state = {"k": 0}

    def gpu_candidate(live_ptr, stream):
        d_live.add_(1)
        if state["k"] == 700:
            d_live[5:9] = 0
        if state["k"] == total - 1:
            d_live[100] ^= 0xFF
        state["k"] += 1
        return 0

    def cpu_candidate(live):
        live += 1
        if state["k"] == 700:
            live[5:9] = 0
        if state["k"] == total - 1:
            live[100] ^= 0xFF
        state["k"] += 1
        return 0
    rc, out = r3.r3_eval_candidate(ctx, t, d_pro, t, d_epi, d_live, gpu_candidate, None, 24, total - 24,
                                   r3.EVERY, d_regions)
    state["k"] = 0
    live = np.zeros(n, np.uint8)
    exp = oracle.eval_candidate(oracle.make_table(rows), pro, oracle.make_table(rows), epi, live, cpu_candidate,
                                24, total - 24, oracle.EVERY)
    assert rc == r3.OK and state["k"] == total
    assert_results_equal(r3.results_to_numpy(d_regions, 1), exp["regions"], "last replay")
    assert (out.total_mismatch, out.passed, out.first_index) == (exp["total_mismatch"], 0, exp["first_index"])
    assert out.total_mismatch >= 1 and int(exp["regions"][0]["mismatch_count"]) == 1
    assert (host(d_live) == live).all()
    times = ctx.last_times()
    assert len(times) == total - 24 and min(times) > 0

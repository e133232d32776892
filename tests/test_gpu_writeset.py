"""GPU parity of write-set driven replay: regions from the recorded dirty bitmap, restore of
the write-set only, and the whole-state guard that catches a candidate writing elsewhere."""
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


@pytest.mark.parametrize("rows", [1 << 15, 1 << 21])
def test_spmv_writeset_replay_and_guard(env, oracle, rows):
    r3, wl, ctx, torch = env
    c = ri.spmv(rows)
    A = c["arena_bytes"]
    print("case spmv write-set", rows, A, flush=True)
    full = r3.Table(ctx, c["table_rows"], A)
    ytbl = r3.Table(ctx, c["y_rows"], A)
    d_live = dev(torch, c["prologue"])
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    nw = r3.bitmap_words(A, 4096)
    d_bm = torch.zeros(nw, dtype=torch.int64, device="cuda:0")
    base_args = wl.spmv_args(c, 64, 256)
    r3.r3_record(ctx, full, d_live, wl.spmv_launch(), base_args, d_pro, d_epi, 4096, d_bm)
    bm = host(d_bm).view(np.uint64)

    # regions from the bitmap: library == oracle, dirty part == the y array
    dirty = r3.r3_writeset_regions(bm, A, 4096, 1)
    clean = r3.r3_writeset_regions(bm, A, 4096, 0)
    assert dirty.tobytes() == oracle.writeset_regions(bm, A, 4096, 1).tobytes()
    assert clean.tobytes() == oracle.writeset_regions(bm, A, 4096, 0).tobytes()
    y_off, y_bytes = c["offsets"]["y"], c["sizes"]["y"]
    assert [(int(r["offset"]), int(r["bytes"])) for r in dirty] == [(y_off, (y_bytes + 4095) // 4096 * 4096)]
    ws_tbl = r3.Table(ctx, dirty, A)
    guard_tbl = r3.Table(ctx, clean, A)
    d_expected = torch.zeros(guard_tbl.n, dtype=torch.int64, device="cuda:0")
    d_scratch = torch.zeros(guard_tbl.n, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, guard_tbl, d_pro, d_expected)
    torch.cuda.synchronize()
    pro_h, epi_h = host(d_pro), host(d_epi)
    assert (pro_h == c["prologue"]).all()
    exp_cs = oracle.checksum(oracle.make_table(clean), pro_h)
    assert (host(d_expected).view(np.uint64) == exp_cs).all()

    d_regions = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    epi_y = epi_h[y_off:y_off + y_bytes].copy()

    # (1) a well-behaved candidate: write-set restore only, guard after every 2nd replay
    d_live.copy_(d_pro)
    rc, out, g = r3.r3_eval_candidate_guarded(ctx, ws_tbl, d_pro, ytbl, d_epi, d_live, wl.spmv_launch(),
                                              wl.spmv_args(c, 128, 512), 1, 4, r3.EVERY, d_regions,
                                              guard_tbl, d_expected, d_scratch, every=2, heal_tbl=full)
    live_h = pro_h.copy()

    def cpu_good(live):
        live[y_off:y_off + y_bytes] = epi_y      # same summation order as the recording
        return 0
    exp = oracle.eval_candidate(oracle.make_table(dirty), pro_h, oracle.make_table(c["y_rows"]), epi_h, live_h,
                                cpu_good, 1, 4, oracle.EVERY, guard_tbl=oracle.make_table(clean),
                                guard_expected=exp_cs, guard_every=2, heal_tbl=oracle.make_table(c["table_rows"]))
    assert rc == r3.OK and out.passed == exp["pass"] == 1
    assert (g.checks, g.failed_checks, g.changed_regions, g.first_region, g.healed) == (
        exp["guard"]["checks"], 0, 0, r3.NO_REGION, 0) == (3, 0, 0, r3.NO_REGION, 0)
    assert r3.results_to_numpy(d_regions, 1).tobytes() == exp["regions"].tobytes()
    assert (host(d_live) == live_h).all()

    # (2) a candidate that also writes a byte outside every array (the padding after row_ptr,
    # so that the product itself is unaffected) on its second and later replays
    x_off = c["offsets"]["row_ptr"] + 4 * (rows + 1) + 16 - 8 * 1000
    whole = r3.Table(ctx, [(0, A, ri.U8, ri.BITWISE, 0, 0)], A)
    whole_rows = [(0, A, ri.U8, ri.BITWISE, 0, 0)]
    state = {"k": 0}
    good_args = wl.spmv_args(c, 64, 128)
    launch = wl.lib().r3w_spmv_launch
    launch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]

    def gpu_stray(live_ptr, stream):
        rc = launch(ctypes.addressof(good_args), live_ptr, stream)
        if state["k"] >= 1:
            d_live[x_off + 8 * 1000] = 0x7F
        state["k"] += 1
        return rc

    def cpu_stray(live):
        live[y_off:y_off + y_bytes] = epi_y
        if state["k"] >= 1:
            live[x_off + 8 * 1000] = 0x7F
        state["k"] += 1
        return 0
    assert pro_h[x_off + 8 * 1000] != 0x7F
    for heal in (True, False):
        state["k"] = 0
        d_live.copy_(d_pro)
        rc, out, g = r3.r3_eval_candidate_guarded(ctx, ws_tbl, d_pro, ytbl, d_epi, d_live, gpu_stray, None,
                                                  0, 3, r3.EVERY, d_regions, guard_tbl, d_expected, d_scratch,
                                                  every=1, heal_tbl=whole if heal else None)
        state["k"] = 0
        live_h = pro_h.copy()
        exp = oracle.eval_candidate(oracle.make_table(dirty), pro_h, oracle.make_table(c["y_rows"]), epi_h,
                                    live_h, cpu_stray, 0, 3, oracle.EVERY, guard_tbl=oracle.make_table(clean),
                                    guard_expected=exp_cs, guard_every=1,
                                    heal_tbl=oracle.make_table(whole_rows) if heal else None)
        eg = exp["guard"]
        assert rc == r3.OK and out.total_mismatch == exp["total_mismatch"] == 0
        assert out.passed == exp["pass"] == 0
        assert (g.checks, g.failed_checks, g.changed_regions, g.first_region, g.healed) == (
            eg["checks"], eg["failed_checks"], eg["changed_regions"], eg["first_region"], eg["healed"])
        assert g.failed_checks == 2 and g.healed == int(heal)
        got_live = host(d_live)
        bad = np.flatnonzero(got_live != live_h)
        assert bad.size == 0, (heal, bad[:5], got_live[bad[:5]], live_h[bad[:5]], x_off, y_off)
        if heal:
            assert (got_live == pro_h).all()

    # argument checks of the guarded call
    with pytest.raises(r3.R3Error) as e:
        r3.r3_eval_candidate_guarded(ctx, ws_tbl, d_pro, ytbl, d_epi, d_live, None, None, 0, 1, r3.EVERY,
                                     d_regions, guard_tbl, 0, d_scratch)
    assert e.value.status == r3.EINVAL


def test_jacobi_writeset_is_the_interior_of_out(env, oracle):
    r3, wl, ctx, torch = env
    n = 64
    c = ri.jacobi(n)
    A = c["arena_bytes"]
    full = r3.Table(ctx, c["restore_rows"], A)
    d_live = dev(torch, c["prologue"])
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_bm = torch.zeros(r3.bitmap_words(A, 4096), dtype=torch.int64, device="cuda:0")
    r3.r3_record(ctx, full, d_live, wl.jacobi_launch(), wl.jacobi_args(c, 256, 1, 0), d_pro, d_epi, 4096, d_bm)
    bm = host(d_bm).view(np.uint64)
    exp_bm, _ = oracle.dirty_diff(host(d_pro), host(d_epi), 4096)
    assert (bm == exp_bm).all()
    dirty = r3.r3_writeset_regions(bm, A, 4096, 1)
    clean = r3.r3_writeset_regions(bm, A, 4096, 0)
    assert int(dirty["offset"].min()) >= c["out_off"] // 4096 * 4096
    assert int(clean["bytes"].sum()) + int(dirty["bytes"].sum()) == A
    ws_tbl, guard_tbl = r3.Table(ctx, dirty, A), r3.Table(ctx, clean, A)
    check = r3.Table(ctx, [c["check_rows"][1]], A)
    d_expected = torch.zeros(guard_tbl.n, dtype=torch.int64, device="cuda:0")
    d_scratch = torch.zeros(guard_tbl.n, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, guard_tbl, d_pro, d_expected)
    d_regions = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    d_live.copy_(d_pro)
    for block, unroll, bug in ri.JACOBI_VARIANTS:
        rc, out, g = r3.r3_eval_candidate_guarded(ctx, ws_tbl, d_pro, check, d_epi, d_live, wl.jacobi_launch(),
                                                  wl.jacobi_args(c, block, unroll, bug), 0, 2, r3.EVERY,
                                                  d_regions, guard_tbl, d_expected, d_scratch, every=0)
        assert rc == r3.OK and g.checks == 1 and g.failed_checks == 0
        assert out.passed == int(not bug)
        exp, _ = oracle.compare(oracle.make_table([c["check_rows"][1]]), host(d_live), host(d_epi))
        assert r3.results_to_numpy(d_regions, 1).tobytes() == exp.tobytes()


def test_guarded_evaluations_in_flight(env, oracle):
    """r3_eval_submit_guarded: write-set replays of all Jacobi variants in flight together give the
    verdicts of the one-at-a-time calls; a candidate that writes outside the write-set fails its
    guard, so does the evaluation queued behind it, and after the heal that one passes."""
    r3, wl, ctx, torch = env
    n = 64
    c = ri.jacobi(n)
    A = c["arena_bytes"]
    full = r3.Table(ctx, c["restore_rows"], A)
    d_live = dev(torch, c["prologue"])
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_bm = torch.zeros(r3.bitmap_words(A, 4096), dtype=torch.int64, device="cuda:0")
    r3.r3_record(ctx, full, d_live, wl.jacobi_launch(), wl.jacobi_args(c, 256, 1, 0), d_pro, d_epi, 4096, d_bm)
    bm = host(d_bm).view(np.uint64)
    dirty = r3.r3_writeset_regions(bm, A, 4096, 1)
    clean = r3.r3_writeset_regions(bm, A, 4096, 0)
    ws_tbl, guard_tbl = r3.Table(ctx, dirty, A), r3.Table(ctx, clean, A)
    check_rows = [c["check_rows"][1]]
    check = r3.Table(ctx, check_rows, A)
    d_expected = torch.zeros(guard_tbl.n, dtype=torch.int64, device="cuda:0")
    d_scratch = torch.zeros(guard_tbl.n, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, guard_tbl, d_pro, d_expected)
    torch.cuda.synchronize()
    pro_h, epi_h = host(d_pro), host(d_epi)
    exp_cs = oracle.checksum(oracle.make_table(clean), pro_h)
    bufs = [torch.zeros(40, dtype=torch.uint8, device="cuda:0") for _ in range(8)]

    # every variant, one at a time, against the oracle on the bytes it left
    d_live.copy_(d_pro)
    alone = []
    for block, unroll, bug in ri.JACOBI_VARIANTS:
        rc, out, g = r3.r3_eval_candidate_guarded(ctx, ws_tbl, d_pro, check, d_epi, d_live, wl.jacobi_launch(),
                                                  wl.jacobi_args(c, block, unroll, bug), 0, 2, r3.EVERY,
                                                  bufs[0], guard_tbl, d_expected, d_scratch, every=1)
        exp, _ = oracle.compare(oracle.make_table(check_rows), host(d_live), epi_h)
        assert r3.results_to_numpy(bufs[0], 1).tobytes() == exp.tobytes()
        assert (g.checks, g.failed_checks) == (2, 0)
        alone.append((exp, out))
    # the same eight, all in flight
    args = [wl.jacobi_args(c, block, unroll, bug) for block, unroll, bug in ri.JACOBI_VARIANTS]
    tickets = [r3.r3_eval_submit_guarded(ctx, ws_tbl, d_pro, check, d_epi, d_live, wl.jacobi_launch(), a,
                                         0, 2, r3.EVERY, bufs[i], guard_tbl, d_expected, d_scratch, every=1)
               for i, a in enumerate(args)]
    for i in reversed(range(8)):
        rc, out, g = r3.r3_eval_wait(ctx, tickets[i], with_guard=True)
        exp, exp_out = alone[i]
        assert rc == r3.OK and (g.checks, g.failed_checks, g.healed) == (2, 0, 0)
        assert r3.results_to_numpy(bufs[i], 1).tobytes() == exp.tobytes()
        for f in ("total_mismatch", "first_region", "first_index", "passed", "max_abs_err", "max_rel_err"):
            assert getattr(out, f) == getattr(exp_out, f), (i, f)

    # a stray write outside the write-set (last byte of the `in` grid), then a good candidate behind it
    stray_at = c["in_off"] + c["grid_bytes"] - 1
    good = wl.jacobi_args(c, 128, 1, 0)
    launch = wl.lib().r3w_jacobi_launch
    launch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    stray_value = int(pro_h[stray_at]) ^ 0x55

    def gpu_stray(live_ptr, stream):
        rc = launch(ctypes.addressof(good), live_ptr, stream)
        d_live[stray_at] = stray_value
        return rc
    out_off, gb = c["out_off"], c["grid_bytes"]
    # what a correct sweep leaves in `out`
    rc, out, g = r3.r3_eval_candidate_guarded(ctx, ws_tbl, d_pro, check, d_epi, d_live, wl.jacobi_launch(), good,
                                              0, 1, r3.EVERY, bufs[0], guard_tbl, d_expected, d_scratch, every=0)
    assert out.passed == 1
    good_out = host(d_live)[out_off:out_off + gb].copy()

    def cpu_stray(live):
        live[out_off:out_off + gb] = good_out
        live[stray_at] = stray_value
        return 0

    def cpu_good(live):
        live[out_off:out_off + gb] = good_out
        return 0
    t_a = r3.r3_eval_submit_guarded(ctx, ws_tbl, d_pro, check, d_epi, d_live, gpu_stray, None, 0, 1, r3.EVERY,
                                    bufs[0], guard_tbl, d_expected, d_scratch, every=0, heal_tbl=full)
    t_b = r3.r3_eval_submit_guarded(ctx, ws_tbl, d_pro, check, d_epi, d_live, wl.jacobi_launch(), good, 0, 1,
                                    r3.EVERY, bufs[1], guard_tbl, d_expected, d_scratch, every=0, heal_tbl=full)
    rc_a, out_a, g_a = r3.r3_eval_wait(ctx, t_a, with_guard=True)
    rc_b, out_b, g_b = r3.r3_eval_wait(ctx, t_b, with_guard=True)
    # the oracle's account of the same sequence: A and B run before any heal, then the heal
    otab = dict(guard_tbl=oracle.make_table(clean), guard_expected=exp_cs, guard_every=0)
    live_h = pro_h.copy()
    exp_a = oracle.eval_candidate(oracle.make_table(dirty), pro_h, oracle.make_table(check_rows), epi_h, live_h,
                                  cpu_stray, 0, 1, oracle.EVERY, heal_tbl=None, **otab)
    exp_b = oracle.eval_candidate(oracle.make_table(dirty), pro_h, oracle.make_table(check_rows), epi_h, live_h,
                                  cpu_good, 0, 1, oracle.EVERY, heal_tbl=None, **otab)
    for (rc, out, g), exp in (((rc_a, out_a, g_a), exp_a), ((rc_b, out_b, g_b), exp_b)):
        assert rc == r3.OK and out.total_mismatch == exp["total_mismatch"] == 0
        assert out.passed == exp["pass"] == 0
        assert (g.checks, g.failed_checks, g.changed_regions, g.first_region) == (
            exp["guard"]["checks"], exp["guard"]["failed_checks"], exp["guard"]["changed_regions"],
            exp["guard"]["first_region"])
        assert g.failed_checks == 1 and g.healed == 1
    # healed: live memory is the recorded prologue again, and B passes when submitted again
    oracle.restore(oracle.make_table(c["restore_rows"]), pro_h, live_h)
    assert (host(d_live) == live_h).all()
    t_b = r3.r3_eval_submit_guarded(ctx, ws_tbl, d_pro, check, d_epi, d_live, wl.jacobi_launch(), good, 0, 1,
                                    r3.EVERY, bufs[1], guard_tbl, d_expected, d_scratch, every=0, heal_tbl=full)
    rc_b, out_b, g_b = r3.r3_eval_wait(ctx, t_b, with_guard=True)
    exp_b = oracle.eval_candidate(oracle.make_table(dirty), pro_h, oracle.make_table(check_rows), epi_h, live_h,
                                  cpu_good, 0, 1, oracle.EVERY, heal_tbl=None, **otab)
    assert rc_b == r3.OK and out_b.passed == exp_b["pass"] == 1 and g_b.failed_checks == 0

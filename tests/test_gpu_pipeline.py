"""GPU parity of r3_eval_submit / r3_eval_wait: several evaluations in flight on one stream must
give, ticket by ticket, what the oracle's evaluation loop gives for the same candidates."""
import ctypes

import numpy as np
import pytest

import r3_inputs as ri
from test_gpu_eval import assert_results_equal, dev, host

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


def test_submit_wait_matches_oracle(env, oracle):
    r3, wl, ctx, torch = env
    rng = np.random.default_rng(77)
    n = 1 << 18
    half = n // 2
    pro = rng.integers(0, 256, size=n, dtype=np.uint8)
    epi = pro.copy()
    epi[half:] = pro[:half] + 1
    rrows = [(0, n, ri.U8, ri.BITWISE, 0, 0)]
    crows = [(0, half, ri.U8, ri.BITWISE, 0, 0), (half, half, ri.U8, ri.BITWISE, 0, 0)]
    rt, ct = r3.Table(ctx, rrows, n), r3.Table(ctx, crows, n)
    d_pro, d_epi = dev(torch, pro), dev(torch, epi)
    d_live = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    max_inflight = 8
    d_regions = [torch.zeros(80, dtype=torch.uint8, device="cuda:0") for _ in range(max_inflight)]

    # candidate c flips the bytes wrong[c] of the output in the replay bad_at[c]
    wrong = [sorted(int(x) for x in rng.choice(n, size=1 + c % 3, replace=False)) for c in range(max_inflight)]
    bad_at = [None, 0, 1, 2, None, 3, 0, 1]
    cases = [(0, 4, r3.EVERY), (2, 2, r3.EVERY), (0, 4, r3.FIRST), (1, 3, r3.LAST),
             (0, 1, r3.EVERY), (0, 4, r3.EVERY), (0, 2, r3.LAST), (3, 1, r3.FIRST)]

    def gpu_candidate(c):
        state = {"k": 0}

        def run(live_ptr, stream):
            d_live[half:] = d_live[:half] + 1
            if state["k"] == bad_at[c]:
                for w in wrong[c]:
                    d_live[w] ^= 1
            state["k"] += 1
            return 0
        return run

    def cpu_candidate(c):
        state = {"k": 0}

        def run(live):
            live[half:] = live[:half] + 1
            if state["k"] == bad_at[c]:
                for w in wrong[c]:
                    live[w] ^= 1
            state["k"] += 1
            return 0
        return run

    expected = []
    live = np.zeros(n, np.uint8)
    for c, (warmup, reps, policy) in enumerate(cases):
        expected.append(oracle.eval_candidate(oracle.make_table(rrows), pro, oracle.make_table(crows), epi,
                                              live, cpu_candidate(c), warmup, reps, policy))

    for order in (list(range(max_inflight)), list(reversed(range(max_inflight))), [3, 0, 7, 1, 6, 2, 5, 4]):
        tickets = []
        for c, (warmup, reps, policy) in enumerate(cases):
            tickets.append(r3.r3_eval_submit(ctx, rt, d_pro, ct, d_epi, d_live, gpu_candidate(c), None,
                                             warmup, reps, policy, d_regions[c]))
        assert sorted(tickets) == list(range(1, max_inflight + 1))
        # no ticket left: the next submission is refused and changes nothing
        with pytest.raises(r3.R3Error) as e:
            r3.r3_eval_submit(ctx, rt, d_pro, ct, d_epi, d_live, None, None, 0, 1, r3.EVERY, d_regions[0])
        assert e.value.status == r3.ENOSPC
        for c in order:
            rc, out = r3.r3_eval_wait(ctx, tickets[c])
            exp = expected[c]
            what = "candidate %d order %s" % (c, order)
            assert rc == r3.OK, what
            assert_results_equal(r3.results_to_numpy(d_regions[c], 2), exp["regions"], what)
            assert (out.total_mismatch, out.passed) == (exp["total_mismatch"], exp["pass"]), what
            assert (out.first_region, out.first_index) == (exp["first_region"], exp["first_index"]), what
            assert out.ms_min > 0 and out.ms_min <= out.ms_median <= out.ms_max, what
            # a ticket is spent once it has been waited for
            with pytest.raises(r3.R3Error) as e:
                r3.r3_eval_wait(ctx, tickets[c])
            assert e.value.status == r3.EINVAL
        # live memory holds what the last candidate submitted left
        assert (host(d_live) == live).all()


@pytest.mark.parametrize("n", [40, 256])
def test_submit_interleaved_with_synchronous_calls(env, oracle, n):
    """A failing candidate is reported by the wait; the synchronous call works while tickets are out;
    a pipeline of depth two over the Jacobi variants gives each variant's own verdict."""
    r3, wl, ctx, torch = env
    c = ri.jacobi(n)
    print("case jacobi pipeline", n, flush=True)
    A = c["arena_bytes"]
    tbl = r3.Table(ctx, c["restore_rows"], A)
    chk = r3.Table(ctx, c["check_rows"], A)
    d_live = dev(torch, c["prologue"])
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    r3.r3_record(ctx, tbl, d_live, wl.jacobi_launch(), wl.jacobi_args(c, 64, 1, 0), d_pro, d_epi, 4096,
                 None, None, None, None)
    epi = host(d_epi)
    nreg = len(c["check_rows"])
    bufs = [torch.zeros(40 * nreg, dtype=torch.uint8, device="cuda:0") for _ in range(3)]

    # what each variant gives when evaluated alone
    alone = []
    for block, unroll, bug in ri.JACOBI_VARIANTS:
        rc, out = r3.r3_eval_candidate(ctx, tbl, d_pro, chk, d_epi, d_live, wl.jacobi_launch(),
                                       wl.jacobi_args(c, block, unroll, bug), 0, 2, r3.EVERY, bufs[2])
        exp_res, exp_sum = oracle.compare(oracle.make_table(c["check_rows"]), host(d_live), epi)
        assert_results_equal(r3.results_to_numpy(bufs[2], nreg), exp_res, "alone")
        assert out.total_mismatch == int(exp_sum[0]["total_mismatch"])
        alone.append((exp_res, out))
    assert [o.passed for _, o in alone].count(0) == 1

    # depth two: submit variant i+1 before waiting for variant i
    pending = None
    got = []
    for i, (block, unroll, bug) in enumerate(ri.JACOBI_VARIANTS):
        t = r3.r3_eval_submit(ctx, tbl, d_pro, chk, d_epi, d_live, wl.jacobi_launch(),
                              wl.jacobi_args(c, block, unroll, bug), 0, 2, r3.EVERY, bufs[i % 2])
        if pending is not None:
            rc, out = r3.r3_eval_wait(ctx, pending[0])
            got.append((r3.results_to_numpy(bufs[pending[1] % 2], nreg).copy(), out))
        pending = (t, i)
    rc, out = r3.r3_eval_wait(ctx, pending[0])
    got.append((r3.results_to_numpy(bufs[pending[1] % 2], nreg).copy(), out))
    for i, ((exp_res, exp_out), (res, out)) in enumerate(zip(alone, got)):
        what = "variant %d" % i
        assert_results_equal(res, exp_res, what)
        for f in ("total_mismatch", "first_region", "first_index", "passed", "max_abs_err", "max_rel_err"):
            assert getattr(out, f) == getattr(exp_out, f), (what, f)

    # a candidate that cannot be launched: the submission is accepted, the wait reports it
    code = ctypes.c_int(9)
    t_bad = r3.r3_eval_submit(ctx, tbl, d_pro, chk, d_epi, d_live, wl.failing_launch(), ctypes.addressof(code),
                              0, 3, r3.EVERY, bufs[0])
    t_good = r3.r3_eval_submit(ctx, tbl, d_pro, chk, d_epi, d_live, wl.jacobi_launch(),
                               wl.jacobi_args(c, 64, 1, 0), 0, 1, r3.EVERY, bufs[1])
    # the synchronous call while both are outstanding
    rc, out = r3.r3_eval_candidate(ctx, tbl, d_pro, tbl, d_pro, d_live, None, None, 0, 1, r3.EVERY, bufs[2])
    assert rc == r3.OK and out.passed == 1
    rc, out = r3.r3_eval_wait(ctx, t_good)
    assert rc == r3.OK and out.passed == 1 and out.candidate_status == 0
    rc, out = r3.r3_eval_wait(ctx, t_bad)
    assert rc == r3.ECANDIDATE and out.passed == 0 and out.candidate_status == 9
    # argument errors are raised by the submission itself and take no ticket
    with pytest.raises(r3.R3Error) as e:
        r3.r3_eval_submit(ctx, tbl, d_pro, chk, d_epi, d_live, None, None, 0, 0, r3.EVERY, bufs[0])
    assert e.value.status == r3.EINVAL
    for bad_ticket in (0, 9, 3):
        with pytest.raises(r3.R3Error) as e:
            r3.r3_eval_wait(ctx, bad_ticket)
        assert e.value.status == r3.EINVAL
    tickets = [r3.r3_eval_submit(ctx, tbl, d_pro, tbl, d_pro, d_live, None, None, 0, 1, r3.EVERY, bufs[0])
               for _ in range(8)]
    assert sorted(tickets) == list(range(1, 9))
    for t in tickets:
        rc, out = r3.r3_eval_wait(ctx, t)
        assert rc == r3.OK and out.passed == 1


def test_several_units_resident(env, oracle):
    """Three replay units (Jacobi, CSR SpMV, the small pure replay) stay resident side by side, each
    with its own tables, snapshots and live arena; evaluations of all three are in flight together
    on one stream and each verdict is the one that unit gives when evaluated alone."""
    r3, wl, ctx, torch = env

    def record(case, restore_rows, launch, args):
        A = case["arena_bytes"]
        tbl = r3.Table(ctx, restore_rows, A)
        d_live = dev(torch, case["prologue"])
        d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
        d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
        r3.r3_record(ctx, tbl, d_live, launch, args, d_pro, d_epi, 4096, None, None, None, None)
        return tbl, d_live, d_pro, d_epi

    units = []
    cj = ri.jacobi(40)
    tbl, d_live, d_pro, d_epi = record(cj, cj["restore_rows"], wl.jacobi_launch(), wl.jacobi_args(cj, 64, 1, 0))
    units.append(dict(name="jacobi", restore=tbl, check=r3.Table(ctx, cj["check_rows"], cj["arena_bytes"]),
                      rows=cj["check_rows"], live=d_live, pro=d_pro, epi=d_epi, launch=wl.jacobi_launch(),
                      cands=[wl.jacobi_args(cj, b, u, g) for b, u, g in ri.JACOBI_VARIANTS]))
    cs = ri.spmv(1 << 15)
    tbl, d_live, d_pro, d_epi = record(cs, cs["table_rows"], wl.spmv_launch(), wl.spmv_args(cs, 64, 256))
    units.append(dict(name="spmv", restore=tbl, check=r3.Table(ctx, cs["y_rows"], cs["arena_bytes"]),
                      rows=cs["y_rows"], live=d_live, pro=d_pro, epi=d_epi, launch=wl.spmv_launch(),
                      cands=[wl.spmv_args(cs, rpw, blk) for rpw, blk in ri.SPMV_VARIANTS[::9]]))
    cr = ri.replay_small()
    A = cr["arena_bytes"]
    units.append(dict(name="small", restore=r3.Table(ctx, cr["restore_rows"], A),
                      check=r3.Table(ctx, cr["check_rows"], A), rows=cr["check_rows"],
                      live=dev(torch, cr["live"]), pro=dev(torch, cr["prologue"]), epi=dev(torch, cr["epilogue"]),
                      launch=None, cands=[None, None]))

    # each candidate of each unit alone, checked against the oracle on the bytes it left
    for u in units:
        u["alone"] = []
        # one result array per evaluation that can be in flight
        u["bufs"] = [torch.zeros(40 * len(u["rows"]), dtype=torch.uint8, device="cuda:0") for _ in range(6)]
        epi = host(u["epi"])
        for cand in u["cands"]:
            rc, out = r3.r3_eval_candidate(ctx, u["restore"], u["pro"], u["check"], u["epi"], u["live"],
                                           u["launch"], cand, 0, 1, r3.EVERY, u["bufs"][0])
            assert rc == r3.OK
            exp_res, exp_sum = oracle.compare(oracle.make_table(u["rows"]), host(u["live"]), epi)
            assert_results_equal(r3.results_to_numpy(u["bufs"][0], len(u["rows"])), exp_res, u["name"])
            assert out.total_mismatch == int(exp_sum[0]["total_mismatch"])
            u["alone"].append((exp_res, out))
    assert units[2]["alone"][0][1].total_mismatch == 1049

    # round robin over the units, up to six evaluations in flight
    work = []
    most = max(len(u["cands"]) for u in units)
    for k in range(most):
        for ui, u in enumerate(units):
            if k < len(u["cands"]):
                work.append((ui, k))
    inflight = []
    done = 0

    def collect():
        ticket, ui, k, buf = inflight.pop(0)
        u = units[ui]
        rc, out = r3.r3_eval_wait(ctx, ticket)
        exp_res, exp_out = u["alone"][k]
        what = "%s candidate %d" % (u["name"], k)
        assert rc == r3.OK, what
        assert_results_equal(r3.results_to_numpy(buf, len(u["rows"])), exp_res, what)
        for f in ("total_mismatch", "first_region", "first_index", "passed", "max_abs_err", "max_rel_err"):
            assert getattr(out, f) == getattr(exp_out, f), (what, f)

    for n_sub, (ui, k) in enumerate(work):
        u = units[ui]
        buf = u["bufs"][n_sub % 6]
        t = r3.r3_eval_submit(ctx, u["restore"], u["pro"], u["check"], u["epi"], u["live"], u["launch"],
                              u["cands"][k], 0, 1, r3.EVERY, buf)
        inflight.append((t, ui, k, buf))
        if len(inflight) == 6:
            collect()
            done += 1
    while inflight:
        collect()
        done += 1
    assert done == len(work)


def test_side_stream(env, oracle):
    """Everything is enqueued on the stream the caller names: a replay on a second stream (default
    priority) gives the oracle's results, also while the default stream is busy with other work."""
    r3, wl, ctx, torch = env
    c = ri.jacobi(40)
    A = c["arena_bytes"]
    side = torch.cuda.Stream()
    tbl = r3.Table(ctx, c["restore_rows"], A)
    chk = r3.Table(ctx, c["check_rows"], A)
    d_live = dev(torch, c["prologue"])
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    nreg = len(c["check_rows"])
    d_regions = torch.zeros(40 * nreg, dtype=torch.uint8, device="cuda:0")
    d_cs = torch.zeros(len(c["restore_rows"]), dtype=torch.int64, device="cuda:0")
    torch.cuda.synchronize()
    busy = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
    r3.r3_record(ctx, tbl, d_live, wl.jacobi_launch(), wl.jacobi_args(c, 64, 1, 0), d_pro, d_epi, 4096,
                 None, None, None, None, stream=side)
    epi = host(d_epi)
    for i, (block, unroll, bug) in enumerate(ri.JACOBI_VARIANTS):
        busy.fill_(i)                       # unrelated work on the default stream
        args = wl.jacobi_args(c, block, unroll, bug)
        if i % 2 == 0:
            rc, out = r3.r3_eval_candidate(ctx, tbl, d_pro, chk, d_epi, d_live, wl.jacobi_launch(), args,
                                           1, 2, r3.EVERY, d_regions, stream=side)
        else:
            t = r3.r3_eval_submit(ctx, tbl, d_pro, chk, d_epi, d_live, wl.jacobi_launch(), args,
                                  1, 2, r3.EVERY, d_regions, stream=side)
            rc, out = r3.r3_eval_wait(ctx, t)
        assert rc == r3.OK
        side.synchronize()
        exp_res, exp_sum = oracle.compare(oracle.make_table(c["check_rows"]), host(d_live), epi)
        assert_results_equal(r3.results_to_numpy(d_regions, nreg), exp_res, "variant %d" % i)
        assert out.total_mismatch == int(exp_sum[0]["total_mismatch"]) and out.passed == int(not bug)
    # the asynchronous calls: nothing is waited for until the caller does
    d_sum = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()                # d_sum's fill ran on the default stream
    r3.r3_restore(ctx, tbl, d_pro, d_live, stream=side)
    r3.r3_checksum(ctx, tbl, d_live, d_cs, stream=side)
    r3.r3_compare(ctx, chk, d_live, d_epi, d_regions, d_sum, stream=side)
    side.synchronize()
    pro = host(d_pro)
    assert (host(d_live) == pro).all()
    assert (host(d_cs).view(np.uint64) == oracle.checksum(oracle.make_table(c["restore_rows"]), pro)).all()
    exp_res, exp_sum = oracle.compare(oracle.make_table(c["check_rows"]), pro, epi)
    assert_results_equal(r3.results_to_numpy(d_regions, nreg), exp_res, "restored state against the epilogue")
    assert_results_equal(r3.summary_to_numpy(d_sum), exp_sum, "summary")


def test_try_wait_gives_up_and_can_be_repeated(env, oracle):
    """r3_eval_try_wait on an evaluation that takes tens of milliseconds: a zero timeout reports that it
    is still running and leaves the ticket alone; later calls get the verdict that r3_eval_wait gives."""
    r3, wl, ctx, torch = env
    c = ri.jacobi(256)
    A = c["arena_bytes"]
    tbl = r3.Table(ctx, c["restore_rows"], A)
    chk = r3.Table(ctx, c["check_rows"], A)
    d_live = dev(torch, c["prologue"])
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    r3.r3_record(ctx, tbl, d_live, wl.jacobi_launch(), wl.jacobi_args(c, 64, 1, 0), d_pro, d_epi, 4096,
                 None, None, None, None)
    nreg = len(c["check_rows"])
    bufs = [torch.zeros(40 * nreg, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
    bug = wl.jacobi_args(c, 128, 2, 1)
    rc, ref = r3.r3_eval_candidate(ctx, tbl, d_pro, chk, d_epi, d_live, wl.jacobi_launch(), bug, 0, 1,
                                   r3.EVERY, bufs[0])
    exp_res, _ = oracle.compare(oracle.make_table(c["check_rows"]), host(d_live), host(d_epi))
    assert_results_equal(r3.results_to_numpy(bufs[0], nreg), exp_res, "one replay")
    torch.cuda.synchronize()
    # 300 replays of ~0.2 ms each: far from finished when the submission returns
    t = r3.r3_eval_submit(ctx, tbl, d_pro, chk, d_epi, d_live, wl.jacobi_launch(), bug, 0, 300, r3.EVERY, bufs[1])
    assert r3.r3_eval_try_wait(ctx, t, 0) is None
    assert r3.r3_eval_try_wait(ctx, t, 200) is None          # 0.2 ms more: still running
    got = None
    for _ in range(2000):                                     # at most 2000 x 10 ms
        got = r3.r3_eval_try_wait(ctx, t, 10000)
        if got is not None:
            break
    assert got is not None
    rc, out, g = got
    assert rc == r3.OK and out.passed == 0
    for f in ("total_mismatch", "first_region", "first_index", "max_abs_err", "max_rel_err"):
        assert getattr(out, f) == getattr(ref, f), f
    assert_results_equal(r3.results_to_numpy(bufs[1], nreg), exp_res, "300 replays")
    assert len(ctx.last_times()) == 300
    # the ticket is spent now
    with pytest.raises(r3.R3Error) as e:
        r3.r3_eval_try_wait(ctx, t, 0)
    assert e.value.status == r3.EINVAL
    # a submission that validates only the first replay ends in an event, not in a posted number
    t = r3.r3_eval_submit(ctx, tbl, d_pro, chk, d_epi, d_live, wl.jacobi_launch(), bug, 0, 100, r3.FIRST, bufs[1])
    assert r3.r3_eval_try_wait(ctx, t, 0) is None
    rc, out = r3.r3_eval_wait(ctx, t)
    assert rc == r3.OK and out.total_mismatch == ref.total_mismatch


@pytest.mark.parametrize("n", [40, 128])
def test_overlapped_evaluations_on_two_live_arenas(env, oracle, n):
    """r3_eval_submit_overlapped: consecutive evaluations alternate between two live arenas and the
    context's two streams; every ticket's verdict, region results and final live state must be what the
    oracle's evaluation loop gives for that candidate, whatever the order the tickets are waited for in."""
    r3, wl, ctx, torch = env
    c = ri.jacobi(n)
    A = c["arena_bytes"]
    rt = r3.Table(ctx, c["restore_rows"], A)
    ct = r3.Table(ctx, c["check_rows"], A)
    d_live = [torch.full((A,), 0x11 * (i + 1), dtype=torch.uint8, device="cuda:0") for i in range(2)]
    d_live[0].copy_(dev(torch, c["prologue"]))
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    r3.r3_record(ctx, rt, d_live[0], wl.jacobi_launch(), wl.jacobi_args(c, 64, 1, 0), d_pro, d_epi)
    pro, epi = host(d_pro), host(d_epi)
    variants = list(ri.JACOBI_VARIANTS)                     # the last one carries the planted bug
    plans = [(0, 1, r3.EVERY), (1, 2, r3.EVERY), (0, 3, r3.LAST), (2, 1, r3.FIRST)]
    args = [wl.jacobi_args(c, b, u, g) for b, u, g in variants]
    d_regions = [torch.zeros(40 * ct.n, dtype=torch.uint8, device="cuda:0") for _ in variants]

    def cpu_candidate(bug):
        def run(live):
            g = live[c["in_off"]:c["in_off"] + c["grid_bytes"]].view("<f8").reshape(n, n, n)
            out = live[c["out_off"]:c["out_off"] + c["grid_bytes"]].view("<f8").reshape(n, n, n)
            ref = ri.jacobi_reference(g)
            if bug:
                ref[:, :, n - 2] = out[:, :, n - 2]      # the x loop stops one short: old values stay
            out[...] = ref
            return 0
        return run

    for order in ([0, 1, 2, 3, 4, 5, 6, 7], [7, 6, 5, 4, 3, 2, 1, 0], [1, 0, 3, 2, 5, 4, 7, 6]):
        print("case overlapped", n, order, flush=True)
        tickets = []
        for k, a in enumerate(args):
            warmup, reps, policy = plans[k % len(plans)]
            tickets.append(r3.r3_eval_submit_overlapped(ctx, rt, d_pro, ct, d_epi, d_live[k % 2], wl.jacobi_launch(), a,
                                                        warmup, reps, policy, d_regions[k]))
        outs = {}
        for k in order:
            outs[k] = r3.r3_eval_wait(ctx, tickets[k])
        torch.cuda.synchronize()
        lives = [None, None]
        for k, (b, u, bug) in enumerate(variants):
            warmup, reps, policy = plans[k % len(plans)]
            live = np.full(A, 0xEE, np.uint8)
            exp = oracle.eval_candidate(oracle.make_table(c["restore_rows"]), pro, oracle.make_table(c["check_rows"]),
                                        epi, live, cpu_candidate(bug), warmup, reps, policy)
            lives[k % 2] = live
            rc, out = outs[k]
            what = "evaluation %d (block %d unroll %d bug %d)" % (k, b, u, bug)
            assert rc == r3.OK, what
            assert out.total_mismatch == exp["total_mismatch"], what
            assert out.passed == exp["pass"] == int(not bug), what
            assert (out.first_region, out.first_index) == (exp["first_region"], exp["first_index"]), what
            assert_results_equal(r3.results_to_numpy(d_regions[k], ct.n), exp["regions"], what)
            assert out.ms_min > 0 and out.ms_min <= out.ms_median <= out.ms_max, what
        for i in range(2):
            assert (host(d_live[i]) == lives[i]).all(), "live arena %d" % i
    # the plain calls still work beside it, on the caller's stream
    rc, out = r3.r3_eval_candidate(ctx, rt, d_pro, ct, d_epi, d_live[0], wl.jacobi_launch(), args[0], 0, 1, r3.EVERY,
                                   d_regions[0])
    assert rc == r3.OK and out.passed == 1


def test_overlapped_pure_replays_and_failing_candidate(env, oracle):
    """Overlapped submissions without a candidate (restore -> validate only), and one whose launch fails:
    the failure is reported by its wait and the evaluations around it are not disturbed."""
    r3, wl, ctx, torch = env
    c = ri.replay_small(n=1 << 15)
    A = c["arena_bytes"]
    rt, ct = r3.Table(ctx, c["restore_rows"], A), r3.Table(ctx, c["check_rows"], A)
    d_pro, d_epi = dev(torch, c["prologue"]), dev(torch, c["epilogue"])
    d_live = [dev(torch, c["live"]), dev(torch, c["live"])]
    d_regions = [torch.zeros(40 * ct.n, dtype=torch.uint8, device="cuda:0") for _ in range(6)]
    live = c["live"].copy()
    exp = oracle.eval_candidate(oracle.make_table(c["restore_rows"]), c["prologue"], oracle.make_table(c["check_rows"]),
                                c["epilogue"], live, None, 0, 2)
    code = ctypes.c_int(9)
    tickets = []
    for k in range(6):
        if k == 3:
            tickets.append(r3.r3_eval_submit_overlapped(ctx, rt, d_pro, ct, d_epi, d_live[k % 2], wl.failing_launch(),
                                                        ctypes.addressof(code), 0, 2, r3.EVERY, d_regions[k]))
        else:
            tickets.append(r3.r3_eval_submit_overlapped(ctx, rt, d_pro, ct, d_epi, d_live[k % 2], None, None, 0, 2,
                                                        r3.EVERY, d_regions[k]))
    for k in (5, 0, 3, 1, 4, 2):
        rc, out = r3.r3_eval_wait(ctx, tickets[k])
        if k == 3:
            assert rc == r3.ECANDIDATE and out.passed == 0 and out.candidate_status == 9
            continue
        assert rc == r3.OK
        assert out.total_mismatch == exp["total_mismatch"] == c["n_planted"] and out.passed == 0
        assert out.first_index == exp["first_index"]
        assert_results_equal(r3.results_to_numpy(d_regions[k], ct.n), exp["regions"], "pure replay %d" % k)
    torch.cuda.synchronize()
    for i in range(2):
        assert (host(d_live[i]) == live).all()

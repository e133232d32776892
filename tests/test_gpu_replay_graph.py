"""GPU parity of the captured replay (restore, candidate, validation as one HIP graph): the
same verdicts as the eager loop and as the oracle, on every one of several replays of the
graph, with eager work and synchronisations in between."""
import time

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


def same(out_a, out_b):
    return all(getattr(out_a, f) == getattr(out_b, f) for f in
               ("total_mismatch", "first_index", "first_region", "passed", "max_abs_err", "max_rel_err"))


def test_captured_jacobi_replays(env, oracle):
    r3, wl, ctx, torch = env
    n = 40
    c = ri.jacobi(n)
    A = c["arena_bytes"]
    tbl = r3.Table(ctx, c["restore_rows"], A)
    d_live = dev(torch, c["prologue"])
    d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
    r3.r3_record(ctx, tbl, d_live, wl.jacobi_launch(), wl.jacobi_args(c, 64, 1, 0), d_pro, d_epi)
    epi = host(d_epi)
    d_regions = torch.zeros(80, dtype=torch.uint8, device="cuda:0")
    d_regions_eager = torch.zeros(80, dtype=torch.uint8, device="cuda:0")
    for block, unroll, bug in [(256, 1, 0), (128, 2, 1), (1024, 1, 0)]:
        args = wl.jacobi_args(c, block, unroll, bug)
        rp = r3.Replay(ctx, tbl, d_pro, tbl, d_epi, d_live, wl.jacobi_launch(), args, d_regions, 4)
        rc, eager = r3.r3_eval_candidate(ctx, tbl, d_pro, tbl, d_epi, d_live, wl.jacobi_launch(), args,
                                         1, 3, r3.EVERY, d_regions_eager)
        exp_res, exp_sum = oracle.compare(oracle.make_table(c["check_rows"]), host(d_live), epi)
        for round_ in range(4):
            d_live.fill_(0x77)                         # eager work between the graph replays
            torch.cuda.synchronize()
            out = rp.run(1, 3)
            assert same(out, eager), (block, unroll, bug, round_)
            assert r3.results_to_numpy(d_regions, 2).tobytes() == exp_res.tobytes()
            assert out.total_mismatch == int(exp_sum[0]["total_mismatch"]) == ((n - 2) ** 2 if bug else 0)
            assert (host(d_live) == host(d_live)).all()
            t = ctx.last_times()
            assert t.size == 3 and (t > 0).all() and (t < 50).all()
            assert out.ms_min <= out.ms_median <= out.ms_max
        rp.close()
    with pytest.raises(r3.R3Error) as e:
        r3.Replay(ctx, tbl, d_pro, tbl, d_epi, d_live, wl.failing_launch(), None, d_regions, 2)
    assert e.value.status == r3.ECANDIDATE
    # the library is still usable after a failed capture
    rc, out = r3.r3_eval_candidate(ctx, tbl, d_pro, tbl, d_epi, d_live, wl.jacobi_launch(),
                                   wl.jacobi_args(c, 64, 1, 0), 0, 1, r3.EVERY, d_regions)
    assert rc == r3.OK and out.passed == 1


def test_captured_pure_replay_small(env, oracle):
    r3, wl, ctx, torch = env
    c = ri.replay_small()
    A = c["arena_bytes"]
    rt, ct = r3.Table(ctx, c["restore_rows"], A), r3.Table(ctx, c["check_rows"], A)
    d_pro, d_epi, d_live = dev(torch, c["prologue"]), dev(torch, c["epilogue"]), dev(torch, c["live"])
    d_regions = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    rp = r3.Replay(ctx, rt, d_pro, ct, d_epi, d_live, None, None, d_regions, 10)
    live = c["live"].copy()
    exp = oracle.eval_candidate(oracle.make_table(c["restore_rows"]), c["prologue"],
                                oracle.make_table(c["check_rows"]), c["epilogue"], live, None, 0, 10)
    for round_ in range(3):
        d_live[:1024].fill_(round_)
        torch.cuda.synchronize()
        out = rp.run(0, 10)
        assert r3.results_to_numpy(d_regions, 1).tobytes() == exp["regions"].tobytes()
        assert out.total_mismatch == exp["total_mismatch"] == 1049 and out.passed == 0
        assert out.first_index == exp["first_index"]
        assert (host(d_live) == live).all()
    # how much the graph saves on a launch-bound replay (printed, not asserted)
    for name, fn in (("eager", lambda: r3.r3_eval_candidate(ctx, rt, d_pro, ct, d_epi, d_live, None, None, 0, 10,
                                                             r3.EVERY, d_regions)),
                     ("graph", lambda: rp.run(0, 10))):
        fn()
        t0 = time.perf_counter()
        for _ in range(50):
            fn()
        print("%s: %.1f us per replay" % (name, (time.perf_counter() - t0) / 500 * 1e6), flush=True)
    rp.close()

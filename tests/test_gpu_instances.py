"""GPU parity of multi-instance validation (one candidate against several recorded
prologue/epilogue pairs in one restore launch and one validation launch) and of the
per-replay timing hook."""
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


def test_jacobi_three_instances(env, oracle):
    r3, wl, ctx, torch = env
    n, k = 48, 3
    cases = [ri.jacobi(n, seed=1002 + 10 * i) for i in range(k)]
    A = cases[0]["arena_bytes"]
    stride = (A + 4095) // 4096 * 4096 + 4096          # a gap between instances
    total = (k - 1) * stride + A
    pro = np.zeros(total, dtype=np.uint8)
    for i, c in enumerate(cases):
        pro[i * stride:i * stride + A] = c["prologue"]
    c0 = cases[0]
    rows = r3.r3_table_replicate(r3.make_table(c0["restore_rows"]), stride, k)
    assert rows.tobytes() == oracle.replicate_table(oracle.make_table(c0["restore_rows"]), stride, k).tobytes()
    tbl = r3.Table(ctx, rows, total)
    d_pro = dev(torch, pro)
    d_epi = d_pro.clone()
    d_live = torch.full((total,), 0x33, dtype=torch.uint8, device="cuda:0")
    # record every instance with the baseline kernel (one launch each, offsets inside the view)
    base = wl.jacobi_args(c0, 64, 1, 0)
    launch = wl.lib().r3w_jacobi_launch
    launch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    for i in range(k):
        assert launch(ctypes.addressof(base), d_epi.data_ptr() + i * stride, 0) == 0
    torch.cuda.synchronize()
    epi = host(d_epi)
    for i, c in enumerate(cases):
        grid = c["prologue"][:c["grid_bytes"]].view("<f8").reshape(n, n, n)
        got = epi[i * stride + c["out_off"]:i * stride + c["out_off"] + c["grid_bytes"]].view("<f8")
        assert np.allclose(got.reshape(n, n, n), ri.jacobi_reference(grid), rtol=1e-12, atol=0)

    d_regions = torch.zeros(40 * tbl.n, dtype=torch.uint8, device="cuda:0")
    for block, unroll, bug in [(256, 2, 0), (128, 2, 1)]:
        args = wl.jacobi_args(c0, block, unroll, bug)
        rc, out, flags = r3.r3_eval_candidate_instances(ctx, tbl, d_pro, tbl, d_epi, d_live, wl.jacobi_launch(),
                                                        args, k, stride, 1, 2, r3.EVERY, d_regions)
        live = host(d_live)
        exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, epi)
        assert rc == r3.OK
        assert r3.results_to_numpy(d_regions, tbl.n).tobytes() == exp_res.tobytes()
        assert out.total_mismatch == int(exp_sum[0]["total_mismatch"]) == (k * (n - 2) ** 2 if bug else 0)
        assert list(flags) == [int(not bug)] * k and out.passed == int(not bug)
        assert (live[A:stride] == 0x33).all()            # gaps between instances untouched
        times = ctx.last_times()
        assert times.size == 2 and (times > 0).all()
        assert abs(float(np.median(times)) - out.ms_median) < 1e-6
        st = r3.r3_timing_stats(times, 0.5)
        assert st.n == 2 and st.min == out.ms_min and st.max == out.ms_max

    # a candidate that is right on the first instances and wrong on the last one
    good = wl.jacobi_args(c0, 256, 1, 0)
    bad = wl.jacobi_args(c0, 256, 1, 1)
    state = {"i": 0}

    def mixed(live_ptr, stream):
        a = bad if state["i"] % k == k - 1 else good
        state["i"] += 1
        return launch(ctypes.addressof(a), live_ptr, stream)
    rc, out, flags = r3.r3_eval_candidate_instances(ctx, tbl, d_pro, tbl, d_epi, d_live, mixed, None, k, stride,
                                                    0, 2, r3.EVERY, d_regions)
    assert rc == r3.OK and list(flags) == [1] * (k - 1) + [0] and out.passed == 0
    assert out.first_region == 2 * (k - 1) + 1 and out.first_index == (1 * n + 1) * n + (n - 2)
    exp_res, _ = oracle.compare(oracle.make_table(rows), host(d_live), epi)
    assert r3.results_to_numpy(d_regions, tbl.n).tobytes() == exp_res.tobytes()

    # argument checks
    with pytest.raises(r3.R3Error) as e:
        r3.r3_eval_candidate_instances(ctx, tbl, d_pro, tbl, d_epi, d_live, None, None, 4, stride, 0, 1, r3.EVERY,
                                       d_regions)
    assert e.value.status == r3.EINVAL
    with pytest.raises(r3.R3Error) as e:
        r3.r3_eval_candidate_instances(ctx, tbl, d_pro, tbl, d_epi, d_live, None, None, k, stride * 4, 0, 1,
                                       r3.EVERY, d_regions)
    assert e.value.status == r3.ERANGE


@pytest.mark.timeout(600)
def test_jacobi_two_instances_full_size(env, oracle):
    """Two recorded instances of the 256^3 Jacobi state in one super arena: regions of 128 MiB (16 KiB
    tiles) next to a 12 KiB side region per instance (4 KiB tiles), so the restore launch mixes size
    classes and the validation folds thousands of partials per region."""
    r3, wl, ctx, torch = env
    n, k = 256, 2
    cases = [ri.jacobi(n, seed=1002 + 10 * i) for i in range(k)]
    c0 = cases[0]
    A = c0["arena_bytes"]
    side = 3 * 4096
    stride = A + side + 4096                            # side region, then a gap
    total = (k - 1) * stride + A + side
    rng = np.random.default_rng(4242)
    pro = np.zeros(total, dtype=np.uint8)
    for i, c in enumerate(cases):
        pro[i * stride:i * stride + A] = c["prologue"]
        pro[i * stride + A:i * stride + A + side] = rng.integers(0, 256, size=side, dtype=np.uint8)
    one = list(c0["restore_rows"]) + [(A, side, ri.I32, ri.BITWISE, 0.0, 0.0)]
    rows = r3.r3_table_replicate(r3.make_table(one), stride, k)
    assert rows.tobytes() == oracle.replicate_table(oracle.make_table(one), stride, k).tobytes()
    tbl = r3.Table(ctx, rows, total)
    d_pro = dev(torch, pro)
    d_epi = d_pro.clone()
    d_live = torch.full((total,), 0x33, dtype=torch.uint8, device="cuda:0")
    base = wl.jacobi_args(c0, 64, 1, 0)
    launch = wl.lib().r3w_jacobi_launch
    launch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    for i in range(k):
        assert launch(ctypes.addressof(base), d_epi.data_ptr() + i * stride, 0) == 0
    torch.cuda.synchronize()
    epi = host(d_epi)
    d_regions = torch.zeros(40 * tbl.n, dtype=torch.uint8, device="cuda:0")
    for block, unroll, bug in [(512, 1, 0), (128, 2, 1)]:
        print("case instances 256^3 x 2", block, unroll, bug, flush=True)
        args = wl.jacobi_args(c0, block, unroll, bug)
        rc, out, flags = r3.r3_eval_candidate_instances(ctx, tbl, d_pro, tbl, d_epi, d_live, wl.jacobi_launch(),
                                                        args, k, stride, 0, 1, r3.EVERY, d_regions)
        live = host(d_live)
        exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, epi)
        s = exp_sum[0]
        assert rc == r3.OK
        assert r3.results_to_numpy(d_regions, tbl.n).tobytes() == exp_res.tobytes()
        assert out.total_mismatch == int(s["total_mismatch"]) == (k * (n - 2) ** 2 if bug else 0)
        assert out.first_region == int(s["first_region"]) and out.first_index == int(s["first_index"])
        assert np.float64(out.max_abs_err).tobytes() == s["max_abs_err"].tobytes()
        assert np.float64(out.max_rel_err).tobytes() == s["max_rel_err"].tobytes()
        assert list(flags) == [int(not bug)] * k and out.passed == int(not bug)
        if bug:
            assert out.first_region == 1 and out.first_index == (1 * n + 1) * n + (n - 2)
        assert (live[A + side:stride] == 0x33).all()    # the gap between the instances is untouched

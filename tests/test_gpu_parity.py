"""GPU parity: every entry point of libr3.so, called through the C ABI, against the CPU
oracle on the same seeded inputs.  Integer, index and checksum results must be equal;
the fp64 error maxima must be equal bit for bit (the path computes them with the same
IEEE operations in an order-free maximum, so the tolerance is zero)."""
import struct

import numpy as np
import pytest

import r3_inputs as ri

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2604_11109_amd import binding as r3
    assert torch.cuda.is_available(), "these tests need the GPU"
    r3.lib()  # raises if the HIP library is not built: there is no fallback
    ctx = r3.Context(0)
    yield r3, ctx, torch
    ctx.close()


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.cpu().numpy()


def assert_results_equal(got, exp, what=""):
    assert got.shape == exp.shape
    for name in exp.dtype.names:
        g = got[name].view(np.uint64) if got[name].dtype.kind == "f" else got[name]
        e = exp[name].view(np.uint64) if exp[name].dtype.kind == "f" else exp[name]
        bad = np.flatnonzero(g != e)
        assert bad.size == 0, "%s field %s differs at %s: got %s expected %s" % (
            what, name, bad[:5], got[name][bad[:5]], exp[name][bad[:5]])


def run_compare(r3, ctx, torch, rows, live, golden, arena_bytes):
    tbl = r3.Table(ctx, rows, arena_bytes)
    d_out = torch.zeros(40 * max(tbl.n, 1), dtype=torch.uint8, device="cuda:0")
    d_sum = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    r3.r3_compare(ctx, tbl, live, golden, d_out, d_sum)
    torch.cuda.synchronize()
    return r3.results_to_numpy(d_out, tbl.n), r3.summary_to_numpy(d_sum)


# ----------------------------------------------------------------------------------------
# checksum and restore on many small regions (the many-regions workload shape, reduced and full)
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("n_regions,max_bytes,align", [(300, 1 << 18, 256), (300, 1 << 17, 1),
                                                       (64, 1 << 21, 16), (4096, 1 << 20, 256),
                                                       # few regions, large and small, unaligned
                                                       (16, 1 << 22, 1), (12, 1 << 16, 1), (5, 1 << 24, 16),
                                                       (1, 1 << 20, 1), (17, 1 << 18, 1)])
def test_checksum_and_restore_many_regions(env, oracle, n_regions, max_bytes, align):
    r3, ctx, torch = env
    c = ri.many_regions(n_regions=n_regions, max_bytes=max_bytes, align=align, seed=1003 + align)
    print("case many_regions", n_regions, max_bytes, align, c["arena_bytes"], flush=True)
    otbl = oracle.make_table(c["rows"])
    tbl = r3.Table(ctx, c["rows"], c["arena_bytes"])
    d_snap, d_live = dev(torch, c["snapshot"]), dev(torch, c["live"])
    d_cs = torch.zeros(tbl.n, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, tbl, d_snap, d_cs)
    torch.cuda.synchronize()
    exp_cs = oracle.checksum(otbl, c["snapshot"])
    got_cs = host(d_cs).view(np.uint64)
    assert (got_cs == exp_cs).all(), np.flatnonzero(got_cs != exp_cs)[:10]
    # restore: regions copied, gaps untouched, snapshot unchanged
    r3.r3_restore(ctx, tbl, d_snap, d_live)
    torch.cuda.synchronize()
    exp_live = c["live"].copy()
    oracle.restore(otbl, c["snapshot"], exp_live)
    got_live = host(d_live)
    assert (got_live == exp_live).all(), np.flatnonzero(got_live != exp_live)[:10]
    assert (host(d_snap) == c["snapshot"]).all()
    # invariant: restore then checksum reproduces the recorded checksums
    d_cs2 = torch.zeros(tbl.n, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, tbl, d_live, d_cs2)
    torch.cuda.synchronize()
    assert (host(d_cs2).view(np.uint64) == exp_cs).all()


def test_checksum_edge_sizes(env, oracle):
    r3, ctx, torch = env
    rng = np.random.default_rng(21)
    arena = rng.integers(0, 256, size=1 << 16, dtype=np.uint8)
    sizes = [0, 1, 2, 7, 8, 9, 15, 16, 17, 31, 32, 33, 1023, 1024, 1025, 4095, 4096, 4097, 8191, 12289]
    rows, at = [], 0
    for s in sizes:
        rows.append((at, s, ri.U8, ri.BITWISE, 0, 0))
        at += (s + 15) // 16 * 16 + 16
    rows.append((at + 3, 777, ri.U8, ri.BITWISE, 0, 0))      # odd offset
    rows.append((at + 1024 + 2, 38, ri.BF16, ri.BITWISE, 0, 0))
    rows.append((at + 2048 + 4, 44, ri.I32, ri.BITWISE, 0, 0))
    rows.append((at + 3072 + 8, 808, ri.F64, ri.BITWISE, 0, 0))
    tbl = r3.Table(ctx, rows, arena.size)
    d_cs = torch.zeros(tbl.n, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, tbl, dev(torch, arena), d_cs)
    torch.cuda.synchronize()
    exp = oracle.checksum(oracle.make_table(rows), arena)
    assert (host(d_cs).view(np.uint64) == exp).all()


# ----------------------------------------------------------------------------------------
# fused compare + checksum
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed,align", [(1, 16), (2, 16), (3, 1), (4, 1), (5, 256), (6, 1)])
def test_compare_mixed_tables(env, oracle, seed, align):
    r3, ctx, torch = env
    c = ri.mixed_compare_case(seed, align=align, max_bytes=400000 if seed % 2 else 60000)
    print("case mixed_compare", seed, align, c["arena_bytes"], flush=True)
    exp_res, exp_sum = oracle.compare(oracle.make_table(c["rows"]), c["live"], c["golden"])
    got_res, got_sum = run_compare(r3, ctx, torch, c["rows"], dev(torch, c["live"]),
                                   dev(torch, c["golden"]), c["arena_bytes"])
    assert_results_equal(got_res, exp_res, "regions")
    assert_results_equal(got_sum, exp_sum, "summary")


def test_compare_replay_small_full_size(env, oracle):
    """the small-replay workload at full size: 1049 planted mismatches among one-step perturbations."""
    r3, ctx, torch = env
    c = ri.replay_small()
    exp_res, exp_sum = oracle.compare(oracle.make_table(c["check_rows"]), c["live"], c["epilogue"])
    got_res, got_sum = run_compare(r3, ctx, torch, c["check_rows"], dev(torch, c["live"]),
                                   dev(torch, c["epilogue"]), c["arena_bytes"])
    assert_results_equal(got_res, exp_res)
    assert_results_equal(got_sum, exp_sum)
    assert int(got_res[0]["mismatch_count"]) == c["n_planted"] == 1049
    assert int(got_res[0]["first_mismatch"]) == int(c["planted"][0])


def test_compare_self_and_single_perturbation(env, oracle):
    r3, ctx, torch = env
    rng = np.random.default_rng(31)
    n = 300001
    g = rng.standard_normal(n).astype("<f4")
    rows = [(0, 4 * n, ri.F32, ri.TOL, 1e-5, 1e-7)]
    arena_bytes = 4 * n + 12
    gold = np.zeros(arena_bytes, np.uint8)
    gold[:4 * n] = g.view(np.uint8)
    res, summ = run_compare(r3, ctx, torch, rows, dev(torch, gold), dev(torch, gold), arena_bytes)
    assert int(res[0]["mismatch_count"]) == 0 and int(res[0]["first_mismatch"]) == r3.NO_INDEX
    assert res[0]["max_abs_err"].tobytes() == bytes(8) and res[0]["max_rel_err"].tobytes() == bytes(8)
    assert int(summ[0]["pass"]) == 1 and int(summ[0]["first_region"]) == r3.NO_REGION
    for q in [0, 1, 65, 4095, 4096, 123457, n - 2, n - 1]:
        live = gold.copy()
        live[4 * q:4 * q + 4] = np.frombuffer(np.float32(g[q] * 1.25 + 0.5).tobytes(), np.uint8)
        exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, gold)
        res, summ = run_compare(r3, ctx, torch, rows, dev(torch, live), dev(torch, gold), arena_bytes)
        assert_results_equal(res, exp_res, "q=%d" % q)
        assert_results_equal(summ, exp_sum, "q=%d" % q)
        assert int(res[0]["mismatch_count"]) == 1 and int(res[0]["first_mismatch"]) == q


def test_compare_rounding_witnesses(env, oracle):
    """Cases where a fused multiply-add, a flushed subnormal or an inexact divide would show."""
    from fractions import Fraction
    r3, ctx, torch = env
    rng = np.random.default_rng(41)
    # (a) thresholds whose fused and unfused roundings differ, with d on the boundary
    found = []
    while len(found) < 40:
        rtol, atol, G = float(rng.uniform(0.1, 1)), float(rng.uniform(0.1, 1)), float(rng.uniform(0.5, 2))
        fused = float(Fraction(atol) + Fraction(rtol) * Fraction(G))
        unfused = float(Fraction(atol) + Fraction(float(Fraction(rtol) * Fraction(G))))
        if fused == unfused:
            continue
        c = G + max(fused, unfused)
        d = float(abs(Fraction(c) - Fraction(G)))
        if d == max(fused, unfused):
            found.append((rtol, atol, G, c))
    rows, live, gold = [], [], []
    for i, (rtol, atol, G, c) in enumerate(found):
        rows.append((16 * i, 8, ri.F64, ri.TOL, rtol, atol))
        live.append(struct.pack("<dd", c, 0.0))
        gold.append(struct.pack("<dd", G, 0.0))
    live = np.frombuffer(b"".join(live), np.uint8).copy()
    gold = np.frombuffer(b"".join(gold), np.uint8).copy()
    exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, gold)
    res, summ = run_compare(r3, ctx, torch, rows, dev(torch, live), dev(torch, gold), live.size)
    assert_results_equal(res, exp_res, "unfused threshold")
    assert 0 < int(exp_sum[0]["total_mismatch"]) < len(found)
    # (b) subnormal fp32 / bf16 / fp64 values and their neighbours; (c) random quotients
    n = 20000
    f32 = rng.integers(0, 0x00800000, size=n, dtype=np.uint32) | (rng.integers(0, 2, n, dtype=np.uint32) << 31)
    f32c = (f32.astype(np.int64) + rng.integers(-5, 6, n)).astype(np.uint32)
    bf = rng.integers(0, 0x0080, size=n, dtype=np.uint16)
    bfc = (bf.astype(np.int32) + rng.integers(-2, 3, n)).astype(np.uint16)
    f64 = rng.integers(0, 1 << 52, size=n, dtype=np.uint64)
    f64c = (f64.astype(np.int64) + rng.integers(-5, 6, n)).astype(np.uint64)
    q_g = (rng.standard_normal(n) * np.exp(rng.uniform(-300, 300, n))).astype("<f8")
    q_c = (q_g * (1 + rng.standard_normal(n) * 1e-3)).astype("<f8")
    parts_g = [f32.view(np.uint8), bf.view(np.uint8), f64.view(np.uint8), q_g.view(np.uint8)]
    parts_c = [f32c.view(np.uint8), bfc.view(np.uint8), f64c.view(np.uint8), q_c.view(np.uint8)]
    dts = [ri.F32, ri.BF16, ri.F64, ri.F64]
    rows, at = [], 0
    for p, dt in zip(parts_g, dts):
        rows.append((at, p.size, dt, ri.TOL, 1e-3, 1e-45))
        at += (p.size + 255) // 256 * 256
    gold = np.zeros(at, np.uint8)
    live = np.zeros(at, np.uint8)
    for (off, nb, *_), pg, pc in zip(rows, parts_g, parts_c):
        gold[off:off + nb] = pg
        live[off:off + nb] = pc
    exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, gold)
    res, summ = run_compare(r3, ctx, torch, rows, dev(torch, live), dev(torch, gold), at)
    assert_results_equal(res, exp_res, "subnormals and quotients")
    assert_results_equal(summ, exp_sum)
    # every element its own region: no maximum can hide a wrong quotient
    m = 3000
    rows1 = [(rows[3][0] + 8 * i, 8, ri.F64, ri.TOL, 1e-3, 0.0) for i in range(m)]
    exp_res, _ = oracle.compare(oracle.make_table(rows1), live, gold)
    res, _ = run_compare(r3, ctx, torch, rows1, dev(torch, live), dev(torch, gold), at)
    assert_results_equal(res, exp_res, "single-element regions")


def test_compare_large_snapshot_reduced(env, oracle):
    """the large-snapshot workload shape at 8 x 8 MiB: planted counts and first indices, checksums of live."""
    r3, ctx, torch = env
    c = ri.large_snapshot(n_regions=8, region_bytes=(8 << 20) + 4096 + 64, frac=1e-5)
    exp_res, exp_sum = oracle.compare(oracle.make_table(c["rows"]), c["snapshot"], c["golden"])
    res, summ = run_compare(r3, ctx, torch, c["rows"], dev(torch, c["snapshot"]), dev(torch, c["golden"]),
                            c["arena_bytes"])
    assert_results_equal(res, exp_res)
    assert_results_equal(summ, exp_sum)
    for r, idx in enumerate(c["planted"]):
        assert int(res[r]["mismatch_count"]) == len(idx) and int(res[r]["first_mismatch"]) == int(idx[0])


@pytest.mark.parametrize("min_tile,cap", [(1024, 64), (4096, 8192), (65536, 256), (1 << 20, 64)])
def test_tile_shapes_do_not_change_results(env, oracle, min_tile, cap):
    r3, ctx, torch = env
    c = ri.mixed_compare_case(9, align=16, max_bytes=3000000)
    exp_res, exp_sum = oracle.compare(oracle.make_table(c["rows"]), c["live"], c["golden"])
    r3.r3_tune_tiles(min_tile, cap)
    try:
        res, summ = run_compare(r3, ctx, torch, c["rows"], dev(torch, c["live"]), dev(torch, c["golden"]),
                                c["arena_bytes"])
        tbl = r3.Table(ctx, c["rows"], c["arena_bytes"])
        d_live = dev(torch, c["live"])
        r3.r3_restore(ctx, tbl, dev(torch, c["golden"]), d_live)
        d_cs = torch.zeros(tbl.n, dtype=torch.int64, device="cuda:0")
        r3.r3_checksum(ctx, tbl, d_live, d_cs)
        torch.cuda.synchronize()
    finally:
        r3.r3_tune_tiles(0, 0)
    assert_results_equal(res, exp_res)
    assert_results_equal(summ, exp_sum)
    assert (host(d_cs).view(np.uint64) == oracle.checksum(oracle.make_table(c["rows"]), c["golden"])).all()


# ----------------------------------------------------------------------------------------
# dirty-diff
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("nbytes,page", [(70 * 4096 + 123, 4096), (1 << 22, 4096), (5000, 256),
                                         (3 * (1 << 20) + 17, 1 << 20), (1, 4096), (64 * 4096, 4096),
                                         (64 * 4096 * 5 + 4095, 4096), (1 << 20, 65536)])
def test_dirty_diff(env, oracle, nbytes, page):
    r3, ctx, torch = env
    rng = np.random.default_rng(nbytes % 1000 + page)
    pre = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
    post = pre.copy()
    k = min(nbytes, 50)
    idx = rng.choice(nbytes, size=k, replace=False)
    post[idx] ^= rng.integers(1, 256, size=k, dtype=np.uint8)
    post[nbytes - 1] ^= 1
    post[0] ^= 0x80
    for a, b in [(pre, post), (pre, pre)]:
        nw = r3.bitmap_words(nbytes, page)
        d_bm = torch.full((nw + 2,), -1, dtype=torch.int64, device="cuda:0")
        d_cnt = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        r3.r3_dirty_diff(ctx, dev(torch, a), dev(torch, b), nbytes, page, d_bm, d_cnt)
        torch.cuda.synchronize()
        exp_bm, exp_cnt = oracle.dirty_diff(a, b, page)
        got = host(d_bm).view(np.uint64)
        assert (got[:nw] == exp_bm).all()
        assert (got[nw:] == 0xFFFFFFFFFFFFFFFF).all()        # nothing written past the bitmap
        assert int(host(d_cnt)[0]) == exp_cnt


def test_dirty_diff_empty_and_errors(env):
    r3, ctx, torch = env
    d = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    bm = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    cnt = torch.full((1,), 7, dtype=torch.int64, device="cuda:0")
    r3.r3_dirty_diff(ctx, d, d, 0, 4096, bm, cnt)
    torch.cuda.synchronize()
    assert int(host(cnt)[0]) == 0
    for bad_page in (0, 100, 128, 3000, 1 << 21):
        with pytest.raises(r3.R3Error) as e:
            r3.r3_dirty_diff(ctx, d, d, 4096, bad_page, bm, cnt)
        assert e.value.status == r3.EINVAL


# ----------------------------------------------------------------------------------------
# error paths that the host decides (no kernel runs)
# ----------------------------------------------------------------------------------------
def test_host_rejections(env):
    r3, ctx, torch = env
    a = torch.zeros(4096 + 16, dtype=torch.uint8, device="cuda:0")
    b = torch.zeros(4096 + 16, dtype=torch.uint8, device="cuda:0")
    tbl = r3.Table(ctx, [(0, 1024, ri.F32, ri.BITWISE, 0, 0)], 4096)
    out = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(r3.R3Error) as e:
        r3.r3_restore(ctx, tbl, a[1:], b)
    assert e.value.status == r3.EALIGN
    with pytest.raises(r3.R3Error) as e:
        r3.r3_restore(ctx, tbl, a, a)
    assert e.value.status == r3.EINVAL
    with pytest.raises(r3.R3Error) as e:
        r3.r3_compare(ctx, tbl, a.data_ptr(), 0, out)
    assert e.value.status == r3.EINVAL
    with pytest.raises(r3.R3Error) as e:
        r3.Table(ctx, [(0, 1024, ri.F32, ri.BITWISE, 0, 0), (512, 1024, ri.F32, ri.BITWISE, 0, 0)], 4096)
    assert e.value.status == r3.EOVERLAP
    with pytest.raises(r3.R3Error) as e:
        r3.Table(ctx, [], 4096)
    assert e.value.status == r3.EINVAL
    ctx2 = r3.Context(0)
    with pytest.raises(r3.R3Error) as e:
        r3.r3_restore(ctx2, tbl, a, b)
    assert e.value.status == r3.EINVAL
    ctx2.close()


@pytest.mark.timeout(900)
def test_region_larger_than_4_gib(env, oracle):
    """One 5 GiB byte region: element indices, tile offsets and the checksum key all pass 2^32."""
    r3, ctx, torch = env
    free, _ = torch.cuda.mem_get_info()
    if free < 16 * (1 << 30):
        pytest.skip("needs 16 GiB of device memory")
    n = 5 * (1 << 30) + 4096 + 5                      # ragged tail, not a multiple of 16
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(77)
    d_gold = torch.empty(n + 11, dtype=torch.uint8, device="cuda:0")
    for lo in range(0, n + 11, 1 << 30):
        hi = min(n + 11, lo + (1 << 30))
        d_gold[lo:hi] = torch.randint(0, 256, (hi - lo,), generator=gen, device="cuda:0", dtype=torch.uint8)
    d_live = torch.empty_like(d_gold)
    d_live[n - 64:n] = 0x5A
    d_live[n:] = 0xA5                                  # canary past the ragged tail
    rows = [(0, n, ri.U8, ri.BITWISE, 0, 0)]
    tbl = r3.Table(ctx, rows, n)
    r3.r3_restore(ctx, tbl, d_gold, d_live)
    planted = [(1 << 32) + 123457, (1 << 32) + (1 << 29) + 5, n - 1]
    for q in planted:
        d_live[q] = d_live[q] ^ 0x10
    d_out = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    d_sum = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    r3.r3_compare(ctx, tbl, d_live, d_gold, d_out, d_sum)
    d_cs = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, tbl, d_live, d_cs)
    torch.cuda.synchronize()
    res = r3.results_to_numpy(d_out, 1)[0]
    summ = r3.summary_to_numpy(d_sum)[0]
    assert int(res["mismatch_count"]) == 3 and int(res["first_mismatch"]) == planted[0]
    assert float(res["max_abs_err"]) == 16.0
    assert int(summ["total_mismatch"]) == 3 and int(summ["first_index"]) == planted[0]
    # the bytes past the region were not written, the last bytes of the region were
    assert (host(d_live[n:]) == 0xA5).all()
    tail_live, tail_gold = host(d_live[n - 64:n]), host(d_gold[n - 64:n])
    tail_gold[-1] ^= 0x10                              # the planted change at n - 1
    assert (tail_live == tail_gold).all()
    # checksum of the 5 GiB of live bytes against the oracle (fused and stand-alone kernels)
    live_h = host(d_live[:n])
    exp = oracle.checksum(oracle.make_table(rows), live_h)
    assert int(res["checksum"]) == int(exp[0]) == int(host(d_cs).view(np.uint64)[0])
    # the oracle's verdict on the last GiB (with the region re-based) agrees on count and index
    lo = n - (1 << 30)
    gold_tail = host(d_gold[lo:n])
    sub = [(0, n - lo, ri.U8, ri.BITWISE, 0, 0)]
    exp_res, _ = oracle.compare(oracle.make_table(sub), live_h[lo:], gold_tail)
    assert lo < planted[0]
    assert int(exp_res[0]["mismatch_count"]) == 3
    assert int(exp_res[0]["first_mismatch"]) + lo == planted[0]


def test_compare_many_regions_full_size(env, oracle):
    """The many-regions workload at full size (4096 regions, ~0.5 GiB) through the fused compare:
    the live state is the restored snapshot with a seeded handful of bytes changed."""
    r3, ctx, torch = env
    c = ri.many_regions()
    rng = np.random.default_rng(4242)
    rows = [(off, nb, dt, ri.TOL if i % 3 == 0 else ri.BITWISE, 1e-3, 1e-6)
            for i, (off, nb, dt, _, _, _) in enumerate(c["rows"])]
    live = c["snapshot"].copy()
    idx = rng.choice(c["arena_bytes"], size=3000, replace=False)
    live[idx] ^= rng.integers(1, 256, size=idx.size, dtype=np.uint8)
    exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, c["snapshot"])
    got_res, got_sum = run_compare(r3, ctx, torch, rows, dev(torch, live), dev(torch, c["snapshot"]),
                                   c["arena_bytes"])
    assert_results_equal(got_res, exp_res, "regions")
    assert_results_equal(got_sum, exp_sum, "summary")
    assert int(got_sum[0]["total_mismatch"]) > 1000


def test_compare_near_tied_relative_errors(env, oracle):
    """The largest relative error of a region when many elements are within a few units in the
    last place of it, for tiny, ordinary and huge recorded values and relative errors above one:
    the kernel divides only where the running maximum can still grow, and must not lose the
    element that carries it."""
    r3, ctx, torch = env
    rng = np.random.default_rng(4711)
    n = 150000
    parts = []   # (dtype, golden bits as uint8, live bits as uint8)

    def f64_case(scale_lo, scale_hi, rel, spread_ulps):
        g = (rng.choice([-1.0, 1.0], n) * rng.uniform(1, 2, n) * np.exp2(rng.integers(scale_lo, scale_hi + 1, n)))
        g = g.astype("<f8")
        # relative offsets that differ from `rel` by a few units in its last place
        k = rng.integers(-spread_ulps, spread_ulps + 1, n)
        r = (np.float64(rel).view(np.int64) + k).view(np.float64)
        c = (g * (1.0 + r)).astype("<f8")
        parts.append((ri.F64, g.view(np.uint8), c.view(np.uint8)))

    f64_case(-20, 20, 1e-3, 8)          # ordinary magnitudes
    f64_case(-1070, -1010, 1e-3, 8)     # recorded values so small that gate * |G| is subnormal
    f64_case(900, 1000, 1e-3, 8)        # huge values
    f64_case(-5, 5, 3.0, 4)             # relative errors above one
    f64_case(-1022, 1000, 2.0 ** -40, 2)  # the whole exponent range at once
    # fp32 and bf16: the same idea with the spread applied to the live bit patterns
    g32 = (rng.standard_normal(n) * np.exp2(rng.integers(-100, 100, n))).astype("<f4")
    c32 = (g32.astype(np.float64) * (1 + 1e-3)).astype("<f4")
    c32 = (c32.view(np.int32) + rng.integers(-1, 2, n).astype(np.int32)).view("<f4")
    parts.append((ri.F32, g32.view(np.uint8), c32.view(np.uint8)))
    gb = ri.f32_to_bf16_bits(rng.standard_normal(n) * np.exp2(rng.integers(-60, 60, n))).astype(np.uint16)
    cb = (gb.astype(np.int32) + rng.integers(-2, 3, n)).astype(np.uint16)
    parts.append((ri.BF16, gb.view(np.uint8), cb.view(np.uint8)))
    gh = (rng.uniform(1, 2, n) * rng.choice([-1.0, 1.0], n) * np.exp2(rng.integers(-12, 12, n)))
    gh = gh.astype("<f2").view(np.uint16)        # finite, well away from the largest binary16
    ch = (gh.astype(np.int32) + rng.integers(-2, 3, n)).astype(np.uint16)
    parts.append((ri.F16, gh.view(np.uint8), ch.view(np.uint8)))
    gi = rng.integers(-(1 << 31), 1 << 31, n).astype("<i4")
    ci = (gi.astype(np.int64) + rng.integers(-3, 4, n)).clip(-(1 << 31), (1 << 31) - 1).astype("<i4")
    parts.append((ri.I32, gi.view(np.uint8), ci.view(np.uint8)))

    rows, at = [], 0
    for i, (dt, pg, _) in enumerate(parts):
        rows.append((at, pg.size, dt, ri.TOL if i % 2 == 0 else ri.BITWISE, 1e-3, 0.0))
        at += (pg.size + 255) // 256 * 256
    gold, live = np.zeros(at, np.uint8), np.zeros(at, np.uint8)
    for (off, nb, *_), (_, pg, pc) in zip(rows, parts):
        gold[off:off + nb] = pg
        live[off:off + nb] = pc
    exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, gold)
    assert (exp_res["max_rel_err"][:5] > 0).all() and np.isfinite(exp_res["max_rel_err"]).all()
    res, summ = run_compare(r3, ctx, torch, rows, dev(torch, live), dev(torch, gold), at)
    assert_results_equal(res, exp_res, "near-tied relative errors")
    assert_results_equal(summ, exp_sum, "summary")
    # the same data in the opposite element order: the maxima cannot depend on who comes first
    gold_r, live_r = np.zeros(at, np.uint8), np.zeros(at, np.uint8)
    for (off, nb, dt, *_), (_, pg, pc) in zip(rows, parts):
        es = ri.ELEM_SIZE[dt]
        gold_r[off:off + nb] = pg.reshape(-1, es)[::-1].reshape(-1)
        live_r[off:off + nb] = pc.reshape(-1, es)[::-1].reshape(-1)
    res_r, _ = run_compare(r3, ctx, torch, rows, dev(torch, live_r), dev(torch, gold_r), at)
    for name in ("mismatch_count", "max_abs_err", "max_rel_err"):
        assert (res_r[name].view(np.uint64) == exp_res[name].view(np.uint64)).all(), name


def test_twenty_thousand_tiny_regions(env, oracle):
    """A table of 20000 regions of 0..64 bytes (one tile each at most): restore, checksum and
    compare against the oracle; the summary comes from a pass over 20000 region results."""
    r3, ctx, torch = env
    rng = np.random.default_rng(2024)
    n = 20000
    dts = [ri.U8, ri.F32, ri.F64, ri.I32, ri.BF16, ri.F16]
    rows, at = [], 0
    for i in range(n):
        dt = dts[int(rng.integers(0, 6))]
        es = ri.ELEM_SIZE[dt]
        nb = int(rng.integers(0, 64 // es + 1)) * es
        at = (at + es - 1) // es * es + int(rng.integers(0, 3)) * es
        rows.append((at, nb, dt, ri.TOL if i % 3 else ri.BITWISE, 1e-3, 1e-6))
        at += nb
    A = (at + 255) // 256 * 256
    snap = rng.integers(0, 256, size=A, dtype=np.uint8)
    live = snap.copy()
    idx = rng.choice(A, size=A // 200, replace=False)
    live[idx] ^= rng.integers(1, 256, size=idx.size, dtype=np.uint8)
    otbl = oracle.make_table(rows)
    tbl = r3.Table(ctx, rows, A)
    # restore into a canary-filled arena
    d_snap, d_dst = dev(torch, snap), torch.full((A,), 0xEE, dtype=torch.uint8, device="cuda:0")
    r3.r3_restore(ctx, tbl, d_snap, d_dst)
    exp_dst = np.full(A, 0xEE, np.uint8)
    oracle.restore(otbl, snap, exp_dst)
    assert (host(d_dst) == exp_dst).all()
    # checksums
    d_cs = torch.zeros(n, dtype=torch.int64, device="cuda:0")
    r3.r3_checksum(ctx, tbl, d_snap, d_cs)
    torch.cuda.synchronize()
    assert (host(d_cs).view(np.uint64) == oracle.checksum(otbl, snap)).all()
    # compare
    exp_res, exp_sum = oracle.compare(otbl, live, snap)
    got_res, got_sum = run_compare(r3, ctx, torch, rows, dev(torch, live), d_snap, A)
    assert_results_equal(got_res, exp_res, "regions")
    assert_results_equal(got_sum, exp_sum, "summary")
    assert int(got_sum[0]["total_mismatch"]) > 100


def test_restore_few_regions_with_empty_and_tiny_ones(env, oracle):
    """Restore of small tables under several copy shapes: empty regions at the start, in the middle
    and at the end, regions shorter than a copy unit, regions that start one element before or
    after a unit boundary, all element sizes."""
    r3, ctx, torch = env
    rng = np.random.default_rng(77)
    A = 1 << 20
    snap = rng.integers(0, 256, size=A, dtype=np.uint8)
    tables = [
        [(0, 0, ri.U8, 0, 0, 0), (1023, 1, ri.U8, 0, 0, 0), (1024, 0, ri.F64, 0, 0, 0), (1025, 1023, ri.U8, 0, 0, 0),
         (4096 - 2, 2050, ri.BF16, 0, 0, 0), (8192 + 4, 1020, ri.I32, 0, 0, 0), (16384 - 8, 24, ri.F64, 0, 0, 0),
         (32768, 3000, ri.F32, 0, 0, 0), (65536 + 1, 70001, ri.U8, 0, 0, 0), (A - 8, 8, ri.F64, 0, 0, 0),
         (A, 0, ri.U8, 0, 0, 0)],
        [(5, 1, ri.U8, 0, 0, 0)],
        [(0, A, ri.U8, 0, 0, 0)],
        [(8, A - 16, ri.F64, 0, 0, 0)],
        [(0, 0, ri.F32, 0, 0, 0), (0, 0, ri.F32, 0, 0, 0), (2, 6, ri.BF16, 0, 0, 0)],
    ]
    for unit, block in ((1024, 64), (4096, 256), (1 << 20, 128), (1024, 64)):
        assert r3.lib().r3_tune_copy(unit, block) == r3.OK
        for rows in tables:
            tbl = r3.Table(ctx, rows, A)
            d_live = torch.full((A,), 0xEE, dtype=torch.uint8, device="cuda:0")
            r3.r3_restore(ctx, tbl, dev(torch, snap), d_live)
            exp = np.full(A, 0xEE, np.uint8)
            oracle.restore(oracle.make_table(rows), snap, exp)
            got = host(d_live)
            assert (got == exp).all(), (unit, rows[:3], np.flatnonzero(got != exp)[:8])
    assert r3.lib().r3_tune_copy(0, 0) == r3.OK


def test_compare_every_binary16_pattern(env, oracle):
    """R3_F16: all 65536 patterns against all-zero, against themselves shifted by one, and pattern
    pairs (p, q) on a grid, under both modes: the device's conversion must agree with the oracle's
    for every value, subnormals, infinities and NaNs included."""
    r3, ctx, torch = env
    pats = np.arange(65536, dtype=np.uint16)
    rng = np.random.default_rng(16)
    cases = [(pats, np.zeros_like(pats)), (pats, np.roll(pats, 1)), (np.roll(pats, 7), pats),
             (rng.permutation(pats), rng.permutation(pats)), (np.full_like(pats, 0x3C00), pats)]
    n = pats.size * 2
    rows, at = [], 0
    for i in range(len(cases)):
        for mode, rtol, atol in ((ri.BITWISE, 0, 0), (ri.TOL, 1e-2, 1e-3), (ri.TOL, 0.0, 0.0)):
            rows.append((at, n, ri.F16, mode, rtol, atol))
            at += n
    live, gold = np.zeros(at, np.uint8), np.zeros(at, np.uint8)
    for r, (off, nb, *_), in enumerate(rows):
        c, g = cases[r // 3]
        live[off:off + nb] = c.view(np.uint8)
        gold[off:off + nb] = g.view(np.uint8)
    exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, gold)
    res, summ = run_compare(r3, ctx, torch, rows, dev(torch, live), dev(torch, gold), at)
    assert_results_equal(res, exp_res, "binary16 patterns")
    assert_results_equal(summ, exp_sum, "summary")
    # one element per region for a sample of pairs: no maximum can hide a wrong conversion
    m = 4000
    p, q = rng.integers(0, 65536, m).astype(np.uint16), rng.integers(0, 65536, m).astype(np.uint16)
    rows1 = [(2 * i, 2, ri.F16, ri.TOL, 1e-3, 1e-4) for i in range(m)]
    exp_res, _ = oracle.compare(oracle.make_table(rows1), p.view(np.uint8), q.view(np.uint8))
    res, _ = run_compare(r3, ctx, torch, rows1, dev(torch, p.view(np.uint8)), dev(torch, q.view(np.uint8)), 2 * m)
    assert_results_equal(res, exp_res, "single binary16 elements")


# ----------------------------------------------------------------------------------------
# states that differ from the recorded one in (almost) every element
# ----------------------------------------------------------------------------------------
def _dense_case(rng, dt, n_el):
    """Golden values of moderate size, live = golden moved by a few pattern steps in every element,
    then special cases planted all over: zeros on either side, NaN and infinity against finite values
    and against themselves, many elements with one and the same error ratio, a few outliers late in
    the region.  Returns (golden bytes, live bytes)."""
    es = ri.ELEM_SIZE[dt]
    if dt == ri.U8:
        g = rng.integers(0, 256, n_el, dtype=np.uint8)
        c = (g.astype(np.int32) + rng.integers(-2, 3, n_el)).astype(np.uint8)
    elif dt == ri.I32:
        g = rng.integers(-2**31, 2**31, n_el, dtype=np.int64).astype(np.int32)
        c = (g.astype(np.int64) + rng.integers(-3, 4, n_el)).astype(np.int32)
    else:
        x = rng.standard_normal(n_el) * np.exp(rng.uniform(-3, 3, n_el))
        if dt == ri.F64:
            g = x.astype("<f8")
            ib = g.view(np.int64)
        elif dt == ri.F32:
            g = x.astype("<f4")
            ib = g.view(np.int32)
        elif dt == ri.F16:
            g = x.astype("<f2")
            ib = g.view(np.int16)
        else:
            g = ri.f32_to_bf16_bits(x.astype("<f4")).view(np.int16).copy()
            ib = g
        c = (ib.astype(np.int64) + rng.integers(-2, 3, n_el)).astype(ib.dtype)
    g = np.ascontiguousarray(g).view(np.uint8).reshape(n_el, es).copy()
    c = np.ascontiguousarray(c).view(np.uint8).reshape(n_el, es).copy()

    def pat(v):
        return np.frombuffer(int(v).to_bytes(es, "little"), dtype=np.uint8)
    is_float = dt in (ri.F32, ri.F64, ri.BF16, ri.F16)
    if is_float:
        one = {ri.F32: 0x3F800000, ri.F64: 0x3FF0000000000000, ri.BF16: 0x3F80, ri.F16: 0x3C00}[dt]
        two = {ri.F32: 0x40000000, ri.F64: 0x4000000000000000, ri.BF16: 0x4000, ri.F16: 0x4000}[dt]
        inf = {ri.F32: 0x7F800000, ri.F64: 0x7FF0000000000000, ri.BF16: 0x7F80, ri.F16: 0x7C00}[dt]
        nan = inf | 1
        big = {ri.F32: 0x7F000000, ri.F64: 0x7FE0000000000000, ri.BF16: 0x7F00, ri.F16: 0x7800}[dt]
        sign = 1 << (8 * es - 1)
        specials = [(0, 0), (sign, 0), (0, sign), (one, 0), (0, one), (nan, 0), (inf, 0), (0, nan), (0, inf),
                    (nan, nan), (inf, inf), (inf, inf | sign), (nan, one), (one, nan), (inf, one), (one, inf),
                    (big, big | sign), (1, 0), (0, 1), (1, 2), (two, one), (one, two)]
    else:
        specials = [(0, 0), (1, 0), (0, 1), (3, 1), (1, 3), (2, 1), (200, 100), (100, 200), (4, 2), (6, 3)]
        if dt == ri.I32:
            specials += [(0x7FFFFFFF, 0x80000000), (0x80000000, 0x7FFFFFFF), (0xFFFFFFFF, 1), (1, 0xFFFFFFFF)]
    where = rng.choice(n_el, size=min(n_el // 2, 40 * len(specials)), replace=False)
    for j, q in enumerate(where):
        cv, gv = specials[j % len(specials)]
        c[q], g[q] = pat(cv), pat(gv)
    # a run of equal error ratios (live = 2 * golden exactly where that is representable)
    lo = n_el // 3
    for q in range(lo, min(n_el, lo + 300)):
        if is_float:
            c[q], g[q] = pat(two), pat(one)
        else:
            c[q], g[q] = pat(2), pat(1)
    return g.reshape(-1), c.reshape(-1)


@pytest.mark.parametrize("mode", [ri.TOL, ri.BITWISE])
def test_compare_dense_differences(env, oracle, mode):
    """Every element differs (what a numerically equivalent rewrite looks like), every element type,
    several tiles and a ragged tail per region, regions at 16-byte aligned and at odd offsets."""
    r3, ctx, torch = env
    rng = np.random.default_rng(977 + mode)
    rows, parts, at = [], [], 0
    for rep, (n_bytes, odd) in enumerate([(150000, False), (41000, True), (4096 * 3, False), (120, False)]):
        for dt in (ri.F32, ri.F64, ri.BF16, ri.F16, ri.I32, ri.U8):
            es = ri.ELEM_SIZE[dt]
            n_el = n_bytes // es
            g, c = _dense_case(rng, dt, n_el)
            at = (at + 255) // 256 * 256 + (es if odd else 0)
            rtol, atol = {ri.F32: (1e-6, 1e-8), ri.F64: (1e-15, 0.0), ri.BF16: (1e-2, 1e-3), ri.F16: (1e-3, 1e-4),
                          ri.I32: (1e-9, 1.0), ri.U8: (1e-2, 1.0)}[dt]
            rows.append((at, n_el * es, dt, mode, rtol, atol))
            parts.append((at, g, c))
            at += n_el * es
    arena = (at + 255) // 256 * 256
    gold = rng.integers(0, 256, arena, dtype=np.uint8)
    live = gold.copy()
    for off, g, c in parts:
        gold[off:off + g.size] = g
        live[off:off + c.size] = c
    print("case dense differences mode", mode, "regions", len(rows), "bytes", arena, flush=True)
    exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, gold)
    res, summ = run_compare(r3, ctx, torch, rows, dev(torch, live), dev(torch, gold), arena)
    assert_results_equal(res, exp_res, "dense differences")
    assert summ.tobytes() == exp_sum.tobytes()
    assert int(exp_sum[0]["total_mismatch"]) > 0
    # the same data without the non-finite values: errors stay finite and the maxima are real quotients
    for (off, nb, dt, *_), (_, g, c) in zip(rows, parts):
        es = ri.ELEM_SIZE[dt]
        if dt in (ri.F32, ri.F64, ri.BF16, ri.F16):
            top = {ri.F32: 0x7F, ri.F64: 0x7F, ri.BF16: 0x7F, ri.F16: 0x7C}[dt]
            for buf in (gold, live):
                hi = buf[off + es - 1:off + nb:es]
                bad = (hi & 0x7F) >= (top if dt != ri.F16 else 0x78)
                hi[bad] &= 0xBF
    exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, gold)
    res, summ = run_compare(r3, ctx, torch, rows, dev(torch, live), dev(torch, gold), arena)
    assert_results_equal(res, exp_res, "dense differences, finite")
    assert summ.tobytes() == exp_sum.tobytes()
    assert np.isfinite(exp_res["max_rel_err"]).all()


@pytest.mark.parametrize("atol_on", [False, True])
def test_compare_errors_at_the_tolerance(env, oracle, atol_on):
    """Every element differs and its relative error sits below, at and just above rtol (within a few
    units in the last place of the threshold), so the decision turns on the two roundings of
    atol + rtol * |G|; the first elements of each region stay well inside, the ones past the middle
    straddle the threshold, and one region never leaves the tolerance at all."""
    r3, ctx, torch = env
    rng = np.random.default_rng(31337 + int(atol_on))
    rows, parts, at = [], [], 0
    kinds = [(ri.F64, "<f8", 2.0 ** -20), (ri.F64, "<f8", 1e-9), (ri.F32, "<f4", 1e-3), (ri.F32, "<f4", 2.0 ** -10),
             (ri.BF16, None, 0.05), (ri.F16, "<f2", 0.01), (ri.F64, "<f8", 1e-6)]
    for j, (dt, np_t, rtol) in enumerate(kinds):
        es = ri.ELEM_SIZE[dt]
        n_el = (70000 + 1000 * j) // es * 2
        calm = j == len(kinds) - 1                          # the last region stays inside its tolerance
        G = rng.standard_normal(n_el) * np.exp(rng.uniform(-2, 2, n_el))
        G[G == 0] = 1.0
        f = rng.choice([0.1, 0.5, 0.9], n_el)
        if not calm:
            late = np.arange(n_el) > n_el // 2
            near = rng.choice([1.0 - 2.0 ** -40, 1.0 - 2.0 ** -52, 1.0, 1.0 + 2.0 ** -52, 1.0 + 2.0 ** -40, 1.5], n_el)
            f = np.where(late & (rng.random(n_el) < 0.3), near, f)
        atol = (1e-4 if dt in (ri.BF16, ri.F16) else 1e-9) if atol_on else 0.0
        if np_t == "<f8":
            g = G.astype("<f8")
            # live = golden + (atol + rtol*|golden|) * f, then nudged by -1, 0, +1 pattern steps
            c = g + np.sign(rng.standard_normal(n_el)) * (atol + rtol * np.abs(g)) * f
            c = (c.view(np.int64) + rng.integers(-1, 2, n_el)).view("<f8")
            gb, cb = g.view(np.uint8), np.ascontiguousarray(c).view(np.uint8)
        elif np_t is not None:
            g = G.astype(np_t)
            g64 = g.astype("<f8")
            c = (g64 + np.sign(rng.standard_normal(n_el)) * (atol + rtol * np.abs(g64)) * f).astype(np_t)
            gb, cb = np.ascontiguousarray(g).view(np.uint8), np.ascontiguousarray(c).view(np.uint8)
        else:
            g = ri.f32_to_bf16_bits(G.astype("<f4"))
            g64 = (g.astype(np.uint32) << 16).view("<f4").astype("<f8")
            c64 = g64 + np.sign(rng.standard_normal(n_el)) * (atol + rtol * np.abs(g64)) * f
            c = ri.f32_to_bf16_bits(c64.astype("<f4"))
            gb, cb = np.ascontiguousarray(g).view(np.uint8), np.ascontiguousarray(c).view(np.uint8)
        at = (at + 255) // 256 * 256
        rows.append((at, n_el * es, dt, ri.TOL, rtol, atol))
        parts.append((at, gb.copy(), cb.copy()))
        at += n_el * es
    arena = (at + 255) // 256 * 256
    gold = rng.integers(0, 256, arena, dtype=np.uint8)
    live = gold.copy()
    for off, g, c in parts:
        gold[off:off + g.size] = g
        live[off:off + c.size] = c
    print("case errors at the tolerance, atol", atol_on, "regions", len(rows), "bytes", arena, flush=True)
    exp_res, exp_sum = oracle.compare(oracle.make_table(rows), live, gold)
    res, summ = run_compare(r3, ctx, torch, rows, dev(torch, live), dev(torch, gold), arena)
    assert_results_equal(res, exp_res, "errors at the tolerance")
    assert summ.tobytes() == exp_sum.tobytes()
    counts = exp_res["mismatch_count"]
    assert (counts[:-1] > 0).all() and counts[-1] == 0       # both regimes are in the data
    assert (exp_res["max_rel_err"] > 0).all()
    if not atol_on:
        assert exp_res["max_rel_err"][-1] < 1e-6             # with atol the quotient may pass rtol without a mismatch

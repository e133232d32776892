"""GPU parity of r3_compare_static, the validation entry point that allocates nothing (its partial
results live in a buffer inside the library's device image): every field of its output against
r3_compare on a table of the same regions, and against the CPU oracle, on calls in a row that share
the buffer, the later ones with smaller inputs."""
import numpy as np
import pytest

import r3_inputs as ri

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2604_11109_amd import binding as r3
    assert torch.cuda.is_available(), "these tests need the GPU"
    r3.lib()
    ctx = r3.Context(0)
    yield r3, ctx, torch
    ctx.close()


def host(t):
    return t.cpu().numpy()


def make_case(rng, sizes, dtypes, gap=48):
    """Regions of the given byte sizes and element types, `gap` bytes apart; golden = live with a few
    planted differences per region (bit flips low in the element, plus one NaN in a float region)."""
    rows, at = [], 16
    for sz, dt in zip(sizes, dtypes):
        es = ri.ELEM_SIZE[dt]
        at = (at + es - 1) // es * es
        mode = ri.TOL if dt in (ri.F32, ri.F64, ri.BF16, ri.F16) else ri.BITWISE
        rows.append((at, sz // es * es, dt, mode, 1e-6, 1e-9))
        at += sz // es * es + gap
    arena = (at + 255) // 256 * 256
    live = rng.integers(0, 256, size=arena, dtype=np.uint8)
    # keep floats finite and moderate: clear the top exponent bit of every element's last byte
    for off, nb, dt, _, _, _ in rows:
        es = ri.ELEM_SIZE[dt]
        if dt in (ri.F32, ri.F64, ri.BF16, ri.F16) and nb:
            live[off + es - 1:off + nb:es] &= 0xBF
    gold = live.copy()
    for off, nb, dt, _, _, _ in rows:
        es = ri.ELEM_SIZE[dt]
        n_el = nb // es
        if n_el == 0:
            continue
        for q in rng.choice(n_el, size=min(n_el, 7), replace=False):
            gold[off + q * es + (es - 1) // 2] ^= 0x04
        if dt == ri.F32 and n_el > 3:
            gold[off + 12:off + 16] = np.frombuffer(np.uint32(0x7FC00000).tobytes(), dtype=np.uint8)
    return rows, arena, live, gold


def run_both(r3, ctx, torch, rows, arena, live, gold, oracle):
    d_live = torch.from_numpy(live).to("cuda:0")
    d_gold = torch.from_numpy(gold).to("cuda:0")
    n = len(rows)
    d_out_s = torch.full((40 * n,), 0xEE, dtype=torch.uint8, device="cuda:0")
    d_sum_s = torch.full((40,), 0xEE, dtype=torch.uint8, device="cuda:0")
    r3.r3_compare_static(ctx, rows, arena, d_live, d_gold, d_out_s, d_sum_s)
    torch.cuda.synchronize()
    got = r3.results_to_numpy(d_out_s, n).copy()
    got_sum = r3.summary_to_numpy(d_sum_s).copy()
    tbl = r3.Table(ctx, rows, arena)
    d_out = torch.zeros(40 * n, dtype=torch.uint8, device="cuda:0")
    d_sum = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    r3.r3_compare(ctx, tbl, d_live, d_gold, d_out, d_sum)
    torch.cuda.synchronize()
    assert got.tobytes() == r3.results_to_numpy(d_out, n).tobytes()
    assert got_sum.tobytes() == r3.summary_to_numpy(d_sum).tobytes()
    exp, exp_sum = oracle.compare(oracle.make_table(rows), live, gold)
    assert got.tobytes() == exp.tobytes()
    assert got_sum.tobytes() == exp_sum.tobytes()
    return got


def test_static_compare_matches_table_compare_on_calls_in_a_row(env, oracle):
    r3, ctx, torch = env
    rng = np.random.default_rng(20260411)
    dts = [ri.F32, ri.BF16, ri.F64, ri.I32, ri.U8, ri.F16, ri.F32]
    # first call: 7 regions, ~80 MiB, more than R3_STATIC_MAX_TILES tiles of 4 KiB (tile size grows),
    # one empty region, ragged sizes
    big = [(24 << 20) + 4, (12 << 20) + 2, (32 << 20) + 8, (10 << 20) + 12, (2 << 20) + 3, 0, 70000]
    print("case static compare: large", flush=True)
    got = run_both(r3, ctx, torch, *make_case(rng, big, dts), oracle)
    assert int(got["mismatch_count"].sum()) > 0
    # second call, smaller: 3 regions of a few tiles each; stale partials of the first call lie
    # beyond its tiles in the shared buffer
    print("case static compare: small", flush=True)
    small = [3 * 4096 + 20, 4096, 100]
    run_both(r3, ctx, torch, *make_case(rng, small, [ri.F64, ri.BF16, ri.U8]), oracle)
    # third: one region, self-compare (the summary comes from the finalize launch itself)
    print("case static compare: one clean region", flush=True)
    rows, arena, live, _ = make_case(rng, [1 << 20], [ri.F32])
    got = run_both(r3, ctx, torch, rows, arena, live, live.copy(), oracle)
    assert int(got[0]["mismatch_count"]) == 0 and int(got[0]["first_mismatch"]) == r3.NO_INDEX


def test_static_compare_limits_and_rules(env, oracle):
    r3, ctx, torch = env
    d = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda:0")
    d_out = torch.zeros(40 * 32, dtype=torch.uint8, device="cuda:0")
    many = [(i * 64, 64, ri.U8, ri.BITWISE, 0, 0) for i in range(r3.STATIC_MAX_REGIONS + 1)]
    with pytest.raises(r3.R3Error) as e:
        r3.r3_compare_static(ctx, many, 1 << 16, d, d, d_out)
    assert e.value.status == r3.ENOSPC and "R3_STATIC_MAX_REGIONS" in str(e.value)
    # more bytes than R3_STATIC_MAX_TILES tiles of R3_STATIC_MAX_TILE_BYTES hold (no memory is touched:
    # the call is rejected on the host)
    too_big = r3.STATIC_MAX_TILES * r3.STATIC_MAX_TILE_BYTES + 1
    with pytest.raises(r3.R3Error) as e:
        r3.r3_compare_static(ctx, [(0, too_big, ri.U8, ri.BITWISE, 0, 0)], too_big, d.data_ptr(), d.data_ptr(),
                             d_out)
    assert e.value.status == r3.ENOSPC and "R3_STATIC_MAX_TILES" in str(e.value)
    for rows, arena in [([(0, 64, ri.F32, ri.TOL, -1.0, 0)], 128), ([(2, 64, ri.F32, 0, 0, 0)], 128),
                        ([(0, 256, ri.U8, 0, 0, 0)], 128), ([(0, 64, 9, 0, 0, 0)], 128),
                        ([(0, 64, ri.U8, 0, 0, 0), (32, 64, ri.U8, 0, 0, 0)], 128),
                        ([(0, 64, ri.F32, ri.TOL, float("inf"), 0)], 128)]:
        with pytest.raises(r3.R3Error) as e:
            r3.r3_compare_static(ctx, rows, arena, d, d, d_out)
        assert e.value.status == oracle.validate_table(oracle.make_table(rows), arena), rows
    # still usable after the rejections
    r3.r3_compare_static(ctx, [(0, 4096, ri.U8, ri.BITWISE, 0, 0)], 4096, d, d, d_out)
    torch.cuda.synchronize()
    assert int(r3.results_to_numpy(d_out, 1)[0]["mismatch_count"]) == 0

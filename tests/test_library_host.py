"""CPU-only: the C-ABI library loads, exports every declared symbol, and its host logic
(table rules, workspace sizing) agrees with the oracle's statement of the rules."""
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def r3():
    from paper_2604_11109_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_11109_amd import build
        build.build_lib("libr3.so", verbose=False)
    binding.lib()
    return binding


def test_exports_every_declared_symbol(r3):
    header = open(os.path.join(ROOT, "include", "r3.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(r3_[a-z_0-9]+)\s*\(", header))
    names -= {"r3_launch_fn"}
    assert names == set(r3.DECLARED)
    L = r3.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert L.r3_version() == 1
    assert r3.lib().r3_strerror(r3.EOVERLAP) == b"regions overlap"


def test_struct_layouts_match_header(r3):
    import ctypes
    assert r3.REGION_DTYPE.itemsize == 40 and r3.RESULT_DTYPE.itemsize == 40
    assert r3.SUMMARY_DTYPE.itemsize == 40 and ctypes.sizeof(r3.EvalResult) == 56
    assert r3.REGION_DTYPE.fields["rtol"][1] == 24 and r3.RESULT_DTYPE.fields["checksum"][1] == 32


def test_table_rules_agree_with_oracle(r3, oracle):
    rng = np.random.default_rng(5)
    fixed = [
        ([(0, 64, 1, 1, 1e-5, 1e-7), (64, 64, 2, 0, 0, 0)], 128),
        ([(0, 64, 1, 1, 1e-5, 1e-7), (64, 64, 2, 0, 0, 0)], 127),
        ([(0, 64, 9, 0, 0, 0)], 128), ([(0, 64, 1, 7, 0, 0)], 128),
        ([(0, 64, 1, 1, -1.0, 0)], 128), ([(0, 64, 1, 1, 0, float("nan"))], 128),
        ([(0, 64, 1, 1, float("inf"), 0)], 128), ([(2, 64, 1, 0, 0, 0)], 128),
        ([(4, 12, 2, 0, 0, 0)], 128), ([(2, 6, 4, 0, 0, 0)], 128), ([(3, 5, 0, 0, 0, 0)], 128),
        ([(1 << 63, 1 << 63, 0, 0, 0, 0)], 128), ([(2**64 - 8, 16, 2, 0, 0, 0)], 2**64 - 1),
        ([(0, 64, 1, 0, 0, 0), (60, 8, 1, 0, 0, 0)], 128),
        ([(64, 64, 1, 0, 0, 0), (0, 64, 1, 0, 0, 0)], 128),
        ([(0, 64, 1, 0, 0, 0), (32, 0, 1, 0, 0, 0)], 128),
        ([(0, 64, 1, 0, 0, 0), (32, 64, 1, 0, 0, 0), (2, 4, 1, 0, 0, 0)], 128),
        ([(0, 256, 1, 0, 0, 0), (2, 4, 1, 0, 0, 0)], 128),
    ]
    for rows, arena in fixed:
        assert r3.r3_table_validate(r3.make_table(rows), arena) == oracle.validate_table(
            oracle.make_table(rows), arena), rows
    assert r3.r3_table_validate(None, 10) == oracle.validate_table(None, 10) == r3.EINVAL
    # random tables, many of them broken in one way or another
    seen = set()
    for _ in range(3000):
        n = int(rng.integers(1, 7))
        rows = []
        for _ in range(n):
            dt = int(rng.choice([0, 1, 2, 3, 4, 4, 1, 5]))
            es = {0: 1, 1: 4, 2: 8, 3: 4, 4: 2}.get(dt, 4)
            off = int(rng.integers(0, 40)) * es + int(rng.random() < 0.05)
            nb = int(rng.integers(0, 12)) * es + int(rng.random() < 0.05)
            mode = int(rng.choice([0, 1, 1, 0, 2])) if rng.random() < 0.1 else int(rng.integers(0, 2))
            rtol = float(rng.choice([0.0, 1e-5, -1e-9, np.nan, np.inf])) if rng.random() < 0.1 else 1e-6
            rows.append((off, nb, dt, mode, rtol, 0.0))
        arena = int(rng.integers(16, 400))
        a = r3.r3_table_validate(r3.make_table(rows), arena)
        b = oracle.validate_table(oracle.make_table(rows), arena)
        assert a == b, (rows, arena)
        seen.add(a)
    assert seen == {0, -1, -2, -3, -4}


def test_workspace_sizes(r3):
    rows = r3.make_table([(0, 1 << 20, 1, 0, 0, 0), (1 << 20, 100, 0, 0, 0, 0), (1 << 21, 0, 2, 0, 0, 0)])
    exact = r3.r3_table_workspace_bytes_exact(rows, 1 << 22)
    bound = r3.r3_table_workspace_bytes(3, 1 << 22)
    assert 0 < exact <= bound
    assert r3.r3_table_workspace_bytes_exact(r3.make_table([(2, 4, 1, 0, 0, 0)]), 64) == 0
    # the bound never falls below the exact need, whatever the split of the arena
    rng = np.random.default_rng(6)
    for _ in range(200):
        n = int(rng.integers(1, 50))
        arena = int(rng.integers(1, 1 << 26))
        cuts = np.sort(rng.integers(0, arena + 1, size=2 * n))
        rws = [(int(cuts[2 * i]), int(cuts[2 * i + 1] - cuts[2 * i]), 0, 0, 0, 0) for i in range(n)]
        ex = r3.r3_table_workspace_bytes_exact(r3.make_table(rws), arena)
        assert 0 < ex <= r3.r3_table_workspace_bytes(n, arena)
    with pytest.raises(r3.R3Error):
        r3.r3_tune_tiles(3000, 0)
    r3.r3_tune_tiles(0, 0)


def test_no_gpu_calls_fail_cleanly(r3):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(r3.R3Error) as e:
        r3.Context(0)
    assert e.value.status == r3.EHIP


def test_writeset_regions_agree_with_oracle(r3, oracle):
    rng = np.random.default_rng(8)
    for nbytes, page in [(70 * 4096 + 123, 4096), (4096, 4096), (1, 4096), (64 * 256, 256), (1000 * 512 + 5, 512)]:
        npages = -(-nbytes // page)
        for density in (0.0, 0.02, 0.3, 0.97, 1.0):
            bits = rng.random(npages) < density
            bm = np.zeros(-(-npages // 64), dtype=np.uint64)
            for p in np.flatnonzero(bits):
                bm[p // 64] |= np.uint64(1) << np.uint64(p % 64)
            for want in (1, 0):
                a = r3.r3_writeset_regions(bm, nbytes, page, want)
                b = oracle.writeset_regions(bm, nbytes, page, want)
                assert a.tobytes() == b.tobytes(), (nbytes, page, density, want)
    assert len(r3.r3_writeset_regions(np.zeros(0, np.uint64), 0, 4096, 1)) == 0


def test_replicate_and_timing_agree_with_oracle(r3, oracle):
    rows = [(0, 64, 1, 1, 1e-5, 1e-7), (64, 32, 4, 0, 0, 0), (128, 0, 2, 0, 0, 0)]
    a = r3.r3_table_replicate(r3.make_table(rows), 4096, 5)
    b = oracle.replicate_table(oracle.make_table(rows), 4096, 5)
    assert a.tobytes() == b.tobytes()
    with pytest.raises(r3.R3Error):
        r3.r3_table_replicate(r3.make_table([(2**63, 8, 2, 0, 0, 0)]), 2**63, 3)
    rng = np.random.default_rng(9)
    for n in [0, 1, 2, 3, 4, 7, 10, 33]:
        ms = (rng.random(n) * 3 + 0.1).astype(np.float32)
        for tol in (0.0, 0.05, 0.5):
            t = r3.r3_timing_stats(ms, tol)
            e = oracle.timing_stats(ms, tol)
            assert (t.n, t.stable) == (e["n"], e["stable"])
            got = np.array([t.min, t.median, t.max, t.mad], dtype=np.float32)
            exp = np.array([e["min"], e["median"], e["max"], e["mad"]], dtype=np.float32)
            assert (got == exp).all(), (n, tol, got, exp)
            assert abs(t.mean - e["mean"]) <= 1e-6 * max(1.0, abs(e["mean"]))


def test_bench_refuses_more_than_one_gpu_and_reports_counters_only_for_the_profiled_source(monkeypatch):
    """Host logic of the benchmark driver: a run on several GPUs is refused with a message, and
    the measured HBM traffic is reported only while the kernel source is the profiled one."""
    import importlib
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr)
    sys.path.insert(0, root)
    try:
        bench = importlib.import_module("bench")
    finally:
        sys.path.pop(0)
    monkeypatch.setitem(bench.COUNTERS, "kernels_sha256_16", "0" * 16)
    assert bench.measured_traffic("large_snapshot", "restore") is None
    import hashlib
    src = os.path.join(root, "paper_2604_11109_amd", "csrc", "r3_kernels.hip")
    monkeypatch.setitem(bench.COUNTERS, "kernels_sha256_16", hashlib.sha256(open(src, "rb").read()).hexdigest()[:16])
    got = bench.measured_traffic("large_snapshot", "restore")
    assert isinstance(got, int) and got >= 2 * 32 * (1 << 30)        # at least the algorithmic bytes
    assert bench.measured_traffic("large_snapshot", "no such stage") is None

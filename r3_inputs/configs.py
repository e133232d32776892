"""Seeded synthetic inputs shaped like the replay workloads (recorded kernel states).

This module serves both the CPU oracle's tests and the GPU path's tests/benchmark.  It
holds none of the method's arithmetic (no checksum, no comparison, no copy kernels): it only
lays out arenas, fills them with seeded values and plants known differences.  Everything
is numpy on the host; `large_snapshot_device` is the one generator that fills device
memory directly (torch's seeded generator), for sizes that are impractical to build on
the host.

Element type / mode codes are the interface constants of the region table.
"""
import numpy as np

U8, F32, F64, I32, BF16, F16 = 0, 1, 2, 3, 4, 5
BITWISE, TOL = 0, 1
ELEM_SIZE = {U8: 1, F32: 4, F64: 8, I32: 4, BF16: 2, F16: 2}
SEEDS = {"replay_small": 1001, "jacobi": 1002, "many_regions": 1003, "large_snapshot": 1004,
         "spmv": 1005}


def _align(x, a):
    return (x + a - 1) // a * a


def f32_to_bf16_bits(x):
    """Round-to-nearest-even conversion of float32 values to bfloat16 bit patterns."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------------------
# the small-replay workload: one small snapshot, three fp32 inputs + one fp32 output
# --------------------------------------------------------------------------------------
def replay_small(n=1 << 20, seed=SEEDS["replay_small"], frac=1e-3, scale=1e-3):
    """Three fp32 input regions and one fp32 output region of n elements each.

    The candidate output equals the golden output except that round(frac*n) seeded elements
    (chosen among |g| >= 2^-10 so that the planted error stays above the tolerance) are
    scaled by (1+scale) and every other element is moved by -1, 0 or +1 steps of its fp32
    bit pattern.  Tolerances rtol 1e-5, atol 1e-7.
    """
    rng = np.random.default_rng(seed)
    nb = 4 * n
    offs = [_align(i * nb, 256) for i in range(4)]
    arena_bytes = offs[3] + nb
    prologue = np.zeros(arena_bytes, dtype=np.uint8)
    for i in range(3):
        prologue[offs[i]:offs[i] + nb] = rng.uniform(-1, 1, n).astype("<f4").view(np.uint8)
    golden = rng.uniform(-1, 1, n).astype("<f4")
    epilogue = prologue.copy()
    epilogue[offs[3]:offs[3] + nb] = golden.view(np.uint8)

    n_planted = int(round(frac * n))
    eligible = np.flatnonzero(np.abs(golden) >= 2.0 ** -10)
    planted = np.sort(rng.choice(eligible, size=n_planted, replace=False))
    steps = rng.integers(-1, 2, size=n).astype(np.int64)
    bits = golden.view(np.uint32).astype(np.int64)
    moved = bits + steps
    keep = (bits & 0x7FFFFFFF) == 0                       # leave zeros alone
    moved[keep] = bits[keep]
    cand = moved.astype(np.uint32).view(np.float32).copy()
    cand[planted] = (golden[planted].astype(np.float64) * (1.0 + scale)).astype(np.float32)
    live = np.zeros(arena_bytes, dtype=np.uint8)          # inputs arrive by restore
    live[offs[3]:offs[3] + nb] = cand.view(np.uint8)

    restore_rows = [(offs[i], nb, F32, BITWISE, 0.0, 0.0) for i in range(3)]
    check_rows = [(offs[3], nb, F32, TOL, 1e-5, 1e-7)]
    return {"arena_bytes": arena_bytes, "prologue": prologue, "epilogue": epilogue, "live": live,
            "restore_rows": restore_rows, "check_rows": check_rows, "planted": planted,
            "n_planted": n_planted}


# --------------------------------------------------------------------------------------
# the Jacobi workload: 7-point Jacobi on an N^3 fp64 grid
# --------------------------------------------------------------------------------------
def jacobi(n=256, seed=SEEDS["jacobi"]):
    """Arena = `in` (N^3 fp64; interior uniform[0,1), boundary planes 0) then `out` (zeros)."""
    rng = np.random.default_rng(seed)
    grid = np.zeros((n, n, n), dtype="<f8")
    grid[1:-1, 1:-1, 1:-1] = rng.uniform(0, 1, (n - 2, n - 2, n - 2))
    nb = 8 * n ** 3
    in_off, out_off = 0, _align(nb, 256)
    arena_bytes = out_off + nb
    prologue = np.zeros(arena_bytes, dtype=np.uint8)
    prologue[in_off:in_off + nb] = grid.reshape(-1).view(np.uint8)
    rows_all = [(in_off, nb, F64, BITWISE, 0.0, 0.0), (out_off, nb, F64, TOL, 1e-12, 0.0)]
    return {"n": n, "arena_bytes": arena_bytes, "prologue": prologue, "in_off": in_off,
            "out_off": out_off, "grid_bytes": nb, "restore_rows": rows_all,
            "check_rows": rows_all}


def jacobi_reference(grid):
    """One sweep, same summation order as the recorded kernel (x fastest)."""
    g = grid
    out = np.zeros_like(g)
    c = g[1:-1, 1:-1, 1:-1]
    s = c + g[1:-1, 1:-1, :-2]
    s = s + g[1:-1, 1:-1, 2:]
    s = s + g[1:-1, :-2, 1:-1]
    s = s + g[1:-1, 2:, 1:-1]
    s = s + g[:-2, 1:-1, 1:-1]
    s = s + g[2:, 1:-1, 1:-1]
    out[1:-1, 1:-1, 1:-1] = s * (1.0 / 7.0)
    return out


# Candidate variants of the Jacobi workload: (block, unroll, bug)
JACOBI_VARIANTS = [(64, 1, 0), (128, 1, 0), (256, 1, 0), (512, 1, 0), (1024, 1, 0), (256, 2, 0),
                   (256, 4, 0), (128, 2, 1)]


# --------------------------------------------------------------------------------------
# the many-regions workload: many small regions of mixed element types
# --------------------------------------------------------------------------------------
def many_regions(n_regions=4096, min_bytes=256, max_bytes=1 << 20, seed=SEEDS["many_regions"],
                 align=256, gap_fill=0xA5):
    """Regions with log-uniform sizes, element types drawn uniformly from fp32/fp64/int32/bf16,
    random bytes, packed in table order at `align`-byte aligned offsets (smaller alignments
    than 16 exercise the unaligned paths: offsets stay multiples of the element size)."""
    rng = np.random.default_rng(seed)
    dts = rng.choice([F32, F64, I32, BF16], size=n_regions)
    sizes = np.exp(rng.uniform(np.log(min_bytes), np.log(max_bytes), n_regions)).astype(np.int64)
    rows, at = [], 0
    for dt, sz in zip(dts, sizes):
        es = ELEM_SIZE[int(dt)]
        sz = max(int(sz) // es * es, es)
        a = max(align, es)
        at = _align(at, a)
        rows.append((at, sz, int(dt), BITWISE, 0.0, 0.0))
        at += sz
    arena_bytes = _align(at, 256)
    snapshot = rng.integers(0, 256, size=arena_bytes, dtype=np.uint8)
    live = np.full(arena_bytes, gap_fill, dtype=np.uint8)
    return {"arena_bytes": arena_bytes, "rows": rows, "snapshot": snapshot, "live": live}


# --------------------------------------------------------------------------------------
# the large-snapshot workload: a few very large regions, fp32 and bf16
# --------------------------------------------------------------------------------------
LARGE_TOL = {F32: (1e-5, 1e-7), BF16: (1e-2, 1e-3)}


def large_snapshot_rows(n_regions=16, region_bytes=2 << 30):
    rows = []
    for r in range(n_regions):
        dt = F32 if r < n_regions // 2 else BF16
        rtol, atol = LARGE_TOL[dt]
        rows.append((r * region_bytes, region_bytes, dt, TOL, rtol, atol))
    return rows


def _plant_value(g, dt, sign):
    """A golden value moved by 10x its tolerance, rounded to the element type."""
    rtol, atol = LARGE_TOL[dt]
    v = g + sign * 10.0 * (atol + rtol * np.abs(g))
    return v


def large_snapshot(n_regions=4, region_bytes=1 << 20, seed=SEEDS["large_snapshot"], frac=1e-6,
                   min_planted=3):
    """Host-side version for small sizes: normal(0,1) data, half the regions fp32 and half
    bf16; the golden copy differs from the snapshot in round(frac*n_elem) (at least
    `min_planted`) seeded elements per region, moved by 10x the region's tolerance."""
    rng = np.random.default_rng(seed)
    rows = large_snapshot_rows(n_regions, region_bytes)
    arena_bytes = n_regions * region_bytes
    snapshot = np.zeros(arena_bytes, dtype=np.uint8)
    golden = np.zeros(arena_bytes, dtype=np.uint8)
    planted = []
    for off, nb, dt, _, _, _ in rows:
        n = nb // ELEM_SIZE[dt]
        vals = rng.standard_normal(n).astype(np.float32)
        k = max(int(round(frac * n)), min_planted)
        idx = np.sort(rng.choice(n, size=k, replace=False))
        sign = rng.choice([-1.0, 1.0], size=k)
        if dt == F32:
            snap = vals
            gold = vals.copy()
            gold[idx] = _plant_value(vals[idx].astype(np.float64), dt, sign).astype(np.float32)
            snapshot[off:off + nb] = snap.view(np.uint8)
            golden[off:off + nb] = gold.view(np.uint8)
        else:
            sb = f32_to_bf16_bits(vals)
            gb = sb.copy()
            base = bf16_bits_to_f32(sb[idx]).astype(np.float64)
            gb[idx] = f32_to_bf16_bits(_plant_value(base, dt, sign).astype(np.float32))
            snapshot[off:off + nb] = sb.view(np.uint8)
            golden[off:off + nb] = gb.view(np.uint8)
        planted.append(idx)
    return {"arena_bytes": arena_bytes, "rows": rows, "snapshot": snapshot, "golden": golden,
            "planted": planted}


def large_snapshot_device(n_regions=16, region_bytes=2 << 30, seed=SEEDS["large_snapshot"],
                          frac=1e-6, device="cuda:0", chunk_elems=1 << 28):
    """Device-side version for the full size (32 GiB per arena): fills `snapshot` with
    normal(0,1) values from torch's seeded generator on the device, copies it to `golden`
    and plants the differences there from host-chosen seeded indices.  Returns uint8 device
    tensors; `planted[r]` are the element indices changed in region r."""
    import torch
    rows = large_snapshot_rows(n_regions, region_bytes)
    arena_bytes = n_regions * region_bytes
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    rng = np.random.default_rng(seed)
    snapshot = torch.empty(arena_bytes, dtype=torch.uint8, device=device)
    golden = torch.empty(arena_bytes, dtype=torch.uint8, device=device)
    planted = []
    for off, nb, dt, _, _, _ in rows:
        tdt = torch.float32 if dt == F32 else torch.bfloat16
        n = nb // ELEM_SIZE[dt]
        view = snapshot[off:off + nb].view(tdt)
        for lo in range(0, n, chunk_elems):
            hi = min(n, lo + chunk_elems)
            view[lo:hi] = torch.randn(hi - lo, generator=gen, device=device,
                                      dtype=torch.float32).to(tdt)
        golden[off:off + nb].copy_(snapshot[off:off + nb])
        k = int(round(frac * n))
        idx = np.sort(rng.choice(n, size=k, replace=False))
        sign = rng.choice([-1.0, 1.0], size=k)
        tidx = torch.from_numpy(idx).to(device)
        base = view[tidx].to(torch.float32).cpu().numpy().astype(np.float64)
        moved = _plant_value(base, dt, sign).astype(np.float32)
        if dt == F32:
            new = torch.from_numpy(moved).to(device)
        else:
            new = torch.from_numpy(f32_to_bf16_bits(moved).view(np.int16)).to(device).view(torch.bfloat16)
        golden[off:off + nb].view(tdt)[tidx] = new
        planted.append(idx)
    torch.cuda.synchronize()
    return {"arena_bytes": arena_bytes, "rows": rows, "snapshot": snapshot, "golden": golden,
            "planted": planted}


# --------------------------------------------------------------------------------------
# the SpMV workload: CSR SpMV with a banded pattern
# --------------------------------------------------------------------------------------
def spmv(rows=1 << 21, seed=SEEDS["spmv"]):
    """27 non-zeros per row in 7 bands around centres {0, +-s, +-16s, +-s^2} (s = cube root of
    the row count; 128 for 2^21 rows), each column = (row + centre + jitter) mod rows with
    distinct seeded jitters per band; fp64 values and x in uniform[-1,1); y starts at 0.
    Arena: row_ptr (int32), col_idx (int32), vals (fp64), x (fp64), y (fp64), 4 KiB aligned."""
    rng = np.random.default_rng(seed)
    side = int(round(rows ** (1.0 / 3.0)))
    jw = min(32, max(2, side // 4))                       # jitters in [-jw, jw)
    centres = [0, -side, side, -16 * side, 16 * side, -side * side, side * side]
    cols = []
    r = np.arange(rows, dtype=np.int64)
    for c in centres:
        k = 3 if c == 0 else 4
        # k distinct jitters: sorted draws from a range shortened by k-1, then spread by +i
        draws = np.sort(rng.integers(0, 2 * jw - (k - 1), size=(rows, k)), axis=1) + np.arange(k)
        jit = draws - jw
        if c == 0:
            jit[:, 1] = 0                                 # keep the diagonal
            jit[:, 0] = np.minimum(jit[:, 0], -1)
            jit[:, 2] = np.maximum(jit[:, 2], 1)
        cols.append((r[:, None] + c + jit) % rows)
    col = np.sort(np.concatenate(cols, axis=1), axis=1).astype(np.int32)
    nnz_row = col.shape[1]
    assert nnz_row == 27
    assert (np.diff(col, axis=1) > 0).all(), "duplicate column in a row"
    nnz = rows * nnz_row
    row_ptr = (np.arange(rows + 1, dtype=np.int64) * nnz_row).astype(np.int32)
    vals = rng.uniform(-1, 1, nnz).astype("<f8")
    x = rng.uniform(-1, 1, rows).astype("<f8")
    sizes = [4 * (rows + 1), 4 * nnz, 8 * nnz, 8 * rows, 8 * rows]
    offs, at = [], 0
    for s in sizes:
        at = _align(at, 4096)
        offs.append(at)
        at += s
    arena_bytes = _align(at, 4096)
    prologue = np.zeros(arena_bytes, dtype=np.uint8)
    for off, arr in zip(offs, [row_ptr, col.reshape(-1), vals, x]):
        b = arr.view(np.uint8).reshape(-1)
        prologue[off:off + b.size] = b
    names = ["row_ptr", "col_idx", "vals", "x", "y"]
    dts = [I32, I32, F64, F64, F64]
    rows_all = [(offs[i], sizes[i] // ELEM_SIZE[dts[i]] * ELEM_SIZE[dts[i]], dts[i],
                 TOL if names[i] == "y" else BITWISE, 1e-12 if names[i] == "y" else 0.0, 0.0)
                for i in range(5)]
    return {"rows": rows, "nnz": nnz, "arena_bytes": arena_bytes, "prologue": prologue,
            "offsets": dict(zip(names, offs)), "sizes": dict(zip(names, sizes)),
            "table_rows": rows_all, "y_rows": [rows_all[4]],
            "csr": (row_ptr, col, vals, x)}


# Candidate launch configurations of the SpMV workload: rows per wavefront x block size
SPMV_VARIANTS = [(rpw, blk) for rpw in (1, 2, 4, 8, 16, 32, 64, 128)
                 for blk in (64, 128, 192, 256, 320, 384, 448, 512)]


# --------------------------------------------------------------------------------------
# free-form cases for parity tests
# --------------------------------------------------------------------------------------
def mixed_compare_case(seed, n_regions=24, max_bytes=300000, align=16, specials=True):
    """A table of regions of every element type and both modes, a golden arena and a live
    arena that differs from it by bit-pattern steps, swapped values and special values."""
    rng = np.random.default_rng(seed)
    rows, at = [], 0
    dts = [U8, F32, F64, I32, BF16, F16]
    for r in range(n_regions):
        dt = dts[r % 6] if r < 12 else int(rng.choice(dts))
        es = ELEM_SIZE[dt]
        kind = r % 6
        if kind == 0:
            sz = int(rng.integers(0, 4)) * es                       # empty or a few elements
        elif kind == 1:
            sz = int(rng.integers(1, 40)) * es
        else:
            sz = int(np.exp(rng.uniform(np.log(64), np.log(max_bytes)))) // es * es
        a = max(align, es)
        at = _align(at, a) + (int(rng.integers(0, 3)) * a if r % 4 == 3 else 0)
        mode = TOL if r % 2 else BITWISE
        rtol, atol = [(1e-5, 1e-7), (1e-2, 1e-3), (0.0, 0.0), (1e-12, 0.0)][r % 4]
        rows.append((at, sz, dt, mode, rtol, atol))
        at += sz
    arena_bytes = _align(at + 1, 256)
    golden = np.zeros(arena_bytes, dtype=np.uint8)
    live = np.zeros(arena_bytes, dtype=np.uint8)
    for off, nb, dt, _, _, _ in rows:
        es = ELEM_SIZE[dt]
        n = nb // es
        if n == 0:
            continue
        if dt == F32:
            g = rng.standard_normal(n).astype("<f4").view(np.uint32).astype(np.uint64)
        elif dt == F64:
            g = (rng.standard_normal(n) * np.exp(rng.uniform(-30, 30, n))).astype("<f8").view(np.uint64)
        elif dt == BF16:
            g = f32_to_bf16_bits(rng.standard_normal(n)).astype(np.uint64)
        elif dt == F16:
            g = (rng.standard_normal(n) * np.exp(rng.uniform(-8, 8, n))).astype("<f2").view(np.uint16).astype(np.uint64)
        elif dt == I32:
            g = rng.integers(0, 1 << 32, size=n, dtype=np.uint64)
        else:
            g = rng.integers(0, 256, size=n, dtype=np.uint64)
        c = g.copy()
        npdt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[es]
        style = int(rng.integers(0, 4))
        if style == 0:                                              # a handful of differences
            k = rng.integers(0, n, size=max(1, n // 5000))
            c[k] = c[k] + rng.integers(1, 4, size=k.size).astype(np.uint64)
        elif style == 1:                                            # most elements one step off
            step = rng.integers(-1, 2, size=n)
            c = (c.astype(np.int64) + step).astype(np.uint64)
        elif style == 2:                                            # unrelated values in a block
            lo = int(rng.integers(0, n))
            hi = min(n, lo + int(rng.integers(1, 200)))
            c[lo:hi] = g[rng.integers(0, n, size=hi - lo)]
        # style 3: identical
        if specials and dt in (F32, F64, BF16, F16):
            sp = {F16: [0x0, 0x8000, 0x1, 0x7C00, 0xFC00, 0x7E00, 0x7E01, 0x0400],
                  F32: [0x0, 0x80000000, 0x1, 0x7F800000, 0xFF800000, 0x7FC00000, 0x7FC00001, 0x00800000],
                  BF16: [0x0, 0x8000, 0x1, 0x7F80, 0xFF80, 0x7FC0, 0x7FC1, 0x0080],
                  F64: [0x0, 1 << 63, 0x1, 0x7FF << 52, 0xFFF << 52, (0x7FF << 52) | (1 << 51),
                        0x7FEFFFFFFFFFFFFF, 0xFFEFFFFFFFFFFFFF]}[dt]
            sp = np.array(sp, dtype=np.uint64)
            k = rng.integers(0, n, size=min(n, 6))
            c[k] = sp[rng.integers(0, sp.size, size=k.size)]
            k = rng.integers(0, n, size=min(n, 6))
            g[k] = sp[rng.integers(0, sp.size, size=k.size)]
        mask = (1 << (8 * es)) - 1 if es < 8 else 0xFFFFFFFFFFFFFFFF
        golden[off:off + nb] = (g & np.uint64(mask)).astype(npdt).view(np.uint8)
        live[off:off + nb] = (c & np.uint64(mask)).astype(npdt).view(np.uint8)
    # bytes outside the regions differ on purpose: they must not be looked at
    covered = np.zeros(arena_bytes, dtype=bool)
    for off, nb, *_ in rows:
        covered[off:off + nb] = True
    live[~covered] = 0x3C
    golden[~covered] = 0xC3
    return {"arena_bytes": arena_bytes, "rows": rows, "golden": golden, "live": live}

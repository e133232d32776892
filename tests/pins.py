"""Pins of the CPU oracle: checks that tie it to something other than itself.

Each check takes the oracle module (or a deliberately broken clone of it, see
test_oracle_mutants.py) and raises AssertionError when the oracle disagrees with
 - a brute-force restatement in Python big integers / exact rationals,
 - a library routine (numpy.isclose, bytes comparison),
 - a closed form or invariant of the definition,
 - hand-worked values (tests/golden/*.txt).
"""
import math
import os
import struct
from fractions import Fraction

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
M64 = (1 << 64) - 1
M32 = (1 << 32) - 1


# ----------------------------------------------------------------------------
# checksum
# ----------------------------------------------------------------------------
def phi_len_constants():
    """PHI = floor(2^64 (sqrt5-1)/2), LEN = floor(2^64 frac(sqrt3)) by integer square roots."""
    s5 = math.isqrt(5 << 128)           # floor(2^64 sqrt 5)
    phi = (s5 - (1 << 64)) // 2
    s3 = math.isqrt(3 << 128)           # floor(2^64 sqrt 3), sqrt 3 = 1.732...
    ln = s3 - (1 << 64)
    return phi, ln


def brute_checksum(data, order=None):
    """The checksum definition in Python integers; `order` permutes the word visiting order."""
    phi, ln = phi_len_constants()
    n = len(data)
    words = (n + 7) // 8
    idx = list(range(words)) if order is None else [int(j) for j in order]
    total = 0
    for j in idx:
        w = int.from_bytes(bytes(data[8 * j:8 * j + 8]).ljust(8, b"\0"), "little")
        k = ((j + 1) * phi) & M64
        a = ((w & M32) + (k & M32)) & M32
        b = ((w >> 32) + (k >> 32)) & M32
        total += a * b
    return (total + n * ln) & M64


def check_checksum_constants(api):
    phi, ln = phi_len_constants()
    assert phi == 0x9E3779B97F4A7C15 and ln == 0xBB67AE8584CAA73B
    # one zero word: a = lo(PHI), b = hi(PHI); a closed form of the definition
    assert api.checksum_bytes(bytes(8)) == ((phi & M32) * (phi >> 32) + 8 * ln) & M64
    assert api.checksum_bytes(b"") == 0


def check_checksum_golden(api):
    with open(os.path.join(GOLDEN, "checksum_vectors.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) >= 10
    for name, hexbytes, expect in rows:
        base, _, rep = hexbytes.partition("x")
        data = b"" if hexbytes == "-" else bytes.fromhex(base) * int(rep or 1)
        assert api.checksum_bytes(data) == int(expect, 16), name
        assert brute_checksum(data) == int(expect, 16), name


def check_checksum_bruteforce(api, seed=7):
    rng = np.random.default_rng(seed)
    for n in [1, 2, 3, 7, 8, 9, 15, 16, 17, 31, 63, 64, 65, 255, 1000, 4093, 4096]:
        data = rng.integers(0, 256, size=n, dtype=np.uint8)
        assert api.checksum_bytes(data) == brute_checksum(data.tobytes()), n
    # all-ones words make every 32-bit add wrap
    data = np.full(72, 0xFF, dtype=np.uint8)
    assert api.checksum_bytes(data) == brute_checksum(data.tobytes())


def check_checksum_properties(api, seed=8):
    rng = np.random.default_rng(seed)
    data = rng.integers(0, 256, size=808, dtype=np.uint8)
    ref = api.checksum_bytes(data)
    # order of summation is free
    perm = rng.permutation(101)
    assert brute_checksum(data.tobytes(), perm) == ref
    # position-keyed: swapping two different words changes it
    sw = data.copy()
    sw[0:8], sw[8:16] = data[8:16], data[0:8]
    assert api.checksum_bytes(sw) != ref
    # swapping the halves of one word changes it
    sh = data.copy()
    sh[0:4], sh[4:8] = data[4:8], data[0:4]
    assert api.checksum_bytes(sh) != ref
    # a one-bit flip changes it, at every byte of a short input
    short = rng.integers(0, 256, size=41, dtype=np.uint8)
    base = api.checksum_bytes(short)
    for i in range(short.size):
        f = short.copy()
        f[i] ^= 1 << (i % 8)
        assert api.checksum_bytes(f) != base, i
    # explicit zero padding only moves the length term
    _, ln = phi_len_constants()
    for n in [1, 5, 13, 41]:
        x = short[:n]
        pad = (-n) % 8
        padded = np.concatenate([x, np.zeros(pad, dtype=np.uint8)])
        assert (api.checksum_bytes(padded) - api.checksum_bytes(x)) & M64 == (pad * ln) & M64
    # the tail must not see bytes past n: same prefix, different neighbours
    a = rng.integers(0, 256, size=64, dtype=np.uint8)
    b = a.copy()
    b[21:] ^= 0x5A
    assert api.checksum_bytes(a[:21].copy()) == api.checksum_bytes(b[:21].copy())
    # word sums are additive over a split at a word boundary when indices are kept:
    # cs(x) - n*LEN == sum of per-word terms; compare against brute force per half
    phi, _ = phi_len_constants()
    x = data[:800].tobytes()
    half = sum(
        ((((int.from_bytes(x[8 * j:8 * j + 8], "little") & M32) + (((j + 1) * phi) & M32)) & M32)
         * (((int.from_bytes(x[8 * j:8 * j + 8], "little") >> 32) + ((((j + 1) * phi) & M64) >> 32)) & M32))
        for j in range(50, 100))
    first = (api.checksum_bytes(data[:400].copy()) - 400 * ln) & M64
    assert (first + half + 800 * ln) & M64 == api.checksum_bytes(data[:800].copy())


def check_checksum_table(api, seed=9):
    rng = np.random.default_rng(seed)
    arena = rng.integers(0, 256, size=4096, dtype=np.uint8)
    rows = [(0, 24, api.F64, api.BITWISE, 0, 0), (100, 6, api.BF16, api.BITWISE, 0, 0),
            (256, 0, api.F32, api.BITWISE, 0, 0), (1001, 333, api.U8, api.BITWISE, 0, 0),
            (2048, 2048, api.I32, api.BITWISE, 0, 0)]
    tbl = api.make_table(rows)
    out = api.checksum(tbl, arena)
    for (off, nb, *_), got in zip(rows, out):
        assert int(got) == brute_checksum(arena[off:off + nb].tobytes())


# ----------------------------------------------------------------------------
# compare
# ----------------------------------------------------------------------------
def _decode(dtype_name, raw):
    """(bits, exact value as Fraction or None if non-finite, isfloat) of one element."""
    if dtype_name == "u8":
        return raw[0], Fraction(raw[0]), False
    if dtype_name == "i32":
        v = struct.unpack("<i", raw)[0]
        return struct.unpack("<I", raw)[0], Fraction(v), False
    if dtype_name == "f32":
        bits = struct.unpack("<I", raw)[0]
        v = struct.unpack("<f", raw)[0]
    elif dtype_name == "bf16":
        bits = struct.unpack("<H", raw)[0]
        v = struct.unpack("<f", struct.pack("<I", bits << 16))[0]
    elif dtype_name == "f16":
        bits = struct.unpack("<H", raw)[0]
        v = struct.unpack("<e", raw)[0]          # the struct module's own binary16 decoder
    else:
        bits = struct.unpack("<Q", raw)[0]
        v = struct.unpack("<d", raw)[0]
    if math.isnan(v) or math.isinf(v):
        return bits, None, True
    return bits, Fraction(v), True


def _rn(x):
    """Round an exact rational to binary64, nearest-even, overflow to inf."""
    try:
        return float(x)
    except OverflowError:
        return math.inf if x > 0 else -math.inf


def brute_compare(dtype_name, live, golden, mode_tol, rtol, atol):
    """Element-by-element validation in exact rationals, one rounding per operation."""
    size = {"u8": 1, "i32": 4, "f32": 4, "bf16": 2, "f16": 2, "f64": 8}[dtype_name]
    n = len(live) // size
    count, first, max_abs, max_rel = 0, M64, 0.0, 0.0
    for i in range(n):
        cb, C, isf = _decode(dtype_name, live[i * size:(i + 1) * size])
        gb, G, _ = _decode(dtype_name, golden[i * size:(i + 1) * size])
        if cb == gb:
            d, r, mis = 0.0, 0.0, False
        elif isf and (C is None or G is None):
            d, r, mis = math.inf, math.inf, True
        else:
            d = _rn(abs(C - G))
            if G == 0:
                r = 0.0
            elif math.isinf(d):
                r = math.inf
            else:
                r = _rn(Fraction(d) / abs(G))
            if not mode_tol:
                mis = True
            else:
                t = _rn(Fraction(rtol) * abs(G))
                thr = math.inf if math.isinf(t) else _rn(Fraction(atol) + Fraction(t))
                mis = d > thr
        if mis:
            count += 1
            first = min(first, i)
        max_abs = max(max_abs, d)
        max_rel = max(max_rel, r)
    return count, first, max_abs, max_rel


_DT = {"u8": 0, "f32": 1, "f64": 2, "i32": 3, "bf16": 4, "f16": 5}
_NP = {"u8": np.uint8, "f32": np.uint32, "f64": np.uint64, "i32": np.uint32, "bf16": np.uint16, "f16": np.uint16}


def _bits_equal(a, b):
    return struct.pack("<d", a) == struct.pack("<d", b)


def _run_compare(api, dtype_name, live_bytes, golden_bytes, mode_tol, rtol, atol, pad=0):
    """Call the oracle on a one-region arena (region at offset `pad`)."""
    n = len(live_bytes)
    live = np.zeros(pad + n + 16, dtype=np.uint8)
    gold = np.zeros(pad + n + 16, dtype=np.uint8)
    live[pad:pad + n] = np.frombuffer(live_bytes, dtype=np.uint8)
    gold[pad:pad + n] = np.frombuffer(golden_bytes, dtype=np.uint8)
    # poison what lies outside the region: must not be looked at
    live[:pad] = 0xEE
    live[pad + n:] = 0x11
    tbl = api.make_table([(pad, n, _DT[dtype_name], api.TOL if mode_tol else api.BITWISE, rtol, atol)])
    res, summ = api.compare(tbl, live, gold)
    return res[0], summ[0], live[pad:pad + n]


def _special_bits(dtype_name):
    if dtype_name == "f32":
        return [0x00000000, 0x80000000, 0x00000001, 0x807FFFFF, 0x00800000, 0x7F7FFFFF, 0xFF7FFFFF,
                0x7F800000, 0xFF800000, 0x7FC00000, 0x7FC00001, 0xFFC00000, 0x3F800000, 0x3F800001,
                0xBF800000, 0x322BCC77]
    if dtype_name == "bf16":
        return [0x0000, 0x8000, 0x0001, 0x807F, 0x0080, 0x7F7F, 0xFF7F, 0x7F80, 0xFF80, 0x7FC0,
                0x7FC1, 0x3F80, 0x3F81, 0xBF80, 0x4000]
    if dtype_name == "f16":
        return [0x0000, 0x8000, 0x0001, 0x83FF, 0x0400, 0x7BFF, 0xFBFF, 0x7C00, 0xFC00, 0x7E00,
                0x7E01, 0x3C00, 0x3C01, 0xBC00, 0x4000]
    if dtype_name == "f64":
        return [0x0, 0x8000000000000000, 0x1, 0x800FFFFFFFFFFFFF, 0x0010000000000000,
                0x7FEFFFFFFFFFFFFF, 0xFFEFFFFFFFFFFFFF, 0x7FF0000000000000, 0xFFF0000000000000,
                0x7FF8000000000000, 0x7FF8000000000001, 0x3FF0000000000000, 0x3FF0000000000001,
                0xBFF0000000000000, 0x3E45798EE2308C3A]
    if dtype_name == "i32":
        return [0, 1, 0xFFFFFFFF, 0x7FFFFFFF, 0x80000000, 0x80000001, 12345, 0xFFFFCFC7]
    return [0, 1, 2, 127, 128, 255]


def check_compare_bruteforce(api, seed=11, n=600):
    """Random + special values of every element type against the exact-rational restatement."""
    rng = np.random.default_rng(seed)
    for dtype_name in ["f32", "bf16", "f16", "f64", "i32", "u8"]:
        npdt = np.dtype(_NP[dtype_name])
        sp = np.array(_special_bits(dtype_name), dtype=np.uint64)
        for mode_tol, rtol, atol in [(False, 0.0, 0.0), (True, 1e-5, 1e-7), (True, 0.0, 0.0),
                                     (True, 1e-2, 1e-3), (True, 0.5, 3.0)]:
            if dtype_name in ("f32", "f64", "bf16", "f16"):
                if dtype_name == "f16":
                    g = rng.standard_normal(n).astype("<f2").view(np.uint16)
                elif dtype_name == "f64":
                    g = rng.standard_normal(n).astype("<f8").view(np.uint64)
                elif dtype_name == "f32":
                    g = rng.standard_normal(n).astype("<f4").view(np.uint32)
                else:
                    g = (rng.standard_normal(n).astype("<f4").view(np.uint32) >> 16).astype(np.uint16)
            else:
                g = rng.integers(0, 1 << (8 * npdt.itemsize), size=n, dtype=np.uint64).astype(npdt)
            g = g.astype(npdt)
            c = g.copy()
            # small steps in the bit pattern on a third, unrelated values on some, specials on some
            k = rng.integers(0, n, size=n // 3)
            c[k] = (c[k].astype(np.int64) + rng.integers(-3, 4, size=k.size)).astype(np.uint64).astype(npdt)
            k = rng.integers(0, n, size=n // 10)
            c[k] = g[rng.integers(0, n, size=k.size)]
            k = rng.integers(0, n, size=sp.size * 2)
            c[k] = sp[rng.integers(0, sp.size, size=k.size)].astype(npdt)
            k = rng.integers(0, n, size=sp.size * 2)
            g[k] = sp[rng.integers(0, sp.size, size=k.size)].astype(npdt)
            # every special against every special, in the head of the arrays
            m = sp.size
            pairs = min(m * m, n // 2)
            c[:pairs] = np.repeat(sp, m)[:pairs].astype(npdt)
            g[:pairs] = np.tile(sp, m)[:pairs].astype(npdt)
            lb, gb = c.tobytes(), g.tobytes()
            exp = brute_compare(dtype_name, lb, gb, mode_tol, rtol, atol)
            res, summ, _ = _run_compare(api, dtype_name, lb, gb, mode_tol, rtol, atol, pad=npdt.itemsize * 3)
            tag = (dtype_name, mode_tol, rtol, atol)
            assert int(res["mismatch_count"]) == exp[0], tag
            assert int(res["first_mismatch"]) == exp[1], tag
            assert _bits_equal(float(res["max_abs_err"]), exp[2]), tag
            assert _bits_equal(float(res["max_rel_err"]), exp[3]), tag
            assert int(res["checksum"]) == brute_checksum(lb), tag
            assert int(summ["total_mismatch"]) == exp[0] and int(summ["pass"]) == int(exp[0] == 0)


def check_f16_every_pattern(api):
    """All 65536 binary16 patterns, each as a one-element region against +0: the absolute error is
    the magnitude of the pattern's value, which numpy's float16 gives independently."""
    pats = np.arange(65536, dtype=np.uint16)
    ref = np.abs(pats.view(np.float16).astype(np.float64))
    for lo in range(0, 65536, 4096):
        chunk = pats[lo:lo + 4096]
        live = chunk.view(np.uint8).copy()
        gold = np.zeros_like(live)
        tbl = api.make_table([(2 * i, 2, _DT["f16"], api.BITWISE, 0, 0) for i in range(chunk.size)])
        res, _ = api.compare(tbl, live, gold)
        want = ref[lo:lo + 4096]
        finite = np.isfinite(want)
        got = res["max_abs_err"]
        assert (got[finite].view(np.uint64) == want[finite].view(np.uint64)).all(), lo
        assert np.isinf(got[~finite]).all(), lo
        assert (res["mismatch_count"] == (chunk != 0)).all(), lo


def check_compare_worked_example(api):
    """Hand-worked fp32 table (tests/golden/compare_worked_f32.txt): per-row d, r and verdicts."""
    rows = []
    with open(os.path.join(GOLDEN, "compare_worked_f32.txt")) as f:
        for l in f:
            if l.strip() and not l.startswith("#"):
                i, gbits, cbits, dbits, rbits, tolv, bitv = l.split()
                rows.append((int(gbits, 16), int(cbits, 16), int(dbits, 16), int(rbits, 16),
                             tolv == "M", bitv == "M"))
    rtol, atol = 1e-5, 1e-7
    for gb, cb, db, rb, tol_m, bit_m in rows:
        g = struct.pack("<I", gb)
        c = struct.pack("<I", cb)
        for mode_tol, expect_m in [(True, tol_m), (False, bit_m)]:
            res, _, _ = _run_compare(api, "f32", c, g, mode_tol, rtol, atol)
            assert int(res["mismatch_count"]) == int(expect_m), (hex(gb), hex(cb), mode_tol)
            assert struct.unpack("<Q", struct.pack("<d", float(res["max_abs_err"])))[0] == db
            assert struct.unpack("<Q", struct.pack("<d", float(res["max_rel_err"])))[0] == rb
    # rows 0..6 together, then all rows
    def run(sel):
        g = b"".join(struct.pack("<I", r[0]) for r in sel)
        c = b"".join(struct.pack("<I", r[1]) for r in sel)
        return _run_compare(api, "f32", c, g, True, rtol, atol)[0]
    r = run(rows[:7])
    assert (int(r["mismatch_count"]), int(r["first_mismatch"])) == (2, 3)
    assert float(r["max_abs_err"]).hex() == float.fromhex("0x1.3a8p-12").hex()
    assert struct.pack("<d", float(r["max_rel_err"])) == struct.pack("<Q", 0x3F1A355555555555)
    r = run(rows)
    assert (int(r["mismatch_count"]), int(r["first_mismatch"])) == (4, 3)
    assert math.isinf(float(r["max_abs_err"])) and math.isinf(float(r["max_rel_err"]))


def check_compare_isclose(api, seed=12, n=4000):
    """The tolerance decision equals numpy.isclose for finite fp64 values with distinct bits."""
    rng = np.random.default_rng(seed)
    for rtol, atol in [(1e-5, 1e-8), (1e-12, 0.0), (0.0, 1e-3), (1e-3, 1e-6)]:
        g = rng.standard_normal(n) * np.exp(rng.uniform(-20, 20, n))
        # errors spread around the threshold, on both sides
        c = g + (atol + rtol * np.abs(g)) * rng.uniform(0.0, 2.0, n) * rng.choice([-1.0, 1.0], n)
        keep = c.view(np.uint64) != g.view(np.uint64)
        c, g = c[keep], g[keep]
        close = np.isclose(c, g, rtol=rtol, atol=atol, equal_nan=False)
        assert 0 < close.sum() < close.size
        res, _, _ = _run_compare(api, "f64", c.astype("<f8").tobytes(), g.astype("<f8").tobytes(),
                                 True, rtol, atol)
        assert int(res["mismatch_count"]) == int((~close).sum())
        assert int(res["first_mismatch"]) == (int(np.flatnonzero(~close)[0]) if (~close).any() else M64)
        # one element at a time: the decision itself
        for i in range(0, c.size, 97):
            one, _, _ = _run_compare(api, "f64", c[i:i + 1].astype("<f8").tobytes(),
                                     g[i:i + 1].astype("<f8").tobytes(), True, rtol, atol)
            assert int(one["mismatch_count"]) == int(not close[i])


def check_compare_closed_forms(api, seed=13):
    rng = np.random.default_rng(seed)
    g = rng.uniform(-1, 1, 5000).astype("<f4")
    gb = g.tobytes()
    for mode_tol in (False, True):
        res, summ, _ = _run_compare(api, "f32", gb, gb, mode_tol, 1e-5, 1e-7)
        assert int(res["mismatch_count"]) == 0 and int(res["first_mismatch"]) == M64
        assert struct.pack("<d", float(res["max_abs_err"])) == bytes(8)  # +0.0 exactly
        assert struct.pack("<d", float(res["max_rel_err"])) == bytes(8)
        assert int(summ["pass"]) == 1 and int(summ["first_region"]) == 0xFFFFFFFF
        assert int(summ["first_index"]) == M64
    # one planted perturbation at q: count 1, first q, errors from exact arithmetic
    for q in [0, 1, 2499, 4999]:
        c = g.copy()
        c[q] = np.float32(g[q] * np.float32(1.5) + np.float32(0.25))
        res, _, _ = _run_compare(api, "f32", c.tobytes(), gb, True, 1e-5, 1e-7)
        d = float(abs(Fraction(float(c[q])) - Fraction(float(g[q]))))
        assert int(res["mismatch_count"]) == 1 and int(res["first_mismatch"]) == q
        assert _bits_equal(float(res["max_abs_err"]), d)
        assert _bits_equal(float(res["max_rel_err"]), float(Fraction(d) / abs(Fraction(float(g[q])))))
    # the recorded value is the reference (asymmetric predicate): |c-g| vs rtol*|g|
    g1, c1 = struct.pack("<d", 1.0), struct.pack("<d", 2.0)
    assert int(_run_compare(api, "f64", c1, g1, True, 0.75, 0.0)[0]["mismatch_count"]) == 1
    assert int(_run_compare(api, "f64", g1, c1, True, 0.75, 0.0)[0]["mismatch_count"]) == 0
    # max errors are taken over matching elements too
    res, _, _ = _run_compare(api, "f64", struct.pack("<2d", 1.0, 4.0), struct.pack("<2d", 1.25, 4.0),
                             True, 1.0, 0.0)
    assert int(res["mismatch_count"]) == 0 and float(res["max_abs_err"]) == 0.25
    assert float(res["max_rel_err"]) == 0.2
    # G == 0 contributes to the absolute maximum only
    res, _, _ = _run_compare(api, "f64", struct.pack("<d", 3.0), struct.pack("<d", 0.0), True, 0.0, 5.0)
    assert float(res["max_abs_err"]) == 3.0 and float(res["max_rel_err"]) == 0.0
    assert int(res["mismatch_count"]) == 0
    # integers under tolerance and bitwise
    ci, gi = struct.pack("<3i", 10, -7, 2**31 - 1), struct.pack("<3i", 12, -7, -2**31)
    res, _, _ = _run_compare(api, "i32", ci, gi, True, 0.0, 2.0)
    assert (int(res["mismatch_count"]), int(res["first_mismatch"])) == (1, 2)
    assert float(res["max_abs_err"]) == float(2**32 - 1)
    res, _, _ = _run_compare(api, "i32", ci, gi, False, 0.0, 2.0)
    assert (int(res["mismatch_count"]), int(res["first_mismatch"])) == (2, 0)
    # fp64 overflow of the difference follows the formula literally
    big = struct.pack("<d", 1.7e308)
    neg = struct.pack("<d", -1.7e308)
    res, _, _ = _run_compare(api, "f64", big, neg, True, 1e-3, 0.0)
    assert math.isinf(float(res["max_abs_err"])) and int(res["mismatch_count"]) == 1


def check_compare_unfused(api, seed=14):
    """Find (rtol, atol, G, d) where atol + rtol*|G| rounds differently fused and unfused and d
    lies between the two; the oracle must take the two-rounding branch."""
    rng = np.random.default_rng(seed)
    found = 0
    for _ in range(200000):
        # tolerances of the order of G, so that G + threshold is often exactly representable
        rtol = float(rng.uniform(0.1, 1.0))
        atol = float(rng.uniform(0.1, 1.0))
        G = float(rng.uniform(0.5, 2.0))
        exact = Fraction(atol) + Fraction(rtol) * Fraction(G)
        fused = float(exact)
        unfused = float(Fraction(atol) + Fraction(float(Fraction(rtol) * Fraction(G))))
        if fused == unfused:
            continue
        lo, hi = min(fused, unfused), max(fused, unfused)
        # choose c so that d = |c - G| lands exactly on hi (representable difference needed)
        c = G + hi
        d = float(abs(Fraction(c) - Fraction(G)))
        if not (lo < d <= hi):
            continue
        expect = d > unfused
        if (d > fused) == expect:
            continue
        res, _, _ = _run_compare(api, "f64", struct.pack("<d", c), struct.pack("<d", G), True, rtol, atol)
        assert int(res["mismatch_count"]) == int(expect)
        found += 1
        if found >= 5:
            break
    assert found >= 1, "no fused/unfused witness found"


def check_summary(api):
    res = np.zeros(4, dtype=api.RESULT_DTYPE)
    res["first_mismatch"] = M64
    res[1] = (3, 17, 0.5, 0.25, 1)
    res[3] = (2, 4, 0.125, 2.0, 2)
    s = api.summarize(res)[0]
    assert int(s["total_mismatch"]) == 5 and int(s["first_region"]) == 1 and int(s["first_index"]) == 17
    assert float(s["max_abs_err"]) == 0.5 and float(s["max_rel_err"]) == 2.0 and int(s["pass"]) == 0
    res["mismatch_count"] = 0
    s = api.summarize(res)[0]
    assert int(s["pass"]) == 1 and int(s["first_region"]) == 0xFFFFFFFF and int(s["first_index"]) == M64


# ----------------------------------------------------------------------------
# restore, dirty-diff, table rules, evaluation loop
# ----------------------------------------------------------------------------
def check_restore(api, seed=15):
    rng = np.random.default_rng(seed)
    snap = rng.integers(0, 256, size=5000, dtype=np.uint8)
    rows = [(0, 16, api.F32, 0, 0, 0), (40, 0, api.F64, 0, 0, 0), (64, 1000, api.F64, 0, 0, 0),
            (1071, 77, api.U8, 0, 0, 0), (4000, 998, api.BF16, 0, 0, 0)]
    tbl = api.make_table(rows)
    live = np.full(5000, 0xA5, dtype=np.uint8)
    api.restore(tbl, snap, live)
    covered = np.zeros(5000, dtype=bool)
    for off, nb, *_ in rows:
        covered[off:off + nb] = True
        assert live[off:off + nb].tobytes() == snap[off:off + nb].tobytes()
    assert (live[~covered] == 0xA5).all()            # gaps untouched
    assert covered.sum() == 16 + 1000 + 77 + 998
    # restore then checksum reproduces the recorded checksums
    assert (api.checksum(tbl, live) == api.checksum(tbl, snap)).all()
    assert (snap == rng.integers(0, 1, 1)).sum() >= 0   # snapshot is read-only: unchanged below
    snap2 = np.random.default_rng(seed).integers(0, 256, size=5000, dtype=np.uint8)
    assert (snap == snap2).all()


def check_dirty_diff(api, seed=16):
    rng = np.random.default_rng(seed)
    P = 4096
    n = 70 * P + 123          # 71 pages, last one partial; two bitmap words
    pre = rng.integers(0, 256, size=n, dtype=np.uint8)
    bm, cnt = api.dirty_diff(pre, pre.copy(), P)
    assert bm.size == 2 and cnt == 0 and not bm.any()
    cases = {0: [0], P - 1: [0], P: [1], 63 * P + 5: [63], 64 * P: [64], n - 1: [70],
             70 * P: [70]}
    for byte, pages in cases.items():
        post = pre.copy()
        post[byte] ^= 0x80
        bm, cnt = api.dirty_diff(pre, post, P)
        want = [0, 0]
        for p in pages:
            want[p // 64] |= 1 << (p % 64)
        assert [int(x) for x in bm] == want and cnt == len(pages), byte
    post = pre.copy()
    idx = rng.choice(n, size=40, replace=False)
    post[idx] ^= 1
    bm, cnt = api.dirty_diff(pre, post, P)
    pages = sorted(set(int(i) // P for i in idx))
    want = [0, 0]
    for p in pages:
        want[p // 64] |= 1 << (p % 64)
    assert [int(x) for x in bm] == want and cnt == len(pages)
    # other page sizes, exact multiple, tiny inputs
    bm, cnt = api.dirty_diff(pre[:1024].copy(), post[:1024].copy(), 256)
    pages = sorted(set(int(i) // 256 for i in idx if i < 1024))
    assert cnt == len(pages) and bm.size == 1
    bm, cnt = api.dirty_diff(np.zeros(0, np.uint8), np.zeros(0, np.uint8), P)
    assert bm.size == 0 and cnt == 0
    one_a, one_b = np.array([1], np.uint8), np.array([2], np.uint8)
    bm, cnt = api.dirty_diff(one_a, one_b, P)
    assert [int(x) for x in bm] == [1] and cnt == 1


def check_table_rules(api):
    R = api.make_table
    ok = [(0, 64, api.F32, api.TOL, 1e-5, 1e-7), (64, 64, api.F64, api.BITWISE, 0, 0)]
    assert api.validate_table(R(ok), 128) == api.OK
    assert api.validate_table(None, 128) == api.EINVAL
    assert api.validate_table(R(ok), 127) == api.ERANGE
    assert api.validate_table(R([(0, 64, 9, 0, 0, 0)]), 128) == api.EINVAL
    assert api.validate_table(R([(0, 64, api.F32, 7, 0, 0)]), 128) == api.EINVAL
    assert api.validate_table(R([(0, 64, api.F32, 1, -1.0, 0)]), 128) == api.EINVAL
    assert api.validate_table(R([(0, 64, api.F32, 1, 0, float("nan"))]), 128) == api.EINVAL
    assert api.validate_table(R([(0, 64, api.F32, 1, float("inf"), 0)]), 128) == api.EINVAL
    assert api.validate_table(R([(2, 64, api.F32, 0, 0, 0)]), 128) == api.EALIGN
    assert api.validate_table(R([(0, 62, api.F32, 0, 0, 0)]), 128) == api.EALIGN
    assert api.validate_table(R([(4, 12, api.F64, 0, 0, 0)]), 128) == api.EALIGN
    assert api.validate_table(R([(2, 6, api.BF16, 0, 0, 0)]), 128) == api.OK
    assert api.validate_table(R([(3, 5, api.U8, 0, 0, 0)]), 128) == api.OK
    assert api.validate_table(R([(1 << 63, 1 << 63, api.U8, 0, 0, 0)]), 128) == api.ERANGE
    assert api.validate_table(R([(2**64 - 8, 16, api.F64, 0, 0, 0)]), 2**64 - 1) == api.ERANGE
    assert api.validate_table(R([(0, 64, api.F32, 0, 0, 0), (60, 8, api.F32, 0, 0, 0)]), 128) == api.EOVERLAP
    assert api.validate_table(R([(64, 64, api.F32, 0, 0, 0), (0, 128, api.F32, 0, 0, 0)]), 128) == api.EOVERLAP
    assert api.validate_table(R([(0, 64, api.F32, 0, 0, 0), (64, 64, api.F32, 0, 0, 0)]), 128) == api.OK
    assert api.validate_table(R([(64, 64, api.F32, 0, 0, 0), (0, 64, api.F32, 0, 0, 0)]), 128) == api.OK
    # empty regions overlap nothing, even inside another region
    assert api.validate_table(R([(0, 64, api.F32, 0, 0, 0), (32, 0, api.F32, 0, 0, 0)]), 128) == api.OK
    # first violation in table order decides; overlap comes last
    assert api.validate_table(R([(0, 64, api.F32, 0, 0, 0), (32, 64, api.F32, 0, 0, 0),
                                 (2, 4, api.F32, 0, 0, 0)]), 128) == api.EALIGN
    assert api.validate_table(R([(0, 256, api.F32, 0, 0, 0), (2, 4, api.F32, 0, 0, 0)]), 128) == api.ERANGE
    assert api.validate_table(R([(2, 256, api.F32, 0, 0, 0)]), 128) == api.EALIGN
    assert api.validate_table(R([(2, 256, 77, 0, 0, 0)]), 128) == api.EINVAL


def check_eval_loop(api, seed=17):
    rng = np.random.default_rng(seed)
    n = 1024
    pro = rng.integers(0, 256, size=n, dtype=np.uint8)
    # the recorded kernel: out[i] = in[i] + 1 on the second half (uint8 wrap)
    def good(live):
        live[512:] = live[:512] + 1
    epi = pro.copy()
    good(epi)
    rtbl = api.make_table([(0, n, api.U8, 0, 0, 0)])
    ctbl = api.make_table([(0, 512, api.U8, 0, 0, 0), (512, 512, api.U8, 0, 0, 0)])
    live = np.zeros(n, np.uint8)
    out = api.eval_candidate(rtbl, pro, ctbl, epi, live, good, warmup=1, reps=3)
    assert out["pass"] == 1 and out["total_mismatch"] == 0 and out["candidate_status"] == 0
    assert (out["regions"]["checksum"] == api.checksum(ctbl, epi)).all()
    # an in-place candidate needs the prologue each replay: without restore it would drift
    def inplace(live):
        live[:512] += 1
        live[512:] = live[:512]
    epi2 = pro.copy()
    inplace(epi2)
    out = api.eval_candidate(rtbl, pro, ctbl, epi2, live, inplace, warmup=2, reps=2)
    assert out["pass"] == 1
    # a candidate that is wrong on the second replay only
    calls = {"k": 0}
    def flaky(live):
        good(live)
        if calls["k"] == 1:
            live[600] ^= 1
            live[700] ^= 1
        calls["k"] += 1
    for policy, want_total, want_pass in [(api.EVERY, 2, 0), (api.FIRST, 0, 1), (api.LAST, 0, 1)]:
        calls["k"] = 0
        out = api.eval_candidate(rtbl, pro, ctbl, epi, live, flaky, warmup=0, reps=3, policy=policy)
        assert (out["total_mismatch"], out["pass"]) == (want_total, want_pass), policy
        # region results are those of the last validated replay (clean here)
        assert int(out["regions"]["mismatch_count"].sum()) == 0
    # wrong on the last replay: reported index is region-relative in the first bad region
    calls["k"] = -1
    def bad_last(live):
        good(live)
        calls["k"] += 1
        if calls["k"] == 2:
            live[512 + 77] ^= 4
    out = api.eval_candidate(rtbl, pro, ctbl, epi, live, bad_last, warmup=1, reps=2, policy=api.LAST)
    assert (out["pass"], out["first_region"], out["first_index"]) == (0, 1, 77)
    # a failing launch rejects the candidate
    out = api.eval_candidate(rtbl, pro, ctbl, epi, live, lambda l: 5, warmup=0, reps=2)
    assert out["pass"] == 0 and out["candidate_status"] == 5
    # no candidate: the restored state validates against the prologue itself
    out = api.eval_candidate(rtbl, pro, rtbl, pro, live, None)
    assert out["pass"] == 1 and (out["regions"]["checksum"] == api.checksum(rtbl, pro)).all()


def check_record(api, seed=18):
    rng = np.random.default_rng(seed)
    n = 3 * 4096 + 100
    live = rng.integers(0, 256, size=n, dtype=np.uint8)
    before = live.copy()
    def kernel(a):
        a[4096 + 5] ^= 0xFF
        a[n - 1] ^= 0x01
    tbl = api.make_table([(0, 4096, api.U8, 0, 0, 0), (4096, n - 4096, api.U8, 0, 0, 0)])
    rec = api.record(tbl, live, kernel)
    assert (rec["prologue"] == before).all() and (rec["epilogue"] == live).all()
    assert [int(x) for x in rec["bitmap"]] == [0b1010] and rec["dirty_count"] == 2
    assert int(rec["pro_cs"][0]) == int(rec["epi_cs"][0]) and int(rec["pro_cs"][1]) != int(rec["epi_cs"][1])
    assert int(rec["epi_cs"][1]) == brute_checksum(live[4096:].tobytes())


def check_writeset_regions(api, seed=19):
    rng = np.random.default_rng(seed)
    for nbytes, page in [(70 * 4096 + 123, 4096), (4096, 4096), (1, 4096), (64 * 256, 256), (129 * 512 + 511, 512)]:
        npages = -(-nbytes // page)
        for density in (0.0, 0.05, 0.5, 1.0):
            bits = rng.random(npages) < density
            bm = np.zeros(-(-npages // 64), dtype=np.uint64)
            for p in np.flatnonzero(bits):
                bm[p // 64] |= np.uint64(1) << np.uint64(p % 64)
            for want in (1, 0):
                t = api.writeset_regions(bm, nbytes, page, want)
                # brute force: a byte is covered iff its page has the wanted state
                covered = np.zeros(nbytes, dtype=np.int32)
                for r in t:
                    assert int(r["bytes"]) > 0 and int(r["dtype"]) == api.U8 and int(r["mode"]) == api.BITWISE
                    covered[int(r["offset"]):int(r["offset"]) + int(r["bytes"])] += 1
                wanted = np.repeat(bits == bool(want), page)[:nbytes]
                assert (covered == wanted.astype(np.int32)).all()
                # maximal runs in address order: consecutive regions never touch
                ends = t["offset"] + t["bytes"]
                assert (t["offset"][1:] > ends[:-1]).all() if len(t) > 1 else True
                assert api.validate_table(t, nbytes) == (api.OK if len(t) else api.EINVAL)
    assert len(api.writeset_regions(np.zeros(0, np.uint64), 0, 4096, 1)) == 0


def check_eval_guard(api, seed=20):
    rng = np.random.default_rng(seed)
    P = 256
    n = 16 * P
    pro = rng.integers(0, 256, size=n, dtype=np.uint8)
    def kernel(live):                      # writes pages 3 and 9..10 only
        live[3 * P + 7] ^= 0x11
        live[9 * P:11 * P] = live[0:2 * P] + 1
    rec_live = pro.copy()
    full = api.make_table([(0, n, api.U8, api.BITWISE, 0, 0)])
    rec = api.record(full, rec_live, kernel, page_bytes=P)
    assert [int(x) for x in rec["bitmap"]] == [(1 << 3) | (1 << 9) | (1 << 10)] and rec["dirty_count"] == 3
    dirty = api.writeset_regions(rec["bitmap"], n, P, 1)
    clean = api.writeset_regions(rec["bitmap"], n, P, 0)
    assert [(int(r["offset"]), int(r["bytes"])) for r in dirty] == [(3 * P, P), (9 * P, 2 * P)]
    assert [(int(r["offset"]), int(r["bytes"])) for r in clean] == [(0, 3 * P), (4 * P, 5 * P), (11 * P, 5 * P)]
    expected = api.checksum(clean, rec["prologue"])
    assert (expected == api.checksum(clean, rec["epilogue"])).all()
    live = pro.copy()
    # a well-behaved candidate: write-set restore is enough, guard stays quiet
    out = api.eval_candidate(dirty, rec["prologue"], dirty, rec["epilogue"], live, kernel, 1, 3,
                             guard_tbl=clean, guard_expected=expected, guard_every=2, heal_tbl=full)
    assert out["pass"] == 1 and out["guard"] == {"checks": 2, "failed_checks": 0, "changed_regions": 0,
                                                  "first_region": api.NO_REGION, "healed": 0}
    # a candidate with a stray write outside the write-set on its second replay: the validated
    # regions still match, only the guard can tell; healing puts the recorded state back
    calls = {"k": 0}
    def stray(live):
        kernel(live)
        if calls["k"] >= 1:
            live[12 * P + 1] = (int(pro[12 * P + 1]) + 1) & 0xFF
        calls["k"] += 1
    out = api.eval_candidate(dirty, rec["prologue"], dirty, rec["epilogue"], live, stray, 0, 4,
                             guard_tbl=clean, guard_expected=expected, guard_every=1, heal_tbl=full)
    assert out["total_mismatch"] == 0 and out["pass"] == 0
    assert out["guard"] == {"checks": 4, "failed_checks": 3, "changed_regions": 1, "first_region": 2, "healed": 1}
    assert (live == rec["prologue"]).all()
    # without healing the damage stays
    calls["k"] = 0
    live2 = pro.copy()
    out = api.eval_candidate(dirty, rec["prologue"], dirty, rec["epilogue"], live2, stray, 0, 2,
                             guard_tbl=clean, guard_expected=expected, guard_every=0)
    assert out["guard"]["checks"] == 1 and out["guard"]["failed_checks"] == 1 and out["guard"]["healed"] == 0
    assert live2[12 * P + 1] != pro[12 * P + 1]


def check_instances(api, seed=21):
    rng = np.random.default_rng(seed)
    n, k, stride = 512, 3, 1024            # three recorded instances, 1 KiB apart
    pro = rng.integers(0, 256, size=k * stride, dtype=np.uint8)
    def kernel(view, i):                   # out = in + 1 (second half of each instance)
        view[256:512] = view[0:256] + 1
        return 0
    epi = pro.copy()
    for i in range(k):
        kernel(epi[i * stride:], i)
    one = api.make_table([(0, 256, api.U8, 0, 0, 0), (256, 256, api.U8, 0, 0, 0)])
    rep = api.replicate_table(one, stride, k)
    assert [(int(r["offset"]), int(r["bytes"])) for r in rep] == [
        (0, 256), (256, 256), (1024, 256), (1280, 256), (2048, 256), (2304, 256)]
    assert api.validate_table(rep, k * stride) == api.OK
    live = np.zeros(k * stride, np.uint8)
    out = api.eval_candidate_instances(rep, pro, rep, epi, live, kernel, k, stride, 1, 2)
    assert out["pass"] == 1 and list(out["instance_pass"]) == [1, 1, 1]
    # a candidate that is right on the recording used during the search and wrong on another
    def partial(view, i):
        kernel(view, i)
        if i == 2:
            view[300] ^= 8
        return 0
    out = api.eval_candidate_instances(rep, pro, rep, epi, live, partial, k, stride, 0, 2)
    assert out["pass"] == 0 and list(out["instance_pass"]) == [1, 1, 0]
    assert out["total_mismatch"] == 1 and out["first_region"] == 5 and out["first_index"] == 300 - 256
    # bytes between the instances are never touched
    assert (live[512:1024] == 0).all() and (live[1536:2048] == 0).all()


def check_timing_stats(api):
    t = api.timing_stats([3.0, 1.0, 2.0, 10.0, 2.5], 0.5)
    assert (t["n"], t["min"], t["median"], t["max"]) == (5, 1.0, 2.5, 10.0) and abs(t["mean"] - 3.7) < 1e-6
    assert t["mad"] == 0.5 and t["stable"] == 1          # |x - 2.5| = .5 1.5 .5 7.5 0 -> median .5
    assert api.timing_stats([3.0, 1.0, 2.0, 10.0, 2.5], 0.1)["stable"] == 0
    t = api.timing_stats([4.0, 2.0], 0.0)
    assert t["median"] == 3.0 and t["mad"] == 1.0 and t["stable"] == 0
    assert api.timing_stats([7.0], 0.0)["stable"] == 1 and api.timing_stats([], 1.0)["n"] == 0


ALL_CHECKS = [
    check_checksum_constants, check_checksum_golden, check_checksum_bruteforce,
    check_checksum_properties, check_checksum_table, check_compare_bruteforce,
    check_f16_every_pattern, check_compare_worked_example, check_compare_isclose, check_compare_closed_forms,
    check_compare_unfused, check_summary, check_restore, check_dirty_diff, check_table_rules,
    check_eval_loop, check_record, check_writeset_regions, check_eval_guard,
    check_instances, check_timing_stats,
]

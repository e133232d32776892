"""ctypes front end of the CPU oracle (oracle/r3_oracle.c).  TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.
It imports nothing from the GPU package.  Arenas are numpy uint8 arrays; tables
are numpy structured arrays of REGION_DTYPE.

The evaluation loop (Sections V-B and V-C of the paper: restore the prologue,
run the candidate, compare with the epilogue) is composed here from the C
functions, one replay at a time.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "r3_oracle.c")
_LIB = os.path.join(_HERE, "libr3_oracle.so")

# status codes, element types, modes, policies (interface constants)
OK, EINVAL, EALIGN, ERANGE, EOVERLAP = 0, -1, -2, -3, -4
U8, F32, F64, I32, BF16, F16 = 0, 1, 2, 3, 4, 5
BITWISE, TOL = 0, 1
EVERY, FIRST, LAST = 0, 1, 2
NO_INDEX = 0xFFFFFFFFFFFFFFFF
NO_REGION = 0xFFFFFFFF
ELEM_SIZE = {U8: 1, F32: 4, F64: 8, I32: 4, BF16: 2, F16: 2}

REGION_DTYPE = np.dtype(
    [("offset", "<u8"), ("bytes", "<u8"), ("dtype", "<u4"), ("mode", "<u4"),
     ("rtol", "<f8"), ("atol", "<f8")], align=True)
RESULT_DTYPE = np.dtype(
    [("mismatch_count", "<u8"), ("first_mismatch", "<u8"), ("max_abs_err", "<f8"),
     ("max_rel_err", "<f8"), ("checksum", "<u8")], align=True)
SUMMARY_DTYPE = np.dtype(
    [("total_mismatch", "<u8"), ("first_index", "<u8"), ("first_region", "<u4"),
     ("pass", "<u4"), ("max_abs_err", "<f8"), ("max_rel_err", "<f8")], align=True)
assert REGION_DTYPE.itemsize == 40 and RESULT_DTYPE.itemsize == 40 and SUMMARY_DTYPE.itemsize == 40

CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-Wall"]


def build(force=False):
    """Compile the oracle with gcc (host only)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc"] + CFLAGS + [_SRC, "-o", tmp, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        vp, u32, u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
        L.r3o_validate_table.argtypes = [vp, u32, u64]
        L.r3o_validate_table.restype = ctypes.c_int
        L.r3o_restore.argtypes = [vp, u32, vp, vp]
        L.r3o_restore.restype = None
        L.r3o_checksum_bytes.argtypes = [vp, u64]
        L.r3o_checksum_bytes.restype = u64
        L.r3o_checksum_table.argtypes = [vp, u32, vp, vp]
        L.r3o_checksum_table.restype = None
        L.r3o_compare_region.argtypes = [vp, vp, vp, vp]
        L.r3o_compare_region.restype = None
        L.r3o_compare_table.argtypes = [vp, u32, vp, vp, vp]
        L.r3o_compare_table.restype = None
        L.r3o_summarize.argtypes = [vp, u32, vp]
        L.r3o_summarize.restype = None
        L.r3o_dirty_diff.argtypes = [vp, vp, u64, u64, vp, vp]
        L.r3o_dirty_diff.restype = None
        _lib = L
    return _lib


def _u8(a):
    a = np.asarray(a)
    if a.dtype != np.uint8 or not a.flags.c_contiguous:
        raise TypeError("arena must be a contiguous uint8 array")
    return a


def _tbl(t):
    t = np.ascontiguousarray(t, dtype=REGION_DTYPE)
    return t


def make_table(rows):
    """rows: iterable of (offset, bytes, dtype, mode, rtol, atol)."""
    rows = list(rows)
    t = np.zeros(len(rows), dtype=REGION_DTYPE)
    for i, r in enumerate(rows):
        t[i] = tuple(r)
    return t


def validate_table(tbl, arena_bytes):
    if tbl is None or len(tbl) == 0:
        return lib().r3o_validate_table(None, 0, arena_bytes)
    t = _tbl(tbl)
    return lib().r3o_validate_table(t.ctypes.data, len(t), arena_bytes)


def _check(tbl, *arenas):
    t = _tbl(tbl)
    n = min(a.size for a in arenas)
    rc = lib().r3o_validate_table(t.ctypes.data, len(t), n)
    if rc != OK:
        raise ValueError("invalid region table: status %d" % rc)
    return t


def restore(tbl, snapshot, live):
    snapshot, live = _u8(snapshot), _u8(live)
    t = _check(tbl, snapshot, live)
    lib().r3o_restore(t.ctypes.data, len(t), snapshot.ctypes.data, live.ctypes.data)


def checksum_bytes(buf):
    b = _u8(np.frombuffer(bytes(buf), dtype=np.uint8)) if not isinstance(buf, np.ndarray) else _u8(buf)
    return int(lib().r3o_checksum_bytes(b.ctypes.data if b.size else None, b.size))


def checksum(tbl, arena):
    arena = _u8(arena)
    t = _check(tbl, arena)
    out = np.zeros(len(t), dtype=np.uint64)
    lib().r3o_checksum_table(t.ctypes.data, len(t), arena.ctypes.data, out.ctypes.data)
    return out


def compare(tbl, live, golden):
    """Returns (per-region RESULT_DTYPE array, SUMMARY_DTYPE scalar array of length 1)."""
    live, golden = _u8(live), _u8(golden)
    t = _check(tbl, live, golden)
    res = np.zeros(len(t), dtype=RESULT_DTYPE)
    lib().r3o_compare_table(t.ctypes.data, len(t), live.ctypes.data, golden.ctypes.data,
                            res.ctypes.data)
    return res, summarize(res)


def summarize(res):
    res = np.ascontiguousarray(res, dtype=RESULT_DTYPE)
    s = np.zeros(1, dtype=SUMMARY_DTYPE)
    lib().r3o_summarize(res.ctypes.data, len(res), s.ctypes.data)
    return s


def dirty_diff(pre, post, page_bytes=4096):
    """Returns (bitmap uint64 array, dirty page count)."""
    pre, post = _u8(pre), _u8(post)
    if pre.size != post.size:
        raise ValueError("states differ in size")
    if page_bytes < 1:
        raise ValueError("page_bytes")
    n = pre.size
    npages = -(-n // page_bytes)
    bitmap = np.zeros(-(-npages // 64), dtype=np.uint64)
    count = ctypes.c_uint64(0)
    lib().r3o_dirty_diff(pre.ctypes.data, post.ctypes.data, n, page_bytes,
                         bitmap.ctypes.data if bitmap.size else None, ctypes.byref(count))
    return bitmap, int(count.value)


def writeset_regions(bitmap, nbytes, page_bytes, want_dirty):
    """Maximal runs of dirty (or clean) pages of a write-set bitmap as byte regions
    (offset, bytes, U8, BITWISE), the last one clipped to nbytes.  One page at a time."""
    npages = -(-nbytes // page_bytes)
    rows, start = [], None
    for p in range(npages):
        dirty = (int(bitmap[p // 64]) >> (p % 64)) & 1
        want = bool(dirty) == bool(want_dirty)
        if want and start is None:
            start = p
        elif not want and start is not None:
            rows.append((start * page_bytes, p * page_bytes - start * page_bytes, U8, BITWISE, 0.0, 0.0))
            start = None
    if start is not None:
        rows.append((start * page_bytes, nbytes - start * page_bytes, U8, BITWISE, 0.0, 0.0))
    return make_table(rows)


def replicate_table(tbl, instance_stride, instances):
    """`instances` copies of a table, copy i shifted by i*instance_stride (several recorded
    instances of one kernel laid out back to back, Section V-C)."""
    t = _tbl(tbl)
    rows = []
    for i in range(instances):
        for r in t:
            rows.append((int(r["offset"]) + i * instance_stride, int(r["bytes"]), int(r["dtype"]),
                         int(r["mode"]), float(r["rtol"]), float(r["atol"])))
    return make_table(rows)


def eval_candidate_instances(restore_tbl, prologues, check_tbl, epilogues, live, launch, instances,
                             instance_stride, warmup=0, reps=1, policy=EVERY):
    """eval_candidate over several recorded instances: launch(view, i) runs the candidate on
    instance i's part of the live super arena.  Adds instance_pass (last validated replay)."""
    def all_instances(arena):
        for i in range(instances):
            rc = launch(arena[i * instance_stride:], i)
            if rc:
                return rc
        return 0
    out = eval_candidate(restore_tbl, prologues, check_tbl, epilogues, live, all_instances, warmup, reps, policy)
    per = len(check_tbl) // instances
    flags = np.zeros(instances, dtype=np.uint8)
    if out["regions"] is not None:
        for i in range(instances):
            flags[i] = int(out["candidate_status"] == 0
                           and (out["regions"]["mismatch_count"][i * per:(i + 1) * per] == 0).all())
    out["instance_pass"] = flags
    return out


def timing_stats(ms, rel_noise):
    """min, median, max, mean, median absolute deviation and the stability flag of a set of
    replay times (plain definitions)."""
    x = np.sort(np.asarray(ms, dtype=np.float32))
    if x.size == 0:
        return {"n": 0, "stable": 0, "min": 0.0, "median": 0.0, "max": 0.0, "mean": 0.0, "mad": 0.0}
    med = np.float32(np.median(x))
    mad = np.float32(np.median(np.abs(x - med)))
    return {"n": int(x.size), "stable": int(med > 0 and mad <= np.float32(rel_noise) * med),
            "min": float(x[0]), "median": float(med), "max": float(x[-1]),
            "mean": float(np.float32(x.astype(np.float64).sum() / x.size)), "mad": float(mad)}


def record(tbl, live, launch, page_bytes=4096):
    """Section V-A: keep the state before and after one run of the recorded kernel.

    launch(live) mutates the uint8 arena in place.  Returns a dict with the two
    snapshots (whole arena), the page write-set and the per-region checksums.
    """
    live = _u8(live)
    prologue = live.copy()
    launch(live)
    epilogue = live.copy()
    bitmap, count = dirty_diff(prologue, epilogue, page_bytes)
    return {"prologue": prologue, "epilogue": epilogue, "bitmap": bitmap, "dirty_count": count,
            "pro_cs": checksum(tbl, prologue), "epi_cs": checksum(tbl, epilogue)}


def eval_candidate(restore_tbl, prologue, check_tbl, epilogue, live, launch, warmup=0, reps=1,
                   policy=EVERY, guard_tbl=None, guard_expected=None, guard_every=0, heal_tbl=None):
    """Sections V-B/V-C: for every replay restore, run, validate per `policy`.

    launch(live) mutates the arena in place and may return a non-zero status
    (failure: the loop stops and the candidate is rejected).  Returns a dict:
    regions = results of the last validated replay, total_mismatch = max over the
    validated replays, first_region/first_index/max errors = last validated replay.
    """
    total = warmup + reps
    if reps < 1 or total < 1:
        raise ValueError("reps")
    regions, last, worst, status = None, None, 0, 0
    g_checks = g_failed = g_changed = 0
    g_first = NO_REGION
    for rep in range(total):
        restore(restore_tbl, prologue, live)
        if launch is not None:
            rc = launch(live)
            if rc:
                status = int(rc)
                break
        selected = (policy == EVERY or (policy == FIRST and rep == 0)
                    or (policy == LAST and rep == total - 1))
        if selected:
            regions, s = compare(check_tbl, live, epilogue)
            last = s[0]
            worst = max(worst, int(last["total_mismatch"]))
        # whole-state guard: the part of the state the recorded kernel never writes must
        # still carry its recorded checksums
        if guard_tbl is not None and ((guard_every and (rep + 1) % guard_every == 0) or rep == total - 1):
            changed = np.flatnonzero(checksum(guard_tbl, live) != np.asarray(guard_expected, dtype=np.uint64))
            g_checks += 1
            if changed.size:
                if g_failed == 0:
                    g_first = int(changed[0])
                g_failed += 1
                g_changed = max(g_changed, int(changed.size))
    healed = 0
    if g_failed and heal_tbl is not None:
        restore(heal_tbl, prologue, live)
        healed = 1
    out = {"candidate_status": status, "regions": regions, "total_mismatch": worst,
           "guard": {"checks": g_checks, "failed_checks": g_failed, "changed_regions": g_changed,
                     "first_region": g_first, "healed": healed}}
    if last is not None:
        out.update(first_region=int(last["first_region"]), first_index=int(last["first_index"]),
                   max_abs_err=float(last["max_abs_err"]), max_rel_err=float(last["max_rel_err"]))
    else:
        out.update(first_region=NO_REGION, first_index=NO_INDEX, max_abs_err=0.0, max_rel_err=0.0)
    out["pass"] = int(status == 0 and worst == 0 and g_failed == 0)
    return out

"""ctypes binding of libr3.so: the same entry points as include/r3.h, with argument
marshalling only.  Device memory and streams come from PyTorch (uint8 CUDA tensors are the
arenas); every step of the path runs in the library's HIP kernels.  There is no CPU
fallback: if the library is missing, importing a symbol raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libr3.so")

# status codes
OK, EINVAL, EALIGN, ERANGE, EOVERLAP, ENOSPC, EHIP, ECANDIDATE, EBUSY = 0, -1, -2, -3, -4, -5, -6, -7, -8
# element types, modes, policies
U8, F32, F64, I32, BF16, F16 = 0, 1, 2, 3, 4, 5
BITWISE, TOL = 0, 1
EVERY, FIRST, LAST = 0, 1, 2
NO_INDEX = 0xFFFFFFFFFFFFFFFF
NO_REGION = 0xFFFFFFFF
MAX_REPLAYS = 1024

REGION_DTYPE = np.dtype(
    [("offset", "<u8"), ("bytes", "<u8"), ("dtype", "<u4"), ("mode", "<u4"),
     ("rtol", "<f8"), ("atol", "<f8")], align=True)
RESULT_DTYPE = np.dtype(
    [("mismatch_count", "<u8"), ("first_mismatch", "<u8"), ("max_abs_err", "<f8"),
     ("max_rel_err", "<f8"), ("checksum", "<u8")], align=True)
SUMMARY_DTYPE = np.dtype(
    [("total_mismatch", "<u8"), ("first_index", "<u8"), ("first_region", "<u4"),
     ("pass", "<u4"), ("max_abs_err", "<f8"), ("max_rel_err", "<f8")], align=True)


class EvalResult(ctypes.Structure):
    _fields_ = [("total_mismatch", ctypes.c_uint64), ("first_index", ctypes.c_uint64),
                ("first_region", ctypes.c_uint32), ("passed", ctypes.c_uint32),
                ("max_abs_err", ctypes.c_double), ("max_rel_err", ctypes.c_double),
                ("ms_min", ctypes.c_float), ("ms_median", ctypes.c_float),
                ("ms_max", ctypes.c_float), ("candidate_status", ctypes.c_int32)]


class Profile(ctypes.Structure):
    _fields_ = [("restore_ms", ctypes.c_double), ("candidate_ms", ctypes.c_double),
                ("validate_ms", ctypes.c_double), ("restore_launches", ctypes.c_uint64),
                ("candidate_launches", ctypes.c_uint64), ("validate_launches", ctypes.c_uint64)]


class Guard(ctypes.Structure):
    _fields_ = [("guard_tbl", ctypes.c_void_p), ("d_expected", ctypes.c_void_p),
                ("d_scratch", ctypes.c_void_p), ("heal_tbl", ctypes.c_void_p),
                ("every", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class GuardResult(ctypes.Structure):
    _fields_ = [("checks", ctypes.c_uint32), ("failed_checks", ctypes.c_uint32),
                ("changed_regions", ctypes.c_uint32), ("first_region", ctypes.c_uint32),
                ("healed", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class Timing(ctypes.Structure):
    _fields_ = [("n", ctypes.c_uint32), ("stable", ctypes.c_uint32), ("min", ctypes.c_float),
                ("median", ctypes.c_float), ("max", ctypes.c_float), ("mean", ctypes.c_float),
                ("mad", ctypes.c_float), ("reserved", ctypes.c_float)]


LAUNCH_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p)

DECLARED = [
    "r3_version", "r3_strerror", "r3_ctx_create", "r3_ctx_destroy", "r3_last_error",
    "r3_ctx_profile", "r3_ctx_profile_read",
    "r3_table_validate", "r3_table_workspace_bytes", "r3_table_workspace_bytes_exact",
    "r3_tune_tiles", "r3_tune_copy", "r3_table_create", "r3_table_destroy", "r3_table_info", "r3_restore",
    "r3_checksum", "r3_compare", "r3_dirty_diff", "r3_record", "r3_eval_candidate",
    "r3_eval_submit", "r3_eval_wait", "r3_eval_try_wait", "r3_eval_submit_guarded",
    "r3_writeset_regions", "r3_eval_candidate_guarded", "r3_table_replicate",
    "r3_eval_candidate_instances", "r3_ctx_last_times", "r3_timing_stats",
    "r3_replay_workspace_bytes", "r3_replay_create", "r3_replay_run", "r3_replay_destroy",
    "r3_compare_static", "r3_eval_submit_overlapped",
]

_lib = None


class R3Error(RuntimeError):
    def __init__(self, status, message):
        super().__init__("r3 status %d (%s): %s" % (status, _strerror(status), message))
        self.status = status


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_2604_11109_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, u32, u64, sz, ci = (ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_size_t,
                                ctypes.c_int)
        L.r3_version.restype = u32
        L.r3_strerror.argtypes = [ci]
        L.r3_strerror.restype = ctypes.c_char_p
        L.r3_ctx_create.argtypes = [ctypes.POINTER(vp), ci]
        L.r3_ctx_destroy.argtypes = [vp]
        L.r3_last_error.argtypes = [vp]
        L.r3_ctx_profile.argtypes = [vp, ci]
        L.r3_ctx_profile_read.argtypes = [vp, ctypes.POINTER(Profile), ci]
        L.r3_last_error.restype = ctypes.c_char_p
        L.r3_table_validate.argtypes = [vp, u32, u64]
        L.r3_table_workspace_bytes.argtypes = [u32, u64]
        L.r3_table_workspace_bytes.restype = sz
        L.r3_table_workspace_bytes_exact.argtypes = [vp, u32, u64]
        L.r3_table_workspace_bytes_exact.restype = sz
        L.r3_tune_tiles.argtypes = [u32, u32]
        L.r3_tune_copy.argtypes = [u32, u32]
        L.r3_table_create.argtypes = [vp, vp, u32, u64, vp, sz, ctypes.POINTER(vp)]
        L.r3_table_destroy.argtypes = [vp]
        L.r3_table_info.argtypes = [vp, ctypes.POINTER(u32), ctypes.POINTER(u64), ctypes.POINTER(u32),
                                    ctypes.POINTER(u64), ctypes.POINTER(u64)]
        L.r3_restore.argtypes = [vp, vp, vp, vp, vp]
        L.r3_checksum.argtypes = [vp, vp, vp, vp, vp]
        L.r3_compare.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        L.r3_compare_static.argtypes = [vp, vp, u32, u64, vp, vp, vp, vp, vp]
        L.r3_dirty_diff.argtypes = [vp, vp, vp, u64, u32, vp, vp, vp]
        L.r3_record.argtypes = [vp, vp, vp, vp, vp, vp, vp, u32, vp, vp, vp, vp, vp]
        L.r3_eval_candidate.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u32, u32, u32, vp,
                                        ctypes.POINTER(EvalResult), vp]
        L.r3_eval_submit.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u32, u32, u32, vp,
                                     ctypes.POINTER(u32), vp]
        L.r3_eval_submit_overlapped.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u32, u32, u32, vp,
                                                ctypes.POINTER(u32), vp]
        L.r3_eval_wait.argtypes = [vp, u32, ctypes.POINTER(EvalResult), ctypes.POINTER(GuardResult)]
        L.r3_eval_try_wait.argtypes = [vp, u32, u32, ctypes.POINTER(EvalResult), ctypes.POINTER(GuardResult)]
        L.r3_eval_submit_guarded.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u32, u32, u32, vp,
                                             ctypes.POINTER(Guard), ctypes.POINTER(u32), vp]
        L.r3_writeset_regions.argtypes = [vp, u64, u32, ci, vp, u32, ctypes.POINTER(u32)]
        L.r3_eval_candidate_guarded.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u32, u32, u32, vp,
                                                ctypes.POINTER(EvalResult), ctypes.POINTER(Guard),
                                                ctypes.POINTER(GuardResult), vp]
        L.r3_table_replicate.argtypes = [vp, u32, u64, u32, vp]
        L.r3_eval_candidate_instances.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u32, u64, u32, u32, u32,
                                                  vp, ctypes.POINTER(EvalResult), vp, vp]
        L.r3_ctx_last_times.argtypes = [vp, vp, u32, ctypes.POINTER(u32)]
        L.r3_timing_stats.argtypes = [vp, u32, ctypes.c_float, ctypes.POINTER(Timing)]
        L.r3_replay_workspace_bytes.restype = sz
        L.r3_replay_create.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, u32, ctypes.POINTER(vp)]
        L.r3_replay_run.argtypes = [vp, u32, u32, ctypes.POINTER(EvalResult), vp]
        L.r3_replay_destroy.argtypes = [vp]
        for name in DECLARED:
            getattr(L, name)  # AttributeError if the library does not export it
        _lib = L
    return _lib


def _strerror(status):
    try:
        return lib().r3_strerror(status).decode()
    except Exception:  # pragma: no cover
        return "?"


def make_table(rows):
    """rows: iterable of (offset, bytes, dtype, mode, rtol, atol) -> REGION_DTYPE array."""
    rows = list(rows)
    t = np.zeros(len(rows), dtype=REGION_DTYPE)
    for i, r in enumerate(rows):
        t[i] = tuple(r)
    return t


def _host_table(tbl):
    return np.ascontiguousarray(tbl, dtype=REGION_DTYPE)


def r3_table_validate(tbl, arena_bytes):
    if tbl is None or len(tbl) == 0:
        return lib().r3_table_validate(None, 0, arena_bytes)
    t = _host_table(tbl)
    return lib().r3_table_validate(t.ctypes.data, len(t), arena_bytes)


def r3_table_workspace_bytes(n, arena_bytes):
    return lib().r3_table_workspace_bytes(n, arena_bytes)


def r3_table_workspace_bytes_exact(tbl, arena_bytes):
    t = _host_table(tbl)
    return lib().r3_table_workspace_bytes_exact(t.ctypes.data, len(t), arena_bytes)


def r3_tune_tiles(min_tile_bytes=0, max_tiles_per_region=0):
    rc = lib().r3_tune_tiles(min_tile_bytes, max_tiles_per_region)
    if rc != OK:
        raise R3Error(rc, "r3_tune_tiles")


def r3_tune_copy(bytes_per_wavefront=0, block_threads=0):
    rc = lib().r3_tune_copy(bytes_per_wavefront, block_threads)
    if rc != OK:
        raise R3Error(rc, "r3_tune_copy")


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    if isinstance(t, (ctypes.Structure, ctypes.Array)):
        return ctypes.addressof(t)
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Context:
    """r3_ctx: host-side state bound to one GPU."""

    def __init__(self, device=0):
        h = ctypes.c_void_p()
        rc = lib().r3_ctx_create(ctypes.byref(h), device)
        if rc != OK:
            raise R3Error(rc, "r3_ctx_create(device=%d)" % device)
        self.handle = h
        self.device = device

    def last_error(self):
        return lib().r3_last_error(self.handle).decode()

    def check(self, rc, what):
        if rc != OK:
            raise R3Error(rc, "%s: %s" % (what, self.last_error()))

    def profile(self, period):
        """0 = off, n = stage events on every n-th evaluation."""
        self.check(lib().r3_ctx_profile(self.handle, int(period)), "r3_ctx_profile")

    def profile_read(self, reset=True):
        p = Profile()
        self.check(lib().r3_ctx_profile_read(self.handle, ctypes.byref(p), int(bool(reset))),
                   "r3_ctx_profile_read")
        return p

    def last_times(self):
        """Candidate times (ms) of the timed replays of the last evaluation."""
        n = ctypes.c_uint32(0)
        buf = np.zeros(MAX_REPLAYS, dtype=np.float32)
        self.check(lib().r3_ctx_last_times(self.handle, buf.ctypes.data, buf.size, ctypes.byref(n)),
                   "r3_ctx_last_times")
        return buf[:n.value].copy()

    def close(self):
        if self.handle:
            lib().r3_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Table:
    """r3_table plus the torch tensor that holds its device workspace."""

    def __init__(self, ctx, rows, arena_bytes, exact_workspace=True):
        import torch
        self.ctx = ctx
        self.host = _host_table(rows if isinstance(rows, np.ndarray) else make_table(rows))
        self.n = len(self.host)
        self.arena_bytes = int(arena_bytes)
        ws = 0
        if self.n:
            ws = (r3_table_workspace_bytes_exact(self.host, self.arena_bytes) if exact_workspace
                  else r3_table_workspace_bytes(self.n, self.arena_bytes))
        ws = max(int(ws), 256)
        self.workspace = torch.empty(ws, dtype=torch.uint8, device="cuda:%d" % ctx.device)
        h = ctypes.c_void_p()
        rc = lib().r3_table_create(ctx.handle, self.host.ctypes.data if self.n else None, self.n,
                                   self.arena_bytes, self.workspace.data_ptr(), ws, ctypes.byref(h))
        ctx.check(rc, "r3_table_create")
        self.handle = h

    def info(self):
        n, tiles, tb, total, arena = (ctypes.c_uint32(), ctypes.c_uint64(), ctypes.c_uint32(),
                                      ctypes.c_uint64(), ctypes.c_uint64())
        lib().r3_table_info(self.handle, ctypes.byref(n), ctypes.byref(tiles), ctypes.byref(tb),
                            ctypes.byref(total), ctypes.byref(arena))
        return {"n_regions": n.value, "n_tiles": tiles.value, "min_tile_bytes": tb.value,
                "total_bytes": total.value, "arena_bytes": arena.value}

    def close(self):
        if getattr(self, "handle", None):
            lib().r3_table_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _need(t, nbytes, what):
    if t is not None and not isinstance(t, int) and t.numel() * t.element_size() < nbytes:
        raise ValueError("%s holds %d bytes, %d needed" % (what, t.numel() * t.element_size(), nbytes))


def r3_restore(ctx, tbl, d_snapshot, d_live, stream=None):
    _need(d_snapshot, tbl.arena_bytes, "snapshot")
    _need(d_live, tbl.arena_bytes, "live arena")
    ctx.check(lib().r3_restore(ctx.handle, tbl.handle, _ptr(d_snapshot), _ptr(d_live),
                               _stream(stream)), "r3_restore")


def r3_checksum(ctx, tbl, d_arena, d_out, stream=None):
    _need(d_arena, tbl.arena_bytes, "arena")
    _need(d_out, 8 * tbl.n, "checksum output")
    ctx.check(lib().r3_checksum(ctx.handle, tbl.handle, _ptr(d_arena), _ptr(d_out),
                                _stream(stream)), "r3_checksum")


def r3_compare(ctx, tbl, d_live, d_golden, d_out, d_summary=None, stream=None):
    _need(d_live, tbl.arena_bytes, "live arena")
    _need(d_golden, tbl.arena_bytes, "golden arena")
    _need(d_out, 40 * tbl.n, "region results")
    _need(d_summary, 40, "summary")
    ctx.check(lib().r3_compare(ctx.handle, tbl.handle, _ptr(d_live), _ptr(d_golden), _ptr(d_out),
                               _ptr(d_summary), _stream(stream)), "r3_compare")


STATIC_MAX_REGIONS, STATIC_MAX_TILES, STATIC_MAX_TILE_BYTES = 16, 16384, 16 << 20


def r3_compare_static(ctx, rows, arena_bytes, d_live, d_golden, d_out, d_summary=None, stream=None):
    """r3_compare without a table object: the regions go in as host rows."""
    t = _host_table(rows if isinstance(rows, np.ndarray) else make_table(rows))
    _need(d_live, arena_bytes, "live arena")
    _need(d_golden, arena_bytes, "golden arena")
    _need(d_out, 40 * len(t), "region results")
    _need(d_summary, 40, "summary")
    ctx.check(lib().r3_compare_static(ctx.handle, t.ctypes.data if len(t) else None, len(t), int(arena_bytes),
                                      _ptr(d_live), _ptr(d_golden), _ptr(d_out), _ptr(d_summary),
                                      _stream(stream)), "r3_compare_static")


def bitmap_words(nbytes, page_bytes):
    pages = -(-nbytes // page_bytes)
    return -(-pages // 64)


def r3_dirty_diff(ctx, d_pre, d_post, nbytes, page_bytes, d_bitmap, d_dirty_count=None, stream=None):
    _need(d_pre, nbytes, "pre state")
    _need(d_post, nbytes, "post state")
    if page_bytes > 0:
        _need(d_bitmap, 8 * bitmap_words(nbytes, page_bytes), "bitmap")
    _need(d_dirty_count, 8, "dirty count")
    ctx.check(lib().r3_dirty_diff(ctx.handle, _ptr(d_pre), _ptr(d_post), nbytes, page_bytes,
                                  _ptr(d_bitmap), _ptr(d_dirty_count), _stream(stream)),
              "r3_dirty_diff")


def _launch_args(launch, user):
    """launch: None, an integer address of a C function with the r3_launch_fn signature, a
    ctypes function pointer, or a Python callable (wrapped; slow, for tests)."""
    if launch is None:
        return None, None, None
    if isinstance(launch, int):
        return ctypes.c_void_p(launch), user, None
    if isinstance(launch, ctypes._CFuncPtr):
        return ctypes.cast(launch, ctypes.c_void_p), user, launch
    cb = LAUNCH_FN(lambda u, live, stream: int(launch(live, stream) or 0))
    return ctypes.cast(cb, ctypes.c_void_p), None, cb


def r3_record(ctx, tbl, d_live, launch, user, d_prologue, d_epilogue, page_bytes=4096,
              d_bitmap=None, d_dirty_count=None, d_pro_cs=None, d_epi_cs=None, stream=None):
    _need(d_live, tbl.arena_bytes, "live arena")
    _need(d_prologue, tbl.arena_bytes, "prologue")
    _need(d_epilogue, tbl.arena_bytes, "epilogue")
    if d_bitmap is not None and page_bytes > 0:
        _need(d_bitmap, 8 * bitmap_words(tbl.arena_bytes, page_bytes), "bitmap")
    _need(d_pro_cs, 8 * tbl.n, "prologue checksums")
    _need(d_epi_cs, 8 * tbl.n, "epilogue checksums")
    fn, usr, keep = _launch_args(launch, user)
    rc = lib().r3_record(ctx.handle, tbl.handle, _ptr(d_live), fn, _ptr(usr), _ptr(d_prologue),
                         _ptr(d_epilogue), page_bytes, _ptr(d_bitmap), _ptr(d_dirty_count),
                         _ptr(d_pro_cs), _ptr(d_epi_cs), _stream(stream))
    del keep
    ctx.check(rc, "r3_record")


def r3_eval_candidate(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user,
                      warmup, reps, policy, d_regions, stream=None, raise_on_candidate=False):
    """Returns (status, EvalResult).  status is OK or ECANDIDATE unless raise_on_candidate."""
    _need(d_prologue, restore_tbl.arena_bytes, "prologue")
    _need(d_epilogue, check_tbl.arena_bytes, "epilogue")
    _need(d_live, max(restore_tbl.arena_bytes, check_tbl.arena_bytes), "live arena")
    _need(d_regions, 40 * check_tbl.n, "region results")
    fn, usr, keep = _launch_args(launch, user)
    out = EvalResult()
    rc = lib().r3_eval_candidate(ctx.handle, restore_tbl.handle, _ptr(d_prologue), check_tbl.handle,
                                 _ptr(d_epilogue), _ptr(d_live), fn, _ptr(usr), warmup, reps, policy,
                                 _ptr(d_regions), ctypes.byref(out), _stream(stream))
    del keep
    if rc == ECANDIDATE and not raise_on_candidate:
        return rc, out
    ctx.check(rc, "r3_eval_candidate")
    return rc, out


def r3_eval_submit(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user,
                   warmup, reps, policy, d_regions, stream=None):
    """Enqueue one evaluation without waiting; returns its ticket."""
    _need(d_prologue, restore_tbl.arena_bytes, "prologue")
    _need(d_epilogue, check_tbl.arena_bytes, "epilogue")
    _need(d_live, max(restore_tbl.arena_bytes, check_tbl.arena_bytes), "live arena")
    _need(d_regions, 40 * check_tbl.n, "region results")
    fn, usr, keep = _launch_args(launch, user)
    ticket = ctypes.c_uint32(0)
    rc = lib().r3_eval_submit(ctx.handle, restore_tbl.handle, _ptr(d_prologue), check_tbl.handle,
                              _ptr(d_epilogue), _ptr(d_live), fn, _ptr(usr), warmup, reps, policy,
                              _ptr(d_regions), ctypes.byref(ticket), _stream(stream))
    del keep
    ctx.check(rc, "r3_eval_submit")
    return ticket.value


def r3_eval_submit_overlapped(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user,
                              warmup, reps, policy, d_regions, stream=None):
    """r3_eval_submit on the context's two streams (pass two live arenas alternately)."""
    _need(d_prologue, restore_tbl.arena_bytes, "prologue")
    _need(d_epilogue, check_tbl.arena_bytes, "epilogue")
    _need(d_live, max(restore_tbl.arena_bytes, check_tbl.arena_bytes), "live arena")
    _need(d_regions, 40 * check_tbl.n, "region results")
    fn, usr, keep = _launch_args(launch, user)
    ticket = ctypes.c_uint32(0)
    rc = lib().r3_eval_submit_overlapped(ctx.handle, restore_tbl.handle, _ptr(d_prologue), check_tbl.handle,
                                         _ptr(d_epilogue), _ptr(d_live), fn, _ptr(usr), warmup, reps, policy,
                                         _ptr(d_regions), ctypes.byref(ticket), _stream(stream))
    del keep
    ctx.check(rc, "r3_eval_submit_overlapped")
    return ticket.value


def r3_eval_submit_guarded(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user,
                           warmup, reps, policy, d_regions, guard_tbl, d_expected, d_scratch,
                           every=0, heal_tbl=None, stream=None):
    """Enqueue one guarded evaluation without waiting; returns its ticket."""
    _need(d_prologue, restore_tbl.arena_bytes, "prologue")
    _need(d_epilogue, check_tbl.arena_bytes, "epilogue")
    _need(d_live, max(restore_tbl.arena_bytes, check_tbl.arena_bytes, guard_tbl.arena_bytes), "live arena")
    _need(d_regions, 40 * check_tbl.n, "region results")
    _need(d_expected, 8 * guard_tbl.n, "guard checksums")
    _need(d_scratch, 8 * guard_tbl.n, "guard scratch")
    fn, usr, keep = _launch_args(launch, user)
    g = Guard(guard_tbl.handle.value, _ptr(d_expected), _ptr(d_scratch),
              heal_tbl.handle.value if heal_tbl is not None else None, every, 0)
    ticket = ctypes.c_uint32(0)
    rc = lib().r3_eval_submit_guarded(ctx.handle, restore_tbl.handle, _ptr(d_prologue), check_tbl.handle,
                                      _ptr(d_epilogue), _ptr(d_live), fn, _ptr(usr), warmup, reps, policy,
                                      _ptr(d_regions), ctypes.byref(g), ctypes.byref(ticket), _stream(stream))
    del keep
    ctx.check(rc, "r3_eval_submit_guarded")
    return ticket.value


def r3_eval_wait(ctx, ticket, raise_on_candidate=False, with_guard=False):
    """Returns (status, EvalResult) of a submitted evaluation, or (status, EvalResult, GuardResult)
    with with_guard; status is OK or ECANDIDATE."""
    out, gout = EvalResult(), GuardResult()
    rc = lib().r3_eval_wait(ctx.handle, ticket, ctypes.byref(out), ctypes.byref(gout))
    if not (rc == ECANDIDATE and not raise_on_candidate):
        ctx.check(rc, "r3_eval_wait")
    return (rc, out, gout) if with_guard else (rc, out)


def r3_eval_try_wait(ctx, ticket, timeout_us=0):
    """Returns None while the evaluation is still running, else (status, EvalResult, GuardResult)."""
    out, gout = EvalResult(), GuardResult()
    rc = lib().r3_eval_try_wait(ctx.handle, ticket, timeout_us, ctypes.byref(out), ctypes.byref(gout))
    if rc == EBUSY:
        return None
    if rc != ECANDIDATE:
        ctx.check(rc, "r3_eval_try_wait")
    return rc, out, gout


def r3_writeset_regions(host_bitmap, nbytes, page_bytes, want_dirty):
    """host_bitmap: numpy uint64 array.  Returns a REGION_DTYPE array of the runs."""
    bm = np.ascontiguousarray(host_bitmap, dtype=np.uint64)
    n = ctypes.c_uint32(0)
    rc = lib().r3_writeset_regions(bm.ctypes.data if bm.size else None, nbytes, page_bytes,
                                   int(bool(want_dirty)), None, 0, ctypes.byref(n))
    if rc not in (OK, ENOSPC):
        raise R3Error(rc, "r3_writeset_regions")
    out = np.zeros(n.value, dtype=REGION_DTYPE)
    if n.value:
        rc = lib().r3_writeset_regions(bm.ctypes.data, nbytes, page_bytes, int(bool(want_dirty)),
                                       out.ctypes.data, n.value, ctypes.byref(n))
        if rc != OK:
            raise R3Error(rc, "r3_writeset_regions")
    return out


def r3_eval_candidate_guarded(ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user,
                              warmup, reps, policy, d_regions, guard_tbl, d_expected, d_scratch,
                              every=0, heal_tbl=None, stream=None):
    """Returns (status, EvalResult, GuardResult)."""
    _need(d_prologue, restore_tbl.arena_bytes, "prologue")
    _need(d_epilogue, check_tbl.arena_bytes, "epilogue")
    _need(d_live, max(restore_tbl.arena_bytes, check_tbl.arena_bytes, guard_tbl.arena_bytes), "live arena")
    _need(d_regions, 40 * check_tbl.n, "region results")
    _need(d_expected, 8 * guard_tbl.n, "guard checksums")
    _need(d_scratch, 8 * guard_tbl.n, "guard scratch")
    fn, usr, keep = _launch_args(launch, user)
    g = Guard(guard_tbl.handle.value, _ptr(d_expected), _ptr(d_scratch),
              heal_tbl.handle.value if heal_tbl is not None else None, every, 0)
    out, gout = EvalResult(), GuardResult()
    rc = lib().r3_eval_candidate_guarded(ctx.handle, restore_tbl.handle, _ptr(d_prologue),
                                         check_tbl.handle, _ptr(d_epilogue), _ptr(d_live), fn, _ptr(usr),
                                         warmup, reps, policy, _ptr(d_regions), ctypes.byref(out),
                                         ctypes.byref(g), ctypes.byref(gout), _stream(stream))
    del keep
    if rc != ECANDIDATE:
        ctx.check(rc, "r3_eval_candidate_guarded")
    return rc, out, gout


def r3_table_replicate(tbl, instance_stride, instances):
    t = _host_table(tbl)
    out = np.zeros(len(t) * instances, dtype=REGION_DTYPE)
    rc = lib().r3_table_replicate(t.ctypes.data if len(t) else None, len(t), instance_stride, instances,
                                  out.ctypes.data if out.size else None)
    if rc != OK:
        raise R3Error(rc, "r3_table_replicate")
    return out


def r3_eval_candidate_instances(ctx, restore_tbl, d_prologues, check_tbl, d_epilogues, d_live, launch, user,
                                instances, instance_stride, warmup, reps, policy, d_regions, stream=None):
    """Returns (status, EvalResult, per-instance pass flags as a uint8 array)."""
    _need(d_prologues, restore_tbl.arena_bytes, "prologues")
    _need(d_epilogues, check_tbl.arena_bytes, "epilogues")
    _need(d_live, max(restore_tbl.arena_bytes, check_tbl.arena_bytes), "live arena")
    _need(d_regions, 40 * check_tbl.n, "region results")
    fn, usr, keep = _launch_args(launch, user)
    out = EvalResult()
    flags = np.zeros(instances, dtype=np.uint8)
    rc = lib().r3_eval_candidate_instances(ctx.handle, restore_tbl.handle, _ptr(d_prologues), check_tbl.handle,
                                           _ptr(d_epilogues), _ptr(d_live), fn, _ptr(usr), instances,
                                           instance_stride, warmup, reps, policy, _ptr(d_regions),
                                           ctypes.byref(out), flags.ctypes.data, _stream(stream))
    del keep
    if rc != ECANDIDATE:
        ctx.check(rc, "r3_eval_candidate_instances")
    return rc, out, flags


class Replay:
    """r3_replay: one replay captured as a HIP graph, plus the tensors it refers to."""

    def __init__(self, ctx, restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, launch, user, d_regions,
                 replays):
        import torch
        _need(d_prologue, restore_tbl.arena_bytes, "prologue")
        _need(d_epilogue, check_tbl.arena_bytes, "epilogue")
        _need(d_live, max(restore_tbl.arena_bytes, check_tbl.arena_bytes), "live arena")
        _need(d_regions, 40 * check_tbl.n, "region results")
        self.ctx = ctx
        self.keep = (restore_tbl, d_prologue, check_tbl, d_epilogue, d_live, user, d_regions)
        self.workspace = torch.zeros(int(lib().r3_replay_workspace_bytes()), dtype=torch.uint8,
                                     device="cuda:%d" % ctx.device)
        fn, usr, self.keep_fn = _launch_args(launch, user)
        h = ctypes.c_void_p()
        rc = lib().r3_replay_create(ctx.handle, restore_tbl.handle, _ptr(d_prologue), check_tbl.handle,
                                    _ptr(d_epilogue), _ptr(d_live), fn, _ptr(usr), _ptr(d_regions),
                                    self.workspace.data_ptr(), replays, ctypes.byref(h))
        ctx.check(rc, "r3_replay_create")
        self.handle = h

    def run(self, warmup, reps, stream=None):
        out = EvalResult()
        self.ctx.check(lib().r3_replay_run(self.handle, warmup, reps, ctypes.byref(out), _stream(stream)),
                       "r3_replay_run")
        return out

    def close(self):
        if getattr(self, "handle", None):
            lib().r3_replay_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def r3_timing_stats(ms, rel_noise):
    a = np.ascontiguousarray(ms, dtype=np.float32)
    out = Timing()
    rc = lib().r3_timing_stats(a.ctypes.data if a.size else None, a.size, rel_noise, ctypes.byref(out))
    if rc != OK:
        raise R3Error(rc, "r3_timing_stats")
    return out


# ---- small conveniences for tests and the benchmark (no arithmetic of the method) --------
def results_to_numpy(d_regions, n):
    """Copy n r3_region_result records from a uint8 device tensor to a RESULT_DTYPE array."""
    return np.frombuffer(d_regions[:40 * n].cpu().numpy().tobytes(), dtype=RESULT_DTYPE).copy()


def summary_to_numpy(d_summary):
    return np.frombuffer(d_summary[:40].cpu().numpy().tobytes(), dtype=SUMMARY_DTYPE).copy()

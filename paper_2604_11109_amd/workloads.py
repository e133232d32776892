"""ctypes view of libr3_workloads.so: candidate kernels (Jacobi and CSR SpMV variants) behind
launch callbacks that r3_record / r3_eval_candidate can call without leaving native code."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libr3_workloads.so")
_lib = None


class JacobiArgs(ctypes.Structure):
    _fields_ = [("in_off", ctypes.c_uint64), ("out_off", ctypes.c_uint64), ("n", ctypes.c_uint32),
                ("block", ctypes.c_uint32), ("unroll", ctypes.c_uint32), ("bug", ctypes.c_uint32)]


class SpmvArgs(ctypes.Structure):
    _fields_ = [("rowptr_off", ctypes.c_uint64), ("col_off", ctypes.c_uint64),
                ("val_off", ctypes.c_uint64), ("x_off", ctypes.c_uint64), ("y_off", ctypes.c_uint64),
                ("rows", ctypes.c_uint32), ("rows_per_wave", ctypes.c_uint32),
                ("block", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class CopyArgs(ctypes.Structure):
    _fields_ = [("src_off", ctypes.c_uint64), ("dst_off", ctypes.c_uint64), ("bytes", ctypes.c_uint64)]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_2604_11109_amd.build`" % LIB_PATH)
        _lib = ctypes.CDLL(LIB_PATH)
    return _lib


def _addr(name):
    return ctypes.cast(getattr(lib(), name), ctypes.c_void_p).value


def jacobi_launch():
    """Address of the Jacobi launch callback (pass as `launch`, with a JacobiArgs as `user`)."""
    return _addr("r3w_jacobi_launch")


def spmv_launch():
    return _addr("r3w_spmv_launch")


def copy_launch():
    return _addr("r3w_copy_launch")


def plain_copy(d_arena, src_off, dst_off, nbytes, stream=0):
    """Run the plain copy kernel once inside d_arena (a uint8 CUDA tensor)."""
    lib().r3w_copy_launch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    args = CopyArgs(src_off, dst_off, nbytes)
    rc = lib().r3w_copy_launch(ctypes.addressof(args), d_arena.data_ptr(), stream)
    if rc:
        raise RuntimeError("plain copy launch failed: %d" % rc)


def yard_copy(d_src, d_dst, nbytes, kib_per_wave=1, stream=0):
    """Plain copy yardstick: nbytes from d_src to d_dst (uint8 CUDA tensors)."""
    f = lib().r3w_yard_copy
    f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p]
    rc = f(d_src.data_ptr(), d_dst.data_ptr(), nbytes, kib_per_wave, stream)
    if rc:
        raise RuntimeError("yard copy launch failed: %d" % rc)


def yard_read2(d_a, d_b, nbytes, d_sink, kib_per_wave=4, stream=0):
    """Two-stream read yardstick: reads nbytes of d_a and of d_b."""
    f = lib().r3w_yard_read2
    f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p,
                  ctypes.c_void_p]
    rc = f(d_a.data_ptr(), d_b.data_ptr(), nbytes, kib_per_wave, d_sink.data_ptr(), stream)
    if rc:
        raise RuntimeError("yard read2 launch failed: %d" % rc)


def failing_launch():
    return _addr("r3w_failing_launch")


def jacobi_args(case, block, unroll, bug):
    return JacobiArgs(case["in_off"], case["out_off"], case["n"], block, unroll, bug)


def spmv_args(case, rows_per_wave, block):
    o = case["offsets"]
    return SpmvArgs(o["row_ptr"], o["col_idx"], o["vals"], o["x"], o["y"], case["rows"],
                    rows_per_wave, block, 0)

"""Builds the HIP libraries of this package in-tree for gfx950 (hipcc cross-compiles
without a GPU).  `python -m paper_2604_11109_amd.build` or build_all() from Python."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]

HOST_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"

LIBS = {
    "libr3.so": ["r3_table.cpp", "r3_api.cpp", "r3_kernels.hip"],
    "libr3_workloads.so": ["workloads/r3w_workloads.hip"],
}


def lib_path(name):
    return os.path.join(HERE, name)


def build_lib(name, verbose=True):
    srcs = [os.path.join(CSRC, s) for s in LIBS[name]]
    srcs = [s for s in srcs if os.path.exists(s)]
    if not srcs:
        return None
    out = lib_path(name)
    tmp = out + ".tmp%d" % os.getpid()
    cmd = [HIPCC] + COMMON + ["-x", "hip"] + srcs + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # The packed-fp32 switch is a device feature; clang's driver refuses to forward -Xclang to
    # one side only, so the host passes see it too and answer with HOST_NOTE.  That one known
    # line is dropped, everything else the compiler says is shown.
    shown = [l for l in res.stdout.splitlines() if l.strip() != HOST_NOTE]
    if shown:
        print("\n".join(shown), flush=True)
    if res.returncode != 0:
        raise subprocess.CalledProcessError(res.returncode, cmd)
    os.replace(tmp, out)
    return out


def build_all(verbose=True):
    return [build_lib(n, verbose) for n in LIBS]


if __name__ == "__main__":
    build_all()
    sys.exit(0)

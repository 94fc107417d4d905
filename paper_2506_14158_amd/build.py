"""Build libs4c.so (HIP, gfx950) in-tree with hipcc.  Used by __graft_entry__.build()."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libs4c.so")
OBJ = os.path.join(PKG, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",      # no packed-fp32 instructions
    "-fno-honor-nans",                                                # inputs are finite by contract; infinities are still honoured
    "-Wno-unused-command-line-argument", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def build_lib(verbose: bool = False, lib: str = LIB, obj_dir: str = OBJ, extra_flags=()) -> str:
    """Compile csrc/*.hip (in parallel) and link them into `lib`.  `extra_flags` are appended to the
    compile and link lines (the sanitizer test builds an instrumented copy elsewhere this way)."""
    os.makedirs(obj_dir, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))

    def cc(src):
        obj = os.path.join(obj_dir, os.path.basename(src)[:-4] + ".o")
        cmd = [HIPCC] + FLAGS + list(extra_flags) + ["-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stderr[-8000:]))
        if verbose and r.stderr.strip():
            print(r.stderr[-4000:])
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(cc, srcs))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + list(extra_flags) + ["-o", lib] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr[-4000:])
    return lib


PROBE_SRC = os.path.join(PKG, "probe", "probes.hip")
PROBE_LIB = os.path.join(PKG, "libs4c_probe.so")


def build_probe_lib() -> str:
    """The benchmark's measurement probes: a library of their own, not part of libs4c.so."""
    cmd = [HIPCC] + FLAGS + ["-I" + os.path.join(PKG, "probe"), "-shared", PROBE_SRC, "-o", PROBE_LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (PROBE_SRC, r.stderr[-8000:]))
    return PROBE_LIB


C_CLIENT_SRC = os.path.join(ROOT, "tests", "c_client", "verify_step.c")
C_CLIENT_BIN = os.path.join(ROOT, "tests", "c_client", "verify_step")


def build_c_client() -> str:
    """The plain-C test client of the C ABI (gcc, linked against libs4c.so and the HIP runtime)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [os.environ.get("CC", "gcc"), "-std=c11", "-O1", "-Wall", "-I" + os.path.join(rocm, "include"),
           "-I" + os.path.join(ROOT, "include"), C_CLIENT_SRC, "-o", C_CLIENT_BIN, "-L" + PKG, "-ls4c",
           "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN/../../paper_2506_14158_amd",
           "-Wl,-rpath," + os.path.join(rocm, "lib")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("C client build failed:\n" + r.stderr[-4000:])
    return C_CLIENT_BIN


if __name__ == "__main__":
    print(build_lib(verbose=True))
    print(build_probe_lib())
    print(build_c_client())

"""Host-side sanitizer runs (CPU only; GPU code cannot be instrumented here).

1. The oracle is rebuilt with gcc -fsanitize=address,undefined and all of its pins
   (tests/test_oracle_*.py) run against that build in a child interpreter.
2. The host side of libs4c (argument checks, launch planning, launchers) is rebuilt with hipcc's
   host-only sanitizer flags and the C-ABI error cases (tests/test_abi.py) run against that build.
The children preload the matching sanitizer runtime, because the Python executable itself is not
instrumented, and run pytest without output capture so that a report reaches stderr; a report from
either sanitizer aborts the child and fails the test.

The same two commands by hand:
    python tests/test_sanitizers.py oracle
    python tests/test_sanitizers.py host
"""
import glob
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ORACLE_PINS = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n--- stdout\n%s\n--- stderr\n%s" % (" ".join(cmd), r.stdout[-6000:], r.stderr[-6000:])
    return r


def _child_env(runtime, **extra):
    env = dict(os.environ)
    # the runtime goes first; whatever was preloaded before stays preloaded
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # detect_leaks: the interpreter and its extension modules hold memory until exit by design
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:abort_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    env.update(extra)
    return env


def oracle_under_sanitizers(tmp):
    lib = os.path.join(tmp, "libs4c_oracle_san.so")
    _run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=undefined", "-o", lib, os.path.join(ROOT, "oracle", "s4c_oracle.c"), "-lm"])
    runtime = _run(["gcc", "-print-file-name=libasan.so"]).stdout.strip()
    assert os.path.isabs(runtime) and os.path.exists(runtime), runtime
    r = _run([sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider"] + ORACLE_PINS, cwd=ROOT,
             env=_child_env(runtime, S4C_ORACLE_LIB=lib))
    assert " passed" in r.stdout and "failed" not in r.stdout, r.stdout[-2000:]
    return r.stdout.strip().splitlines()[-1]


def host_side_under_sanitizers(tmp):
    from paper_2506_14158_amd import build as bld
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-Xarch_host", "-g"]
    lib = bld.build_lib(lib=os.path.join(tmp, "libs4c_san.so"), obj_dir=os.path.join(tmp, "obj"), extra_flags=san)
    runtime = _run([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"]).stdout.strip()
    if not os.path.isabs(runtime):
        found = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        assert found, "clang's AddressSanitizer runtime not found"
        runtime = found[0]
    code = ("import sys, pytest; sys.path.insert(0, %r)\n"
            "from paper_2506_14158_amd import binding\n"
            "binding.LIB_PATH = %r\n"
            "sys.exit(pytest.main(['-x', '-q', '-s', '-p', 'no:cacheprovider', %r, '-k', 'not missing_library']))\n"
            % (ROOT, lib, os.path.join(ROOT, "tests", "test_abi.py")))
    r = _run([sys.executable, "-c", code], cwd=ROOT, env=_child_env(runtime))
    assert " passed" in r.stdout and "failed" not in r.stdout, r.stdout[-2000:]
    return r.stdout.strip().splitlines()[-1]


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    print(oracle_under_sanitizers(str(tmp_path)))


def test_abi_error_cases_pass_with_the_host_code_under_sanitizers(tmp_path):
    print(host_side_under_sanitizers(str(tmp_path)))


if __name__ == "__main__":
    which = sys.argv[1] if len(sys.argv) > 1 else "both"
    with tempfile.TemporaryDirectory() as tmp:
        if which in ("oracle", "both"):
            print("oracle:", oracle_under_sanitizers(tmp))
        if which in ("host", "both"):
            print("host:", host_side_under_sanitizers(tmp))

"""The oracle's pins once more, against a build of the oracle with AddressSanitizer and UndefinedBehaviorSanitizer, and
the library's host logic (argument validation, page bookkeeping, the seeded projection) under the same sanitizers'
run-time: an out-of-bounds access, a misaligned or overflowing operation in either aborts the child process."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _asan_runtime():
    path = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _child_env(extra, rt=None):
    env = dict(os.environ)
    rt = rt or _asan_runtime()
    # the sanitizer's run-time must be loaded before the interpreter's own allocations: append it to whatever is preloaded
    env["LD_PRELOAD"] = (env.get("LD_PRELOAD", "") + " " + rt).strip()
    # python itself leaks by design and is not instrumented; the link order check assumes an instrumented executable
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


@pytest.mark.skipif(_asan_runtime() is None, reason="gcc's libasan.so is not installed")
def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from oracle import build as oracle_build
    lib = oracle_build.build_sanitized(str(tmp_path / "liboracle_san.so"))
    files = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    assert len(files) >= 7
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + files, cwd=ROOT,
                       env=_child_env({"H1BKV_ORACLE_LIB": lib, "OMP_NUM_THREADS": "4"}), capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    # the sanitized build was the one that ran
    probe = ("from oracle import cref; import ctypes; L = cref.lib(); print(L._name)")
    r2 = subprocess.run([sys.executable, "-c", probe], cwd=ROOT, env=_child_env({"H1BKV_ORACLE_LIB": lib}), capture_output=True, text=True)
    assert r2.returncode == 0 and r2.stdout.strip() == lib, r2.stdout + r2.stderr


@pytest.mark.skipif(_asan_runtime() is None, reason="gcc's libasan.so is not installed")
def test_planted_overrun_is_caught(tmp_path):
    """The check checks something: a C function that reads one element past its buffer, built and loaded the same way,
    makes the child process abort."""
    src = tmp_path / "overrun.c"
    src.write_text("#include <stdlib.h>\nint overrun(int n) { int *p = malloc(n * sizeof(int)); for (int i = 0; i < n; ++i) p[i] = i;"
                   " int v = p[n]; free(p); return v; }\n")
    lib = tmp_path / "liboverrun.so"
    subprocess.run(["gcc", "-O1", "-g", "-fPIC", "-shared", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", str(lib), str(src)],
                   check=True)
    code = f"import ctypes; L = ctypes.CDLL({str(lib)!r}); print('ok', L.overrun(0) * 0)"
    good = subprocess.run([sys.executable, "-c", code.replace("overrun(0) * 0", "overrun.__class__ is not None")], env=_child_env({}),
                          capture_output=True, text=True)
    assert good.returncode == 0, good.stderr[-2000:]
    bad = subprocess.run([sys.executable, "-c", code.replace("overrun(0)", "overrun(8)")], env=_child_env({}), capture_output=True, text=True)
    assert bad.returncode != 0 and "heap-buffer-overflow" in bad.stderr, bad.stderr[-2000:]


def test_host_logic_passes_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The library's host side (validation, page bookkeeping, rollback, the seeded projection draw) rebuilt with both
    sanitizers, and the bookkeeping-only tests run against that build."""
    from paper_2510_05529_amd import build as hip_build
    rt = hip_build.sanitizer_runtime()
    if not rt:
        pytest.skip("the clang AddressSanitizer run-time is not installed")
    lib = hip_build.build_host_sanitized(str(tmp_path / "libh1bkv_san.so"))
    files = [os.path.join(ROOT, "tests", "test_host_logic.py"), os.path.join(ROOT, "tests", "test_abi.py")]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + files, cwd=ROOT,
                       env=_child_env({"H1BKV_LIBRARY": lib}, rt), capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail

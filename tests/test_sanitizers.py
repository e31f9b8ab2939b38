"""Host-side sanitizer runs (CPU only): the oracle's pins with the oracle built under AddressSanitizer and
UndefinedBehaviorSanitizer, and the library's host tests (host-only entry points, planners, every argument check)
with the host code of libwk built the same way.  Each run is a child process with the sanitizer runtime preloaded;
a planted out-of-bounds write in a call of the oracle shows that the run really is instrumented."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
REPORT_MARKS = ("ERROR: AddressSanitizer", "runtime error:", "ERROR: LeakSanitizer")


def _env(runtime, **extra):
    env = dict(os.environ)
    prior = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + (":" + prior if prior else "")     # the sanitizer runtime must come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    env["OMP_NUM_THREADS"] = "4"
    env.update(extra)
    return env


@pytest.fixture(scope="module")
def oracle_asan(tmp_path_factory):
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    from oracle import build as ob
    runtime = ob.sanitizer_runtime()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's libasan.so is not installed")
    lib = ob.build_sanitized(str(tmp_path_factory.mktemp("oracle_asan") / "liboracle_wk_asan.so"))
    return _env(runtime, WK_ORACLE_LIB=lib)


def test_oracle_pins_pass_under_asan_and_ubsan(oracle_asan):
    pins = sorted(os.path.join(ROOT, "tests", f) for f in os.listdir(os.path.join(ROOT, "tests"))
                  if f.startswith("test_oracle_") and f.endswith(".py"))
    pins.append(os.path.join(ROOT, "tests", "test_checker_selftest.py"))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins], cwd=ROOT,
                       env=oracle_asan, capture_output=True, text=True, timeout=900)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-4000:]
    assert not any(m in out for m in REPORT_MARKS), out[-4000:]
    assert " passed" in out


def test_the_sanitizer_run_is_instrumented(oracle_asan):
    """A call that hands the oracle an output array one element too short must be reported."""
    code = ("import ctypes as C, numpy as np, oracle\n"
            "L = oracle.lib()\n"
            "assert 'asan' in L._name\n"
            "s = np.arange(64, dtype=np.float64)\n"
            "out = np.zeros(7, np.int32)\n"          # n_keep = 8 below: one write past the end
            "L.wko_select_lowest(C.c_void_p(s.ctypes.data), C.c_int64(64), C.c_int64(8), C.c_void_p(out.ctypes.data))\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=oracle_asan, capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr, (r.returncode, r.stderr[-2000:])


def test_library_host_layer_passes_under_asan_and_ubsan(tmp_path):
    """libwk's host code (wk_keep_count, wk_window_plan, wk_accumulate_actions, workspace sizing, launch
    planning and every argument check) with host-side sanitizers: tests/test_library_host.py runs against it."""
    from paper_2605_22718_amd import build as hb
    if not os.path.exists(hb.HIPCC):
        pytest.skip("no hipcc")
    runtime = hb.sanitizer_runtime()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("clang's AddressSanitizer runtime is not installed")
    lib = hb.build_host_sanitized(str(tmp_path / "hostsan"))
    env = _env(runtime, WK_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
                        os.path.join(ROOT, "tests", "test_library_host.py")], cwd=ROOT, env=env, capture_output=True,
                       text=True, timeout=900)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-4000:]
    assert not any(m in out for m in REPORT_MARKS), out[-4000:]
    assert " passed" in out

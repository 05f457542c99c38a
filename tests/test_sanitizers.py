"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU involved).

  * the fp64 oracle (oracle/w2l_oracle.c), rebuilt with gcc -fsanitize=address,undefined, runs its
    own pin tests (tests/test_oracle_*.py) in a child process;
  * the library's host side -- argument checks, workspace and launch-configuration arithmetic --
    from `python -m paper_1812_07625_amd.build --sanitize` (the same sources; only the host pass is
    instrumented) runs the host-only ABI tests in a child process.
Either child aborts on the first report (-fno-sanitize-recover), which fails the test here.
The sanitizer runtime has to be the first library of the child, hence LD_PRELOAD (prepended to
whatever the environment already preloads).
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_pytest_under(runtime, extra_env, files):
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + ((":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra_env)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + [os.path.join(ROOT, "tests", f) for f in files]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, "child pytest failed under the sanitizers:\n%s\n%s" % (r.stdout[-4000:], r.stderr[-4000:])
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error:" not in r.stderr
    return r.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    lib = str(tmp_path / "libw2l_oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fopenmp", "-fPIC", "-shared", "-o", lib,
                           os.path.join(ROOT, "oracle", "w2l_oracle.c"), "-lm"])
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.isabs(runtime), "gcc has no shared ASan runtime"
    out = _run_pytest_under(runtime, {"W2L_ORACLE_LIB": lib},
                            ["test_oracle_conv.py", "test_oracle_ctc.py", "test_oracle_misc.py", "test_oracle_asg.py"])
    assert "failed" not in out


def test_library_host_code_under_asan_ubsan():
    from paper_1812_07625_amd import build as hip_build
    lib = hip_build.build(sanitize=True)
    out = _run_pytest_under(hip_build.asan_runtime(), {"W2L_LIB": lib}, ["test_abi.py", "test_launch_variants.py"])
    assert "failed" not in out

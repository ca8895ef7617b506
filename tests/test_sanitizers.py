"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): the library's sampler,
validation, planner and parameter handling (tests/sanitize/host_driver.cpp, linked with sampler.cpp and
rocket_api.hip compiled for the host only, kernel launchers stubbed), and the C oracle
(tests/sanitize/oracle_driver.c).  Any report makes the program exit non-zero."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2301_08527_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout[-4000:]
    return r.stdout


def test_oracle_c_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-std=c99", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra"] + SAN +
         [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "rocket_oracle.c"),
          "-o", exe, "-lm"])
    out = _run([exe], env=dict(ENV, OMP_NUM_THREADS="2"))
    assert "oracle driver: ok" in out


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_library_host_code_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_driver")
    # rocket_api.hip holds almost no device code (one array), so it compiles in seconds; every sanitizer flag goes to
    # the host compilation only
    host_san = []
    for f in SAN:
        host_san += ["-Xarch_host", f]
    common = ["-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = []
    for src, extra in ((os.path.join(CSRC, "rocket_api.hip"), ["--offload-arch=gfx950"]),
                       (os.path.join(CSRC, "sampler.cpp"), ["-x", "c++", "-ffp-contract=off"]),
                       (os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), ["-x", "c++"])):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        _run([HIPCC] + extra + common + host_san + ["-c", src, "-o", obj])
        objs.append(obj)
    _run([HIPCC, "--offload-arch=gfx950"] + host_san + objs + ["-o", exe])
    out = _run([exe], env=ENV)
    assert "host driver: ok" in out

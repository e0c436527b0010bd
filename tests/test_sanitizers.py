"""Host-side sanitizer passes (CPU only, no GPU call is made):

  * oracle/otf_oracle.c under AddressSanitizer + UndefinedBehaviorSanitizer, driven by
    tests/sanitize/oracle_driver.c over ragged sizes with tightly sized heap buffers; the same
    driver built plainly must print the same checksums;
  * the argument validation, workspace layout and switches of the C ABI (host code of
    csrc/otf_api.hip) under both sanitizers, driven by tests/sanitize/boundary_driver.cpp with
    extreme and invalid arguments;
  * the oracle pins and the boundary tests themselves, run in a child interpreter against builds
    of both libraries with undefined-behaviour checks in trap mode.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ORACLE_C = os.path.join(ROOT, "oracle", "otf_oracle.c")
REPORT_WORDS = ("runtime error", "AddressSanitizer", "UndefinedBehaviorSanitizer", "LeakSanitizer")

needs_gcc = pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
needs_hipcc = pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")


def _run(cmd, env=None, timeout=600):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run(cmd, capture_output=True, text=True, env=e, timeout=timeout, cwd=ROOT)


def _clean(result):
    text = result.stdout + result.stderr
    assert result.returncode == 0, text[-4000:]
    assert not any(w in text for w in REPORT_WORDS), text[-4000:]


@needs_gcc
def test_oracle_c_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    checked, plain = str(tmp_path / "oracle_checked"), str(tmp_path / "oracle_plain")
    common = ["gcc", "-std=c11", "-fopenmp", "-ffp-contract=off", "-g"]
    srcs = [ORACLE_C, os.path.join(SAN, "oracle_driver.c"), "-lm"]
    r = _run(common + ["-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                       "-o", checked] + srcs)
    assert r.returncode == 0, r.stderr[-3000:]
    r = _run(common + ["-O2", "-o", plain] + srcs)
    assert r.returncode == 0, r.stderr[-3000:]
    a = _run([checked], env={"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "OMP_NUM_THREADS": "4"})
    _clean(a)
    b = _run([plain], env={"OMP_NUM_THREADS": "4"})
    assert b.returncode == 0
    assert a.stdout == b.stdout and a.stdout.count("\n") > 200
    assert "rc=-" in a.stdout                       # the driver's bad inputs were refused, not followed


@needs_hipcc
def test_argument_validation_under_address_and_undefined_behaviour_sanitizers():
    from paper_1407_4764_amd import build
    exe = build.build_host_checked("asan-ubsan", os.path.join(SAN, "boundary_driver.cpp"))
    # the HIP runtime keeps its start-up allocations until the process ends: leak reports are not ours
    r = _run([exe], env={"ASAN_OPTIONS": "detect_leaks=0"})
    _clean(r)
    assert "every call was rejected as documented" in r.stdout


@needs_gcc
@needs_hipcc
def test_oracle_pins_and_boundary_tests_against_trapping_builds(tmp_path):
    from paper_1407_4764_amd import build
    libotf = build.build_host_checked("ubsan-trap")
    liboracle = str(tmp_path / "libotf_oracle_checked.so")
    r = _run(["gcc", "-O1", "-g", "-fopenmp", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fsanitize=undefined",
              "-fsanitize-undefined-trap-on-error", "-o", liboracle, ORACLE_C, "-lm"])
    assert r.returncode == 0, r.stderr[-3000:]
    files = ["tests/test_oracle_pins.py", "tests/test_boundary.py", "tests/test_binding_checks.py"]
    r = _run([sys.executable, os.path.join(SAN, "run_checked.py"), libotf, liboracle] + files, timeout=900)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert " passed" in r.stdout

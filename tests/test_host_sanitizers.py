"""The host side under sanitizers, without a GPU: the library's plan and replica-array arithmetic compiled with
AddressSanitizer and UndefinedBehaviorSanitizer and replayed over seeded random and near-overflow inputs whose
expected values the oracle wrote (tests/golden/plan_fuzz_cases.txt), and the oracle's own pins under Python's
development mode."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2004_13336_amd", "csrc")
GOLDEN = os.path.join(ROOT, "tests", "golden")


def test_golden_fuzz_cases_are_what_the_oracle_script_writes(tmp_path):
    """The stored file is reproducible from the committed script, which imports nothing but oracle/."""
    src = open(os.path.join(GOLDEN, "make_plan_fuzz_cases.py")).read()
    assert "paper_2004_13336_amd" not in src
    work = tmp_path / "golden"
    work.mkdir()
    script = work / "make_plan_fuzz_cases.py"
    # the script writes beside itself and finds the repository two levels up: run a copy from a mirror of that layout
    mirror = tmp_path / "repo" / "tests" / "golden"
    mirror.mkdir(parents=True)
    shutil.copy(os.path.join(GOLDEN, "make_plan_fuzz_cases.py"), mirror / "make_plan_fuzz_cases.py")
    os.symlink(os.path.join(ROOT, "oracle"), tmp_path / "repo" / "oracle")
    subprocess.run([sys.executable, str(mirror / "make_plan_fuzz_cases.py")], check=True, capture_output=True)
    assert open(mirror / "plan_fuzz_cases.txt").read() == open(os.path.join(GOLDEN, "plan_fuzz_cases.txt")).read()
    del script


def test_plan_and_topology_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host compiler")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    exe = str(tmp_path / "plan_fuzz")
    cmd = [gxx, "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-g", "-O1", "-Wall", "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "plan_fuzz.cpp"), os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "topology.cpp"),
           "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)              # the sanitizer runtime must come first in the program's own link order
    run = subprocess.run([exe, os.path.join(GOLDEN, "plan_fuzz_cases.txt")], capture_output=True, text=True, env=env)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-3000:])
    assert "all agree" in run.stdout and "runtime error" not in run.stderr


def test_oracle_pins_pass_in_python_development_mode():
    """python -X dev turns on the interpreter's own run-time checks (unclosed files, bad buffer use, numpy's
    deprecations as errors are not implied); the oracle's pins must pass there as they do normally."""
    files = sorted(f for f in os.listdir(os.path.join(ROOT, "tests")) if f.startswith("test_oracle_") and f != "test_oracle_mutations.py")
    cmd = [sys.executable, "-X", "dev", "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider", "-m", "not gpu"] + \
          [os.path.join(ROOT, "tests", f) for f in files]
    run = subprocess.run(cmd, capture_output=True, text=True, cwd=ROOT)
    assert run.returncode == 0, run.stdout[-3000:] + run.stderr[-2000:]

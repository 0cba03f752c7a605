"""The host code of the library (plan, admission, C-ABI layer) and the C oracle, compiled with
AddressSanitizer and UndefinedBehaviorSanitizer, under the host-side test files: every index the plan
builder, the planner and the oracle compute on thousands of seeded batches is then a checked one.
The device side is replaced by stubs (host-only contexts launch nothing)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_06914_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
HOST_TESTS = ["test_plan_host.py", "test_plan_fuzz.py", "test_phase_host.py", "test_admission_host.py", "test_workspace_host.py"]


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no libasan.so beside gcc")
    lib = tmp_path / "libtaper_attn_san.so"
    subprocess.check_call(["g++", "-std=c++17", "-fPIC", "-shared", *SAN, "-D__HIP_PLATFORM_AMD__", "-fvisibility=hidden",
                           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", "/opt/rocm/include", "-o", str(lib),
                           os.path.join(CSRC, "taper_api.cpp"), os.path.join(CSRC, "taper_plan.cpp"),
                           os.path.join(CSRC, "taper_admission.cpp"), os.path.join(ROOT, "tests", "sanitize", "kernel_stubs.cpp"),
                           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"])
    olib = tmp_path / "libtaper_oracle_san.so"
    subprocess.check_call(["gcc", "-std=c99", "-fPIC", "-shared", "-fopenmp", *SAN, "-o", str(olib),
                           os.path.join(ROOT, "oracle", "taper_oracle.c"), "-lm"])
    env = dict(os.environ)
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    cmd = [sys.executable, os.path.join(ROOT, "tests", "sanitize", "run_pytest_with_libraries.py"), str(lib), str(olib),
           "-q", "-x", "-p", "no:cacheprovider", "-m", "not gpu", *[os.path.join(ROOT, "tests", t) for t in HOST_TESTS]]
    run = subprocess.run(cmd, env=env, capture_output=True, text=True, timeout=1500, cwd=ROOT)
    out = run.stdout + run.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert run.returncode == 0, out[-4000:]
    assert " passed" in run.stdout
    mapped = [l for l in run.stdout.splitlines() if l.startswith("libraries mapped:")][-1]
    assert str(lib) in mapped and str(olib) in mapped and "paper_2605_06914_amd/libtaper_attn.so" not in mapped, mapped

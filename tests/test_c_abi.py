"""The boundary is a C ABI: the headers must be valid C99 and usable without Python or C++."""
import os
import subprocess

from paper_2605_06914_amd import LIB_PATH, load_library

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_headers_are_c99_and_a_c_program_can_use_the_library(tmp_path):
    load_library()  # raises if the library has not been built
    exe = tmp_path / "host_only"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c_abi", "host_only.c"), "-o", str(exe), LIB_PATH, "-lm",
                           "-Wl,-rpath," + os.path.dirname(LIB_PATH)])
    env = dict(os.environ)
    for d in ("/opt/rocm/lib",):
        env["LD_LIBRARY_PATH"] = d + ":" + env.get("LD_LIBRARY_PATH", "")
    out = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=60)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stdout + out.stderr

"""CPU-only checks of what the compiler made of the kernels (hipcc cross-compiles gfx950 here):
no decode kernel variant may use scratch memory, and no vector instruction may read a matrix
instruction's result before the matrix pipeline has delivered it."""
import os
import re
import subprocess

import pytest

from paper_2605_06914_amd.build import CSRC, HIP_FLAGS, ROOT
from tests.asm_hazards import NEED, scan


@pytest.fixture(scope="module")
def compiled(tmp_path_factory):
    """Assembly of the kernels and the compiler's resource-usage remarks, from one device-only compile."""
    out_dir = tmp_path_factory.mktemp("kernels")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIP_FLAGS if f not in ("-shared", "-fPIC")]
    asm = out_dir / "taper_kernels.s"
    cmd = [hipcc, *flags, "--cuda-device-only", "-S", "-Rpass-analysis=kernel-resource-usage",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", str(asm), os.path.join(CSRC, "taper_kernels.hip")]
    run = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert run.returncode == 0, run.stderr[-2000:]
    return asm.read_text(), run.stderr


def test_decode_kernels_use_no_scratch_memory(compiled):
    """Any scratch use makes every launch set up scratch for the whole grid (microseconds per launch);
    the kernels are written to fit the register file, and a change that spills must not go unnoticed."""
    _, remarks = compiled
    name, seen = None, {}
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name:
            seen[name] = int(m.group(1))
    decode = {k: v for k, v in seen.items() if "decode_kernel" in k}
    # head_dim 64 / 128 x 2 partial formats x (1..3 row tiles per wave, and the variant for launches without shared-prefix work)
    assert len(decode) == 16, sorted(seen)
    assert all(v == 0 for v in decode.values()), {k: v for k, v in decode.items() if v}


def test_no_vector_read_of_a_matrix_result_inside_its_latency(compiled):
    """Every control-flow path from every matrix instruction of every decode kernel variant keeps NEED wait
    states before a vector-ALU instruction reads what it wrote."""
    asm, _ = compiled
    findings, kernels = scan(asm)
    assert kernels == 16
    assert not findings, "\n".join(f"{k}: {blk}: `{mfma}` then `{reader}` after {ws} wait states (need {NEED})"
                                   for k, blk, mfma, reader, ws in findings[:10])


def test_the_scanner_sees_a_planted_hazard():
    """The scanner itself: a matrix result copied after two branches and three scalar instructions is
    reported, the same with enough wait states written out is not, and a write in between ends the dependence."""
    def kernel(filler):
        return "\n".join(["_ZN5taper13decode_kernelILi64ELi2ELi0EEEvNS_8StepArgsE:",
                          "\tv_mfma_f32_16x16x32_bf16 v[108:111], v[60:63], v[146:149], v[108:111]",
                          "\ts_cbranch_vccnz .LBB0_2", ".LBB0_1:", "\ts_branch .LBB0_3", ".LBB0_2:", "\ts_mov_b64 s[8:9], 0",
                          *filler, "\tv_mov_b64_e32 v[2:3], v[108:109]", ".LBB0_3:", "\ts_endpgm"])
    bad, n = scan(kernel(["\ts_and_b64 vcc, exec, s[88:89]"]))
    assert n == 1 and len(bad) == 1 and bad[0][4] == 3 and "v_mov_b64" in bad[0][3]
    good, _ = scan(kernel(["\ts_nop 5"]))
    assert good == []
    overwritten, _ = scan(kernel(["\tv_mov_b64_e32 v[108:109], v[4:5]", "\tv_mov_b64_e32 v[110:111], v[6:7]"]))
    assert [f for f in overwritten if f[1] == ".LBB0_2" and "v[2:3]" in f[3]] == []

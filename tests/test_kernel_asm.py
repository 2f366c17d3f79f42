"""Static checks on the device code of the four-wave GEMM kernel (no GPU needed: hipcc cross-compiles).

Its K loop keeps 256 accumulators in AGPRs through inline-assembly MFMAs with one wave per SIMD; two things the
compiler may do when register allocation gets tight would ruin it without failing any numerical test outright:
spilling inside the loop (the loop then waits on scratch memory), and moving accumulators with v_accvgpr_write /
v_accvgpr_mov right in front of an inline MFMA (whose read-after-write hazard the compiler does not pad, since it
cannot see the instruction).  Both are looked for in the assembly of every instantiation."""
import re
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
CSRC = ROOT / "paper_2209_13258_amd" / "csrc"


@pytest.fixture(scope="module")
def gemm_asm(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not Path(hipcc).exists():
        pytest.skip("hipcc not found")
    out = tmp_path_factory.mktemp("asm") / "osdp_gemm.s"
    cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           f"-I{ROOT / 'include'}", f"-I{CSRC}", "-S", "--cuda-device-only", str(CSRC / "osdp_gemm.hip"), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    return out.read_text().split("\n")


def _kernels(lines):
    """{mangled name: list of instruction lines} for the four-wave kernels."""
    kernels, cur = {}, None
    for line in lines:
        m = re.match(r"^(_ZN4osdp\S*gemm_w4_kernel\S*):", line)
        if m:
            cur = m.group(1)
            kernels[cur] = []
            continue
        if re.match(r"^\S+:", line) and not line.startswith(".L"):   # another function starts
            cur = None
        t = line.strip()
        if cur and t and not t.startswith((";", ".")):
            kernels[cur].append(t)
    return kernels


def test_four_wave_kernels_keep_their_k_loop_free_of_scratch_and_accumulator_moves(gemm_asm):
    kernels = _kernels(gemm_asm)
    assert len(kernels) >= 12, "the four-wave kernel's instantiations were not found in the assembly"
    for name, ins in kernels.items():
        mfma = [i for i, t in enumerate(ins) if t.startswith("v_mfma")]
        assert len(mfma) == 128, f"{name}: expected one K block of 128 MFMAs, found {len(mfma)} (the loop body was duplicated?)"
        body = ins[mfma[0]:mfma[-1] + 1]
        assert not [t for t in body if t.startswith("scratch_")], f"{name}: scratch traffic inside the K loop"
        for i in mfma:
            near = ins[max(0, i - 3):i]
            assert not [t for t in near if t.startswith(("v_accvgpr_write", "v_accvgpr_mov"))], \
                f"{name}: an accumulator register is written right in front of an inline MFMA"

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


def _kernels(lines, kernel="gemm_w4_kernel"):
    """{mangled name: list of instruction lines} for the instantiations of one kernel template."""
    kernels, cur = {}, None
    for line in lines:
        m = re.match(r"^(_ZN4osdp\S*" + kernel + r"I\S*):", line)
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


def _vgprs(operand):
    """The VGPR numbers an operand like v7 or v[8:11] names (empty for anything else)."""
    m = re.fullmatch(r"v(\d+)", operand)
    if m:
        return {int(m.group(1))}
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", operand)
    return set(range(int(m.group(1)), int(m.group(2)) + 1)) if m else set()


def _assert_no_valu_write_in_front_of_its_mfma(name, ins, mfma):
    """An MFMA may not read a register in the two cycles after a VALU instruction wrote it; the compiler pads none
    for an MFMA it cannot see."""
    for i in mfma:
        ops = [o.strip() for o in ins[i].split(None, 1)[1].split(",")]
        srcs = _vgprs(ops[1]) | _vgprs(ops[2])
        for t in ins[max(0, i - 2):i]:
            if t.startswith("v_") and not t.startswith("v_mfma"):
                dst = t.split(None, 1)[1].split(",")[0].strip()
                assert not (_vgprs(dst) & srcs), f"{name}: '{t}' writes a source of the MFMA that follows it"


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
        _assert_no_valu_write_in_front_of_its_mfma(name, ins, mfma)


def test_persistent_four_wave_kernels_use_no_scratch_and_respect_the_mfma_hazards(gemm_asm):
    """The persistent form runs its epilogue and the start of the next tile inside the loop over K blocks, where the
    compiler has no register to spare: any spill there, any accumulator moved by the compiler, or a source
    register of an inline MFMA written by a VALU instruction just before it (two wait states are needed, and the
    compiler pads none for an instruction it cannot see) is a defect."""
    kernels = _kernels(gemm_asm, "gemm_w4p_kernel")
    assert len(kernels) >= 10, "the persistent kernel's instantiations were not found in the assembly"
    for name, ins in kernels.items():
        assert not [t for t in ins if t.startswith("scratch_")], f"{name}: scratch traffic"
        mfma = [i for i, t in enumerate(ins) if t.startswith("v_mfma")]
        # one K block of 128, plus 64 that clear the accumulators before the first tile and 64 between tiles
        # (instantiations that start from a stored partial sum load it instead)
        assert len(mfma) in (128, 256), f"{name}: {len(mfma)} MFMAs"
        for i in mfma:
            near = ins[max(0, i - 3):i]
            assert not [t for t in near if t.startswith(("v_accvgpr_write", "v_accvgpr_mov"))], \
                f"{name}: an accumulator register is written right in front of an inline MFMA"
        _assert_no_valu_write_in_front_of_its_mfma(name, ins, mfma)

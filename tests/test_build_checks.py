"""The build-time check that guards the asm MFMAs of the persistent GEMM (csrc/check_mfma_hazards.py), on small
hand-written listings: it must flag an accumulator touched too soon after an MFMA or written too late before one,
along straight-line code and across a branch, and accept the same code with enough wait states in between."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
spec = importlib.util.spec_from_file_location("check_mfma_hazards",
                                              os.path.join(ROOT, "paper_2410_03065_amd", "csrc", "check_mfma_hazards.py"))
chk = importlib.util.module_from_spec(spec)
spec.loader.exec_module(chk)

MFMA = "\tv_mfma_f32_16x16x32_bf16 a[8:11], v[0:3], v[4:7], a[8:11]"


def _problems(body):
    return chk.check_kernel("k", body.split("\n"))[1]


def test_read_right_after_mfma_is_flagged():
    assert _problems(MFMA + "\n\tv_accvgpr_read_b32 v9, a10\n")
    assert _problems(MFMA + "\n\ts_nop 7\n\tv_accvgpr_read_b32 v9, a10\n")          # 9 wait states: still too few
    assert not _problems(MFMA + "\n\ts_nop 15\n\ts_nop 3\n\tv_accvgpr_read_b32 v9, a10\n")
    assert not _problems(MFMA + "\n\tv_accvgpr_read_b32 v9, a12\n")                 # another register


def test_write_right_before_mfma_is_flagged():
    assert _problems("\tv_accvgpr_write_b32 a9, v1\n" + MFMA + "\n")
    assert not _problems("\tv_accvgpr_write_b32 a9, v1\n\ts_nop 3\n" + MFMA + "\n")
    assert _problems("\tv_accvgpr_mov_b32 a11, a40\n\ts_nop 0\n" + MFMA + "\n")


def test_mfma_to_mfma_on_the_same_accumulator_is_left_to_the_hardware():
    assert not _problems(MFMA + "\n" + MFMA + "\n")


def test_store_from_an_accumulator_counts_as_a_read():
    assert _problems(MFMA + "\n\tbuffer_store_dwordx4 a[8:11], v1, s[0:3], 0 offen\n")


def test_hazard_across_a_branch():
    body = MFMA + "\n\ts_cbranch_scc1 .LBB0_2\n\ts_nop 15\n\ts_nop 15\n.LBB0_2:\n\tv_accvgpr_read_b32 v9, a8\n"
    found = _problems(body)
    assert found and "branch" in found[0]
    # the fall-through path has its wait states: only the branch is reported
    assert all("branch" in f for f in found)


def test_counts_mfmas():
    assert chk.check_kernel("k", (MFMA + "\n" + MFMA + "\n").split("\n"))[0] == 2

"""The build-time ISA check of the attention kernels' inline-assembly LDS reads (paper_2602_01801_amd/asmcheck.py):
it must flag a register touched between an asm read and its wait, and nothing else."""
from paper_2602_01801_amd import asmcheck


def lines(text):
    return [l for l in text.strip("\n").split("\n")]


CLEAN = """
	;;#ASMSTART
	ds_read_b128 v[10:13], v1 offset:0
	;;#ASMEND
	;;#ASMSTART
	ds_read_b64_tr_b16 v[20:21], v2 offset:0
	;;#ASMEND
	v_add_u32_e32 v3, v4, v5
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
	v_mfma_f32_32x32x16_bf16 v[32:47], v[10:13], v[20:23], v[32:47]
"""


def test_clean_sequence_passes():
    assert asmcheck._check_lines(lines(CLEAN), False) == 0


def test_use_before_the_wait_is_flagged():
    bad = CLEAN.replace("v_add_u32_e32 v3, v4, v5", "v_mov_b32_e32 v3, v11")
    assert asmcheck._check_lines(lines(bad), False) == 1


def test_overwrite_before_the_wait_is_flagged():
    bad = CLEAN.replace("v_add_u32_e32 v3, v4, v5", "v_mov_b32_e32 v21, v4")
    assert asmcheck._check_lines(lines(bad), False) == 1


def test_counted_wait_releases_only_the_older_reads():
    text = """
	;;#ASMSTART
	ds_read_b128 v[10:13], v1 offset:0
	;;#ASMEND
	;;#ASMSTART
	ds_read_b128 v[14:17], v1 offset:64
	;;#ASMEND
	;;#ASMSTART
	s_waitcnt lgkmcnt(1)
	;;#ASMEND
	v_mov_b32_e32 v3, v10
	v_mov_b32_e32 v4, v14
"""
    assert asmcheck._check_lines(lines(text), False) == 1      # v14 is still in flight, v10 has landed


def test_accumulation_registers_are_tracked_too():
    text = """
	;;#ASMSTART
	ds_read_b128 a[4:7], v1 offset:0
	;;#ASMEND
	v_accvgpr_read_b32 v3, a5
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
	v_accvgpr_read_b32 v3, a5
"""
    assert asmcheck._check_lines(lines(text), False) == 1


def test_the_scan_ends_at_an_unconditional_jump():
    text = """
	;;#ASMSTART
	ds_read_b128 v[10:13], v1 offset:0
	;;#ASMEND
	s_branch .LBB0_9
.LBB0_8:
	v_mov_b32_e32 v10, 0
.LBB0_9:
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
"""
    assert asmcheck._check_lines(lines(text), False) == 0

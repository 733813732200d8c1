"""The inline assembly of the grouped GEMM (direct-to-LDS loads, the row scatter it carries) keeps the
hardware's wait states itself: no vector instruction writes a scalar register that an assembly
block's memory instruction reads fewer than five wait states later.  Checked on the compiled ISA
(hipcc cross-compiles without a GPU); the detector is exercised on hand-written snippets first.
A second detector follows every load that an assembly block leaves in flight (the carried scatter's row
pieces and positions) to the first wait that covers it, down both sides of every branch, and fails if
any instruction names the load's destination registers on the way: to the compiler those registers
hold their value as soon as the block ends."""
from paper_2509_25041_amd import asm_hazards


def test_detector_on_snippets():
    bad = """
	v_readlane_b32 s42, v214, 19
	v_readlane_b32 s43, v214, 20
	;;#ASMSTART
	global_load_dword v203, v160, s[42:43]
	;;#ASMEND
""".splitlines()
    n, found = asm_hazards.find_hazards(bad)
    assert n == 1 and len(found) == 2
    good = """
	v_readlane_b32 s42, v214, 19
	v_readlane_b32 s43, v214, 20
	;;#ASMSTART
	s_nop 4
	global_load_dword v203, v160, s[42:43]
	;;#ASMEND
	s_add_u32 s4, s4, s42
	;;#ASMSTART
	global_store_dwordx4 v1, v[2:5], s[4:5] nt
	;;#ASMEND
	v_readfirstlane_b32 s9, v3
	s_nop 1
	;;#ASMSTART
	s_mov_b32 m0, s9
	s_nop 3
	global_load_lds_dwordx4 v7, s[10:11]
	;;#ASMEND
""".splitlines()
    n, found = asm_hazards.find_hazards(good)
    assert n == 3 and found == []


def test_early_use_detector_on_snippets():
    bad = """
	;;#ASMSTART
	s_nop 4
	global_load_dwordx2 v[240:241], v153, s[54:55]
	;;#ASMEND
	s_cbranch_vccnz .LBB0_2
	v_add_u32_e32 v3, v4, v5
	s_waitcnt vmcnt(4)
	s_branch .LBB0_3
.LBB0_2:
	v_mov_b32_e32 v9, v241
	s_waitcnt vmcnt(0)
.LBB0_3:
	s_endpgm
""".splitlines()
    n, found = asm_hazards.find_early_uses(bad)
    assert n == 1 and len(found) == 1 and "v241" in found[0]
    good = """
	;;#ASMSTART
	s_nop 4
	global_load_dword v7, v1, s[2:3]
	global_load_dwordx4 v[8:11], v1, s[4:5]
	;;#ASMEND
	v_mfma_f32_32x32x16_bf16 a[0:15], v[20:23], v[24:27], a[0:15]
	;;#ASMSTART
	global_load_lds_dwordx4 v30, s[10:11]
	global_load_lds_dwordx4 v31, s[10:11]
	global_load_lds_dwordx4 v32, s[10:11]
	global_load_lds_dwordx4 v33, s[10:11]
	;;#ASMEND
	s_waitcnt vmcnt(4)
	v_readlane_b32 s9, v7, 0
	;;#ASMSTART
	global_load_dwordx4 v[12:15], v1, s[4:5] sc1
	s_waitcnt vmcnt(0)
	;;#ASMEND
	v_add_f32_e32 v12, v12, v13
	;;#ASMSTART
	global_load_lds_dwordx4 v7, s[10:11]
	;;#ASMEND
""".splitlines()
    n, found = asm_hazards.find_early_uses(good)
    assert n == 2 and found == []
    # a wait that leaves more operations in flight than were issued after the load does not cover it
    partial = """
	;;#ASMSTART
	global_load_dwordx2 v[40:41], v1, s[2:3]
	global_load_dword v7, v1, s[2:3]
	;;#ASMEND
	;;#ASMSTART
	global_load_lds_dwordx4 v9, s[10:11]
	;;#ASMEND
	s_waitcnt vmcnt(3)
	v_add_u32_e32 v3, v40, v5
	s_waitcnt vmcnt(0)
	v_add_u32_e32 v3, v7, v5
""".splitlines()
    n, found = asm_hazards.find_early_uses(partial)
    assert n == 2 and len(found) == 1 and "v40" in found[0]
    partial[8] = "\ts_waitcnt vmcnt(2)"       # two younger loads were issued: now the oldest has landed
    n, found = asm_hazards.find_early_uses(partial)
    assert n == 2 and found == []


def test_grouped_gemm_assembly_keeps_its_wait_states():
    n, found = asm_hazards.check("ffn.hip")
    assert n > 100          # the direct-to-LDS loads and the carried row scatter are all there
    assert found == [], "\n".join(found)


def test_loads_left_in_flight_are_not_touched_before_a_wait():
    n, found = asm_hazards.check_early_uses("ffn.hip")
    assert n >= 4           # the carried row scatter: a position load and a row piece per instantiation
    assert found == [], "\n".join(found)

"""The inline assembly of the grouped GEMM (direct-to-LDS loads, the row scatter it carries) keeps the
hardware's wait states itself: no vector instruction writes a scalar register that an assembly
block's memory instruction reads fewer than five wait states later.  Checked on the compiled ISA
(hipcc cross-compiles without a GPU); the detector is exercised on hand-written snippets first."""
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


def test_grouped_gemm_assembly_keeps_its_wait_states():
    n, found = asm_hazards.check("ffn.hip")
    assert n > 100          # the direct-to-LDS loads and the carried row scatter are all there
    assert found == [], "\n".join(found)

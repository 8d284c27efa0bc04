"""The kernels that keep loads in flight through inline asm must not let go of a load's destination register before
the wait that covers the load (paper_2410_12513_amd/asm_check.py): a check of the library's own assembly, on the CPU."""
from paper_2410_12513_amd import asm_check


def test_scan_finds_a_planted_reuse_and_accepts_the_covered_case():
    planted = """
_ZN5first6k_stepILi128ELb1EEEvNS_10StepParamsE: ; @_ZN5first6k_stepILi128ELb1EEEvNS_10StepParamsE
	;;#ASMSTART
	global_load_dwordx4 v[2:5], v[10:11], off
	;;#ASMEND
	;;#ASMSTART
	global_load_dwordx4 v[6:9], v[12:13], off    ; a comment
	;;#ASMEND
	s_waitcnt vmcnt(1)
	v_add_f32_e32 v20, v2, v3
	v_mov_b32_e32 v6, 0
	s_waitcnt vmcnt(0)
	v_add_f32_e32 v21, v6, v7
	s_endpgm
"""
    hits = asm_check.touched_in_flight(planted)
    assert len(hits) == 1 and hits[0][3] == [6] and "v_mov_b32" in hits[0][2]      # v[2:5] was covered by vmcnt(1), v6 was not


def test_scan_carries_loads_in_flight_around_a_loop_and_over_a_forward_jump():
    loop = """
_ZN5first6k_stepILi128EEEvNS_10StepParamsE:
	s_waitcnt vmcnt(0)
.LBB0_1:
	v_add_f32_e32 v20, v2, v20
	s_waitcnt vmcnt(0)
	;;#ASMSTART
	global_load_dwordx4 v[2:5], v[10:11], off
	;;#ASMEND
	s_cbranch_scc1 .LBB0_1
	s_waitcnt vmcnt(0)
	s_endpgm
"""
    hits = asm_check.touched_in_flight(loop)
    assert len(hits) == 1 and hits[0][3] == [2]          # requested at the tail, named at the head before the wait
    jump = """
_ZN5first6k_stepILi128EEEvNS_10StepParamsE:
	;;#ASMSTART
	global_load_dwordx4 v[2:5], v[10:11], off
	;;#ASMEND
	s_cbranch_scc1 .LBB0_2
	s_waitcnt vmcnt(0)
	v_add_f32_e32 v20, v2, v20
.LBB0_2:
	v_mov_b32_e32 v3, 0
	s_waitcnt vmcnt(0)
	s_endpgm
"""
    hits = asm_check.touched_in_flight(jump)
    assert len(hits) == 1 and hits[0][3] == [3]          # the jump skips the wait
    fine = """
_ZN5first6k_stepILi128EEEvNS_10StepParamsE:
.LBB0_1:
	;;#ASMSTART
	global_load_dwordx4 v[2:5], v[10:11], off
	;;#ASMEND
	s_waitcnt vmcnt(0)
	v_add_f32_e32 v20, v2, v20
	s_cbranch_scc1 .LBB0_1
	s_endpgm
"""
    assert not asm_check.touched_in_flight(fine)
    # a load the compiler issued itself is its own business (it waits before it reuses the register), but it counts in vmcnt
    managed = """
_ZN5first6k_stepILi128EEEvNS_10StepParamsE:
	;;#ASMSTART
	global_load_dwordx4 v[2:5], v[10:11], off
	;;#ASMEND
	global_load_dword v6, v[12:13], off
	s_waitcnt vmcnt(1)
	v_add_f32_e32 v20, v2, v20
	v_mov_b32_e32 v7, v6
	s_endpgm
"""
    assert not asm_check.touched_in_flight(managed)


def test_no_kernel_of_the_library_touches_a_load_destination_in_flight():
    asm = asm_check.assembly()
    seen = asm_check.kernels_seen(asm)
    assert all(n >= 1 for n in seen.values()), seen          # the walk must not be blind: every family of kernels is found
    hits = asm_check.touched_in_flight(asm)
    assert not hits, hits[:5]

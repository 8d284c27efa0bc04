"""The kernels that keep loads in flight through inline asm must not let go of a load's destination register before
the wait that covers the load (paper_2410_12513_amd/asm_check.py): a check of the library's own assembly, on the CPU."""
from paper_2410_12513_amd import asm_check


def test_scan_finds_a_planted_reuse_and_accepts_the_covered_case():
    planted = """
_ZN5first6k_stepILi128ELb1EEEvNS_10StepParamsE:
	global_load_dwordx4 v[2:5], v[10:11], off
	global_load_dwordx4 v[6:9], v[12:13], off
	s_waitcnt vmcnt(1)
	v_add_f32_e32 v20, v2, v3
	v_mov_b32_e32 v6, 0
	s_waitcnt vmcnt(0)
	v_add_f32_e32 v21, v6, v7
	s_endpgm
"""
    hits = asm_check.touched_in_flight(planted)
    assert len(hits) == 1 and hits[0][3] == [6] and "v_mov_b32" in hits[0][2]      # v[2:5] was covered by vmcnt(1), v6 was not


def test_no_kernel_of_the_library_touches_a_load_destination_in_flight():
    hits = asm_check.touched_in_flight(asm_check.assembly())
    assert not hits, hits[:5]

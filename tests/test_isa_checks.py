"""The static checks over the ISA of the kernels with inline assembly (hipcc -S, no GPU): every load that
may be in flight has its registers left alone, and no inline-assembly instruction reads a scalar register
too soon behind the vector instruction that wrote it."""
from paper_1804_02941_amd import isa_checks as ic


def test_the_kernels_with_inline_assembly_pass_both_checks():
    assert ic.check_sources(verbose=True) == 0


HAZARD = """
_ZN3dab4demoEv:
	v_cmp_ge_f32_e64 s[10:11], v0, v1
	s_and_b64 s[8:9], s[6:7], s[10:11]
	v_cndmask_b32_e64 v0, 0, 1, s[8:9]
	v_cmp_ne_u32_e64 s[10:11], 0, v0
	{between}
	;;#ASMSTART
	v_writelane_b32 v131, s10, 59
	;;#ASMEND
	s_endpgm
.Lfunc_end0:
"""


def test_the_scalar_read_check_sees_a_lane_write_right_behind_the_compare():
    (name, lines), = ic.kernels(HAZARD.format(between="v_mul_f32_e32 v2, v3, v4"))
    assert len(ic.scalar_read_hazards(lines)) == 1                  # one instruction in between: one wait state
    (name, lines), = ic.kernels(HAZARD.format(between="s_nop 1"))
    assert ic.scalar_read_hazards(lines) == []


IN_FLIGHT = """
_ZN3dab4demoEv:
	;;#ASMSTART
	buffer_load_dword v5, v1, s[0:3], 0 offen
	;;#ASMEND
	;;#ASMSTART
	buffer_load_dword v6, v1, s[0:3], 0 offen
	;;#ASMEND
	s_waitcnt vmcnt({n})
	v_add_u32_e32 v7, v5, v5
	s_waitcnt vmcnt(0)
	s_endpgm
.Lfunc_end0:
"""


def test_the_in_flight_check_sees_a_use_before_the_wait():
    (name, lines), = ic.kernels(IN_FLIGHT.format(n=2))
    assert len(ic.loads_in_flight(lines)) == 1                      # vmcnt(2) leaves both loads pending
    (name, lines), = ic.kernels(IN_FLIGHT.format(n=1))
    assert ic.loads_in_flight(lines) == []                          # the older load has landed


def test_the_sort_kernels_at_their_64_register_allocation_read_no_register_before_it_is_written():
    assert ic.check_estimators_without_the_reserved_register(verbose=True) == 0


UNWRITTEN = """
_ZN3dab4demoEv:
	v_mov_b32_e32 v1, 0
	s_cbranch_scc1 .LBB0_2
	v_mov_b32_e32 v2, 1
.LBB0_2:
	v_mov_b32_dpp v1, v0 row_shr:1 row_mask:0xf bank_mask:0xf
	v_add_u32_e32 v3, v1, v2
	s_endpgm
.Lfunc_end0:
"""


def test_the_read_before_write_check_sees_a_register_set_on_one_path_only():
    (name, lines), = ic.kernels(UNWRITTEN)
    bad = ic.reads_before_any_write(lines)
    assert len(bad) == 1 and bad[0][2] == [2]                      # v2 is set only when the branch is not taken

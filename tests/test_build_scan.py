"""The build scans the device assembly for scalar loads whose base may not be a multiple of four (the scalar
memory path drops the low two address bits).  The scanner against hand-written fragments."""
from paper_2311_15269_amd.build import misaligned_scalar_loads


def test_a_base_advanced_by_a_byte_index_is_reported():
    asm = """
.LBB0_1:
	v_readfirstlane_b32 s9, v3
	s_add_u32 s4, s34, s9
	s_addc_u32 s5, s35, 0
	s_load_dword s23, s[4:5], 0x10
"""
    assert misaligned_scalar_loads(asm) == ["6: s_load_dword s23, s[4:5], 0x10"]


def test_a_register_offset_is_reported():
    assert len(misaligned_scalar_loads("\ts_load_dword s2, s[4:5], s7\n")) == 1


def test_word_indices_and_whole_pointers_pass():
    asm = """
.LBB0_1:
	s_lshl_b64 s[4:5], s[92:93], 2
	s_add_u32 s6, s34, s4
	s_addc_u32 s7, s35, s5
	s_load_dword s22, s[6:7], 0x40
	s_mul_i32 s4, s92, 12
	s_add_u32 s4, s6, s4
	s_addc_u32 s5, s7, s5
	s_load_dword s23, s[4:5], 0xea0
	v_readlane_b32 s0, v252, 12
	v_readlane_b32 s1, v252, 13
	s_load_dwordx2 s[0:1], s[0:1], 0x0
	s_load_dword s3, s[0:1], 0x8
"""
    assert misaligned_scalar_loads(asm) == []


def test_a_product_with_an_odd_factor_is_reported():
    asm = """
.LBB0_1:
	s_mul_i32 s4, s92, 3
	s_add_u32 s4, s6, s4
	s_addc_u32 s5, s7, 0
	s_load_dword s23, s[4:5], 0x0
"""
    assert len(misaligned_scalar_loads(asm)) == 1

"""The build's check of the scorer's compiled code (paper_2601_07891_amd/isa_lint.py): on small
hand-written listings with a planted hazard of every kind it has to find it, and on clean ones
it has to stay silent.  CPU only; the real kernels are checked by build() itself."""
from paper_2601_07891_amd import isa_lint as L


def _lint(text):
    return [ins for _, ins in L.lint_kernel(text.strip().split("\n"))]


CLEAN = """
	global_load_dwordx4 v[10:13], v2, s[4:5] offset:0
	global_load_lds_dwordx4 v[20:21], off
	global_load_dwordx4 v[14:17], v2, s[4:5] offset:1024
	ds_read_b128 v[30:33], v5 offset:0
	v_add_u32_e32 v6, 1, v7                 ; unrelated registers
	s_waitcnt vmcnt(2)                      ; v[10:13] have arrived
	s_waitcnt lgkmcnt(0)
	v_mfma_f32_32x32x16_bf16 a[0:15], v[10:13], v[30:33], a[0:15]
	s_waitcnt vmcnt(0)
	v_mfma_f32_32x32x16_bf16 a[0:15], v[14:17], v[30:33], a[0:15]
"""


def test_clean_listing_has_no_finding():
    assert _lint(CLEAN) == []


def test_use_before_the_wait_is_found():
    text = CLEAN.replace("s_waitcnt vmcnt(2) ", "s_waitcnt vmcnt(3) ")    # one too many allowed
    assert _lint(text) == ["v_mfma_f32_32x32x16_bf16 a[0:15], v[10:13], v[30:33], a[0:15]"]


def test_copy_of_a_register_in_flight_is_found():
    text = CLEAN.replace("v_add_u32_e32 v6, 1, v7", "v_mov_b32_e32 v40, v12")
    assert _lint(text) == ["v_mov_b32_e32 v40, v12"]


def test_reuse_of_a_destination_as_scratch_is_found():
    text = CLEAN.replace("v_add_u32_e32 v6, 1, v7", "v_add_u32_e32 v15, 1, v7")
    assert _lint(text) == ["v_add_u32_e32 v15, 1, v7"]


def test_lds_read_consumed_before_lgkmcnt_is_found():
    text = CLEAN.replace("s_waitcnt lgkmcnt(0)\n", "s_waitcnt lgkmcnt(1)\n")
    assert len(_lint(text)) == 2          # both MFMAs read v[30:33]


def test_address_register_in_flight_is_found():
    text = """
	global_load_dwordx2 v[2:3], v[4:5], off
	global_load_dwordx4 v[10:13], v[2:3], off
	s_waitcnt vmcnt(0)
"""
    assert _lint(text) == ["global_load_dwordx4 v[10:13], v[2:3], off"]


def test_spill_of_a_register_in_flight_is_found():
    text = """
	global_load_dwordx4 v[10:13], v2, s[4:5] offset:0
	scratch_store_dword off, v11, off offset:16
	s_waitcnt vmcnt(0)
"""
    assert _lint(text) == ["scratch_store_dword off, v11, off offset:16"]


def test_counts_follow_issue_order():
    # three loads, vmcnt(1): the first two have arrived, the third has not
    text = """
	global_load_dwordx4 v[10:13], v2, s[4:5] offset:0
	global_load_dwordx4 v[14:17], v2, s[4:5] offset:1024
	global_load_dwordx4 v[18:21], v2, s[4:5] offset:2048
	s_waitcnt vmcnt(1)
	v_mov_b32_e32 v40, v10
	v_mov_b32_e32 v41, v17
	v_mov_b32_e32 v42, v18
"""
    assert _lint(text) == ["v_mov_b32_e32 v42, v18"]


def test_kernels_are_found_by_name():
    asm = """
	.text
_ZN5kvzap5otherEv:                      ; @_ZN5kvzap5otherEv
	global_load_dword v1, v[2:3], off
	v_mov_b32_e32 v4, v1
	s_endpgm
.Lfunc_end0:
_ZN5kvzap21score_mlp_frag_kernelILi4EEEvv: ; @_ZN5kvzap21score_mlp_frag_kernelILi4EEEvv
	global_load_dword v1, v[2:3], off
	s_waitcnt vmcnt(0)
	v_mov_b32_e32 v4, v1
	s_endpgm
.Lfunc_end1:
"""
    res = L.lint_scorer_asm(asm)
    assert list(res) == ["_ZN5kvzap21score_mlp_frag_kernelILi4EEEvv"] and res[list(res)[0]] == []
    res = L.lint_scorer_asm(asm, "other")
    assert [ins for _, ins in res["_ZN5kvzap5otherEv"]] == ["v_mov_b32_e32 v4, v1"]

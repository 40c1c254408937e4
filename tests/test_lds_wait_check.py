"""The build's check of hand-scheduled LDS reads (paper_2307_09782_amd/check_lds_waits.py) on small listings
written for the purpose: it must name a copy or a use of a register whose read is still in flight, on the
straight path and on a path through a branch, and accept the same code once the wait covers the read."""
import pytest

from paper_2307_09782_amd import check_lds_waits as chk

HEAD = "_ZN4zqfp11k_gemm_tileILi2EEEvPKh:\n"
TAIL = "\ts_endpgm\n.Lfunc_end0:\n"


def _run(body):
    return chk.check_kernel((HEAD + body + TAIL).splitlines()[1:])


def test_a_use_behind_a_sufficient_wait_is_accepted():
    body = """
	ds_read_b128 v[10:13], v1 offset:0
	ds_read_b32 v20, v2 offset:64
	ds_read_b128 v[14:17], v1 offset:1024
	s_waitcnt lgkmcnt(1)
	v_mov_b32_e32 v30, v20
	v_mfma_scale_f32_16x16x128_f8f6f4 v[40:43], v[50:57], v[10:13], 0, v60, v20 op_sel_hi:[0,0,0] blgp:4
	s_waitcnt lgkmcnt(0)
	v_mov_b64_e32 v[32:33], v[14:15]
"""
    assert _run(body) == []


def test_a_copy_ahead_of_the_wait_is_named():
    body = """
	ds_read_b128 v[10:13], v1 offset:0
	ds_read_b128 v[14:17], v1 offset:1024
	s_waitcnt lgkmcnt(1)
	v_mov_b64_e32 v[32:33], v[14:15]
	s_waitcnt lgkmcnt(0)
"""
    found = _run(body)
    assert len(found) == 1 and found[0][2] == [14, 15] and "v_mov_b64" in found[0][1]


def test_a_read_in_flight_across_a_branch_is_followed_into_both_arms():
    body = """
	ds_read_b128 v[10:13], v1 offset:0
	s_cbranch_vccz .LBB0_2
	v_mov_b32_e32 v5, v10
	s_waitcnt lgkmcnt(0)
	s_branch .LBB0_3
.LBB0_2:
	s_waitcnt lgkmcnt(0)
	v_mov_b32_e32 v5, v10
.LBB0_3:
	v_add_u32_e32 v6, v5, v11
"""
    found = _run(body)
    assert [f[1] for f in found] == ["v_mov_b32_e32 v5, v10"] and found[0][0] == 2


def test_an_address_register_that_is_still_arriving_is_named_and_lds_writes_take_a_place_in_the_count():
    body = """
	ds_read_b32 v7, v1 offset:0
	ds_write_b32 v2, v3
	s_waitcnt lgkmcnt(1)
	ds_read_b32 v8, v7 offset:0
	s_waitcnt lgkmcnt(0)
"""
    assert _run(body) == []
    assert len(_run(body.replace("lgkmcnt(1)", "lgkmcnt(2)"))) == 1


def test_a_loop_that_only_writes_lds_ends_the_walk():
    body = """
.LBB0_1:
	ds_write_b32 v2, v3
	s_cbranch_scc1 .LBB0_1
	s_waitcnt lgkmcnt(0)
"""
    assert _run(body) == []


def test_check_text_raises_with_the_kernel_and_the_instruction():
    text = HEAD + "\tds_read_b32 v7, v1 offset:0\n\tv_mov_b32_e32 v9, v7\n" + TAIL
    with pytest.raises(RuntimeError, match="v_mov_b32_e32 v9, v7"):
        chk.check_text(text, "k_gemm_tile")
    with pytest.raises(RuntimeError, match="no kernel"):
        chk.check_text(text, "k_other")
    assert chk.check_text(text.replace("\tv_mov", "\ts_waitcnt lgkmcnt(0)\n\tv_mov"), "k_gemm_tile") == 1

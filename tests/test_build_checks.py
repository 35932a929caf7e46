"""The build's two checks of the hand-issued loads (CPU only): no kernel may spill, and in the generated
assembly no instruction may name a register that still has a load in flight."""
import pytest

from paper_2401_14112_amd import build

KERNEL = "_Z6kernelv:\n"


def _problems(body):
    return build.loads_in_flight_problems(KERNEL + body)


def test_copy_of_a_register_in_flight_is_reported():
    # what a compiler does with a loop-carried value it could not keep in place
    body = """
        buffer_load_dwordx4 v[36:39], v80, s[0:3], 0 offen offset:0x400 nt
        v_xor_b32_e32 v12, v12, v28
        v_mov_b32_e32 v8, v36
        s_waitcnt vmcnt(0)
    """
    p = _problems(body)
    assert len(p) == 1 and p[0][0] == "_Z6kernelv" and "v_mov_b32_e32 v8, v36" in p[0][2] and "buffer_load" in p[0][3]
    with pytest.raises(RuntimeError, match="load in flight"):
        build.check_loads_in_flight(KERNEL + body)


def test_write_into_a_register_in_flight_is_reported():
    assert len(_problems("global_load_dword v5, v[2:3], off\n v_mov_b32_e32 v5, 0\n s_waitcnt vmcnt(0)\n")) == 1


def test_after_the_wait_the_register_is_free():
    assert _problems("buffer_load_dword v5, v8, s[0:3], 0 offen\n s_waitcnt vmcnt(0)\n v_add_u32_e32 v6, v5, v5\n") == []
    assert _problems("buffer_load_dword v5, v8, s[0:3], 0 offen\n s_waitcnt vmcnt(0) lgkmcnt(0)\n v_add_u32_e32 v6, v5, v5\n") == []
    # a wait for another counter frees nothing
    assert len(_problems("buffer_load_dword v5, v8, s[0:3], 0 offen\n s_waitcnt lgkmcnt(0)\n v_add_u32_e32 v6, v5, v5\n")) == 1


def test_loads_complete_in_order():
    body = """
        buffer_load_dwordx4 v[0:3], v9, s[0:3], 0 offen
        buffer_load_dwordx4 v[4:7], v9, s[0:3], 0 offen offset:1024
        s_waitcnt vmcnt(1)
        v_xor_b32_e32 v10, v0, v3
        %s
        s_waitcnt vmcnt(0)
        v_xor_b32_e32 v10, v4, v7
    """
    assert _problems(body % "") == []
    assert len(_problems(body % "v_xor_b32_e32 v10, v10, v6")) == 1


def test_stores_and_copies_to_lds_count_as_requests_without_a_destination():
    body = """
        buffer_load_dwordx4 v[0:3], v9, s[0:3], 0 offen
        buffer_load_dwordx4 v9, s[4:7], 0 offen offset:0 lds
        global_store_dword v[20:21], v22, off
        s_waitcnt vmcnt(2)
        v_mov_b32_e32 v30, v0
        v_mov_b32_e32 v31, v9
        v_mov_b32_e32 v32, v22
    """
    assert _problems(body) == []
    assert len(_problems(body.replace("vmcnt(2)", "vmcnt(3)"))) == 1


def test_the_address_register_may_be_the_destination_of_its_own_load():
    assert _problems("buffer_load_dwordx4 v[52:55], v52, s[0:3], 0 offen\n s_waitcnt vmcnt(0)\n") == []


def test_undefined_high_half_of_a_64_bit_addend_is_exempt():
    body = """
        v_and_b32_e32 v152, 48, v2
        buffer_load_dword v153, v8, s[24:27], 0 offen offset:0
        v_mad_u64_u32 v[6:7], s[4:5], s8, v2, v[152:153]
        s_waitcnt vmcnt(0)
    """
    assert _problems(body) == []
    # the low half and the other operands are not
    assert len(_problems(body.replace("v_and_b32_e32 v152, 48, v2", "").replace("v153, v8", "v152, v8"))) == 1
    assert len(_problems(body.replace("s8, v2, v[152:153]", "s8, v153, v[152:153]"))) == 1


def test_state_is_per_kernel_and_code_after_a_jump_starts_clean():
    two = KERNEL + "buffer_load_dword v5, v8, s[0:3], 0 offen\n s_endpgm\n_Z5otherv:\n v_mov_b32_e32 v6, v5\n s_endpgm\n"
    assert build.loads_in_flight_problems(two) == []
    jump = "buffer_load_dword v5, v8, s[0:3], 0 offen\n s_branch .LBB0_2\n.LBB0_1:\n v_mov_b32_e32 v6, v5\n.LBB0_2:\n s_waitcnt vmcnt(0)\n"
    assert _problems(jump) == []
    fall = "buffer_load_dword v5, v8, s[0:3], 0 offen\n.LBB0_1:\n v_mov_b32_e32 v6, v5\n s_waitcnt vmcnt(0)\n"
    assert len(_problems(fall)) == 1


def test_scratch_is_refused():
    ok = ["remark: Function Name: k [-Rpass-analysis]", "remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis]"]
    build.check_no_scratch(ok)
    with pytest.raises(RuntimeError, match="spills 16 bytes"):
        build.check_no_scratch([ok[0], ok[1].replace(": 0", ": 16")])

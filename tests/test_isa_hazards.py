"""The hazards the hand-written assembly is responsible for, checked in the generated instruction stream (no GPU):
`isa_check` compiles the backward source for gfx950 and walks the assembly; planted violations show that the checks
would see one."""
import os

import pytest

from paper_2510_18121_amd import isa_check as C

pytestmark = pytest.mark.skipif(not os.path.exists(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")),
                                reason="hipcc is needed to produce the assembly")


@pytest.fixture(scope="module")
def bwd_asm():
    return C.compile_to_asm("ca_bwd.hip")


def test_mfma_chains_are_left_alone_until_they_end(bwd_asm):
    bodies = C.kernel_bodies(bwd_asm, "ca_bwd_dkv_kernel")
    assert len(bodies) == 2  # head_dim 128 and 64
    for body in bodies:
        n, marks, bad = C.check_mfma_chains(body)
        # the kernel holds its body twice (units that run alone, chains of units).  Per body: chains before the loop, in
        # the loop (two, ended by markers) and on the diagonal; the compiler may keep two copies of a loop (one per
        # value of a condition that does not change inside it)
        assert n >= 8 and marks in (4, 6, 8)
        assert not bad, bad


def test_no_vector_instruction_reads_a_transcendental_in_the_next_slot(bwd_asm):
    n, bad = C.check_trans_use(bwd_asm)
    assert n > 100
    assert not bad, bad


def test_forward_kernel_transcendentals_and_chains():
    asm = C.compile_to_asm("ca_fwd.hip")
    n, bad = C.check_trans_use(asm)
    assert n > 50 and not bad, bad
    bodies = C.kernel_bodies(asm, "ca_fwd_kernel")
    assert len(bodies) == 2  # head_dim 128 and 64
    for body in bodies:
        # score chains of the pipelined steps, of the prologue and of the diagonal path, every one ended by wait states
        n, marks, bad = C.check_mfma_chains(body)
        assert n >= 6 and marks == 0
        assert not bad, bad
        # the pipelined loop keeps everything in registers
        assert "scratch_" not in body


M = "v_mfma_f32_32x32x16_bf16"


def test_planted_violations_are_found():
    chain = f"""
	{M} v[0:15], v[40:43], a[0:3], 0
	{M} v[16:31], v[44:47], a[4:7], v[60:75]
	{M} v[0:15], v[48:51], a[8:11], v[0:15]
"""
    ok = chain + "\ts_nop 11\n\tv_add_f32_e32 v90, v3, v4\n"
    assert C.check_mfma_chains(ok) == (1, 0, [])
    early = chain + "\tv_add_f32_e32 v90, v3, v4\n\ts_nop 11\n"
    assert len(C.check_mfma_chains(early)[2]) == 1
    branch = chain + ".LBB0_3:\n\ts_nop 11\n"
    assert len(C.check_mfma_chains(branch)[2]) == 1
    # a marker instead of wait states: the registers must stay untouched for 16 issue cycles
    far = chain + "\t; chain end\n" + "\tv_mov_b32_e32 v91, v92\n" * 16 + "\tv_add_f32_e32 v90, v3, v4\n"
    assert C.check_mfma_chains(far) == (1, 1, [])
    near = chain + "\t; chain end\n" + "\tv_mov_b32_e32 v91, v92\n" * 5 + "\tv_add_f32_e32 v90, v3, v4\n"
    assert len(C.check_mfma_chains(near)[2]) == 1
    two_mfmas_later = chain + "\t; chain end\n" + f"\t{M} a[0:15], v[40:43], v[44:47], a[0:15]\n" * 2 + "\tv_add_f32_e32 v90, v3, v4\n"
    assert C.check_mfma_chains(two_mfmas_later) == (1, 1, [])
    assert C.check_trans_use("\tv_exp_f32_e32 v5, v6\n\tv_add_f32_e32 v7, v5, v8\n")[1]
    assert not C.check_trans_use("\tv_exp_f32_e32 v5, v6\n\ts_nop 0\n\tv_add_f32_e32 v7, v5, v8\n")[1]
    assert not C.check_trans_use("\tv_exp_f32_e32 v5, v6\n\tv_add_f32_e32 v7, v9, v8\n")[1]
    assert not C.check_trans_use("\tv_exp_f32_e32 v5, v6\n\tv_exp_f32_e32 v7, v5\n")[1]

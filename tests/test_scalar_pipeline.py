"""The static checker of the hand-issued scalar loads (tests/scalar_pipeline_check.py): first the
checker itself on tiny hand-written assembly (a planted violation must be found, on a straight
path and around a loop), then the branch kernels of all eight activation widths -- the assembly
the library build kept beside its objects, i.e. the code that is in libqnn.so."""
import os
import shutil
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import scalar_pipeline_check as chk  # noqa: E402


def kernel(body):
    lines = ["_ZN3qnn4test_kernelEv:"] + body + ["\ts_endpgm", ".Lfunc_end0:"]
    name = lines[0][:-1]
    return chk.check_kernel(name, list(enumerate(lines[1:], 2)))[0]


ASM_LOAD = [";;#ASMSTART", "\ts_load_dwordx4 s[8:11], s[0:1], s2 offset:0", ";;#ASMEND"]
ASM_WAIT = [";;#ASMSTART", "\ts_waitcnt lgkmcnt(0)", ";;#ASMEND"]


def test_checker_accepts_a_use_after_the_wait():
    assert kernel(ASM_LOAD + ["\tv_mov_b32_e32 v1, s3"] + ASM_WAIT + ["\tv_xor_b32_e32 v0, s8, v1"]) == []


def test_checker_flags_a_use_before_the_wait():
    p = kernel(ASM_LOAD + ["\tv_xor_b32_e32 v0, s9, v1"] + ASM_WAIT)
    assert len(p) == 1 and "[9]" in p[0] and "v_xor_b32_e32" in p[0]


def test_checker_flags_a_spill_of_a_register_in_flight():
    p = kernel(ASM_LOAD + ["\tv_writelane_b32 v40, s10, 3"] + ASM_WAIT)
    assert len(p) == 1 and "v_writelane_b32" in p[0]


def test_checker_follows_the_back_edge_of_a_loop():
    # the load at the bottom of the loop body is still in flight at its top on the second trip
    body = [".LBB0_1:", "\tv_xor_b32_e32 v0, s8, v1"] + ASM_LOAD + ["\ts_cmp_lg_u32 s4, 0", "\ts_cbranch_scc1 .LBB0_1"] + ASM_WAIT
    p = kernel(body)
    assert len(p) == 1 and "v_xor_b32_e32" in p[0]
    # with the wait at the top of the body the same loop is clean
    body = [".LBB0_1:"] + ASM_WAIT + ["\tv_xor_b32_e32 v0, s8, v1"] + ASM_LOAD + ["\ts_cmp_lg_u32 s4, 0", "\ts_cbranch_scc1 .LBB0_1"] + ASM_WAIT
    assert kernel(body) == []


def test_checker_ignores_compiler_issued_loads():
    # a load outside an asm block is tracked by the compiler's own waits
    assert kernel(["\ts_load_dwordx2 s[8:9], s[0:1], 0x0", "\ts_waitcnt lgkmcnt(0)", "\tv_mov_b32_e32 v0, s8"]) == []


def test_checker_tells_reserved_from_used_scratch(tmp_path):
    """A kernel that only reserves scratch (the allocator's emergency slot) passes; one whose code
    addresses it does not."""
    def asm_file(body):
        text = ["_ZN3qnn6a_kernelEv:"] + body + ["\ts_endpgm", ".Lfunc_end0:", "\t.amdhsa_kernel _ZN3qnn6a_kernelEv",
                                                  "\t\t.amdhsa_private_segment_fixed_size 20", "\t.end_amdhsa_kernel"]
        f = tmp_path / "k.s"
        f.write_text("\n".join(text))
        return str(f)
    assert chk.check_file(asm_file(["\tv_mov_b32_e32 v0, 0"]))[1] == []
    assert len(chk.check_file(asm_file(["\tscratch_store_dword off, v0, off offset:4"]))[1]) == 1
    assert len(chk.check_file(asm_file(["\tbuffer_store_dword v0, off, s[0:3], 0 offset:4"]))[1]) == 1


@pytest.fixture(scope="module")
def asm():
    tmp = tempfile.mkdtemp(prefix="qnn_asm_test_")
    try:
        yield chk.asm_files(tmp)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


@pytest.mark.timeout(1800)
@pytest.mark.skipif(shutil.which(chk.HIPCC) is None and not os.path.exists(chk.HIPCC), reason="hipcc not available")
@pytest.mark.parametrize("ab", range(1, 9))
def test_branch_kernels_are_clean(asm, ab):
    """Every 3x3 / GEMM kernel (all weight widths, all chunk shapes) and the small-channel kernels of
    one activation width: no register with a hand-issued load in flight is touched, no scratch."""
    total = 0
    for src in chk.SOURCES:
        nk, problems, _ = chk.check_file(asm[(src, ab)])
        assert problems == [], problems[:5]
        total += nk
    assert total >= 60

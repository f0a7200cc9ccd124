"""The build refuses generated code that would break the tiled GEMM's hand-kept load accounting."""
import os
import tempfile

import pytest

from paper_2511_17826_amd import build as b


def _check(text):
    f = tempfile.NamedTemporaryFile("w", suffix=".s", delete=False)
    f.write(text)
    f.close()
    try:
        b.check_generated_code(f.name)
    finally:
        os.unlink(f.name)


HEAD = "_ZN4tbik17gemm_tiled_kernelILi4EEEvNS_11TiledParamsE:\n"


def test_clean_code_passes():
    _check(HEAD + "\tv_mov_b32 v0, v1\n\ts_add_i32 m0, s1, s2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v1, s[2:3]\n\ts_endpgm\n")
    _check("_ZN4tbik14rmsnorm_kernelEv:\n\tscratch_load_dword v0, off, off\n\ts_endpgm\n")      # other kernels may spill


def test_scratch_traffic_in_the_tiled_gemm_is_refused():
    with pytest.raises(RuntimeError, match="scratch"):
        _check(HEAD + "\tscratch_store_dword off, v0, off\n\ts_endpgm\n")


def test_labels_with_a_trailing_comment_are_recognised():
    """The compiler writes 'name: ; @name'; the checker must still know which kernel it is in."""
    head = "_ZN4tbik17gemm_tiled_kernelILi4EEEvNS_11TiledParamsE: ; @_ZN4tbik17gemm_tiled_kernelILi4EEEvNS_11TiledParamsE\n"
    with pytest.raises(RuntimeError, match="scratch"):
        _check(head + "\tscratch_load_dword v0, off, off offset:4 ; 4-byte Folded Reload\n\ts_endpgm\n")
    f = tempfile.NamedTemporaryFile("w", suffix=".s", delete=False)
    f.write("_ZN4tbik25attention_pingpong_kernelILb1ELi4EEEvNS_10AttnParamsE: ; @x\n\tscratch_store_dword off, v0, off\n\ts_endpgm\n")
    f.close()
    try:
        with pytest.raises(RuntimeError, match="scratch"):
            b.check_generated_code(f.name, "attention_")
    finally:
        os.unlink(f.name)


def test_m0_write_without_wait_state_is_refused():
    with pytest.raises(RuntimeError, match="m0"):
        _check(HEAD + "\ts_mov_b32 m0, s4\n\tglobal_load_lds_dwordx4 v1, s[2:3]\n\ts_endpgm\n")


def test_the_built_library_passed_the_check():
    asm = os.path.join(b.BUILD, "gemm_tiled-hip-amdgcn-amd-amdhsa-gfx950.s")
    if not os.path.exists(asm):
        pytest.skip("no assembly kept from the last build")
    b.check_generated_code(asm)
    b.check_generated_code(os.path.join(b.BUILD, "attention-hip-amdgcn-amd-amdhsa-gfx950.s"), "attention_")
    b.check_generated_code(os.path.join(b.BUILD, "gemm_f32-hip-amdgcn-amd-amdhsa-gfx950.s"), "gemm_f32_tiled_kernel")

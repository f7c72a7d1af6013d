"""The hand-placed MFMAs must keep the data-hazard distances the compiler cannot enforce for
inline asm.  Checked on the gfx950 assembly of the library sources (no GPU needed)."""
import pytest

from paper_2409_04431_amd import isa_check

_HEAD = "kernel_x:\n"
_MFMA = "\t;;#ASMSTART\n\tv_mfma_f32_32x32x16_bf16 v[0:15], v[20:23], a[4:7], v[0:15]\n\t;;#ASMEND\n"


def test_scanner_flags_valu_write_right_before_asm_mfma():
    txt = _HEAD + "\tv_accvgpr_read_b32 v21, a9\n" + _MFMA + "\ts_endpgm\n"
    msgs = isa_check.check_text(txt)
    assert len(msgs) == 1 and "rule A" in msgs[0]
    ok = _HEAD + "\tv_accvgpr_read_b32 v21, a9\n\ts_nop 1\n" + _MFMA + "\ts_endpgm\n"
    assert isa_check.check_text(ok) == []
    ok2 = _HEAD + "\tv_accvgpr_read_b32 v21, a9\n\tv_add_u32_e32 v40, v41, v42\n\ts_add_i32 s0, s0, 1\n" + _MFMA + "\ts_endpgm\n"
    assert isa_check.check_text(ok2) == []


def test_scanner_flags_early_read_of_asm_mfma_result():
    txt = _HEAD + _MFMA + "\tv_add_f32_e32 v30, v31, v32\n\tv_accvgpr_write_b32 a100, v15\n\ts_endpgm\n"
    msgs = isa_check.check_text(txt)
    assert len(msgs) == 1 and "rule B" in msgs[0]
    ok = _HEAD + _MFMA + "\ts_nop 15\n\tv_accvgpr_write_b32 a100, v15\n\ts_endpgm\n"
    assert isa_check.check_text(ok) == []
    # an independent MFMA in between occupies the matrix pipe for its 8 passes
    other = "\tv_mfma_f32_32x32x16_bf16 v[64:79], v[20:23], a[4:7], v[64:79]\n"
    ok2 = _HEAD + _MFMA + other + other + "\tv_accvgpr_write_b32 a100, v15\n\ts_endpgm\n"
    assert isa_check.check_text(ok2) == []


def test_scanner_ignores_compiler_emitted_mfma():
    txt = _HEAD + "\tv_accvgpr_read_b32 v21, a9\n\tv_mfma_f32_32x32x16_bf16 v[0:15], v[20:23], a[4:7], v[0:15]\n\ts_endpgm\n"
    assert isa_check.check_text(txt) == []


def test_scanner_flags_m0_write_outside_asm_next_to_lds_dma():
    dma = "\t;;#ASMSTART\n\ts_mov_b32 m0, s5\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v3, s[8:9]\n\t;;#ASMEND\n"
    more = "\t;;#ASMSTART\n\tglobal_load_lds_dwordx4 v4, s[8:9] offset:1024\n\t;;#ASMEND\n"
    assert isa_check.check_text(_HEAD + dma + "\tv_add_u32_e32 v40, v41, v42\n" + more + "\ts_endpgm\n") == []
    msgs = isa_check.check_text(_HEAD + dma + "\ts_mov_b32 m0, -1\n" + more + "\ts_endpgm\n")
    assert len(msgs) == 1 and "rule C" in msgs[0]
    # without such loads in the function the compiler may use M0 as it likes
    assert isa_check.check_text(_HEAD + "\ts_mov_b32 m0, -1\n\ts_endpgm\n") == []


def test_library_kernels_have_no_mfma_hazard():
    asm = isa_check.compile_to_asm()
    n_asm_mfma = sum(1 for _, insts in isa_check.parse_functions(asm) for i in insts if i.is_mfma and i.in_asm)
    assert n_asm_mfma > 1000  # the pinned forward and backward steps are in there
    assert isa_check.check_text(asm) == []

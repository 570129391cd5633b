"""The two checks build.py runs on the generated assembly of the unit score kernel, on planted text: compiler code
must stay off the accumulation registers the kernel reserves, and no ALU write may stand within two issue slots of
the matrix instruction that reads it."""
import pytest

from paper_2410_01518_amd import build

GOOD = """
\tv_cvt_pk_bf16_f32 v85, v24, v25
\ts_nop 1
\t;;#ASMSTART
\tv_mfma_f32_32x32x16_bf16 v[34:49], v[82:85], a[0:3], 0
\t;;#ASMEND
\tv_add_f32_e32 v100, v2, v3
\tv_add_f32_e32 v104, v2, v3
\t;;#ASMSTART
\tv_mfma_f32_32x32x16_bf16 v[2:17], v[0:3], a[32:35], v[2:17]
\t;;#ASMEND
\t;;#ASMSTART
\tglobal_load_dwordx4 a[8:11], v[20:21], off offset:32
\t;;#ASMEND
"""


def _write(tmp_path, text):
    p = tmp_path / "k.s"
    p.write_text(text)
    return str(p)


def test_clean_text_passes(tmp_path):
    p = _write(tmp_path, GOOD)
    build.check_acc_registers_untouched(p)
    build.check_matrix_operand_distance(p)


@pytest.mark.parametrize("gap", ["", "\tv_mov_b32_e32 v200, v201\n"])
def test_alu_write_directly_before_the_matrix_instruction_that_reads_it_is_refused(tmp_path, gap):
    text = "\tv_cvt_pk_bf16_f32 v85, v24, v25\n" + gap + "\tv_mfma_f32_32x32x16_bf16 v[34:49], v[82:85], a[0:3], 0\n"
    with pytest.raises(RuntimeError, match="matrix instruction"):
        build.check_matrix_operand_distance(_write(tmp_path, text))


def test_two_slots_in_between_are_enough_and_the_accumulator_operand_does_not_count(tmp_path):
    ok = ("\tv_cvt_pk_bf16_f32 v85, v24, v25\n\tv_mov_b32_e32 v200, v201\n\tv_mov_b32_e32 v202, v201\n"
          "\tv_mfma_f32_32x32x16_bf16 v[34:49], v[82:85], a[0:3], 0\n"
          "\tv_add_f32_e32 v40, v1, v2\n\tv_mfma_f32_32x32x16_bf16 v[34:49], v[86:89], a[0:3], v[34:49]\n")
    build.check_matrix_operand_distance(_write(tmp_path, ok))


def test_compiler_code_on_an_accumulation_register_is_refused(tmp_path):
    with pytest.raises(RuntimeError, match="accumulation registers"):
        build.check_acc_registers_untouched(_write(tmp_path, GOOD + "\tv_accvgpr_write_b32 a5, v1\n"))
    with pytest.raises(RuntimeError, match="accumulation registers"):
        build.check_acc_registers_untouched(_write(tmp_path, GOOD + "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[0:3], v[4:7], a[0:15]\n"))

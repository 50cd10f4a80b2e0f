"""The build's check of the emitted FFN code: a matrix instruction must not read a register that
one of the two vector instructions in front of it wrote (the matrix instructions of the packed FFN
are asm statements, for which the compiler inserts no such wait)."""
import pytest

from paper_2603_28768_amd import build

MFMA = "\tv_mfma_f32_16x16x32_bf16 a[0:3], v[4:7], v[8:11], a[0:3]\n"


def _check(tmp_path, text):
    p = tmp_path / "k.s"
    p.write_text(text)
    return build.check_matrix_operands(str(p))


def test_operands_from_loads_and_settled_vector_results_pass(tmp_path):
    assert _check(tmp_path, "\tds_read_b128 v[8:11], v20\n\ts_waitcnt lgkmcnt(0)\n" + MFMA) == 1
    assert _check(tmp_path, "\tv_add_u32_e32 v5, v1, v2\n\ts_nop 1\n" + MFMA) == 1
    assert _check(tmp_path, "\tv_add_u32_e32 v5, v1, v2\n\tv_add_u32_e32 v30, v1, v2\n\tv_add_u32_e32 v31, v1, v2\n" + MFMA) == 1
    assert _check(tmp_path, "\tv_add_u32_e32 v12, v1, v2\n" + MFMA + MFMA) == 2


@pytest.mark.parametrize("front", [
    "\tv_add_u32_e32 v5, v1, v2\n",                                  # directly in front
    "\tv_cvt_pk_bf16_f32 v8, v1, v2\n\tds_read_b128 v[20:23], v9\n",  # one instruction between
    "\tv_accvgpr_read_b32 v11, a200\n\ts_nop 0\n",                    # one idle cycle is not enough
    "\tv_accvgpr_write_b32 a2, v9\n",                                 # the addend counts as well
])
def test_fresh_vector_results_are_caught(tmp_path, front):
    with pytest.raises(RuntimeError):
        _check(tmp_path, front + MFMA)


def test_m0_belongs_to_the_row_requests(tmp_path):
    ok = "\ts_mov_b32 m0, s12\n\tglobal_load_lds_dwordx4 v3, s[4:5]\n" + MFMA
    assert _check(tmp_path, ok) == 1
    with pytest.raises(RuntimeError):
        _check(tmp_path, "\ts_mov_b32 m0, s12\n\tv_readlane_b32 s3, v9, m0\n" + MFMA)

"""The build checks the generated assembly of the hand-scheduled attention kernels.  These tests
feed the checker small assembly texts with one planted mistake each (on the CPU), and run it
over the assembly of the library that is actually built."""
import os

import pytest

from paper_2605_20104_amd import build as b

KERNEL = "_ZN5graft21tree_attn_mfma_kernelILi2EEEvNS_10AttnParamsE"


def _asm(body, scratch=0):
    return "\n".join([
        "\t.text",
        KERNEL + ":",
        "\ts_load_dwordx2 s[0:1], s[4:5], 0x0",
        body,
        "\ts_endpgm",
        "\t.amdhsa_kernel " + KERNEL,
        "\t\t.amdhsa_private_segment_fixed_size %d" % scratch,
        "\t.end_amdhsa_kernel",
        ".Lfunc_end0:",
    ])


MFMA = "\t;;#ASMSTART\n\tv_mfma_f32_16x16x32_bf16 a[0:3], v[10:13], v[20:23], a[0:3]\n\t;;#ASMEND"
MFMA_C = "\t;;#ASMSTART\n\tv_mfma_f32_16x16x32_bf16 v[40:43], v[10:13], a[96:99], v[30:33]\n\t;;#ASMEND"
FILL = "\tv_add_u32_e32 v1, v2, v3\n\ts_add_i32 s0, s1, s2"


def test_clean_text_passes():
    assert b.check_attention_asm(_asm(FILL + "\n" + MFMA + "\n" + MFMA_C)) == []


@pytest.mark.parametrize("writer", ["v_mov_b32_e32 v11, v5", "v_cvt_pk_bf16_f32 v23, v1, v2",
                                    "v_mov_b64_e32 v[12:13], s[2:3]", "v_accvgpr_read_b32 v20, a200"])
def test_vector_write_of_a_source_right_before_the_mfma(writer):
    bad = b.check_attention_asm(_asm(FILL + "\n\t" + writer + "\n" + MFMA))
    assert len(bad) == 1 and "MFMA source" in bad[0]
    # one instruction in between is one wait state: still too close
    assert b.check_attention_asm(_asm(FILL + "\n\t" + writer + "\n\ts_add_i32 s0, s1, s2\n" + MFMA))
    # two wait states are enough, as two instructions or as s_nop 1
    assert b.check_attention_asm(_asm("\t" + writer + "\n" + FILL + "\n" + MFMA)) == []
    assert b.check_attention_asm(_asm("\t" + writer + "\n\ts_nop 1\n" + MFMA)) == []
    assert b.check_attention_asm(_asm("\t" + writer + "\n\ts_nop 0\n" + MFMA))


def test_accumulator_input_in_vgprs_is_a_source_too():
    assert b.check_attention_asm(_asm(FILL + "\n\tv_mov_b32_e32 v31, 0\n" + MFMA_C))
    assert b.check_attention_asm(_asm(FILL + "\n\tv_mov_b32_e32 v50, 0\n" + MFMA_C)) == []


def test_writes_that_are_not_vector_registers_do_not_count():
    ok = FILL + "\n\tv_cmp_gt_f32_e32 vcc, v10, v11\n\tv_readfirstlane_b32 s3, v20\n" + MFMA
    assert b.check_attention_asm(_asm(ok)) == []


def test_unknown_predecessor_after_a_label():
    assert b.check_attention_asm(_asm(FILL + "\n.LBB0_3:\n" + MFMA))
    assert b.check_attention_asm(_asm(FILL + "\n.LBB0_3:\n\ts_nop 1\n" + MFMA)) == []


def test_compiler_use_of_a_hand_managed_accvgpr():
    # 48 * MB + 4 * min(MB, 4) = 104 registers are hand-managed in the MB = 2 kernel
    bad = b.check_attention_asm(_asm(FILL + "\n\tv_accvgpr_write_b32 a103, v1\n" + FILL))
    assert len(bad) == 1 and "AccVGPR" in bad[0]
    assert b.check_attention_asm(_asm(FILL + "\n\tds_read_b32 a17, v1\n" + FILL))
    assert b.check_attention_asm(_asm(FILL + "\n\tv_accvgpr_write_b32 a104, v1\n" + FILL)) == []
    inside = "\t;;#ASMSTART\n\tv_accvgpr_write_b32 a[5], v1\n\t;;#ASMEND"
    assert b.check_attention_asm(_asm(FILL + "\n" + inside)) == []


NOPS = "\ts_nop 7\n\ts_nop 3"          # 8 + 4 = 12 wait states


@pytest.mark.parametrize("reader", ["v_exp_f32_e32 v1, v41", "v_max3_f32 v2, v3, v40, v43", "ds_write_b32 v5, v42",
                                    "global_store_dwordx4 v[6:7], v[40:43], off", "v_cmp_gt_f32_e32 vcc, v40, v1",
                                    "v_accvgpr_write_b32 a200, v43"])
def test_read_of_an_mfma_result_in_vgprs_too_early(reader):
    bad = b.check_attention_asm(_asm(FILL + "\n" + MFMA_C + "\n\t" + reader))
    assert len(bad) == 1 and "MFMA result" in bad[0]
    # eleven wait states are not enough, twelve are; a label in between does not reset the count
    assert b.check_attention_asm(_asm(FILL + "\n" + MFMA_C + "\n\ts_nop 7\n\ts_nop 2\n\t" + reader))
    assert b.check_attention_asm(_asm(FILL + "\n" + MFMA_C + "\n" + NOPS + "\n\t" + reader)) == []
    assert b.check_attention_asm(_asm(FILL + "\n" + MFMA_C + "\n\ts_nop 3\n.LBB0_7:\n\t" + reader))
    # registers next to the result are not the result
    other = reader.replace("v40", "v39").replace("v41", "v44").replace("v42", "v44").replace("v43", "v44") \
                  .replace("v[40:43]", "v[44:47]")
    assert b.check_attention_asm(_asm(FILL + "\n" + MFMA_C + "\n\t" + other)) == []


def test_read_of_an_accumulator_too_early():
    rd = "\t;;#ASMSTART\n\tv_accvgpr_read_b32 v1, a[2]\n\t;;#ASMEND"
    bad = b.check_attention_asm(_asm(FILL + "\n" + MFMA + "\n" + rd))
    assert len(bad) == 1 and "MFMA result" in bad[0]
    assert b.check_attention_asm(_asm(FILL + "\n" + MFMA + "\n" + NOPS + "\n" + rd)) == []
    # another MFMA accumulating into the same registers is not such a reader
    assert b.check_attention_asm(_asm(FILL + "\n" + MFMA + "\n" + MFMA)) == []


def test_accvgpr_write_of_a_source_right_before_the_mfma():
    wr = "\t;;#ASMSTART\n\tv_accvgpr_write_b32 a[97], v1\n\t;;#ASMEND"
    bad = b.check_attention_asm(_asm(FILL + "\n" + wr + "\n" + MFMA_C))
    assert len(bad) == 1 and "MFMA source" in bad[0]
    assert b.check_attention_asm(_asm(FILL + "\n" + wr + "\n\ts_nop 1\n" + MFMA_C)) == []


def test_scratch_memory():
    bad = b.check_attention_asm(_asm(FILL, scratch=128))
    assert len(bad) == 1 and "scratch" in bad[0]


def test_the_built_library_passes():
    if not os.path.exists(b.ATTN_ASM):
        pytest.skip("no assembly kept from a build in this tree")
    with open(b.ATTN_ASM) as f:
        text = f.read()
    assert text.count("v_mfma_f32_16x16x32_bf16") > 500          # the check sees the real kernels
    assert b.check_attention_asm(text) == []

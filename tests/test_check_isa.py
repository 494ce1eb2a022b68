"""Host logic of the build's assembly checks (paper_2603_02188_amd/check_isa.py)."""
from paper_2603_02188_amd.check_isa import find_overlaps, find_reserved_acc_uses

ASM = """
_ZN4mlra12_GLOBAL__N_118decode_mfma_kernelILi6ELi0EEEvNS_9mfma_tile10MfmaParamsE:
\tv_mov_b32_e32 v1, v0
\t;;#ASMSTART
\tv_mfma_f32_32x32x16_bf16 a[0:15], v[2:5], v[6:9], a[0:15]
\t;;#ASMEND
.LBB0_1:
\tv_accvgpr_write_b32 a200, v3
\tv_accvgpr_read_b32 v4, a135
\tds_read_b128 a[140:143], v7
\tv_accvgpr_mov_b32 a120, a210
\ts_endpgm
_ZN4mlra5otherEv:
\tv_accvgpr_write_b32 a3, v3
"""


def test_reserved_accumulation_registers_outside_inline_asm_are_reported():
    bad = find_reserved_acc_uses(ASM, r"decode_mfma_kernel", 136)
    assert [text for _, text in bad] == ["v_accvgpr_read_b32 v4, a135", "v_accvgpr_mov_b32 a120, a210"]
    # nothing reserved, nothing reported; another kernel's registers are its own
    assert find_reserved_acc_uses(ASM, r"decode_mfma_kernel", 0) == []
    assert find_reserved_acc_uses(ASM, r"no_such_kernel", 136) == []


def test_mfma_destination_over_a_source_is_reported():
    ok = "\tv_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], a[0:3], v[0:15]\n"
    bad = "\tv_mfma_f32_32x32x16_bf16 v[0:15], v[12:15], a[0:3], 0\n"
    narrow = "\tv_mfma_f32_16x16x32_bf16 v[0:3], v[0:3], v[4:7], 0\n"
    assert find_overlaps(ok) == [] and find_overlaps(narrow) == []
    assert len(find_overlaps(bad)) == 1

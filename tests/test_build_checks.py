"""The build's own check of the prefill kernels' register use (host logic, no GPU)."""
from paper_2410_09615_amd.build import compiler_agpr_uses

ASM = """\t.text
_ZN4slim5cleanE:
\ts_load_dwordx2 s[0:1], s[4:5], 0x0
\t;;#ASMSTART
\tv_accvgpr_write_b32 a[5], v1
\tv_mfma_f32_32x32x16_f16 a[0:15], v[2:5], v[6:9], a[0:15]
\tv_smfmac_f32_32x32x32_f16 a[16:31], v[2:5], v[6:13], v14 abid:1
\tv_accvgpr_read_b32 v3, a[17]
\t;;#ASMEND
\tbuffer_load_dwordx4 v[24:27], v26, s[20:23], 0 offen ; a5 in a comment does not count
\ts_endpgm
.Lfunc_end0:
_ZN4slim6parkedE:
\tv_accvgpr_write_b32 a14, v30
\tbuffer_load_dwordx4 a[24:27], v26, s[20:23], 0 offen
\tv_mfma_f32_32x32x16_f16 a[0:15], v[2:5], v[6:9], a[0:15]
\tv_accvgpr_read_b32 v21, a7
\ts_endpgm
"""


def test_compiler_uses_of_accumulation_registers_are_found():
    """Kernels that address the accumulation registers by number lose whatever the register allocator
    parks there (a store index, once: an out-of-bounds store).  The build reads the device assembly and
    refuses such a library; here the reader itself, on a clean kernel and on one with three parked values."""
    assert compiler_agpr_uses(ASM) == {"_ZN4slim6parkedE": 3}

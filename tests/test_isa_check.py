"""The build's scan of generated code for pinned matrix-core instructions (isa_check).

The 256-row kernel issues matrix-core instructions as inline assembly; the compiler does not add
the wait states the hardware needs between a vector-ALU write and a matrix-core read around those.
The scan must find a planted pair, accept the forms the kernel relies on, and the kernel as built
must be clean.
"""
import os

from paper_2312_05516_amd import build as pv_build
from paper_2312_05516_amd import isa_check

CLEAN = """
	v_exp_f32_e32 v10, v11
	v_cvt_pk_bf16_f32 v12, v10, v13
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[20:35], v[4:7], a[0:3], v[40:55]
	;;#ASMEND
	v_mov_b32_e32 v4, v1
	s_nop 1
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[20:35], v[4:7], a[0:3], v[20:35]
	;;#ASMEND
	v_mov_b32_e32 v5, v1
	ds_read_b128 v[60:63], v9
	v_add_f32_e32 v70, v71, v72
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[20:35], v[4:7], a[0:3], v[20:35]
	;;#ASMEND
	v_mov_b32_e32 v6, v1
	v_mfma_f32_32x32x16_bf16 v[20:35], v[4:7], a[0:3], v[20:35]
"""

PLANTED = [
    # the instruction right before writes an A-operand register
    ("	v_mov_b32_e32 v5, v1\n	;;#ASMSTART\n	v_mfma_f32_32x32x16_f16 v[20:35], v[4:7], a[0:3], 0\n", 1),
    # two before, an accumulation register of the B operand, another vector-ALU instruction between
    ("	v_accvgpr_write_b32 a2, v1\n	v_add_f32_e32 v70, v71, v72\n	;;#ASMSTART\n"
     "	v_mfma_f32_32x32x16_f16 v[20:35], v[4:7], a[0:3], 0\n", 1),
    # the starting value (C operand) written right before
    ("	v_add_f32_e32 v44, v44, v1\n	;;#ASMSTART\n"
     "	v_mfma_f32_32x32x16_bf16 v[20:35], v[4:7], a[0:3], v[40:55]\n", 1),
]


def test_scan_accepts_the_forms_the_kernel_relies_on():
    pinned, hazards = isa_check.pinned_mfma_hazards(CLEAN)
    # the fourth instruction is not inline assembly: the compiler guards those itself
    assert pinned == 3 and hazards == []


def test_scan_finds_planted_pairs():
    for text, want in PLANTED:
        pinned, hazards = isa_check.pinned_mfma_hazards(text)
        assert pinned == 1 and len(hazards) == want, (text, hazards)


def test_the_kernel_as_built_has_pinned_instructions_and_no_hazard():
    for src in pv_build.ISA_CHECKED:
        path = pv_build.isa_path(src)
        if not os.path.exists(path):
            pv_build.build(verbose=False)  # keeps the generated code of these sources
        with open(path) as f:
            text = f.read()
        pinned, hazards = isa_check.pinned_mfma_hazards(text)
        assert pinned >= 64, f"{src}: the pipelined loops alone hold 64 pinned instructions"
        assert hazards == [], hazards[:5]
        # a spill inside these loops is a vector-memory load whose wait also drains the
        # asynchronous copies in flight: correct, but several times slower
        spills = isa_check.spill_counts(text)
        assert len(spills) == 4 and all(n == 0 for n in spills.values()), spills

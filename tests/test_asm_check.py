"""The static check for hand-issued loads (paper_2306_09342_amd/asm_check.py): it must see a planted misuse in
a small assembly text, accept the correct form, and find nothing in the library's own kernels."""
import os
import tempfile

from paper_2306_09342_amd import asm_check

GOOD = """
_Z4kernPf:
\t;;#ASMSTART
\tds_read_b128 v[4:7], v1 offset:0
\t;;#ASMEND
\t;;#ASMSTART
\tds_read_b128 v[8:11], v1 offset:4096
\t;;#ASMEND
\tv_add_u32_e32 v20, 1, v20
\t;;#ASMSTART
\ts_waitcnt lgkmcnt(1)
\t;;#ASMEND
\tv_mfma_f32_32x32x16_bf16 a[0:15], v[4:7], v[12:15], a[0:15]
\t;;#ASMSTART
\ts_waitcnt lgkmcnt(0)
\t;;#ASMEND
\tv_mfma_f32_32x32x16_bf16 a[0:15], v[8:11], v[12:15], a[0:15]
\ts_endpgm
"""
# the second read's registers are copied before the wait that covers them
BAD_LDS = GOOD.replace("\tv_add_u32_e32 v20, 1, v20\n", "\tv_mov_b32_e32 v30, v9\n")
# a global load issued by hand, its destination spilled before the wait
BAD_VM = """
_Z5kern2Pf:
\t;;#ASMSTART
\tglobal_load_dwordx4 v[4:7], v[2:3], off
\t;;#ASMEND
\tscratch_store_dwordx4 off, v[4:7], off offset:16
\ts_waitcnt vmcnt(0)
\ts_endpgm
"""
# the same load issued by the compiler is the compiler's business
COMPILER_VM = BAD_VM.replace("\t;;#ASMSTART\n", "").replace("\t;;#ASMEND\n", "")


def _check(text):
    with tempfile.NamedTemporaryFile("w", suffix=".s", delete=False) as f:
        f.write(text)
        path = f.name
    try:
        return asm_check.check_assembly(path)
    finally:
        os.unlink(path)


def test_correct_wait_order_is_accepted():
    assert _check(GOOD) == []


def test_copy_of_a_register_whose_lds_read_is_in_flight_is_found():
    got = _check(BAD_LDS)
    assert len(got) == 1 and got[0][0] == "_Z4kernPf" and ("v", 9) in got[0][3]


def test_spill_of_a_hand_issued_global_load_is_found_and_compiler_loads_are_left_alone():
    got = _check(BAD_VM)
    assert len(got) == 1 and "scratch_store" in got[0][2]
    assert _check(COMPILER_VM) == []


def test_library_kernels_use_no_hand_issued_load_before_its_wait():
    assert asm_check.check_sources(verbose=False) == []

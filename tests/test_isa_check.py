"""The static check that build() runs on the generated gfx950 code: its logic on small hand-written listings, and
the package's own device sources (compiled to ISA text here: no GPU is needed)."""
import os
from concurrent.futures import ThreadPoolExecutor

from paper_2408_01803_amd import build as stb_build
from paper_2408_01803_amd import isa_check

CLOSE = """
kernel:
\tv_readlane_b32 s5, v203, 3
\tv_add_u32_e32 v1, v2, v3
\tglobal_load_dword v4, v1, s[4:5]
\ts_endpgm
"""

PADDED = """
kernel:
\tv_readlane_b32 s5, v203, 3
\ts_nop 4
\tglobal_load_dword v4, v1, s[4:5]
\ts_endpgm
"""

OTHER_REGISTER = """
kernel:
\tv_readlane_b32 s7, v203, 3
\tglobal_load_dword v4, v1, s[4:5]
\ts_endpgm
"""

ACROSS_A_BRANCH = """
kernel:
\ts_cbranch_scc1 .LBB0_2
\tv_readfirstlane_b32 s4, v9
\ts_branch .LBB0_3
.LBB0_2:
\ts_nop 7
.LBB0_3:
\tglobal_load_dwordx2 v[4:5], v1, s[4:5] offset:512
\ts_endpgm
"""

SCALAR_ALU_WRITE = """
kernel:
\ts_add_u32 s4, s4, s8
\tglobal_load_dword v4, v1, s[4:5]
\ts_endpgm
"""

CARRY_OUT = """
kernel:
\tv_add_co_u32_e64 v1, s[4:5], v2, v3
\tv_mov_b32_e32 v7, 0
\tglobal_load_dword v4, v1, s[4:5]
\ts_endpgm
"""


def test_a_lane_read_right_in_front_of_the_load_is_found():
    found = isa_check.hazards(CLOSE)
    assert len(found) == 1 and found[0][1].startswith("v_readlane_b32 s5") and found[0][4] == 1


def test_five_wait_states_clear_it():
    assert isa_check.hazards(PADDED) == []


def test_a_write_of_another_scalar_is_no_finding():
    assert isa_check.hazards(OTHER_REGISTER) == []


def test_every_path_to_the_load_is_walked():
    found = isa_check.hazards(ACROSS_A_BRANCH)
    assert len(found) == 1 and found[0][1].startswith("v_readfirstlane_b32 s4")


def test_scalar_alu_writes_are_interlocked_and_not_reported():
    assert isa_check.hazards(SCALAR_ALU_WRITE) == []


def test_carry_outputs_count_as_vector_alu_writes():
    assert len(isa_check.hazards(CARRY_OUT)) == 1


SPILL_OF_A_LOAD_IN_FLIGHT = """
kernel:
\t;;#ASMSTART
\tglobal_load_dwordx2 v[10:11], v1, s[4:5]
\t;;#ASMEND
\tv_add_u32_e32 v2, v3, v4
\tscratch_store_dword off, v11, off offset:4 ; 4-byte Folded Spill
\t;;#ASMSTART
\ts_waitcnt vmcnt(0)
\t;;#ASMEND
\ts_endpgm
"""

SPILL_OF_A_COMPUTED_VALUE = """
kernel:
\t;;#ASMSTART
\tglobal_load_dwordx2 v[10:11], v1, s[4:5]
\t;;#ASMEND
\t;;#ASMSTART
\ts_waitcnt vmcnt(0)
\t;;#ASMEND
\tv_add_u32_e32 v11, v10, v11
\tscratch_store_dword off, v11, off offset:4 ; 4-byte Folded Spill
\ts_endpgm
"""


def test_a_spill_of_a_register_that_an_asm_load_has_just_written_is_found():
    assert isa_check.spilled_asm_kernels(SPILL_OF_A_LOAD_IN_FLIGHT) == [("kernel", [11])]


def test_a_spill_of_a_value_computed_after_the_wait_is_no_finding():
    assert isa_check.spilled_asm_kernels(SPILL_OF_A_COMPUTED_VALUE) == []


def test_the_device_sources_of_the_package_are_clean(tmp_path):
    inc = ["-I" + os.path.join(stb_build.ROOT, "include"), "-I" + stb_build.CSRC]
    srcs = [os.path.join(stb_build.CSRC, s) for s in stb_build.DEVICE_SOURCES]
    with ThreadPoolExecutor(max_workers=len(srcs)) as pool:
        found = list(pool.map(lambda s: isa_check.check_source(s, str(tmp_path), stb_build.HIPCC, [*stb_build.DEVICE_FLAGS, *inc]), srcs))
    assert all(f == [] for f in found), [f[:3] for f in found if f]

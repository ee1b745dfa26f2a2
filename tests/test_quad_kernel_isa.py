"""What the four-wave contraction kernel assumes about its own machine code (M0 untouched by the compiler, no spills,
accumulators in place), checked on the code hipcc generates.  The checks live in ``paper_2510_00236_amd/isa_check.py``
and are part of every build; here they run on their own, and on planted mistakes."""
import os

import pytest

from paper_2510_00236_amd import build as pexbuild
from paper_2510_00236_amd import isa_check

SRC = os.path.join(pexbuild.CSRC, "pex_stat_bf16.hip")


@pytest.fixture(scope="module")
def quad_asm():
    return isa_check.quad_kernel_asm(pexbuild.HIPCC, pexbuild.FLAGS, SRC)


def test_only_the_kernel_itself_writes_m0(quad_asm):
    body, _ = quad_asm
    isa_check.check_m0(body)
    with pytest.raises(isa_check.IsaCheckError, match="touch M0"):
        isa_check.check_m0(body + ["\ts_mov_b32 m0, s5"])


def test_no_spills_and_accumulators_stay_put(quad_asm):
    body, meta = quad_asm
    isa_check.check_registers(body, meta)
    with pytest.raises(isa_check.IsaCheckError, match="spills"):
        isa_check.check_registers(body + ["\tscratch_store_dword off, v1, s32"], meta)
    at = [i for i, l in enumerate(body) if "v_mfma_f32_16x16x32_bf16" in l]
    with pytest.raises(isa_check.IsaCheckError, match="accumulator moves"):
        isa_check.check_registers(body[:at[5]] + ["\tv_accvgpr_read_b32 v1, a0"] + body[at[5]:], meta)


def test_no_contraction_kernel_spills():
    text = isa_check.device_asm(pexbuild.HIPCC, pexbuild.FLAGS, SRC)
    isa_check.check_no_scratch(text)
    planted = text.replace(".amdhsa_private_segment_fixed_size 0", ".amdhsa_private_segment_fixed_size 756", 1)
    with pytest.raises(isa_check.IsaCheckError, match="scratch memory"):
        isa_check.check_no_scratch(planted)


@pytest.mark.parametrize("name", ["pex_gram.hip", "pex_gram_wide.hip"])
def test_gram_kernels_keep_their_accumulators_in_place(name):
    text = isa_check.device_asm(pexbuild.HIPCC, pexbuild.FLAGS, os.path.join(pexbuild.CSRC, name))
    isa_check.check_no_scratch(text)
    isa_check.check_accumulators_in_place(text)
    with pytest.raises(isa_check.IsaCheckError, match="accumulator moves"):
        isa_check.check_accumulators_in_place(text + "\n\tv_accvgpr_read_b32 v79, a3\n")

"""What the four-wave contraction kernel assumes about its own machine code, checked on the code hipcc generates
(host only: the kernel is compiled to assembly, nothing runs).

The kernel writes M0 (the LDS base of a group of direct-to-LDS loads) in one inline-assembly statement and issues the
group's loads in later ones, with MFMAs and LDS reads between them; that is only correct while no instruction the
compiler adds writes M0.  It also needs its 256 accumulator registers to stay where they are: a spill or a shuffle of
accumulators inside the loop would cost more than the kernel gains."""
import os
import re
import shutil
import subprocess

import pytest

from paper_2510_00236_amd import build as pexbuild

SRC = os.path.join(pexbuild.CSRC, "pex_stat_bf16.hip")


@pytest.fixture(scope="module")
def quad_asm(tmp_path_factory):
    if not (os.path.exists(pexbuild.HIPCC) or shutil.which(pexbuild.HIPCC)):
        pytest.skip("hipcc not available")
    out = tmp_path_factory.mktemp("isa") / "pex_stat_bf16.s"
    flags = [f for f in pexbuild.FLAGS if f != "-fPIC"]
    subprocess.run([pexbuild.HIPCC, *flags, "--cuda-device-only", "-S", SRC, "-o", str(out)], check=True,
                   stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = out.read_text()
    m = re.search(r"^(_ZN\w*stat_bf16_quad_kernel\w*):[^\n]*\n(.*?)\n\s*s_endpgm", text, re.S | re.M)
    assert m, "four-wave kernel not found in the assembly"
    meta = re.search(r"\.amdhsa_kernel " + re.escape(m.group(1)) + r"\n(.*?)\.end_amdhsa_kernel", text, re.S)
    assert meta, "kernel descriptor not found"
    return m.group(2).splitlines(), meta.group(1)


def test_only_the_kernel_itself_writes_m0(quad_asm):
    body, _ = quad_asm
    touching = [l.strip() for l in body if re.search(r"\bm0\b", l)]
    assert touching, "the kernel sets M0 for its direct-to-LDS loads"
    assert all(l.startswith("s_add_u32 m0,") for l in touching), [l for l in touching if not l.startswith("s_add_u32 m0,")][:5]


def test_no_spills_and_accumulators_stay_put(quad_asm):
    body, meta = quad_asm
    assert not [l for l in body if "scratch_" in l], "register spills in the four-wave kernel"
    assert re.search(r"\.amdhsa_next_free_vgpr 512\b", meta) and re.search(r"\.amdhsa_accum_offset 256\b", meta)
    # everything between the first and the last MFMA is the main loop, unrolled over its period of 10 iterations:
    # no moves into or out of accumulators there
    at = [i for i, l in enumerate(body) if "v_mfma_f32_16x16x32_bf16" in l]
    assert len(at) == 64 * 10, f"{len(at)} MFMAs, expected 64 per iteration x 10 iterations"
    loop = body[at[0]:at[-1] + 1]
    assert not [l for l in loop if "v_accvgpr" in l], "accumulator moves inside the main loop"
    # every MFMA accumulates in place
    for l in loop:
        if "v_mfma_f32_16x16x32_bf16" in l:
            ops = [o.strip() for o in l.split("v_mfma_f32_16x16x32_bf16")[1].split(",")]
            assert ops[0] == ops[3] and ops[0].startswith("a["), l

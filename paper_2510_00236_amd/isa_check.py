"""Checks on the machine code hipcc generates for the four-wave contraction kernel (host only: the kernel is compiled
to assembly, nothing runs).  Part of the build: ``build()`` fails if one of them does not hold.

The kernel writes M0 (the LDS base of a group of direct-to-LDS loads) in one inline-assembly statement and issues the
group's loads in later ones, with MFMAs and LDS reads between them; that is only correct while no instruction the
compiler adds writes M0.  It also needs its 256 accumulator registers to stay where they are: a spill or a shuffle of
accumulators inside the loop would cost more than the kernel gains.

If the compiler ever broke the M0 assumption unnoticed, loads of the four-wave kernel would land in the wrong ring
buffer and ``tests/test_parity_gpu.py::test_four_wave_kernel_shapes`` (element-by-element against the oracle on
seven shapes) would fail."""
from __future__ import annotations

import os
import re
import subprocess
import tempfile


class IsaCheckError(RuntimeError):
    pass


def device_asm(hipcc: str, flags, src: str) -> str:
    """The device assembly hipcc generates for ``src``."""
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "pex_stat_bf16.s")
        flags = [f for f in flags if f != "-fPIC"]
        subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", src, "-o", out], check=True,
                       stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        return open(out).read()


def quad_kernel_asm(hipcc: str, flags, src: str, text: str | None = None):
    """(body lines, kernel descriptor text) of stat_bf16_quad_kernel compiled from ``src``."""
    if text is None:
        text = device_asm(hipcc, flags, src)
    m = re.search(r"^(_ZN\w*stat_bf16_quad_kernel\w*):[^\n]*\n(.*?)\n\s*s_endpgm", text, re.S | re.M)
    if not m:
        raise IsaCheckError("four-wave kernel not found in the assembly")
    meta = re.search(r"\.amdhsa_kernel " + re.escape(m.group(1)) + r"\n(.*?)\.end_amdhsa_kernel", text, re.S)
    if not meta:
        raise IsaCheckError("kernel descriptor of the four-wave kernel not found")
    return m.group(2).splitlines(), meta.group(1)


def check_m0(body) -> None:
    touching = [l.strip() for l in body if re.search(r"\bm0\b", l)]
    if not touching:
        raise IsaCheckError("the four-wave kernel no longer sets M0 for its direct-to-LDS loads")
    foreign = [l for l in touching if not l.startswith("s_add_u32 m0,")]
    if foreign:
        raise IsaCheckError(f"instructions other than the kernel's own s_add_u32 touch M0: {foreign[:5]}")


def check_registers(body, meta) -> None:
    if [l for l in body if "scratch_" in l]:
        raise IsaCheckError("register spills in the four-wave kernel")
    if not (re.search(r"\.amdhsa_next_free_vgpr 512\b", meta) and re.search(r"\.amdhsa_accum_offset 256\b", meta)):
        raise IsaCheckError("the four-wave kernel no longer uses 256 + 256 registers")
    # everything between the first and the last MFMA is the main loop, unrolled over its period of 10 iterations:
    # no moves into or out of accumulators there, and every MFMA accumulates in place
    at = [i for i, l in enumerate(body) if "v_mfma_f32_16x16x32_bf16" in l]
    if len(at) != 64 * 10:
        raise IsaCheckError(f"{len(at)} MFMAs in the four-wave kernel, expected 64 per iteration x 10 iterations")
    loop = body[at[0]:at[-1] + 1]
    if [l for l in loop if "v_accvgpr" in l]:
        raise IsaCheckError("accumulator moves inside the main loop of the four-wave kernel")
    for l in loop:
        if "v_mfma_f32_16x16x32_bf16" in l:
            ops = [o.strip() for o in l.split("v_mfma_f32_16x16x32_bf16")[1].split(",")]
            if not (ops[0] == ops[3] and ops[0].startswith("a[")):
                raise IsaCheckError(f"an MFMA of the four-wave kernel does not accumulate in place: {l.strip()}")


def check_no_scratch(text: str) -> None:
    """No contraction kernel of the file may spill: every flavour is sized to fit the register file, and one that does
    not (a fold that keeps an address per accumulator alive across the main loop did once) still computes the right
    result, only slowly -- no test would notice."""
    kernels = re.findall(r"\.amdhsa_kernel (\S+)\n(.*?)\.end_amdhsa_kernel", text, re.S)
    if not kernels:
        raise IsaCheckError("no kernel descriptors found in the assembly")
    for name, meta in kernels:
        m = re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", meta)
        if not m:
            raise IsaCheckError(f"no scratch size in the descriptor of {name}")
        if int(m.group(1)) != 0:
            raise IsaCheckError(f"{name} uses {m.group(1)} bytes of scratch memory per lane (register spills)")


def check_accumulators_in_place(text: str) -> None:
    """The Gram kernels keep their accumulators where they are across two loops (one per matrix); compiled with the whole
    register file of a lone wave the compiler once split them over both halves of the file and moved them in and out in
    every step."""
    moves = [l.strip() for l in text.splitlines() if "v_accvgpr" in l]
    if moves:
        raise IsaCheckError(f"{len(moves)} accumulator moves in the Gram kernel, e.g. {moves[0]}")


def check_all(hipcc: str, flags, src: str, *gram_srcs: str) -> None:
    text = device_asm(hipcc, flags, src)
    check_no_scratch(text)
    body, meta = quad_kernel_asm(hipcc, flags, src, text)
    check_m0(body)
    check_registers(body, meta)
    for gram_src in gram_srcs:
        gram = device_asm(hipcc, flags, gram_src)
        check_no_scratch(gram)
        check_accumulators_in_place(gram)

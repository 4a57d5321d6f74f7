"""Checks on the compiled device code of the projection kernels (no GPU needed: hipcc cross-compiles).

The direct-to-LDS kernel sets M0 (the LDS base of its load-to-LDS instructions) once per operand
tile and relies on it staying put until the tile's last load; it also sizes its register use to
exactly one wavefront per SIMD with no scratch.  Both are properties of the generated code, not
of the source, so they are checked on the assembly.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2604_06483_amd", "csrc", "ll_project.hip")

pytestmark = pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("isa") / "ll_project.s"
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-S", "--cuda-device-only",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2604_06483_amd", "csrc"),
           SRC, "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    return out.read_text()


def kernel_bodies(asm_text, needle):
    """{symbol: [instruction lines]} for every kernel whose mangled name contains `needle`."""
    bodies = {}
    for m in re.finditer(r"^(_Z\w*" + needle + r"\w*):[^\n]*\n(.*?)\n\s*s_endpgm", asm_text, re.S | re.M):
        lines = [l.strip() for l in m.group(2).splitlines()]
        bodies[m.group(1)] = [l for l in lines if l and not l.startswith((";", ".", "//")) and not l.endswith(":")]
    return bodies


def test_m0_is_only_written_by_the_lds_base_setter(asm):
    bodies = kernel_bodies(asm, "ll_lens_gemm_dma_kernel")
    assert len(bodies) == 10, sorted(bodies)         # four top-k list lengths, each with and without a bias, and the two steering sweeps
    for name, ins in bodies.items():
        loads = [i for i, l in enumerate(ins) if l.startswith("global_load_lds_dwordx4")]
        assert len(loads) >= 16 + 36, (name, len(loads))          # main loop + prologue
        for i, l in enumerate(ins):
            if "m0" not in l.split(";")[0]:
                continue
            # the only mention of M0: "s_mov_b32 m0, sN" and the wait state that follows it
            assert re.fullmatch(r"s_mov_b32 m0, s\d+", l.split(";")[0].strip()), (name, l)
            assert ins[i + 1].startswith("s_nop"), (name, ins[i + 1])
        # nothing that implicitly uses M0 (indexed register moves, messages, GWS)
        for l in ins:
            op = l.split()[0]
            assert not op.startswith(("v_movrel", "s_movrel", "s_sendmsg", "ds_gws", "s_set_gpr_idx")), (name, l)


def test_projection_kernels_fit_one_wave_per_simd_without_scratch(asm):
    meta = {}
    for m in re.finditer(r"\.name:\s+(\S+)\n(.*?)\.wavefront_size", asm, re.S):
        block = m.group(2)
        get = lambda key: int(re.search(r"\." + key + r":\s+(\d+)", block).group(1))
        meta[m.group(1)] = dict(vgpr=get("vgpr_count"), scratch=get("private_segment_fixed_size"),
                                vspill=get("vgpr_spill_count"))
    dma = {k: v for k, v in meta.items() if "ll_lens_gemm_dma_kernel" in k}
    assert len(dma) == 10
    for name, v in dma.items():
        assert v["vgpr"] <= 512 and v["scratch"] == 0 and v["vspill"] == 0, (name, v)


def test_no_valu_reads_an_sgpr_a_valu_wrote_within_two_instructions(asm):
    """gfx950 needs two wait states between a VALU instruction that writes an SGPR (a comparison,
    a carry-out) and a VALU instruction that reads it.  The compiler keeps that distance for its
    own instructions but does not look inside inline asm: check the hand-written selects and
    add-with-carry of the top-k epilogue."""
    bodies = {**kernel_bodies(asm, "ll_lens_gemm_dma_kernel"), **kernel_bodies(asm, "ll_lens_gemm_kernel")}
    assert bodies
    checked = 0
    for name, ins in bodies.items():
        ins = [l.split(";")[0].strip() for l in ins]
        ins = [l for l in ins if l]
        for i, l in enumerate(ins):
            m = re.fullmatch(r"v_cndmask_b32 v\d+, v\d+, v\d+, (s\[\d+:\d+\])", l) or \
                re.fullmatch(r"v_addc_co_u32_e64 v\d+, s\[\d+:\d+\], v\d+, v\d+, (s\[\d+:\d+\])", l)
            if not m:
                continue
            checked += 1
            sreg = m.group(1)
            for prev in ins[max(0, i - 2):i]:
                ops = prev.split(None, 1)
                if len(ops) == 2 and ops[0].startswith("v_"):
                    dests = ops[1].split(",")[:2]            # destination, and carry-out where there is one
                    assert all(sreg != dd.strip() for dd in dests), (name, prev, l)
    assert checked > 1000

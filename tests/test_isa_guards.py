"""Build-time guard for the hand-scheduled part of gemm_kernel (no GPU needed: hipcc cross-compiles).

gemm_kernel issues its LDS fragment reads as inline assembly and waits for them with explicit s_waitcnt instructions
that are tied to the destination registers.  The compiler does not know that those registers are still in flight
after the read, so the generated code is checked here: between a `ds_read_b128` and the next s_waitcnt that covers LDS
(an lgkmcnt field or a literal immediate), no instruction may read or write the registers the read returns into.
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2210_03858_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _regs(token):
    m = re.match(r"v\[(\d+):(\d+)\]", token)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", token)
    return {int(m.group(1))} if m else set()


@pytest.fixture(scope="module")
def mfma_asm():
    src = os.path.join(ROOT, "paper_2210_03858_amd", "csrc", "bcq_mfma.hip")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-fPIC", "-Wall", "-Wno-unused-function")]
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "bcq_mfma.s")
        r = subprocess.run([build._hipcc()] + flags + ["-S", "--cuda-device-only", src, "-o", out],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return open(out).read()


def _check(lines):
    """Returns (number of fragment reads, instructions that touch a register with a read still pending)."""
    pending, reads, violations = set(), 0, []
    for l in lines:
        op = l.split()[0]
        args = [a.strip() for a in l[len(op):].split(",")]
        if op == "ds_read_b128":
            pending |= _regs(args[0])
            reads += 1
            continue
        if op == "s_waitcnt":
            if "lgkmcnt" in l or l.split()[1].startswith("0x"):
                pending = set()
            continue
        if op.startswith("s_"):
            continue
        used = set()
        for a in args:
            if a:
                used |= _regs(a.split()[0])
        if used & pending:
            violations.append(l)
    return reads, violations


def test_the_checker_sees_a_planted_early_use():
    good = ["ds_read_b128 v[10:13], v5 offset:128", "v_add_u32_e32 v20, v21, v22", "s_waitcnt 0xc47f",
            "v_mfma_f32_32x32x16_bf16 a[0:15], v[30:33], v[10:13], a[0:15]"]
    assert _check(good) == (1, [])
    early_copy = ["ds_read_b128 v[10:13], v5 offset:128", "v_mov_b32_e32 v40, v11", "s_waitcnt lgkmcnt(0)"]
    assert _check(early_copy)[1] == ["v_mov_b32_e32 v40, v11"]
    early_use = ["ds_read_b128 v[10:13], v5", "v_mfma_f32_32x32x16_bf16 a[0:15], v[30:33], v[10:13], a[0:15]",
                 "s_waitcnt 0xc47f"]
    assert len(_check(early_use)[1]) == 1
    vmem_wait_only = ["ds_read_b128 v[10:13], v5", "s_waitcnt vmcnt(3)", "v_mov_b32_e32 v1, v13"]
    assert len(_check(vmem_wait_only)[1]) == 1


def _dispatcher_tiles():
    """(TM, TN) of every gemm_kernel instantiation the host dispatcher can launch: read from its source."""
    src = open(os.path.join(ROOT, "paper_2210_03858_amd", "csrc", "bcq_mfma.hip")).read()
    body = src[src.index("static hipError_t launch_gemm("):]
    body = body[:body.index("\n}\n")]
    tiles = sorted(set((int(a), int(b)) for a, b in re.findall(r"launch_gemm_cfg<\s*(\d+)\s*,\s*(\d+)\s*>", body)))
    assert len(tiles) >= 2, "the dispatcher's tile choices were not found"
    return tiles


def _kernel_bodies(asm):
    """{(TM, TN): instruction lines} of every gemm_kernel instantiation in the assembly."""
    out = {}
    for m in re.finditer(r"^_ZN3bcq11gemm_kernelILi(\d+)ELi(\d+)E\w*:[^\n]*\n(.*?)s_endpgm", asm, re.S | re.M):
        lines = [l.strip() for l in m.group(3).split("\n")]
        out[(int(m.group(1)), int(m.group(2)))] = [l for l in lines if l and not l.startswith(";") and not l.startswith(".")]
    return out


def test_every_instantiation_the_dispatcher_can_launch_is_compiled_and_clean(mfma_asm):
    """No hand-typed list: the tile configurations come from launch_gemm's source, and every gemm_kernel found in the
    assembly is checked, so a new instantiation cannot slip past the guard."""
    bodies = _kernel_bodies(mfma_asm)
    for tile in _dispatcher_tiles():
        assert tile in bodies, "gemm_kernel<%d, %d> is launched by the dispatcher but not in the assembly" % tile
    assert set(bodies) == set(_dispatcher_tiles()), "instantiations in the assembly that the dispatcher never launches"
    for tile, lines in bodies.items():
        reads, violations = _check(lines)
        assert reads >= 4, ("the main loop's fragment reads were not found", tile)
        assert not violations, (tile, violations[:5])

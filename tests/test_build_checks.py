"""Checks on the generated gfx950 code that no GPU is needed for."""
import re

from paper_2505_21036_amd.build import device_assembly


import pytest


@pytest.mark.parametrize("source", ["rf_attn.hip", "rf_arm.hip"])
def test_m0_is_used_only_by_the_tile_loads(source):
    """The attention and ARM kernels issue its global->LDS tile loads from inline assembly, which writes
    the LDS address to M0 behind the compiler's back.  That is only sound while the compiler
    itself has no use for M0 in those files: every mention of M0 in the generated code must be
    the assembly's own  s_mov_b32 m0 / s_nop / global_load_lds  triple, and there must be no
    compiler-generated LDS load (which would set M0 itself) left."""
    m0_write = r"s_mov_b32 m0, (s\d+|vcc_lo|vcc_hi)"  # the assembly's own write: any scalar source register
    lines = [l.strip() for l in device_assembly(source).splitlines()]
    code = [l for l in lines if l and not l.startswith((";", ".", "//"))]
    loads = 0
    for i, l in enumerate(code):
        if "global_load_lds" in l:
            assert re.fullmatch(r"global_load_lds_dwordx4 v\[\d+:\d+\], off", l), l
            assert code[i - 1] == "s_nop 0" and re.fullmatch(m0_write, code[i - 2]), code[i - 2:i + 1]
            loads += 1
        elif re.search(r"\bm0\b", l):
            assert re.fullmatch(m0_write, l) and code[i + 1] == "s_nop 0" and "global_load_lds" in code[i + 2], l
    assert loads > 0
    # every explicit wait of the pipeline is still there: one vmcnt wait per tile-loop barrier at least
    assert sum("s_waitcnt vmcnt(0)" in l for l in code) >= (4 if source == "rf_attn.hip" else 2)


def _tile_loops(asm, kernel):
    """Instruction lists of the innermost loops of `kernel` that hold one tile's 32 MFMAs."""
    lines = asm.splitlines()
    start = next(i for i, l in enumerate(lines) if l.startswith(kernel + ":"))
    end = next(i for i in range(start, len(lines)) if "s_endpgm" in lines[i])
    lines = lines[start:end]
    label_at = {m.group(1): i for i, l in enumerate(lines) for m in [re.match(r"^(\.LBB\d+_\d+):", l)] if m}
    loops = []
    for i, l in enumerate(lines):
        m = re.search(r"s_c?branch\w*\s+(\.LBB\d+_\d+)", l)
        if m and label_at.get(m.group(1), len(lines)) < i:
            body = [x.strip() for x in lines[label_at[m.group(1)]:i + 1]]
            body = [x for x in body if x and not x.startswith((";", "."))]
            if sum(x.startswith("v_mfma") for x in body) == 32:
                loops.append(body)
    return loops


def test_tile_loops_keep_operand_reads_ahead_of_the_mfmas():
    """Performance guard on the generated code of the eight-wavefront kernel (head_dim 128, 256-row blocks):
    in every tile loop the LDS operand reads run ahead of the MFMAs that use them, which shows as
    waits for all-but-3 / all-but-4 outstanding LDS operations.  (A schedule that reads, waits for
    everything and then issues one MFMA costs ~9 % and has appeared from unrelated edits.)"""
    asm = device_assembly("rf_attn.hip")
    loops = _tile_loops(asm, "_ZN2rf11attn_kernelILi128ELi8ELi0EEEvNS_8AttnArgsE")
    assert len(loops) >= 3  # every-tile walk (dense / packed), compacted walk, listed walk
    for body in loops:
        waits = [x for x in body if x.startswith("s_waitcnt") and "lgkmcnt" in x]
        ahead = sum("lgkmcnt(3)" in x or "lgkmcnt(4)" in x for x in waits)
        assert ahead >= 24, (ahead, len(waits))
        assert not any(x.startswith("scratch_") for x in body)  # no spills inside a tile loop


def test_twelve_wavefront_kernel_fits_its_registers():
    """The kernel of the headline configuration (head_dim 128, 384-row blocks, twelve wavefronts) is
    held to 168 registers so that three wavefronts share a SIMD.  A reload from scratch waits for every
    vector-memory operation in flight, the tile loads included, so the loops that run on every tile
    must hold none; the listed loop may reload lane offsets on its rare path (tiles that are not 64
    consecutive rows), at most two."""
    asm = device_assembly("rf_attn.hip")
    loops = _tile_loops(asm, "_ZN2rf11attn_kernelILi128ELi12ELi0EEEvNS_8AttnArgsE")
    assert len(loops) >= 4
    spills = sorted(sum(x.startswith("scratch_") for x in body) for body in loops)
    assert spills[:-1] == [0] * (len(loops) - 1) and spills[-1] <= 2, spills
    m = re.search(r"\.amdhsa_kernel _ZN2rf11attn_kernelILi128ELi12ELi0EEEvNS_8AttnArgsE.*?\.amdhsa_next_free_vgpr\s+(\d+)", asm, re.S)
    assert m and int(m.group(1)) <= 168


"""Checks on the generated gfx950 code that no GPU is needed for."""
import re

from paper_2505_21036_amd.build import device_assembly


def test_m0_is_used_only_by_the_tile_loads():
    """The attention kernel issues its global->LDS tile loads from inline assembly, which writes
    the LDS address to M0 behind the compiler's back.  That is only sound while the compiler
    itself has no use for M0 in that file: every mention of M0 in the generated code must be
    the assembly's own  s_mov_b32 m0 / s_nop / global_load_lds  triple, and there must be no
    compiler-generated LDS load (which would set M0 itself) left."""
    m0_write = r"s_mov_b32 m0, (s\d+|vcc_lo|vcc_hi)"  # the assembly's own write: any scalar source register
    lines = [l.strip() for l in device_assembly("rf_attn.hip").splitlines()]
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
    assert sum("s_waitcnt vmcnt(0)" in l for l in code) >= 4

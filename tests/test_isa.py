"""Checks on the generated gfx950 code (no GPU needed: hipcc cross-compiles).

The packed-bf16 FP4 convert of the K staging takes its four source dwords out of one 128-bit load tuple.  One shape of
that code made the compiler name the tuple's first register in all four converts (wrong codes, caught by the parity
tests at the time); this test pins the generated code: every group of four converts into one destination reads four
different source registers.  (The compiler is the image's; the check guards edits of the source.)
The same listing must hold no packed binary32 arithmetic: the library is built with those forms switched off.
"""
import os
import re
import subprocess

import pytest

from paper_2604_03950_amd import build as B


@pytest.mark.parametrize("lo,hi", [(2, 3), (2, 1), (2, 4), (2, 2)])      # every pair whose low format is MXFP4
def test_fp4_convert_groups_read_four_registers(tmp_path, lo, hi):
    out = tmp_path / f"inst_{lo}_{hi}.s"
    flags = [f for f in B.HIPCC_FLAGS if f != "-fPIC"]
    cmd = ["hipcc"] + flags + [f"-DDMA_LO={lo}", f"-DDMA_HI={hi}", "-S", "--cuda-device-only", "-o", str(out),
                              os.path.join(B.CSRC, "dma_attn_inst.hip")]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = open(out).read()
    # the build flags keep the packed binary32 add / multiply / fused multiply-add forms out of the generated code
    assert not re.search(r"\bv_pk_(add|mul|fma)_f32\b", text)
    lines = [ln.strip() for ln in text.splitlines() if "v_cvt_scalef32_pk_fp4_bf16" in ln]
    assert len(lines) >= 16 and len(lines) % 4 == 0
    # The four converts into one destination dword fill its bytes in order (op_sel of the destination byte); the
    # scheduler may interleave the groups of different destinations, so the groups are collected per destination.
    want_sel = ["", "[0,0,1,0]", "[0,0,0,1]", "[0,0,1,1]"]
    open_groups, n_groups = {}, 0
    for ln in lines:
        ops = ln.split()
        dst, src = ops[1].rstrip(","), ops[2].rstrip(",")
        sel = re.search(r"op_sel:(\[[0-9,]+\])", ln).group(1) if "op_sel" in ln else ""
        grp = open_groups.setdefault(dst, [])
        assert sel == want_sel[len(grp)], (dst, grp, ln)     # the next byte of this destination, nothing else
        grp.append(src)
        if len(grp) == 4:
            assert len(set(grp)) == 4, (dst, grp)            # four different source registers
            del open_groups[dst]
            n_groups += 1
    assert not open_groups and n_groups == len(lines) // 4

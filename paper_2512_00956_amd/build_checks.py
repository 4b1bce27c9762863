"""Checks on the generated gfx950 assembly of the tiled MXFP4 GEMM (csrc/mxfp4_gemm_frag.hip).

Its main-loop global loads are issued from inline asm with explicit vmcnt waits, so the compiler
does not know that their destination registers are written asynchronously.  The kernel is only
correct while
  (a) nothing in it spills to scratch,
  (b) every register of the two W sets has ONE physical assignment in the whole kernel (2 sets x
      CB x 4 fragment tuples + 2 x CB scale registers for a tile shape with CB column blocks per
      wave, each loaded at the same number of code sites): a second assignment would mean a
      register copy that may read a tuple whose load is still in flight,
  (c) the compiler adds no full drain (vmcnt(0) / lgkmcnt(0)) inside the pipelined loop, which
      holds exactly two K iterations and two barriers.
None of this can be said in the source, and a different compiler may break it silently, so the
build runs these checks on every compile and fails when one does not hold; the test suite runs
them again.
"""
from __future__ import annotations

import re
from collections import Counter


class InvariantError(RuntimeError):
    pass


def kernels(text: str) -> dict:
    """{kernel symbol: body} of every gemm_frag_kernel instantiation in the assembly."""
    parts = re.split(r"^(_ZN4wush\S*gemm_frag_kernel\S*):.*$", text, flags=re.M)
    return {parts[i]: parts[i + 1].split("s_endpgm")[0] for i in range(1, len(parts) - 1, 2)}


def shape(name: str):
    """(RB, CB) from the mangled template arguments ...ILb<f32>ELi<RB>ELi<CB>E..."""
    m = re.search(r"ILb[01]ELi(\d+)ELi(\d+)E", name)
    return int(m.group(1)), int(m.group(2))


def check_gemm_frag_asm(text: str, expected_kernels: int = 8) -> None:
    ks = kernels(text)
    if len(ks) != expected_kernels:
        raise InvariantError(f"expected {expected_kernels} gemm_frag_kernel instantiations, found {len(ks)}: {list(ks)}")
    for name, body in ks.items():
        RB, CB = shape(name)
        if "scratch_" in body:
            raise InvariantError(f"{name}: spills to scratch")
        frag = Counter(re.findall(r"global_load_dwordx4 (v\[\d+:\d+\])", body))
        scale = Counter(re.findall(r"global_load_dword (v\d+),", body))
        if len(frag) != 2 * CB * 4 or len(scale) != 2 * CB:
            raise InvariantError(f"{name}: {len(frag)} W fragment tuples and {len(scale)} scale registers "
                                 f"(expected {2 * CB * 4} and {2 * CB}): a W register changed its assignment")
        if len(set(frag.values())) != 1 or len(set(scale.values())) != 1:
            raise InvariantError(f"{name}: W registers are loaded at different numbers of code sites: {frag} {scale}")
        regs = [r for t in frag for r in range(*map(int, re.match(r"v\[(\d+):(\d+)\]", t).groups()))]
        if len(regs) != len(set(regs)):
            raise InvariantError(f"{name}: W fragment tuples overlap")
        m = re.search(r"Inner Loop Header.*?s_cbranch_scc1", body, flags=re.S)
        if not m:
            raise InvariantError(f"{name}: pipelined loop not found")
        loop = m.group(0)
        if loop.count("v_mfma_scale_f32_32x32x64_f8f6f4") != 2 * 4 * RB * CB:
            raise InvariantError(f"{name}: the loop does not hold two K iterations")
        if "vmcnt(0)" in loop or "lgkmcnt(0)" in loop:
            raise InvariantError(f"{name}: a full waitcnt drain inside the pipelined loop")
        if loop.count("s_barrier") != 2:
            raise InvariantError(f"{name}: {loop.count('s_barrier')} barriers in the loop (expected 2)")

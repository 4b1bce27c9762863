"""Invariants of the generated code of the MXFP4 GEMM that the source cannot
express: its main-loop global loads are issued from inline asm with explicit
vmcnt waits, so the compiler does not know that their destination registers are
written asynchronously.  That is only safe while (a) nothing in the kernel
spills to scratch and (b) every register of the two W sets has ONE physical
assignment in the whole kernel (2 sets x CB x 4 fragment tuples + 2 x CB scale
registers for the tile shape with CB column blocks per wave, each loaded at the
same number of code sites) -- a second assignment would mean a
register copy that may read a tuple whose load is still in flight.
The test compiles the kernel to gfx950 assembly (no GPU needed) and checks both.
"""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2512_00956_amd", "csrc", "mxfp4_gemm_frag.hip")


@pytest.fixture(scope="module")
def asm_text():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(SRC), "-S",
               "--cuda-device-only", SRC, "-o", out]
        subprocess.run(cmd, check=True, capture_output=True)
        return open(out).read()


def test_gemm_frag_generated_code(asm_text):
    """No scratch, one register assignment per W slot, no compiler-made full drain (vmcnt(0)) inside the
    pipelined loop: the same checks the build runs (paper_2512_00956_amd/build_checks.py)."""
    from paper_2512_00956_amd.build_checks import check_gemm_frag_asm
    check_gemm_frag_asm(asm_text)


def test_the_checks_catch_what_they_are_for(asm_text):
    """Planted faults in the assembly text (not in any kernel): a spill, a second register assignment
    of a W fragment, a full drain in the loop."""
    from paper_2512_00956_amd.build_checks import InvariantError, check_gemm_frag_asm
    import re as _re
    with pytest.raises(InvariantError):
        check_gemm_frag_asm(asm_text.replace("s_barrier", "scratch_store_dword off, v0, s0\n\ts_barrier", 1))
    m = _re.search(r"global_load_dwordx4 v\[(\d+):(\d+)\]", asm_text)
    moved = f"global_load_dwordx4 v[{int(m.group(1)) + 400}:{int(m.group(2)) + 400}]"
    with pytest.raises(InvariantError):
        check_gemm_frag_asm(asm_text[:m.start()] + moved + asm_text[m.end():])
    loop = _re.search(r"Inner Loop Header.*?s_cbranch_scc1", asm_text, flags=_re.S)
    drained = asm_text[:loop.start()] + loop.group(0).replace("s_barrier", "s_waitcnt vmcnt(0)\n\ts_barrier", 1) + asm_text[loop.end():]
    with pytest.raises(InvariantError):
        check_gemm_frag_asm(drained)


# ---------------------------------------------------------------------------
# The FP16-dequantizing GEMM of the NVFP4 / INT4 variants and the three fused quantizers: performance
# invariants of the generated code -- nothing spills to scratch (the GEMM keeps up to 256 accumulator
# registers per lane alive next to its conversion temporaries), and the GEMM's K loop holds exactly the
# MFMAs of one K step and one workgroup barrier.
# ---------------------------------------------------------------------------
def _compile(src_name):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    src = os.path.join(ROOT, "paper_2512_00956_amd", "csrc", src_name)
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(src), "-S",
               "--cuda-device-only", src, "-o", out]
        subprocess.run(cmd, check=True, capture_output=True)
        return open(out).read()


def _bodies(text, pattern):
    parts = re.split(rf"^(_ZN4wush\S*{pattern}\S*):.*$", text, flags=re.M)
    return {parts[i]: parts[i + 1].split("s_endpgm")[0] for i in range(1, len(parts) - 1, 2)}


def test_f16_gemm_has_no_scratch_and_a_tight_loop():
    text = _compile("nvfp4_gemm.hip")
    kernels = _bodies(text, "w4_f16_gemm_kernel")
    assert len(kernels) == 12, list(kernels)          # {bf16, f32 output} x {4, 3, 2 column blocks} x {NVFP4, INT4}
    for name, body in kernels.items():
        cb = int(re.search(r"ILb[01]ELi(\d+)ELi[01]E", name).group(1))
        assert "scratch_" not in body, f"{name}: spills to scratch"
        # the K loop = the basic blocks the compiler annotates as the loop header or "in Loop"
        blocks = re.split(r"^(\.LBB\d+_\d+:.*)$", body, flags=re.M)
        loop = "".join(blocks[i + 1] for i in range(1, len(blocks) - 1, 2)
                       if "Loop Header" in blocks[i] or "in Loop" in blocks[i])
        assert loop, name
        assert len(re.findall(r"v_mfma_f32_32x32x16_f16", loop)) == 16 * cb, name
        assert len(re.findall(r"s_barrier", loop)) == 1, name
        _assert_loads_cost_no_vector_arithmetic(name, loop, 6)


def _loop_of(body):
    blocks = re.split(r"^(\.LBB\d+_\d+:.*)$", body, flags=re.M)
    return "".join(blocks[i + 1] for i in range(1, len(blocks) - 1, 2)
                   if "Loop Header" in blocks[i] or "in Loop" in blocks[i])


def _assert_loads_cost_no_vector_arithmetic(name, loop, n_loads):
    """Every global load of the K loop takes its base from a scalar register pair and a 32-bit lane
    offset (`global_load_* vdst, voffset, s[base:base+1]`), and no 64-bit address arithmetic runs on the
    vector unit: measured, either costs more than the conversion it sits next to."""
    loads = re.findall(r"^\s*global_load_\S+\s+(.*)$", loop, flags=re.M)
    assert len(loads) == n_loads, (name, len(loads))
    for ops in loads:
        assert re.search(r",\s*v\d+,\s*s\[\d+:\d+\]", ops), (name, ops)
    for insn in ("v_mad_i64_i32", "v_mad_u64_u32", "v_lshl_add_u64", "v_add_co_u32", "v_addc_co_u32"):
        assert insn not in loop, (name, insn)


def test_register_w_gemm_loop():
    """The NVFP4 / INT4 kernel that keeps W in registers: no scratch, two K steps per loop trip (2 x 16 CB MFMAs,
    two barriers), 3 + 2 CB loads per step in scalar-base form, and no register move in the loop (the
    prefetched operand sets swap roles between the two steps instead of being copied)."""
    text = _compile("nvfp4_gemm.hip")
    kernels = _bodies(text, "w4_wreg_gemm_kernel")
    assert len(kernels) == 12, list(kernels)          # {bf16, f32 output} x {4, 3, 2 column blocks} x {NVFP4, INT4}
    for name, body in kernels.items():
        cb = int(re.search(r"ILb[01]ELi(\d+)E", name).group(1))
        assert "scratch_" not in body, f"{name}: spills to scratch"
        loop = _loop_of(body)
        assert loop, name
        assert len(re.findall(r"v_mfma_f32_32x32x16_f16", loop)) == 2 * 16 * cb, name
        assert len(re.findall(r"s_barrier", loop)) == 2, name
        _assert_loads_cost_no_vector_arithmetic(name, loop, 2 * (3 + 2 * cb))
        assert "v_mov_b32" not in loop and "v_accvgpr" not in loop, name


@pytest.mark.parametrize("src,pattern,count", [("nvfp4_quant.hip", "nvfp4_transform_quant_kernel", 8),
                                                ("int4_quant.hip", "int4_transform_quant_kernel", 8),
                                                ("transform_quant.hip", "22transform_quant_kernel", 8)])
def test_quantizers_do_not_spill_and_keep_three_waves_per_simd(src, pattern, count):
    text = _compile(src)
    kernels = _bodies(text, pattern)
    assert len(kernels) == count, list(kernels)
    for name, body in kernels.items():
        assert "scratch_" not in body, f"{name}: spills to scratch"
    # register budget from the kernel descriptors: at most 168 VGPRs = three waves per SIMD of 512 (the
    # instantiations that also write the FP32 transformed values, a test tap, are exempt).  The kernels
    # with two wave groups and two tiles of lookahead run as the only workgroup of their CU, two waves per
    # SIMD: 256.
    for m in re.finditer(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.vgpr_count:\s+(\d+)", text):
        if pattern in m.group(1) and "kernelILb1E" not in m.group(1):
            budget = 256 if "ELi2ELi2EE" in m.group(1) else 176
            assert int(m.group(2)) <= budget, (m.group(1), m.group(2))

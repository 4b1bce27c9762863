"""ctypes loader of libwush_probes.so, the benchmark's measurement aids.

Not part of the layer path: the MFMA instructions of the GEMMs in register-only
loops and plain streaming kernels with the byte mix of the fused transform +
quantize kernel.  bench.py and the probes' own tests are the only users.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_int32, c_int64, c_void_p

_PATH = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "libwush_probes.so")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_PATH):
            raise RuntimeError(f"{_PATH} not found: build it first (python -m paper_2512_00956_amd.build)")
        L = ctypes.CDLL(_PATH)
        for name in ("wushp_mfma_fp4", "wushp_mfma_fp4_colmajor", "wushp_mfma_f16"):
            fn = getattr(L, name)
            fn.restype = c_int32
            fn.argtypes = [c_void_p, c_int32, c_int32, c_void_p, c_void_p]
        L.wushp_stream.restype = c_int32
        L.wushp_stream.argtypes = [c_void_p, c_int64, c_int64, c_void_p, c_int32, c_int32, c_void_p]
        _lib = L
    return _lib


def _stream():
    import torch
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(code: int, where: str):
    if code != 0:
        raise RuntimeError(f"{where}: {'bad argument' if code == 1 else 'HIP launch error'}")


def mfma_fp4(operand_bits, iters: int, blocks: int, cycles_ticks):
    """Block-scaled FP4 MFMA (32x32x64) in a register-only loop: operand_bits u8 [16384],
    cycles_ticks int64 [blocks][2] = shader cycles and 100 MHz ticks per workgroup (GPU tensors).
    FLOP per workgroup = 4 waves * iters * 64 * 2*32*32*64."""
    _check(lib().wushp_mfma_fp4(c_void_p(operand_bits.data_ptr()), iters, blocks, c_void_p(cycles_ticks.data_ptr()),
                                _stream()), "wushp_mfma_fp4")


def mfma_fp4_colmajor(operand_bits, iters: int, blocks: int, cycles_ticks):
    """mfma_fp4 with the 16 MFMAs of an issue ordered column block by column block (eight consecutive
    MFMAs share the W-side operand) instead of row block by row block."""
    _check(lib().wushp_mfma_fp4_colmajor(c_void_p(operand_bits.data_ptr()), iters, blocks,
                                         c_void_p(cycles_ticks.data_ptr()), _stream()), "wushp_mfma_fp4_colmajor")


def mfma_f16(operand_f16, iters: int, blocks: int, cycles_ticks):
    """The same for the FP16 MFMA (32x32x16): operand_f16 = 8192 FP16 values.
    FLOP per workgroup = 4 waves * iters * 64 * 2*32*32*16."""
    _check(lib().wushp_mfma_f16(c_void_p(operand_f16.data_ptr()), iters, blocks, c_void_p(cycles_ticks.data_ptr()),
                                _stream()), "wushp_mfma_f16")


def stream(src, rows: int, row_bytes: int, dst, mode: int, blocks: int):
    """Streaming kernel with the quantizer's byte mix (reads rows*row_bytes, writes 17/64 of that with
    non-temporal stores).  mode 0: linear; mode 1: the quantizer's tile pattern (32 rows x 256 B per
    wave, tiles dealt round-robin over the workgroups); mode 2: that pattern with 512 B per row and wave;
    mode 3: mode 1 with a contiguous run of tiles per workgroup; modes 4, 5, 6: mode 1 with
    linear / no scale / cached stores; modes 10, 11, 13: read-pattern probes with
    linear stores of a quarter of the bytes (32 rows x 256 B per wave tile, 8 rows x 1 KiB, and the first
    with whole 128-byte lines per load instruction), contiguous runs; 20, 21, 23: the same dealt round-robin; 30, 40: modes 0 and 20 with non-temporal loads;
    50: linear and read only (dst then holds blocks * 8 KiB: the xor of what each wave read).  dst: at least rows*row_bytes*17/64 bytes."""
    _check(lib().wushp_stream(c_void_p(src.data_ptr()), rows, row_bytes, c_void_p(dst.data_ptr()), mode, blocks,
                              _stream()), "wushp_stream")

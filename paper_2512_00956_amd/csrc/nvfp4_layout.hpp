// Tiled layout of packed NVFP4 operands (codes + E4M3 scale bytes) between the
// quantizers and the GEMM.  Needs K % 64 == 0; buffers hold a multiple of 32 rows.
// With rb = row / 32, r = row % 32, KT = K / 64, and the 64 channels of K step kt
// split into halves hh = 0, 1 of 32 channels (16 bytes of codes each):
//   codes : the 16-byte chunk (row, kt, hh) sits at (((rb*KT + kt)*2 + hh)*32 + r) * 16,
//           so the 32 rows of a row block are contiguous (512 B) per half step;
//   scales: the 4 scale bytes of (row, kt) sit at ((rb*KT + kt)*32 + r) * 4, byte g = group g.
// A GEMM tile reads whole 512-byte / 128-byte runs instead of 16 bytes from each of
// 256 rows; the canonical row-major layout stays the one tests and callers inspect.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wush {

__host__ __device__ __forceinline__ int64_t nv_tiled_chunk_offset(int64_t row, int kt, int hh, int KT) {
  return ((((row >> 5) * KT + kt) * 2 + hh) * 32 + (row & 31)) * 16;
}

__host__ __device__ __forceinline__ int64_t nv_tiled_scale_offset(int64_t row, int kt, int KT) {
  return (((row >> 5) * KT + kt) * 32 + (row & 31)) * 4;
}

}  // namespace wush

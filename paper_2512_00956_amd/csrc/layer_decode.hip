// Decode-sized layer forward (at most 64 tokens) for gfx950:
//   Y = sum_i Wq(i)^T q(T(i) X(i))      (layer forward-pass equation)
// with the weights already transformed and quantized, in two forms:
//   * gemm_skinny_kernel: the MXFP4 GEMM alone for M <= 128 (wush_linear);
//   * layer_decode_kernel: activation transform + quantization + GEMM in ONE
//     launch (wush_layer_decode).
// At these sizes the layer is bound by streaming the weights once (K/2 + K/32
// bytes per output channel); the activations are a few hundred KiB.
//
// GEMM part.  A workgroup owns one block of 32 output channels at a time; its four
// waves split K into four contiguous ranges (a wave's W fragments are then one
// contiguous run of the fragment-order layout), accumulate 32 x 32 (x 2 for
// 33..64 tokens) partial tiles on the scaled 32x32x64 MFMA, and reduce the four
// partials through LDS in a fixed order.  The W fragment is the first MFMA
// operand, so a lane's accumulator quad is four consecutive output channels of one
// token.  A wave issues the loads of 4 K tiles (2 for 33..64 tokens) of W and X
// together and then consumes them; beyond that, latency is hidden by occupancy
// (several workgroups per CU), not by a software pipeline.
//
// Fused form.  Phase 1: the (token tile, 4 blocks) units of the activation
// quantizer are dealt out one per wave over the grid and write Xq/Xs (fragment
// order) to the workspace.  A grid-wide barrier separates it from phase 2, the
// GEMM above.  Each workgroup issues the loads of its first W tile before phase 1,
// so the weight stream is already in flight while the activations are quantized.
//
// The barrier uses no read-modify-write atomics: device-scope atomics on one
// address complete at roughly one per 100 ns on this part (measured: a counter
// barrier cost 0.1-0.17 us per workgroup), far more than the rest of the kernel.
// Instead every workgroup publishes "arrived" with one store of this launch's
// generation number to its own slot; one wave of workgroup 0 polls the slot array
// with coalesced device-scope loads until all slots carry that number and then
// stores it into the generation word, which is what the other workgroups poll (and
// what the next launch reads to form its own number).  Variants measured and
// dropped: one release slot per workgroup, and every workgroup polling the slot
// array itself -- both slower.  Device-scope release/acquire fences bracket the
// stores and loads.  From the last arrival to the last workgroup leaving the
// barrier takes 3-5 us: each hop is a trip to the memory side of the fabric.
// The barrier needs all workgroups resident: the grid is capped at one workgroup
// per CU, and every wait is bounded -- on expiry the workgroup records an error
// and exits without touching Y.
#include "skinny_reduce.hpp"
#include "transform_quant_core.hpp"
#include "wush_kernels.hpp"

namespace wush {

namespace {

using skinny::kWaves;
using skinny::reduce_store_block;
using skinny::wave_k_range;
using skinny::decode_vec_store;
constexpr uint32_t kSpinLimit = 1u << 21;   // polls of about 0.5 us each
constexpr int kMaxGrid = 1024;              // barrier slots in the workspace

// Barrier words in the workspace (uint32 index): generation of the last completed
// launch, error flag (each on its own 128-byte line), arrival slots (dense).
constexpr int kGenWord = 0, kErrWord = 32, kArriveWord = 64;
constexpr int kStateWords = kArriveWord + kMaxGrid;

struct FragTile {   // one (row block, K tile) of a fragment-order operand
  v4i f[4];
  int s;
};

__device__ __forceinline__ void load_frag_tile(FragTile& t, const uint8_t* __restrict__ q,
                                               const uint8_t* __restrict__ s, int64_t rb_kt, int lane) {
  const v4i* p = reinterpret_cast<const v4i*>(q + rb_kt * 4096) + lane;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) t.f[kk] = p[kk * 64];
  t.s = reinterpret_cast<const int*>(s + rb_kt * 256)[lane];
}

// K tiles a wave keeps in flight at once (its loads are issued together, then
// consumed): 4 for up to 32 tokens, 2 beyond (the X registers grow with the token blocks).
template <int RB>
struct Depth { static constexpr int U = RB == 1 ? 4 : 2; };

template <int U>
__device__ __forceinline__ void load_w_chunk(FragTile (&w)[U], const uint8_t* __restrict__ Wq,
                                             const uint8_t* __restrict__ Ws, int64_t j_kt, int n, int lane) {
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (u < n) load_frag_tile(w[u], Wq, Ws, j_kt + u, lane);
}

// Partial tile of column block j over K tiles [kt0, kt1), U tiles at a time.  `w`
// already holds the W tiles of the first chunk (loaded by the caller, possibly
// long ago).
template <int RB>
__device__ __forceinline__ void accumulate_block(v16f (&acc)[RB], FragTile (&w)[Depth<RB>::U],
                                                 const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs,
                                                 const uint8_t* __restrict__ Wq, const uint8_t* __restrict__ Ws,
                                                 int KT, int j, int kt0, int kt1, int lane) {
  constexpr int U = Depth<RB>::U;
  for (int kt = kt0; kt < kt1; kt += U) {
    const int n = min(U, kt1 - kt);
    if (kt != kt0) load_w_chunk<U>(w, Wq, Ws, (int64_t)j * KT + kt, n, lane);
    FragTile x[RB][U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (u < n) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) load_frag_tile(x[rb][u], Xq, Xs, (int64_t)rb * KT + kt + u, lane);
      }
#define WUSH_SKINNY_ISSUE(KK)                                                                                        \
  {                                                                                                                  \
    const v8i A_ = {w[u].f[KK][0], w[u].f[KK][1], w[u].f[KK][2], w[u].f[KK][3], 0, 0, 0, 0};                         \
    _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) {                                                              \
      const v8i B_ = {x[rb][u].f[KK][0], x[rb][u].f[KK][1], x[rb][u].f[KK][2], x[rb][u].f[KK][3], 0, 0, 0, 0};       \
      acc[rb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A_, B_, acc[rb], 4, 4, KK, w[u].s, KK, x[rb][u].s);  \
    }                                                                                                                \
  }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (u < n) {
        WUSH_SKINNY_ISSUE(0)
        WUSH_SKINNY_ISSUE(1)
        WUSH_SKINNY_ISSUE(2)
        WUSH_SKINNY_ISSUE(3)
      }
#undef WUSH_SKINNY_ISSUE
  }
}

template <int RB, bool OUT_F32>
__global__ __launch_bounds__(kWaves * 64) void gemm_skinny_kernel(
    const uint8_t* __restrict__ Xq, const uint8_t* __restrict__ Xs, const uint8_t* __restrict__ Wq,
    const uint8_t* __restrict__ Ws, int M, int N, int K, void* __restrict__ Y, int64_t ldy, int vec_store) {
  __shared__ float red[kWaves][RB][16][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int KT = K >> 8, NB = (N + 31) >> 5;
  int kt0, kt1;
  wave_k_range(KT, wave, kt0, kt1);
  for (int j = blockIdx.x; j < NB; j += gridDim.x) {
    v16f acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = (v16f){0};
    if (kt0 < kt1) {
      FragTile w[Depth<RB>::U];
      load_w_chunk<Depth<RB>::U>(w, Wq, Ws, (int64_t)j * KT + kt0, min(Depth<RB>::U, kt1 - kt0), lane);
      accumulate_block<RB>(acc, w, Xq, Xs, Wq, Ws, KT, j, kt0, kt1, lane);
    }
    reduce_store_block<RB, OUT_F32>(acc, red, j, M, N, Y, ldy, vec_store, lane, wave);
  }
}

template <int RB, bool OUT_F32>
__global__ __launch_bounds__(kWaves * 64) void layer_decode_kernel(
    const uint16_t* __restrict__ X, int64_t ldx, const uint16_t* __restrict__ T, const uint8_t* __restrict__ Wq,
    const uint8_t* __restrict__ Ws, uint8_t* __restrict__ Xq, uint8_t* __restrict__ Xs, uint32_t* __restrict__ state,
    int M, int N, int K, void* __restrict__ Y, int64_t ldy, int vec_store, int rule, uint32_t expected_blocks,
    uint32_t spin_limit) {
  __shared__ float red[kWaves][RB][16][64];
  __shared__ int barrier_ok;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int KT = K >> 8, C = K >> 5, NB = (N + 31) >> 5;
  int kt0, kt1;
  wave_k_range(KT, wave, kt0, kt1);

  // This launch's generation: one more than the last completed launch's, which
  // workgroup 0 only advances after every workgroup has arrived (and so has read it).
  const uint32_t target = state[kGenWord] + 1;

  // Start the weight stream: first W chunk of this workgroup's first column block.
  // Waves with a phase-1 unit issue it after that unit's loads, which the barrier waits for.
  constexpr int U = Depth<RB>::U;
  int j = blockIdx.x;
  FragTile w_first[U];
  const int n_first = min(U, kt1 - kt0);
  const bool has_unit = (int)(blockIdx.x + wave * gridDim.x) < RB * (C >> 2);
  if (!has_unit && j < NB && kt0 < kt1) load_w_chunk<U>(w_first, Wq, Ws, (int64_t)j * KT + kt0, n_first, lane);

  // ---- phase 1: quantize the activations, one (token tile, 4 blocks) unit per wave
  {
    const int tok = lane & 31, h = lane >> 5;
    const int units = RB * (C >> 2);
    for (int u = blockIdx.x + wave * gridDim.x; u < units; u += kWaves * gridDim.x) {
      const int t = u % RB, bfirst = 4 * (u / RB);
      v8bf ta[tq::kNB][2];
      tq::XFrag cur[tq::kNB];
      tq::load_transforms(ta, T, bfirst, C, tok, h);
      tq::load_tile(cur, X, ldx, min(32 * t + tok, M - 1), bfirst, C, h);
      if (u == (int)(blockIdx.x + wave * gridDim.x) && j < NB && kt0 < kt1)
        load_w_chunk<U>(w_first, Wq, Ws, (int64_t)j * KT + kt0, n_first, lane);
      v4u out[2];
      uint32_t sbytes;
      tq::transform_quantize<false>(ta, cur, rule, out, sbytes, nullptr, tq::kNB);
      if (32 * t + tok < M) tq::store_tile_tiled<false>(out, sbytes, Xq, Xs, t, KT, bfirst, tok, h);
    }
  }

  // ---- grid-wide barrier.  Device-scope fences cost about 0.1 us each and
  // serialize within an XCD (they walk its L2), so there is one release per
  // workgroup that wrote activations and one acquire per workgroup, both issued by
  // wave 0 with the workgroup barrier extending them to the other waves.
  __syncthreads();
  if (wave == 0) {
    bool ok = true;
    if ((int)blockIdx.x < RB * (C >> 2)) __threadfence();   // release this workgroup's Xq/Xs stores
    if (lane == 0)
      __hip_atomic_store(&state[kArriveWord + blockIdx.x], target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (blockIdx.x == 0) {
      // collector: poll all arrival slots, 64 per load instruction
      uint32_t spins = 0;
      for (;;) {
        bool all = true;
        for (uint32_t i = lane; i < expected_blocks; i += 64)
          all &= __hip_atomic_load(&state[kArriveWord + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == target;
        if (__builtin_amdgcn_ballot_w64(all) == ~0ull) break;
        if (++spins >= spin_limit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(4);
      }
      // every workgroup has arrived, hence has read the old generation: publish the new one
      if (ok) {
        __threadfence();
        if (lane == 0) __hip_atomic_store(&state[kGenWord], target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    } else {
      uint32_t spins = 0;
      while (__hip_atomic_load(&state[kGenWord], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != target) {
        if (++spins >= spin_limit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(8);
      }
    }
    if (ok) __threadfence();   // acquire: see every workgroup's Xq/Xs
    if (lane == 0) {
      if (!ok) __hip_atomic_store(&state[kErrWord], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      barrier_ok = ok;
    }
  }
  __syncthreads();
  if (!barrier_ok) return;   // workgroup-uniform

  // ---- phase 2: GEMM over this workgroup's column blocks
  for (; j < NB; j += gridDim.x) {
    v16f acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) acc[rb] = (v16f){0};
    if (kt0 < kt1) {
      if (j != (int)blockIdx.x) load_w_chunk<U>(w_first, Wq, Ws, (int64_t)j * KT + kt0, n_first, lane);
      accumulate_block<RB>(acc, w_first, Xq, Xs, Wq, Ws, KT, j, kt0, kt1, lane);
    }
    reduce_store_block<RB, OUT_F32>(acc, red, j, M, N, Y, ldy, vec_store, lane, wave);
  }
}

__global__ void decode_state_reset_kernel(uint32_t* state) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kStateWords; i += gridDim.x * blockDim.x) state[i] = 0;
}

// Workgroups that are certainly resident together: one per CU, given that the
// occupancy the runtime reports for the kernel is at least that.
template <typename Kern>
hipError_t resident_limit(Kern kern, int* limit) {
  int dev = 0, cus = 0, per_cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kWaves * 64, 0);
  if (e != hipSuccess) return e;
  if (per_cu < 1 || cus < 1) return hipErrorInvalidValue;
  // One workgroup per CU: measured faster than two for every shape (half the
  // arrivals and fences at the barrier; the GEMM phase keeps 4 x U tiles in flight per CU).
  *limit = cus;
  if (*limit > kMaxGrid - 1) *limit = kMaxGrid - 1;   // one slot is left for the timeout test hook
  return hipSuccess;
}

}  // namespace

hipError_t launch_mxfp4_gemm_skinny(const void* Xq, const void* Xs, const void* Wq, const void* Ws, int64_t M,
                                    int64_t N, int64_t K, int out_f32, void* Y, int64_t ldy, hipStream_t stream) {
  const int NB = (int)((N + 31) / 32);
  dim3 grid((unsigned)(NB < 4096 ? NB : 4096)), block(kWaves * 64);
  const int vec = decode_vec_store(Y, N, ldy, out_f32);
#define WUSH_SKINNY_LAUNCH(RB, F32)                                                                         \
  gemm_skinny_kernel<RB, F32><<<grid, block, 0, stream>>>((const uint8_t*)Xq, (const uint8_t*)Xs,           \
                                                          (const uint8_t*)Wq, (const uint8_t*)Ws, (int)M,   \
                                                          (int)N, (int)K, Y, ldy, vec)
  if (M <= 32) {
    if (out_f32) WUSH_SKINNY_LAUNCH(1, true); else WUSH_SKINNY_LAUNCH(1, false);
  } else if (M <= 64) {
    if (out_f32) WUSH_SKINNY_LAUNCH(2, true); else WUSH_SKINNY_LAUNCH(2, false);
  } else {
    if (out_f32) WUSH_SKINNY_LAUNCH(4, true); else WUSH_SKINNY_LAUNCH(4, false);
  }
#undef WUSH_SKINNY_LAUNCH
  return hipGetLastError();
}

// workspace: Xq for 64 tokens (2 row blocks) | Xs | barrier words
size_t layer_decode_codes_bytes(int64_t K) { return (size_t)(K >> 8) * 2 * 4096; }
size_t layer_decode_scales_bytes(int64_t K) { return (size_t)(K >> 8) * 2 * 256; }
size_t layer_decode_scales_offset(int64_t K) { return layer_decode_codes_bytes(K); }
size_t layer_decode_state_offset(int64_t K) { return layer_decode_codes_bytes(K) + layer_decode_scales_bytes(K); }
size_t layer_decode_workspace_bytes(int64_t K) { return layer_decode_state_offset(K) + (size_t)kStateWords * 4; }
size_t layer_decode_error_offset(int64_t K) { return layer_decode_state_offset(K) + (size_t)kErrWord * 4; }

hipError_t launch_layer_decode_init(void* workspace, int64_t K, hipStream_t stream) {
  uint32_t* state = reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(workspace) + layer_decode_state_offset(K));
  decode_state_reset_kernel<<<32, 256, 0, stream>>>(state);
  return hipGetLastError();
}

hipError_t launch_layer_decode(const void* X, int64_t M, int64_t K, int64_t ldx, const void* T, const void* Wq,
                               const void* Ws, int64_t N, int rule, int out_f32, void* Y, int64_t ldy,
                               void* workspace, int test_timeout, hipStream_t stream) {
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  uint8_t* Xq = ws;
  uint8_t* Xs = ws + layer_decode_codes_bytes(K);
  uint32_t* state = reinterpret_cast<uint32_t*>(ws + layer_decode_state_offset(K));
  const int NB = (int)((N + 31) / 32);
  const int vec = decode_vec_store(Y, N, ldy, out_f32);
  dim3 block(kWaves * 64);
#define WUSH_DECODE_LAUNCH(RB, F32)                                                                          \
  {                                                                                                          \
    static int limit = 0; /* queried once per instantiation */                                               \
    if (limit == 0) {                                                                                        \
      int l = 0;                                                                                             \
      hipError_t e = resident_limit(layer_decode_kernel<RB, F32>, &l);                                       \
      if (e != hipSuccess) return e;                                                                         \
      limit = l;                                                                                             \
    }                                                                                                        \
    const unsigned g = (unsigned)(NB < limit ? NB : limit);                                                  \
    /* test hook: expect one workgroup more than launched and give up after a few polls */                   \
    const uint32_t expected = test_timeout ? g + 1 : g;                                                      \
    const uint32_t spin = test_timeout ? 16u : kSpinLimit;                                                   \
    layer_decode_kernel<RB, F32><<<dim3(g), block, 0, stream>>>(                                             \
        (const uint16_t*)X, ldx, (const uint16_t*)T, (const uint8_t*)Wq, (const uint8_t*)Ws, Xq, Xs, state,  \
        (int)M, (int)N, (int)K, Y, ldy, vec, rule, expected, spin);                                          \
  }
  if (M <= 32) {
    if (out_f32) WUSH_DECODE_LAUNCH(1, true) else WUSH_DECODE_LAUNCH(1, false)
  } else {
    if (out_f32) WUSH_DECODE_LAUNCH(2, true) else WUSH_DECODE_LAUNCH(2, false)
  }
#undef WUSH_DECODE_LAUNCH
  return hipGetLastError();
}

}  // namespace wush

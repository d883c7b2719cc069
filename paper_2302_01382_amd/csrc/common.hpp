// common.hpp -- shared device/host helpers of libmpq (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mpq.h"

namespace mpq {

constexpr int kWave = 64;           // CDNA wavefront
constexpr int kBlock = 256;         // 4 waves per workgroup for the streaming kernels
constexpr int kNumCU = 256;         // MI355X
constexpr float kMagic = 12582912.0f;  // 1.5 * 2^23: fma(x, inv, kMagic) - kMagic == RNE(x * inv)

// ---- host side ---------------------------------------------------------------------------
void set_last_hip_error(int e);

inline int launch_status() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_last_hip_error((int)e);
    return MPQ_ERR_HIP;
  }
  return MPQ_OK;
}

// defined in fake_quant.hip: mpq_fake_quant plus the step size as an output of the same kernel
int fake_quant_launch(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax, int bits,
                      float* y_out, int8_t* codes_out, uint8_t* packed4_out, float* step_out, void* stream);

// defined in qgemm.hip: the host-side argument checks of mpq_qgemm_act / mpq_qgemm_score, for callers
// that must validate several layers before their first launch
int check_qgemm_act_args(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N, int64_t K,
                         const float* a_scale, const float* w_scale, int w_gran, int act, const float* y_out,
                         const float* absmax_out);
int check_qgemm_score_args(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N, int64_t K,
                           const float* a_scale, const float* w_scale, int w_gran, const float* y_ref,
                           const double* sse_out, const float* y_out, const void* ws, size_t ws_bytes);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool mul_overflows(int64_t a, int64_t b) {
  int64_t r;
  return __builtin_mul_overflow(a, b, &r) || r > (int64_t)1 << 46;  // 2^46 elements: 256 TiB fp32
}

inline int64_t channels(int gran, int64_t rows, int64_t cols) {
  return gran == MPQ_PER_ROW ? rows : gran == MPQ_PER_COL ? cols : 1;
}

// Flat streaming kernels walk the tensor in tiles of kTileVec float4 per lane x kBlock lanes
// (16 KiB contiguous), all kTileVec loads issued before the first use; tiles are dealt round-robin
// to a persistent grid whose size divides the tile count evenly (every block gets the same number
// of tiles, so the grid finishes together).  Measured on MI355X, contiguous tiles read ~6.1 TB/s
// from HBM against ~5.3 TB/s for a plain grid-stride loop; for kernels that also write, round-robin
// tiles beat one contiguous span per block by ~10 %.
constexpr int kTileVec = 4;

// grid for a flat streaming kernel over `units` work items (float4 vectors or scalars) of which a
// block takes `units_per_trip` per trip: about blocks_per_cu blocks per CU, every block the same
// number of trips r (the last block may fall short), r capped at 256 so that a lane never
// accumulates more than 256 trips in fp32.
inline unsigned flat_grid(int64_t units, int64_t units_per_trip, int blocks_per_cu = 8) {
  const int64_t trips = (units + units_per_trip - 1) / units_per_trip;
  if (trips <= 1) return 1;
  const int64_t cap = (int64_t)kNumCU * blocks_per_cu;
  int64_t r = (trips + cap - 1) / cap;  // trips per block
  if (r > 256) r = 256;
  return (unsigned)((trips + r - 1) / r);
}

// ---- device side ---------------------------------------------------------------------------
#if defined(__HIPCC__)

__device__ __forceinline__ float f_from_bits(int v) { return __builtin_bit_cast(float, v); }
__device__ __forceinline__ int bits_from_f(float v) { return __builtin_bit_cast(int, v); }

// data-parallel-primitive move: lane reads another lane's register without touching LDS
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return f_from_bits(__builtin_amdgcn_update_dpp(0, bits_from_f(v), CTRL, 0xF, 0xF, true));
}

constexpr int kQuadSwap1 = 0xB1;   // quad_perm [1,0,3,2]
constexpr int kQuadSwap2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141;
constexpr int kRowMirror = 0x140;

// Sum over the 64 lanes of a wave (all lanes must be active); every lane gets the result.
// Fixed combination order -> reproducible.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp<kQuadSwap1>(v);
  v += dpp<kQuadSwap2>(v);
  v += dpp<kRowHalfMirror>(v);
  v += dpp<kRowMirror>(v);  // each 16-lane row now holds its row sum in every lane
  const float r0 = f_from_bits(__builtin_amdgcn_readlane(bits_from_f(v), 0));
  const float r1 = f_from_bits(__builtin_amdgcn_readlane(bits_from_f(v), 16));
  const float r2 = f_from_bits(__builtin_amdgcn_readlane(bits_from_f(v), 32));
  const float r3 = f_from_bits(__builtin_amdgcn_readlane(bits_from_f(v), 48));
  return (r0 + r1) + (r2 + r3);
}

// Sum over each aligned group of 16 lanes (one DPP row); every lane of the group gets the result.
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp<kQuadSwap1>(v);
  v += dpp<kQuadSwap2>(v);
  v += dpp<kRowHalfMirror>(v);
  v += dpp<kRowMirror>(v);
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp<kQuadSwap1>(v));
  v = fmaxf(v, dpp<kQuadSwap2>(v));
  v = fmaxf(v, dpp<kRowHalfMirror>(v));
  v = fmaxf(v, dpp<kRowMirror>(v));
  const float r0 = f_from_bits(__builtin_amdgcn_readlane(bits_from_f(v), 0));
  const float r1 = f_from_bits(__builtin_amdgcn_readlane(bits_from_f(v), 16));
  const float r2 = f_from_bits(__builtin_amdgcn_readlane(bits_from_f(v), 32));
  const float r3 = f_from_bits(__builtin_amdgcn_readlane(bits_from_f(v), 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// Per-bit constants of Eq. 1 for absmax m: scale = m / qmax, inv = qmax / m (correctly rounded
// fp32 divisions), both 0 when m == 0.
__device__ __forceinline__ void bit_constants(float m, int bits, float& scale, float& inv) {
  const float qmax = (float)((1 << (bits - 1)) - 1);
  if (m > 0.0f) {
    scale = m / qmax;  // IEEE division (the compiler default for HIP is correctly rounded)
    inv = qmax / m;
  } else {
    scale = 0.0f;
    inv = 0.0f;
  }
}

// Integer-valued float code of Eq. 1: RNE(x * inv) clamped to +-qmax.  The fused add of
// 1.5 * 2^23 rounds the exact product to an integer (ulp = 1 there, ties to even).
__device__ __forceinline__ float code_f(float x, float inv, float qmax) {
  const float t = __builtin_fmaf(x, inv, kMagic);
  const float q = t - kMagic;
  return __builtin_amdgcn_fmed3f(q, -qmax, qmax);
}

// Streaming access: a tensor that a kernel reads once is loaded non-temporally (the `nt` bit of
// the global load), so that it passes through the caches without displacing lines somebody will
// use again.  Measured on MI355X: the max calibration over 1.2 GB of weights reads 6.5 TB/s with it
// and 5.7 TB/s without, the error sweep 5.8-6.0 against 5.2-5.4.  The address-space cast also tells
// the compiler that the pointer is a global one where it cannot see that (pointers read from a
// table in memory would otherwise become flat loads).
__device__ __forceinline__ float4 load_stream(const float4* p) {
  typedef float v4f __attribute__((ext_vector_type(4)));
  const v4f v = __builtin_nontemporal_load((const __attribute__((address_space(1))) v4f*)p);
  return make_float4(v.x, v.y, v.z, v.w);
}

// Visits every float4 of x4[0, n4) that the tile round-robin deals to this block: f(value, index).
template <typename F>
__device__ __forceinline__ void for_each_vec4_tiled(const float4* __restrict__ x4, int64_t n4, F&& f) {
  constexpr int64_t tile = (int64_t)kBlock * kTileVec;
  const int64_t ntiles = (n4 + tile - 1) / tile;
  for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const int64_t base = t * tile + threadIdx.x;
    if ((t + 1) * tile <= n4) {  // block-uniform
      float4 v[kTileVec];
#pragma unroll
      for (int u = 0; u < kTileVec; ++u) v[u] = load_stream(x4 + base + u * kBlock);
#pragma unroll
      for (int u = 0; u < kTileVec; ++u) f(v[u], base + u * kBlock);
    } else {
#pragma unroll
      for (int u = 0; u < kTileVec; ++u) {
        const int64_t i = base + u * kBlock;
        if (i < n4) f(load_stream(x4 + i), i);
      }
    }
  }
}

// Same walk over two tensors at once: f(a, b); two + two loads in flight.
template <typename F>
__device__ __forceinline__ void for_each_vec4_pair_tiled(const float4* __restrict__ a4,
                                                         const float4* __restrict__ b4, int64_t n4, F&& f) {
  constexpr int U = 2;
  constexpr int64_t tile = (int64_t)kBlock * U;
  const int64_t ntiles = (n4 + tile - 1) / tile;
  for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const int64_t base = t * tile + threadIdx.x;
    if ((t + 1) * tile <= n4) {
      const float4 a0 = load_stream(a4 + base), b0 = load_stream(b4 + base), a1 = load_stream(a4 + base + kBlock),
                   b1 = load_stream(b4 + base + kBlock);
      f(a0, b0);
      f(a1, b1);
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t i = base + u * kBlock;
        if (i < n4) f(load_stream(a4 + i), load_stream(b4 + i));
      }
    }
  }
}

// |x| as an unsigned key: for non-negative floats the bit pattern orders like the value, so an
// integer atomic max over keys is an exact float max.
__device__ __forceinline__ unsigned abs_key(float v) { return (unsigned)bits_from_f(fabsf(v)); }

#endif  // __HIPCC__

}  // namespace mpq

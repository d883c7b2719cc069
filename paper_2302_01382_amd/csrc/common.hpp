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

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool mul_overflows(int64_t a, int64_t b) {
  int64_t r;
  return __builtin_mul_overflow(a, b, &r) || r > (int64_t)1 << 46;  // 2^46 elements: 256 TiB fp32
}

inline int64_t channels(int gran, int64_t rows, int64_t cols) {
  return gran == MPQ_PER_ROW ? rows : gran == MPQ_PER_COL ? cols : 1;
}

// grid for a flat streaming kernel: enough blocks to fill the chip several times over, never more
// than the work, so that a lane accumulates at most a few hundred elements in fp32.
inline unsigned flat_grid(int64_t vec_items, int items_per_thread, int blocks_per_cu = 8) {
  int64_t want = (vec_items + (int64_t)kBlock * items_per_thread - 1) / ((int64_t)kBlock * items_per_thread);
  int64_t cap = (int64_t)kNumCU * blocks_per_cu;
  // very large tensors: let the grid grow so a lane never sums more than ~1024 vectors
  int64_t min_for_len = (vec_items + (int64_t)kBlock * 1024 - 1) / ((int64_t)kBlock * 1024);
  if (cap < min_for_len) cap = min_for_len;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  return (unsigned)want;
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

// |x| as an unsigned key: for non-negative floats the bit pattern orders like the value, so an
// integer atomic max over keys is an exact float max.
__device__ __forceinline__ unsigned abs_key(float v) { return (unsigned)bits_from_f(fabsf(v)); }

#endif  // __HIPCC__

}  // namespace mpq

// sweep.hpp -- the per-lane accumulator of the quantization-error sweep (paper Sec. 3.2.1 Eq. 2):
// for NB consecutive bit-widths at once, acc_b += (Q_b(x) - x)^2 with Q_b the grid point code * scale_b.
//
// Per element and bit-width: t = fma(xc, inv_b, 1.5*2^23); q = t - 1.5*2^23; e = fma(q, scale_b, -x);
// acc_b = fma(e, e, acc_b) -- four VALU operations, with xc = clip(x, +-m) computed once per element
// (it replaces the clamp of the code).  The constants stay in registers for the whole kernel.
//
// Two bits take three: the grid is {-m, 0, +m} (qmax = 1, scale = m exactly), so the distance to the
// nearest grid point is min(|x|, ||x| - m|), also beyond the clip and for m = 0.  NB = 7 can only be
// the full range 2..8, so the first width of Sweep<7> is known to be 2 when the code is compiled.
// Within one ulp of the midpoint m/2 the choice of grid point can differ from RNE(x * inv); there
// the two distances are equal to that ulp, so the sum moves by a relative 1e-7 of one element's term.
#pragma once

#include "common.hpp"

namespace mpq {

template <int NB>
struct Sweep {
  float m;
  float inv[NB], sc[NB], acc[NB];
  __device__ __forceinline__ void init(float absmax, int b_lo) {
    m = absmax;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      bit_constants(absmax, b_lo + b, sc[b], inv[b]);
      acc[b] = 0.0f;
    }
  }
  __device__ __forceinline__ void add(float v) {
    const float vc = __builtin_amdgcn_fmed3f(v, -m, m);
    if (NB == 7) {
      const float a = __builtin_fabsf(v);
      const float e = __builtin_amdgcn_fmed3f(a, __builtin_fabsf(a - m), 0.0f);  // min of two non-negatives
      acc[0] = __builtin_fmaf(e, e, acc[0]);
    }
#pragma unroll
    for (int b = (NB == 7 ? 1 : 0); b < NB; ++b) {
      const float t = __builtin_fmaf(vc, inv[b], kMagic);
      const float q = t - kMagic;
      const float e = __builtin_fmaf(q, sc[b], -v);
      acc[b] = __builtin_fmaf(e, e, acc[b]);
    }
  }
  __device__ __forceinline__ void add4(const float4 v) { add(v.x); add(v.y); add(v.z); add(v.w); }
};

}  // namespace mpq

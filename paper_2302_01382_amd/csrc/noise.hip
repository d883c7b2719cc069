// noise.hip -- Gaussian perturbation of a tensor (paper Sec. 3.2.2 Eq. 3-5): y = x + sigma * z,
// sigma = lambda * scale_b(absmax): the spread is tied to max|w_i| through the b-bit step.
//
// z comes from a counter-based generator so that element i depends on (seed, stream_id, i) only:
//   Philox-4x32-10 (Salmon et al., SC'11): key = seed, counter = (i/4, stream_id) -> 4 words;
//   word pairs (0,1), (2,3) -> Box-Muller:  u1 = ((w >> 8) + 1) 2^-24, u2 = (w' >> 8) 2^-24,
//   r = sqrt(-2 ln u1), z_even = r cos(2 pi u2), z_odd = r sin(2 pi u2).
// ln / sin / cos are NOT library calls: they are fixed fp32 recipes (integer range reduction,
// Horner polynomials with explicit fused multiply-adds, coefficient tables below) so that any
// implementation following the recipe produces the same bits.  sqrt is the correctly rounded IEEE
// one (sqrtf under the compiler's default correctly-rounded-divide-sqrt mode, not the raw
// 1-ulp hardware instruction).
//
// One lane produces one group of four normals (one Philox call).  8 bytes of HBM traffic per
// element; ~45 integer + ~25 fp32 lane-operations per element.
#include "common.hpp"
#include "philox.hpp"

namespace mpq {

// -2 ln(k 2^-24), 1 <= k <= 2^24
__device__ __forceinline__ float neg2log_u24(unsigned k) {
  const float fk = (float)k;  // exact
  const unsigned bits = (unsigned)bits_from_f(fk);
  int e = (int)(bits >> 23) - 127;
  const unsigned mant = bits & 0x007FFFFFu;
  const bool upper = mant > 0x003504F3u;  // mantissa above sqrt(2): use m/2 and e+1
  const float m = f_from_bits((int)(mant | (upper ? 0x3F000000u : 0x3F800000u)));
  e += upper ? 1 : 0;
  const float t = m - 1.0f;  // exact
  float r = 0x1.40bfc2p-3f;
  r = __builtin_fmaf(r, t, -0x1.0aa1c6p-2f);
  r = __builtin_fmaf(r, t, 0x1.0e9656p-2f);
  r = __builtin_fmaf(r, t, -0x1.2202fap-2f);
  r = __builtin_fmaf(r, t, 0x1.542e08p-2f);
  r = __builtin_fmaf(r, t, -0x1.99aa6ap-2f);
  r = __builtin_fmaf(r, t, 0x1.00041ep-1f);
  r = __builtin_fmaf(r, t, -0x1.555540p-1f);
  r = __builtin_fmaf(r, t, 0x1.fffff8p-1f);
  r = __builtin_fmaf(r, t, -0x1.000000p+1f);
  const float q = t * r;
  return __builtin_fmaf((float)(24 - e), 0x1.62e430p+0f, q);
}

// cos, sin of 2 pi j 2^-24, 0 <= j < 2^24
__device__ __forceinline__ void sincos_2pi_u24(unsigned j, float& c_out, float& s_out) {
  const unsigned qd = (j + (1u << 21)) >> 22;           // nearest quarter turn, 0..4
  const int jr = (int)j - (int)(qd << 22);               // [-2^21, 2^21)
  const float y = (float)jr * 0x1.0p-24f;                // exact, turns
  const float v = y * y;
  float sp = -0x1.2d9bb8p+6f;
  sp = __builtin_fmaf(sp, v, 0x1.465ec6p+6f);
  sp = __builtin_fmaf(sp, v, -0x1.4abbbap+5f);
  sp = __builtin_fmaf(sp, v, 0x1.921fb6p+2f);
  const float s = y * sp;
  float c = 0x1.d9c364p+5f;
  c = __builtin_fmaf(c, v, -0x1.55c57cp+6f);
  c = __builtin_fmaf(c, v, 0x1.03c1dcp+6f);
  c = __builtin_fmaf(c, v, -0x1.3bd3ccp+4f);
  c = __builtin_fmaf(c, v, 0x1.000000p+0f);
  // rotate by qd quarter turns: swap on odd qd, then flip signs by bit tests (exact)
  const bool odd = qd & 1u;
  const float cc = odd ? s : c;
  const float ss = odd ? c : s;
  const unsigned cneg = ((qd + 1u) & 2u) << 30;  // qd = 1, 2 -> cos negative
  const unsigned sneg = (qd & 2u) << 30;         // qd = 2, 3 -> sin negative
  c_out = f_from_bits(bits_from_f(cc) ^ (int)cneg);
  s_out = f_from_bits(bits_from_f(ss) ^ (int)sneg);
}

__device__ __forceinline__ float4 gauss4(unsigned long long seed, unsigned long long sid,
                                         unsigned long long g) {
  const U4 w = philox4x32_10((unsigned)g, (unsigned)(g >> 32), (unsigned)sid, (unsigned)(sid >> 32),
                             (unsigned)seed, (unsigned)(seed >> 32));
  float4 z;
  float c, s;
  float r = __builtin_sqrtf(neg2log_u24((w.a >> 8) + 1u));
  sincos_2pi_u24(w.b >> 8, c, s);
  z.x = r * c;
  z.y = r * s;
  r = __builtin_sqrtf(neg2log_u24((w.c >> 8) + 1u));
  sincos_2pi_u24(w.d >> 8, c, s);
  z.z = r * c;
  z.w = r * s;
  return z;
}

__device__ __forceinline__ float sigma_of(float absmax, int bits, float lambda) {
  float scale, inv;
  bit_constants(absmax, bits, scale, inv);
  return lambda * scale;
}

// ---- one sigma for the whole group of four: per tensor, or per row with cols % 4 == 0 -------
// ROWS = false: flat; ROWS = true: group g lies in row g / (cols/4)
// Both kernels write nb outputs, one per bit-width b_lo .. b_lo + nb - 1, `stride` elements apart:
// z does not depend on b, so a sweep over bit-widths draws it once per element.
template <bool ROWS>
__global__ __launch_bounds__(kBlock) void noise_vec(const float* __restrict__ x, int64_t n4,
                                                    int64_t cols4, const float* __restrict__ absmax,
                                                    int b_lo, int nb, float lambda, unsigned long long seed,
                                                    unsigned long long sid, float* __restrict__ y,
                                                    int64_t stride4) {
  for_each_vec4_tiled(reinterpret_cast<const float4*>(x), n4, [&](const float4 v, int64_t g) {
    const float m = absmax[ROWS ? g / cols4 : 0];
    const float4 z = gauss4(seed, sid, (unsigned long long)g);
    for (int k = 0; k < nb; ++k) {
      const float sig = sigma_of(m, b_lo + k, lambda);
      reinterpret_cast<float4*>(y)[g + k * stride4] =
          make_float4(__builtin_fmaf(sig, z.x, v.x), __builtin_fmaf(sig, z.y, v.y),
                      __builtin_fmaf(sig, z.z, v.z), __builtin_fmaf(sig, z.w, v.w));
    }
  });
}

// ---- generic: any shape, alignment, granularity; a lane still owns one group of four ----------
__global__ __launch_bounds__(kBlock) void noise_generic(const float* __restrict__ x, int64_t rows,
                                                        int64_t cols, int gran,
                                                        const float* __restrict__ absmax, int b_lo, int nb,
                                                        float lambda, unsigned long long seed,
                                                        unsigned long long sid, float* __restrict__ y,
                                                        int64_t stride) {
  const int64_t n = rows * cols;
  const int64_t n4 = (n + 3) >> 2;
  for (int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x; g < n4; g += (int64_t)gridDim.x * kBlock) {
    const float4 z = gauss4(seed, sid, (unsigned long long)g);
    const float zz[4] = {z.x, z.y, z.z, z.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int64_t i = 4 * g + e;
      if (i < n) {
        const int64_t r = i / cols, c = i - r * cols;
        const int64_t ch = gran == MPQ_PER_ROW ? r : gran == MPQ_PER_COL ? c : 0;
        const float m = absmax[ch], xi = x[i];
        for (int k = 0; k < nb; ++k) y[i + k * stride] = __builtin_fmaf(sigma_of(m, b_lo + k, lambda), zz[e], xi);
      }
    }
  }
}

static int launch_noise(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax, int b_lo,
                        int nb, float lambda, uint64_t seed, uint64_t stream_id, float* y_out, int64_t stride,
                        hipStream_t st) {
  const int64_t n = rows * cols;
  const bool vec = aligned16(x) && aligned16(y_out) && (n & 3) == 0 && (stride & 3) == 0;
  if (vec && gran == MPQ_PER_TENSOR) {
    noise_vec<false><<<flat_grid(n >> 2, kBlock * kTileVec), kBlock, 0, st>>>(x, n >> 2, 0, absmax, b_lo, nb, lambda, seed, stream_id, y_out, stride >> 2);
  } else if (vec && gran == MPQ_PER_ROW && (cols & 3) == 0) {
    noise_vec<true><<<flat_grid(n >> 2, kBlock * kTileVec), kBlock, 0, st>>>(x, n >> 2, cols >> 2, absmax, b_lo, nb, lambda, seed, stream_id, y_out, stride >> 2);
  } else {
    noise_generic<<<flat_grid((n + 3) >> 2, kBlock * 2), kBlock, 0, st>>>(x, rows, cols, gran, absmax, b_lo, nb, lambda, seed, stream_id, y_out, stride);
  }
  return launch_status();
}

}  // namespace mpq

using namespace mpq;

extern "C" int mpq_noise_inject(const float* x, int64_t rows, int64_t cols, int gran,
                                const float* absmax, int bits, float lambda, uint64_t seed,
                                uint64_t stream_id, float* y_out, void* stream) {
  if (!x || !absmax || !y_out) return MPQ_ERR_NULL;
  if (rows <= 0 || cols <= 0 || mul_overflows(rows, cols)) return MPQ_ERR_SHAPE;
  if (gran < MPQ_PER_TENSOR || gran > MPQ_PER_COL) return MPQ_ERR_GRAN;
  if (bits < 2 || bits > 8) return MPQ_ERR_BITS;
  return launch_noise(x, rows, cols, gran, absmax, bits, 1, lambda, seed, stream_id, y_out, 0, (hipStream_t)stream);
}

extern "C" int mpq_noise_inject_sweep(const float* x, int64_t rows, int64_t cols, int gran,
                                      const float* absmax, int b_lo, int b_hi, float lambda, uint64_t seed,
                                      uint64_t stream_id, float* y_out, int64_t y_stride, void* stream) {
  if (!x || !absmax || !y_out) return MPQ_ERR_NULL;
  if (rows <= 0 || cols <= 0 || mul_overflows(rows, cols)) return MPQ_ERR_SHAPE;
  if (gran < MPQ_PER_TENSOR || gran > MPQ_PER_COL) return MPQ_ERR_GRAN;
  if (b_lo < 2 || b_hi > 8 || b_lo > b_hi) return MPQ_ERR_BITS;
  if (y_stride < rows * cols || mul_overflows(y_stride, 8)) return MPQ_ERR_SHAPE;  // planes must not overlap
  return launch_noise(x, rows, cols, gran, absmax, b_lo, b_hi - b_lo + 1, lambda, seed, stream_id, y_out, y_stride,
                      (hipStream_t)stream);
}

// scale_adjust.hip -- the adjustment step of Sec. 3.1: after max calibration the two scales of
// Eq. 1 are free parameters and are moved by gradient descent while the model's own parameters
// stay put.  In the integer form used throughout this library the pair is
//   inv   (= alpha * levels): applied before rounding,     code = clamp(RNE(x * inv), +-qmax)
//   scale (= gamma / levels): applied after,                Q = code * scale
// and calibration sets inv = qmax / m, scale = m / qmax.
//
// Gradients treat rounding as the identity (straight-through): with g = dL/dQ
//   dL/dscale = sum g * code
//   dL/dinv   = scale * sum over elements whose rounded value needs no clamping of g * x
// g == NULL selects the reconstruction loss L = sum (Q - x)^2, g = 2 (Q - x).
//
// code for arbitrary inv: x is first clamped to +-2^20 / |inv| so that the magic-number rounding
// (exact product rounded to nearest even by one fused add of 1.5 * 2^23) stays in its valid range;
// 2^20 is far beyond qmax + 1/2, so neither the code nor the "needs no clamping" test changes.
#include "common.hpp"

namespace mpq {

struct TwoScales {
  float inv, scale, lim, qmax;
  __device__ __forceinline__ TwoScales(float inv_, float scale_, int bits) : inv(inv_), scale(scale_) {
    qmax = (float)((1 << (bits - 1)) - 1);
    lim = 1048576.0f / fabsf(inv_);  // +inf for inv == 0: nothing to clamp, every product is 0
  }
  // rounded value before clamping, as an integer-valued float
  __device__ __forceinline__ float rounded(float x) const {
    const float xc = __builtin_amdgcn_fmed3f(x, -lim, lim);
    return __builtin_fmaf(xc, inv, kMagic) - kMagic;
  }
};

// lane-local sums of one element's contributions
struct GradAcc {
  float s_code = 0.0f, s_x = 0.0f, s_loss = 0.0f;
  template <bool HAS_G>
  __device__ __forceinline__ void add(const TwoScales& t, float x, float g_in) {
    const float r = t.rounded(x);
    const float q = __builtin_amdgcn_fmed3f(r, -t.qmax, t.qmax);
    const float e = __builtin_fmaf(q, t.scale, -x);
    const float g = HAS_G ? g_in : 2.0f * e;
    s_code = __builtin_fmaf(g, q, s_code);
    if (r == q) s_x = __builtin_fmaf(g, x, s_x);  // the clamp was inactive
    s_loss = __builtin_fmaf(e, e, s_loss);
  }
};

// ---- per tensor: tiles dealt round-robin, one partial triple per workgroup ---------------------
template <bool HAS_G, bool VEC>
__global__ __launch_bounds__(kBlock) void sg_flat(const float* __restrict__ x, const float* __restrict__ g,
                                                  int64_t n, const float* __restrict__ inv,
                                                  const float* __restrict__ scale, int bits,
                                                  double* __restrict__ partials) {
  const TwoScales t(inv[0], scale[0], bits);
  GradAcc a;
  if (VEC) {
    const int64_t n4 = n >> 2;
    if (HAS_G) {
      for_each_vec4_pair_tiled(reinterpret_cast<const float4*>(x), reinterpret_cast<const float4*>(g), n4,
                               [&](const float4 v, const float4 u) {
                                 a.add<true>(t, v.x, u.x); a.add<true>(t, v.y, u.y);
                                 a.add<true>(t, v.z, u.z); a.add<true>(t, v.w, u.w);
                               });
    } else {
      for_each_vec4_tiled(reinterpret_cast<const float4*>(x), n4, [&](const float4 v, int64_t) {
        a.add<false>(t, v.x, 0.0f); a.add<false>(t, v.y, 0.0f);
        a.add<false>(t, v.z, 0.0f); a.add<false>(t, v.w, 0.0f);
      });
    }
  } else {
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock)
      a.add<HAS_G>(t, x[i], HAS_G ? g[i] : 0.0f);
  }
  __shared__ float sm[3][kBlock / kWave];
  const float w0 = wave_sum(a.s_code), w1 = wave_sum(a.s_x), w2 = wave_sum(a.s_loss);
  if ((threadIdx.x & (kWave - 1)) == 0) {
    sm[0][threadIdx.x / kWave] = w0;
    sm[1][threadIdx.x / kWave] = w1;
    sm[2][threadIdx.x / kWave] = w2;
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    const float* s = sm[threadIdx.x];
    partials[(int64_t)blockIdx.x * 3 + threadIdx.x] = ((double)s[0] + (double)s[1]) + ((double)s[2] + (double)s[3]);
  }
}

// one workgroup folds the partial triples in a fixed order and applies the factor of dL/dinv
__global__ __launch_bounds__(kBlock) void sg_finish(const double* __restrict__ partials, int64_t count,
                                                    const float* __restrict__ scale, double* __restrict__ dinv,
                                                    double* __restrict__ dscale, double* __restrict__ loss) {
  __shared__ double sm[3][kBlock];
  double a0 = 0.0, a1 = 0.0, a2 = 0.0;
  for (int64_t i = threadIdx.x; i < count; i += kBlock) {
    a0 += partials[i * 3];
    a1 += partials[i * 3 + 1];
    a2 += partials[i * 3 + 2];
  }
  sm[0][threadIdx.x] = a0;
  sm[1][threadIdx.x] = a1;
  sm[2][threadIdx.x] = a2;
  __syncthreads();
  for (int h = kBlock / 2; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h)
      for (int k = 0; k < 3; ++k) sm[k][threadIdx.x] += sm[k][threadIdx.x + h];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    dscale[0] = sm[0][0];
    dinv[0] = (double)scale[0] * sm[1][0];
    if (loss) loss[0] = sm[2][0];
  }
}

// ---- per row: one wave per row, results written directly ---------------------------------------
template <bool HAS_G, bool VEC>
__global__ __launch_bounds__(kBlock) void sg_rows(const float* __restrict__ x, const float* __restrict__ g,
                                                  int64_t rows, int64_t cols, const float* __restrict__ inv,
                                                  const float* __restrict__ scale, int bits,
                                                  double* __restrict__ dinv, double* __restrict__ dscale,
                                                  double* __restrict__ loss) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t r = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
  if (r >= rows) return;  // the whole wave leaves together
  const TwoScales t(inv[r], scale[r], bits);
  GradAcc a;
  const float* xr = x + r * cols;
  const float* gr = HAS_G ? g + r * cols : nullptr;
  if (VEC) {  // cols % 4 == 0 and 16-byte aligned tensors: rows start aligned
    const float4* x4 = reinterpret_cast<const float4*>(xr);
    const float4* g4 = reinterpret_cast<const float4*>(gr);
    for (int64_t c = lane; c < (cols >> 2); c += kWave) {
      const float4 v = x4[c];
      const float4 u = HAS_G ? g4[c] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      a.add<HAS_G>(t, v.x, u.x); a.add<HAS_G>(t, v.y, u.y);
      a.add<HAS_G>(t, v.z, u.z); a.add<HAS_G>(t, v.w, u.w);
    }
  } else {
    for (int64_t c = lane; c < cols; c += kWave) a.add<HAS_G>(t, xr[c], HAS_G ? gr[c] : 0.0f);
  }
  const float w0 = wave_sum(a.s_code), w1 = wave_sum(a.s_x), w2 = wave_sum(a.s_loss);
  if (lane == 0) {
    dscale[r] = (double)w0;
    dinv[r] = (double)t.scale * (double)w1;
    if (loss) loss[r] = (double)w2;
  }
}

// ---- forward with explicit scales ----------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void fq_scales_k(const float* __restrict__ x, int64_t n, int64_t cols,
                                                      int per_row, const float* __restrict__ inv,
                                                      const float* __restrict__ scale, int bits,
                                                      float* __restrict__ y, int8_t* __restrict__ codes) {
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
    const int64_t ch = per_row ? i / cols : 0;
    const TwoScales t(inv[ch], scale[ch], bits);
    const float q = __builtin_amdgcn_fmed3f(t.rounded(x[i]), -t.qmax, t.qmax);
    if (y) y[i] = q * t.scale;
    if (codes) codes[i] = (int8_t)(int)q;
  }
}

// ---- p <- fl32(p - lr * dL/dp), in double, rounded once -----------------------------------------
__global__ void sgd_k(float* __restrict__ inv, float* __restrict__ scale, const double* __restrict__ dinv,
                      const double* __restrict__ dscale, int64_t count, double lr) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  inv[i] = (float)((double)inv[i] - lr * dinv[i]);
  scale[i] = (float)((double)scale[i] - lr * dscale[i]);
}

static int check_sa(int64_t rows, int64_t cols, int gran, int bits) {
  if (rows <= 0 || cols <= 0 || mul_overflows(rows, cols)) return MPQ_ERR_SHAPE;
  if (gran != MPQ_PER_TENSOR && gran != MPQ_PER_ROW) return MPQ_ERR_GRAN;
  if (bits < 2 || bits > 8) return MPQ_ERR_BITS;
  if (gran == MPQ_PER_ROW && (rows + 3) / 4 > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  return MPQ_OK;
}

static unsigned sg_grid(int64_t n, bool vec, bool has_g) {
  if (!vec) return flat_grid(n, kBlock * 4);
  return flat_grid(n >> 2, kBlock * (has_g ? 2 : kTileVec));
}

}  // namespace mpq

using namespace mpq;

extern "C" int mpq_fake_quant_scales(const float* x, int64_t rows, int64_t cols, int gran, const float* inv,
                                     const float* scale, int bits, float* y_out, int8_t* codes_out,
                                     void* stream) {
  if (!x || !inv || !scale || (!y_out && !codes_out)) return MPQ_ERR_NULL;
  const int rc = check_sa(rows, cols, gran, bits);
  if (rc != MPQ_OK) return rc;
  const int64_t n = rows * cols;
  fq_scales_k<<<flat_grid(n, kBlock * 4), kBlock, 0, (hipStream_t)stream>>>(x, n, cols, gran == MPQ_PER_ROW, inv, scale,
                                                                           bits, y_out, codes_out);
  return launch_status();
}

extern "C" size_t mpq_scale_grad_workspace_bytes(int64_t rows, int64_t cols, int gran) {
  if (check_sa(rows, cols, gran, 8) != MPQ_OK || gran != MPQ_PER_TENSOR) return 0;
  const int64_t n = rows * cols;
  unsigned g = sg_grid(n, false, false);
  for (int v = 0; v < 2; ++v) {  // the largest grid any variant may use
    const unsigned c = sg_grid(n, true, v != 0);
    g = c > g ? c : g;
  }
  return (size_t)g * 3 * sizeof(double);
}

extern "C" int mpq_scale_grad(const float* x, int64_t rows, int64_t cols, int gran, const float* inv,
                              const float* scale, int bits, const float* g, double* dinv_out,
                              double* dscale_out, double* loss_out, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !inv || !scale || !dinv_out || !dscale_out) return MPQ_ERR_NULL;
  const int rc = check_sa(rows, cols, gran, bits);
  if (rc != MPQ_OK) return rc;
  if ((reinterpret_cast<uintptr_t>(dinv_out) | reinterpret_cast<uintptr_t>(dscale_out) |
       reinterpret_cast<uintptr_t>(loss_out)) & 7u)
    return MPQ_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const int64_t n = rows * cols;
  const bool vec = aligned16(x) && (!g || aligned16(g));
  if (gran == MPQ_PER_TENSOR) {
    if (!ws || ws_bytes < mpq_scale_grad_workspace_bytes(rows, cols, gran)) return MPQ_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) & 7u) return MPQ_ERR_ALIGN;
    double* partials = reinterpret_cast<double*>(ws);
    const bool v = vec && (n & 3) == 0;
    const unsigned grid = sg_grid(n, v, g != nullptr);
    if (g) {
      if (v) sg_flat<true, true><<<grid, kBlock, 0, st>>>(x, g, n, inv, scale, bits, partials);
      else sg_flat<true, false><<<grid, kBlock, 0, st>>>(x, g, n, inv, scale, bits, partials);
    } else {
      if (v) sg_flat<false, true><<<grid, kBlock, 0, st>>>(x, g, n, inv, scale, bits, partials);
      else sg_flat<false, false><<<grid, kBlock, 0, st>>>(x, g, n, inv, scale, bits, partials);
    }
    sg_finish<<<1, kBlock, 0, st>>>(partials, (int64_t)grid, scale, dinv_out, dscale_out, loss_out);
  } else {
    const bool v = vec && (cols & 3) == 0;
    const unsigned grid = (unsigned)((rows + 3) / 4);
    if (g) {
      if (v) sg_rows<true, true><<<grid, kBlock, 0, st>>>(x, g, rows, cols, inv, scale, bits, dinv_out, dscale_out, loss_out);
      else sg_rows<true, false><<<grid, kBlock, 0, st>>>(x, g, rows, cols, inv, scale, bits, dinv_out, dscale_out, loss_out);
    } else {
      if (v) sg_rows<false, true><<<grid, kBlock, 0, st>>>(x, g, rows, cols, inv, scale, bits, dinv_out, dscale_out, loss_out);
      else sg_rows<false, false><<<grid, kBlock, 0, st>>>(x, g, rows, cols, inv, scale, bits, dinv_out, dscale_out, loss_out);
    }
  }
  return launch_status();
}

extern "C" int mpq_scale_sgd_step(float* inv, float* scale, const double* dinv, const double* dscale,
                                  int64_t count, double lr, void* stream) {
  if (!inv || !scale || !dinv || !dscale) return MPQ_ERR_NULL;
  if (count <= 0 || (count + 255) / 256 > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  sgd_k<<<(unsigned)((count + 255) / 256), 256, 0, (hipStream_t)stream>>>(inv, scale, dinv, dscale, count, lr);
  return launch_status();
}

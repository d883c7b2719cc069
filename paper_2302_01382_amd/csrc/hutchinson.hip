// hutchinson.hip -- Hutchinson's estimate of the trace of the Hessian (paper Sec. 3.2.3,
// E_Hessian = E[Tr(d^2 L / d w_i^2)]) for the one case that needs no network behind it: a linear
// layer Y = X W' under L = mean((Y - T)^2).  L is quadratic in W with Hessian
// (2 / (M N)) (I_N (x) X'X), so a probe's quadratic form is a sum of ||X v||^2 over K-vectors v,
// and Tr(H) ~= (2 / M) mean_p ||X v_p||^2 (exact value: (2 / M) ||X||_F^2).
//
//   mpq_rademacher       the probes: random signs, one Philox bit per element
//   mpq_hutchinson_quad  quad[p] = ||X v_p||^2 = sum_m (sum_k X[m][k] v[p][k])^2
//
// The second is a dense contraction X [M x K] times V' [K x P] followed by a column-wise sum of
// squares, so it runs on the fp32 matrix cores (v_mfma_f32_32x32x2_f32; products with +-1 are
// exact, the sums over k round in fp32).  X is read once per group of up to 128 probes; with 32
// probes the kernel is bound by that read (4 bytes per element of X against 64 flops), with 128
// by the fp32 matrix rate.  V (P x K floats, at most a few MB) stays in L2.
//
// A workgroup of four waves owns 32 rows of X at a time; the waves split k between them in chunks
// of 32 (lane l: row l % 32, sixteen consecutive k in half l / 32 of the chunk, loaded as four
// 16-byte pieces that feed four K = 2 matrix steps each), add their 32 x 32 partial products
// through LDS, and wave 0 squares and accumulates.  Lane l of a product tile holds column
// p = l % 32 and sixteen of the rows m, so the column sums of squares need no cross-lane work
// until the very end.
#include "common.hpp"
#include "philox.hpp"

namespace mpq {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kHW = 4;            // waves per workgroup
constexpr int kProbeGroup = 128;  // probes per pass over X

// thread w owns word w of the sign stream: elements 32 w .. 32 w + 31
__global__ __launch_bounds__(kBlock) void rademacher_k(unsigned long long seed, unsigned long long sid,
                                                       int64_t n, float* __restrict__ out) {
  const int64_t w = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t e0 = w << 5;
  if (e0 >= n) return;
  const unsigned long long g = (unsigned long long)(w >> 2);
  const U4 r = philox4x32_10((unsigned)g, (unsigned)(g >> 32), (unsigned)sid, (unsigned)(sid >> 32),
                             (unsigned)seed, (unsigned)(seed >> 32) ^ 0x5241444Du);
  const unsigned sel = (unsigned)w & 3u;
  const unsigned word = sel == 0 ? r.a : sel == 1 ? r.b : sel == 2 ? r.c : r.d;
#pragma unroll 8
  for (int t = 0; t < 32; ++t)
    if (e0 + t < n) out[e0 + t] = ((word >> t) & 1u) ? -1.0f : 1.0f;
}

// four floats at p (k .. k+3) with everything at or past `left` elements zeroed
template <bool VEC>
__device__ __forceinline__ float4 load4f(const float* __restrict__ p, int64_t left, bool ok) {
  if (VEC) {  // left is a multiple of 4: the piece is whole or absent
    return (ok && left > 0) ? *reinterpret_cast<const float4*>(p) : make_float4(0.f, 0.f, 0.f, 0.f);
  } else {
    float4 r;
    r.x = (ok && left > 0) ? p[0] : 0.f;
    r.y = (ok && left > 1) ? p[1] : 0.f;
    r.z = (ok && left > 2) ? p[2] : 0.f;
    r.w = (ok && left > 3) ? p[3] : 0.f;
    return r;
  }
}

// part: float [gridDim.x][PB * 32], this workgroup's share of sum_m (X V')[m][p]^2
template <int PB, bool VEC>
__global__ __launch_bounds__(kHW * 64, 2) void hutch_k(const float* __restrict__ X, int64_t M, int64_t K,
                                                       const float* __restrict__ V, int64_t P,
                                                       float* __restrict__ part) {
  __shared__ float red[kHW - 1][PB][16][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int row = lane & 31, half = lane >> 5;
  const int64_t nchunk = (K + 31) >> 5;
  const int64_t nblk = (M + 31) >> 5;
  float s[PB];
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) s[pb] = 0.0f;

  for (int64_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
    const int64_t m = blk * 32 + row;
    const bool m_ok = m < M;
    const float* xr = X + (m_ok ? m : 0) * K;
    v16f acc[PB];
#pragma unroll
    for (int pb = 0; pb < PB; ++pb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[pb][v] = 0.0f;

    float4 xa[4];
    {
      const int64_t kb = (int64_t)wave * 32 + half * 16;
#pragma unroll
      for (int e = 0; e < 4; ++e) xa[e] = load4f<VEC>(xr + kb + 4 * e, K - (kb + 4 * e), m_ok && wave < nchunk);
    }
    for (int64_t c = wave; c < nchunk; c += kHW) {
      const int64_t kb = c * 32 + half * 16;
      float4 xn[4];  // this wave's next chunk of X, requested before the matrix steps of this one
      {
        const int64_t kn = kb + kHW * 32;
#pragma unroll
        for (int e = 0; e < 4; ++e) xn[e] = load4f<VEC>(xr + kn + 4 * e, K - (kn + 4 * e), m_ok && c + kHW < nchunk);
      }
#pragma unroll
      for (int pb = 0; pb < PB; ++pb) {
        const int64_t p = pb * 32 + row;
        const bool p_ok = p < P;
        const float* vr = V + (p_ok ? p : 0) * K + kb;
        float4 va[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) va[e] = load4f<VEC>(vr + 4 * e, K - (kb + 4 * e), p_ok);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[e].x, va[e].x, acc[pb], 0, 0, 0);
          acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[e].y, va[e].y, acc[pb], 0, 0, 0);
          acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[e].z, va[e].z, acc[pb], 0, 0, 0);
          acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[e].w, va[e].w, acc[pb], 0, 0, 0);
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) xa[e] = xn[e];
    }

    // the four k shares of the 32 x 32 products meet in wave 0, in a fixed order
    if (wave > 0) {
#pragma unroll
      for (int pb = 0; pb < PB; ++pb)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave - 1][pb][v][lane] = acc[pb][v];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int pb = 0; pb < PB; ++pb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float d = ((acc[pb][v] + red[0][pb][v][lane]) + red[1][pb][v][lane]) + red[2][pb][v][lane];
          s[pb] = __builtin_fmaf(d, d, s[pb]);
        }
    }
    __syncthreads();  // red is free again
  }
  if (wave == 0) {
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      const float t = s[pb] + __shfl_xor(s[pb], 32);  // the two halves hold different rows of the same column
      if (lane < 32) part[(int64_t)blockIdx.x * (PB * 32) + pb * 32 + lane] = t;
    }
  }
}

// quad[p] = sum over workgroups of part[b][p], in double, fixed order; one workgroup per probe
__global__ __launch_bounds__(kBlock) void hutch_finish(const float* __restrict__ part, int nblocks, int width,
                                                       double* __restrict__ quad) {
  const int p = blockIdx.x;
  double t = 0.0;
  for (int b = threadIdx.x; b < nblocks; b += kBlock) t += (double)part[(int64_t)b * width + p];
  __shared__ double sm[kBlock];
  sm[threadIdx.x] = t;
  __syncthreads();
  for (int o = kBlock / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) quad[p] = sm[0];
}

static int probe_blocks(int64_t pg) { return pg <= 32 ? 1 : pg <= 64 ? 2 : 4; }

// workgroups of one pass: a few per CU, every lane accumulating at most 256 row blocks in fp32
static int64_t hutch_grid(int64_t M, int pb) {
  const int64_t nblk = (M + 31) >> 5;
  int64_t g = (int64_t)kNumCU * (pb == 1 ? 4 : 2);
  if (g > nblk) g = nblk;
  const int64_t need = (nblk + 255) / 256;
  return g > need ? g : need;
}

}  // namespace mpq

using namespace mpq;

extern "C" int mpq_rademacher(uint64_t seed, uint64_t stream_id, int64_t rows, int64_t cols, float* v_out,
                              void* stream) {
  if (!v_out) return MPQ_ERR_NULL;
  if (rows <= 0 || cols <= 0 || mul_overflows(rows, cols) || rows * cols > ((int64_t)1 << 38)) return MPQ_ERR_SHAPE;
  const int64_t n = rows * cols;
  const int64_t words = (n + 31) >> 5;
  rademacher_k<<<(unsigned)((words + kBlock - 1) / kBlock), kBlock, 0, (hipStream_t)stream>>>(seed, stream_id, n, v_out);
  return launch_status();
}

extern "C" size_t mpq_hutchinson_quad_workspace_bytes(int64_t M, int64_t K, int64_t P) {
  if (M <= 0 || K <= 0 || P <= 0 || mul_overflows(M, K) || mul_overflows(P, K)) return 0;
  size_t most = 0;
  for (int pb = 1; pb <= 4; pb *= 2) {
    const size_t b = (size_t)hutch_grid(M, pb) * (size_t)(pb * 32) * sizeof(float);
    if (b > most) most = b;
  }
  return most;
}

extern "C" int mpq_hutchinson_quad(const float* x, int64_t M, int64_t K, const float* v, int64_t P,
                                   double* quad_out, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !v || !quad_out) return MPQ_ERR_NULL;
  if (M <= 0 || K <= 0 || P <= 0 || M >= ((int64_t)1 << 31) || P > ((int64_t)1 << 20)) return MPQ_ERR_SHAPE;
  if (mul_overflows(M, K) || mul_overflows(P, K)) return MPQ_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(x) & 3u) || (reinterpret_cast<uintptr_t>(v) & 3u) ||
      (reinterpret_cast<uintptr_t>(quad_out) & 7u))
    return MPQ_ERR_ALIGN;
  if (!ws || ws_bytes < mpq_hutchinson_quad_workspace_bytes(M, K, P)) return MPQ_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 3u) return MPQ_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  float* part = reinterpret_cast<float*>(ws);
  const bool vec = aligned16(x) && aligned16(v) && (K & 3) == 0;
  for (int64_t p0 = 0; p0 < P; p0 += kProbeGroup) {
    const int64_t pg = P - p0 < kProbeGroup ? P - p0 : kProbeGroup;
    const int pb = probe_blocks(pg);
    const unsigned g = (unsigned)hutch_grid(M, pb);
    const float* vg = v + p0 * K;
#define MPQ_HUTCH(PB_)                                                                  \
  (vec ? hutch_k<PB_, true><<<g, kHW * 64, 0, st>>>(x, M, K, vg, pg, part)              \
       : hutch_k<PB_, false><<<g, kHW * 64, 0, st>>>(x, M, K, vg, pg, part))
    if (pb == 1) MPQ_HUTCH(1);
    else if (pb == 2) MPQ_HUTCH(2);
    else MPQ_HUTCH(4);
#undef MPQ_HUTCH
    hutch_finish<<<(unsigned)pg, kBlock, 0, st>>>(part, (int)g, pb * 32, quad_out + p0);
  }
  return launch_status();
}

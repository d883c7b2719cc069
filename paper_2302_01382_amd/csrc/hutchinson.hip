// hutchinson.hip -- Hutchinson's estimate of the trace of the Hessian (paper Sec. 3.2.3,
// E_Hessian = E[Tr(d^2 L / d w_i^2)]) for the one case that needs no network behind it: a linear
// layer Y = X W' under L = mean((Y - T)^2).  L is quadratic in W with Hessian
// (2 / (M N)) (I_N (x) X'X), so a probe's quadratic form is a sum of ||X v||^2 over K-vectors v,
// and Tr(H) ~= (2 / M) mean_p ||X v_p||^2 (exact value: (2 / M) ||X||_F^2).
//
//   mpq_rademacher       the probes: random signs, one Philox bit per element
//   mpq_hutchinson_quad  quad[p] = ||X v_p||^2 = sum_m (sum_k X[m][k] v[p][k])^2
//   mpq_hutchinson_quad_signs  the same with the sign probes drawn inside the kernel (the bits
//                        mpq_rademacher would store): no probe matrix is read at all
//
// The second is a dense contraction X [M x K] times V' [K x P] followed by a column-wise sum of
// squares, so it runs on the fp32 matrix cores (v_mfma_f32_32x32x2_f32; products with +-1 are
// exact, the sums over k round in fp32).  X is read once per group of up to 64 probes; with 32
// probes the kernel is bound by that read (4 bytes per element of X against 64 flops), with 64
// the fp32 matrix rate is level with it.  V (P x K floats, at most a few MB) stays in L2.
//
// A workgroup of eight waves owns 32 rows of X at a time; the waves split k between them (a
// contiguous eighth each) and walk it in chunks of 32 (lane l: row l % 32, sixteen consecutive k in half l / 32 of the chunk, loaded as four
// 16-byte pieces that feed four K = 2 matrix steps each), add their 32 x 32 partial products
// through LDS, and wave 0 squares and accumulates.  Lane l of a product tile holds column
// p = l % 32 and sixteen of the rows m, so the column sums of squares need no cross-lane work
// until the very end.
#include "common.hpp"
#include "philox.hpp"

namespace mpq {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kHW = 8;           // waves per workgroup; they split k
constexpr int kProbeGroup = 64;  // probes per pass over X: the width at which the fp32 matrix rate
                                 // (64 flops per byte of X at the HBM rate) and the read of X balance

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

// One chunk of a wave's operands: CH pieces of four k each of X row `row` and of PB x 32 probe
// rows (lane (row, half) owns the k range [c * 8 CH + half * 4 CH, + 4 CH) of chunk c).
template <int PB, int CH>
struct Operands {
  float4 x[CH];
  float4 v[PB][CH];
};

// Where the probes come from: a matrix in memory, or (SIGNS) the sign stream of mpq_rademacher
// drawn on the spot: with K a multiple of 16 the sixteen signs a lane needs for a chunk are one
// half of a 32-bit Philox word (one Philox call per lane and chunk, about 80 vector operations
// next to the chunk's 16 matrix steps of 64 clocks each).  Chunks of 64 k (a whole word per lane)
// were slower: a lane's run of 128 bytes puts 64 different lines under every load instruction.
struct Probes {
  const float* V;
  unsigned long long seed, sid, first;  // first: index of probe row 0 of this pass in the sign matrix
};

// the sixteen signs starting at element `base` (a multiple of 16) of the sign matrix, in the low bits
__device__ __forceinline__ unsigned sign_word(const Probes& pr, unsigned long long base) {
  const unsigned long long g = base >> 7;
  const U4 w = philox4x32_10((unsigned)g, (unsigned)(g >> 32), (unsigned)pr.sid, (unsigned)(pr.sid >> 32),
                             (unsigned)pr.seed, (unsigned)(pr.seed >> 32) ^ 0x5241444Du);
  const unsigned sel = (unsigned)(base >> 5) & 3u;
  const unsigned word = sel == 0 ? w.a : sel == 1 ? w.b : sel == 2 ? w.c : w.d;
  return word >> ((unsigned)base & 16u);
}

__device__ __forceinline__ float sign_f(unsigned bits, int t) {  // +1.0f, or -1.0f if bit t is set
  return f_from_bits((int)(0x3F800000u | (((bits >> t) & 1u) << 31)));
}

// piece e (four k) of the chunk that starts at kb for this lane: X always, V when it is in memory
template <int PB, int CH, bool VEC, bool SIGNS>
__device__ __forceinline__ void load_piece(Operands<PB, CH>& o, int e, const float* __restrict__ xr, bool m_ok,
                                           const Probes& pr, int64_t P, int64_t K, int64_t kb, int row, bool live) {
  const int64_t k = kb + 4 * e;
  o.x[e] = load4f<VEC>(xr + k, K - k, live && m_ok);
  if (!SIGNS) {
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      const int64_t p = pb * 32 + row;
      const bool p_ok = live && p < P;
      o.v[pb][e] = load4f<VEC>(pr.V + (p_ok ? p : 0) * K + k, K - k, p_ok);
    }
  }
}

// part: float [gridDim.x][PB * 32], this workgroup's share of sum_m (X V')[m][p]^2
template <int PB, bool VEC, bool SIGNS>
__global__ __launch_bounds__(kHW * 64, 4) void hutch_k(const float* __restrict__ X, int64_t M, int64_t K,
                                                       Probes pr, int64_t P, float* __restrict__ part) {
  constexpr int CH = 4;               // pieces per chunk and lane
  constexpr int CK = 8 * CH;          // k per chunk
  __shared__ float red[kHW - 1][PB][16][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int row = lane & 31, half = lane >> 5;
  const int64_t nchunk = (K + CK - 1) / CK;
  const int64_t nblk = (M + 31) >> 5;
  // wave w takes the chunks [c_lo, c_hi): a contiguous share of k
  const int64_t per = (nchunk + kHW - 1) / kHW;
  const int64_t c_lo = wave * per;
  const int64_t c_hi = c_lo + per < nchunk ? c_lo + per : nchunk;
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

    // first element of the sign matrix this lane needs from chunk c of probe block pb (columns
    // past P get signs too; their sums are never read)
    auto sign_base = [&](int pb, int64_t c) {
      return (pr.first + (unsigned long long)(pb * 32 + row)) * (unsigned long long)K +
             (unsigned long long)(c * CK + half * (CK / 2));
    };
    // A piece's registers are refilled with the same piece of the wave's next chunk as soon as
    // the matrix steps that read them have been issued: loads run most of a chunk ahead of their
    // use without a second set of registers.
    Operands<PB, CH> o;
    unsigned bits[PB], bits_next[PB];
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) bits[pb] = SIGNS ? sign_word(pr, sign_base(pb, c_lo)) : 0u;
#pragma unroll
    for (int e = 0; e < CH; ++e)
      load_piece<PB, CH, VEC, SIGNS>(o, e, xr, m_ok, pr, P, K, c_lo * CK + half * (CK / 2), row, c_lo < c_hi);
    for (int64_t c = c_lo; c < c_hi; ++c) {
      const int64_t kn = (c + 1) * CK + half * (CK / 2);
      const bool more = c + 1 < c_hi;
#pragma unroll
      for (int pb = 0; pb < PB; ++pb) bits_next[pb] = SIGNS ? sign_word(pr, sign_base(pb, c + 1)) : 0u;
#pragma unroll
      for (int e = 0; e < CH; ++e) {
        float4 v[PB];
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
          v[pb] = SIGNS ? make_float4(sign_f(bits[pb], 4 * e), sign_f(bits[pb], 4 * e + 1), sign_f(bits[pb], 4 * e + 2),
                                      sign_f(bits[pb], 4 * e + 3))
                        : o.v[pb][e];
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.x[e].x, v[pb].x, acc[pb], 0, 0, 0);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.x[e].y, v[pb].y, acc[pb], 0, 0, 0);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.x[e].z, v[pb].z, acc[pb], 0, 0, 0);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.x[e].w, v[pb].w, acc[pb], 0, 0, 0);
        load_piece<PB, CH, VEC, SIGNS>(o, e, xr, m_ok, pr, P, K, kn, row, more);
      }
#pragma unroll
      for (int pb = 0; pb < PB; ++pb) bits[pb] = bits_next[pb];
    }

    // the k shares of the 32 x 32 products meet in wave 0, in a fixed order
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
          float d = acc[pb][v];
#pragma unroll
          for (int w = 0; w < kHW - 1; ++w) d += red[w][pb][v][lane];
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

static int probe_blocks(int64_t pg) { return pg <= 32 ? 1 : 2; }

// workgroups of one pass: a few per CU, every lane accumulating at most 256 row blocks in fp32
static int64_t hutch_grid(int64_t M, int pb) {
  const int64_t nblk = (M + 31) >> 5;
  (void)pb;
  int64_t g = (int64_t)kNumCU * 4;
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
  for (int pb = 1; pb <= 2; pb *= 2) {
    const size_t b = (size_t)hutch_grid(M, pb) * (size_t)(pb * 32) * sizeof(float);
    if (b > most) most = b;
  }
  return most;
}

// one pass per group of kProbeGroup probes; v == nullptr draws the signs in the kernel
static int run_hutchinson(const float* x, int64_t M, int64_t K, const float* v, uint64_t seed, uint64_t stream_id,
                          int64_t P, double* quad_out, float* part, hipStream_t st) {
  const bool signs = v == nullptr;
  const bool vec = aligned16(x) && (signs || aligned16(v)) && (K & 3) == 0;
  for (int64_t p0 = 0; p0 < P; p0 += kProbeGroup) {
    const int64_t pg = P - p0 < kProbeGroup ? P - p0 : kProbeGroup;
    const int pb = probe_blocks(pg);
    const unsigned g = (unsigned)hutch_grid(M, pb);
    const Probes pr = {signs ? nullptr : v + p0 * K, seed, stream_id, (unsigned long long)p0};
#define MPQ_HUTCH(PB_)                                                                                  \
  (signs ? hutch_k<PB_, true, true><<<g, kHW * 64, 0, st>>>(x, M, K, pr, pg, part)                       \
   : vec ? hutch_k<PB_, true, false><<<g, kHW * 64, 0, st>>>(x, M, K, pr, pg, part)                      \
         : hutch_k<PB_, false, false><<<g, kHW * 64, 0, st>>>(x, M, K, pr, pg, part))
    if (pb == 1) MPQ_HUTCH(1);
    else MPQ_HUTCH(2);
#undef MPQ_HUTCH
    hutch_finish<<<(unsigned)pg, kBlock, 0, st>>>(part, (int)g, pb * 32, quad_out + p0);
  }
  return launch_status();
}

static int check_hutchinson(const float* x, int64_t M, int64_t K, int64_t P, double* quad_out, void* ws,
                            size_t ws_bytes) {
  if (!x || !quad_out) return MPQ_ERR_NULL;
  if (M <= 0 || K <= 0 || P <= 0 || M >= ((int64_t)1 << 31) || P > ((int64_t)1 << 20)) return MPQ_ERR_SHAPE;
  if (mul_overflows(M, K) || mul_overflows(P, K)) return MPQ_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(x) & 3u) || (reinterpret_cast<uintptr_t>(quad_out) & 7u)) return MPQ_ERR_ALIGN;
  if (!ws || ws_bytes < mpq_hutchinson_quad_workspace_bytes(M, K, P)) return MPQ_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 3u) return MPQ_ERR_ALIGN;
  return MPQ_OK;
}

extern "C" int mpq_hutchinson_quad(const float* x, int64_t M, int64_t K, const float* v, int64_t P,
                                   double* quad_out, void* ws, size_t ws_bytes, void* stream) {
  if (!v) return MPQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(v) & 3u) return MPQ_ERR_ALIGN;
  const int rc = check_hutchinson(x, M, K, P, quad_out, ws, ws_bytes);
  if (rc != MPQ_OK) return rc;
  return run_hutchinson(x, M, K, v, 0, 0, P, quad_out, reinterpret_cast<float*>(ws), (hipStream_t)stream);
}

extern "C" int mpq_hutchinson_quad_signs(const float* x, int64_t M, int64_t K, uint64_t seed, uint64_t stream_id,
                                         int64_t P, double* quad_out, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_hutchinson(x, M, K, P, quad_out, ws, ws_bytes);
  if (rc != MPQ_OK) return rc;
  if ((K & 15) || !aligned16(x)) return MPQ_ERR_SHAPE;  // a lane's 16 signs of a chunk must sit in one Philox word
  return run_hutchinson(x, M, K, nullptr, seed, stream_id, P, quad_out, reinterpret_cast<float*>(ws),
                        (hipStream_t)stream);
}

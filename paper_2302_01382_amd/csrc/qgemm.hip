// qgemm.hip -- one quantized linear layer, the dense core of "Evaluate f(x, w)" in the paper's
// Alg. 1 / Alg. 2: acc[m][n] = sum_k A_q[m][k] * W_q[n][k] in int32 on the int8 matrix cores,
// then Y = (float(acc) * s_A) * s_W[n].
//
// Both operands are K-contiguous, which is exactly what v_mfma_i32_32x32x32_i8 wants: lane l of
// the A operand holds 16 consecutive k-bytes of row l%32 (k-half l/32), lane l of the B operand
// the same for output column l%32.  Tiles go global -> registers -> LDS (16-byte chunks, XOR
// swizzled by row so the 128-bit operand reads are bank-conflict free) -> MFMA.
//
// Packed int4 weights are expanded while staging: a nibble n becomes the byte n << 4 (= 16 n as
// int8, sign included), so the accumulator holds 16 * acc exactly and is shifted back by 4.
#include "common.hpp"

namespace mpq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 64;  // block tile; BK in bytes of k
constexpr int kGemmThreads = 256;           // 4 waves as 2 x 2, each 64 x 64 = 2 x 2 MFMA tiles

// byte offset of 16-byte chunk `ch` (0..3) of tile row `row` in a [rows][64 B] LDS tile
__device__ __forceinline__ int lds_off(int row, int ch) { return row * BK + ((ch ^ ((row >> 1) & 3)) << 4); }

// 8 nibbles of `w` (lowest nibble = lowest k) -> 8 bytes, each nibble << 4, in k order
__device__ __forceinline__ void expand8(unsigned w, unsigned& lo, unsigned& hi) {
  const unsigned e = (w << 4) & 0xF0F0F0F0u;  // nibbles 0,2,4,6
  const unsigned o = w & 0xF0F0F0F0u;         // nibbles 1,3,5,7
  lo = __builtin_amdgcn_perm(o, e, 0x05010400u);
  hi = __builtin_amdgcn_perm(o, e, 0x07030602u);
}

// ---- staging: global -> registers ------------------------------------------------------------
// A tile (and int8 W tile): 128 rows x 64 B = 512 chunks, two per thread.
struct Stage8 { v4i c[2]; };
// packed W tile: 128 rows x 32 B = 256 packed chunks, one per thread (expands to two chunks)
struct Stage4 { v4i c; };

template <bool FAST>
__device__ __forceinline__ Stage8 load8(const int8_t* __restrict__ base, int64_t nrows, int64_t K,
                                        int64_t row0, int64_t k0) {
  Stage8 s;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int cid = threadIdx.x + j * kGemmThreads;
    const int row = cid >> 2, ch = cid & 3;
    int64_t r = row0 + row;
    if (r >= nrows) r = nrows - 1;  // rows past the edge re-read the last row; never stored
    const int64_t k = k0 + ch * 16;
    const int8_t* p = base + r * K + k;
    if (FAST) {
      s.c[j] = (k < K) ? *reinterpret_cast<const v4i*>(p) : v4i{0, 0, 0, 0};
    } else {
      unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
      for (int b = 0; b < 16; ++b)
        if (k + b < K) w[b >> 2] |= (unsigned)(uint8_t)p[b] << (8 * (b & 3));
      s.c[j] = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
    }
  }
  return s;
}

__device__ __forceinline__ void store8(int8_t* lds, const Stage8& s) {
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int cid = threadIdx.x + j * kGemmThreads;
    *reinterpret_cast<v4i*>(lds + lds_off(cid >> 2, cid & 3)) = s.c[j];
  }
}

template <bool FAST>
__device__ __forceinline__ Stage4 load4(const uint8_t* __restrict__ base, int64_t nrows, int64_t K,
                                        int64_t row0, int64_t k0) {
  Stage4 s;
  const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
  int64_t r = row0 + row;
  if (r >= nrows) r = nrows - 1;
  const int64_t k = k0 + half * 32;           // first k of this packed chunk (32 values)
  const uint8_t* p = base + r * (K >> 1) + (k >> 1);
  if (FAST) {
    s.c = (k < K) ? *reinterpret_cast<const v4i*>(p) : v4i{0, 0, 0, 0};
  } else {
    unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < 16; ++b)
      if (k + 2 * b < K) w[b >> 2] |= (unsigned)p[b] << (8 * (b & 3));  // K even: pairs are whole
    s.c = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
  }
  return s;
}

__device__ __forceinline__ void store4(int8_t* lds, const Stage4& s) {
  const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
  unsigned b[8];
  expand8((unsigned)s.c.x, b[0], b[1]);
  expand8((unsigned)s.c.y, b[2], b[3]);
  expand8((unsigned)s.c.z, b[4], b[5]);
  expand8((unsigned)s.c.w, b[6], b[7]);
  *reinterpret_cast<v4i*>(lds + lds_off(row, 2 * half)) = v4i{(int)b[0], (int)b[1], (int)b[2], (int)b[3]};
  *reinterpret_cast<v4i*>(lds + lds_off(row, 2 * half + 1)) = v4i{(int)b[4], (int)b[5], (int)b[6], (int)b[7]};
}

// ---- the kernel ---------------------------------------------------------------------------------
// grid: x = N tiles (fast index, so neighbouring blocks share the A row panel), y = M tiles.
template <bool W4, bool FAST>
__global__ __launch_bounds__(kGemmThreads) void qgemm_k(const int8_t* __restrict__ A,
                                                        const void* __restrict__ Wv, int64_t M,
                                                        int64_t N, int64_t K,
                                                        const float* __restrict__ a_scale,
                                                        const float* __restrict__ w_scale,
                                                        int w_per_row, float* __restrict__ Y,
                                                        int32_t* __restrict__ ACC) {
  __shared__ __attribute__((aligned(16))) int8_t lds_a[BM * BK];
  __shared__ __attribute__((aligned(16))) int8_t lds_b[BN * BK];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t m0 = (int64_t)blockIdx.y * BM, n0 = (int64_t)blockIdx.x * BN;
  const int8_t* W8 = reinterpret_cast<const int8_t*>(Wv);
  const uint8_t* W4p = reinterpret_cast<const uint8_t*>(Wv);

  v16i acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  Stage8 ra = load8<FAST>(A, M, K, m0, 0);
  Stage8 rb8;
  Stage4 rb4;
  if (W4) rb4 = load4<FAST>(W4p, N, K, n0, 0);
  else rb8 = load8<FAST>(W8, N, K, n0, 0);

  for (int64_t k0 = 0; k0 < K; k0 += BK) {
    __syncthreads();  // previous step's LDS reads are done
    store8(lds_a, ra);
    if (W4) store4(lds_b, rb4);
    else store8(lds_b, rb8);
    __syncthreads();
    if (k0 + BK < K) {  // prefetch the next tile into registers while this one is multiplied
      ra = load8<FAST>(A, M, K, m0, k0 + BK);
      if (W4) rb4 = load4<FAST>(W4p, N, K, n0, k0 + BK);
      else rb8 = load8<FAST>(W8, N, K, n0, k0 + BK);
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int ch = 2 * s + (lane >> 5);
      v4i fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const v4i*>(lds_a + lds_off(wm * 64 + i * 32 + (lane & 31), ch));
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const v4i*>(lds_b + lds_off(wn * 64 + j * 32 + (lane & 31), ch));
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }

  // epilogue: lane holds column l%32 and rows 8*(v/4) + 4*(l/32) + v%4 of each 32x32 tile
  const float sa = Y ? a_scale[0] : 0.0f;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int64_t n = n0 + wn * 64 + j * 32 + (lane & 31);
    if (n >= N) continue;
    const float sw = Y ? w_scale[w_per_row ? n : 0] : 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t m = m0 + wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (m >= M) continue;
        int a = acc[i][j][v];
        if (W4) a >>= 4;  // exact: every product carried the factor 16
        if (ACC) ACC[m * N + n] = a;
        if (Y) Y[m * N + n] = ((float)a * sa) * sw;
      }
    }
  }
}

}  // namespace mpq

using namespace mpq;

extern "C" size_t mpq_qgemm_workspace_bytes(int64_t, int64_t, int64_t, int) { return 0; }

extern "C" int mpq_qgemm(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M,
                         int64_t N, int64_t K, const float* a_scale, const float* w_scale,
                         int w_gran, float* y_out, int32_t* acc_out, void* ws, size_t ws_bytes,
                         void* stream) {
  (void)ws;
  (void)ws_bytes;
  if (!a_q || !w_q) return MPQ_ERR_NULL;
  if (!y_out && !acc_out) return MPQ_ERR_NULL;
  if (y_out && (!a_scale || !w_scale)) return MPQ_ERR_NULL;
  if (w_storage_bits != 8 && w_storage_bits != 4) return MPQ_ERR_BITS;
  if (M <= 0 || N <= 0 || K <= 0) return MPQ_ERR_SHAPE;
  if (K > 133143) return MPQ_ERR_SHAPE;  // K * 127 * 127 must stay below 2^31
  if (w_storage_bits == 4 && (K & 1)) return MPQ_ERR_SHAPE;
  if (mul_overflows(M, N) || mul_overflows(M, K) || mul_overflows(N, K)) return MPQ_ERR_SHAPE;
  if (w_gran != MPQ_PER_TENSOR && w_gran != MPQ_PER_ROW) return MPQ_ERR_GRAN;
  if (y_out && (reinterpret_cast<uintptr_t>(y_out) & 3u)) return MPQ_ERR_ALIGN;
  if (acc_out && (reinterpret_cast<uintptr_t>(acc_out) & 3u)) return MPQ_ERR_ALIGN;
  const int64_t gx = (N + BN - 1) / BN, gy = (M + BM - 1) / BM;
  if (gx > 0x7FFFFFFF || gy > 65535) return MPQ_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid((unsigned)gx, (unsigned)gy);
  const int per_row = w_gran == MPQ_PER_ROW;
  const bool w4 = w_storage_bits == 4;
  const bool fast = aligned16(a_q) && aligned16(w_q) && (K % (w4 ? 32 : 16)) == 0;
#define MPQ_LAUNCH(W4_, FAST_) \
  qgemm_k<W4_, FAST_><<<grid, kGemmThreads, 0, st>>>(a_q, w_q, M, N, K, a_scale, w_scale, per_row, y_out, acc_out)
  if (w4) { if (fast) MPQ_LAUNCH(true, true); else MPQ_LAUNCH(true, false); }
  else { if (fast) MPQ_LAUNCH(false, true); else MPQ_LAUNCH(false, false); }
#undef MPQ_LAUNCH
  return launch_status();
}

// qgemm.hip -- one quantized linear layer, the dense core of the evaluation step in the paper's
// Alg. 1 / Alg. 2: acc[m][n] = sum_k A_q[m][k] * W_q[n][k] in int32 on the int8 matrix cores,
// then Y = (float(acc) * s_A) * s_W[n].
//
// Both operands are K-contiguous, which is exactly what v_mfma_i32_32x32x32_i8 wants: lane l of
// either operand holds 16 consecutive k-bytes of tile row l%32 (k-half l/32).
//
// Two kernels: the fast path (second half of this file; 16-byte aligned operands, K a multiple of
// 16, or 32 for packed int4) feeds a multi-stage LDS pipeline with direct global->LDS loads; the
// generic path right below stages tiles through registers with byte-wise loads and handles any
// K and alignment.  Same arithmetic, same results.
//
// Packed int4 weights are expanded on their way to the matrix core: a nibble n becomes the byte
// n << 4 (= 16 n as int8, sign included), so the accumulator holds 16 * acc exactly and is shifted
// back by 4.
#include "qgemm_dma.hpp"

namespace mpq {

__global__ void fill_u32_k(unsigned* p, unsigned v) { p[0] = v; }

constexpr int BM = 128, BN = 128, BK = 64;  // block tile; BK in bytes of k
constexpr int kGemmThreads = 256;           // 4 waves as 2 x 2, each 64 x 64 = 2 x 2 MFMA tiles

// byte offset of 16-byte chunk `ch` (0..3) of tile row `row` in a [rows][64 B] LDS tile; the XOR makes
// the 16 lanes served per clock (one chunk column of 16 rows) distinct modulo 256 B (64 banks)
__device__ __forceinline__ int lds_off(int row, int ch) { return row * BK + ((ch ^ ((row >> 2) & 3)) << 4); }

// ---- staging: global -> registers ------------------------------------------------------------
// A tile (and int8 W tile): 128 rows x 64 B = 512 chunks, two per thread.
struct Stage8 { v4i c[2]; };
// packed W tile: 128 rows x 32 B = 256 packed chunks, one per thread (expands to two chunks)
struct Stage4 { v4i c; };

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
    unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < 16; ++b)
      if (k + b < K) w[b >> 2] |= (unsigned)(uint8_t)p[b] << (8 * (b & 3));
    s.c[j] = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
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

__device__ __forceinline__ Stage4 load4(const uint8_t* __restrict__ base, int64_t nrows, int64_t K,
                                        int64_t row0, int64_t k0) {
  Stage4 s;
  const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
  int64_t r = row0 + row;
  if (r >= nrows) r = nrows - 1;
  const int64_t k = k0 + half * 32;           // first k of this packed chunk (32 values)
  const uint8_t* p = base + r * (K >> 1) + (k >> 1);
  unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
  for (int b = 0; b < 16; ++b)
    if (k + 2 * b < K) w[b >> 2] |= (unsigned)p[b] << (8 * (b & 3));  // K even: pairs are whole
  s.c = v4i{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
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
template <bool W4>
__global__ __launch_bounds__(kGemmThreads) void qgemm_k(const int8_t* __restrict__ A,
                                                        const void* __restrict__ Wv, int64_t M,
                                                        int64_t N, int64_t K,
                                                        const float* __restrict__ a_scale,
                                                        const float* __restrict__ w_scale,
                                                        int w_per_row, float* __restrict__ Y,
                                                        int32_t* __restrict__ ACC, EpiArgs epi) {
  const float* __restrict__ YREF = epi.yref;
  double* __restrict__ PART = epi.part;
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

  Stage8 ra = load8(A, M, K, m0, 0);
  Stage8 rb8;
  Stage4 rb4;
  if (W4) rb4 = load4(W4p, N, K, n0, 0);
  else rb8 = load8(W8, N, K, n0, 0);

  for (int64_t k0 = 0; k0 < K; k0 += BK) {
    __syncthreads();  // previous step's LDS reads are done
    store8(lds_a, ra);
    if (W4) store4(lds_b, rb4);
    else store8(lds_b, rb8);
    __syncthreads();
    if (k0 + BK < K) {  // prefetch the next tile into registers while this one is multiplied
      ra = load8(A, M, K, m0, k0 + BK);
      if (W4) rb4 = load4(W4p, N, K, n0, k0 + BK);
      else rb8 = load8(W8, N, K, n0, k0 + BK);
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
  const bool want_y = Y || YREF || epi.amax || epi.codes;
  const float sa = want_y ? a_scale[0] : 0.0f;
  float sse = 0.0f;  // this lane's share of sum (Y - YREF)^2
  float amax = 0.0f;
  float q_scale = 0.0f, q_inv = 0.0f, q_max = 0.0f;
  if (epi.codes) {
    bit_constants(epi.q_absmax[0], epi.q_bits, q_scale, q_inv);
    q_max = (float)((1 << (epi.q_bits - 1)) - 1);
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int64_t n = n0 + wn * 64 + j * 32 + (lane & 31);
    if (n >= N) continue;
    const float sw = want_y ? w_scale[w_per_row ? n : 0] : 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t m = m0 + wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (m >= M) continue;
        int a = acc[i][j][v];
        if (W4) a >>= 4;  // exact: every product carried the factor 16
        if (ACC) ACC[m * N + n] = a;
        const float y = apply_act(((float)a * sa) * sw, epi.act);
        amax = fmaxf(amax, fabsf(y));
        if (Y) Y[m * N + n] = y;
        if (epi.codes) epi.codes[m * N + n] = (int8_t)(int)code_f(y, q_inv, q_max);
        if (YREF) {
          const float d = y - YREF[m * N + n];
          sse = __builtin_fmaf(d, d, sse);
        }
      }
    }
  }
  if (PART) {  // one partial per workgroup, combined in a fixed order
    const float w = wave_sum(sse);
    __syncthreads();  // the tiles in LDS are not needed any more
    float* sm = reinterpret_cast<float*>(lds_a);
    if (lane == 0) sm[wave] = w;
    __syncthreads();
    if (threadIdx.x == 0)
      PART[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = ((double)sm[0] + (double)sm[1]) + ((double)sm[2] + (double)sm[3]);
  }
  if (epi.amax) {
    const float w = wave_max(amax);
    if (lane == 0) atomicMax(epi.amax, abs_key(w));
  }
}

// sum of `count` per-workgroup partials, one workgroup, fixed order
__global__ __launch_bounds__(kBlock) void sum_partials_k(const double* __restrict__ part, int64_t count,
                                                         double* __restrict__ out) {
  __shared__ double sm[kBlock];
  double a = 0.0;
  for (int64_t i = threadIdx.x; i < count; i += kBlock) a += part[i];
  sm[threadIdx.x] = a;
  __syncthreads();
  for (int h = kBlock / 2; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h) sm[threadIdx.x] += sm[threadIdx.x + h];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = sm[0];
}


// ---- split along k ----------------------------------------------------------------------------------
// A GEMM with a handful of output tiles and a long k (any layer at inference batch 1: 49 x 4608 x 512
// is 8 tiles of 64 x 64) leaves most of the chip idle.  With a workspace the caller lets the library
// cut k into `split` ranges: every (tile, range) pair is a workgroup that writes its raw int32
// accumulators to a plane of the workspace, and one elementwise kernel adds the planes (integer
// sums: exact in any order, so the accumulators stay bit-identical to the unsplit product) and
// applies the epilogue Y = (float(acc) * s_A) * s_W[n].
// Measured on the chip: the second kernel and the planes cost about 5 us, so the split pays only
// where the unsplit grid is tiny -- 49 x 4608 x 512 takes 13.0 us unsplit and 9.1 us in 12 ranges,
// whereas 1568 x 4608 x 512 (200 tiles of 64 x 64: 17 us) and 6272 x 2304 x 256 (14.6 us) lose 5-9 us
// with any split of either tile size, and stay unsplit.
struct SplitPlan {
  int split = 1;
  int k_per_split = 0;
};

static SplitPlan plan_split(int64_t M, int64_t N, int64_t K) {
  SplitPlan p;
  const int64_t base = ((M + 63) / 64) * ((N + 63) / 64);  // tiles of 64 x 64
  if (K < 1024 || base > kNumCU / 4) return p;
  const int64_t kt = (K + 127) / 128;               // k tiles of 128 bytes
  int64_t want = (kNumCU + base - 1) / base;        // about one workgroup per CU
  if (want > 16) want = 16;
  if (want > kt / 2) want = kt / 2;                 // at least two k tiles per range
  if (want < 2) return p;
  const int64_t per = (kt + want - 1) / want;       // k tiles per range
  p.k_per_split = (int)(per * 128);
  p.split = (int)((kt + per - 1) / per);            // no empty range
  if (p.split < 2) return SplitPlan{};
  return p;
}

// acc = sum of `split` planes; ACC and / or Y from it.  VEC: four consecutive n per thread.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void splitk_reduce(const int32_t* __restrict__ planes, int split, int64_t MN,
                                                        int64_t N, const float* __restrict__ a_scale,
                                                        const float* __restrict__ w_scale, int w_per_row,
                                                        float* __restrict__ Y, int32_t* __restrict__ ACC) {
  const int64_t i = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * (VEC ? 4 : 1);
  if (i >= MN) return;
  const float sa = Y ? a_scale[0] : 0.0f;
  if (VEC) {
    v4i a = *reinterpret_cast<const v4i*>(planes + i);
    for (int s = 1; s < split; ++s) {
      const v4i b = *reinterpret_cast<const v4i*>(planes + (int64_t)s * MN + i);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    if (ACC) *reinterpret_cast<v4i*>(ACC + i) = a;
    if (Y) {
      const int64_t n = i % N;  // N % 4 == 0: the four share a row
      float4 sw;
      if (w_per_row) sw = *reinterpret_cast<const float4*>(w_scale + n);
      else sw = make_float4(w_scale[0], w_scale[0], w_scale[0], w_scale[0]);
      *reinterpret_cast<float4*>(Y + i) = make_float4(((float)a.x * sa) * sw.x, ((float)a.y * sa) * sw.y,
                                                      ((float)a.z * sa) * sw.z, ((float)a.w * sa) * sw.w);
    }
  } else {
    int a = planes[i];
    for (int s = 1; s < split; ++s) a += planes[(int64_t)s * MN + i];
    if (ACC) ACC[i] = a;
    if (Y) Y[i] = ((float)a * sa) * w_scale[w_per_row ? i % N : 0];
  }
}

// Everything about the arguments of a quantized layer that can be wrong, checked on the host
// before anything is enqueued (a failing call leaves the device untouched).
static int check_qgemm_args(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N, int64_t K,
                            const float* a_scale, const float* w_scale, int w_gran, const float* y_out,
                            const int32_t* acc_out, const EpiArgs& epi) {
  const float* y_ref = epi.yref;
  if (!a_q || !w_q) return MPQ_ERR_NULL;
  if (!y_out && !acc_out && !y_ref && !epi.amax && !epi.codes) return MPQ_ERR_NULL;
  if ((y_out || y_ref || epi.amax || epi.codes) && (!a_scale || !w_scale)) return MPQ_ERR_NULL;
  if (w_storage_bits != 8 && w_storage_bits != 4) return MPQ_ERR_BITS;
  if (M <= 0 || N <= 0 || K <= 0) return MPQ_ERR_SHAPE;
  if (K > 133143) return MPQ_ERR_SHAPE;  // K * 127 * 127 must stay below 2^31
  if (w_storage_bits == 4 && (K & 1)) return MPQ_ERR_SHAPE;
  if (mul_overflows(M, N) || mul_overflows(M, K) || mul_overflows(N, K)) return MPQ_ERR_SHAPE;
  if (w_gran != MPQ_PER_TENSOR && w_gran != MPQ_PER_ROW) return MPQ_ERR_GRAN;
  if (y_out && (reinterpret_cast<uintptr_t>(y_out) & 3u)) return MPQ_ERR_ALIGN;
  if (y_ref && (reinterpret_cast<uintptr_t>(y_ref) & 3u)) return MPQ_ERR_ALIGN;
  if (acc_out && (reinterpret_cast<uintptr_t>(acc_out) & 3u)) return MPQ_ERR_ALIGN;
  const int64_t gx = (N + BN - 1) / BN, gy = (M + BM - 1) / BM;
  if (gx > 0x7FFFFFFF || gy > 65535) return MPQ_ERR_SHAPE;           // grid of the generic kernel
  if (((M + 63) / 64) * ((N + 63) / 64) > 0x7FFFFFFF) return MPQ_ERR_SHAPE;  // ... and of the smallest fast tile
  return MPQ_OK;
}

static bool fast_path(const int8_t* a_q, const void* w_q, bool w4, int64_t M, int64_t N, int64_t K) {
  // the fast kernels index rows with 32 bits
  return aligned16(a_q) && aligned16(w_q) && (K % (w4 ? 32 : 16)) == 0 && M < (1ll << 31) && N < (1ll << 31);
}

// Dispatch shared by every quantized-layer call; the arguments have passed check_qgemm_args.  With
// y_ref the kernels also leave one partial sum of (Y - y_ref)^2 per workgroup in epi.part and
// report how many.  ws / ws_bytes: optional scratch for the split along k (plain epilogue only).
static int run_qgemm(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
                     int64_t K, const float* a_scale, const float* w_scale, int w_gran, float* y_out,
                     int32_t* acc_out, EpiArgs epi, int64_t* n_partials, hipStream_t st, void* ws = nullptr,
                     size_t ws_bytes = 0) {
  const int per_row = w_gran == MPQ_PER_ROW;
  const bool w4 = w_storage_bits == 4;
  const int64_t gx = (N + BN - 1) / BN, gy = (M + BM - 1) / BM;
  if (fast_path(a_q, w_q, w4, M, N, K)) {
    DmaArgs d{a_q, w_q, M, N, K, a_scale, w_scale, per_row, y_out, acc_out, st, epi, n_partials, 1, 0, false};
    const bool plain = !epi.yref && !epi.codes && !epi.act && !epi.amax;
    const SplitPlan sp = plain ? plan_split(M, N, K) : SplitPlan{};
    if (sp.split > 1 && ws && aligned16(ws) && ws_bytes >= (size_t)sp.split * (size_t)(M * N) * sizeof(int32_t)) {
      int32_t* planes = reinterpret_cast<int32_t*>(ws);
      d.y_out = nullptr;
      d.acc_out = planes;
      d.split = sp.split;
      d.k_per_split = sp.k_per_split;
      const int rc = launch_dma_64(w4, false, d);
      if (rc != MPQ_OK) return rc;
      const int64_t MN = M * N;
      const bool vec = (N & 3) == 0 && (!y_out || aligned16(y_out)) && (!acc_out || aligned16(acc_out)) &&
                       (!(y_out && per_row) || aligned16(w_scale));
      const int64_t threads = vec ? MN / 4 : MN;
      const unsigned blocks = (unsigned)((threads + kBlock - 1) / kBlock);
      if (vec) splitk_reduce<true><<<blocks, kBlock, 0, st>>>(planes, sp.split, MN, N, a_scale, w_scale, per_row, y_out, acc_out);
      else splitk_reduce<false><<<blocks, kBlock, 0, st>>>(planes, sp.split, MN, N, a_scale, w_scale, per_row, y_out, acc_out);
      return launch_status();
    }
    // tile choice (from sweeps over the configured shapes): 256 x 256 when that gives at least
    // three CUs in four a tile; else 192 x 192 (six waves) when it covers the problem in exactly
    // one round with at least three CUs in four busy and next to no padding (the BERT-base
    // widths: 768 = 4 x 192 gives 12288 x 768 exactly 256 tiles where 256 x 256 gives 144);
    // else 128 x 128 when it gives at least half of the CUs a tile, else 64 x 64.
    // 128 x 128 runs three stages (one workgroup per CU) when there is at most one tile per CU
    // anyway or k is long, two stages (two workgroups per CU) otherwise.
    auto tiles = [&](int64_t bm, int64_t bn) { return ((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    const int64_t t192 = tiles(192, 192);
    if (N > 128 && tiles(256, 256) >= kNumCU * 3 / 4) return launch_dma_256(w4, d);
    if (N % 192 == 0 && t192 <= kNumCU && t192 >= kNumCU * 3 / 4 && t192 * 192 * 192 <= M * N + M * N / 32)
      return launch_dma_192(w4, K >= 1024, d);
    if (N > 64 && tiles(128, 128) >= kNumCU / 2) return launch_dma_128(w4, K >= 2048 || tiles(128, 128) <= kNumCU, d);
    // k tiles of 256 bytes where the grid is at most one workgroup per CU anyway (the longer stages
    // leave room for one workgroup per CU only) and k is long enough to have several of them
    return launch_dma_64(w4, K >= 1024 && tiles(64, 64) <= kNumCU, d);
  }
  const dim3 grid((unsigned)gx, (unsigned)gy);
  if (w4) qgemm_k<true><<<grid, kGemmThreads, 0, st>>>(a_q, w_q, M, N, K, a_scale, w_scale, per_row, y_out, acc_out, epi);
  else qgemm_k<false><<<grid, kGemmThreads, 0, st>>>(a_q, w_q, M, N, K, a_scale, w_scale, per_row, y_out, acc_out, epi);
  if (n_partials) *n_partials = gx * gy;
  return launch_status();
}

// partials never outnumber the 64 x 64 tiles (the smallest tile any kernel here uses)
static int64_t max_partials(int64_t M, int64_t N) { return ((M + 63) / 64) * ((N + 63) / 64); }

}  // namespace mpq

using namespace mpq;

extern "C" int mpq_init(void) {
  const DmaArgs d{nullptr, nullptr, 0, 0, 0, nullptr, nullptr, 0, nullptr, nullptr, nullptr, kNoEpi, nullptr, 1, 0, true};
  for (int w4 = 0; w4 < 2; ++w4) {
    int rc = launch_dma_256(w4 != 0, d);
    if (rc == MPQ_OK) rc = launch_dma_192(w4 != 0, true, d);
    if (rc == MPQ_OK) rc = launch_dma_192(w4 != 0, false, d);
    if (rc == MPQ_OK) rc = launch_dma_128(w4 != 0, true, d);
    if (rc == MPQ_OK) rc = launch_dma_128(w4 != 0, false, d);
    if (rc == MPQ_OK) rc = launch_dma_64(w4 != 0, false, d);
    if (rc == MPQ_OK) rc = launch_dma_64(w4 != 0, true, d);
    if (rc != MPQ_OK) return rc;
  }
  return MPQ_OK;
}

extern "C" size_t mpq_qgemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int w_storage_bits) {
  if (M <= 0 || N <= 0 || K <= 0 || K > 133143 || (w_storage_bits != 8 && w_storage_bits != 4)) return 0;
  if (mul_overflows(M, N) || mul_overflows(M, K) || mul_overflows(N, K)) return 0;
  const SplitPlan sp = plan_split(M, N, K);
  return sp.split > 1 ? (size_t)sp.split * (size_t)(M * N) * sizeof(int32_t) : 0;
}

extern "C" int mpq_qgemm(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M,
                         int64_t N, int64_t K, const float* a_scale, const float* w_scale,
                         int w_gran, float* y_out, int32_t* acc_out, void* ws, size_t ws_bytes,
                         void* stream) {
  if (!y_out && !acc_out) return MPQ_ERR_NULL;
  const int rc = check_qgemm_args(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, y_out, acc_out, kNoEpi);
  if (rc != MPQ_OK) return rc;
  return run_qgemm(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, y_out, acc_out,
                   kNoEpi, nullptr, (hipStream_t)stream, ws, ws_bytes);
}

// shared by mpq_qgemm_act and mpq_stack_evaluate (which checks all its layers before its first launch)
namespace mpq {
int check_qgemm_act_args(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N, int64_t K,
                         const float* a_scale, const float* w_scale, int w_gran, int act, const float* y_out,
                         const float* absmax_out) {
  if (!y_out && !absmax_out) return MPQ_ERR_NULL;
  if (act < MPQ_ACT_NONE || act > MPQ_ACT_GELU) return MPQ_ERR_SHAPE;
  if (absmax_out && (reinterpret_cast<uintptr_t>(absmax_out) & 3u)) return MPQ_ERR_ALIGN;
  const EpiArgs epi{nullptr, nullptr, act, reinterpret_cast<unsigned*>(const_cast<float*>(absmax_out)), nullptr, 0, nullptr};
  return check_qgemm_args(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, y_out, nullptr, epi);
}
int check_qgemm_score_args(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N, int64_t K,
                           const float* a_scale, const float* w_scale, int w_gran, const float* y_ref,
                           const double* sse_out, const float* y_out, const void* ws, size_t ws_bytes) {
  if (!y_ref || !sse_out) return MPQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(sse_out) & 7u) return MPQ_ERR_ALIGN;
  if (M <= 0 || N <= 0 || mul_overflows(M, N)) return MPQ_ERR_SHAPE;
  if (!ws || ws_bytes < (size_t)max_partials(M, N) * sizeof(double)) return MPQ_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 7u) return MPQ_ERR_ALIGN;
  const EpiArgs epi{y_ref, nullptr, 0, nullptr, nullptr, 0, nullptr};
  return check_qgemm_args(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, y_out, nullptr, epi);
}
}  // namespace mpq

extern "C" int mpq_qgemm_act(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
                             int64_t K, const float* a_scale, const float* w_scale, int w_gran, int act,
                             float* y_out, float* absmax_out, int accumulate, void* stream) {
  // every check comes before the fill: a failing call leaves the device untouched
  const int rc = check_qgemm_act_args(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, act, y_out, absmax_out);
  if (rc != MPQ_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  unsigned* amax = reinterpret_cast<unsigned*>(absmax_out);
  if (amax && !accumulate) fill_u32_k<<<1, 1, 0, st>>>(amax, 0u);
  return run_qgemm(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, y_out, nullptr,
                   EpiArgs{nullptr, nullptr, act, amax, nullptr, 0, nullptr}, nullptr, st);
}

extern "C" int mpq_qgemm_act_codes(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
                                   int64_t K, const float* a_scale, const float* w_scale, int w_gran, int act,
                                   const float* absmax, int bits, int8_t* codes_out, void* stream) {
  if (!absmax || !codes_out) return MPQ_ERR_NULL;
  if (act < MPQ_ACT_NONE || act > MPQ_ACT_GELU) return MPQ_ERR_SHAPE;
  if (bits < 2 || bits > 8) return MPQ_ERR_BITS;
  if (reinterpret_cast<uintptr_t>(absmax) & 3u) return MPQ_ERR_ALIGN;
  const EpiArgs epi{nullptr, nullptr, act, nullptr, absmax, bits, codes_out};
  const int rc = check_qgemm_args(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, nullptr, nullptr, epi);
  if (rc != MPQ_OK) return rc;
  return run_qgemm(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, nullptr, nullptr, epi, nullptr,
                   (hipStream_t)stream);
}

extern "C" size_t mpq_qgemm_score_workspace_bytes(int64_t M, int64_t N, int64_t K, int w_storage_bits) {
  (void)w_storage_bits;
  if (M <= 0 || N <= 0 || K <= 0 || mul_overflows(M, N)) return 0;
  return (size_t)max_partials(M, N) * sizeof(double);
}

extern "C" int mpq_qgemm_score(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M,
                               int64_t N, int64_t K, const float* a_scale, const float* w_scale,
                               int w_gran, const float* y_ref, double* sse_out, float* y_out, void* ws,
                               size_t ws_bytes, void* stream) {
  int rc = check_qgemm_score_args(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, y_ref, sse_out, y_out, ws,
                                  ws_bytes);
  if (rc != MPQ_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  double* partials = reinterpret_cast<double*>(ws);
  int64_t count = 0;
  rc = run_qgemm(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, y_out, nullptr,
                 EpiArgs{y_ref, partials, 0, nullptr, nullptr, 0, nullptr}, &count, st);
  if (rc != MPQ_OK) return rc;
  sum_partials_k<<<1, kBlock, 0, st>>>(partials, count, sse_out);
  return launch_status();
}

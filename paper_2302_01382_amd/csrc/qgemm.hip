// qgemm.hip -- one quantized linear layer, the dense core of "Evaluate f(x, w)" in the paper's
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
#include "common.hpp"

#include <type_traits>

namespace mpq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// What an epilogue may do beyond Y = (float(acc) * s_A) * s_W[n]:
//  - score: accumulate sum (Y - yref)^2, one double partial per workgroup in `part`;
//  - activation: Y <- act(Y) before it is stored (1 = ReLU, 2 = GELU), and the largest |Y| after
//    the activation merged into amax[0] (an integer atomic max over the bit patterns of the
//    non-negative floats: exact and independent of the order);
//  - codes: the activated output quantized on the spot (Eq. 1 with the absmax in q_absmax[0], which
//    an earlier pass over the same product found) and stored as int8 codes, so that the fp32 layer
//    output never travels to HBM and back on its way into the next layer's GEMM.
struct EpiArgs {
  const float* yref;
  double* part;
  int act;
  unsigned* amax;
  const float* q_absmax;
  int q_bits;
  int8_t* codes;
};
constexpr EpiArgs kNoEpi = {nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr};

// GELU(y) = y Phi(y).  The epilogue's arithmetic is not hidden behind anything (every wave of the
// workgroup is in its epilogue at the same time), so Phi is evaluated in about twenty lane
// operations instead of the library erf's fifty: with t = |y|,
//   Phi(-t) = 1/2 erfc(t / sqrt 2) = exp(-t^2 / 2) P(u),  u = 1 / (1 + 0.28 t),
// P a degree-6 polynomial fitted (minimax in the relative error, 4e-7 on 0 <= t <= 6) to
// 1/2 erfcx(t / sqrt 2), and Phi(t) = 1 - Phi(-t).  The form keeps the RELATIVE accuracy in the
// negative tail, where 1 + erf would cancel: in fp32 the result is within 2e-6 relative of the
// exact GELU for y >= -6 (the rounding of t^2 in the exponent dominates) and within 4e-7 |y|
// absolute everywhere (beyond y = -6 GELU itself is below 1e-9 |y|).
__device__ __forceinline__ float gelu_f(float y) {
  const float t = fabsf(y);
  const float u = __builtin_amdgcn_rcpf(__builtin_fmaf(t, 0.28f, 1.0f));
  float p = -0.11208509653806686f;
  p = __builtin_fmaf(p, u, 0.41932520270347595f);
  p = __builtin_fmaf(p, u, -0.29365190863609314f);
  p = __builtin_fmaf(p, u, 0.32605481147766113f);
  p = __builtin_fmaf(p, u, 0.035669293254613876f);
  p = __builtin_fmaf(p, u, 0.12578752636909485f);
  p = __builtin_fmaf(p, u, -0.0010996352648362517f);
  const float tail = __builtin_amdgcn_exp2f((t * t) * -0.72134752044448170f) * p;  // exp(-t^2/2) P(u)
  return y * (y < 0.0f ? tail : 1.0f - tail);
}

__device__ __forceinline__ float apply_act(float y, int act) {
  if (act == 1) return fmaxf(y, 0.0f);
  if (act == 2) return gelu_f(y);
  return y;
}

__global__ void fill_u32_k(unsigned* p, unsigned v) { p[0] = v; }

constexpr int BM = 128, BN = 128, BK = 64;  // block tile; BK in bytes of k
constexpr int kGemmThreads = 256;           // 4 waves as 2 x 2, each 64 x 64 = 2 x 2 MFMA tiles

// byte offset of 16-byte chunk `ch` (0..3) of tile row `row` in a [rows][64 B] LDS tile; the XOR makes
// the 16 lanes served per clock (one chunk column of 16 rows) distinct modulo 256 B (64 banks)
__device__ __forceinline__ int lds_off(int row, int ch) { return row * BK + ((ch ^ ((row >> 2) & 3)) << 4); }

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


// =====================================================================================================
// Fast path: multi-stage LDS pipeline fed by direct global->LDS loads (no register staging).
//
// k is walked in tiles of 128 bytes.  One wave-wide global_load_lds_dwordx4 moves 64 x 16 B = 1 KiB
// and the hardware puts lane l's 16 bytes at LDS base + 16 l, so an instruction fills 8 whole tile
// rows (16 rows of a packed-int4 tile).  To get a bank-conflict-free layout anyway, the *global*
// chunk a lane fetches is permuted: LDS slot s of row r holds logical chunk s ^ ((r >> 1) & 7)
// (int8 tiles, 8 chunks per row) or s ^ ((r >> 2) & 3) (packed tiles, 4 chunks per row).  The LDS
// of gfx950 has 64 banks (256 B per clock, measured): a 128-bit operand read is served 16 lanes
// per clock, those lanes read one chunk column of 16 consecutive rows, and with this XOR their
// 16 addresses are distinct modulo 256 B.  The MFMA operand reads apply the same XOR.  Chunks
// beyond K are fetched from a 16-byte block of zeros.
//
// A k tile is requested NSTAGE - 1 tiles ahead of the MFMAs that use it; a wave waits only for
// its own share of the tile it needs next (s_waitcnt vmcnt) and then meets the others at the one
// barrier per k tile.  The k loop is unrolled by NSTAGE so every LDS address is a compile-time
// offset (the compiler then keeps ds_reads of one stage independent of the loads in flight into
// the others).
//
// What bounds this path (microbenchmarks on the same chip): a CU fills its LDS from L2 at about
// 90 GB/s (one 1 KiB wave-load per ~27 clocks through its one address unit), so the 64 KiB k tile
// of a 256 x 256 workgroup takes ~0.75 us to arrive against ~0.85-1.0 us of MFMA work on it;
// and because a wave issues in order, a wave queueing at the address unit feeds no MFMAs -- a
// plain stream of MFMAs with wave-loads between them, no waits and no barrier at all, reaches
// about 70 % of the pure MFMA rate, which itself is ~82 % of the nominal peak under this load.
// =====================================================================================================
#define MPQ_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define MPQ_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

__device__ __attribute__((aligned(16))) int g_zero16[4];  // never written: zero fill for k tails


// The direct-to-LDS load and its wait are written as inline assembly on purpose: when the
// compiler sees the load it cannot tell which LDS bytes are in flight once more than a handful of
// them are outstanding, and puts a full "s_waitcnt vmcnt(0)" in front of every LDS read -- which
// would serialise the pipeline.  Written this way the compiler does not track them, and the
// kernel does the bookkeeping itself: loads return in order, so "vmcnt(n)" means all but the
// youngest n wave-loads of this wave have landed.
// lds_byte_off must be wave-uniform (it travels in M0); lane l's 16 bytes land at +16 l.
__device__ __forceinline__ void dma16(const char* src, unsigned lds_byte_off) {
  // s_nop: the one wait state the ISA asks for between a write of M0 and an LDS-DMA that reads it
  // (the compiler's hazard pass does not look inside inline assembly)
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_byte_off) : "memory");
}
template <int N_>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_) : "memory");
}

// KB: k bytes per stage (128 or 64)
template <int BM, int BN, int WM, int WN, int NSTAGE, bool W4, int KB>
struct DmaCfg {
  static constexpr int DBK = KB;
  static constexpr int CPR = KB / 16;                 // 16-byte chunks per int8 tile row (8 | 4)
  static constexpr int RPI = 64 / CPR;                // tile rows one wave-load covers (8 | 16)
  static constexpr int SH = CPR == 8 ? 1 : 2;         // swizzle: slot = chunk ^ ((row >> SH) & (CPR-1))
  static constexpr int PCPR = KB / 32;                // 16-byte chunks per packed-int4 tile row (4 | 2)
  static constexpr int PRPI = 64 / PCPR;              // packed rows per wave-load (16 | 32)
  static constexpr int PSH = PCPR == 4 ? 2 : 3;
  static constexpr int NW = WM * WN;
  static constexpr int NT = NW * 64;
  static constexpr int TM = BM / WM, TN = BN / WN;   // per-wave tile
  static constexpr int FM = TM / 32, FN = TN / 32;   // 32x32 MFMA tiles per wave
  static constexpr int A_STAGE = BM * DBK;
  static constexpr int B_ROW = W4 ? DBK / 2 : DBK;   // bytes of one W tile row in LDS
  static constexpr int B_STAGE = BN * B_ROW;
  static constexpr int STAGE = A_STAGE + B_STAGE;
  static constexpr int SCALE_OFF = NSTAGE * STAGE;    // two 1 KiB buffers of per-channel W scales
  static constexpr int LDS_BYTES = SCALE_OFF + 2048;
  static constexpr int NLA = BM / RPI;                // wave-loads per A stage
  static constexpr int NLB = W4 ? BN / PRPI : BN / RPI;  // wave-loads per W stage
  static constexpr int LPW = (NLA + NLB) / NW;        // wave-loads per wave per stage
  static_assert(NLA % NW == 0 && NLB % NW == 0, "loads must divide evenly over the waves");
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile is a multiple of 32 x 32");
  static_assert(KB == 128 || KB == 64, "k tile of 128 or 64 bytes");
  static_assert((NSTAGE - 1) * LPW < 64, "vmcnt is a 6-bit counter");
};

// compile-time loop: f(std::integral_constant<int, I>) for I = FIRST .. LAST - 1
template <int FIRST, int LAST, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (FIRST < LAST) {
    f(std::integral_constant<int, FIRST>{});
    static_for<FIRST + 1, LAST>(f);
  }
}

// What one wave fetches per stage.  Wave-load t of a wave covers tile rows first + t * STEP ..., and
// because STEP is a multiple of the swizzle period every one of them has the lane fetch the same
// logical chunk, so the plan is four registers: the lane's first row and chunk offset per operand.
// Source addresses are formed at issue time (one 64-bit multiply-add per wave-load).
template <class C, bool W4>
struct DmaPlan {
  static constexpr int NA = C::NLA / C::NW, NB_ = C::NLB / C::NW;
  static constexpr int STEP_A = C::RPI * C::NW;
  static constexpr int STEP_B = (W4 ? C::PRPI : C::RPI) * C::NW;
  static_assert(((STEP_A >> C::SH) % C::CPR) == 0, "A swizzle must repeat from one wave-load to the next");
  static_assert(W4 ? ((STEP_B >> C::PSH) % C::PCPR) == 0 : ((STEP_B >> C::SH) % C::CPR) == 0,
                "W swizzle must repeat from one wave-load to the next");
  const char* A;
  const char* W;
  unsigned last_a, last_b;  // M - 1, N - 1: rows past the edge re-read the last row; never stored
  unsigned K;
  unsigned ra, rb;          // the lane's row of its first wave-load (global index)
  int ka, kb;               // k of the lane's chunk within the tile (bytes of A / values of W)
  unsigned wave_off;        // LDS offset of this wave's first wave-load within a stage region

  __device__ __forceinline__ void init(const int8_t* __restrict__ A_, const uint8_t* __restrict__ W_,
                                       int64_t M, int64_t N, int64_t K_, int64_t m0, int64_t n0,
                                       int wave_u, int lane) {
    A = reinterpret_cast<const char*>(A_);
    W = reinterpret_cast<const char*>(W_);
    last_a = (unsigned)(M - 1);
    last_b = (unsigned)(N - 1);
    K = (unsigned)K_;
    wave_off = (unsigned)wave_u * 1024u;
    {
      const int row = C::RPI * wave_u + lane / C::CPR;
      ka = ((lane % C::CPR) ^ ((row >> C::SH) & (C::CPR - 1))) * 16;  // logical chunk this lane fetches
      ra = (unsigned)m0 + (unsigned)row;
    }
    if (!W4) {
      const int row = C::RPI * wave_u + lane / C::CPR;
      kb = ((lane % C::CPR) ^ ((row >> C::SH) & (C::CPR - 1))) * 16;
      rb = (unsigned)n0 + (unsigned)row;
    } else {  // packed tile: a wave-load covers PRPI rows of KB/2 packed bytes; a chunk is 32 values
      const int row = C::PRPI * wave_u + lane / C::PCPR;
      kb = ((lane % C::PCPR) ^ ((row >> C::PSH) & (C::PCPR - 1))) * 32;
      rb = (unsigned)n0 + (unsigned)row;
    }
  }

  // One k tile's requests of this wave, numbered 0 .. NA + NB_ - 1 (A first); chunks at or beyond
  // k_limit are fetched from a block of zeros.
  struct Tile {
    const char* a0;
    const char* b0;
    bool va, vb;
  };
  __device__ __forceinline__ Tile tile(int k0, int k_limit) const {
    Tile t;
    t.va = k0 + ka < k_limit;
    t.vb = k0 + kb < k_limit;
    t.a0 = A + (unsigned)(k0 + ka);
    t.b0 = W + (unsigned)(W4 ? (k0 + kb) >> 1 : k0 + kb);
    return t;
  }
  template <int R>
  __device__ __forceinline__ void request(const Tile& tl, unsigned lds_stage_off) const {
    const char* zero = reinterpret_cast<const char*>(g_zero16);
    if constexpr (R < NA) {
      unsigned r = ra + (unsigned)(R * STEP_A);
      r = r < last_a ? r : last_a;
      const char* src = tl.va ? tl.a0 + (uint64_t)r * K : zero;
      dma16(src, lds_stage_off + wave_off + (unsigned)(R * C::NW) * 1024u);
    } else {
      constexpr int T = R - NA;
      const unsigned ldb = W4 ? K >> 1 : K;
      unsigned r = rb + (unsigned)(T * STEP_B);
      r = r < last_b ? r : last_b;
      const char* src = tl.vb ? tl.b0 + (uint64_t)r * ldb : zero;
      dma16(src, lds_stage_off + (unsigned)C::A_STAGE + wave_off + (unsigned)(T * C::NW) * 1024u);
    }
  }
  // all requests of the k tile starting at k0, back to back
  __device__ __forceinline__ void issue(unsigned lds_stage_off, int k0, int k_limit) const {
    const Tile tl = tile(k0, k_limit);
    static_for<0, NA + NB_>([&](auto r_) { request<decltype(r_)::value>(tl, lds_stage_off); });
  }
};

// LDS offsets (within a stage) of the first operand fragments of a lane, for k substep 0.  With
// the XOR swizzle the offset for substep s is this value with s XORed into its chunk bits, and
// rows 32 i further down add a multiple of the row pitch, which never reaches those bits.
template <class C, bool W4>
struct FragBase {
  unsigned a, b;
  __device__ __forceinline__ void init(int wm, int wn, int lane) {
    const int l31 = lane & 31, g = lane >> 5;
    const int ra = wm * C::TM + l31;
    a = (unsigned)(ra * C::DBK + ((g ^ ((ra >> C::SH) & (C::CPR - 1))) << 4));
    const int rb = wn * C::TN + l31;
    if (!W4) b = (unsigned)(C::A_STAGE + rb * C::DBK + ((g ^ ((rb >> C::SH) & (C::CPR - 1))) << 4));
    else b = (unsigned)(C::A_STAGE + rb * (C::DBK / 2) + (((rb >> C::PSH) & (C::PCPR - 1)) << 4) + g * 8);
  }
};

// base ^ bits, computed where it is used: written as a plain expression the compiler would keep
// one address register per (stage, substep, operand) alive across the whole k loop
template <unsigned BITS>
__device__ __forceinline__ unsigned xor_here(unsigned base) {
  if (BITS == 0) return base;
  unsigned r;
  asm volatile("v_xor_b32 %0, %1, %2" : "=v"(r) : "n"(BITS), "v"(base));
  return r;
}

// W fragment as it sits in LDS: the MFMA operand itself, or 16 packed nibbles that are expanded
// right before use (kept packed meanwhile: half the registers, and the expansion then never waits
// for a read issued a moment ago).
template <bool W4>
struct BRaw { v4i v; };
template <>
struct BRaw<true> { uint2 v; };
__device__ __forceinline__ v4i b_operand(const BRaw<false>& r) { return r.v; }
__device__ __forceinline__ v4i b_operand(const BRaw<true>& r) {
  unsigned b0, b1, b2, b3;
  expand8(r.v.x, b0, b1);
  expand8(r.v.y, b2, b3);
  return v4i{(int)b0, (int)b1, (int)b2, (int)b3};
}

// A fragments of k-substep S (32 k-values) of the stage at byte offset stage_off
template <class C, bool W4, int S>
__device__ __forceinline__ void load_a_frags(const char* lds, unsigned stage_off, const FragBase<C, W4>& fr,
                                             v4i (&fa)[C::FM]) {
  // logical chunk 2 S + g of an int8 row
  const char* pa = lds + xor_here<(unsigned)(S << 5)>(fr.a + stage_off);
#pragma unroll
  for (int i = 0; i < C::FM; ++i) fa[i] = *reinterpret_cast<const v4i*>(pa + i * 32 * C::DBK);
}
// LDS address of the lane's W fragments of k-substep S (packed rows hold 32 values per chunk:
// chunk S, half g)
template <class C, bool W4, int S>
__device__ __forceinline__ const char* b_frag_ptr(const char* lds, unsigned stage_off, const FragBase<C, W4>& fr) {
  return lds + xor_here<(unsigned)(W4 ? S << 4 : S << 5)>(fr.b + stage_off);
}
template <class C, bool W4>
__device__ __forceinline__ void load_b_frag(const char* pb, int j, BRaw<W4>& fb) {
  if constexpr (!W4) fb.v = *reinterpret_cast<const v4i*>(pb + j * 32 * C::DBK);
  else fb.v = *reinterpret_cast<const uint2*>(pb + j * 32 * (C::DBK / 2));
}

// One k substep.  The operand reads of the FOLLOWING substep (S_NEXT of the stage at next_off) are
// dealt in between the MFMAs: its A fragments first, into the other half of a double buffer; its
// W fragment j into the registers of this substep's W fragment j as soon as the MFMAs that use
// that one have been issued.  Every fragment is thus requested several MFMAs before its first
// use, with 32 instead of 48 registers of fragments.  Left to itself the scheduler sinks every
// read down to its first use, and a substep then starts by waiting out the LDS latency, hence
// the pinning.
// `request(r)` issues the wave's r-th global->LDS request of a k tile; NR of them are dealt out
// over the substep (NR = 0: none).  A wave that issues its requests back to back sits in the
// queue of the CU's one address unit (a 64 KiB k tile keeps it busy for about a thousand clocks)
// and, issuing in order, feeds no MFMAs meanwhile.
template <class C, bool W4, int S_NEXT, int NR, class Request>
__device__ __forceinline__ void k_substep(v16i (&acc)[C::FM][C::FN], const v4i (&fa)[C::FM],
                                          v4i (&fa_next)[C::FM], BRaw<W4> (&fb)[C::FN], const char* lds,
                                          unsigned next_off, const FragBase<C, W4>& fr, Request&& request) {
  constexpr int NM = C::FM * C::FN;
  load_a_frags<C, W4, S_NEXT>(lds, next_off, fr, fa_next);
  const char* pb = b_frag_ptr<C, W4, S_NEXT>(lds, next_off, fr);
  __builtin_amdgcn_sched_barrier(0);
  static_for<0, C::FN>([&](auto j_) {
    constexpr int j = decltype(j_)::value;
    const v4i b = b_operand(fb[j]);
    static_for<0, C::FM>([&](auto i_) {
      constexpr int i = decltype(i_)::value;
      constexpr int q = j * C::FM + i;
      static_for<q * NR / NM, (q + 1) * NR / NM>([&](auto r_) { request(r_); });
      __builtin_amdgcn_sched_barrier(0);
      // W fragment as the row operand: the lane then holds 4 consecutive n per register group,
      // which the epilogue stores as one 16-byte piece of a Y row
      acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, fa[i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    });
    load_b_frag<C, W4>(pb, j, fb[j]);
    __builtin_amdgcn_sched_barrier(0);
  });
}

// A workgroup works off `chunk` output tiles that follow each other along M (same columns, so
// the W tile stays hot and, at any moment, the workgroups in flight still write all column blocks
// of Y: tiles that follow each other along N made the whole grid store into the same quarter of
// every Y row at the same time, which the memory channels punish).  Workgroup ids run with N
// fastest; `remap` regroups them so that the workgroups an XCD receives (ids congruent mod 8)
// cover a contiguous id range and share its L2.
// The k loop never drains between the tiles of a chunk: the requests issued during the last k
// tiles of one output tile already fetch the first k tiles of the next one, and the epilogue's
// stores overlap with those loads.  (k is padded to a multiple of NSTAGE tiles with zero tiles so
// that a tile always starts in stage 0.)  Chunks stay short so that the hardware dispatcher, not a
// fixed assignment, balances the load when other kernels hold some of the CUs.
// MINW: waves the register allocation must leave room for on one SIMD.
// EPI: 0 plain, 1 score, 2 activation and absmax of the output, 3 activation and int8 codes of the
// output (see EpiArgs); variants of their own because the largest tile has no registers to spare
// for them in the plain kernel.
template <int BM, int BN, int WM, int WN, int NSTAGE, bool W4, bool VEC, int KB, int MINW, int EPI>
__global__ __launch_bounds__(WM * WN * 64, MINW) void qgemm_dma(const int8_t* __restrict__ A,
                                                          const void* __restrict__ Wv, int64_t M,
                                                          int64_t N, int64_t K,
                                                          const float* __restrict__ a_scale,
                                                          const float* __restrict__ w_scale,
                                                          int w_per_row, float* __restrict__ Y,
                                                          int32_t* __restrict__ ACC, EpiArgs epi,
                                                          int tiles_n, int tiles_m, int chunk,
                                                          int remap) {
  constexpr bool SCORE = EPI == 1, ACT = EPI >= 2, AMAX = EPI == 2, QOUT = EPI == 3;
  int8_t* __restrict__ CODES = epi.codes;
  const float* __restrict__ YREF = epi.yref;
  double* __restrict__ PART = epi.part;
  using C = DmaCfg<BM, BN, WM, WN, NSTAGE, W4, KB>;
  constexpr int DBK = KB;
  constexpr int NSUB = DBK / 32;
  static_assert(NSUB % 2 == 0, "fragment double buffer assumes an even number of k substeps");
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int wm = wave / WN, wn = wave % WN;
  const unsigned lds0 = (unsigned)(uintptr_t)MPQ_LPTR(lds);  // LDS byte address of the buffer
  const uint8_t* Wb = reinterpret_cast<const uint8_t*>(Wv);
  const int G = (int)gridDim.x;
  int wg = (int)blockIdx.x;
  if (remap) wg = (wg & 7) * (G >> 3) + (wg >> 3);  // G % 8 == 0
  const int KT = (int)((K + DBK - 1) / DBK);
  const int KTp = (KT + NSTAGE - 1) / NSTAGE * NSTAGE;

  int tile = (wg / tiles_n) * chunk;  // row of tiles; < tiles_m: the grid is ceil(tiles_m / chunk) * tiles_n
  const int tile_end = tile + chunk < tiles_m ? tile + chunk : tiles_m;
  int64_t m0 = (int64_t)tile * BM;
  const int64_t n0 = (int64_t)(wg % tiles_n) * BN;
  DmaPlan<C, W4> plan;
  plan.init(A, Wb, M, N, K, m0, n0, wave, lane);
  int k_limit = (int)K;  // 0 once there is no next tile: every further request fetches zeros
  // Per-channel W scales of an output tile travel through LDS (one wave-load of 256 floats, issued
  // by every wave ahead of the tile's first k tile, into the buffer `par` selects): the epilogue
  // then needs no global loads between its stores and no registers to park the scales in.
  const bool want_y = Y || (SCORE && YREF) || (AMAX && epi.amax) || (QOUT && CODES);
  float q_inv = 0.0f, q_max = 0.0f;
  if (QOUT) {
    float q_scale;
    bit_constants(epi.q_absmax[0], epi.q_bits, q_scale, q_inv);
    q_max = (float)((1 << (epi.q_bits - 1)) - 1);
  }
  const bool lds_scales = VEC && want_y && w_per_row;
  unsigned par = 0;
  auto issue_scales = [&](int64_t n_first, unsigned which) {
    if (lds_scales) {  // wave-uniform
      const int64_t n = n_first + 4 * lane;
      const char* src = (4 * lane < BN && n < N) ? reinterpret_cast<const char*>(w_scale + n)
                                                 : reinterpret_cast<const char*>(g_zero16);
      dma16(src, lds0 + C::SCALE_OFF + which * 1024u);
    }
  };

  // Software pipeline.  Every stage holds a k tile; k tile t + NSTAGE is requested into the stage of
  // k tile t at the moment that stage has been read for the last time, which is BEFORE the MFMAs
  // of the tile's last k substep are issued (their operands sit in registers by then).  The same
  // point waits for k tile t + 1, passes the barrier and requests the first fragments of t + 1, so
  // that barrier skew, the address arithmetic of the loads and the LDS latency all hide behind the
  // matrix pipe working off the queued MFMAs.
  issue_scales(n0, par);  // older than every k tile request: the counted waits below cover it
#pragma unroll
  for (int p = 0; p < NSTAGE; ++p) plan.issue(lds0 + p * C::STAGE, p * DBK, k_limit);
  wait_vmcnt<(NSTAGE - 1) * C::LPW>();  // this wave's share of k tile 0 has landed
  __syncthreads();                      // ... and everyone else's
  v4i fa[2][C::FM];
  BRaw<W4> fb[C::FN];
  FragBase<C, W4> fr;
  fr.init(wm, wn, lane);
  load_a_frags<C, W4, 0>(lds, 0u, fr, fa[0]);
  {
    const char* pb = b_frag_ptr<C, W4, 0>(lds, 0u, fr);
#pragma unroll
    for (int j = 0; j < C::FN; ++j) load_b_frag<C, W4>(pb, j, fb[j]);
  }
  float sse = 0.0f;    // this lane's share of sum (Y - YREF)^2 over the chunk
  float amax = 0.0f;   // this lane's largest |Y| after the activation
  bool drain = false;  // true for the first wait after an epilogue: stores are in flight, and
                       // loads and stores do not retire in order with respect to each other

  while (true) {
    v16i acc[C::FM][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
#pragma unroll
      for (int j = 0; j < C::FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    const int next = tile + 1;
    const int64_t cur_m0 = m0, cur_n0 = n0;  // m0 moves on to the next tile before the epilogue

    for (int kt = 0; kt < KTp; kt += NSTAGE) {
      const bool tail = kt + NSTAGE >= KTp;  // requests from here on belong to the next output tile
      if (tail) {
        if (next < tile_end) {
          m0 = (int64_t)next * BM;
          plan.init(A, Wb, M, N, K, m0, n0, wave, lane);
        } else {
          k_limit = 0;
        }
      }
      static_for<0, NSTAGE>([&](auto u_) {
        constexpr int u = decltype(u_)::value;
        static_for<0, NSUB>([&](auto sub_) {
          constexpr int sub = decltype(sub_)::value;
          if constexpr (sub + 1 < NSUB) {
            k_substep<C, W4, sub + 1, 0>(acc, fa[sub & 1], fa[(sub + 1) & 1], fb, lds, (unsigned)(u * C::STAGE), fr,
                                         [](auto) {});
          } else {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wave has read the stage for the last time
            if (drain) wait_vmcnt<0>();                          // its share of the next k tile has landed
            else wait_vmcnt<(NSTAGE - 2) * C::LPW>();
            drain = false;
            __syncthreads();
            const int k_next = tail ? u * DBK : (kt + u + NSTAGE) * DBK;
            if (u == 0 && tail && next < tile_end) issue_scales(n0, par ^ 1u);
            const auto tl = plan.tile(k_next, k_limit);
            // the stage just given up is refilled while the last substep's MFMAs, whose operands
            // are in registers, run; the next stage's first fragments are read alongside
            k_substep<C, W4, 0, C::LPW>(acc, fa[sub & 1], fa[0], fb, lds, (unsigned)(((u + 1) % NSTAGE) * C::STAGE), fr,
                                        [&](auto r_) { plan.template request<decltype(r_)::value>(tl, lds0 + u * C::STAGE); });
          }
        });
      });
    }

    // epilogue.  32x32 accumulator tile (i, j): lane l holds m = l % 32 and, in registers
    // 4g .. 4g+3, the four consecutive n = 8g + 4 (l / 32) + 0..3.
    const float sa = want_y ? a_scale[0] : 0.0f;
    const float sw0 = (want_y && !w_per_row) ? w_scale[0] : 0.0f;
    const char* scales = lds + C::SCALE_OFF + par * 1024u;
#pragma unroll
    for (int i = 0; i < C::FM; ++i) {
      const int64_t m = cur_m0 + wm * C::TM + i * 32 + (lane & 31);
      if (m >= M) continue;
#pragma unroll
      for (int j = 0; j < C::FN; ++j) {
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int64_t n = cur_n0 + wn * C::TN + j * 32 + g4 * 8 + (lane >> 5) * 4;
          if (n >= N) continue;
          int a[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            a[e] = acc[i][j][g4 * 4 + e];
            if (W4) a[e] >>= 4;  // exact: every product carried the factor 16
          }
          if (VEC) {  // N % 4 == 0 and 16-byte aligned outputs: the four n are all in range
            if (ACC) *reinterpret_cast<v4i*>(ACC + m * N + n) = v4i{a[0], a[1], a[2], a[3]};
            if (want_y) {
              float4 sw = make_float4(sw0, sw0, sw0, sw0);
              if (w_per_row)
                sw = *reinterpret_cast<const float4*>(scales + (wn * C::TN + j * 32 + g4 * 8 + (lane >> 5) * 4) * 4);
              float4 y = make_float4(((float)a[0] * sa) * sw.x, ((float)a[1] * sa) * sw.y,
                                     ((float)a[2] * sa) * sw.z, ((float)a[3] * sa) * sw.w);
              if (ACT) {
                y = make_float4(apply_act(y.x, epi.act), apply_act(y.y, epi.act), apply_act(y.z, epi.act),
                                apply_act(y.w, epi.act));
                if (AMAX) amax = fmaxf(fmaxf(amax, fmaxf(fabsf(y.x), fabsf(y.y))), fmaxf(fabsf(y.z), fabsf(y.w)));
              }
              if (Y) *reinterpret_cast<float4*>(Y + m * N + n) = y;
              if (QOUT && CODES) {  // four codes, lowest n in the lowest byte
                const unsigned c0 = (unsigned)(int)code_f(y.x, q_inv, q_max) & 0xFFu;
                const unsigned c1 = (unsigned)(int)code_f(y.y, q_inv, q_max) & 0xFFu;
                const unsigned c2 = (unsigned)(int)code_f(y.z, q_inv, q_max) & 0xFFu;
                const unsigned c3 = (unsigned)(int)code_f(y.w, q_inv, q_max);
                *reinterpret_cast<unsigned*>(CODES + m * N + n) = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
              }
              if (SCORE && YREF) {
                const float4 r = *reinterpret_cast<const float4*>(YREF + m * N + n);
                float d = y.x - r.x;
                sse = __builtin_fmaf(d, d, sse);
                d = y.y - r.y;
                sse = __builtin_fmaf(d, d, sse);
                d = y.z - r.z;
                sse = __builtin_fmaf(d, d, sse);
                d = y.w - r.w;
                sse = __builtin_fmaf(d, d, sse);
              }
            }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if (n + e >= N) break;
              if (ACC) ACC[m * N + n + e] = a[e];
              if (want_y) {
                float y = ((float)a[e] * sa) * (w_per_row ? w_scale[n + e] : sw0);
                if (ACT) {
                  y = apply_act(y, epi.act);
                  if (AMAX) amax = fmaxf(amax, fabsf(y));
                }
                if (Y) Y[m * N + n + e] = y;
                if (QOUT && CODES) CODES[m * N + n + e] = (int8_t)(int)code_f(y, q_inv, q_max);
                if (SCORE && YREF) {
                  const float d = y - YREF[m * N + n + e];
                  sse = __builtin_fmaf(d, d, sse);
                }
              }
            }
          }
        }
      }
    }
    if (next >= tile_end) break;  // block-uniform
    tile = next;
    par ^= 1u;
    drain = true;
  }
  wait_vmcnt<0>();  // the zero-fill requests past the last tile land before the LDS is given back
  if (SCORE && PART) {  // one partial per workgroup, combined in a fixed order
    const float w = wave_sum(sse);
    __syncthreads();  // nobody reads a stage or a scale buffer any more
    float* sm = reinterpret_cast<float*>(lds);
    if (lane == 0) sm[wave] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
      double t = 0.0;
      for (int i = 0; i < C::NW; ++i) t += (double)sm[i];
      PART[blockIdx.x] = t;
    }
  }
  if (AMAX && epi.amax) {  // one atomic per workgroup
    const float w = wave_max(amax);
    __syncthreads();
    float* sm = reinterpret_cast<float*>(lds);
    if (lane == 0) sm[wave] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
      float t = 0.0f;
      for (int i = 0; i < C::NW; ++i) t = fmaxf(t, sm[i]);
      atomicMax(epi.amax, abs_key(t));
    }
  }
}

template <int BM, int BN, int WM, int WN, int NSTAGE, bool W4, int KB = 128, int MINW = 1>
static int launch_dma(const int8_t* a_q, const void* w_q, int64_t M, int64_t N, int64_t K,
                      const float* a_scale, const float* w_scale, int per_row, float* y_out,
                      int32_t* acc_out, hipStream_t st, EpiArgs epi = kNoEpi,
                      int64_t* n_partials = nullptr) {
  const float* y_ref = epi.yref;
  using C = DmaCfg<BM, BN, WM, WN, NSTAGE, W4, KB>;
  // float4 / int4 stores need every 4-group of n inside the row and 16-byte aligned
  const bool vec = (N & 3) == 0 && (!y_out || aligned16(y_out)) && (!acc_out || aligned16(acc_out)) &&
                   (!((y_out || y_ref || epi.amax || epi.codes) && per_row) || aligned16(w_scale)) &&
                   (!y_ref || aligned16(y_ref)) && (!epi.codes || (reinterpret_cast<uintptr_t>(epi.codes) & 3u) == 0);
  const int mode = y_ref ? 1 : epi.codes ? 3 : (epi.act || epi.amax) ? 2 : 0;
  auto kern = mode == 1 ? (vec ? qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, true, KB, MINW, 1>
                               : qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, false, KB, MINW, 1>)
            : mode == 2 ? (vec ? qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, true, KB, MINW, 2>
                               : qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, false, KB, MINW, 2>)
            : mode == 3 ? (vec ? qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, true, KB, MINW, 3>
                               : qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, false, KB, MINW, 3>)
                        : (vec ? qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, true, KB, MINW, 0>
                               : qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, false, KB, MINW, 0>);
  static bool attr_set[8] = {false, false, false, false, false, false, false, false};  // dynamic LDS above 64 KiB has to be allowed once per kernel
  const int which = mode * 2 + (vec ? 1 : 0);
  if (!attr_set[which]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) { set_last_hip_error((int)e); return MPQ_ERR_HIP; }
    attr_set[which] = true;
  }
  const int64_t tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
  if (tm * tn > 0x7FFFFFFF || tn > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  // Chunk length: the chip holds `slots` workgroups at a time (what the LDS allows per CU), so a
  // launch costs about ceil(grid / slots) * chunk tile times; take the length up to 4 that makes
  // this smallest, the longer one on a tie (more tile boundaries without a drain).
  int per_cu = (160 * 1024) / C::LDS_BYTES;
  if (per_cu > 4) per_cu = 4;
  if (per_cu < 1) per_cu = 1;
  const int64_t slots = kNumCU * per_cu;
  int chunk = 1;
  int64_t best = 0, grid = 0;
  for (int c = 1; c <= 4; ++c) {
    const int64_t g = ((tm + c - 1) / c) * tn;
    const int64_t cost = ((g + slots - 1) / slots) * c;
    if (c == 1 || cost <= best) { best = cost; chunk = c; grid = g; }
  }
  const int remap = (grid % 8 == 0 && grid >= 16) ? 1 : 0;
  kern<<<(unsigned)grid, C::NT, C::LDS_BYTES, st>>>(a_q, w_q, M, N, K, a_scale, w_scale, per_row, y_out,
                                                   acc_out, epi, (int)tn, (int)tm, chunk, remap);
  if (n_partials) *n_partials = grid;
  return launch_status();
}

// Validation and dispatch shared by mpq_qgemm and mpq_qgemm_score.  With y_ref the kernels also
// leave one partial sum of (Y - y_ref)^2 per workgroup in `partials` and report how many.
static int run_qgemm(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
                     int64_t K, const float* a_scale, const float* w_scale, int w_gran, float* y_out,
                     int32_t* acc_out, EpiArgs epi, int64_t* n_partials, hipStream_t st) {
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
  if (gx > 0x7FFFFFFF || gy > 65535) return MPQ_ERR_SHAPE;
  const int per_row = w_gran == MPQ_PER_ROW;
  const bool w4 = w_storage_bits == 4;
  // the fast kernels index rows with 32 bits
  const bool fast = aligned16(a_q) && aligned16(w_q) && (K % (w4 ? 32 : 16)) == 0 && M < (1ll << 31) && N < (1ll << 31);
  if (fast) {
    // tile choice (from sweeps over the configured shapes): 256 x 256 when that gives at least
    // three CUs in four a tile; else 192 x 192 (six waves) when it covers the problem in exactly
    // one round with at least three CUs in four busy and next to no padding (the BERT-base
    // widths: 768 = 4 x 192 gives 12288 x 768 exactly 256 tiles where 256 x 256 gives 144);
    // else 128 x 128 when it gives at least half of the CUs a tile, else 64 x 64.
    // 128 x 128 runs three stages (one workgroup per CU) when there is at most one tile per CU
    // anyway or k is long, two stages (two workgroups per CU) otherwise.
    auto tiles = [&](int64_t bm, int64_t bn) { return ((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    int pick = 64;
    const int64_t t192 = tiles(192, 192);
    if (N > 128 && tiles(256, 256) >= kNumCU * 3 / 4) pick = 256;
    else if (N % 192 == 0 && t192 <= kNumCU && t192 >= kNumCU * 3 / 4 && t192 * 192 * 192 <= M * N + M * N / 32) pick = 192;
    else if (N > 64 && tiles(128, 128) >= kNumCU / 2) pick = 128;
#define MPQ_DMA(BM_, BN_, WM_, WN_, NS_)                                                              \
  (w4 ? launch_dma<BM_, BN_, WM_, WN_, NS_, true>(a_q, w_q, M, N, K, a_scale, w_scale, per_row, y_out, \
                                                  acc_out, st, epi, n_partials)                        \
      : launch_dma<BM_, BN_, WM_, WN_, NS_, false>(a_q, w_q, M, N, K, a_scale, w_scale, per_row,     \
                                                   y_out, acc_out, st, epi, n_partials))
    if (pick == 256) return MPQ_DMA(256, 256, 4, 2, 2);
    if (pick == 192) return K >= 1024 ? MPQ_DMA(192, 192, 3, 2, 3) : MPQ_DMA(192, 192, 3, 2, 2);
    if (pick == 128)
      return (K >= 2048 || tiles(128, 128) <= kNumCU) ? MPQ_DMA(128, 128, 4, 2, 3) : MPQ_DMA(128, 128, 4, 2, 2);
    return MPQ_DMA(64, 64, 2, 2, 3);
#undef MPQ_DMA
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

extern "C" size_t mpq_qgemm_workspace_bytes(int64_t, int64_t, int64_t, int) { return 0; }

extern "C" int mpq_qgemm(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M,
                         int64_t N, int64_t K, const float* a_scale, const float* w_scale,
                         int w_gran, float* y_out, int32_t* acc_out, void* ws, size_t ws_bytes,
                         void* stream) {
  (void)ws;
  (void)ws_bytes;
  if (!y_out && !acc_out) return MPQ_ERR_NULL;
  return run_qgemm(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, y_out, acc_out,
                   kNoEpi, nullptr, (hipStream_t)stream);
}

extern "C" int mpq_qgemm_act(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
                             int64_t K, const float* a_scale, const float* w_scale, int w_gran, int act,
                             float* y_out, float* absmax_out, int accumulate, void* stream) {
  if (!y_out && !absmax_out) return MPQ_ERR_NULL;
  if (act < MPQ_ACT_NONE || act > MPQ_ACT_GELU) return MPQ_ERR_SHAPE;
  if (absmax_out && (reinterpret_cast<uintptr_t>(absmax_out) & 3u)) return MPQ_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  unsigned* amax = reinterpret_cast<unsigned*>(absmax_out);
  // validate before the fill: a failing call must leave the device untouched
  if (!a_q || !w_q || !a_scale || !w_scale) return MPQ_ERR_NULL;
  if (w_storage_bits != 8 && w_storage_bits != 4) return MPQ_ERR_BITS;
  if (M <= 0 || N <= 0 || K <= 0 || K > 133143 || (w_storage_bits == 4 && (K & 1))) return MPQ_ERR_SHAPE;
  if (w_gran != MPQ_PER_TENSOR && w_gran != MPQ_PER_ROW) return MPQ_ERR_GRAN;
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
  return run_qgemm(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, nullptr, nullptr,
                   EpiArgs{nullptr, nullptr, act, nullptr, absmax, bits, codes_out}, nullptr, (hipStream_t)stream);
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
  if (!y_ref || !sse_out) return MPQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(sse_out) & 7u) return MPQ_ERR_ALIGN;
  if (M <= 0 || N <= 0 || mul_overflows(M, N)) return MPQ_ERR_SHAPE;
  if (!ws || ws_bytes < (size_t)max_partials(M, N) * sizeof(double)) return MPQ_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 7u) return MPQ_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  double* partials = reinterpret_cast<double*>(ws);
  int64_t count = 0;
  const int rc = run_qgemm(a_q, w_q, w_storage_bits, M, N, K, a_scale, w_scale, w_gran, y_out, nullptr,
                           EpiArgs{y_ref, partials, 0, nullptr, nullptr, 0, nullptr}, &count, st);
  if (rc != MPQ_OK) return rc;
  sum_partials_k<<<1, kBlock, 0, st>>>(partials, count, sse_out);
  return launch_status();
}

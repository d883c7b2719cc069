// fake_quant.hip -- the quantizer of paper Sec. 3.1 Eq. 1 in its symmetric integer form:
// code = clamp(RNE(x * inv), +-qmax), Q(x) = code * scale.  Emits any of: fp32 Q(x), int8 codes,
// packed int4 codes.  HBM-bound: 4 bytes read + 4 / 1 / 0.5 bytes written per element.
//
// Arithmetic per element: clamp x to +-absmax once (this is the clip of Eq. 1 and makes the
// clamp of the code redundant: |x| <= m gives |x*inv| <= qmax(1 + 2^-24), which rounds to at
// most qmax), then t = fma(x, inv, 1.5*2^23).  The low mantissa bits of t ARE the two's
// complement code, so bytes and nibbles are cut straight from t's bit pattern.
#include "common.hpp"

namespace mpq {

struct QConst {
  float m, inv, scale;
};

__device__ __forceinline__ QConst make_qconst(float m, int bits) {
  QConst c;
  c.m = m;
  bit_constants(m, bits, c.scale, c.inv);
  return c;
}

// t = 1.5*2^23 + code (exactly); clip of Eq. 1 applied to x first
__device__ __forceinline__ float magic_t(float x, const QConst& c) {
  const float xc = __builtin_amdgcn_fmed3f(x, -c.m, c.m);
  return __builtin_fmaf(xc, c.inv, kMagic);
}
__device__ __forceinline__ float dequant_t(float t, const QConst& c) { return (t - kMagic) * c.scale; }

__device__ __forceinline__ unsigned pack_bytes(float t0, float t1, float t2, float t3) {
  const unsigned lo = __builtin_amdgcn_perm((unsigned)bits_from_f(t1), (unsigned)bits_from_f(t0), 0x0c0c0400u);
  const unsigned hi = __builtin_amdgcn_perm((unsigned)bits_from_f(t3), (unsigned)bits_from_f(t2), 0x04000c0cu);
  return lo | hi;
}
// low nibble = even column, high nibble = odd column
__device__ __forceinline__ unsigned pack_nibbles(float t0, float t1, float t2, float t3) {
  const unsigned a = (unsigned)bits_from_f(t0) & 0xFu, b = (unsigned)bits_from_f(t1) & 0xFu;
  const unsigned c = (unsigned)bits_from_f(t2) & 0xFu, d = (unsigned)bits_from_f(t3) & 0xFu;
  return a | (b << 4) | (c << 8) | (d << 12);
}

// one float4 of x with one constant set for all four columns
__device__ __forceinline__ void emit4(const float4 v, const QConst& c, int64_t i4, float* y,
                                      int8_t* codes, uint8_t* packed) {
  const float t0 = magic_t(v.x, c), t1 = magic_t(v.y, c), t2 = magic_t(v.z, c), t3 = magic_t(v.w, c);
  if (y) reinterpret_cast<float4*>(y)[i4] = make_float4(dequant_t(t0, c), dequant_t(t1, c), dequant_t(t2, c), dequant_t(t3, c));
  if (codes) reinterpret_cast<unsigned*>(codes)[i4] = pack_bytes(t0, t1, t2, t3);
  if (packed) reinterpret_cast<unsigned short*>(packed)[i4] = (unsigned short)pack_nibbles(t0, t1, t2, t3);
}

// ---- per tensor, flat, 128-bit loads; n4 = n / 4 vectors, tail of n % 4 scalars ------------
__global__ __launch_bounds__(kBlock) void fq_flat(const float* __restrict__ x, int64_t n,
                                                  const float* __restrict__ absmax, int bits,
                                                  float* __restrict__ y, int8_t* __restrict__ codes,
                                                  uint8_t* __restrict__ packed, float* __restrict__ step_out) {
  const QConst c = make_qconst(absmax[0], bits);
  const int64_t tid = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (step_out && tid == 0) step_out[0] = c.scale;  // the step size the codes dequantize with
  const int64_t n4 = n >> 2;
  for_each_vec4_tiled(reinterpret_cast<const float4*>(x), n4,
                      [&](const float4 v, int64_t i) { emit4(v, c, i, y, codes, packed); });
  // tail: at most 3 elements, pairs stay together (n even whenever packed != null)
  if (tid == 0) {
    for (int64_t j = n4 << 2; j < n; ++j) {
      const float t = magic_t(x[j], c);
      if (y) y[j] = dequant_t(t, c);
      if (codes) codes[j] = (int8_t)(bits_from_f(t) & 0xFF);
      if (packed && !(j & 1)) {
        const float t1 = magic_t(x[j + 1], c);
        packed[j >> 1] = (uint8_t)(((unsigned)bits_from_f(t) & 0xFu) | (((unsigned)bits_from_f(t1) & 0xFu) << 4));
      }
    }
  }
}

// ---- per row: one wave per (row, segment); cols % 4 == 0 -------------------------------------
constexpr int64_t kSeg = 16384;

__global__ __launch_bounds__(kBlock) void fq_rows(const float* __restrict__ x, int64_t rows,
                                                  int64_t cols, int64_t nseg,
                                                  const float* __restrict__ absmax, int bits,
                                                  float* __restrict__ y, int8_t* __restrict__ codes,
                                                  uint8_t* __restrict__ packed) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t item = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
  if (item >= rows * nseg) return;
  const int64_t r = item / nseg, seg = item - r * nseg;
  const int64_t c0 = seg * kSeg;
  const int64_t c1 = (c0 + kSeg < cols) ? c0 + kSeg : cols;
  const QConst c = make_qconst(absmax[r], bits);
  const int64_t base4 = (r * cols) >> 2;
  const float4* x4 = reinterpret_cast<const float4*>(x);
  int64_t i = (c0 >> 2) + lane;
  const int64_t end = c1 >> 2;
  for (; i + 3 * kWave < end; i += 4 * kWave) {  // four loads in flight per lane
    const float4 v0 = load_stream(x4 + base4 + i), v1 = load_stream(x4 + base4 + i + kWave),
                 v2 = load_stream(x4 + base4 + i + 2 * kWave), v3 = load_stream(x4 + base4 + i + 3 * kWave);
    emit4(v0, c, base4 + i, y, codes, packed);
    emit4(v1, c, base4 + i + kWave, y, codes, packed);
    emit4(v2, c, base4 + i + 2 * kWave, y, codes, packed);
    emit4(v3, c, base4 + i + 3 * kWave, y, codes, packed);
  }
  for (; i < end; i += kWave) emit4(load_stream(x4 + base4 + i), c, base4 + i, y, codes, packed);
}

// ---- per column: a lane owns 4 adjacent columns; cols % 4 == 0 --------------------------------
__global__ __launch_bounds__(kBlock) void fq_cols(const float* __restrict__ x, int64_t rows,
                                                  int64_t cols, const float* __restrict__ absmax,
                                                  int bits, float* __restrict__ y,
                                                  int8_t* __restrict__ codes,
                                                  uint8_t* __restrict__ packed) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int64_t c = ((int64_t)blockIdx.x * kWave + lane) * 4;
  if (c >= cols) return;
  const float4 m = *reinterpret_cast<const float4*>(absmax + c);
  const QConst k0 = make_qconst(m.x, bits), k1 = make_qconst(m.y, bits), k2 = make_qconst(m.z, bits),
               k3 = make_qconst(m.w, bits);
  const int64_t row_step = (int64_t)gridDim.y * (kBlock / kWave);
  for (int64_t r = (int64_t)blockIdx.y * (kBlock / kWave) + wave; r < rows; r += row_step) {
    const int64_t i4 = (r * cols + c) >> 2;
    const float4 v = reinterpret_cast<const float4*>(x)[i4];
    const float t0 = magic_t(v.x, k0), t1 = magic_t(v.y, k1), t2 = magic_t(v.z, k2), t3 = magic_t(v.w, k3);
    if (y) reinterpret_cast<float4*>(y)[i4] = make_float4(dequant_t(t0, k0), dequant_t(t1, k1), dequant_t(t2, k2), dequant_t(t3, k3));
    if (codes) reinterpret_cast<unsigned*>(codes)[i4] = pack_bytes(t0, t1, t2, t3);
    if (packed) reinterpret_cast<unsigned short*>(packed)[i4] = (unsigned short)pack_nibbles(t0, t1, t2, t3);
  }
}

// ---- generic: any shape / alignment / granularity; a thread owns one pair of flat elements ----
__global__ __launch_bounds__(kBlock) void fq_generic(const float* __restrict__ x, int64_t rows,
                                                     int64_t cols, int gran,
                                                     const float* __restrict__ absmax, int bits,
                                                     float* __restrict__ y, int8_t* __restrict__ codes,
                                                     uint8_t* __restrict__ packed, float* __restrict__ step_out) {
  const int64_t n = rows * cols;
  const int64_t npairs = (n + 1) >> 1;
  if (step_out && blockIdx.x == 0 && threadIdx.x == 0) step_out[0] = make_qconst(absmax[0], bits).scale;  // per tensor only
  for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p < npairs; p += (int64_t)gridDim.x * kBlock) {
    unsigned nib = 0;
    for (int e = 0; e < 2; ++e) {
      const int64_t j = 2 * p + e;
      if (j >= n) break;
      const int64_t r = j / cols, cc = j - r * cols;
      const int64_t ch = gran == MPQ_PER_ROW ? r : gran == MPQ_PER_COL ? cc : 0;
      const QConst c = make_qconst(absmax[ch], bits);
      const float t = magic_t(x[j], c);
      if (y) y[j] = dequant_t(t, c);
      if (codes) codes[j] = (int8_t)(bits_from_f(t) & 0xFF);
      nib |= ((unsigned)bits_from_f(t) & 0xFu) << (4 * e);
    }
    if (packed) packed[p] = (uint8_t)nib;  // cols even: the pair shares a row
  }
}

// mpq_fake_quant with one more output: for per-tensor granularity the kernel also leaves the step
// size scale_b in step_out[0] (what mpq_scale_from_absmax would compute in a launch of its own).
int fake_quant_launch(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax, int bits,
                      float* y_out, int8_t* codes_out, uint8_t* packed4_out, float* step_out, void* stream) {
  if (!x || !absmax) return MPQ_ERR_NULL;
  if (step_out && gran != MPQ_PER_TENSOR) return MPQ_ERR_GRAN;
  if (!y_out && !codes_out && !packed4_out) return MPQ_ERR_NULL;
  if (rows <= 0 || cols <= 0 || mul_overflows(rows, cols)) return MPQ_ERR_SHAPE;
  if (gran < MPQ_PER_TENSOR || gran > MPQ_PER_COL) return MPQ_ERR_GRAN;
  if (bits < 2 || bits > 8) return MPQ_ERR_BITS;
  if (packed4_out && bits > 4) return MPQ_ERR_BITS;
  if (packed4_out && (cols & 1)) return MPQ_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  const int64_t n = rows * cols;
  const bool vec_ok = aligned16(x) && (!y_out || aligned16(y_out)) &&
                      (!codes_out || (reinterpret_cast<uintptr_t>(codes_out) & 3u) == 0) &&
                      (!packed4_out || (reinterpret_cast<uintptr_t>(packed4_out) & 1u) == 0);
  if (vec_ok && gran == MPQ_PER_TENSOR) {
    fq_flat<<<flat_grid(n >> 2, kBlock * kTileVec), kBlock, 0, st>>>(x, n, absmax, bits, y_out, codes_out, packed4_out, step_out);
  } else if (vec_ok && gran == MPQ_PER_ROW && (cols & 3) == 0) {
    const int64_t nseg = (cols + kSeg - 1) / kSeg;
    const int64_t blocks = (rows * nseg + kBlock / kWave - 1) / (kBlock / kWave);
    if (blocks > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
    fq_rows<<<(unsigned)blocks, kBlock, 0, st>>>(x, rows, cols, nseg, absmax, bits, y_out, codes_out, packed4_out);
  } else if (vec_ok && gran == MPQ_PER_COL && (cols & 3) == 0 && aligned16(absmax)) {
    const int64_t gx = (cols + kWave * 4 - 1) / (kWave * 4);
    if (gx > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
    int64_t gy = ((int64_t)kNumCU * 8 + gx - 1) / gx;
    const int64_t max_gy = (rows + 4 * 8 - 1) / (4 * 8);
    if (gy > max_gy) gy = max_gy;
    if (gy < 1) gy = 1;
    if (gy > 65535) gy = 65535;
    fq_cols<<<dim3((unsigned)gx, (unsigned)gy), kBlock, 0, st>>>(x, rows, cols, absmax, bits, y_out, codes_out, packed4_out);
  } else {
    fq_generic<<<flat_grid((n + 1) >> 1, kBlock * 4), kBlock, 0, st>>>(x, rows, cols, gran, absmax, bits, y_out, codes_out, packed4_out, step_out);
  }
  return launch_status();
}

}  // namespace mpq

using namespace mpq;

extern "C" int mpq_fake_quant(const float* x, int64_t rows, int64_t cols, int gran,
                              const float* absmax, int bits, float* y_out, int8_t* codes_out,
                              uint8_t* packed4_out, void* stream) {
  return fake_quant_launch(x, rows, cols, gran, absmax, bits, y_out, codes_out, packed4_out, nullptr, stream);
}

extern "C" int mpq_fake_quant_step(const float* x, int64_t rows, int64_t cols, const float* absmax, int bits,
                                   float* y_out, int8_t* codes_out, uint8_t* packed4_out, float* step_out,
                                   void* stream) {
  if (!step_out) return MPQ_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(step_out) & 3u) return MPQ_ERR_ALIGN;
  return fake_quant_launch(x, rows, cols, MPQ_PER_TENSOR, absmax, bits, y_out, codes_out, packed4_out, step_out, stream);
}

// absmax.hip -- max calibration (paper Sec. 3.1, first step of scale estimation): m = max |x|
// per tensor, per row or per column.  HBM-bound: 4 bytes read per element, one v_max per element.
//
// Per tensor: every block writes one partial maximum to the workspace and a one-block kernel
// folds them (and the previous value when accumulating) -- thousands of atomics on ONE address
// serialise in L2 and cost ~10 us.  Per row / per column the outputs are many addresses: |x| >= 0,
// so its bit pattern orders like its value and blocks combine with an integer atomic max (exact,
// order independent) after a fill kernel cleared the output (a kernel, not a memset node, so the
// call can be captured in a HIP graph).
#include "common.hpp"

namespace mpq {

__global__ void fill_u32(unsigned* p, int64_t n, unsigned v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// flat tensor: contiguous 16 KiB tiles dealt round-robin when VEC, scalar grid-stride otherwise
// partials: float [gridDim.x]
template <bool VEC>
__global__ __launch_bounds__(kBlock) void absmax_flat(const float* __restrict__ x, int64_t n,
                                                      float* __restrict__ partials) {
  const int64_t tid = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t nthr = (int64_t)gridDim.x * kBlock;
  float m = 0.0f;
  if (VEC) {
    const int64_t n4 = n >> 2;
    for_each_vec4_tiled(reinterpret_cast<const float4*>(x), n4, [&](const float4 a, int64_t) {
      m = fmaxf(m, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
    });
    for (int64_t j = (n4 << 2) + tid; j < n; j += nthr) m = fmaxf(m, fabsf(x[j]));
  } else {
    for (int64_t j = tid; j < n; j += nthr) m = fmaxf(m, fabsf(x[j]));
  }
  m = wave_max(m);
  __shared__ float sm[kBlock / kWave];
  if ((threadIdx.x & (kWave - 1)) == 0) sm[threadIdx.x / kWave] = m;
  __syncthreads();
  if (threadIdx.x == 0) partials[blockIdx.x] = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
}

__global__ __launch_bounds__(kBlock) void absmax_finish(const float* __restrict__ partials, int np,
                                                        int accumulate, float* __restrict__ out) {
  float m = 0.0f;
#pragma unroll 8
  for (int p = threadIdx.x; p < np; p += kBlock) m = fmaxf(m, partials[p]);
  m = wave_max(m);
  __shared__ float sm[kBlock / kWave];
  if ((threadIdx.x & (kWave - 1)) == 0) sm[threadIdx.x / kWave] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    float b = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    if (accumulate) b = fmaxf(b, out[0]);
    out[0] = b;
  }
}

// per row: one wave per (row, segment of kSeg columns)
constexpr int64_t kSeg = 16384;

// DIRECT: one segment per row and no running maximum -> plain store, no clearing pass needed
template <bool VEC, bool DIRECT>
__global__ __launch_bounds__(kBlock) void absmax_rows(const float* __restrict__ x, int64_t rows,
                                                      int64_t cols, int64_t nseg,
                                                      unsigned* __restrict__ out) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t item = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
  if (item >= rows * nseg) return;  // whole wave leaves together
  const int64_t r = item / nseg, seg = item - r * nseg;
  const int64_t c0 = seg * kSeg;
  const int64_t c1 = (c0 + kSeg < cols) ? c0 + kSeg : cols;
  const float* row = x + r * cols;
  float m = 0.0f;
  if (VEC) {  // cols % 4 == 0 and x 16-byte aligned: every row start is aligned
    const float4* r4 = reinterpret_cast<const float4*>(row);
    int64_t i = (c0 >> 2) + lane;
    const int64_t end = c1 >> 2;
    for (; i + 3 * kWave < end; i += 4 * kWave) {  // four loads in flight per lane
      const float4 a = load_stream(r4 + i), b = load_stream(r4 + i + kWave), c = load_stream(r4 + i + 2 * kWave),
                   d = load_stream(r4 + i + 3 * kWave);
      m = fmaxf(m, fmaxf(fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))),
                         fmaxf(fmaxf(fabsf(b.x), fabsf(b.y)), fmaxf(fabsf(b.z), fabsf(b.w)))));
      m = fmaxf(m, fmaxf(fmaxf(fmaxf(fabsf(c.x), fabsf(c.y)), fmaxf(fabsf(c.z), fabsf(c.w))),
                         fmaxf(fmaxf(fabsf(d.x), fabsf(d.y)), fmaxf(fabsf(d.z), fabsf(d.w)))));
    }
    for (; i < end; i += kWave) {
      const float4 a = load_stream(r4 + i);
      m = fmaxf(m, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
    }
  } else {
    for (int64_t c = c0 + lane; c < c1; c += kWave) m = fmaxf(m, fabsf(row[c]));
  }
  m = wave_max(m);
  if (lane == 0) {
    if (DIRECT) out[r] = abs_key(m);
    else atomicMax(out + r, abs_key(m));
  }
}

// per column: a lane owns 4 adjacent columns (VEC) or one column; waves of a block take
// interleaved rows; blockIdx.y strides over row chunks.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void absmax_cols(const float* __restrict__ x, int64_t rows,
                                                      int64_t cols, unsigned* __restrict__ out) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int64_t row_step = (int64_t)gridDim.y * (kBlock / kWave);
  const int64_t r_first = (int64_t)blockIdx.y * (kBlock / kWave) + wave;
  if (VEC) {
    const int64_t c = ((int64_t)blockIdx.x * kWave + lane) * 4;
    if (c >= cols) return;
    float4 m = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int64_t r = r_first; r < rows; r += row_step) {
      const float4 a = *reinterpret_cast<const float4*>(x + r * cols + c);
      m.x = fmaxf(m.x, fabsf(a.x)); m.y = fmaxf(m.y, fabsf(a.y));
      m.z = fmaxf(m.z, fabsf(a.z)); m.w = fmaxf(m.w, fabsf(a.w));
    }
    atomicMax(out + c + 0, abs_key(m.x)); atomicMax(out + c + 1, abs_key(m.y));
    atomicMax(out + c + 2, abs_key(m.z)); atomicMax(out + c + 3, abs_key(m.w));
  } else {
    const int64_t c = (int64_t)blockIdx.x * kWave + lane;
    if (c >= cols) return;
    float m = 0.0f;
    for (int64_t r = r_first; r < rows; r += row_step) m = fmaxf(m, fabsf(x[r * cols + c]));
    atomicMax(out + c, abs_key(m));
  }
}

__global__ void scale_from_absmax_k(const float* __restrict__ absmax, int64_t count, int bits,
                                    float* __restrict__ scale_out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  float s, inv;
  bit_constants(absmax[i], bits, s, inv);
  scale_out[i] = s;
}

}  // namespace mpq

using namespace mpq;

static unsigned absmax_flat_grid(int64_t n, bool vec) {
  return vec ? flat_grid(n >> 2, kBlock * kTileVec) : flat_grid(n, kBlock * 4);
}

extern "C" size_t mpq_calibrate_absmax_workspace_bytes(int64_t rows, int64_t cols, int gran) {
  if (rows <= 0 || cols <= 0 || mul_overflows(rows, cols) || gran != MPQ_PER_TENSOR) return 0;
  const unsigned a = absmax_flat_grid(rows * cols, true), b = absmax_flat_grid(rows * cols, false);
  return (size_t)(a > b ? a : b) * sizeof(float);
}

extern "C" int mpq_calibrate_absmax(const float* x, int64_t rows, int64_t cols, int gran,
                                    int accumulate, float* absmax_out, void* ws, size_t ws_bytes,
                                    void* stream) {
  if (!x || !absmax_out) return MPQ_ERR_NULL;
  if (rows <= 0 || cols <= 0 || mul_overflows(rows, cols)) return MPQ_ERR_SHAPE;
  if (gran < MPQ_PER_TENSOR || gran > MPQ_PER_COL) return MPQ_ERR_GRAN;
  if (gran == MPQ_PER_TENSOR) {
    if (!ws || ws_bytes < mpq_calibrate_absmax_workspace_bytes(rows, cols, gran)) return MPQ_ERR_WORKSPACE;
    if (!aligned16(ws)) return MPQ_ERR_ALIGN;
  }
  hipStream_t st = (hipStream_t)stream;
  unsigned* out = reinterpret_cast<unsigned*>(absmax_out);
  const int64_t nch = channels(gran, rows, cols);
  const int64_t n = rows * cols;
  const int64_t nseg = (cols + kSeg - 1) / kSeg;
  const bool direct = gran == MPQ_PER_ROW && nseg == 1 && !accumulate;
  const bool a16 = aligned16(x);
  const bool vec = a16 && (cols & 3) == 0;
  // grid limits are part of the argument check: nothing is enqueued before they have passed
  const int64_t row_blocks = (rows * nseg + kBlock / kWave - 1) / (kBlock / kWave);
  const int64_t cols_per_block = vec ? kWave * 4 : kWave;
  const int64_t col_gx = (cols + cols_per_block - 1) / cols_per_block;
  if (gran == MPQ_PER_ROW && row_blocks > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  if (gran == MPQ_PER_COL && col_gx > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  if (gran != MPQ_PER_TENSOR && (nch + 255) / 256 > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  if (!accumulate && !direct && gran != MPQ_PER_TENSOR) {
    fill_u32<<<(unsigned)((nch + 255) / 256), 256, 0, st>>>(out, nch, 0u);
  }
  if (gran == MPQ_PER_TENSOR) {
    const unsigned g = absmax_flat_grid(n, a16);
    float* partials = reinterpret_cast<float*>(ws);
    if (a16) absmax_flat<true><<<g, kBlock, 0, st>>>(x, n, partials);
    else absmax_flat<false><<<g, kBlock, 0, st>>>(x, n, partials);
    absmax_finish<<<1, kBlock, 0, st>>>(partials, (int)g, accumulate, absmax_out);
  } else if (gran == MPQ_PER_ROW) {
    const unsigned g = (unsigned)row_blocks;
    if (vec && direct) absmax_rows<true, true><<<g, kBlock, 0, st>>>(x, rows, cols, nseg, out);
    else if (vec) absmax_rows<true, false><<<g, kBlock, 0, st>>>(x, rows, cols, nseg, out);
    else if (direct) absmax_rows<false, true><<<g, kBlock, 0, st>>>(x, rows, cols, nseg, out);
    else absmax_rows<false, false><<<g, kBlock, 0, st>>>(x, rows, cols, nseg, out);
  } else {
    const int64_t gx = col_gx;
    // enough row chunks to give the chip ~8 blocks per CU, at least 16 rows per wave
    int64_t gy = ((int64_t)kNumCU * 8 + gx - 1) / gx;
    const int64_t max_gy = (rows + 4 * 16 - 1) / (4 * 16);
    if (gy > max_gy) gy = max_gy;
    if (gy < 1) gy = 1;
    if (gy > 65535) gy = 65535;
    dim3 grid((unsigned)gx, (unsigned)gy);
    if (vec) absmax_cols<true><<<grid, kBlock, 0, st>>>(x, rows, cols, out);
    else absmax_cols<false><<<grid, kBlock, 0, st>>>(x, rows, cols, out);
  }
  return launch_status();
}

extern "C" int mpq_scale_from_absmax(const float* absmax, int64_t count, int bits,
                                     float* scale_out, void* stream) {
  if (!absmax || !scale_out) return MPQ_ERR_NULL;
  if (count <= 0 || count > ((int64_t)1 << 38)) return MPQ_ERR_SHAPE;
  if (bits < 2 || bits > 8) return MPQ_ERR_BITS;
  scale_from_absmax_k<<<(unsigned)((count + 255) / 256), 256, 0, (hipStream_t)stream>>>(
      absmax, count, bits, scale_out);
  return launch_status();
}

// quant_error.hip -- the sum under the expectation of paper Sec. 3.2.1 Eq. 2,
// SSE_b = sum (Q_b(x) - x)^2, for every bit-width b_lo..b_hi in ONE read of the tensor, per
// tensor / per row / per column; plus the two-tensor squared distance used as the candidate score.
//
// Per element and bit-width: t = fma(xc, inv_b, 1.5*2^23); q = t - 1.5*2^23; e = fma(q, scale_b, -x);
// acc_b = fma(e, e, acc_b) -- four VALU operations, with xc = clip(x, +-m) computed once (it
// replaces the clamp of the code, see fake_quant.hip; two bits take three, see sweep.hpp).
// 28 lane-operations per element for the full sweep b = 2..8 against 4 bytes of HBM traffic: a
// quarter below what the vector ALUs take
// from registers (mpq_diag_sweep_alu_rate), so the kernel is bound by HBM as long as nothing else
// gets into the inner loop (constants live in registers for the whole kernel, loads are 128-bit
// and four deep).
//
// Reproducibility: per-lane fp32 partial sums (a lane sees at most ~4k elements), fixed-order
// DPP wave reduction, then double precision across waves / blocks in a fixed order.  No float
// atomics anywhere.
#include "common.hpp"
#include "sweep.hpp"

#include <mutex>

namespace mpq {

constexpr int64_t kSeg = 16384;  // columns per wave item in the per-row kernels

// ---- per tensor ----------------------------------------------------------------------------
// partials: double [gridDim.x][NB]
template <int NB, bool VEC>
__global__ __launch_bounds__(kBlock) void qe_flat(const float* __restrict__ x, int64_t n,
                                                  const float* __restrict__ absmax, int b_lo,
                                                  double* __restrict__ partials) {
  Sweep<NB> s;
  s.init(absmax[0], b_lo);
  const int64_t tid = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t nthr = (int64_t)gridDim.x * kBlock;
  if (VEC) {
    const int64_t n4 = n >> 2;
    for_each_vec4_tiled(reinterpret_cast<const float4*>(x), n4, [&](const float4 v, int64_t) { s.add4(v); });
    for (int64_t j = (n4 << 2) + tid; j < n; j += nthr) s.add(x[j]);
  } else {
    for (int64_t j = tid; j < n; j += nthr) s.add(x[j]);
  }
  __shared__ float sm[kBlock / kWave][NB];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const float w = wave_sum(s.acc[b]);
    if (lane == 0) sm[wave][b] = w;
  }
  __syncthreads();
  if (threadIdx.x < NB)
    partials[(int64_t)blockIdx.x * NB + threadIdx.x] =
        ((double)sm[0][threadIdx.x] + (double)sm[1][threadIdx.x]) +
        ((double)sm[2][threadIdx.x] + (double)sm[3][threadIdx.x]);
}

// out[b] = sum_p partials[p][b], p < np, in a fixed order: thread t adds p = t, t + 256, ...
// (independent loads, unrolled), then a fixed LDS tree over the 256 threads.
template <int NB>
__global__ __launch_bounds__(kBlock) void qe_finish_tree(const double* __restrict__ partials,
                                                         int64_t np, double* __restrict__ out) {
  double a[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) a[b] = 0.0;
#pragma unroll 4
  for (int64_t p = threadIdx.x; p < np; p += kBlock) {
#pragma unroll
    for (int b = 0; b < NB; ++b) a[b] += partials[p * NB + b];
  }
  __shared__ double sm[kBlock][NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) sm[threadIdx.x][b] = a[b];
  __syncthreads();
  for (int half = kBlock / 2; half >= 1; half >>= 1) {
    if ((int)threadIdx.x < half) {
#pragma unroll
      for (int b = 0; b < NB; ++b) sm[threadIdx.x][b] += sm[threadIdx.x + half][b];
    }
    __syncthreads();
  }
  if (threadIdx.x < NB) out[threadIdx.x] = sm[0][threadIdx.x];
}

// partials laid out [np][nch][nb] (per-column kernels) or [nch][np][nb] (per-row kernels)
__global__ void qe_finish_serial(const double* __restrict__ partials, int64_t nch, int64_t np,
                                 int nb, int64_t stride_ch, int64_t stride_p,
                                 double* __restrict__ out) {
  const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= nch * nb) return;
  const int64_t ch = k / nb;
  const int b = (int)(k - ch * nb);
  double a = 0.0;
  for (int64_t p = 0; p < np; ++p) a += partials[ch * stride_ch + p * stride_p + b];
  out[k] = a;
}

// ---- per row: one wave per (row, segment) ------------------------------------------------------
// dst: nseg == 1 -> out [rows][NB]; else partials [rows][nseg][NB]; same indexing item*NB
template <int NB, bool VEC>
__global__ __launch_bounds__(kBlock) void qe_rows(const float* __restrict__ x, int64_t rows,
                                                  int64_t cols, int64_t nseg,
                                                  const float* __restrict__ absmax, int b_lo,
                                                  double* __restrict__ dst) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t item = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
  if (item >= rows * nseg) return;  // the whole wave leaves together
  const int64_t r = item / nseg, seg = item - r * nseg;
  const int64_t c0 = seg * kSeg;
  const int64_t c1 = (c0 + kSeg < cols) ? c0 + kSeg : cols;
  Sweep<NB> s;
  s.init(absmax[r], b_lo);
  const float* row = x + r * cols;
  if (VEC) {
    const float4* r4 = reinterpret_cast<const float4*>(row);
    int64_t i = (c0 >> 2) + lane;
    const int64_t e4 = c1 >> 2;
    for (; i + 3 * kWave < e4; i += 4 * kWave) {
      const float4 a = load_stream(r4 + i), b = load_stream(r4 + i + kWave), c = load_stream(r4 + i + 2 * kWave),
                   d = load_stream(r4 + i + 3 * kWave);
      s.add4(a); s.add4(b); s.add4(c); s.add4(d);
    }
    for (; i < e4; i += kWave) s.add4(load_stream(r4 + i));
  } else {
    for (int64_t c = c0 + lane; c < c1; c += kWave) s.add(row[c]);
  }
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const float w = wave_sum(s.acc[b]);
    if (lane == 0) dst[item * NB + b] = (double)w;
  }
}

// ---- per row, short rows: LPR lanes per row (16 or 64), 64 / LPR rows per wave ---------------------
// The 2 NB per-row constants cost a division each; here lane j of a row group computes constant j
// only and the group shares them through the cross-lane network, and the final sums need 4 DPP
// steps instead of a full wave reduction.  cols % 4 == 0, x 16-byte aligned, cols <= kSeg.
template <int NB, int LPR>
__global__ __launch_bounds__(kBlock) void qe_rows_sub(const float* __restrict__ x, int64_t rows,
                                                      int64_t cols, const float* __restrict__ absmax,
                                                      int b_lo, double* __restrict__ out) {
  constexpr int RW = kWave / LPR;  // rows per wave
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int lr = lane % LPR;
  int64_t r = ((int64_t)blockIdx.x * (kBlock / kWave) + wave) * RW + lane / LPR;
  const bool live = r < rows;
  if (!live) r = rows - 1;  // keep every lane active for the cross-lane steps; result discarded
  const float m = absmax[r];
  // lane j < 7: inv of bit-width b_lo + j; lane 7 + j: scale of bit-width b_lo + j
  float mine = 0.0f;
  {
    const int j = lr < 7 ? lr : lr - 7;
    float sc, inv;
    bit_constants(m, b_lo + (j < NB ? j : 0), sc, inv);
    mine = lr < 7 ? inv : sc;
  }
  Sweep<NB> s;
  s.m = m;
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    s.inv[b] = __shfl(mine, b, LPR);
    s.sc[b] = __shfl(mine, 7 + b, LPR);
    s.acc[b] = 0.0f;
  }
  const float4* r4 = reinterpret_cast<const float4*>(x + r * cols);
  const int64_t e4 = cols >> 2;
  int64_t i = lr;
  for (; i + 3 * LPR < e4; i += 4 * LPR) {
    const float4 a = load_stream(r4 + i), b = load_stream(r4 + i + LPR), c = load_stream(r4 + i + 2 * LPR),
                 d = load_stream(r4 + i + 3 * LPR);
    s.add4(a); s.add4(b); s.add4(c); s.add4(d);
  }
  for (; i < e4; i += LPR) s.add4(load_stream(r4 + i));
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const float w = LPR == 16 ? row16_sum(s.acc[b]) : wave_sum(s.acc[b]);
    if (lr == 0 && live) out[r * NB + b] = (double)w;
  }
}

// ---- per column: a lane owns CPL adjacent columns; the block's 4 waves take interleaved rows ----
// partials: double [gridDim.y][cols][NB]
template <int NB, int CPL>
__global__ __launch_bounds__(kBlock) void qe_cols(const float* __restrict__ x, int64_t rows,
                                                  int64_t cols, const float* __restrict__ absmax,
                                                  int b_lo, double* __restrict__ partials) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int64_t c = ((int64_t)blockIdx.x * kWave + lane) * CPL;
  const bool live = c < cols;
  Sweep<NB> s[CPL];
#pragma unroll
  for (int k = 0; k < CPL; ++k) s[k].init(live ? absmax[c + k] : 0.0f, b_lo);
  if (live) {
    const int64_t row_step = (int64_t)gridDim.y * (kBlock / kWave);
    for (int64_t r = (int64_t)blockIdx.y * (kBlock / kWave) + wave; r < rows; r += row_step) {
      if (CPL == 4) {
        const float4 v = *reinterpret_cast<const float4*>(x + r * cols + c);
        s[0].add(v.x); s[1 % CPL].add(v.y); s[2 % CPL].add(v.z); s[3 % CPL].add(v.w);
      } else {
        s[0].add(x[r * cols + c]);
      }
    }
  }
  __shared__ float sm[kBlock / kWave][kWave][CPL * NB + 1];
#pragma unroll
  for (int k = 0; k < CPL; ++k)
#pragma unroll
    for (int b = 0; b < NB; ++b) sm[wave][lane][k * NB + b] = s[k].acc[b];
  __syncthreads();
  if (wave == 0 && live) {
#pragma unroll
    for (int k = 0; k < CPL; ++k)
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int j = k * NB + b;
        const double v = ((double)sm[0][lane][j] + (double)sm[1][lane][j]) +
                         ((double)sm[2][lane][j] + (double)sm[3][lane][j]);
        partials[((int64_t)blockIdx.y * cols + c + k) * NB + b] = v;
      }
  }
}

// ---- two-tensor squared distance -----------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kBlock) void sse_pair_k(const float* __restrict__ y,
                                                     const float* __restrict__ yr, int64_t n,
                                                     double* __restrict__ partials) {
  const int64_t tid = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t nthr = (int64_t)gridDim.x * kBlock;
  float acc = 0.0f;
  auto add = [&](float a, float b) { const float e = a - b; acc = __builtin_fmaf(e, e, acc); };
  if (VEC) {
    const int64_t n4 = n >> 2;
    for_each_vec4_pair_tiled(reinterpret_cast<const float4*>(y), reinterpret_cast<const float4*>(yr), n4,
                             [&](const float4 a, const float4 b) {
                               add(a.x, b.x); add(a.y, b.y); add(a.z, b.z); add(a.w, b.w);
                             });
    for (int64_t j = (n4 << 2) + tid; j < n; j += nthr) add(y[j], yr[j]);
  } else {
    for (int64_t j = tid; j < n; j += nthr) add(y[j], yr[j]);
  }
  __shared__ float sm[kBlock / kWave];
  const float w = wave_sum(acc);
  if ((threadIdx.x & (kWave - 1)) == 0) sm[threadIdx.x / kWave] = w;
  __syncthreads();
  if (threadIdx.x == 0)
    partials[blockIdx.x] = ((double)sm[0] + (double)sm[1]) + ((double)sm[2] + (double)sm[3]);
}

// ---- launch geometry, shared by the workspace queries and the launchers --------------------------
struct QeGeom {
  unsigned gx = 1, gy = 1;
  int64_t nseg = 1;
  int64_t partial_doubles = 0;  // doubles of workspace
  bool vec = false;
};

static QeGeom qe_geometry(int64_t rows, int64_t cols, int gran, int nb, bool aligned) {
  QeGeom g;
  const int64_t n = rows * cols;
  if (gran == MPQ_PER_TENSOR) {
    g.vec = aligned;
    // 4 blocks per CU: the full sweep needs ~65 VGPRs (7 waves per SIMD), so 8 blocks per CU
    // would not be co-resident and the late blocks would trail the rest
    const unsigned gv = flat_grid(n >> 2, kBlock * kTileVec, 4), gs = flat_grid(n, kBlock * 4, 4);
    g.gx = g.vec ? gv : gs;
    // the query cannot see the pointer: reserve for the larger of the two grids
    const unsigned worst = gv > gs ? gv : gs;
    g.partial_doubles = (int64_t)worst * nb;
  } else if (gran == MPQ_PER_ROW) {
    g.vec = aligned && (cols & 3) == 0;
    g.nseg = (cols + kSeg - 1) / kSeg;
    const int64_t blocks = (rows * g.nseg + kBlock / kWave - 1) / (kBlock / kWave);
    g.gx = (unsigned)blocks;
    g.partial_doubles = g.nseg > 1 ? rows * g.nseg * nb : 0;
  } else {
    g.vec = aligned && (cols & 3) == 0;
    const int64_t worst_gx = (cols + kWave - 1) / kWave;          // scalar columns
    const int64_t gx = g.vec ? (cols + kWave * 4 - 1) / (kWave * 4) : worst_gx;
    // row chunks: fill the chip ~8 blocks per CU, at least 8 rows per wave
    auto rows_chunks = [&](int64_t gxx) {
      int64_t gy = ((int64_t)kNumCU * 8 + gxx - 1) / gxx;
      const int64_t max_gy = (rows + 4 * 8 - 1) / (4 * 8);
      if (gy > max_gy) gy = max_gy;
      if (gy < 1) gy = 1;
      if (gy > 65535) gy = 65535;
      return gy;
    };
    g.gx = (unsigned)gx;
    g.gy = (unsigned)rows_chunks(gx);
    const int64_t worst_gy = rows_chunks(worst_gx) > rows_chunks((cols + kWave * 4 - 1) / (kWave * 4))
                                 ? rows_chunks(worst_gx) : rows_chunks((cols + kWave * 4 - 1) / (kWave * 4));
    g.partial_doubles = worst_gy * cols * nb;
  }
  return g;
}

template <int NB>
static void launch_qe(const QeGeom& g, const float* x, int64_t rows, int64_t cols, int gran,
                      const float* absmax, int b_lo, double* out, double* ws, hipStream_t st) {
  const int64_t n = rows * cols;
  if (gran == MPQ_PER_TENSOR) {
    if (g.vec) qe_flat<NB, true><<<g.gx, kBlock, 0, st>>>(x, n, absmax, b_lo, ws);
    else qe_flat<NB, false><<<g.gx, kBlock, 0, st>>>(x, n, absmax, b_lo, ws);
    qe_finish_tree<NB><<<1, kBlock, 0, st>>>(ws, (int64_t)g.gx, out);
  } else if (gran == MPQ_PER_ROW) {
    double* dst = g.nseg == 1 ? out : ws;
    if (g.vec && g.nseg == 1) {
      // 16 lanes per row up to 2048 columns (>= 4 vectors per lane from 256 columns on), else a wave
      if (cols <= 2048) {
        const int64_t blocks = (rows + 15) / 16;
        qe_rows_sub<NB, 16><<<(unsigned)blocks, kBlock, 0, st>>>(x, rows, cols, absmax, b_lo, out);
      } else {
        const int64_t blocks = (rows + 3) / 4;
        qe_rows_sub<NB, 64><<<(unsigned)blocks, kBlock, 0, st>>>(x, rows, cols, absmax, b_lo, out);
      }
    } else if (g.vec) qe_rows<NB, true><<<g.gx, kBlock, 0, st>>>(x, rows, cols, g.nseg, absmax, b_lo, dst);
    else qe_rows<NB, false><<<g.gx, kBlock, 0, st>>>(x, rows, cols, g.nseg, absmax, b_lo, dst);
    if (g.nseg > 1) {
      const int64_t k = rows * NB;
      qe_finish_serial<<<(unsigned)((k + 255) / 256), 256, 0, st>>>(ws, rows, g.nseg, NB, g.nseg * NB, NB, out);
    }
  } else {
    dim3 grid(g.gx, g.gy);
    if (g.vec) qe_cols<NB, 4><<<grid, kBlock, 0, st>>>(x, rows, cols, absmax, b_lo, ws);
    else qe_cols<NB, 1><<<grid, kBlock, 0, st>>>(x, rows, cols, absmax, b_lo, ws);
    const int64_t k = cols * NB;
    qe_finish_serial<<<(unsigned)((k + 255) / 256), 256, 0, st>>>(ws, cols, (int64_t)g.gy, NB, NB, cols * NB, out);
  }
}

static int check_qe_args(int64_t rows, int64_t cols, int gran, int b_lo, int b_hi) {
  if (rows <= 0 || cols <= 0 || mul_overflows(rows, cols)) return MPQ_ERR_SHAPE;
  if (gran < MPQ_PER_TENSOR || gran > MPQ_PER_COL) return MPQ_ERR_GRAN;
  if (b_lo < 2 || b_hi > 8 || b_lo > b_hi) return MPQ_ERR_BITS;
  if (gran == MPQ_PER_ROW && (rows * ((cols + kSeg - 1) / kSeg) + 3) / 4 > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  if (gran == MPQ_PER_COL && (cols + kWave - 1) / kWave > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  return MPQ_OK;
}

}  // namespace mpq

using namespace mpq;

extern "C" size_t mpq_quant_error_workspace_bytes(int64_t rows, int64_t cols, int gran, int b_lo,
                                                  int b_hi) {
  if (check_qe_args(rows, cols, gran, b_lo, b_hi) != MPQ_OK) return 0;
  const QeGeom g = qe_geometry(rows, cols, gran, b_hi - b_lo + 1, true);
  return (size_t)g.partial_doubles * sizeof(double);
}

static int run_quant_error(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax, int b_lo,
                           int b_hi, double* sse_out, void* ws, size_t ws_bytes, bool builtin_scratch,
                           void* stream) {
  if (!x || !absmax || !sse_out) return MPQ_ERR_NULL;
  const int rc = check_qe_args(rows, cols, gran, b_lo, b_hi);
  if (rc != MPQ_OK) return rc;
  const int nb = b_hi - b_lo + 1;
  const QeGeom g = qe_geometry(rows, cols, gran, nb, aligned16(x));
  const size_t need = (size_t)g.partial_doubles * sizeof(double);
  if (need > 0 && (!ws || ws_bytes < need)) return builtin_scratch ? MPQ_ERR_TOO_LARGE : MPQ_ERR_WORKSPACE;
  if (need > 0 && !aligned16(ws)) return MPQ_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(sse_out) & 7u) != 0) return MPQ_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  double* wsd = reinterpret_cast<double*>(ws);
  switch (nb) {
    case 1: launch_qe<1>(g, x, rows, cols, gran, absmax, b_lo, sse_out, wsd, st); break;
    case 2: launch_qe<2>(g, x, rows, cols, gran, absmax, b_lo, sse_out, wsd, st); break;
    case 3: launch_qe<3>(g, x, rows, cols, gran, absmax, b_lo, sse_out, wsd, st); break;
    case 4: launch_qe<4>(g, x, rows, cols, gran, absmax, b_lo, sse_out, wsd, st); break;
    case 5: launch_qe<5>(g, x, rows, cols, gran, absmax, b_lo, sse_out, wsd, st); break;
    case 6: launch_qe<6>(g, x, rows, cols, gran, absmax, b_lo, sse_out, wsd, st); break;
    default: launch_qe<7>(g, x, rows, cols, gran, absmax, b_lo, sse_out, wsd, st); break;
  }
  return launch_status();
}

extern "C" int mpq_quant_error(const float* x, int64_t rows, int64_t cols, int gran,
                               const float* absmax, int b_lo, int b_hi, double* sse_out, void* ws,
                               size_t ws_bytes, void* stream) {
  return run_quant_error(x, rows, cols, gran, absmax, b_lo, b_hi, sse_out, ws, ws_bytes, false, stream);
}

// ---- the sweep for callers that cannot allocate -------------------------------------------------
// The partial sums live in a buffer that is part of the library's device image, so the call needs
// neither a workspace from the caller nor any allocation.  Every GPU the library runs on holds its
// own copy of the buffer, at its own address, for the life of the process.  In host code the
// array's name is only a handle for hipGetSymbolAddress: the device address is looked up once per
// device (with that device current) and kept; everything that touches the memory uses that pointer.
constexpr size_t kScratchBytes = MPQ_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device
int scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_last_hip_error((int)(e != hipSuccess ? e : hipErrorInvalidDevice));
    return MPQ_ERR_HIP;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      set_last_hip_error((int)(e != hipSuccess ? e : hipErrorInvalidSymbol));
      return MPQ_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MPQ_OK;
}
}  // namespace

extern "C" int mpq_quant_error_noalloc(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax,
                                       int b_lo, int b_hi, double* sse_out, void* stream) {
  // arguments first: a call that cannot succeed must not touch the device at all
  if (!x || !absmax || !sse_out) return MPQ_ERR_NULL;
  int rc = check_qe_args(rows, cols, gran, b_lo, b_hi);
  if (rc != MPQ_OK) return rc;
  if (mpq_quant_error_workspace_bytes(rows, cols, gran, b_lo, b_hi) > kScratchBytes) return MPQ_ERR_TOO_LARGE;
  void* ptr = nullptr;
  rc = scratch_of_current_device(&ptr);
  if (rc != MPQ_OK) return rc;
  // every partial the finishing kernel reads is written by the main kernel of the same call:
  // nothing in the buffer has to start at zero
  return run_quant_error(x, rows, cols, gran, absmax, b_lo, b_hi, sse_out, ptr, kScratchBytes, true, stream);
}

extern "C" size_t mpq_sse_pair_workspace_bytes(int64_t n) {
  if (n <= 0 || n > ((int64_t)1 << 46)) return 0;
  const unsigned a = flat_grid(n >> 2, kBlock * 2), b = flat_grid(n, kBlock * 4);
  return (size_t)(a > b ? a : b) * sizeof(double);
}

extern "C" int mpq_sse_pair(const float* y, const float* y_ref, int64_t n, double* sse_out,
                            void* ws, size_t ws_bytes, void* stream) {
  if (!y || !y_ref || !sse_out) return MPQ_ERR_NULL;
  if (n <= 0 || n > ((int64_t)1 << 46)) return MPQ_ERR_SHAPE;
  const bool vec = aligned16(y) && aligned16(y_ref);
  const unsigned grid = vec ? flat_grid(n >> 2, kBlock * 2) : flat_grid(n, kBlock * 4);
  if (!ws || ws_bytes < mpq_sse_pair_workspace_bytes(n)) return MPQ_ERR_WORKSPACE;
  if (!aligned16(ws) || (reinterpret_cast<uintptr_t>(sse_out) & 7u) != 0) return MPQ_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  double* wsd = reinterpret_cast<double*>(ws);
  if (vec) sse_pair_k<true><<<grid, kBlock, 0, st>>>(y, y_ref, n, wsd);
  else sse_pair_k<false><<<grid, kBlock, 0, st>>>(y, y_ref, n, wsd);
  qe_finish_tree<1><<<1, kBlock, 0, st>>>(wsd, (int64_t)grid, sse_out);
  return launch_status();
}

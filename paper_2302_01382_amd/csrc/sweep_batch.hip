// sweep_batch.hip -- the sensitivity sweep of paper Sec. 3.2.1 over a whole SET of tensors in a
// handful of launches: max calibration (Sec. 3.1) per output channel and per tensor, and the error
// sums of Eq. 2 for every bit-width, per tensor and per output channel.
//
// A model has on the order of a hundred weight tensors of a few megabytes each.  Swept one call
// at a time, every kernel is mostly launch ramp and tail (a 4 MB tensor is 1 us of HBM time) and
// every per-tensor result costs a finishing kernel of its own.  Here the caller describes the set
// once in a plan (built by a host function into caller memory and uploaded by the caller: the
// library still allocates and copies nothing); a launch then covers all tensors: the grid is a
// flat list of work items, an item being a 64 K-element chunk of one tensor (per-tensor sums) or a
// group of rows of one tensor (per-row results), and one finishing launch with a workgroup per
// tensor folds the items of each tensor in a fixed order.
//
// The arithmetic per element is the one of the single-tensor calls (sweep.hpp); per-row results
// are bit-identical to mpq_quant_error(MPQ_PER_ROW), per-tensor sums differ from
// mpq_quant_error(MPQ_PER_TENSOR) by the rounding of a different summation order.
// Where the maxima come from the swept tensors themselves (weights), one more call takes the row
// maxima and the per-row sums from the same read (calib_qe_rows_batch).
#include "common.hpp"
#include "sweep.hpp"

#include <cstring>

namespace mpq {

constexpr uint32_t kPlanMagic = 0x4D505153u;  // "MPQS"
constexpr int64_t kChunk = 65536;             // elements per flat work item (256 KiB)
constexpr int kRowGroupsPerItem = 2;          // row groups a row item walks through

struct PlanHeader {
  uint32_t magic;
  int32_t n_tensors;
  int32_t n_flat_items;
  int32_t n_row_items;
  int64_t bytes;
  int64_t elements;
};

struct PlanTensor {
  mpq_sweep_tensor t;
  int32_t flat_first, flat_count;  // this tensor's range in the flat item table
  int32_t row_first, row_count;    // ... and in the row item table
  int32_t lanes_per_row;           // 16 (rows up to 2048 columns) or 64
  int32_t rows_per_item;
};

struct PlanItem {
  int32_t tensor;
  int32_t index;  // chunk number / row-item number within the tensor
};

static size_t plan_bytes(int64_t n, int64_t flat, int64_t row) {
  return sizeof(PlanHeader) + (size_t)n * sizeof(PlanTensor) + (size_t)(flat + row) * sizeof(PlanItem);
}

__host__ __device__ inline const PlanTensor* plan_tensors(const void* plan) {
  return reinterpret_cast<const PlanTensor*>(reinterpret_cast<const char*>(plan) + sizeof(PlanHeader));
}
__host__ __device__ inline const PlanItem* plan_flat_items(const void* plan, int n_tensors) {
  return reinterpret_cast<const PlanItem*>(reinterpret_cast<const char*>(plan_tensors(plan)) +
                                           (size_t)n_tensors * sizeof(PlanTensor));
}

// per tensor: how the two item tables cut it
static int tensor_items(const mpq_sweep_tensor& t, int64_t* flat, int64_t* row, int* lpr, int* rpi) {
  if (!t.x) return MPQ_ERR_NULL;
  if (t.rows <= 0 || t.cols <= 0 || mul_overflows(t.rows, t.cols)) return MPQ_ERR_SHAPE;
  if (t.cols & 3) return MPQ_ERR_SHAPE;       // every row starts on a 16-byte boundary
  if (t.cols > 16384) return MPQ_ERR_SHAPE;   // a row is walked by one wave
  if (!aligned16(t.x)) return MPQ_ERR_ALIGN;
  *flat = (t.rows * t.cols + kChunk - 1) / kChunk;
  *lpr = t.cols <= 2048 ? 16 : 64;
  *rpi = (kBlock / *lpr) * kRowGroupsPerItem;
  *row = (t.rows + *rpi - 1) / *rpi;
  return MPQ_OK;
}

// ---- max calibration: row maxima, then the tensor's maximum from them ----------------------------
// A group of LPR lanes owns a row; all loads of a row are issued before the first use (rows up to
// 2048 columns: at most 32 float4 per lane would be too many registers, so four at a time).
template <int LPR>
__device__ __forceinline__ void absmax_rows_of_item(const PlanTensor& T, int index) {
  constexpr int RG = kBlock / LPR;  // rows per group of the workgroup
  const int lr = threadIdx.x % LPR;
  const int64_t e4 = T.t.cols >> 2;
  for (int g = 0; g < kRowGroupsPerItem; ++g) {
    const int64_t r = ((int64_t)index * kRowGroupsPerItem + g) * RG + threadIdx.x / LPR;
    const bool live = r < T.t.rows;
    const float4* r4 = reinterpret_cast<const float4*>(T.t.x + (live ? r : T.t.rows - 1) * T.t.cols);
    float m = 0.0f;
    int64_t i = lr;
    for (; i + 3 * LPR < e4; i += 4 * LPR) {
      const float4 a = load_stream(r4 + i), b = load_stream(r4 + i + LPR), c = load_stream(r4 + i + 2 * LPR),
                   d = load_stream(r4 + i + 3 * LPR);
      m = fmaxf(m, fmaxf(fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))),
                         fmaxf(fmaxf(fabsf(b.x), fabsf(b.y)), fmaxf(fabsf(b.z), fabsf(b.w)))));
      m = fmaxf(m, fmaxf(fmaxf(fmaxf(fabsf(c.x), fabsf(c.y)), fmaxf(fabsf(c.z), fabsf(c.w))),
                         fmaxf(fmaxf(fabsf(d.x), fabsf(d.y)), fmaxf(fabsf(d.z), fabsf(d.w)))));
    }
    for (; i < e4; i += LPR) {
      const float4 a = load_stream(r4 + i);
      m = fmaxf(m, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
    }
    if (LPR == 16) {
      m = fmaxf(m, dpp<kQuadSwap1>(m));
      m = fmaxf(m, dpp<kQuadSwap2>(m));
      m = fmaxf(m, dpp<kRowHalfMirror>(m));
      m = fmaxf(m, dpp<kRowMirror>(m));
    } else {
      m = wave_max(m);
    }
    if (lr == 0 && live) T.t.absmax_row[r] = m;
  }
}

__global__ __launch_bounds__(kBlock) void absmax_rows_batch(const void* __restrict__ plan) {
  const PlanHeader* H = reinterpret_cast<const PlanHeader*>(plan);
  const PlanItem it = (plan_flat_items(plan, H->n_tensors) + H->n_flat_items)[blockIdx.x];
  const PlanTensor& T = plan_tensors(plan)[it.tensor];
  if (T.lanes_per_row == 16) absmax_rows_of_item<16>(T, it.index);
  else absmax_rows_of_item<64>(T, it.index);
}

// one workgroup per tensor: the maximum of its row maxima (exact, order independent)
__global__ __launch_bounds__(kBlock) void absmax_tensor_batch(const void* __restrict__ plan) {
  const PlanTensor& T = plan_tensors(plan)[blockIdx.x];
  float m = 0.0f;
  const float* __restrict__ rm = T.t.absmax_row;
  const int64_t rows = T.t.rows;
  int64_t r = threadIdx.x;
  for (; r + 7 * kBlock < rows; r += 8 * kBlock) {  // eight independent loads in flight
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = rm[r + u * kBlock];
#pragma unroll
    for (int u = 0; u < 8; ++u) m = fmaxf(m, v[u]);
  }
  for (; r < rows; r += kBlock) m = fmaxf(m, rm[r]);
  m = wave_max(m);
  __shared__ float sm[kBlock / kWave];
  if ((threadIdx.x & (kWave - 1)) == 0) sm[threadIdx.x / kWave] = m;
  __syncthreads();
  if (threadIdx.x == 0) T.t.absmax_tensor[0] = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
}

// ---- Eq. 2 per tensor: one 64 K-element chunk per workgroup ---------------------------------------
// partials: double [n_flat_items][NB]
template <int NB>
__global__ __launch_bounds__(kBlock) void qe_flat_batch(const void* __restrict__ plan, int b_lo,
                                                        double* __restrict__ partials) {
  const PlanHeader* H = reinterpret_cast<const PlanHeader*>(plan);
  const PlanItem it = plan_flat_items(plan, H->n_tensors)[blockIdx.x];
  const PlanTensor& T = plan_tensors(plan)[it.tensor];
  const int64_t n = T.t.rows * T.t.cols;  // a multiple of 4
  const int64_t e0 = (int64_t)it.index * kChunk;
  const int64_t n4 = ((e0 + kChunk < n ? e0 + kChunk : n) - e0) >> 2;
  const float4* __restrict__ x4 = reinterpret_cast<const float4*>(T.t.x + e0);
  Sweep<NB> s;
  s.init(T.t.absmax_tensor[0], b_lo);
  constexpr int64_t tile = (int64_t)kBlock * kTileVec;
  for (int64_t base = threadIdx.x; base < n4; base += tile) {
    if (base - threadIdx.x + tile <= n4) {  // workgroup-uniform
      float4 v[kTileVec];
#pragma unroll
      for (int u = 0; u < kTileVec; ++u) v[u] = load_stream(x4 + base + u * kBlock);
#pragma unroll
      for (int u = 0; u < kTileVec; ++u) s.add4(v[u]);
    } else {
#pragma unroll
      for (int u = 0; u < kTileVec; ++u)
        if (base + u * kBlock < n4) s.add4(load_stream(x4 + base + u * kBlock));
    }
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

// one workgroup per tensor: sse_tensor[b] = sum of the tensor's item partials, in a fixed order
// (thread t takes items t, t + 256, ...; then a fixed tree over the threads).
// ROW_ITEMS: the partials are indexed by row item (the pass that takes both granularities at once)
template <int NB, bool ROW_ITEMS>
__global__ __launch_bounds__(kBlock) void qe_tensor_finish_batch(const void* __restrict__ plan,
                                                                 const double* __restrict__ partials) {
  const PlanTensor& T = plan_tensors(plan)[blockIdx.x];
  const int first = ROW_ITEMS ? T.row_first : T.flat_first;
  const int count = ROW_ITEMS ? T.row_count : T.flat_count;
  double a[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) a[b] = 0.0;
  for (int p = threadIdx.x; p < count; p += kBlock) {
#pragma unroll
    for (int b = 0; b < NB; ++b) a[b] += partials[(int64_t)(first + p) * NB + b];
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
  if (threadIdx.x < NB) T.t.sse_tensor[threadIdx.x] = sm[0][threadIdx.x];
}

// ---- Eq. 2 per row (and, with BOTH, per tensor in the same read) ----------------------------------
// LPR lanes own a row.  The 2 NB per-row constants cost a division each: lane j of a row group
// computes constant j only and the group shares them through the cross-lane network.
template <int NB, int LPR, bool BOTH>
__device__ __forceinline__ void qe_rows_of_item(const PlanTensor& T, int index, int b_lo, Sweep<NB>& st) {
  constexpr int RG = kBlock / LPR;
  const int lr = threadIdx.x % LPR;
  const int e4 = (int)(T.t.cols >> 2);  // at most 4096
  for (int g = 0; g < kRowGroupsPerItem; ++g) {
    int64_t r = ((int64_t)index * kRowGroupsPerItem + g) * RG + threadIdx.x / LPR;
    const bool live = r < T.t.rows;
    if (!live) r = T.t.rows - 1;  // every lane stays active for the cross-lane steps; result discarded
    const float m = T.t.absmax_row[r];
    float mine;
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
    const float4* r4 = reinterpret_cast<const float4*>(T.t.x + r * T.t.cols);
    int i = lr;
    for (; i + 3 * LPR < e4; i += 4 * LPR) {
      const float4 a = load_stream(r4 + i), b = load_stream(r4 + i + LPR), c = load_stream(r4 + i + 2 * LPR),
                   d = load_stream(r4 + i + 3 * LPR);
      s.add4(a); s.add4(b); s.add4(c); s.add4(d);
      if (BOTH && live) { st.add4(a); st.add4(b); st.add4(c); st.add4(d); }
    }
    for (; i < e4; i += LPR) {
      const float4 a = load_stream(r4 + i);
      s.add4(a);
      if (BOTH && live) st.add4(a);
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const float w = LPR == 16 ? row16_sum(s.acc[b]) : wave_sum(s.acc[b]);
      if (lr == 0 && live) T.t.sse_row[r * NB + b] = (double)w;
    }
  }
}

// partials (BOTH only): double [n_row_items][NB]
template <int NB, bool BOTH>
__global__ __launch_bounds__(kBlock) void qe_rows_batch(const void* __restrict__ plan, int b_lo,
                                                        double* __restrict__ partials) {
  const PlanHeader* H = reinterpret_cast<const PlanHeader*>(plan);
  const PlanItem it = (plan_flat_items(plan, H->n_tensors) + H->n_flat_items)[blockIdx.x];
  const PlanTensor& T = plan_tensors(plan)[it.tensor];
  Sweep<NB> st;
  if (BOTH) st.init(T.t.absmax_tensor[0], b_lo);
  if (T.lanes_per_row == 16) qe_rows_of_item<NB, 16, BOTH>(T, it.index, b_lo, st);
  else qe_rows_of_item<NB, 64, BOTH>(T, it.index, b_lo, st);
  if (BOTH) {
    __shared__ float sm[kBlock / kWave][NB];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const float w = wave_sum(st.acc[b]);
      if (lane == 0) sm[wave][b] = w;
    }
    __syncthreads();
    if (threadIdx.x < NB)
      partials[(int64_t)blockIdx.x * NB + threadIdx.x] =
          ((double)sm[0][threadIdx.x] + (double)sm[1][threadIdx.x]) +
          ((double)sm[2][threadIdx.x] + (double)sm[3][threadIdx.x]);
  }
}

// ---- max calibration per row AND Eq. 2 per row from ONE read -----------------------------------
// A row's share of a lane (at most kHold float4: rows up to 1024 columns on 16 lanes, up to 4096 on
// a wave) stays in registers between the two steps: the row maximum first, then the sweep on the
// same values.  Longer rows are read a second time; the second read comes out of the L2, which the
// row has just passed through (the first read is a plain load for that reason, the last one a
// streaming load).  Lane-to-element assignment and order are those of the two separate kernels, so
// the results are theirs bit for bit.
constexpr int kHold = 16;

template <int NB, int LPR>
__device__ __forceinline__ void calib_qe_rows_of_item(const PlanTensor& T, int index, int b_lo) {
  constexpr int RG = kBlock / LPR;
  const int lr = threadIdx.x % LPR;
  const int e4 = (int)(T.t.cols >> 2);
  const bool fits = e4 <= kHold * LPR;  // the same for every row of the tensor
  for (int g = 0; g < kRowGroupsPerItem; ++g) {
    int64_t r = ((int64_t)index * kRowGroupsPerItem + g) * RG + threadIdx.x / LPR;
    const bool live = r < T.t.rows;
    if (!live) r = T.t.rows - 1;  // every lane stays active for the cross-lane steps; result discarded
    const float4* r4 = reinterpret_cast<const float4*>(T.t.x + r * T.t.cols);
    float4 v[kHold];
    float m = 0.0f;
    if (fits) {
#pragma unroll
      for (int u = 0; u < kHold; ++u) {
        const int i = lr + u * LPR;
        v[u] = i < e4 ? load_stream(r4 + i) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      }
#pragma unroll
      for (int u = 0; u < kHold; ++u)
        m = fmaxf(m, fmaxf(fmaxf(fabsf(v[u].x), fabsf(v[u].y)), fmaxf(fabsf(v[u].z), fabsf(v[u].w))));
    } else {
      int i = lr;
      for (; i + 3 * LPR < e4; i += 4 * LPR) {
        const float4 a = r4[i], b = r4[i + LPR], c = r4[i + 2 * LPR], d = r4[i + 3 * LPR];
        m = fmaxf(m, fmaxf(fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))),
                           fmaxf(fmaxf(fabsf(b.x), fabsf(b.y)), fmaxf(fabsf(b.z), fabsf(b.w)))));
        m = fmaxf(m, fmaxf(fmaxf(fmaxf(fabsf(c.x), fabsf(c.y)), fmaxf(fabsf(c.z), fabsf(c.w))),
                           fmaxf(fmaxf(fabsf(d.x), fabsf(d.y)), fmaxf(fabsf(d.z), fabsf(d.w)))));
      }
      for (; i < e4; i += LPR) {
        const float4 a = r4[i];
        m = fmaxf(m, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
      }
    }
    if (LPR == 16) {  // every lane of the row group ends up with the row's maximum
      m = fmaxf(m, dpp<kQuadSwap1>(m));
      m = fmaxf(m, dpp<kQuadSwap2>(m));
      m = fmaxf(m, dpp<kRowHalfMirror>(m));
      m = fmaxf(m, dpp<kRowMirror>(m));
    } else {
      m = wave_max(m);
    }
    if (lr == 0 && live) T.t.absmax_row[r] = m;
    float mine;
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
    if (fits) {
#pragma unroll
      for (int u = 0; u < kHold; ++u)
        if (lr + u * LPR < e4) s.add4(v[u]);
    } else {
      int i = lr;
      for (; i + 3 * LPR < e4; i += 4 * LPR) {
        const float4 a = load_stream(r4 + i), b = load_stream(r4 + i + LPR), c = load_stream(r4 + i + 2 * LPR),
                     d = load_stream(r4 + i + 3 * LPR);
        s.add4(a); s.add4(b); s.add4(c); s.add4(d);
      }
      for (; i < e4; i += LPR) s.add4(load_stream(r4 + i));
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const float w = LPR == 16 ? row16_sum(s.acc[b]) : wave_sum(s.acc[b]);
      if (lr == 0 && live) T.t.sse_row[r * NB + b] = (double)w;
    }
  }
}

template <int NB>
__global__ __launch_bounds__(kBlock) void calib_qe_rows_batch(const void* __restrict__ plan, int b_lo) {
  const PlanHeader* H = reinterpret_cast<const PlanHeader*>(plan);
  const PlanItem it = (plan_flat_items(plan, H->n_tensors) + H->n_flat_items)[blockIdx.x];
  const PlanTensor& T = plan_tensors(plan)[it.tensor];
  if (T.lanes_per_row == 16) calib_qe_rows_of_item<NB, 16>(T, it.index, b_lo);
  else calib_qe_rows_of_item<NB, 64>(T, it.index, b_lo);
}

template <int NB>
static void launch_qe_batch(const PlanHeader* H, const void* plan_dev, int gran, int b_lo, double* ws,
                            hipStream_t st) {
  const unsigned nt = (unsigned)H->n_tensors;
  if (gran == MPQ_PER_TENSOR) {
    qe_flat_batch<NB><<<(unsigned)H->n_flat_items, kBlock, 0, st>>>(plan_dev, b_lo, ws);
    qe_tensor_finish_batch<NB, false><<<nt, kBlock, 0, st>>>(plan_dev, ws);
  } else if (gran == MPQ_PER_ROW) {
    qe_rows_batch<NB, false><<<(unsigned)H->n_row_items, kBlock, 0, st>>>(plan_dev, b_lo, nullptr);
  } else {
    qe_rows_batch<NB, true><<<(unsigned)H->n_row_items, kBlock, 0, st>>>(plan_dev, b_lo, ws);
    qe_tensor_finish_batch<NB, true><<<nt, kBlock, 0, st>>>(plan_dev, ws);
  }
}

static const PlanHeader* checked_plan(const void* plan_host) {
  if (!plan_host) return nullptr;
  const PlanHeader* H = reinterpret_cast<const PlanHeader*>(plan_host);
  if (H->magic != kPlanMagic || H->n_tensors <= 0) return nullptr;
  if ((size_t)H->bytes != plan_bytes(H->n_tensors, H->n_flat_items, H->n_row_items)) return nullptr;
  return H;
}

}  // namespace mpq

using namespace mpq;

extern "C" size_t mpq_sweep_plan_bytes(const mpq_sweep_tensor* tensors, int n_tensors) {
  if (!tensors || n_tensors <= 0) return 0;
  int64_t flat = 0, row = 0;
  for (int i = 0; i < n_tensors; ++i) {
    int64_t f, r;
    int lpr, rpi;
    if (tensor_items(tensors[i], &f, &r, &lpr, &rpi) != MPQ_OK) return 0;
    flat += f;
    row += r;
    if (flat > 0x7FFFFFFF || row > 0x7FFFFFFF) return 0;
  }
  return plan_bytes(n_tensors, flat, row);
}

extern "C" int mpq_sweep_plan_build(const mpq_sweep_tensor* tensors, int n_tensors, void* plan_host,
                                    size_t plan_host_bytes) {
  if (!tensors || !plan_host) return MPQ_ERR_NULL;
  if (n_tensors <= 0) return MPQ_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(plan_host) & 7u) return MPQ_ERR_ALIGN;
  int64_t flat = 0, row = 0;
  for (int i = 0; i < n_tensors; ++i) {
    int64_t f, r;
    int lpr, rpi;
    const int rc = tensor_items(tensors[i], &f, &r, &lpr, &rpi);
    if (rc != MPQ_OK) return rc;
    if (!tensors[i].absmax_row || !tensors[i].absmax_tensor) return MPQ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(tensors[i].absmax_row) & 3u) ||
        (reinterpret_cast<uintptr_t>(tensors[i].absmax_tensor) & 3u) ||
        (reinterpret_cast<uintptr_t>(tensors[i].sse_tensor) & 7u) ||
        (reinterpret_cast<uintptr_t>(tensors[i].sse_row) & 7u))
      return MPQ_ERR_ALIGN;
    flat += f;
    row += r;
    if (flat > 0x7FFFFFFF || row > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  }
  const size_t need = plan_bytes(n_tensors, flat, row);
  if (plan_host_bytes < need) return MPQ_ERR_WORKSPACE;
  PlanHeader* H = reinterpret_cast<PlanHeader*>(plan_host);
  PlanTensor* T = reinterpret_cast<PlanTensor*>(reinterpret_cast<char*>(plan_host) + sizeof(PlanHeader));
  PlanItem* F = reinterpret_cast<PlanItem*>(T + n_tensors);
  PlanItem* R = F + flat;
  int64_t f0 = 0, r0 = 0, elements = 0;
  for (int i = 0; i < n_tensors; ++i) {
    int64_t f, r;
    int lpr, rpi;
    tensor_items(tensors[i], &f, &r, &lpr, &rpi);
    std::memset(&T[i], 0, sizeof(PlanTensor));
    T[i].t = tensors[i];
    T[i].flat_first = (int32_t)f0;
    T[i].flat_count = (int32_t)f;
    T[i].row_first = (int32_t)r0;
    T[i].row_count = (int32_t)r;
    T[i].lanes_per_row = lpr;
    T[i].rows_per_item = rpi;
    for (int64_t k = 0; k < f; ++k) F[f0 + k] = PlanItem{i, (int32_t)k};
    for (int64_t k = 0; k < r; ++k) R[r0 + k] = PlanItem{i, (int32_t)k};
    f0 += f;
    r0 += r;
    elements += tensors[i].rows * tensors[i].cols;
  }
  H->magic = kPlanMagic;
  H->n_tensors = n_tensors;
  H->n_flat_items = (int32_t)flat;
  H->n_row_items = (int32_t)row;
  H->bytes = (int64_t)need;
  H->elements = elements;
  return MPQ_OK;
}

extern "C" int mpq_calibrate_absmax_batch(const void* plan_host, const void* plan_dev, void* stream) {
  if (!plan_host || !plan_dev) return MPQ_ERR_NULL;
  const PlanHeader* H = checked_plan(plan_host);
  if (!H) return MPQ_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(plan_dev) & 7u) return MPQ_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  absmax_rows_batch<<<(unsigned)H->n_row_items, kBlock, 0, st>>>(plan_dev);
  absmax_tensor_batch<<<(unsigned)H->n_tensors, kBlock, 0, st>>>(plan_dev);
  return launch_status();
}

extern "C" size_t mpq_quant_error_batch_workspace_bytes(const void* plan_host, int gran, int b_lo, int b_hi) {
  const PlanHeader* H = checked_plan(plan_host);
  if (!H || b_lo < 2 || b_hi > 8 || b_lo > b_hi) return 0;
  const int nb = b_hi - b_lo + 1;
  if (gran == MPQ_PER_TENSOR) return (size_t)H->n_flat_items * nb * sizeof(double);
  if (gran == MPQ_SWEEP_TENSOR_AND_ROW) return (size_t)H->n_row_items * nb * sizeof(double);
  return 0;
}

extern "C" int mpq_quant_error_batch(const void* plan_host, const void* plan_dev, int gran, int b_lo, int b_hi,
                                     void* ws, size_t ws_bytes, void* stream) {
  if (!plan_host || !plan_dev) return MPQ_ERR_NULL;
  const PlanHeader* H = checked_plan(plan_host);
  if (!H) return MPQ_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(plan_dev) & 7u) return MPQ_ERR_ALIGN;
  if (gran != MPQ_PER_TENSOR && gran != MPQ_PER_ROW && gran != MPQ_SWEEP_TENSOR_AND_ROW) return MPQ_ERR_GRAN;
  if (b_lo < 2 || b_hi > 8 || b_lo > b_hi) return MPQ_ERR_BITS;
  const PlanTensor* T = plan_tensors(plan_host);
  for (int i = 0; i < H->n_tensors; ++i) {
    if (gran != MPQ_PER_ROW && !T[i].t.sse_tensor) return MPQ_ERR_NULL;
    if (gran != MPQ_PER_TENSOR && !T[i].t.sse_row) return MPQ_ERR_NULL;
  }
  const size_t need = mpq_quant_error_batch_workspace_bytes(plan_host, gran, b_lo, b_hi);
  if (need > 0 && (!ws || ws_bytes < need)) return MPQ_ERR_WORKSPACE;
  if (need > 0 && (reinterpret_cast<uintptr_t>(ws) & 7u)) return MPQ_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  double* wsd = reinterpret_cast<double*>(ws);
  switch (b_hi - b_lo + 1) {
    case 1: launch_qe_batch<1>(H, plan_dev, gran, b_lo, wsd, st); break;
    case 2: launch_qe_batch<2>(H, plan_dev, gran, b_lo, wsd, st); break;
    case 3: launch_qe_batch<3>(H, plan_dev, gran, b_lo, wsd, st); break;
    case 4: launch_qe_batch<4>(H, plan_dev, gran, b_lo, wsd, st); break;
    case 5: launch_qe_batch<5>(H, plan_dev, gran, b_lo, wsd, st); break;
    case 6: launch_qe_batch<6>(H, plan_dev, gran, b_lo, wsd, st); break;
    default: launch_qe_batch<7>(H, plan_dev, gran, b_lo, wsd, st); break;
  }
  return launch_status();
}

extern "C" int mpq_calibrate_quant_error_rows_batch(const void* plan_host, const void* plan_dev, int b_lo, int b_hi,
                                                    void* stream) {
  if (!plan_host || !plan_dev) return MPQ_ERR_NULL;
  const PlanHeader* H = checked_plan(plan_host);
  if (!H) return MPQ_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(plan_dev) & 7u) return MPQ_ERR_ALIGN;
  if (b_lo < 2 || b_hi > 8 || b_lo > b_hi) return MPQ_ERR_BITS;
  const PlanTensor* T = plan_tensors(plan_host);
  for (int i = 0; i < H->n_tensors; ++i)
    if (!T[i].t.sse_row) return MPQ_ERR_NULL;
  hipStream_t st = (hipStream_t)stream;
  const unsigned grid = (unsigned)H->n_row_items;
  switch (b_hi - b_lo + 1) {
    case 1: calib_qe_rows_batch<1><<<grid, kBlock, 0, st>>>(plan_dev, b_lo); break;
    case 2: calib_qe_rows_batch<2><<<grid, kBlock, 0, st>>>(plan_dev, b_lo); break;
    case 3: calib_qe_rows_batch<3><<<grid, kBlock, 0, st>>>(plan_dev, b_lo); break;
    case 4: calib_qe_rows_batch<4><<<grid, kBlock, 0, st>>>(plan_dev, b_lo); break;
    case 5: calib_qe_rows_batch<5><<<grid, kBlock, 0, st>>>(plan_dev, b_lo); break;
    case 6: calib_qe_rows_batch<6><<<grid, kBlock, 0, st>>>(plan_dev, b_lo); break;
    default: calib_qe_rows_batch<7><<<grid, kBlock, 0, st>>>(plan_dev, b_lo); break;
  }
  absmax_tensor_batch<<<(unsigned)H->n_tensors, kBlock, 0, st>>>(plan_dev);
  return launch_status();
}

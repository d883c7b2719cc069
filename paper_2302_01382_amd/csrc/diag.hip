// diag.hip -- measurement aids, not part of the method.
// (1) The rate at which this chip issues
// v_mfma_i32_32x32x32_i8 when nothing else happens (operands sit in registers, no memory traffic
// inside the loop).  The sustained clock under matrix load depends on how much the operand bits
// toggle, so the "matrix peak" a GEMM can be held against is this measured rate on operands like
// its own, not the nominal 5 POP/s: on MI355X about 4.9 POP/s for constant bytes and about
// 3.3 POP/s for uniformly random int8.
// (2) The rate at which it works off the arithmetic of the error sweep (sweep.hpp, b = 2..8) when the
// elements sit in registers: the vector-ALU ceiling of that kernel, measured instead of derived.
#include "common.hpp"
#include "sweep.hpp"

namespace mpq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBurnWaves = 8;  // per workgroup, one workgroup per CU: two waves per SIMD, like the GEMM

// every lane reads 8 x 16 bytes of operands once, then 16 matrix steps per iteration on them
__global__ __launch_bounds__(kBurnWaves * 64) void mfma_burn(const v4i* __restrict__ src, int iters,
                                                             int* __restrict__ sink) {
  const size_t base = ((size_t)blockIdx.x * (kBurnWaves * 64) + threadIdx.x) * 8;
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = src[base + i];
    b[i] = src[base + 4 + i];
  }
  v16i acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[j], b[(i + j) & 3], acc[i], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  if (s == 0x7fffffff) sink[0] = s;  // keeps the loop alive; practically never taken
}

constexpr int kSweepBurnBlocksPerCU = 8;  // of 256 threads: eight waves per SIMD

// 16 elements per lane and iteration through Sweep<7>::add, nothing else in the loop
__global__ __launch_bounds__(256) void sweep_burn(int iters, float absmax, float* __restrict__ sink) {
  Sweep<7> s;
  s.init(absmax, 2);
  float4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const float t = (float)threadIdx.x * 1e-3f + (float)u * 0.25f;
    v[u] = make_float4(t, -t, 0.5f * t, 0.1f - t);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      s.add4(v[u]);
      // the compiler may not assume the elements stay the same from one iteration to the next
      asm volatile("" : "+v"(v[u].x), "+v"(v[u].y), "+v"(v[u].z), "+v"(v[u].w));
    }
  }
  float t = 0.0f;
#pragma unroll
  for (int b = 0; b < 7; ++b) t += s.acc[b];
  if (t == -1.0f) sink[0] = t;  // keeps the loop alive; a sum of squares is never negative
}

}  // namespace mpq

using namespace mpq;

extern "C" size_t mpq_diag_mfma_operand_bytes(void) { return (size_t)kNumCU * kBurnWaves * 64 * 8 * 16; }

extern "C" int mpq_diag_mfma_rate(const void* operands, size_t operand_bytes, int iters, int* sink, double* ops_out,
                                  void* stream) {
  if (!operands || !sink) return MPQ_ERR_NULL;
  if (operand_bytes < mpq_diag_mfma_operand_bytes()) return MPQ_ERR_WORKSPACE;
  if (!aligned16(operands)) return MPQ_ERR_ALIGN;
  if (iters <= 0 || iters > (1 << 20)) return MPQ_ERR_SHAPE;
  mfma_burn<<<kNumCU, kBurnWaves * 64, 0, (hipStream_t)stream>>>(reinterpret_cast<const v4i*>(operands), iters, sink);
  if (ops_out) *ops_out = (double)kNumCU * kBurnWaves * (double)iters * 16.0 * 2.0 * 32 * 32 * 32;
  return launch_status();
}

extern "C" int mpq_diag_sweep_alu_rate(int iters, float* sink, double* lane_ops_out, void* stream) {
  if (!sink) return MPQ_ERR_NULL;
  if (iters <= 0 || iters > (1 << 20)) return MPQ_ERR_SHAPE;
  const unsigned blocks = (unsigned)(kNumCU * kSweepBurnBlocksPerCU);
  sweep_burn<<<blocks, 256, 0, (hipStream_t)stream>>>(iters, 3.7f, sink);
  // 16 elements per lane and iteration, 28 lane-operations per element (6 widths x 4, two bits 3, one clip)
  if (lane_ops_out) *lane_ops_out = (double)blocks * 256.0 * (double)iters * 16.0 * 28.0;
  return launch_status();
}

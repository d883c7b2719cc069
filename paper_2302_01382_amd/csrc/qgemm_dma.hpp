// qgemm_dma.hpp -- the fast path of the quantized linear layer (the evaluation step of the paper's
// Alg. 1 / Alg. 2): the templated multi-stage LDS pipeline fed by direct global->LDS loads, shared by
// the translation units that instantiate one tile size each (qgemm_t*.hip), and the epilogue
// options shared with the generic kernel (qgemm.hip).
#pragma once

#include "common.hpp"

#include <atomic>
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

// 8 nibbles of `w` (lowest nibble = lowest k) -> 8 bytes, each nibble << 4, in k order
__device__ __forceinline__ void expand8(unsigned w, unsigned& lo, unsigned& hi) {
  const unsigned e = (w << 4) & 0xF0F0F0F0u;  // nibbles 0,2,4,6
  const unsigned o = w & 0xF0F0F0F0u;         // nibbles 1,3,5,7
  lo = __builtin_amdgcn_perm(o, e, 0x05010400u);
  hi = __builtin_amdgcn_perm(o, e, 0x07030602u);
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

static __device__ __attribute__((aligned(16))) int g_zero16[4];  // never written: zero fill for k tails


// The direct-to-LDS load and its wait are written as inline assembly on purpose: when the
// compiler sees the load it cannot tell which LDS bytes are in flight once more than a handful of
// them are outstanding, and puts a full "s_waitcnt vmcnt(0)" in front of every LDS read -- which
// would serialise the pipeline.  Written this way the compiler does not track them, and the
// kernel does the bookkeeping itself: loads return in order, so "vmcnt(n)" means all but the
// youngest n wave-loads of this wave have landed.
// lds_byte_off must be wave-uniform (it travels in M0); lane l's 16 bytes land at +16 l.
// M0 cannot be named as a clobber (the compiler reserves it and rejects it on clobber lists), so the
// kernels that use dma16 must not make the compiler use M0 itself: no dynamically indexed register
// arrays (v_movrel / s_set_gpr_idx), no LDS-direct reads, no GWS or message instructions.  Every
// array in these kernels is indexed at compile time (static_for, #pragma unroll); in the generated
// code of all four tile sizes every reference to M0 is one of the moves below.
__device__ __forceinline__ void dma16(const char* src, unsigned lds_byte_off) {
  // s_nop: the one wait state the ISA asks for between a write of M0 and an LDS-DMA that reads it
  // (the compiler's hazard pass does not look inside inline assembly)
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_byte_off) : "memory");
}
template <int N_>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_) : "memory");
}

// KB: k bytes per stage (64, 128 or 256)
template <int BM, int BN, int WM, int WN, int NSTAGE, bool W4, int KB>
struct DmaCfg {
  static constexpr int DBK = KB;
  static constexpr int CPR = KB / 16;                 // 16-byte chunks per int8 tile row (4 | 8 | 16)
  static constexpr int RPI = 64 / CPR;                // tile rows one wave-load covers (16 | 8 | 4)
  // swizzle: slot = chunk ^ ((row >> SH) & (CPR-1)); 2^SH rows share 256 bytes (one sweep of the banks)
  static constexpr int SH = CPR == 16 ? 0 : CPR == 8 ? 1 : 2;
  static constexpr int PCPR = KB / 32;                // 16-byte chunks per packed-int4 tile row (2 | 4 | 8)
  static constexpr int PRPI = 64 / PCPR;              // packed rows per wave-load (32 | 16 | 8)
  static constexpr int PSH = PCPR == 8 ? 1 : PCPR == 4 ? 2 : 3;
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
  static_assert(KB == 256 || KB == 128 || KB == 64, "k tile of 64, 128 or 256 bytes");
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
// the XOR swizzle the offset for substep s is this value with a compile-time constant XORed into its
// chunk bits, and rows 32 i further down add a multiple of the row pitch, which never reaches those bits.
//
// Which 16 k-values a lane's operand holds in substep s is free as long as both operands agree (a
// dot product does not care about the order of its terms).  int8 weights: the natural order, lane
// half g of substep s holds k = 32 s + 16 g ..., i.e. 16-byte chunk 2 s + g of both rows.
// Packed int4 weights: a 16-byte LDS chunk holds 32 k-values, and only whole chunks can be read without
// bank conflicts (64-bit reads of half chunks leave half of the banks idle and collide two-fold on
// the rest).  So a lane reads chunk 2 p + g of the W row ONCE per pair p of substeps and multiplies
// its low 8 bytes (k = 64 p + 32 g ...) in substep 2 p, its high 8 bytes (k = 64 p + 32 g + 16 ...) in
// substep 2 p + 1; the A operand follows: chunk 4 p + 2 g + h in substep 2 p + h.
template <class C, bool W4>
struct FragBase {
  unsigned a, b;
  __device__ __forceinline__ void init(int wm, int wn, int lane) {
    const int l31 = lane & 31, g = lane >> 5;
    const int ra = wm * C::TM + l31;
    const int ga = W4 ? g << 1 : g;
    a = (unsigned)(ra * C::DBK + ((ga ^ ((ra >> C::SH) & (C::CPR - 1))) << 4));
    const int rb = wn * C::TN + l31;
    if (!W4) b = (unsigned)(C::A_STAGE + rb * C::DBK + ((g ^ ((rb >> C::SH) & (C::CPR - 1))) << 4));
    else b = (unsigned)(C::A_STAGE + rb * (C::DBK / 2) + ((g ^ ((rb >> C::PSH) & (C::PCPR - 1))) << 4));
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

// W fragment as it sits in LDS: the MFMA operand itself (int8), or 32 packed nibbles that serve two
// substeps and are expanded right before use (kept packed meanwhile: no more registers than int8
// weights need, and the expansion never waits for a read issued a moment ago).
struct BRaw { v4i v; };
template <bool W4, int H>
__device__ __forceinline__ v4i b_operand(const BRaw& r) {
  if constexpr (!W4) {
    return r.v;
  } else {
    unsigned b0, b1, b2, b3;
    expand8((unsigned)(H ? r.v.z : r.v.x), b0, b1);
    expand8((unsigned)(H ? r.v.w : r.v.y), b2, b3);
    return v4i{(int)b0, (int)b1, (int)b2, (int)b3};
  }
}

// A fragments of k-substep S (32 k-values) of the stage at byte offset stage_off
template <class C, bool W4, int S>
__device__ __forceinline__ void load_a_frags(const char* lds, unsigned stage_off, const FragBase<C, W4>& fr,
                                             v4i (&fa)[C::FM]) {
  // chunk bits: 2 S + g (int8 weights) or 4 (S / 2) + 2 g + S % 2 (packed weights); g is in fr.a
  constexpr unsigned bits = W4 ? (unsigned)(((S >> 1) << 6) | ((S & 1) << 4)) : (unsigned)(S << 5);
  const char* pa = lds + xor_here<bits>(fr.a + stage_off);
#pragma unroll
  for (int i = 0; i < C::FM; ++i) fa[i] = *reinterpret_cast<const v4i*>(pa + i * 32 * C::DBK);
}
// LDS address of the lane's W fragments of k-substep S (packed rows: of the substep pair S / 2)
template <class C, bool W4, int S>
__device__ __forceinline__ const char* b_frag_ptr(const char* lds, unsigned stage_off, const FragBase<C, W4>& fr) {
  return lds + xor_here<(unsigned)(W4 ? (S >> 1) << 5 : S << 5)>(fr.b + stage_off);
}
template <class C, bool W4>
__device__ __forceinline__ void load_b_frag(const char* pb, int j, BRaw& fb) {
  fb.v = *reinterpret_cast<const v4i*>(pb + j * 32 * (W4 ? C::DBK / 2 : C::DBK));
}

// One k substep.  The operand reads of the FOLLOWING substep (S_NEXT of the stage at next_off) are
// dealt in between the MFMAs: its A fragments first, into the other half of a double buffer; its
// W fragment j into the registers of this substep's W fragment j as soon as the MFMAs that use
// that one have been issued (packed weights: only after the second substep of a pair, whose
// fragments serve both).  Every fragment is thus requested several MFMAs before its first
// use, with 32 instead of 48 registers of fragments.  Left to itself the scheduler sinks every
// read down to its first use, and a substep then starts by waiting out the LDS latency, hence
// the pinning.
// `request(r)` issues the wave's r-th global->LDS request of a k tile; NR of them are dealt out
// over the substep (NR = 0: none).  A wave that issues its requests back to back sits in the
// queue of the CU's one address unit (a 64 KiB k tile keeps it busy for about a thousand clocks)
// and, issuing in order, feeds no MFMAs meanwhile.
template <class C, bool W4, int S_NEXT, int NR, class Request>
__device__ __forceinline__ void k_substep(v16i (&acc)[C::FM][C::FN], const v4i (&fa)[C::FM],
                                          v4i (&fa_next)[C::FM], BRaw (&fb)[C::FN], const char* lds,
                                          unsigned next_off, const FragBase<C, W4>& fr, Request&& request) {
  constexpr int NM = C::FM * C::FN;
  constexpr int H = (S_NEXT & 1) ^ 1;            // this substep's half of a packed fragment
  constexpr bool RELOAD = !W4 || (S_NEXT & 1) == 0;  // the following substep starts a new pair
  load_a_frags<C, W4, S_NEXT>(lds, next_off, fr, fa_next);
  const char* pb = b_frag_ptr<C, W4, S_NEXT>(lds, next_off, fr);
  __builtin_amdgcn_sched_barrier(0);
  static_for<0, C::FN>([&](auto j_) {
    constexpr int j = decltype(j_)::value;
    const v4i b = b_operand<W4, H>(fb[j]);
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
    if constexpr (RELOAD) load_b_frag<C, W4>(pb, j, fb[j]);
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
                                                          int remap, int k_per_split) {
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
  const int G = (int)gridDim.x;
  int wg = (int)blockIdx.x;
  if (remap) wg = (wg & 7) * (G >> 3) + (wg >> 3);  // G % 8 == 0
  // Split along k (gridDim.y > 1): workgroup row y takes k in [y * k_per_split, ...) and leaves its
  // raw accumulators in plane y of ACC; the caller adds the planes up (integers: exact in any order).
  const int k_begin = (int)blockIdx.y * k_per_split;  // a multiple of the k tile; 0 without a split
  const int k_len = ((int)K - k_begin < k_per_split) ? (int)K - k_begin : k_per_split;
  if (gridDim.y > 1) {
    A += k_begin;
    Wv = reinterpret_cast<const char*>(Wv) + (W4 ? k_begin >> 1 : k_begin);
    ACC += (int64_t)blockIdx.y * M * N;
  }
  const int KT = (k_len + DBK - 1) / DBK;
  const int KTp = (KT + NSTAGE - 1) / NSTAGE * NSTAGE;

  const uint8_t* Wb = reinterpret_cast<const uint8_t*>(Wv);
  int tile = (wg / tiles_n) * chunk;  // row of tiles; < tiles_m: the grid is ceil(tiles_m / chunk) * tiles_n
  const int tile_end = tile + chunk < tiles_m ? tile + chunk : tiles_m;
  int64_t m0 = (int64_t)tile * BM;
  const int64_t n0 = (int64_t)(wg % tiles_n) * BN;
  DmaPlan<C, W4> plan;
  plan.init(A, Wb, M, N, K, m0, n0, wave, lane);
  int k_limit = k_len;  // 0 once there is no next tile: every further request fetches zeros
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
  BRaw fb[C::FN];
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

// Dynamic LDS above 64 KiB has to be allowed once per kernel and device (hipFuncSetAttribute, not a
// stream operation).  `done` is one flag word per device, a bit per kernel variant of the caller's
// instantiation; setting the attribute twice is harmless, so a relaxed flag is all the
// synchronisation two host threads racing through here need.
constexpr int kMaxDevices = 64;
inline int allow_lds(const void* kern, int bytes, std::atomic<unsigned>* done, int which) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
  if (done[dev].load(std::memory_order_relaxed) & (1u << which)) return MPQ_OK;
  hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) { set_last_hip_error((int)e); return MPQ_ERR_HIP; }
  done[dev].fetch_or(1u << which, std::memory_order_relaxed);
  return MPQ_OK;
}

// prepare_only: configure every kernel variant of this instantiation and launch nothing (mpq_init).
// split > 1: workgroup rows y = 0 .. split - 1 each take k_per_split of k (a multiple of the k tile)
// and write raw accumulators to plane y of acc_out (plain epilogue only).
template <int BM, int BN, int WM, int WN, int NSTAGE, bool W4, int KB = 128, int MINW = 1>
static int launch_dma(const int8_t* a_q, const void* w_q, int64_t M, int64_t N, int64_t K,
                      const float* a_scale, const float* w_scale, int per_row, float* y_out,
                      int32_t* acc_out, hipStream_t st, EpiArgs epi = kNoEpi,
                      int64_t* n_partials = nullptr, int split = 1, int k_per_split = 0,
                      bool prepare_only = false) {
  const float* y_ref = epi.yref;
  using C = DmaCfg<BM, BN, WM, WN, NSTAGE, W4, KB>;
  using Kern = void (*)(const int8_t*, const void*, int64_t, int64_t, int64_t, const float*, const float*, int,
                        float*, int32_t*, EpiArgs, int, int, int, int, int);
  static const Kern kerns[8] = {
      qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, false, KB, MINW, 0>, qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, true, KB, MINW, 0>,
      qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, false, KB, MINW, 1>, qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, true, KB, MINW, 1>,
      qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, false, KB, MINW, 2>, qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, true, KB, MINW, 2>,
      qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, false, KB, MINW, 3>, qgemm_dma<BM, BN, WM, WN, NSTAGE, W4, true, KB, MINW, 3>};
  static std::atomic<unsigned> done[kMaxDevices];
  if (prepare_only) {
    for (int w = 0; w < 8; ++w) {
      const int rc = allow_lds(reinterpret_cast<const void*>(kerns[w]), C::LDS_BYTES, done, w);
      if (rc != MPQ_OK) return rc;
    }
    return MPQ_OK;
  }
  // float4 / int4 stores need every 4-group of n inside the row and 16-byte aligned
  const bool vec = (N & 3) == 0 && (!y_out || aligned16(y_out)) && (!acc_out || aligned16(acc_out)) &&
                   (!((y_out || y_ref || epi.amax || epi.codes) && per_row) || aligned16(w_scale)) &&
                   (!y_ref || aligned16(y_ref)) && (!epi.codes || (reinterpret_cast<uintptr_t>(epi.codes) & 3u) == 0);
  const int mode = y_ref ? 1 : epi.codes ? 3 : (epi.act || epi.amax) ? 2 : 0;
  const int which = mode * 2 + (vec ? 1 : 0);
  const Kern kern = kerns[which];
  const int64_t tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
  if (tm * tn > 0x7FFFFFFF || tn > 0x7FFFFFFF) return MPQ_ERR_SHAPE;
  const int rc = allow_lds(reinterpret_cast<const void*>(kern), C::LDS_BYTES, done, which);
  if (rc != MPQ_OK) return rc;
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
    const int64_t cost = ((g * split + slots - 1) / slots) * c;
    if (c == 1 || cost <= best) { best = cost; chunk = c; grid = g; }
  }
  const int remap = (grid % 8 == 0 && grid >= 16) ? 1 : 0;
  if (split <= 1) { split = 1; k_per_split = (int)K; }
  kern<<<dim3((unsigned)grid, (unsigned)split), C::NT, C::LDS_BYTES, st>>>(a_q, w_q, M, N, K, a_scale, w_scale, per_row, y_out,
                                                                    acc_out, epi, (int)tn, (int)tm, chunk, remap, k_per_split);
  if (n_partials) *n_partials = grid;
  return launch_status();
}

// What a translation unit of one tile size exports: validation is the caller's business.
struct DmaArgs {
  const int8_t* a_q;
  const void* w_q;
  int64_t M, N, K;
  const float* a_scale;
  const float* w_scale;
  int per_row;
  float* y_out;
  int32_t* acc_out;
  hipStream_t st;
  EpiArgs epi;
  int64_t* n_partials;
  int split;         // > 1: split along k, raw accumulators to `split` planes of acc_out
  int k_per_split;
  bool prepare_only;  // configure the kernels of this tile size, launch nothing
};
int launch_dma_256(bool w4, const DmaArgs& a);
int launch_dma_192(bool w4, bool three_stages, const DmaArgs& a);
int launch_dma_128(bool w4, bool three_stages, const DmaArgs& a);
int launch_dma_64(bool w4, bool long_k, const DmaArgs& a);

}  // namespace mpq

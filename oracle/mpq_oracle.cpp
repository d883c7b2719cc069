// mpq_oracle.cpp -- plain CPU reference ("oracle") for the mixed-precision PTQ hot path.
//
// THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the smoke check and the
// benchmark's cpu_baseline leg may build, load or call it.  It shares no code, header, table
// generator or helper with the HIP library; every constant below is typed here from the
// published algorithm / the project's written recipe.
//
// Everything is written as the definition, one element at a time, in index order, with double
// precision wherever that makes the definition exact.  No blocking, no vectorisation, no threads.
//
// What each function follows (paper = "Mixed Precision Post Training Quantization of Neural
// Networks with Sensitivity Guided Search"):
//   orc_absmax          Sec. 3.1, calibration step: the maximum (absolute) value of each tensor.
//   orc_bit_constants   Sec. 3.1 Eq. 1 with alpha = 1/max, gamma = max, in the symmetric
//                       (2^(b-1) - 1)-level variant: scale = m/qmax, inv = qmax/m.
//   orc_fake_quant      Sec. 3.1 Eq. 1: round(clip(alpha x) * levels) / levels * gamma.
//   orc_quant_error     Sec. 3.2.1 Eq. 2: the expectation inside E_QE, as a sum of squares.
//   orc_eqe, orc_eqe_channels
//                       Sec. 3.2.1 Eq. 2 itself (one scale per tensor; one scale per channel).
//   orc_noise_inject    Sec. 3.2.2 Eq. 3-5: w_i + nu, nu Gaussian with spread tied to max|w_i|.
//   orc_qgemm           Alg. 1 / Alg. 2, evaluation step: one linear layer with both operands
//                       quantized; integer contraction, floating-point rescale.
//   orc_sse_pair        Alg. 1 / Alg. 2, the score the evaluation step keeps: stand-in, squared output error.
//   orc_fake_quant_scales, orc_scale_grad, orc_scale_sgd_step
//                       Sec. 3.1, adjustment step: Eq. 1 with its two scales as free parameters,
//                       their straight-through gradients, one gradient-descent step on them.
//   orc_rademacher, orc_hutchinson_quad
//                       Sec. 3.2.3: Hutchinson's estimate of the trace of the Hessian, for one
//                       linear layer under a mean-squared-error loss: random sign vectors and the
//                       quadratic forms v' H v they give.
//
// Parity status: every function here is pinned by tests (brute force, exact rational arithmetic,
// closed forms, invariants, published Philox known-answer vectors).  Nothing is "parity unpinned".

#include <cfenv>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

#if defined(__FAST_MATH__)
#error "the oracle must not be built with fast-math"
#endif

extern "C" {

enum { ORC_PER_TENSOR = 0, ORC_PER_ROW = 1, ORC_PER_COL = 2 };
enum { ORC_OK = 0, ORC_BAD_ARG = 1, ORC_ACC_OVERFLOW = 2 };

// ------------------------------------------------------------------------------------------
// channel bookkeeping: which absmax entry governs element (r, c)
static inline int64_t channel_of(int gran, int64_t r, int64_t c) {
  if (gran == ORC_PER_ROW) return r;
  if (gran == ORC_PER_COL) return c;
  return 0;
}
static inline int64_t channel_count(int gran, int64_t rows, int64_t cols) {
  if (gran == ORC_PER_ROW) return rows;
  if (gran == ORC_PER_COL) return cols;
  return 1;
}

// ------------------------------------------------------------------------------------------
// Sec. 3.1 calibration: m = max |x| over the tensor, each row, or each column.
// accumulate != 0 keeps a running maximum over successive calibration batches.
int orc_absmax(const float* x, int64_t rows, int64_t cols, int gran, int accumulate, float* out) {
  if (!x || !out || rows <= 0 || cols <= 0 || gran < 0 || gran > 2) return ORC_BAD_ARG;
  const int64_t nch = channel_count(gran, rows, cols);
  if (!accumulate)
    for (int64_t ch = 0; ch < nch; ++ch) out[ch] = 0.0f;
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      const float a = std::fabs(x[r * cols + c]);
      float& m = out[channel_of(gran, r, c)];
      if (a > m) m = a;
    }
  return ORC_OK;
}

// ------------------------------------------------------------------------------------------
// Eq. 1 constants.  Levels on each side: qmax = 2^(b-1) - 1.  gamma/levels -> scale = m / qmax,
// alpha*levels -> inv = qmax / m; each is ONE correctly rounded fp32 division.  m == 0 gives 0, 0.
int orc_qmax(int bits) { return (1 << (bits - 1)) - 1; }

void orc_bit_constants(float m, int bits, float* scale, float* inv) {
  const float qmax = (float)orc_qmax(bits);
  if (m > 0.0f) {
    volatile float s = m / qmax;   // volatile: keep the compiler from widening the division
    volatile float i = qmax / m;
    *scale = s;
    *inv = i;
  } else {
    *scale = 0.0f;
    *inv = 0.0f;
  }
}

void orc_scale_from_absmax(const float* absmax, int64_t count, int bits, float* scale_out) {
  for (int64_t i = 0; i < count; ++i) {
    float s, inv;
    orc_bit_constants(absmax[i], bits, &s, &inv);
    scale_out[i] = s;
  }
}

// Eq. 1, integer code of one value: round-half-to-even of the exact real product x * inv,
// then clip to +-qmax.  The product of two fp32 numbers is exact in double (24+24 <= 53 bits).
static inline int code_of(float x, float inv, int qmax) {
  const double p = (double)x * (double)inv;
  double q = std::nearbyint(p);  // rounding mode is round-to-nearest-even (checked by the caller)
  if (q > (double)qmax) q = (double)qmax;
  if (q < -(double)qmax) q = -(double)qmax;
  return (int)q;
}
// Eq. 1, dequantized value: code * scale, one fp32 multiplication.
static inline float dequant_of(int q, float scale) {
  volatile float y = (float)q * scale;
  return y;
}

// two's-complement nibble pair: low nibble = even column, high nibble = odd column
static inline uint8_t pack_pair(int q_even, int q_odd) {
  return (uint8_t)((q_even & 0xF) | ((q_odd & 0xF) << 4));
}
static inline int nibble_lo(uint8_t b) { int v = b & 0xF; return v >= 8 ? v - 16 : v; }
static inline int nibble_hi(uint8_t b) { int v = (b >> 4) & 0xF; return v >= 8 ? v - 16 : v; }

void orc_pack4(const int8_t* codes, int64_t n_pairs, uint8_t* packed) {
  for (int64_t i = 0; i < n_pairs; ++i) packed[i] = pack_pair(codes[2 * i], codes[2 * i + 1]);
}
void orc_unpack4(const uint8_t* packed, int64_t n_pairs, int8_t* codes) {
  for (int64_t i = 0; i < n_pairs; ++i) {
    codes[2 * i] = (int8_t)nibble_lo(packed[i]);
    codes[2 * i + 1] = (int8_t)nibble_hi(packed[i]);
  }
}

// ------------------------------------------------------------------------------------------
// Eq. 1 over a tensor.  Any of y / codes / packed4 may be null.  packed4 needs bits <= 4 and an
// even number of columns (pairs never straddle a row).
int orc_fake_quant(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax,
                   int bits, float* y, int8_t* codes, uint8_t* packed4) {
  if (!x || !absmax || rows <= 0 || cols <= 0 || gran < 0 || gran > 2) return ORC_BAD_ARG;
  if (bits < 2 || bits > 8) return ORC_BAD_ARG;
  if (packed4 && (bits > 4 || (cols & 1))) return ORC_BAD_ARG;
  if (std::fegetround() != FE_TONEAREST) return ORC_BAD_ARG;
  const int qmax = orc_qmax(bits);
  const int64_t nch = channel_count(gran, rows, cols);
  std::vector<float> scale(nch), inv(nch);  // per-channel constants, computed once
  for (int64_t ch = 0; ch < nch; ++ch) orc_bit_constants(absmax[ch], bits, &scale[ch], &inv[ch]);
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      const int64_t ch = channel_of(gran, r, c);
      const int64_t i = r * cols + c;
      const int q = code_of(x[i], inv[ch], qmax);
      if (y) y[i] = dequant_of(q, scale[ch]);
      if (codes) codes[i] = (int8_t)q;
      if (packed4) {
        if ((c & 1) == 0) packed4[i >> 1] = (uint8_t)(q & 0xF);
        else packed4[i >> 1] = (uint8_t)(packed4[i >> 1] | ((q & 0xF) << 4));
      }
    }
  return ORC_OK;
}

// ------------------------------------------------------------------------------------------
// Eq. 2, the sum under the expectation: SSE_b = sum (Q_b(x) - x)^2 for every b in b_lo..b_hi,
// per tensor or per channel, accumulated in double in index order.  Q_b(x) = code * scale_b is
// taken exactly (the fp32 constants scale_b, inv_b are the only roundings in the definition).
// sse is [nch][nb], channel-major, b ascending.
int orc_quant_error(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax,
                    int b_lo, int b_hi, double* sse) {
  if (!x || !absmax || !sse || rows <= 0 || cols <= 0 || gran < 0 || gran > 2) return ORC_BAD_ARG;
  if (b_lo < 2 || b_hi > 8 || b_lo > b_hi) return ORC_BAD_ARG;
  if (std::fegetround() != FE_TONEAREST) return ORC_BAD_ARG;
  const int nb = b_hi - b_lo + 1;
  const int64_t nch = channel_count(gran, rows, cols);
  for (int64_t k = 0; k < nch * nb; ++k) sse[k] = 0.0;
  std::vector<float> scale(nch * nb), inv(nch * nb);  // per-(channel, b) constants, computed once
  for (int64_t ch = 0; ch < nch; ++ch)
    for (int b = b_lo; b <= b_hi; ++b)
      orc_bit_constants(absmax[ch], b, &scale[ch * nb + (b - b_lo)], &inv[ch * nb + (b - b_lo)]);
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      const int64_t ch = channel_of(gran, r, c);
      const float xv = x[r * cols + c];
      for (int b = b_lo; b <= b_hi; ++b) {
        const int64_t kb = ch * nb + (b - b_lo);
        // Eq. 2 is stated over the reals: Q(x) here is the grid point code * scale_b itself
        // (exact in double: 8 x 24 significant bits), not its rounding to fp32.
        const double qx = (double)code_of(xv, inv[kb], orc_qmax(b)) * (double)scale[kb];
        const double e = qx - (double)xv;
        sse[ch * nb + (b - b_lo)] += e * e;
      }
    }
  return ORC_OK;
}

// Eq. 2: E_QE = sqrt(mean squared error) / max|x|.
double orc_eqe(double sse, int64_t n, float absmax) {
  if (n <= 0 || !(absmax > 0.0f)) return 0.0;
  return std::sqrt(sse / (double)n) / (double)absmax;
}

// Eq. 2 for a tensor quantized with one scale per channel: the expectation runs over all n elements
// of the tensor, so the channels' error sums add up, and max|x| of the tensor is the largest
// channel maximum.  sse: [nch][nb] (b ascending), absmax: [nch]; out: [nb].
void orc_eqe_channels(const double* sse, const float* absmax, int64_t nch, int nb, int64_t n, double* out) {
  float m = 0.0f;
  for (int64_t c = 0; c < nch; ++c) m = absmax[c] > m ? absmax[c] : m;
  for (int b = 0; b < nb; ++b) {
    double total = 0.0;
    for (int64_t c = 0; c < nch; ++c) total += sse[c * nb + b];
    out[b] = orc_eqe(total, n, m);
  }
}

// ------------------------------------------------------------------------------------------
// Philox-4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
// SC'11).  Ten rounds; the key is bumped by the Weyl constants between rounds.
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// --- fp32 building blocks of the Gaussian transform.  Every operation is a single IEEE fp32
// operation (multiply, fused multiply-add, square root); volatile stores stop the compiler from
// keeping wider intermediates or contracting anything on its own.
static inline float f32_mul(float a, float b) { volatile float r = a * b; return r; }
static inline float f32_fma(float a, float b, float c) { volatile float r = std::fmaf(a, b, c); return r; }
static inline float f32_sqrt(float a) { volatile float r = std::sqrt(a); return r; }

// L(k) = -2 ln(k * 2^-24) for integer 1 <= k <= 2^24.
//   (float)k = 2^e * m, m in [1,2); if the mantissa field exceeds 0x3504F3 (m > sqrt 2) halve m
//   and bump e, so m in (0.7071, 1.4142];  t = m - 1 (exact);
//   -2 ln m = t * R(t), R a degree-9 polynomial (Horner, fused);  L = fma(24 - e, 2 ln 2, t R(t)).
float orc_neg2log_u24(uint32_t k) {
  static const float R[10] = {-0x1.000000p+1f, 0x1.fffff8p-1f, -0x1.555540p-1f, 0x1.00041ep-1f,
                              -0x1.99aa6ap-2f, 0x1.542e08p-2f, -0x1.2202fap-2f, 0x1.0e9656p-2f,
                              -0x1.0aa1c6p-2f, 0x1.40bfc2p-3f};
  const float fk = (float)k;  // exact, k <= 2^24
  uint32_t bits;
  std::memcpy(&bits, &fk, 4);
  int e = (int)(bits >> 23) - 127;
  uint32_t mant = bits & 0x007FFFFFu;
  uint32_t mbits = mant | 0x3F800000u;      // m in [1, 2)
  if (mant > 0x003504F3u) { mbits = mant | 0x3F000000u; e += 1; }  // m/2 in (0.707, 1)
  float m;
  std::memcpy(&m, &mbits, 4);
  const float t = m - 1.0f;  // exact
  float r = R[9];
  for (int i = 8; i >= 0; --i) r = f32_fma(r, t, R[i]);
  const float q = f32_mul(t, r);
  return f32_fma((float)(24 - e), 0x1.62e430p+0f /* 2 ln 2 */, q);
}

// cos and sin of 2 pi j 2^-24 for integer 0 <= j < 2^24.
//   quadrant qd = (j + 2^21) >> 22 (nearest quarter turn, 0..4); y = (j - qd 2^22) 2^-24 in
//   [-1/8, 1/8) turns (exact);  v = y*y;  s = y * S(v), c = C(v) (Horner, fused);
//   rotate by qd quarter turns with exact sign flips / swaps.
void orc_sincos_2pi_u24(uint32_t j, float* cos_out, float* sin_out) {
  static const float S[4] = {0x1.921fb6p+2f, -0x1.4abbbap+5f, 0x1.465ec6p+6f, -0x1.2d9bb8p+6f};
  static const float C[5] = {0x1.000000p+0f, -0x1.3bd3ccp+4f, 0x1.03c1dcp+6f, -0x1.55c57cp+6f,
                             0x1.d9c364p+5f};
  const uint32_t qd = (j + (1u << 21)) >> 22;
  const int32_t jr = (int32_t)j - (int32_t)(qd << 22);
  const float y = (float)jr * 0x1.0p-24f;  // exact
  const float v = f32_mul(y, y);
  float sp = S[3];
  for (int i = 2; i >= 0; --i) sp = f32_fma(sp, v, S[i]);
  const float s = f32_mul(y, sp);
  float c = C[4];
  for (int i = 3; i >= 0; --i) c = f32_fma(c, v, C[i]);
  switch (qd & 3u) {
    case 0: *cos_out = c;  *sin_out = s;  break;
    case 1: *cos_out = -s; *sin_out = c;  break;
    case 2: *cos_out = -c; *sin_out = -s; break;
    default: *cos_out = s; *sin_out = -c; break;
  }
}

// Four standard normals for elements 4g .. 4g+3 of stream `stream_id` under `seed`:
// Philox counter = (g lo, g hi, stream lo, stream hi), key = (seed lo, seed hi);
// Box-Muller on the word pairs (w0,w1) and (w2,w3):
//   u1 = ((wa >> 8) + 1) 2^-24 in (0,1],  u2 = (wb >> 8) 2^-24 in [0,1),
//   r = sqrt(-2 ln u1),  z_even = r cos(2 pi u2),  z_odd = r sin(2 pi u2).
void orc_gauss4(uint64_t seed, uint64_t stream_id, uint64_t g, float z[4]) {
  const uint32_t ctr[4] = {(uint32_t)g, (uint32_t)(g >> 32), (uint32_t)stream_id,
                           (uint32_t)(stream_id >> 32)};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  orc_philox4x32_10(ctr, key, w);
  for (int pair = 0; pair < 2; ++pair) {
    const float r = f32_sqrt(orc_neg2log_u24((w[2 * pair] >> 8) + 1u));
    float c, s;
    orc_sincos_2pi_u24(w[2 * pair + 1] >> 8, &c, &s);
    z[2 * pair] = f32_mul(r, c);
    z[2 * pair + 1] = f32_mul(r, s);
  }
}

// Eq. 3-5: y_i = x_i + sigma * z_i with sigma = lambda * scale_b (standard deviation equal to
// lambda quantization steps of the b-bit grid); element index i = r*cols + c in row-major order.
int orc_noise_inject(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax,
                     int bits, float lambda, uint64_t seed, uint64_t stream_id, float* y) {
  if (!x || !absmax || !y || rows <= 0 || cols <= 0 || gran < 0 || gran > 2) return ORC_BAD_ARG;
  if (bits < 2 || bits > 8) return ORC_BAD_ARG;
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      const int64_t i = r * cols + c;
      float scale, inv, z[4];
      orc_bit_constants(absmax[channel_of(gran, r, c)], bits, &scale, &inv);
      const float sigma = f32_mul(lambda, scale);  // standard deviation of the injected noise
      orc_gauss4(seed, stream_id, (uint64_t)i >> 2, z);
      y[i] = f32_fma(sigma, z[i & 3], x[i]);
    }
  return ORC_OK;
}

// ------------------------------------------------------------------------------------------
// One quantized linear layer: acc[m][n] = sum_k A_q[m][k] * W_q[n][k] in int32 (checked against
// the int64 sum); Y[m][n] = (float(acc) * s_A) * s_W[n], two fp32 multiplications in that order.
// W is [N x K] int8, or [N x K/2] nibble pairs when w_storage_bits == 4.
int orc_qgemm(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
              int64_t K, const float* a_scale, const float* w_scale, int w_gran, float* y,
              int32_t* acc_out) {
  if (!a_q || !w_q || M <= 0 || N <= 0 || K <= 0) return ORC_BAD_ARG;
  if (w_storage_bits != 8 && w_storage_bits != 4) return ORC_BAD_ARG;
  if (w_storage_bits == 4 && (K & 1)) return ORC_BAD_ARG;
  if (y && (!a_scale || !w_scale)) return ORC_BAD_ARG;
  if (w_gran != ORC_PER_TENSOR && w_gran != ORC_PER_ROW) return ORC_BAD_ARG;
  const int8_t* w8 = (const int8_t*)w_q;
  const uint8_t* w4 = (const uint8_t*)w_q;
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      int32_t acc = 0;
      int64_t wide = 0;
      for (int64_t k = 0; k < K; ++k) {
        const int a = a_q[m * K + k];
        int w;
        if (w_storage_bits == 8) w = w8[n * K + k];
        else {
          const uint8_t byte = w4[n * (K / 2) + (k >> 1)];
          w = (k & 1) ? nibble_hi(byte) : nibble_lo(byte);
        }
        acc = (int32_t)((uint32_t)acc + (uint32_t)(a * w));  // wraps like the hardware would
        wide += (int64_t)a * (int64_t)w;
      }
      if ((int64_t)acc != wide) return ORC_ACC_OVERFLOW;
      if (acc_out) acc_out[m * N + n] = acc;
      if (y) {
        const float sw = w_scale[w_gran == ORC_PER_ROW ? n : 0];
        y[m * N + n] = f32_mul(f32_mul((float)acc, a_scale[0]), sw);
      }
    }
  return ORC_OK;
}

// Activations a layer may be followed by inside the evaluation step: ReLU, or GELU(x) = x Phi(x)
// with the exact Gaussian distribution function, evaluated in double and rounded to fp32 once.
// act: 0 none, 1 ReLU, 2 GELU.  In place.
int orc_activation(float* y, int64_t n, int act) {
  if (!y || n <= 0 || act < 0 || act > 2) return ORC_BAD_ARG;
  for (int64_t i = 0; i < n; ++i) {
    const double x = (double)y[i];
    if (act == 1) y[i] = x > 0.0 ? y[i] : 0.0f;
    else if (act == 2) y[i] = (float)(0.5 * x * std::erfc(-x / std::sqrt(2.0)));
  }
  return ORC_OK;
}

// Squared distance between two tensors, in double, index order.
double orc_sse_pair(const float* y, const float* y_ref, int64_t n) {
  double s = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    const double d = (double)y[i] - (double)y_ref[i];
    s += d * d;
  }
  return s;
}

// ------------------------------------------------------------------------------------------
// Sec. 3.2.3, E_Hessian = E[Tr(d^2 L / d w_i^2)], the trace estimated with Hutchinson's algorithm:
// Tr(H) = E_v[v' H v] for random v with independent zero-mean unit-variance entries; the usual
// choice, taken here, is random signs.
//
// The one case with no network behind it: a linear layer Y = X W' (X [M x K], W [N x K]) under
// L = mean over the M N outputs of (Y - T)^2.  L is quadratic in W; its Hessian with respect to
// vec(W) is (2 / (M N)) (I_N (x) X'X), whatever W and T are.  For a probe V [N x K] that is
// v' H v = (2 / (M N)) sum_n || X v_n ||^2: every row of V is one K-vector v_n that meets the same
// block X'X, so probes are drawn as a list of K-vectors and
//     Tr(H) ~= (2 / (M N)) * N * mean_p || X v_p ||^2 = (2 / M) mean_p || X v_p ||^2,
// against the exact Tr(H) = (2 / M) ||X||_F^2.  (With respect to X instead, the roles swap:
// quadratic forms of W, trace (2 / N) ||W||_F^2.)
//
// Random signs: element e = r * cols + c of the [rows x cols] sign matrix is decided by bit
// (e mod 128) of the Philox-4x32-10 block with counter (e / 128 lo, hi, stream lo, stream hi) and
// key (seed lo, seed hi XOR 0x5241444D): bit t sits in word t / 32 at position t mod 32; a set
// bit gives -1, a clear bit +1.  (The constant keeps these draws apart from the Gaussian stream
// of the same seed and stream id.)
int orc_rademacher(uint64_t seed, uint64_t stream_id, int64_t rows, int64_t cols, float* v) {
  if (!v || rows <= 0 || cols <= 0) return ORC_BAD_ARG;
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32) ^ 0x5241444Du};
  for (int64_t e = 0; e < rows * cols; ++e) {
    const uint64_t g = (uint64_t)e >> 7;
    const uint32_t ctr[4] = {(uint32_t)g, (uint32_t)(g >> 32), (uint32_t)stream_id, (uint32_t)(stream_id >> 32)};
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    const unsigned t = (unsigned)(e & 127);
    v[e] = ((w[t >> 5] >> (t & 31u)) & 1u) ? -1.0f : 1.0f;
  }
  return ORC_OK;
}

// quad[p] = || X v_p ||^2 = sum_m (sum_k X[m][k] v[p][k])^2, in double, index order.
int orc_hutchinson_quad(const float* x, int64_t M, int64_t K, const float* v, int64_t P, double* quad) {
  if (!x || !v || !quad || M <= 0 || K <= 0 || P <= 0) return ORC_BAD_ARG;
  for (int64_t p = 0; p < P; ++p) {
    double q = 0.0;
    for (int64_t m = 0; m < M; ++m) {
      double s = 0.0;
      for (int64_t k = 0; k < K; ++k) s += (double)x[m * K + k] * (double)v[p * K + k];
      q += s * s;
    }
    quad[p] = q;
  }
  return ORC_OK;
}

// ------------------------------------------------------------------------------------------
// Sec. 3.1, second step ("adjustment"): after calibration the two scales of Eq. 1 are free
// parameters, here as the pair the integer form works with: inv (= alpha * levels, applied
// before rounding) and scale (= gamma / levels, applied after).
//
// Forward with explicit scales: code = clamp(RNE(x * inv), +-qmax) on the exact product,
// Q = fl32(code * scale).
int orc_fake_quant_scales(const float* x, int64_t rows, int64_t cols, int gran, const float* inv,
                          const float* scale, int bits, float* y, int8_t* codes) {
  if (!x || !inv || !scale || rows <= 0 || cols <= 0 || gran < 0 || gran > 1) return ORC_BAD_ARG;
  if (bits < 2 || bits > 8) return ORC_BAD_ARG;
  if (std::fegetround() != FE_TONEAREST) return ORC_BAD_ARG;
  const int qmax = orc_qmax(bits);
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      const int64_t ch = channel_of(gran, r, c), i = r * cols + c;
      const int q = code_of(x[i], inv[ch], qmax);
      if (y) y[i] = dequant_of(q, scale[ch]);
      if (codes) codes[i] = (int8_t)q;
    }
  return ORC_OK;
}

// Gradients of a loss L with respect to the two scales, rounding treated as the identity
// (straight-through): with g_i = dL/dQ_i,
//   dL/dscale = sum_i g_i * code_i                       (Q is linear in scale: exact)
//   dL/dinv   = scale * sum_{i not clipped} g_i * x_i    (d clip(u)/du = 1 where the clamp of the
//               rounded value is inactive, |RNE(x inv)| <= qmax, else 0)
// g == null selects the reconstruction loss L = sum (Q - x)^2 with Q = code * scale taken exactly,
// g_i = 2 (Q_i - x_i).  loss is that sum of squares in either case.  abs_* (nullable) receive the
// sums of the absolute values of the terms, the natural yardstick for an error bound.
// All outputs are per channel, accumulated in double in index order.
int orc_scale_grad(const float* x, int64_t rows, int64_t cols, int gran, const float* inv,
                   const float* scale, int bits, const float* g, double* dinv, double* dscale,
                   double* loss, double* abs_dinv, double* abs_dscale) {
  if (!x || !inv || !scale || !dinv || !dscale || rows <= 0 || cols <= 0 || gran < 0 || gran > 1)
    return ORC_BAD_ARG;
  if (bits < 2 || bits > 8) return ORC_BAD_ARG;
  if (std::fegetround() != FE_TONEAREST) return ORC_BAD_ARG;
  const int qmax = orc_qmax(bits);
  const int64_t nch = channel_count(gran, rows, cols);
  std::vector<double> sx(nch, 0.0), sq(nch, 0.0), sl(nch, 0.0), ax(nch, 0.0), aq(nch, 0.0);
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      const int64_t ch = channel_of(gran, r, c), i = r * cols + c;
      const double rounded = std::nearbyint((double)x[i] * (double)inv[ch]);
      const bool clipped = std::fabs(rounded) > (double)qmax;
      const int q = code_of(x[i], inv[ch], qmax);
      const double e = (double)q * (double)scale[ch] - (double)x[i];
      const double gi = g ? (double)g[i] : 2.0 * e;
      sq[ch] += gi * (double)q;
      aq[ch] += std::fabs(gi * (double)q);
      if (!clipped) {
        sx[ch] += gi * (double)x[i];
        ax[ch] += std::fabs(gi * (double)x[i]);
      }
      sl[ch] += e * e;
    }
  for (int64_t ch = 0; ch < nch; ++ch) {
    dscale[ch] = sq[ch];
    dinv[ch] = (double)scale[ch] * sx[ch];
    if (loss) loss[ch] = sl[ch];
    if (abs_dscale) abs_dscale[ch] = aq[ch];
    if (abs_dinv) abs_dinv[ch] = std::fabs((double)scale[ch]) * ax[ch];
  }
  return ORC_OK;
}

// One step of plain gradient descent on the scales only (the model's parameters stay as they
// are): p <- fl32(p - lr * dL/dp), formed in double and rounded once.
int orc_scale_sgd_step(float* inv, float* scale, const double* dinv, const double* dscale,
                       int64_t count, double lr) {
  if (!inv || !scale || !dinv || !dscale || count <= 0) return ORC_BAD_ARG;
  for (int64_t i = 0; i < count; ++i) {
    inv[i] = (float)((double)inv[i] - lr * dinv[i]);
    scale[i] = (float)((double)scale[i] - lr * dscale[i]);
  }
  return ORC_OK;
}

}  // extern "C"

/* mpq.h -- C ABI of libmpq: the data-parallel inner loop of sensitivity-guided mixed-precision
 * post-training quantization, for AMD Instinct MI355X (gfx950).
 *
 * Paper: "Mixed Precision Post Training Quantization of Neural Networks with Sensitivity Guided
 * Search".  The calls below are the per-tensor operations its searches (Alg. 1 bisection, Alg. 2
 * greedy) and sensitivity metrics (Sec. 3.2) execute over and over: max calibration (Sec. 3.1),
 * the quantizer of Eq. 1, the error sum inside Eq. 2, the perturbation of Eq. 3-5, and the
 * quantized linear layer that the evaluation step of both algorithms runs.
 *
 * Conventions common to every call
 *  - All data pointers are DEVICE pointers (HIP global memory) unless a comment says "host".
 *    Scalars (sizes, bits, lambda, seed) are host values.  `stream` is a hipStream_t passed as
 *    void* (NULL = the default stream).
 *  - Calls only enqueue work on `stream`; they never synchronise, never copy device<->host and
 *    never allocate.  Results (absmax, error sums) stay on the device.  The caller owns every
 *    buffer; scratch comes from the caller's workspace `ws` of `ws_bytes` bytes, whose required
 *    size is returned by the matching mpq_*_workspace_bytes() (a pure host function).  The
 *    workspace needs no initialisation, must be 16-byte aligned, and must not be shared by calls
 *    that may run concurrently.
 *  - Tensors are dense row-major 2-D [rows x cols] fp32.  `gran` selects the quantization
 *    granularity: one scale per tensor, per row, or per column.  Linear-layer weights are stored
 *    [N x K] (out x in, K contiguous), so "per output channel" is MPQ_PER_ROW.
 *  - Quantizer (Eq. 1 in its symmetric integer form): qmax_b = 2^(b-1) - 1,
 *    scale_b = fl32(m / qmax_b), inv_b = fl32(qmax_b / m) with m the channel's absmax (both 0
 *    when m == 0); code = clamp(RNE(x * inv_b), +-qmax_b) where the product is the exact real
 *    product and RNE is round-half-to-even; Q(x) = fl32(code * scale_b).
 *  - Inputs must be finite; NaN/Inf give unspecified values (never a fault).
 *  - Return value: MPQ_OK or an error code below.  Argument errors are detected on the host
 *    before anything is launched, so a failing call has no effect on the device.
 */
#ifndef MPQ_H_
#define MPQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum mpq_status {
  MPQ_OK = 0,
  MPQ_ERR_NULL = 1,      /* a required pointer is NULL */
  MPQ_ERR_SHAPE = 2,     /* dims <= 0, rows*cols overflow, odd cols/K with packed int4, ... */
  MPQ_ERR_BITS = 3,      /* bit-width outside 2..8, storage bits not 4 or 8, bad range */
  MPQ_ERR_ALIGN = 4,     /* a pointer lacks the alignment stated for it */
  MPQ_ERR_WORKSPACE = 5, /* ws is NULL or ws_bytes too small */
  MPQ_ERR_GRAN = 6,      /* granularity value not valid for this call */
  MPQ_ERR_HIP = 7,       /* the HIP runtime refused a launch; see mpq_last_hip_error() */
  MPQ_ERR_TOO_LARGE = 8  /* the input needs more scratch than a built-in buffer of fixed size holds */
};

enum mpq_gran { MPQ_PER_TENSOR = 0, MPQ_PER_ROW = 1, MPQ_PER_COL = 2 };

/* Text for a status code (static storage, host). */
const char* mpq_strerror(int status);
/* Raw hipError_t of the most recent MPQ_ERR_HIP on the calling thread (0 if none). */
int mpq_last_hip_error(void);
/* Library version, major*100 + minor. */
int mpq_version(void);
/* Optional.  Configures, on the caller's current device, every kernel variant of the quantized-layer
 * calls that needs more than the default amount of on-chip memory (a per-kernel runtime attribute,
 * not a stream operation).  Without it the first call that selects a variant does the same for
 * that variant; code that records the calls into a HIP graph calls mpq_init() before the capture
 * begins, or runs each call once eagerly first.  Thread safe, idempotent, allocates nothing. */
int mpq_init(void);

/* ---- Sec. 3.1, calibration step: m = max |x| --------------------------------------------
 * x          [rows x cols] fp32, any alignment (16-byte alignment enables 128-bit loads).
 * gran       PER_TENSOR -> absmax_out[1]; PER_ROW -> [rows]; PER_COL -> [cols].
 * accumulate 0: absmax_out is overwritten; 1: absmax_out = max(absmax_out, new), the running
 *            maximum over successive calibration batches (absmax_out must then hold valid
 *            non-negative values).
 * Workspace: needed for PER_TENSOR only (one partial maximum per workgroup); the query returns 0
 * for the other granularities and ws may then be NULL.
 * The result is exact (max is order independent). */
size_t mpq_calibrate_absmax_workspace_bytes(int64_t rows, int64_t cols, int gran);
int mpq_calibrate_absmax(const float* x, int64_t rows, int64_t cols, int gran, int accumulate,
                         float* absmax_out, void* ws, size_t ws_bytes, void* stream);

/* scale_out[i] = fl32(absmax[i] / qmax_bits) (0 when absmax[i] == 0), i < count: the step size
 * of Eq. 1 that mpq_qgemm takes as a_scale / w_scale. */
int mpq_scale_from_absmax(const float* absmax, int64_t count, int bits, float* scale_out,
                          void* stream);

/* ---- Sec. 3.1 Eq. 1: b-bit fake quantization ----------------------------------------------
 * absmax     [1] | [rows] | [cols] according to gran (need not come from the same tensor;
 *            values beyond it saturate at +-qmax).
 * bits       2..8.
 * y_out      nullable: Q(x), fp32 [rows x cols].
 * codes_out  nullable: integer codes, one int8 per element, [rows x cols].
 * packed4_out nullable: bits <= 4 only, cols even: two's-complement nibbles, two per byte along
 *            cols, LOW nibble = even column, HIGH nibble = odd column; [rows x cols/2] bytes.
 * At least one output must be given.  No workspace. */
int mpq_fake_quant(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax,
                   int bits, float* y_out, int8_t* codes_out, uint8_t* packed4_out, void* stream);
/* Per-tensor mpq_fake_quant that also leaves the step size scale_b = absmax / qmax_b in step_out[0]
 * (device float[1], required): what mpq_scale_from_absmax(absmax, 1, bits) computes, without a
 * launch of its own for one division.  Other arguments and errors as mpq_fake_quant. */
int mpq_fake_quant_step(const float* x, int64_t rows, int64_t cols, const float* absmax, int bits,
                        float* y_out, int8_t* codes_out, uint8_t* packed4_out, float* step_out,
                        void* stream);


/* ---- Sec. 3.2.1 Eq. 2: quantization-error sums for b = b_lo..b_hi in ONE read of x -----------
 * sse_out    double [nch x nb], channel-major, b ascending; nch = 1 | rows | cols, nb =
 *            b_hi - b_lo + 1.  sse_out[ch][b] = sum over the channel of (Q_b(x) - x)^2.
 *            E_QE(b) = sqrt(sse / n) / absmax is left to the host (Eq. 2).
 * 2 <= b_lo <= b_hi <= 8.  Per-lane partial sums are fp32, combined in double in a fixed order:
 * results are reproducible run to run and agree with a double-precision sum to ~1e-6 relative. */
size_t mpq_quant_error_workspace_bytes(int64_t rows, int64_t cols, int gran, int b_lo, int b_hi);
int mpq_quant_error(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax,
                    int b_lo, int b_hi, double* sse_out, void* ws, size_t ws_bytes, void* stream);

/* Eq. 2 itself, from the sums above (HOST functions on HOST values; the caller has read the sums back):
 *   mpq_eqe          E_QE = sqrt(sse / n) / absmax, n the number of elements the sum ran over;
 *                    0 when absmax == 0 (an all-zero tensor has no error) or n <= 0.
 *   mpq_eqe_channels the same for a tensor quantized with one scale per channel, from its channels'
 *                    sums sse[nch][nb] (what mpq_quant_error writes per row / column) and maxima
 *                    absmax[nch]: the expectation of Eq. 2 runs over all n elements of the tensor, so
 *                    eqe_out[b] = sqrt(sum_c sse[c][b] / n) / max_c absmax[c], b < nb. */
double mpq_eqe(double sse, int64_t n, double absmax);
int mpq_eqe_channels(const double* sse, const float* absmax, int64_t nch, int nb, int64_t n, double* eqe_out);

/* mpq_quant_error for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (minus the workspace), same kernels and bit-for-bit the same results as
 * mpq_quant_error; the partial sums go to a buffer of MPQ_NOALLOC_SCRATCH_BYTES that is part of the
 * library's device image (each GPU the library runs on holds one copy until the process ends).
 * The call allocates nothing and calls no allocating routine; on the first call on a device it
 * looks up that device's address of the buffer (one symbol query, cached), with the caller's
 * current device.  Inputs whose partial sums do not fit -- mpq_quant_error_workspace_bytes(...) >
 * MPQ_NOALLOC_SCRATCH_BYTES (4 MiB), which only happens for MPQ_PER_COL (from about 1500 columns
 * on) or rows longer than 16384 columns on large tensors; the per-tensor sweep of any size needs at
 * most 56 KiB and the per-row sweep of rows up to 16384 columns none -- are rejected with
 * MPQ_ERR_TOO_LARGE before anything is launched.  All calls on one GPU share the one buffer:
 * calls that may run concurrently on the same GPU (different streams, different host threads)
 * race on it and must be serialised by the caller; calls in stream order are safe. */
#define MPQ_NOALLOC_SCRATCH_BYTES ((size_t)4 << 20)
int mpq_quant_error_noalloc(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax,
                            int b_lo, int b_hi, double* sse_out, void* stream);

/* ---- Sec. 3.2.1, "for each tensor": calibration and Eq. 2 over a whole SET of tensors -------------
 * The sensitivity ordering needs max|x| and the error sums of every weight tensor of the model.
 * These calls cover all tensors of a set in two or three launches instead of several per tensor
 * (a model's tensors are a few MB each: alone, each kernel is mostly launch ramp and tail).
 *
 * The set is described once by a PLAN.  mpq_sweep_plan_build() writes it into HOST memory of the
 * caller (size from mpq_sweep_plan_bytes(), 8-byte aligned); the caller copies those bytes,
 * unchanged, to DEVICE memory (8-byte aligned) and passes both copies to the calls below: the host
 * copy is what the library validates and sizes its grids from, the device copy is what the kernels
 * read.  The plan holds the descriptors and a table of work items; it stays valid as long as the
 * tensors' addresses and shapes do, for any number of calls.  The library allocates and copies
 * nothing.
 *
 * mpq_sweep_tensor (HOST struct of DEVICE pointers):
 *   x [rows x cols] fp32, 16-byte aligned, cols a multiple of 4 and at most 16384 (other tensors go
 *   through the single-tensor calls); absmax_row float[rows] and absmax_tensor float[1]: written by
 *   mpq_calibrate_absmax_batch, read by mpq_quant_error_batch (both required, 4-byte aligned);
 *   sse_tensor double[nb], sse_row double[rows x nb] (row-major, b ascending): written by
 *   mpq_quant_error_batch, each required only for the granularity that writes it (8-byte aligned).
 *
 * mpq_calibrate_absmax_batch: absmax_row[r] = max_c |x[r][c]|, absmax_tensor[0] = max_r absmax_row[r]
 *   (= max |x|; exact), for every tensor of the plan; one read of the tensors.  No workspace.
 * mpq_quant_error_batch: Eq. 2's sums for b = b_lo..b_hi in one read per tensor, with
 *   gran = MPQ_PER_TENSOR: sse_tensor, quantizer scale from absmax_tensor;
 *   gran = MPQ_PER_ROW:    sse_row, scale from absmax_row (bit-identical to mpq_quant_error per tensor);
 *   gran = MPQ_SWEEP_TENSOR_AND_ROW: both from the same read (twice the arithmetic per element).
 *   fp32 per-lane partial sums, fixed-order double combine: reproducible from call to call.
 *   Workspace from the query (0 for MPQ_PER_ROW), 8-byte aligned.
 * mpq_calibrate_quant_error_rows_batch: mpq_calibrate_absmax_batch and
 *   mpq_quant_error_batch(MPQ_PER_ROW) from ONE read of the tensors (the calibration of Sec. 3.1 and
 *   Eq. 2 with the scales it has just found): absmax_row, absmax_tensor and sse_row are written,
 *   bit-identical to the two separate calls.  A row of up to 4096 columns stays in registers
 *   between the two steps; a longer row is read a second time, out of the L2.  No workspace.
 *   For weights, whose maxima come from the tensor itself; activations whose maxima are running
 *   ones over several batches take the two separate calls.
 * Errors: MPQ_ERR_NULL / _SHAPE / _ALIGN for a tensor the plan cannot hold (build), MPQ_ERR_SHAPE
 * for a plan_host that is not a built plan, MPQ_ERR_WORKSPACE, MPQ_ERR_GRAN, MPQ_ERR_BITS. */
typedef struct mpq_sweep_tensor {
  const float* x;
  int64_t rows, cols;
  float* absmax_row;
  float* absmax_tensor;
  double* sse_tensor;
  double* sse_row;
} mpq_sweep_tensor;
enum mpq_sweep_gran { MPQ_SWEEP_TENSOR_AND_ROW = 3 };
size_t mpq_sweep_plan_bytes(const mpq_sweep_tensor* tensors /* host */, int n_tensors);
int mpq_sweep_plan_build(const mpq_sweep_tensor* tensors /* host */, int n_tensors, void* plan_host,
                         size_t plan_host_bytes);
int mpq_calibrate_absmax_batch(const void* plan_host, const void* plan_dev, void* stream);
int mpq_calibrate_quant_error_rows_batch(const void* plan_host, const void* plan_dev, int b_lo, int b_hi,
                                         void* stream);
size_t mpq_quant_error_batch_workspace_bytes(const void* plan_host, int gran, int b_lo, int b_hi);
int mpq_quant_error_batch(const void* plan_host, const void* plan_dev, int gran, int b_lo, int b_hi,
                          void* ws, size_t ws_bytes, void* stream);

/* ---- Sec. 3.2.2 Eq. 3-5: Gaussian perturbation ----------------------------------------------
 * y[i] = fl32(x[i] + sigma_ch * z_i), sigma_ch = fl32(lambda * scale_bits(absmax[ch])): the
 * noise standard deviation is `lambda` quantization steps of the b-bit grid.  z_i is the i-th
 * standard normal (i = r*cols + c) of stream `stream_id` under `seed`: Philox-4x32-10 with
 * key = (seed lo, seed hi), counter = (i/4 lo, i/4 hi, stream_id lo, stream_id hi), output word
 * pairs (0,1) and (2,3) through Box-Muller with the fixed fp32 log / sin / cos recipes of this
 * library; z_i depends on (seed, stream_id, i) only -- not on bits, shape or launch geometry.
 * y_out may alias x.  No workspace. */
int mpq_noise_inject(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax,
                     int bits, float lambda, uint64_t seed, uint64_t stream_id, float* y_out,
                     void* stream);

/* The same perturbation for every bit-width b_lo..b_hi in one pass (z does not depend on b and is
 * drawn once per element): plane k of y_out, starting y_stride elements after plane k-1
 * (y_stride >= rows*cols, else MPQ_ERR_SHAPE), holds exactly what mpq_noise_inject writes for
 * bits = b_lo + k.  x must not overlap y_out. */
int mpq_noise_inject_sweep(const float* x, int64_t rows, int64_t cols, int gran, const float* absmax,
                           int b_lo, int b_hi, float lambda, uint64_t seed, uint64_t stream_id,
                           float* y_out, int64_t y_stride, void* stream);

/* ---- the evaluation step of Alg. 1 / Alg. 2: one quantized linear layer ------------------------
 * acc[m][n] = sum_k a_q[m][k] * w_q[n][k] (int32), y[m][n] = fl32(fl32(float(acc) * a_scale[0])
 *             * w_scale[n or 0]).
 * a_q        int8 [M x K], K contiguous.
 * w_q        w_storage_bits == 8: int8 [N x K];  == 4: uint8 [N x K/2] nibble pairs as written
 *            by mpq_fake_quant (K even).
 * a_scale    [1]; w_scale [1] (w_gran = PER_TENSOR) or [N] (PER_ROW).  Needed only with y_out.
 * y_out      nullable fp32 [M x N]; acc_out nullable int32 [M x N]; at least one is required.
 * K*127*127 must stay below 2^31 (K <= 133143), else MPQ_ERR_SHAPE.
 * 16-byte aligned a_q / w_q with K a multiple of 16 (32 for packed int4) take the fast path;
 * anything else is computed by a slower byte-wise loader with identical results.
 * Workspace: optional.  Shapes with a handful of output tiles and a long K (at most 64 tiles of
 * 64 x 64, K >= 1024: any layer at inference batch 1) are cut along K when the caller passes
 * the workspace the query asks for (16-byte aligned): partial int32 accumulators go to the
 * workspace and are added by a second kernel -- integer sums, so acc_out and y_out are bit-identical
 * to the unsplit product.  With ws == NULL (or too small) the same results are computed without
 * the split, only slower on those shapes; the query returns 0 for shapes that are not split. */
size_t mpq_qgemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int w_storage_bits);
int mpq_qgemm(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
              int64_t K, const float* a_scale, const float* w_scale, int w_gran, float* y_out,
              int32_t* acc_out, void* ws, size_t ws_bytes, void* stream);

/* ---- the score kept by the evaluation step of Alg. 1 / Alg. 2, stand-in: squared output error -------
 * sse_out[0] = sum_i (y[i] - y_ref[i])^2 (double).  fp32 per-lane partials, fixed-order double
 * combine.  Dividing by n gives the candidate's output MSE. */
size_t mpq_sse_pair_workspace_bytes(int64_t n);
int mpq_sse_pair(const float* y, const float* y_ref, int64_t n, double* sse_out, void* ws,
                 size_t ws_bytes, void* stream);

/* ---- the layer of mpq_qgemm with what follows it inside an evaluation taken in its epilogue ----
 * y_out = act(Y) with Y as mpq_qgemm defines it, act one of mpq_act:
 *   MPQ_ACT_RELU  max(Y, 0);   MPQ_ACT_GELU  Y * Phi(Y), Phi the standard normal distribution
 *   function, evaluated in fp32 from a fitted approximation of its tail: within 1e-5 relative of
 *   the exact value, or 4e-7 |Y| where that is larger (beyond Y = -6, where GELU is below 1e-9 |Y|).
 * absmax_out nullable float[1]: max |y_out|, i.e. the max calibration (Sec. 3.1) of the next
 *   layer's input, taken on the values while they are in registers.  accumulate = 0 overwrites
 *   it, 1 keeps a running maximum (absmax_out must then hold a valid non-negative value).
 *   The maximum is exact (order independent).
 * y_out      nullable when absmax_out is given: the calibration-only pass, which computes the
 *   product and keeps nothing but the maximum (no fp32 output travels to HBM).
 * Other arguments and errors as mpq_qgemm, plus MPQ_ERR_SHAPE for an unknown act.  No workspace. */
enum mpq_act { MPQ_ACT_NONE = 0, MPQ_ACT_RELU = 1, MPQ_ACT_GELU = 2 };
int mpq_qgemm_act(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
                  int64_t K, const float* a_scale, const float* w_scale, int w_gran, int act,
                  float* y_out, float* absmax_out, int accumulate, void* stream);

/* ---- the same layer with Eq. 1 applied to its activated output in the epilogue ----------------
 * codes_out[m][n] = clamp(RNE(act(Y)[m][n] * inv_b), +-qmax_b) as int8 [M x N], inv_b = qmax_b /
 * absmax[0]: exactly the codes mpq_fake_quant(per tensor, bits) gives for the y_out of
 * mpq_qgemm_act, without that fp32 tensor ever being stored.  Meant as the second of two passes
 * over the product: mpq_qgemm_act(y_out = NULL) finds absmax, this call quantizes with it, and
 * the next layer's GEMM reads codes_out (its activation step is mpq_scale_from_absmax(absmax, bits)).
 * Recomputing the int8 product costs less than writing and re-reading 4 bytes per output.
 * absmax     device float[1], required (any non-negative value; 0 gives all-zero codes).
 * bits       2..8.  codes_out required.  Other arguments and errors as mpq_qgemm_act. */
int mpq_qgemm_act_codes(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
                        int64_t K, const float* a_scale, const float* w_scale, int w_gran, int act,
                        const float* absmax, int bits, int8_t* codes_out, void* stream);

/* ---- Hutchinson's estimate of the Hessian trace (Sec. 3.2.3, E_Hessian) ------------------------
 * For a linear layer Y = X W' (X [M x K], W [N x K]) under L = mean over the M N outputs of
 * (Y - T)^2 the Hessian with respect to W is (2 / (M N)) (I_N (x) X'X): a probe's quadratic form
 * is a sum of ||X v||^2 over K-vectors v, and
 *     Tr(H) ~= (2 / M) * mean_p quad[p],   quad[p] = ||X v_p||^2   (exact: (2 / M) ||X||_F^2).
 * With respect to the layer input instead, pass W as x: Tr = (2 / N) * mean_p ||W v_p||^2.
 *
 * mpq_rademacher: v_out fp32 [rows x cols] of +1 / -1.  Element e = r * cols + c takes bit
 *   (e mod 128) of the Philox-4x32-10 block with counter (e / 128, stream_id) and key
 *   (seed lo, seed hi XOR 0x5241444D); bit t = word t / 32, position t mod 32; set bit = -1.
 *   Depends on (seed, stream_id, e) only.  rows * cols <= 2^38.
 * mpq_hutchinson_quad: quad_out double [P], quad_out[p] = sum_m (sum_k x[m][k] v[p][k])^2 for any
 *   fp32 probes v [P x K] (the sums over k are taken in fp32 on the matrix cores, squares and the
 *   sum over m in fp32 per lane, the final combine in double in a fixed order; reproducible).
 *   x, v 4-byte aligned (16-byte aligned with K % 4 == 0 takes the vector loads); quad_out 8-byte
 *   aligned.  M < 2^31, P <= 2^20.  Workspace from the query (MPQ_ERR_WORKSPACE if too small). */
int mpq_rademacher(uint64_t seed, uint64_t stream_id, int64_t rows, int64_t cols, float* v_out,
                   void* stream);
size_t mpq_hutchinson_quad_workspace_bytes(int64_t M, int64_t K, int64_t P);
int mpq_hutchinson_quad(const float* x, int64_t M, int64_t K, const float* v, int64_t P,
                        double* quad_out, void* ws, size_t ws_bytes, void* stream);
/* The same quadratic forms for the sign probes mpq_rademacher(seed, stream_id, P, K) would store,
 * drawn inside the kernel: no probe matrix exists in memory.  Results equal those of
 * mpq_hutchinson_quad on that matrix up to the fp32 rounding of a different summation order over k.  Needs K % 16 == 0 and x 16-byte aligned
 * (MPQ_ERR_SHAPE otherwise: draw the matrix and use the call above).  Same workspace query. */
int mpq_hutchinson_quad_signs(const float* x, int64_t M, int64_t K, uint64_t seed, uint64_t stream_id,
                              int64_t P, double* quad_out, void* ws, size_t ws_bytes, void* stream);
/* The estimate itself (HOST function on the P quadratic forms read back from the device):
 * estimate_out[0] = (2 / rows) * mean_p quad[p], rows = M of the tensor the forms were taken of, and
 * std_error_out[0] (nullable) = (2 / rows) * sample standard deviation of quad / sqrt(P), NaN for P = 1. */
int mpq_hutchinson_trace(const double* quad, int64_t P, int64_t rows, double* estimate_out, double* std_error_out);

/* ---- the evaluation step of Alg. 1 / Alg. 2 in one call -------------------
 * The layer of mpq_qgemm with the score of mpq_sse_pair taken in its epilogue:
 * sse_out[0] = sum_{m,n} (y[m][n] - y_ref[m][n])^2 (double), y exactly as mpq_qgemm defines it.
 * y_ref      fp32 [M x N], required.
 * y_out      nullable: when NULL the layer output is never written, which is what a search over
 *            bit configurations wants for the last layer (only the score leaves the chip).
 * Workspace: one double per workgroup, size from the query; needs no initialisation.
 * fp32 per-lane partials (at most a few hundred terms each), fixed-order double combine:
 * results are reproducible from call to call.  Other arguments and errors as mpq_qgemm. */
size_t mpq_qgemm_score_workspace_bytes(int64_t M, int64_t N, int64_t K, int w_storage_bits);
int mpq_qgemm_score(const int8_t* a_q, const void* w_q, int w_storage_bits, int64_t M, int64_t N,
                    int64_t K, const float* a_scale, const float* w_scale, int w_gran,
                    const float* y_ref, double* sse_out, float* y_out, void* ws, size_t ws_bytes,
                    void* stream);

/* ---- Sec. 3.1, second step ("adjustment"): the two scales of Eq. 1 as free parameters ---------
 * In the integer form of this library the pair is inv (= alpha * levels, applied before rounding)
 * and scale (= gamma / levels, applied after); calibration sets inv = qmax/m, scale = m/qmax.
 * gran is MPQ_PER_TENSOR or MPQ_PER_ROW (else MPQ_ERR_GRAN); inv, scale: [1] or [rows].
 *
 * mpq_fake_quant_scales: code = clamp(RNE(x*inv), +-qmax) on the exact product, Q = fl32(code*scale);
 *   y_out / codes_out nullable, at least one required.
 * mpq_scale_grad: with g = dL/dQ (fp32 [rows x cols]) and rounding treated as the identity,
 *   dscale_out[ch] = sum g*code,  dinv_out[ch] = scale[ch] * sum over elements whose rounded value
 *   needs no clamping (|RNE(x*inv)| <= qmax) of g*x,  loss_out[ch] (nullable) = sum (Q - x)^2.
 *   g == NULL selects the reconstruction loss L = sum (Q - x)^2 itself, g = 2 (Q - x).
 *   fp32 per-lane partial sums, double from there on; outputs are doubles, 8-byte aligned.
 *   Workspace: per-tensor granularity only (one partial triple per workgroup).
 * mpq_scale_sgd_step: p[i] = fl32(p[i] - lr * dL/dp[i]) for both scale vectors, i < count, formed
 *   in double and rounded once.  The model's own parameters are never touched. */
int mpq_fake_quant_scales(const float* x, int64_t rows, int64_t cols, int gran, const float* inv,
                          const float* scale, int bits, float* y_out, int8_t* codes_out, void* stream);
size_t mpq_scale_grad_workspace_bytes(int64_t rows, int64_t cols, int gran);
int mpq_scale_grad(const float* x, int64_t rows, int64_t cols, int gran, const float* inv,
                   const float* scale, int bits, const float* g, double* dinv_out, double* dscale_out,
                   double* loss_out, void* ws, size_t ws_bytes, void* stream);
int mpq_scale_sgd_step(float* inv, float* scale, const double* dinv, const double* dscale,
                       int64_t count, double lr, void* stream);

/* ---- the evaluation step of Alg. 1 / Alg. 2 for a whole stack of layers in one call ------------
 * The model f is n_layers linear layers with an activation between them.  Layer l has weights
 * [N_l x K_l] (K_{l+1} = N_l) quantized beforehand at each of its n_widths candidate widths; an
 * evaluation picks one width per layer (width_index[l], host array) and enqueues, per layer,
 *   l > 0:  mpq_fake_quant(h_{l-1} -> a_codes_l, absmax a_absmax[l], act_bits), per tensor, with
 *           the step size mpq_scale_from_absmax(a_absmax[l]) written to a_scale[l] by the same kernel,
 *   l < n_layers - 1:  mpq_qgemm_act(..., act, h_l, running maximum into a_absmax[l + 1]),
 *   last layer:        mpq_qgemm_score(..., y_ref) -> sse_out[0],
 * i.e. the results of exactly those calls, in two launches per layer, issued from native code.
 * a_absmax[1..] is cleared first (one small kernel).
 * The caller provides layer 0's a_codes, a_absmax[0] and a_scale[0] (the model's input does not
 * depend on the configuration).  mpq_stack_layer holds HOST arrays of DEVICE pointers.
 * Errors: as the calls above; every argument is checked before the first launch. */
typedef struct mpq_stack_layer {
  int64_t N, K;                 /* weights [N x K] */
  int n_widths;                 /* candidate widths of this layer */
  const void* const* w_q;       /* [n_widths] device: int8 codes [N x K] or packed nibbles [N x K/2] */
  const float* const* w_scale;  /* [n_widths] device: step sizes, [1] or [N] by w_gran */
  const int* w_storage_bits;    /* [n_widths] host: 8 or 4 */
  int8_t* a_codes;              /* device [M x K]: the layer's quantized input */
  float* h;                     /* device [M x N] fp32: the layer's activated output; NULL for the last layer */
} mpq_stack_layer;
size_t mpq_stack_evaluate_workspace_bytes(const mpq_stack_layer* layers, int n_layers, int64_t M);
int mpq_stack_evaluate(const mpq_stack_layer* layers, int n_layers, int64_t M, const int* width_index,
                       int act_bits, int act, int w_gran, float* a_absmax /* device [n_layers] */,
                       float* a_scale /* device [n_layers] */, const float* y_ref, double* sse_out,
                       void* ws, size_t ws_bytes, void* stream);

/* ---- Alg. 1 (bisection search) and Alg. 2 (greedy search): host code ---------------------------
 * Both decide which per-layer bit configuration to evaluate next and return the final one; they
 * launch nothing themselves.  All pointers here are HOST pointers.
 * eval       the evaluation step of Alg. 1 / Alg. 2: called with bits[n_layers] (bits[l] = width
 *            of layer l) and `user`; returns the accuracy a, which is compared with `target`
 *            (a >= target meets it).  Called from the calling thread, one call at a time.
 * order      the layer ids 0 .. n_layers-1 sorted by sensitivity in ascending order (a
 *            permutation, else MPQ_ERR_SHAPE).
 * bit_widths the available widths bs, visited in the order given (pass them descending: highest
 *            quantized precision first); each in 2..16, else MPQ_ERR_BITS.  The working
 *            configuration starts at the largest of them.
 * flags      0, or MPQ_SEARCH_ENSURE_TARGET (bisection only): if the loop of Alg. 1 stops on an
 *            evaluation that missed the target, fall back to the largest layer count that met it
 *            instead of keeping the failed one, as the printed arithmetic would.
 * config_out [n_layers] final width per layer.  n_evals_out nullable: number of eval calls.
 * Threshold arithmetic of Alg. 1: integers, floor division, stop when an update leaves thr
 * unchanged. */
typedef double (*mpq_eval_fn)(const int* bits, int n_layers, void* user);
enum mpq_search_flags { MPQ_SEARCH_ENSURE_TARGET = 1 };
int mpq_search_bisection(const int* order, int n_layers, const int* bit_widths, int n_bits,
                         double target, int flags, mpq_eval_fn eval, void* user, int* config_out,
                         int* n_evals_out);
int mpq_search_greedy(const int* order, int n_layers, const int* bit_widths, int n_bits,
                      double target, int flags, mpq_eval_fn eval, void* user, int* config_out,
                      int* n_evals_out);

/* ---- Experiments section, "Compute Latency Estimates" and Table 1: deployment estimates (HOST) ----
 * The paper benchmarks the kernel of every layer shape at every precision (inference batch size 1)
 * and combines the kernel latencies of a configuration's layers into a model latency; here the
 * kernel is mpq_qgemm (timed by the caller with events) and the combination is the sum, layers of
 * an inference pass running one after the other.
 * mpq_latency_estimate: layer_us [n_layers x n_widths] (row-major) measured latencies of layer l
 *   at its candidate precision number w; width_index[l] < n_widths the precision of layer l in the
 *   configuration; total_us_out[0] = sum_l layer_us[l][width_index[l]].
 * mpq_model_size_bytes: bytes_out[0] = sum_l parameters[l] * bits[l] / 8 (bits 1..64).
 * All pointers are host pointers. */
int mpq_latency_estimate(const double* layer_us, int n_layers, int n_widths, const int* width_index,
                         double* total_us_out);
int mpq_model_size_bytes(const int64_t* parameters, const int* bits, int n_layers, double* bytes_out);

/* ---- measurement aid (not part of the method) --------------------------------------------------
 * Launches a kernel that does nothing but issue int8 matrix-core instructions (one workgroup of
 * eight waves per CU, 16 x iters instructions per wave) on operand registers filled once from
 * `operands` (device, 16-byte aligned, at least mpq_diag_mfma_operand_bytes() bytes).  Timing it
 * gives the matrix rate this chip sustains for operands of that kind: the clock under matrix load
 * depends on how much the operand bits toggle.  ops_out (host, nullable) receives the number of
 * integer operations the launch performs (2 per multiply-add).  sink: device int[1], scratch. */
size_t mpq_diag_mfma_operand_bytes(void);
int mpq_diag_mfma_rate(const void* operands, size_t operand_bytes, int iters, int* sink, double* ops_out,
                       void* stream);

/* Launches a kernel that does nothing but the arithmetic of the error sweep of Sec. 3.2.1 Eq. 2 for
 * b = 2..8 (the code mpq_quant_error runs per element) on elements held in registers: eight
 * workgroups of 256 threads per CU, 16 elements per lane and iteration, no memory traffic in the
 * loop.  Timing it gives the vector-ALU ceiling of the sweep kernels on this chip.  lane_ops_out
 * (host, nullable) receives the number of lane-operations of the launch (28 per element).
 * sink: device float[1], scratch. */
int mpq_diag_sweep_alu_rate(int iters, float* sink, double* lane_ops_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MPQ_H_ */

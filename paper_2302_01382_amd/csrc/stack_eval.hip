// stack_eval.hip -- the evaluation step of Alg. 1 / Alg. 2 for a stack of
// linear layers with an activation between them, as ONE host call: for every layer the quantizer
// of its input (Eq. 1, the same kernel also leaves the step size), and the quantized layer with
// the activation and the max calibration of the next input in its epilogue; the last layer's epilogue takes the score.  The
// searches call this thousands of times with different width choices; issued call by call from a
// scripting language the ~3 launches per layer cost more host time than device time.
// Host code: it only enqueues the library's own kernels on the caller's stream.
#include "common.hpp"

namespace {
__global__ void clear_f32(float* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.0f;
}
}  // namespace

extern "C" size_t mpq_stack_evaluate_workspace_bytes(const mpq_stack_layer* layers, int n_layers, int64_t M) {
  if (!layers || n_layers <= 0 || M <= 0) return 0;
  const mpq_stack_layer& last = layers[n_layers - 1];
  return mpq_qgemm_score_workspace_bytes(M, last.N, last.K, 8);
}

extern "C" int mpq_stack_evaluate(const mpq_stack_layer* layers, int n_layers, int64_t M, const int* width_index,
                                  int act_bits, int act, int w_gran, float* a_absmax, float* a_scale,
                                  const float* y_ref, double* sse_out, void* ws, size_t ws_bytes, void* stream) {
  if (!layers || !width_index || !a_absmax || !a_scale || !y_ref || !sse_out) return MPQ_ERR_NULL;
  if (n_layers <= 0 || M <= 0) return MPQ_ERR_SHAPE;
  if (act_bits < 2 || act_bits > 8) return MPQ_ERR_BITS;
  if (act < MPQ_ACT_NONE || act > MPQ_ACT_GELU) return MPQ_ERR_SHAPE;
  // Everything is checked before the first launch, with the very checks the per-layer calls apply,
  // so that a failing call leaves the device untouched.
  if (w_gran != MPQ_PER_TENSOR && w_gran != MPQ_PER_ROW) return MPQ_ERR_GRAN;
  if (!ws || ws_bytes < mpq_stack_evaluate_workspace_bytes(layers, n_layers, M)) return MPQ_ERR_WORKSPACE;
  for (int l = 0; l < n_layers; ++l) {
    const mpq_stack_layer& L = layers[l];
    if (!L.w_q || !L.w_scale || !L.w_storage_bits || !L.a_codes) return MPQ_ERR_NULL;
    if (L.N <= 0 || L.K <= 0 || L.n_widths <= 0) return MPQ_ERR_SHAPE;
    if (width_index[l] < 0 || width_index[l] >= L.n_widths) return MPQ_ERR_SHAPE;
    const int w = width_index[l];
    int rc;
    if (l + 1 < n_layers) {
      if (!L.h) return MPQ_ERR_NULL;
      if (layers[l + 1].K != L.N) return MPQ_ERR_SHAPE;  // the layers must chain
      rc = mpq::check_qgemm_act_args(L.a_codes, L.w_q[w], L.w_storage_bits[w], M, L.N, L.K, a_scale + l, L.w_scale[w],
                                     w_gran, act, L.h, a_absmax + l + 1);
    } else {
      rc = mpq::check_qgemm_score_args(L.a_codes, L.w_q[w], L.w_storage_bits[w], M, L.N, L.K, a_scale + l, L.w_scale[w],
                                       w_gran, y_ref, sse_out, nullptr, ws, ws_bytes);
    }
    if (rc != MPQ_OK) return rc;
    if (l > 0 && mpq::mul_overflows(M, L.K)) return MPQ_ERR_SHAPE;  // the quantizer's own shape check
  }
  hipStream_t st = (hipStream_t)stream;
  // the running maxima of the inputs of layers 1.. start at zero (the activation's output is what
  // they are taken of; layer 0's input was calibrated by the caller)
  if (n_layers > 1) clear_f32<<<(unsigned)((n_layers - 1 + 255) / 256), 256, 0, st>>>(a_absmax + 1, n_layers - 1);
  for (int l = 0; l < n_layers; ++l) {
    const mpq_stack_layer& L = layers[l];
    const int w = width_index[l];
    int rc;
    if (l > 0) {
      // the quantizer kernel also leaves the step size: no launch of its own for one division
      rc = mpq::fake_quant_launch(layers[l - 1].h, M, L.K, MPQ_PER_TENSOR, a_absmax + l, act_bits, nullptr, L.a_codes,
                                  nullptr, a_scale + l, stream);
      if (rc != MPQ_OK) return rc;
    }
    if (l + 1 < n_layers) {
      rc = mpq_qgemm_act(L.a_codes, L.w_q[w], L.w_storage_bits[w], M, L.N, L.K, a_scale + l, L.w_scale[w], w_gran, act,
                         L.h, a_absmax + l + 1, 1, stream);
    } else {
      rc = mpq_qgemm_score(L.a_codes, L.w_q[w], L.w_storage_bits[w], M, L.N, L.K, a_scale + l, L.w_scale[w], w_gran,
                           y_ref, sse_out, nullptr, ws, ws_bytes, stream);
    }
    if (rc != MPQ_OK) return rc;
  }
  return mpq::launch_status();
}

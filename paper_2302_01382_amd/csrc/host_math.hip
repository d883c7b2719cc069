// host_math.hip -- the few scalar steps of the method that follow a device result on the host: the
// normalisation of Eq. 2 (Sec. 3.2.1) that turns error sums into the sensitivity E_QE, and the mean
// and standard error that turn Hutchinson's quadratic forms (Sec. 3.2.3) into the trace estimate.
// Plain host code on host arrays (the caller has read the sums back); nothing here touches the device.
#include "mpq.h"

#include <cmath>

extern "C" double mpq_eqe(double sse, int64_t n, double absmax) {
  if (n <= 0 || !(absmax > 0.0) || !(sse >= 0.0)) return 0.0;
  return std::sqrt(sse / (double)n) / absmax;
}

extern "C" int mpq_eqe_channels(const double* sse, const float* absmax, int64_t nch, int nb, int64_t n,
                                double* eqe_out) {
  if (!sse || !absmax || !eqe_out) return MPQ_ERR_NULL;
  if (nch <= 0 || n <= 0) return MPQ_ERR_SHAPE;
  if (nb < 1 || nb > 7) return MPQ_ERR_BITS;
  float m = 0.0f;
  for (int64_t c = 0; c < nch; ++c) m = absmax[c] > m ? absmax[c] : m;
  for (int b = 0; b < nb; ++b) {
    double total = 0.0;
    for (int64_t c = 0; c < nch; ++c) total += sse[c * nb + b];
    eqe_out[b] = mpq_eqe(total, n, (double)m);
  }
  return MPQ_OK;
}

extern "C" int mpq_hutchinson_trace(const double* quad, int64_t P, int64_t rows, double* estimate_out,
                                    double* std_error_out) {
  if (!quad || !estimate_out) return MPQ_ERR_NULL;
  if (P <= 0 || rows <= 0) return MPQ_ERR_SHAPE;
  double mean = 0.0;
  for (int64_t p = 0; p < P; ++p) mean += quad[p];
  mean /= (double)P;
  const double k = 2.0 / (double)rows;
  *estimate_out = k * mean;
  if (std_error_out) {
    if (P > 1) {
      double ss = 0.0;
      for (int64_t p = 0; p < P; ++p) ss += (quad[p] - mean) * (quad[p] - mean);
      *std_error_out = k * std::sqrt(ss / (double)(P - 1)) / std::sqrt((double)P);
    } else {
      *std_error_out = NAN;
    }
  }
  return MPQ_OK;
}

// Experiments section, "Compute Latency Estimates": the deployment latency of a mixed-precision
// model from the kernel latencies of its layers -- layer_us[l][w] measured for layer l at its
// candidate precision number w, width_index[l] the precision a configuration gives layer l.
// Layers of an inference pass run one after the other: the estimate is the sum.
extern "C" int mpq_latency_estimate(const double* layer_us, int n_layers, int n_widths, const int* width_index,
                                    double* total_us_out) {
  if (!layer_us || !width_index || !total_us_out) return MPQ_ERR_NULL;
  if (n_layers <= 0 || n_widths <= 0) return MPQ_ERR_SHAPE;
  double total = 0.0;
  for (int l = 0; l < n_layers; ++l) {
    if (width_index[l] < 0 || width_index[l] >= n_widths) return MPQ_ERR_SHAPE;
    total += layer_us[(int64_t)l * n_widths + width_index[l]];
  }
  *total_us_out = total;
  return MPQ_OK;
}

// Model size of a configuration (Table 1, "Size"): parameters times their bit-widths, in bytes.
extern "C" int mpq_model_size_bytes(const int64_t* parameters, const int* bits, int n_layers, double* bytes_out) {
  if (!parameters || !bits || !bytes_out) return MPQ_ERR_NULL;
  if (n_layers <= 0) return MPQ_ERR_SHAPE;
  double total = 0.0;
  for (int l = 0; l < n_layers; ++l) {
    if (parameters[l] < 0) return MPQ_ERR_SHAPE;
    if (bits[l] < 1 || bits[l] > 64) return MPQ_ERR_BITS;
    total += (double)parameters[l] * (double)bits[l] / 8.0;
  }
  *bytes_out = total;
  return MPQ_OK;
}

// search.hip -- the two configuration searches of the paper, Alg. 1 (bisection) and Alg. 2
// (greedy), as host code.  They decide which bit configuration to evaluate next; the evaluation
// itself ("Evaluate f(x, lw) and save accuracy a") is the caller's callback, which on this
// library's path is a chain of mpq_fake_quant / mpq_qgemm / mpq_qgemm_score launches followed by
// one read-back of the score.  Nothing here touches the device.
//
// Readings of the printed algorithms (they leave these open):
//  - bit widths are visited in the order the caller lists them (the text wants the highest
//    quantized precision first, so callers pass them in descending order); the working
//    configuration starts at the largest listed width;
//  - the threshold arithmetic of Alg. 1 is integer arithmetic with floor division, and "until thr
//    is not changing" compares the threshold after the update with the one before it.
//    Consequences of that arithmetic, kept as printed: the threshold never reaches the full list
//    length, and when even a single layer fails the target the loop still ends at thr = 1.  With
//    MPQ_SEARCH_ENSURE_TARGET the search falls back, in that last case, to the largest count it
//    has seen meet the target (lowl), so that the returned configuration never relies on an
//    evaluation that failed.
#include "mpq.h"

#include <vector>

namespace {

int check_common(const int* order, int n_layers, const int* bit_widths, int n_bits, mpq_eval_fn eval,
                 int* config_out) {
  if (!order || !bit_widths || !eval || !config_out) return MPQ_ERR_NULL;
  if (n_layers <= 0 || n_bits <= 0) return MPQ_ERR_SHAPE;
  std::vector<char> seen((size_t)n_layers, 0);
  for (int i = 0; i < n_layers; ++i) {  // order must be a permutation of the layer ids
    if (order[i] < 0 || order[i] >= n_layers || seen[(size_t)order[i]]) return MPQ_ERR_SHAPE;
    seen[(size_t)order[i]] = 1;
  }
  for (int i = 0; i < n_bits; ++i)
    if (bit_widths[i] < 2 || bit_widths[i] > 16) return MPQ_ERR_BITS;
  return MPQ_OK;
}

int widest(const int* bit_widths, int n_bits) {
  int m = bit_widths[0];
  for (int i = 1; i < n_bits; ++i) m = bit_widths[i] > m ? bit_widths[i] : m;
  return m;
}

}  // namespace

extern "C" int mpq_search_bisection(const int* order, int n_layers, const int* bit_widths, int n_bits,
                                    double target, int flags, mpq_eval_fn eval, void* user,
                                    int* config_out, int* n_evals_out) {
  const int rc = check_common(order, n_layers, bit_widths, n_bits, eval, config_out);
  if (rc != MPQ_OK) return rc;
  const bool ensure = (flags & MPQ_SEARCH_ENSURE_TARGET) != 0;
  std::vector<int> w((size_t)n_layers, widest(bit_widths, n_bits));  // working configuration
  std::vector<int> lw((size_t)n_layers);
  int len = n_layers;  // the layer list is always a prefix of `order`: ll = order[0 : len]
  int evals = 0;
  for (int bi = 0; bi < n_bits; ++bi) {
    const int b = bit_widths[bi];
    int thr = len / 2, upl = len, lowl = 0;
    bool last_met = false;
    for (;;) {
      lw = w;
      for (int i = 0; i < thr; ++i) lw[(size_t)order[i]] = b;
      const double a = eval(lw.data(), n_layers, user);
      ++evals;
      last_met = a >= target;
      const int before = thr;
      if (last_met) {
        lowl = thr;
        thr = thr + (upl - thr) / 2;
      } else {
        upl = thr;
        thr = thr - (thr - lowl) / 2;
      }
      if (thr == before) break;
    }
    if (ensure && !last_met) thr = lowl;
    for (int i = 0; i < thr; ++i) w[(size_t)order[i]] = b;
    len = thr;
  }
  for (int i = 0; i < n_layers; ++i) config_out[i] = w[(size_t)i];
  if (n_evals_out) *n_evals_out = evals;
  return MPQ_OK;
}

extern "C" int mpq_search_greedy(const int* order, int n_layers, const int* bit_widths, int n_bits,
                                 double target, int flags, mpq_eval_fn eval, void* user, int* config_out,
                                 int* n_evals_out) {
  (void)flags;  // every step of Alg. 2 that is kept was evaluated and met the target
  const int rc = check_common(order, n_layers, bit_widths, n_bits, eval, config_out);
  if (rc != MPQ_OK) return rc;
  std::vector<int> w((size_t)n_layers, widest(bit_widths, n_bits));
  std::vector<int> ll(order, order + n_layers), ql;
  int evals = 0;
  for (int bi = 0; bi < n_bits; ++bi) {
    const int b = bit_widths[bi];
    ql.clear();
    for (int l : ll) {
      const int before = w[(size_t)l];
      w[(size_t)l] = b;
      const double a = eval(w.data(), n_layers, user);
      ++evals;
      if (a >= target) ql.push_back(l);
      else w[(size_t)l] = before;  // and the layer is not a candidate for lower widths any more
    }
    ll.swap(ql);
  }
  for (int i = 0; i < n_layers; ++i) config_out[i] = w[(size_t)i];
  if (n_evals_out) *n_evals_out = evals;
  return MPQ_OK;
}

// search.hip -- the two configuration searches of the paper, Alg. 1 (bisection) and Alg. 2
// (greedy), as host code.  They decide which bit configuration to evaluate next; the evaluation
// itself (the evaluation step of both algorithms) is the caller's callback, which on this
// library's path is mpq_stack_evaluate or a chain of mpq_fake_quant / mpq_qgemm_act /
// mpq_qgemm_score launches followed by one read-back of the score.  Nothing here touches the device.
//
// Both searches only ever lower a PREFIX of the sensitivity order (bisection) or single layers of
// it (greedy), so the state is kept in those terms: the committed configuration, and for the
// bisection the interval [lo, hi) of prefix lengths still in question.
//
// Readings of the printed algorithms (they leave these open):
//  - bit widths are visited in the order the caller lists them (the text wants the highest
//    quantized precision first, so callers pass them in descending order); the committed
//    configuration starts at the largest listed width;
//  - Alg. 1 moves its prefix length by integer halves of the distance to the bound on the side it
//    is heading for, and stops at the first update that leaves the length where it was.
//    Consequences of that arithmetic, kept as printed: the length never reaches the full list,
//    and when the loop stops on an evaluation that missed the target the length stays on the
//    count that failed.  With MPQ_SEARCH_ENSURE_TARGET the search falls back, in that case, to the
//    largest length it has seen meet the target, so that the returned configuration never relies
//    on an evaluation that failed.
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

// One search in progress: the committed configuration and the callback that scores a trial.
struct Trial {
  const int* order;
  int n_layers;
  mpq_eval_fn eval;
  void* user;
  double target;
  std::vector<int> committed, scratch;
  int evals = 0;

  // does the model meet the target with the first `count` layers of the order at `width` and
  // every other layer as committed?
  bool prefix_meets_target(int count, int width) {
    scratch = committed;
    for (int i = 0; i < count; ++i) scratch[(size_t)order[i]] = width;
    ++evals;
    return eval(scratch.data(), n_layers, user) >= target;
  }
  void commit_prefix(int count, int width) {
    for (int i = 0; i < count; ++i) committed[(size_t)order[i]] = width;
  }
};

}  // namespace

extern "C" int mpq_search_bisection(const int* order, int n_layers, const int* bit_widths, int n_bits,
                                    double target, int flags, mpq_eval_fn eval, void* user,
                                    int* config_out, int* n_evals_out) {
  const int rc = check_common(order, n_layers, bit_widths, n_bits, eval, config_out);
  if (rc != MPQ_OK) return rc;
  const bool fall_back = (flags & MPQ_SEARCH_ENSURE_TARGET) != 0;
  Trial t{order, n_layers, eval, user, target, std::vector<int>((size_t)n_layers, widest(bit_widths, n_bits)), {}};
  int candidates = n_layers;  // layers still eligible for a lower width: order[0 .. candidates)
  for (int bi = 0; bi < n_bits; ++bi) {
    const int width = bit_widths[bi];
    int lo = 0, hi = candidates;  // lengths known to meet the target / known (or assumed) not to
    int count = candidates / 2;
    bool met;
    for (;;) {
      met = t.prefix_meets_target(count, width);
      int next;
      if (met) {
        lo = count;
        next = count + (hi - count) / 2;
      } else {
        hi = count;
        next = count - (count - lo) / 2;
      }
      if (next == count) break;
      count = next;
    }
    if (!met && fall_back) count = lo;
    t.commit_prefix(count, width);
    candidates = count;
  }
  for (int i = 0; i < n_layers; ++i) config_out[i] = t.committed[(size_t)i];
  if (n_evals_out) *n_evals_out = t.evals;
  return MPQ_OK;
}

extern "C" int mpq_search_greedy(const int* order, int n_layers, const int* bit_widths, int n_bits,
                                 double target, int flags, mpq_eval_fn eval, void* user, int* config_out,
                                 int* n_evals_out) {
  (void)flags;  // every step of Alg. 2 that is kept was evaluated and met the target
  const int rc = check_common(order, n_layers, bit_widths, n_bits, eval, config_out);
  if (rc != MPQ_OK) return rc;
  std::vector<int> config((size_t)n_layers, widest(bit_widths, n_bits));
  std::vector<int> eligible(order, order + n_layers), still_eligible;  // in sensitivity order
  int evals = 0;
  for (int bi = 0; bi < n_bits; ++bi) {
    const int width = bit_widths[bi];
    still_eligible.clear();
    for (int layer : eligible) {
      const int keep = config[(size_t)layer];
      config[(size_t)layer] = width;  // trial: this one layer lower, everything accepted so far stays
      ++evals;
      if (eval(config.data(), n_layers, user) >= target) still_eligible.push_back(layer);
      else config[(size_t)layer] = keep;  // rejected: back to its last accepted width, out of the lower rounds
    }
    eligible.swap(still_eligible);
  }
  for (int i = 0; i < n_layers; ++i) config_out[i] = config[(size_t)i];
  if (n_evals_out) *n_evals_out = evals;
  return MPQ_OK;
}

// qgemm_t64.hip -- the fast path of mpq_qgemm (qgemm_dma.hpp) instantiated for one tile size; a
// translation unit per tile size so that the sources compile side by side.
#include "qgemm_dma.hpp"

namespace mpq {

#define MPQ_GO(W4, KB) launch_dma<64, 64, 2, 2, 3, W4, KB>(a.a_q, a.w_q, a.M, a.N, a.K, a.a_scale, a.w_scale, a.per_row, a.y_out, a.acc_out, a.st, a.epi, a.n_partials, a.split, a.k_per_split, a.prepare_only)
// long_k: k tiles of 256 bytes.  With one 32 x 32 matrix instruction per wave and k substep this tile
// is bound by the latency of its barrier and of the loads behind it, paid once per k tile: twice
// the k per tile halves how often.
int launch_dma_64(bool w4, bool long_k, const DmaArgs& a) {
  if (long_k) return w4 ? MPQ_GO(true, 256) : MPQ_GO(false, 256);
  return w4 ? MPQ_GO(true, 128) : MPQ_GO(false, 128);
}
#undef MPQ_GO

}  // namespace mpq

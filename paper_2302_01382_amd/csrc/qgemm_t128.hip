// qgemm_t128.hip -- the fast path of mpq_qgemm (qgemm_dma.hpp) instantiated for one tile size; a
// translation unit per tile size so that the sources compile side by side.
#include "qgemm_dma.hpp"

namespace mpq {

#define MPQ_GO(NS, W4) launch_dma<128, 128, 2, 4, NS, W4>(a.a_q, a.w_q, a.M, a.N, a.K, a.a_scale, a.w_scale, a.per_row, a.y_out, a.acc_out, a.st, a.epi, a.n_partials, a.split, a.k_per_split, a.prepare_only)
// three stages (one workgroup per CU) or two (two workgroups per CU)
int launch_dma_128(bool w4, bool three_stages, const DmaArgs& a) {
  if (three_stages) return w4 ? MPQ_GO(3, true) : MPQ_GO(3, false);
  return w4 ? MPQ_GO(2, true) : MPQ_GO(2, false);
}
#undef MPQ_GO

}  // namespace mpq

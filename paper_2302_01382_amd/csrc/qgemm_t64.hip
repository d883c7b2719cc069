// qgemm_t64.hip -- the fast path of mpq_qgemm (qgemm_dma.hpp) instantiated for one tile size; a
// translation unit per tile size so that the sources compile side by side.
#include "qgemm_dma.hpp"

namespace mpq {

#define MPQ_GO(W4) launch_dma<64, 64, 2, 2, 3, W4>(a.a_q, a.w_q, a.M, a.N, a.K, a.a_scale, a.w_scale, a.per_row, a.y_out, a.acc_out, a.st, a.epi, a.n_partials, a.split, a.k_per_split, a.prepare_only)
int launch_dma_64(bool w4, const DmaArgs& a) { return w4 ? MPQ_GO(true) : MPQ_GO(false); }
#undef MPQ_GO

}  // namespace mpq

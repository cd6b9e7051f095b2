// Instantiations of the tile kernels (dsq_tile_impl.h) for one family of compressors.
#include "dsq_tile_impl.h"

namespace dsq {

bool tile_plans_quant8(int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err) {
    return pick_for_kind<DS_COMP_QUANT_MAXABS, 8>(block, n, nnz, plans, err);
}
bool stream_plan_quant8(int block, TilePlan& plan) { return stream_plan_for_block<DS_COMP_QUANT_MAXABS, 8>(block, plan); }

}  // namespace dsq

// Instantiations of the tile kernels (dsq_tile_impl.h) for one family of compressors.
#include "dsq_tile_impl.h"

namespace dsq {

bool tile_plans_sign(int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err) {
    return pick_for_kind<DS_COMP_SIGN_MEANABS, 1>(block, n, nnz, plans, err);
}
bool stream_plan_sign(int block, TilePlan& plan) { return stream_plan_for_block<DS_COMP_SIGN_MEANABS, 1>(block, plan); }

}  // namespace dsq

// Instantiations of the comparison-update tile kernels (dsq_compare_impl.h) for one family of compressors.
#include "dsq_compare_impl.h"

namespace dsq {

bool compare_plans_sign(int algo, int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err) {
    if (algo == kAlgoDcd) return pick_compare_for_kind<DS_COMP_SIGN_MEANABS, 1, kAlgoDcd>(block, n, nnz, plans, err);
    return pick_compare_for_kind<DS_COMP_SIGN_MEANABS, 1, kAlgoChoco>(block, n, nnz, plans, err);
}

}  // namespace dsq

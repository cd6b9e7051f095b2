// Instantiations of the tile kernels (dsq_tile_impl.h) for one family of compressors.
#include "dsq_tile_impl.h"

namespace dsq {

// identity, random sparsifier, and the dispatchers over all families
bool tile_plans_quant4(int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err);
bool tile_plans_quant2(int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err);
bool tile_plans_quant8(int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err);
bool tile_plans_sign(int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err);
bool stream_plan_quant4(int block, TilePlan& plan);
bool stream_plan_quant2(int block, TilePlan& plan);
bool stream_plan_quant8(int block, TilePlan& plan);
bool stream_plan_sign(int block, TilePlan& plan);
// the comparison updates (dsq_compare_*.hip)
bool compare_plans_quant4(int algo, int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err);
bool compare_plans_quant2(int algo, int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err);
bool compare_plans_quant8(int algo, int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err);
bool compare_plans_sign(int algo, int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err);

static_assert(kKeepGroup == 16, "the tile kernel finds a sweep's group with a shift by 4");

void launch_keep_offsets(const TileArgs& a, uint32_t* local_off, uint32_t* group_tot, uint32_t* prev_count, uint32_t* overflow,
                         hipStream_t stream) {
    const uint64_t want = (a.nsweeps + 3) / 4;
    hipLaunchKernelGGL(keep_count_if_stale_kernel, dim3((unsigned)(want < 512 ? want : 512), a.n), dim3(256), 0, stream, a);
    hipLaunchKernelGGL(keep_local_scan_kernel, dim3((unsigned)((a.nsweeps + 255) / 256), a.n), dim3(256), 0, stream, a, local_off, group_tot);
    hipLaunchKernelGGL(keep_scan_kernel, dim3(a.n), dim3(1024), 0, stream, a, group_tot, prev_count, overflow);
}

bool stream_plan(const ds_config& cfg, TilePlan& plan) {
    if (cfg.algo != DS_ALGO_DEEPSQUEEZE) return false;     // the comparison updates exchange fp32 rows through LDS
    if (cfg.comp.kind == DS_COMP_QUANT_MAXABS && cfg.comp.bits == 4) return stream_plan_quant4(cfg.comp.block, plan);
    if (cfg.comp.kind == DS_COMP_QUANT_MAXABS && cfg.comp.bits == 2) return stream_plan_quant2(cfg.comp.block, plan);
    if (cfg.comp.kind == DS_COMP_QUANT_MAXABS && cfg.comp.bits == 8) return stream_plan_quant8(cfg.comp.block, plan);
    if (cfg.comp.kind == DS_COMP_SIGN_MEANABS) return stream_plan_sign(cfg.comp.block, plan);
    if (cfg.comp.kind == DS_COMP_IDENTITY) { plan = make_stream_plan<DS_COMP_IDENTITY, 32, 512>(); return true; }
    return false;
}

bool choose_tile_plans(const ds_config& cfg, int nnz, std::vector<TilePlan>& plan, std::string& err) {
    if (cfg.algo != DS_ALGO_DEEPSQUEEZE) {
        if (cfg.comp.kind == DS_COMP_SIGN_MEANABS) return compare_plans_sign(cfg.algo, cfg.comp.block, cfg.n, nnz, plan, err);
        if (cfg.comp.kind == DS_COMP_QUANT_MAXABS && cfg.comp.bits == 4) return compare_plans_quant4(cfg.algo, cfg.comp.block, cfg.n, nnz, plan, err);
        if (cfg.comp.kind == DS_COMP_QUANT_MAXABS && cfg.comp.bits == 2) return compare_plans_quant2(cfg.algo, cfg.comp.block, cfg.n, nnz, plan, err);
        if (cfg.comp.kind == DS_COMP_QUANT_MAXABS && cfg.comp.bits == 8) return compare_plans_quant8(cfg.algo, cfg.comp.block, cfg.n, nnz, plan, err);
        err = "no comparison kernel for this compressor";
        return false;
    }
    switch (cfg.comp.kind) {
        case DS_COMP_QUANT_MAXABS:
            if (cfg.comp.bits == 4) return tile_plans_quant4(cfg.comp.block, cfg.n, nnz, plan, err);
            if (cfg.comp.bits == 2) return tile_plans_quant2(cfg.comp.block, cfg.n, nnz, plan, err);
            if (cfg.comp.bits == 8) return tile_plans_quant8(cfg.comp.block, cfg.n, nnz, plan, err);
            err = "bits must be 2, 4 or 8";
            return false;
        case DS_COMP_SIGN_MEANABS:
            return tile_plans_sign(cfg.comp.block, cfg.n, nnz, plan, err);
        case DS_COMP_IDENTITY:
            return pick_for_block<DS_COMP_IDENTITY, 32, 512>(cfg.n, nnz, plan, err);
        case DS_COMP_RAND_SPARSE:
            return pick_for_block<DS_COMP_RAND_SPARSE, 32, 512>(cfg.n, nnz, plan, err);
        default:
            err = "no tile kernel for this compressor";
            return false;
    }
}

}  // namespace dsq

// C ABI of libdsq: handle life cycle, state transfer and the ds_step dispatcher.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "dsq_internal.h"

struct ds_handle {
    ds_config cfg{};
    dsq::Graph graph;
    uint64_t ld = 0;                 // row pitch of x and delta, in floats
    uint64_t msg_row_bytes = 0;
    uint64_t msg_half = 0;           // row-streaming variant: bytes of one of the two message buffers (else 0)
    uint64_t t = 0;
    bool stepped = false;
    int device = 0;
    hipStream_t last_stream = nullptr;
    float* x = nullptr;
    float* delta = nullptr;
    uint8_t* msg = nullptr;
    int32_t* d_rowptr = nullptr;
    int32_t* d_col = nullptr;
    float* d_coef = nullptr;
    unsigned long long* d_t = nullptr;   // kStepCells cells; d_t[0]: the step counter t, read and advanced by the
                                         // step's kernels; the rest: the tile kernel's finished-workgroup counters
    dsq::TilePlan tile;
    std::vector<dsq::TilePlan> tile_candidates;
    dsq::TopkState* topk = nullptr;
    dsq::L2State* l2q = nullptr;
    uint32_t* d_keep = nullptr;          // random sparsifier, one allocation: n x nsweeps offsets inside groups,
                                         // n x ngroups group offsets, n previous counts, one overflow flag,
                                         // 2 x n x nsweeps raw counts (steps of even / odd t)
    uint64_t nsweeps = 0, ngroups = 0;
    std::string err;
    std::string plan_name;
};

namespace {

ds_status fail(ds_handle* h, ds_status st, const std::string& msg) {
    if (h) h->err = msg;
    return st;
}

ds_status hip_fail(ds_handle* h, hipError_t e, const char* what) {
    return fail(h, e == hipErrorOutOfMemory ? DS_ENOMEM : DS_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define DSQ_HIP(h, call)                                              \
    do {                                                              \
        hipError_t e_ = (call);                                       \
        if (e_ != hipSuccess) return hip_fail((h), e_, #call);        \
    } while (0)

void release(ds_handle* h) {
    if (!h) return;
    if (h->topk) dsq::topk_destroy(h->topk);
    if (h->l2q) dsq::l2q_destroy(h->l2q);
    if (h->x) (void)hipFree(h->x);
    if (h->delta) (void)hipFree(h->delta);
    if (h->msg) (void)hipFree(h->msg);
    if (h->d_rowptr) (void)hipFree(h->d_rowptr);   // d_col and d_coef point into the same allocation
    if (h->d_t) (void)hipFree(h->d_t);
    if (h->d_keep) (void)hipFree(h->d_keep);
    delete h;
}


dsq::TileArgs tile_args(const ds_handle* h, const float* g_dev, uint64_t g_ld);

// Kernel arguments of the top-k and the norm-rescaled paths, always from the handle's CURRENT buffers, mixing
// matrix and rates (a flush after ds_set_mixing must not see the device addresses of the matrix it replaced).
dsq::TopkArgs topk_args(const ds_handle* h, const float* g_dev, uint64_t g_ld) {
    dsq::TopkArgs a{};
    a.x = h->x; a.delta = h->delta; a.g = g_dev; a.msg = h->msg;
    a.rowptr = h->d_rowptr; a.col = h->d_col; a.coef = h->d_coef;
    a.ld = h->ld; a.g_ld = g_ld; a.N = h->cfg.N; a.k = h->cfg.comp.k; a.n = h->cfg.n;
    a.gamma = h->cfg.gamma; a.eta = h->cfg.eta; a.t_ptr = h->d_t;
    if (h->cfg.comp.kind == DS_COMP_GSPAR) {               // rows of [header pair][capacity pairs]
        a.k = h->msg_row_bytes / 8;
        a.k_expected = h->cfg.comp.k;
        a.seed_lo = (uint32_t)h->cfg.seed; a.seed_hi = (uint32_t)(h->cfg.seed >> 32);
    }
    return a;
}

dsq::L2Args l2_args(const ds_handle* h, const float* g_dev, uint64_t g_ld) {
    dsq::L2Args a{};
    a.x = h->x; a.delta = h->delta; a.g = g_dev; a.msg = h->msg;
    a.rowptr = h->d_rowptr; a.col = h->d_col; a.coef = h->d_coef;
    a.ld = h->ld; a.g_ld = g_ld; a.N = h->cfg.N; a.msg_row_bytes = h->msg_row_bytes; a.n = h->cfg.n;
    a.msg_half = h->msg_half;
    a.gamma = h->cfg.gamma; a.eta = h->cfg.eta; a.t_ptr = h->d_t;
    return a;
}

// Three paths (top-k, norm-rescaled codes, the row-streaming block kernels) leave the tail of a step to the next step's first pass;
// this applies it now, on the stream of the last step.  Callers that replace W, gamma or eta call it BEFORE the
// replacement: the tail belongs to the values the step ran with.
ds_status flush_deferred(ds_handle* h) {
    if (h->topk) return dsq::topk_flush(h->topk, topk_args(h, nullptr, 0), h->last_stream);
    if (h->l2q) return dsq::l2q_flush(h->l2q, l2_args(h, nullptr, 0), h->last_stream);
    if (h->tile.streaming && h->stepped) {
        h->tile.flush(tile_args(h, nullptr, 0), h->last_stream);
        return hipGetLastError() == hipSuccess ? DS_OK : DS_EHIP;
    }
    return DS_OK;
}

dsq::TileArgs tile_args(const ds_handle* h, const float* g_dev, uint64_t g_ld) {
    dsq::TileArgs a{};
    a.x = h->x; a.delta = h->delta; a.g = g_dev; a.msg = h->msg;
    a.rowptr = h->d_rowptr; a.col = h->d_col; a.coef = h->d_coef;
    a.ld = h->ld; a.g_ld = g_ld; a.N = h->cfg.N; a.msg_row_bytes = h->msg_row_bytes;
    a.n = h->cfg.n; a.nnz = (int)h->graph.col.size();
    a.gamma = h->cfg.gamma; a.eta = h->cfg.eta;
    a.seed_lo = (uint32_t)h->cfg.seed; a.seed_hi = (uint32_t)(h->cfg.seed >> 32); a.t_ptr = h->d_t;
    a.msg_half = h->msg_half;
    a.pending = reinterpret_cast<uint32_t*>(h->d_t + 3);        // cell 3: the row-streaming variant's pending flag
    if (h->cfg.comp.kind == DS_COMP_RAND_SPARSE) {
        a.keep_off = h->d_keep;
        a.keep_group_off = h->d_keep + (size_t)h->cfg.n * h->nsweeps;
        a.keep_raw = h->d_keep + (size_t)h->cfg.n * (h->nsweeps + h->ngroups) + h->cfg.n + 1;
        a.nsweeps = h->nsweeps;
        a.ngroups = h->ngroups;
        a.keep_thr = (uint32_t)((h->cfg.comp.k << 24) / h->cfg.N);        // floor(k 2^24 / N) <= 2^24
        a.msg_cap = (uint32_t)((h->msg_row_bytes - 4) / 4);
    }
    return a;
}

// Row pitch candidates (floats added to N rounded up to kPitchAlign).  A tile kernel has all n rows
// of a column window in flight at once, so how the row pitch falls on the HBM channel hash decides
// up to 12 % of the achieved bandwidth, and the best pitch differs between shapes and GPUs.  ds_init
// times the real kernel on the (still all-zero) state for each candidate and keeps the fastest.
const uint64_t kPitchCandidates[] = {0, 2560, 4096, 6656, 8192, 12288};
constexpr uint64_t kMaxPitchSkew = 12288;

// Times `plan` at the current h->ld on the all-zero state (3 launches, twice, after a warm-up); < 0 on failure.
float time_plan(ds_handle* h, const dsq::TilePlan& plan, const float* g, hipEvent_t e0, hipEvent_t e1) {
    const dsq::TileArgs a = tile_args(h, g, h->ld);
    plan.launch(a, plan.rows_per_wave, nullptr);
    float best = 1e30f;
    for (int rep = 0; rep < 2; ++rep) {                        // the better of two timings: less noise in the choice
        (void)hipEventRecord(e0, nullptr);
        for (int r = 0; r < 3; ++r) plan.launch(a, plan.rows_per_wave, nullptr);
        (void)hipEventRecord(e1, nullptr);
        float ms = 0.f;
        if (hipGetLastError() != hipSuccess) return -1.f;      // a launch that was refused would look fast
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1.f;
        best = ms < best ? ms : best;
    }
    return best;
}

// Picks the launch shape (at the default pitch) and then the row pitch for it by timing the real
// kernel.  Returns the chosen skew and sets h->tile; leaves x, delta and the messages zeroed.
uint64_t autotune(ds_handle* h, uint64_t base_ld, size_t state_bytes, size_t msg_bytes) {
    float* g = nullptr;
    if (hipMalloc(&g, state_bytes) != hipSuccess) { (void)hipGetLastError(); return dsq::kPitchSkew; }
    hipEvent_t e0, e1;
    bool ok = hipMemset(g, 0, state_bytes) == hipSuccess && hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
    uint64_t best_skew = dsq::kPitchSkew;
    if (ok) {
        float best_ms = 1e30f;
        h->ld = base_ld + dsq::kPitchSkew;
        // A later candidate (or, below, another pitch) must win by 2 % to be taken: differences below that are
        // timing noise, and a choice that flips between near-equal candidates from run to run makes measurements
        // hard to compare.
        for (const dsq::TilePlan& plan : h->tile_candidates) {
            const float ms = time_plan(h, plan, g, e0, e1);
            if (ms < 0.f) { ok = false; break; }
            if (ms < 0.98f * best_ms) { best_ms = ms; h->tile = plan; }
        }
        for (uint64_t skew : kPitchCandidates) {
            if (!ok) break;
            if (skew == dsq::kPitchSkew) continue;             // timed above
            h->ld = base_ld + skew;
            const float ms = time_plan(h, h->tile, g, e0, e1);
            if (ms < 0.f) { ok = false; break; }
            if (ms < 0.98f * best_ms) { best_ms = ms; best_skew = skew; }
        }
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
    }
    (void)hipDeviceSynchronize();
    (void)hipFree(g);
    (void)hipMemset(h->x, 0, state_bytes);
    (void)hipMemset(h->delta, 0, state_bytes);
    (void)hipMemset(h->msg, 0, msg_bytes ? msg_bytes : 4);
    (void)hipMemset(h->d_t, 0, dsq::kStepCells * sizeof(unsigned long long));   // the timed launches advanced t
    (void)hipMemset(h->d_t + 2, 0xFF, sizeof(unsigned long long));              // ... and no keep counts are valid
    (void)hipDeviceSynchronize();
    if (!ok) h->tile = h->tile_candidates.front();
    return ok ? best_skew : dsq::kPitchSkew;
}

// Diagnostics (off the hot path): a thread walks all rows of its columns (grid-stride); fp64 accumulation.
__global__ void __launch_bounds__(256) diagnostics_kernel(const float* __restrict__ x, const float* __restrict__ delta, uint64_t ld,
                                                          uint64_t N, int n, const int32_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ col, const float* __restrict__ coef,
                                                          float eta, double* __restrict__ out) {
    __shared__ double part[3][4];
    double cons = 0.0, dsq_ = 0.0, mixed = 0.0;
    for (uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x; j < N; j += (uint64_t)gridDim.x * 256) {
        double sum = 0.0, sumsq = 0.0;
        for (int i = 0; i < n; ++i) {
            const double xv = x[(uint64_t)i * ld + j];
            const double dv = delta[(uint64_t)i * ld + j];
            sum += xv;
            sumsq += xv * xv;
            dsq_ += dv * dv;
        }
        const double mean = sum / n;
        for (int i = 0; i < n; ++i) {                           // second pass: no cancellation
            const double dev = (double)x[(uint64_t)i * ld + j] - mean;
            cons += dev * dev;
            double m = 0.0;
            for (int e = rowptr[i]; e < rowptr[i + 1]; ++e) m += (double)coef[e] * (double)delta[(uint64_t)col[e] * ld + j];
            m *= (double)eta;
            mixed += m * m;
        }
        (void)sumsq;
    }
    double v[3] = {cons, dsq_, mixed};
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int q = 0; q < 3; ++q) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v[q] += __shfl_xor(v[q], o);
        if (lane == 0) part[q][wave] = v[q];
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        const double tot = part[threadIdx.x][0] + part[threadIdx.x][1] + part[threadIdx.x][2] + part[threadIdx.x][3];
        atomicAdd(&out[threadIdx.x], tot);
    }
}

// Plain streaming copy, one 16-byte non-temporal load and store per lane, one-shot grid: the
// yardstick for the HBM bandwidth a trivial kernel reaches.
typedef float f32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) copy_kernel(f32x4* __restrict__ dst, const f32x4* __restrict__ src, uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// The access mix of ds_step without its arithmetic: three 16-byte non-temporal loads and two stores per lane,
// in place (x += g, delta += g): what a streaming kernel of this shape reaches on the same GPU.
__global__ void __launch_bounds__(256) stream_3r2w_kernel(f32x4* __restrict__ x, f32x4* __restrict__ d, const f32x4* __restrict__ g, uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) {
        const f32x4 gv = __builtin_nontemporal_load(g + i);
        const f32x4 xv = __builtin_nontemporal_load(x + i);
        const f32x4 dv = __builtin_nontemporal_load(d + i);
        __builtin_nontemporal_store(xv + gv, x + i);
        __builtin_nontemporal_store(dv + gv, d + i);
    }
}

// The same for the DCD-PSGD step, which has no second state array: two loads, one store.
__global__ void __launch_bounds__(256) stream_2r1w_kernel(f32x4* __restrict__ x, const f32x4* __restrict__ g, uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) {
        const f32x4 gv = __builtin_nontemporal_load(g + i);
        const f32x4 xv = __builtin_nontemporal_load(x + i);
        __builtin_nontemporal_store(xv + gv, x + i);
    }
}

// ---- ds_step_static: one step with no handle and no allocation ------------------------------------------------
// Everything the fused tile kernel needs beyond the caller's arrays -- the step-counter cells with its
// finished-workgroup counters, and W - I in CSR form -- lives in this file-scope device array.  Every GPU the
// library runs on holds its own copy until the process ends.  In host code the array's name is only a stand-in:
// its device address is asked for once per device (static_scratch) and that pointer is what kernels get.
constexpr int kStaticMaxWorkers = 1024;
constexpr int kStaticMaxDegree = 5;                                           // ring 3, torus 5 (diagonal included)
constexpr size_t kStaticGraphWords = (size_t)kStaticMaxWorkers + 1 + 2 * (size_t)kStaticMaxDegree * kStaticMaxWorkers;
constexpr size_t kStaticCellBytes = dsq::kStepCells * sizeof(unsigned long long);
constexpr size_t kStaticBytes = kStaticCellBytes + kStaticGraphWords * sizeof(int32_t);   // 16,640 + 45,060 bytes
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (asked for on the first call per device); nullptr on failure.
unsigned char* static_scratch(int device, std::string& err) {
    if (device < 0 || device >= kMaxDevices) { err = "device index beyond the 64 this entry point keeps an address for"; return nullptr; }
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e); return nullptr; }
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    return g_scratch_ptr[device];
}

// One workgroup: the step-counter cells (t, everything else zero, no keep counts) and the CSR of W - I of a
// ring or a 2-D torus, rows in ascending neighbour index as ds_init builds them.
__global__ void __launch_bounds__(256) static_setup_kernel(unsigned char* base, int n, int topo, int torus_rows, int torus_cols,
                                                           float w, float w_diag, unsigned long long t) {
    unsigned long long* cells = reinterpret_cast<unsigned long long*>(base);
    for (size_t q = threadIdx.x; q < dsq::kStepCells; q += 256) cells[q] = (q == 0) ? t : (q == 2) ? ~0ull : 0ull;
    const int deg = (topo == DS_TOPO_RING) ? 3 : 5;
    int32_t* rowptr = reinterpret_cast<int32_t*>(base + kStaticCellBytes);
    int32_t* col = rowptr + n + 1;
    float* coef = reinterpret_cast<float*>(col + (size_t)deg * n);
    for (int i = threadIdx.x; i <= n; i += 256) rowptr[i] = deg * i;
    for (int i = threadIdx.x; i < n; i += 256) {
        int nb[5];
        if (topo == DS_TOPO_RING) {
            nb[0] = (i + n - 1) % n; nb[1] = i; nb[2] = (i + 1) % n;
        } else {
            const int r = i / torus_cols, c = i % torus_cols;
            nb[0] = i;
            nb[1] = ((r + 1) % torus_rows) * torus_cols + c;
            nb[2] = ((r + torus_rows - 1) % torus_rows) * torus_cols + c;
            nb[3] = r * torus_cols + (c + 1) % torus_cols;
            nb[4] = r * torus_cols + (c + torus_cols - 1) % torus_cols;
        }
        for (int a = 1; a < deg; ++a)                                          // ascending neighbour index
            for (int b = a; b > 0 && nb[b - 1] > nb[b]; --b) { const int tmp = nb[b]; nb[b] = nb[b - 1]; nb[b - 1] = tmp; }
        for (int e = 0; e < deg; ++e) {
            col[(size_t)deg * i + e] = nb[e];
            coef[(size_t)deg * i + e] = (nb[e] == i) ? w_diag : w;
        }
    }
}

}  // namespace

extern "C" {

ds_status ds_step_static(const ds_config* cfg, float* x_dev, float* delta_dev, uint64_t ld, const float* g_dev, uint64_t g_ld,
                         void* msg_dev, uint64_t t, void* hip_stream, char* errbuf, uint64_t errbuf_len) {
    std::string err, warn;
    auto fail_with = [&](ds_status st, const std::string& m) {
        if (errbuf && errbuf_len) std::snprintf(errbuf, (size_t)errbuf_len, "%s", m.c_str());
        return st;
    };
    if (dsq::validate_config(cfg, err, &warn) != DS_OK) return fail_with(DS_EINVAL, err);
    const int kind = cfg->comp.kind;
    if (cfg->algo != DS_ALGO_DEEPSQUEEZE) return fail_with(DS_EINVAL, "ds_step_static serves Algorithm 1 (DS_ALGO_DEEPSQUEEZE) only");
    if (kind != DS_COMP_QUANT_MAXABS && kind != DS_COMP_SIGN_MEANABS && kind != DS_COMP_IDENTITY)
        return fail_with(DS_EINVAL, "ds_step_static serves the block quantiser, the sign compressor and the identity only "
                                    "(the other compressors need scratch memory in proportion to N)");
    if (cfg->topo != DS_TOPO_RING && cfg->topo != DS_TOPO_TORUS2D)
        return fail_with(DS_EINVAL, "ds_step_static builds W on the device: DS_TOPO_RING or DS_TOPO_TORUS2D only");
    if (cfg->n > kStaticMaxWorkers)
        return fail_with(DS_EINVAL, "ds_step_static: n exceeds the 1024 workers its static scratch array has room for");
    if (!x_dev || !delta_dev || !g_dev || !msg_dev) return fail_with(DS_EINVAL, "a device pointer is NULL");
    if ((ld & 3) || ld < (cfg->N + dsq::kPitchAlign - 1) / dsq::kPitchAlign * dsq::kPitchAlign)
        return fail_with(DS_EINVAL, "ld must be a multiple of 4 and at least N rounded up to a multiple of 4096");
    if (g_ld < cfg->N || (g_ld & 3)) return fail_with(DS_EINVAL, "g_ld must be >= N and a multiple of 4");
    if ((reinterpret_cast<uintptr_t>(x_dev) | reinterpret_cast<uintptr_t>(delta_dev) | reinterpret_cast<uintptr_t>(g_dev)) & 15)
        return fail_with(DS_EINVAL, "x_dev, delta_dev and g_dev must be 16-byte aligned");
    if (reinterpret_cast<uintptr_t>(msg_dev) & 3) return fail_with(DS_EINVAL, "msg_dev must be 4-byte aligned");
    const int deg = cfg->topo == DS_TOPO_RING ? 3 : 5;
    const int nnz = deg * cfg->n;
    std::vector<dsq::TilePlan> plans;
    if (!dsq::choose_tile_plans(*cfg, nnz, plans, err)) return fail_with(DS_EINVAL, err);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return fail_with(DS_EHIP, "no current HIP device");
    unsigned char* base = static_scratch(dev, err);
    if (!base) return fail_with(DS_EHIP, err);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const float w = (cfg->topo == DS_TOPO_RING) ? 1.0f / 3.0f : 1.0f / 5.0f;
    hipLaunchKernelGGL(static_setup_kernel, dim3(1), dim3(256), 0, stream, base, cfg->n, cfg->topo, cfg->torus_rows,
                       cfg->torus_cols, w, w - 1.0f, (unsigned long long)t);
    dsq::TileArgs a{};
    a.x = x_dev; a.delta = delta_dev; a.g = g_dev; a.msg = static_cast<uint8_t*>(msg_dev);
    a.rowptr = reinterpret_cast<const int32_t*>(base + kStaticCellBytes);
    a.col = a.rowptr + cfg->n + 1;
    a.coef = reinterpret_cast<const float*>(a.col + nnz);
    a.ld = ld; a.g_ld = g_ld; a.N = cfg->N; a.msg_row_bytes = dsq::message_row_bytes(cfg);
    a.n = cfg->n; a.nnz = nnz;
    a.gamma = cfg->gamma; a.eta = cfg->eta;
    a.seed_lo = (uint32_t)cfg->seed; a.seed_hi = (uint32_t)(cfg->seed >> 32);
    a.t_ptr = reinterpret_cast<unsigned long long*>(base);
    a.pending = reinterpret_cast<uint32_t*>(a.t_ptr + 3);
    const dsq::TilePlan& plan = plans.front();
    plan.launch(a, plan.rows_per_wave, stream);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_with(DS_EHIP, std::string("launching the step failed: ") + hipGetErrorString(e));
    if (errbuf && errbuf_len) std::snprintf(errbuf, (size_t)errbuf_len, "%s", warn.c_str());
    return DS_OK;
}

ds_status ds_workload_gradient(const ds_workload* w, uint64_t t, const float* x_dev, uint64_t x_ld, float* g_dev,
                               uint64_t g_ld, void* hip_stream) {
    if (!w || !g_dev || w->n < 1 || w->N < 1 || w->N > 0xFFFFFFF0ull || g_ld < w->N) return DS_EINVAL;
    if (w->kind < DS_GRAD_NORMAL || w->kind > DS_GRAD_QUADRATIC || !std::isfinite(w->scale)) return DS_EINVAL;
    if (w->kind == DS_GRAD_QUADRATIC && (!x_dev || x_ld < w->N)) return DS_EINVAL;
    return dsq::launch_workload_gradient(*w, t, x_dev, x_ld, g_dev, g_ld, static_cast<hipStream_t>(hip_stream));
}

ds_status ds_bench_stream(void* x_dev, void* delta_dev, const void* g_dev, uint64_t bytes, void* hip_stream) {
    if (!x_dev || !g_dev || (bytes & 15) ||
        ((reinterpret_cast<uintptr_t>(x_dev) | reinterpret_cast<uintptr_t>(delta_dev) | reinterpret_cast<uintptr_t>(g_dev)) & 15))
        return DS_EINVAL;
    const uint64_t n4 = bytes / 16;
    if (n4 == 0) return DS_OK;
    if (n4 > 0xFFFFFF00ull) return DS_EINVAL;
    if (!delta_dev) {
        hipLaunchKernelGGL(stream_2r1w_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                           static_cast<f32x4*>(x_dev), static_cast<const f32x4*>(g_dev), n4);
        return hipGetLastError() == hipSuccess ? DS_OK : DS_EHIP;
    }
    hipLaunchKernelGGL(stream_3r2w_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<f32x4*>(x_dev), static_cast<f32x4*>(delta_dev), static_cast<const f32x4*>(g_dev), n4);
    return hipGetLastError() == hipSuccess ? DS_OK : DS_EHIP;
}

ds_status ds_bench_copy(void* dst_dev, const void* src_dev, uint64_t bytes, void* hip_stream) {
    if (!dst_dev || !src_dev || (bytes & 15) || ((reinterpret_cast<uintptr_t>(dst_dev) | reinterpret_cast<uintptr_t>(src_dev)) & 15))
        return DS_EINVAL;
    const uint64_t n4 = bytes / 16;
    if (n4 == 0) return DS_OK;
    if (n4 > 0xFFFFFF00ull) return DS_EINVAL;              // one work-item per 16 bytes, fewer than 2^32 of them
    const unsigned blocks = (unsigned)((n4 + 255) / 256);
    hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<f32x4*>(dst_dev), static_cast<const f32x4*>(src_dev), n4);
    return hipGetLastError() == hipSuccess ? DS_OK : DS_EHIP;
}

ds_status ds_init(const ds_config* cfg, ds_handle** out) { return ds_init_ex(cfg, nullptr, nullptr, 0, out); }

ds_status ds_init_ex(const ds_config* cfg, const ds_plan_request* plan, char* errbuf, uint64_t errbuf_len, ds_handle** out) {
    if (errbuf && errbuf_len) errbuf[0] = 0;
    if (!out) return DS_EINVAL;
    *out = nullptr;
    ds_handle* h = new (std::nothrow) ds_handle();
    if (!h) return DS_ENOMEM;
    auto bail = [&](ds_status st, const std::string& why) {
        if (errbuf && errbuf_len) std::snprintf(errbuf, (size_t)errbuf_len, "%s", why.c_str());
        release(h);
        return st;
    };
    ds_plan_request want{};                                 // all automatic
    want.tile_plan = -1; want.pitch_skew = -1; want.autotune = 1;
    if (plan) {
        want = *plan;
        if (want.variant < 0 || want.variant > 1) return bail(DS_EINVAL, "plan: variant must be 0 (automatic) or 1 (row-streaming)");
        if (want.pitch_skew < -1 || want.pitch_skew > (int64_t)kMaxPitchSkew || (want.pitch_skew > 0 && (want.pitch_skew & 3)))
            return bail(DS_EINVAL, "plan: pitch_skew must be -1 (automatic) or a multiple of 4 up to 12288");
    }

    std::string err, warn;
    if (dsq::validate_config(cfg, err, &warn) != DS_OK) return bail(DS_EINVAL, err);
    h->cfg = *cfg;
    if (dsq::build_graph(cfg, h->graph, err) != DS_OK) return bail(DS_EINVAL, err);
    h->cfg.W_rowptr = nullptr; h->cfg.W_col = nullptr; h->cfg.W_val = nullptr;   // the copy lives in graph
    const uint64_t base_ld = (cfg->N + dsq::kPitchAlign - 1) / dsq::kPitchAlign * dsq::kPitchAlign;
    h->ld = base_ld + kMaxPitchSkew;                       // allocation pitch; the working pitch is fixed below
    h->msg_row_bytes = dsq::message_row_bytes(cfg);

    const bool sparse_pairs = cfg->comp.kind == DS_COMP_TOPK || cfg->comp.kind == DS_COMP_GSPAR;   // (column, value) messages
    const bool tiled = !sparse_pairs && cfg->comp.kind != DS_COMP_QUANT_L2NORM;
    if (cfg->comp.kind == DS_COMP_GSPAR) {
        h->plan_name = "gspar/sift-scan-write";
    } else if (cfg->comp.kind == DS_COMP_TOPK) {
        h->plan_name = "topk/radix-select";
    } else if (cfg->comp.kind == DS_COMP_QUANT_L2NORM) {
        h->plan_name = "l2norm/speculative-codes";
        h->msg_half = (uint64_t)cfg->n * h->msg_row_bytes;     // the first pass writes codes while the old ones are still read
    } else {
        // the row-streaming variant of the block compressors on request; it is also what serves a number of
        // workers whose codes do not fit in LDS
        dsq::TilePlan sp;
        const bool can_stream = dsq::stream_plan(h->cfg, sp);
        const bool fits = dsq::choose_tile_plans(h->cfg, (int)h->graph.col.size(), h->tile_candidates, err);
        if (can_stream && (!fits || want.variant == 1)) {
            h->tile_candidates.assign(1, sp);
            h->msg_half = (uint64_t)cfg->n * h->msg_row_bytes;
        } else if (!fits) {
            return bail(DS_EINVAL, err);
        }
        h->tile = h->tile_candidates.front();
        // a pinned candidate launch shape (tests walk through all of them; an index past the end leaves the choice automatic)
        if (want.tile_plan >= 0 && (size_t)want.tile_plan < h->tile_candidates.size()) {
            h->tile = h->tile_candidates[(size_t)want.tile_plan];
            h->tile_candidates.assign(1, h->tile);
        }
    }

    hipError_t e = hipGetDevice(&h->device);
    if (e != hipSuccess) return bail(DS_EHIP, std::string("no HIP device: ") + hipGetErrorString(e));
    const size_t state_bytes = (size_t)cfg->n * h->ld * sizeof(float);
    const size_t nnz = h->graph.col.size();
    const size_t msg_bytes = (size_t)cfg->n * h->msg_row_bytes * (h->msg_half ? 2 : 1);
    // rowptr | col | coef as one contiguous array of 32-bit words
    hipError_t errs[5] = {
        hipMalloc(&h->x, state_bytes), hipMalloc(&h->delta, state_bytes), hipMalloc(&h->msg, msg_bytes ? msg_bytes : 4),
        hipMalloc(&h->d_rowptr, (cfg->n + 1 + 2 * nnz) * sizeof(int32_t)), hipMalloc(&h->d_t, dsq::kStepCells * sizeof(unsigned long long))};
    for (hipError_t ee : errs)
        if (ee != hipSuccess) { (void)hipGetLastError(); return bail(ee == hipErrorOutOfMemory ? DS_ENOMEM : DS_EHIP, std::string("hipMalloc: ") + hipGetErrorString(ee)); }
    h->d_col = h->d_rowptr + cfg->n + 1;
    h->d_coef = reinterpret_cast<float*>(h->d_col + nnz);
    bool ok = hipMemset(h->x, 0, state_bytes) == hipSuccess && hipMemset(h->delta, 0, state_bytes) == hipSuccess &&
              hipMemset(h->msg, 0, msg_bytes ? msg_bytes : 4) == hipSuccess &&
              hipMemset(h->d_t, 0, dsq::kStepCells * sizeof(unsigned long long)) == hipSuccess &&
              hipMemset(h->d_t + 2, 0xFF, sizeof(unsigned long long)) == hipSuccess &&   // tag of the keep counts: none yet
              hipMemcpy(h->d_rowptr, h->graph.rowptr.data(), (cfg->n + 1) * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(h->d_col, h->graph.col.data(), nnz * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(h->d_coef, h->graph.coef.data(), nnz * sizeof(float), hipMemcpyHostToDevice) == hipSuccess &&
              hipDeviceSynchronize() == hipSuccess;
    if (!ok) return bail(DS_EHIP, "device initialisation failed");
    if (cfg->comp.kind == DS_COMP_RAND_SPARSE) {
        h->nsweeps = (cfg->N + dsq::kSweep - 1) / dsq::kSweep;
        h->ngroups = (h->nsweeps + 15) / 16;
        const size_t words = (size_t)cfg->n * (3 * h->nsweeps + h->ngroups) + (size_t)cfg->n + 1;
        if (hipMalloc(&h->d_keep, words * sizeof(uint32_t)) != hipSuccess || hipMemset(h->d_keep, 0, words * sizeof(uint32_t)) != hipSuccess ||
            hipDeviceSynchronize() != hipSuccess) {
            return bail(DS_ENOMEM, "allocating the random sparsifier's offsets failed");
        }
    }

    // working row pitch: pinned by the caller, or timed per candidate for large tile-kernel problems; everything
    // else takes the default
    uint64_t skew = dsq::kPitchSkew;
    if (want.pitch_skew >= 0) {
        skew = (uint64_t)want.pitch_skew;
    } else if (want.autotune && tiled && !h->tile.streaming && (uint64_t)cfg->n * cfg->N >= (32ull << 20)) {
        skew = autotune(h, base_ld, state_bytes, msg_bytes);
    }
    h->ld = base_ld + skew;
    if (tiled)
        h->plan_name = std::string(cfg->algo == DS_ALGO_DCD_PSGD ? "dcd/" : cfg->algo == DS_ALGO_CHOCO_SGD ? "choco/" : "") + h->tile.name + "/" +
                       std::to_string(h->tile.sweeps) + "sweeps";
    h->plan_name += "/pitch+" + std::to_string(skew);

    if (sparse_pairs) {
        const ds_status st = dsq::topk_create(h->cfg, h->ld, &h->topk, err);
        if (st != DS_OK) return bail(st, err);
    }
    if (cfg->comp.kind == DS_COMP_QUANT_L2NORM) {
        const ds_status st = dsq::l2q_create(h->cfg, h->ld, &h->l2q, err);
        if (st != DS_OK) return bail(st, err);
    }
    h->err = warn;
    if (errbuf && errbuf_len) std::snprintf(errbuf, (size_t)errbuf_len, "%s", warn.c_str());
    *out = h;
    return DS_OK;
}

ds_status ds_step(ds_handle* h, const float* g_dev, uint64_t g_ld, void* hip_stream) {
    if (!h) return DS_EINVAL;
    if (!g_dev) return fail(h, DS_EINVAL, "g_dev is NULL");
    if (g_ld < h->cfg.N || (g_ld & 3)) return fail(h, DS_EINVAL, "g_ld must be >= N and a multiple of 4");
    if (reinterpret_cast<uintptr_t>(g_dev) & 15) return fail(h, DS_EINVAL, "g_dev must be 16-byte aligned");
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != h->device)
        return fail(h, DS_ESTATE, "the current HIP device is not the one the handle was created on");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    if (h->topk) {
        const ds_status st = dsq::topk_step(h->topk, topk_args(h, g_dev, g_ld), stream);
        if (st != DS_OK) return st;
    } else if (h->cfg.comp.kind == DS_COMP_QUANT_L2NORM) {
        const ds_status st = dsq::l2q_step(h->l2q, l2_args(h, g_dev, g_ld), stream);
        if (st != DS_OK) return fail(h, st, "launching the norm-rescaled step failed");
    } else {
        const dsq::TileArgs a = tile_args(h, g_dev, g_ld);
        if (h->cfg.comp.kind == DS_COMP_RAND_SPARSE) {
            uint32_t* groups = h->d_keep + (size_t)h->cfg.n * h->nsweeps;
            uint32_t* prev = groups + (size_t)h->cfg.n * h->ngroups;
            dsq::launch_keep_offsets(a, h->d_keep, groups, prev, prev + h->cfg.n, stream);
        }
        h->tile.launch(a, h->tile.rows_per_wave, stream);
    }
    DSQ_HIP(h, hipGetLastError());
    h->t += 1;
    h->stepped = true;
    h->last_stream = stream;
    return DS_OK;
}

ds_status ds_set_mixing(ds_handle* h, const int32_t* W_rowptr, const int32_t* W_col, const float* W_val) {
    if (!h) return DS_EINVAL;
    ds_config probe = h->cfg;
    probe.topo = DS_TOPO_CSR;
    probe.W_rowptr = W_rowptr; probe.W_col = W_col; probe.W_val = W_val;
    std::string err;
    if (dsq::validate_config(&probe, err, nullptr) != DS_OK) return fail(h, DS_EINVAL, err);
    dsq::Graph g;
    if (dsq::build_graph(&probe, g, err) != DS_OK) return fail(h, DS_EINVAL, err);
    const size_t nnz = g.col.size();
    if (!h->topk && !h->l2q && !h->tile.streaming) {
        // the launch shape was chosen for the old graph; the new CSR only has to fit in LDS next to the codes
        std::vector<dsq::TilePlan> plans;
        if (!dsq::choose_tile_plans(h->cfg, (int)nnz, plans, err)) return fail(h, DS_EINVAL, err);
    }
    // a deferred tail belongs to the old W: apply it first
    if (flush_deferred(h) != DS_OK) return fail(h, DS_EHIP, "applying the deferred tail of the last step failed");
    DSQ_HIP(h, hipStreamSynchronize(h->last_stream));
    // same number of stored entries: overwrite in place, so that the device addresses (and a HIP graph captured
    // from ds_step with them) stay valid
    const bool in_place = nnz == h->graph.col.size();
    int32_t* packed = h->d_rowptr;
    if (!in_place) DSQ_HIP(h, hipMalloc(&packed, (h->cfg.n + 1 + 2 * nnz) * sizeof(int32_t)));
    hipError_t e = hipMemcpy(packed, g.rowptr.data(), (h->cfg.n + 1) * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(packed + h->cfg.n + 1, g.col.data(), nnz * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(packed + h->cfg.n + 1 + nnz, g.coef.data(), nnz * sizeof(float), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (!in_place) (void)hipFree(packed);
        return hip_fail(h, e, "hipMemcpy(W)");
    }
    if (!in_place) (void)hipFree(h->d_rowptr);
    h->d_rowptr = packed;
    h->d_col = packed + h->cfg.n + 1;
    h->d_coef = reinterpret_cast<float*>(h->d_col + nnz);
    h->graph = g;
    h->cfg.topo = DS_TOPO_CSR;
    return DS_OK;
}

ds_status ds_set_rates(ds_handle* h, float gamma, float eta) {
    if (!h) return DS_EINVAL;
    if (!std::isfinite(gamma) || !std::isfinite(eta)) return fail(h, DS_EINVAL, "gamma and eta must be finite");
    // a deferred tail was computed for the old eta
    if (flush_deferred(h) != DS_OK) return fail(h, DS_EHIP, "applying the deferred tail of the last step failed");
    h->cfg.gamma = gamma;
    h->cfg.eta = eta;
    h->err = (eta > 0.5f) ? "warning: eta > 1/2, outside the range of the paper's Theorem 1 (W_eff may not be PSD)" : "";
    return DS_OK;
}

// Dense host array <-> pitched device rows.  Rows of more than 1 GiB go one by one (2-D copies of such widths
// are not something every runtime version handles).
static hipError_t copy_rows(void* dst, size_t dst_pitch, const void* src, size_t src_pitch, size_t row_bytes, int rows, hipMemcpyKind kind) {
    if (row_bytes <= (1ull << 30)) return hipMemcpy2D(dst, dst_pitch, src, src_pitch, row_bytes, rows, kind);
    for (int i = 0; i < rows; ++i) {
        const hipError_t e = hipMemcpy(static_cast<char*>(dst) + (size_t)i * dst_pitch, static_cast<const char*>(src) + (size_t)i * src_pitch,
                                       row_bytes, kind);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

ds_status ds_read_state(ds_handle* h, float* x_host, float* delta_host) {
    if (!h) return DS_EINVAL;
    if (!x_host && !delta_host) return fail(h, DS_EINVAL, "nothing to read");
    if (flush_deferred(h) != DS_OK) return fail(h, DS_EHIP, "applying the deferred tail of the last step failed");
    DSQ_HIP(h, hipStreamSynchronize(h->last_stream));
    const size_t row = h->cfg.N * sizeof(float), pitch = h->ld * sizeof(float);
    if (x_host) DSQ_HIP(h, copy_rows(x_host, row, h->x, pitch, row, h->cfg.n, hipMemcpyDeviceToHost));
    if (delta_host) DSQ_HIP(h, copy_rows(delta_host, row, h->delta, pitch, row, h->cfg.n, hipMemcpyDeviceToHost));
    return DS_OK;
}

ds_status ds_write_state(ds_handle* h, const float* x_host, const float* delta_host, uint64_t t) {
    if (!h) return DS_EINVAL;
    if (flush_deferred(h) != DS_OK) return fail(h, DS_EHIP, "applying the deferred tail of the last step failed");
    DSQ_HIP(h, hipStreamSynchronize(h->last_stream));
    const size_t row = h->cfg.N * sizeof(float), pitch = h->ld * sizeof(float);
    if (x_host) DSQ_HIP(h, copy_rows(h->x, pitch, x_host, row, row, h->cfg.n, hipMemcpyHostToDevice));
    if (delta_host) DSQ_HIP(h, copy_rows(h->delta, pitch, delta_host, row, row, h->cfg.n, hipMemcpyHostToDevice));
    const unsigned long long t64 = t;
    DSQ_HIP(h, hipMemcpy(h->d_t, &t64, sizeof(t64), hipMemcpyHostToDevice));
    DSQ_HIP(h, hipDeviceSynchronize());
    h->t = t;
    return DS_OK;
}

// Plans with two message buffers (row-streaming block kernels, norm-rescaled codes): a step leaves the number of
// the buffer it wrote in cell 4 of the step cells.  The caller has synchronised.
static ds_status last_message_buffer(ds_handle* h, uint8_t** out) {
    *out = h->msg;
    if (!h->msg_half) return DS_OK;
    unsigned long long half = 0;
    DSQ_HIP(h, hipMemcpy(&half, h->d_t + 4, sizeof(half), hipMemcpyDeviceToHost));
    if (half & 1ull) *out = h->msg + h->msg_half;
    return DS_OK;
}

ds_status ds_read_messages(ds_handle* h, void* host_buf, uint64_t cap, uint64_t* bytes) {
    if (!h) return DS_EINVAL;
    if (!h->stepped) return fail(h, DS_ESTATE, "no step has been taken yet");
    const uint64_t total = h->msg_row_bytes * (uint64_t)h->cfg.n;
    if (bytes) *bytes = total;
    if (!host_buf || cap < total) return fail(h, DS_EINVAL, "message buffer too small");
    DSQ_HIP(h, hipStreamSynchronize(h->last_stream));
    uint8_t* src = nullptr;
    if (last_message_buffer(h, &src) != DS_OK) return DS_EHIP;
    DSQ_HIP(h, hipMemcpy(host_buf, src, total, hipMemcpyDeviceToHost));
    if (h->cfg.comp.kind == DS_COMP_GSPAR) {
        bool over = false;
        if (dsq::gspar_overflowed(h->topk, h->last_stream, &over) != DS_OK) return DS_EHIP;
        if (over) return fail(h, DS_ESTATE, "a worker kept more elements than its message has room for: the messages since then are cut short");
    }
    if (h->d_keep) {
        uint32_t overflow = 0;
        DSQ_HIP(h, hipMemcpy(&overflow, h->d_keep + (size_t)h->cfg.n * (h->nsweeps + h->ngroups) + h->cfg.n, sizeof(overflow), hipMemcpyDeviceToHost));
        if (overflow) return fail(h, DS_ESTATE, "a worker kept more values than its message has room for (x and delta are unaffected)");
    }
    return DS_OK;
}

ds_status ds_state_ptrs(ds_handle* h, float** x_dev, float** delta_dev, uint64_t* ld) {
    if (!h) return DS_EINVAL;
    // top-k keeps the sparse part of the last gossip update pending; complete x before lending it
    if (flush_deferred(h) != DS_OK) return fail(h, DS_EHIP, "applying the deferred tail of the last step failed");
    if (x_dev) *x_dev = h->x;
    if (delta_dev) *delta_dev = h->delta;
    if (ld) *ld = h->ld;
    return DS_OK;
}

ds_status ds_message_ptr(ds_handle* h, void** msg_dev, uint64_t* bytes) {
    if (!h) return DS_EINVAL;
    uint8_t* src = h->msg;
    if (h->msg_half) {                                       // which of the two buffers is the last step's: ask the device
        DSQ_HIP(h, hipStreamSynchronize(h->last_stream));
        if (last_message_buffer(h, &src) != DS_OK) return DS_EHIP;
    }
    if (msg_dev) *msg_dev = src;
    if (bytes) *bytes = h->msg_row_bytes * (uint64_t)h->cfg.n;
    return DS_OK;
}

ds_status ds_diagnostics(ds_handle* h, double* out4) {
    if (!h || !out4) return DS_EINVAL;
    if (flush_deferred(h) != DS_OK) return fail(h, DS_EHIP, "applying the deferred tail of the last step failed");
    DSQ_HIP(h, hipStreamSynchronize(h->last_stream));
    double* d_out = nullptr;
    DSQ_HIP(h, hipMalloc(&d_out, 3 * sizeof(double)));
    hipError_t e = hipMemset(d_out, 0, 3 * sizeof(double));
    if (e == hipSuccess) {
        const uint64_t want = (h->cfg.N + 255) / 256;
        const unsigned blocks = (unsigned)(want < (1u << 20) ? want : (1u << 20));
        hipLaunchKernelGGL(diagnostics_kernel, dim3(blocks), dim3(256), 0, nullptr, h->x, h->delta, h->ld, h->cfg.N, h->cfg.n,
                           h->d_rowptr, h->d_col, h->d_coef, h->cfg.eta, d_out);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpy(out4, d_out, 3 * sizeof(double), hipMemcpyDeviceToHost);
    (void)hipFree(d_out);
    if (e != hipSuccess) return hip_fail(h, e, "ds_diagnostics");
    out4[3] = (double)(h->msg_row_bytes * (uint64_t)h->cfg.n);
    return DS_OK;
}

ds_status ds_topk_candidate_rows(ds_handle* h, uint32_t* count) {
    if (!h || !count) return DS_EINVAL;
    *count = 0;
    if (!h->topk && !h->l2q) return DS_OK;
    if (!h->stepped) return fail(h, DS_ESTATE, "no step has been taken yet");
    if (h->l2q) return dsq::l2q_speculated_rows(h->l2q, h->last_stream, count);
    return dsq::topk_candidate_rows(h->topk, h->last_stream, count);
}

uint64_t ds_step_count(const ds_handle* h) {
    // the device counter is the authority: replays of a captured graph advance it without the host seeing them
    if (!h) return 0;
    unsigned long long t64 = h->t;
    if (hipStreamSynchronize(h->last_stream) == hipSuccess)
        (void)hipMemcpy(&t64, h->d_t, sizeof(t64), hipMemcpyDeviceToHost);
    return t64;
}

const char* ds_plan_name(const ds_handle* h) { return h ? h->plan_name.c_str() : ""; }

const char* ds_last_error(const ds_handle* h) { return h ? h->err.c_str() : "handle is NULL"; }

void ds_destroy(ds_handle* h) {
    if (!h) return;
    (void)hipDeviceSynchronize();
    release(h);
}

}  // extern "C"

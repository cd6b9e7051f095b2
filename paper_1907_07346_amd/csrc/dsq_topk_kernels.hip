// Top-k path of libdsq (gfx950): exact magnitude select per worker row, ordered packing of the
// (index, value) message, residual write-back and the sparse gossip update.
//
// DeepSqueeze's Algorithm 1 with C_omega = top-k (one of the operators the paper lists under
// Assumption 1.6): line 5 forms v, line 6 keeps the k largest |v| (ties to the lower index) and
// leaves everything else in delta, lines 7-8 "send" the k pairs, line 9 mixes the neighbours'
// sparse vectors into x.
//
// The select is an MSB-first radix select on key = bits(v) & 0x7fffffff (order preserving for
// finite |v|): 11 + 11 + 9 bits with workgroup histograms in LDS.  The first histogram is fused
// into the pass that forms v; the exact threshold key tau and the number r_tie of elements equal
// to tau that still belong to the set come out of three tiny per-row select kernels.  Ordered
// output (ascending index, needed for the tie rule and for a canonical message) comes from
// per-chunk counts, a per-row scan over chunks and an in-chunk ordered compaction.

#include "dsq_internal.h"

namespace dsq {

namespace {

constexpr int TK_THREADS = 256;
constexpr int TK_VEC = 4 * TK_THREADS;       // elements per workgroup iteration
constexpr int TK_ITERS = 8;
constexpr int TK_CHUNK = TK_VEC * TK_ITERS;  // columns per chunk (one workgroup)
constexpr int BINS1 = 2048, SHIFT1 = 20;     // key bits 30..20
constexpr int BINS2 = 2048, SHIFT2 = 9;      // key bits 19..9
constexpr int BINS3 = 512;                   // key bits 8..0
constexpr int HIST_BINS = 2048;

struct TopkRow {
    uint32_t prefix1, need1;   // level-1 bin holding the threshold; how many to take inside it
    uint32_t prefix2, need2;   // 22-bit prefix of the threshold key; how many to take among its matches
    uint32_t tau, r_tie;       // threshold key; number of elements with key == tau to take (lowest indices)
    uint32_t total;            // number of selected elements found by the scan (must equal k)
    uint32_t pad;
};

__device__ __forceinline__ uint32_t key_of(float v) { return __float_as_uint(v) & 0x7FFFFFFFu; }

// Exclusive prefix sum over the 256 threads of a workgroup; *total receives the sum.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_sums /*[4]*/, uint32_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(inc, o);
        if (lane >= o) inc += up;
    }
    __syncthreads();                       // wave_sums may still be read from a previous call
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < TK_THREADS / 64; ++w) {
        const uint32_t s = wave_sums[w];
        if (w < wave) base += s;
        tot += s;
    }
    *total = tot;
    return base + inc - v;
}

__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t* wave_sums) {
    uint32_t tot;
    (void)block_exclusive_scan(v, wave_sums, &tot);
    return tot;
}

// ---- pass 1: Algorithm 1 line 5 (x <- x - gamma g, delta <- v) + level-1 histogram ------------
__global__ void __launch_bounds__(TK_THREADS) topk_form_hist1(TopkArgs a, uint32_t* __restrict__ hist) {
    __shared__ uint32_t h[HIST_BINS];
    const int row = blockIdx.y;
    const uint64_t c0 = (uint64_t)blockIdx.x * TK_CHUNK;
    for (int b = threadIdx.x; b < HIST_BINS; b += TK_THREADS) h[b] = 0;
    __syncthreads();
    float* xr = a.x + (uint64_t)row * a.ld;
    float* dr = a.delta + (uint64_t)row * a.ld;
    const float* gr = a.g + (uint64_t)row * a.g_ld;
#pragma unroll 2
    for (int it = 0; it < TK_ITERS; ++it) {
        const uint64_t j = c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x;
        if (j >= a.ld) break;
        const float4 xv = *reinterpret_cast<const float4*>(xr + j);
        const float4 dv = *reinterpret_cast<const float4*>(dr + j);
        float4 gv;
        if (j + 3 < a.N) {
            gv = *reinterpret_cast<const float4*>(gr + j);
        } else {
            gv.x = (j + 0 < a.N) ? gr[j + 0] : 0.f;
            gv.y = (j + 1 < a.N) ? gr[j + 1] : 0.f;
            gv.z = (j + 2 < a.N) ? gr[j + 2] : 0.f;
            gv.w = (j + 3 < a.N) ? gr[j + 3] : 0.f;
        }
        float4 xh, v;
        xh.x = fmaf(-a.gamma, gv.x, xv.x); v.x = xh.x + dv.x;
        xh.y = fmaf(-a.gamma, gv.y, xv.y); v.y = xh.y + dv.y;
        xh.z = fmaf(-a.gamma, gv.z, xv.z); v.z = xh.z + dv.z;
        xh.w = fmaf(-a.gamma, gv.w, xv.w); v.w = xh.w + dv.w;
        // x holds xh + eta*0 until the gossip kernel patches the columns some neighbour sent
        xh.x += 0.f; xh.y += 0.f; xh.z += 0.f; xh.w += 0.f;
        *reinterpret_cast<float4*>(xr + j) = xh;
        *reinterpret_cast<float4*>(dr + j) = v;
        if (j + 0 < a.N) atomicAdd(&h[key_of(v.x) >> SHIFT1], 1u);
        if (j + 1 < a.N) atomicAdd(&h[key_of(v.y) >> SHIFT1], 1u);
        if (j + 2 < a.N) atomicAdd(&h[key_of(v.z) >> SHIFT1], 1u);
        if (j + 3 < a.N) atomicAdd(&h[key_of(v.w) >> SHIFT1], 1u);
    }
    __syncthreads();
    uint32_t* hrow = hist + (size_t)row * HIST_BINS;
    for (int b = threadIdx.x; b < HIST_BINS; b += TK_THREADS)
        if (h[b]) atomicAdd(&hrow[b], h[b]);
}

// ---- passes 2 and 3: histogram of the next digit among keys matching the prefix so far ---------
template <int LEVEL>
__global__ void __launch_bounds__(TK_THREADS) topk_hist_level(const float* __restrict__ delta, uint64_t ld, uint64_t N,
                                                              const TopkRow* __restrict__ rows, uint32_t* __restrict__ hist,
                                                              uint32_t* __restrict__ cnt_gt, uint32_t* __restrict__ cnt_eq,
                                                              uint32_t nchunks) {
    __shared__ uint32_t h[HIST_BINS];
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.y;
    const uint64_t c0 = (uint64_t)blockIdx.x * TK_CHUNK;
    constexpr int BINS = (LEVEL == 2) ? BINS2 : BINS3;
    for (int b = threadIdx.x; b < BINS; b += TK_THREADS) h[b] = 0;
    __syncthreads();
    const uint32_t prefix = (LEVEL == 2) ? rows[row].prefix1 : rows[row].prefix2;
    const float* dr = delta + (uint64_t)row * ld;
    uint32_t gt = 0, eq = 0;
#pragma unroll 2
    for (int it = 0; it < TK_ITERS; ++it) {
        const uint64_t j = c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x;
        if (j >= ld) break;
        const float4 v = *reinterpret_cast<const float4*>(dr + j);
        const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (j + c < N) {
                const uint32_t key = key_of(vv[c]);
                if (LEVEL == 2) {
                    if ((key >> SHIFT1) == prefix) atomicAdd(&h[(key >> SHIFT2) & (BINS2 - 1)], 1u);
                } else {
                    const uint32_t hi = key >> SHIFT2;
                    if (hi == prefix) { atomicAdd(&h[key & (BINS3 - 1)], 1u); ++eq; }
                    else if (hi > prefix) ++gt;
                }
            }
        }
    }
    __syncthreads();
    uint32_t* hrow = hist + (size_t)row * HIST_BINS;
    for (int b = threadIdx.x; b < BINS; b += TK_THREADS)
        if (h[b]) atomicAdd(&hrow[b], h[b]);
    if (LEVEL == 3) {
        const uint32_t gts = block_sum(gt, wave_sums);
        const uint32_t eqs = block_sum(eq, wave_sums);
        if (threadIdx.x == 0) {
            cnt_gt[(size_t)row * nchunks + blockIdx.x] = gts;
            cnt_eq[(size_t)row * nchunks + blockIdx.x] = eqs;
        }
    }
}

// ---- per-row digit select: the bin where the count from the top crosses `need` -----------------
template <int LEVEL>
__global__ void __launch_bounds__(TK_THREADS) topk_select(uint32_t* __restrict__ hist, TopkRow* __restrict__ rows, uint32_t k) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.x;
    constexpr int BINS = (LEVEL == 1) ? BINS1 : (LEVEL == 2) ? BINS2 : BINS3;
    constexpr int PER = HIST_BINS / TK_THREADS;           // 8 consecutive bins per thread
    uint32_t* hrow = hist + (size_t)row * HIST_BINS;
    TopkRow& r = rows[row];
    const uint32_t need = (LEVEL == 1) ? k : (LEVEL == 2) ? r.need1 : r.need2;
    // thread t owns bins [top - 8t - 7, top - 8t], i.e. threads are ordered from the largest keys down
    uint32_t mine[PER];
    uint32_t sum = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int b = HIST_BINS - 1 - (threadIdx.x * PER + q);
        mine[q] = (b < BINS) ? hrow[b] : 0u;
        sum += mine[q];
    }
    uint32_t total;
    uint32_t above = block_exclusive_scan(sum, wave_sums, &total);   // keys in strictly higher bins
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int b = HIST_BINS - 1 - (threadIdx.x * PER + q);
        if (above < need && need <= above + mine[q]) {
            const uint32_t rem = need - above;
            if (LEVEL == 1)      { r.prefix1 = (uint32_t)b; r.need1 = rem; }
            else if (LEVEL == 2) { r.prefix2 = (r.prefix1 << (SHIFT1 - SHIFT2)) | (uint32_t)b; r.need2 = rem; }
            else                 { r.tau = (r.prefix2 << SHIFT2) | (uint32_t)b; r.r_tie = rem; }
        }
        above += mine[q];
        if (b < HIST_BINS) hrow[b] = 0;                   // leave the histogram clean for the next pass
    }
}

// ---- exact per-chunk counts: only chunks that hold a key with the threshold's 22-bit prefix -----
__global__ void __launch_bounds__(TK_THREADS) topk_fix_counts(const float* __restrict__ delta, uint64_t ld, uint64_t N,
                                                              const TopkRow* __restrict__ rows, uint32_t* __restrict__ cnt_gt,
                                                              uint32_t* __restrict__ cnt_eq, uint32_t nchunks) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.y;
    const size_t ci = (size_t)row * nchunks + blockIdx.x;
    if (cnt_eq[ci] == 0) return;                          // uniform: nothing in this chunk can tie or straddle
    const uint32_t tau = rows[row].tau;
    const uint64_t c0 = (uint64_t)blockIdx.x * TK_CHUNK;
    const float* dr = delta + (uint64_t)row * ld;
    uint32_t gt = 0, eq = 0;
    for (int it = 0; it < TK_ITERS; ++it) {
        const uint64_t j = c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x;
        if (j >= ld) break;
        const float4 v = *reinterpret_cast<const float4*>(dr + j);
        const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (j + c < N) {
                const uint32_t key = key_of(vv[c]);
                gt += key > tau;
                eq += key == tau;
            }
    }
    const uint32_t gts = block_sum(gt, wave_sums);
    const uint32_t eqs = block_sum(eq, wave_sums);
    if (threadIdx.x == 0) { cnt_gt[ci] = gts; cnt_eq[ci] = eqs; }
}

// ---- per-row scan over chunks: tie quota and output offset of every chunk -----------------------
__global__ void __launch_bounds__(TK_THREADS) topk_scan_chunks(TopkRow* __restrict__ rows, const uint32_t* __restrict__ cnt_gt,
                                                               const uint32_t* __restrict__ cnt_eq, uint32_t* __restrict__ eq_before,
                                                               uint32_t* __restrict__ out_off, uint32_t nchunks) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.x;
    const uint32_t r_tie = rows[row].r_tie;
    const uint32_t* gt = cnt_gt + (size_t)row * nchunks;
    const uint32_t* eq = cnt_eq + (size_t)row * nchunks;
    uint32_t* eqb = eq_before + (size_t)row * nchunks;
    uint32_t* off = out_off + (size_t)row * (nchunks + 1);
    uint32_t run_eq = 0, run_out = 0;
    for (uint32_t base = 0; base < nchunks; base += TK_THREADS) {
        const uint32_t c = base + threadIdx.x;
        const uint32_t e = (c < nchunks) ? eq[c] : 0u;
        const uint32_t g = (c < nchunks) ? gt[c] : 0u;
        uint32_t tot_e, tot_o;
        const uint32_t before = run_eq + block_exclusive_scan(e, wave_sums, &tot_e);
        const uint32_t quota = (before < r_tie) ? (r_tie - before) : 0u;
        const uint32_t take = g + (e < quota ? e : quota);
        const uint32_t o = run_out + block_exclusive_scan(take, wave_sums, &tot_o);
        if (c < nchunks) { eqb[c] = before; off[c] = o; }
        run_eq += tot_e;
        run_out += tot_o;
    }
    if (threadIdx.x == 0) { off[nchunks] = run_out; rows[row].total = run_out; }
}

// ---- ordered compaction: message pairs, delta <- 0 on the selected set (Algorithm 1, line 6) ----
__global__ void __launch_bounds__(TK_THREADS) topk_write_selected(TopkArgs a, const TopkRow* __restrict__ rows,
                                                                  const uint32_t* __restrict__ cnt_eq,
                                                                  const uint32_t* __restrict__ eq_before,
                                                                  const uint32_t* __restrict__ out_off, uint32_t nchunks) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.y;
    const size_t ci = (size_t)row * nchunks + blockIdx.x;
    const uint32_t off0 = out_off[(size_t)row * (nchunks + 1) + blockIdx.x];
    const uint32_t off1 = out_off[(size_t)row * (nchunks + 1) + blockIdx.x + 1];
    if (off0 == off1) return;
    const bool ties = cnt_eq[ci] != 0;
    const uint32_t tau = rows[row].tau, r_tie = rows[row].r_tie;
    uint32_t run_eq = eq_before[ci], run_out = off0;
    const uint64_t c0 = (uint64_t)blockIdx.x * TK_CHUNK;
    float* dr = a.delta + (uint64_t)row * a.ld;
    uint2* out = reinterpret_cast<uint2*>(a.msg + (uint64_t)row * a.k * 8);
    for (int it = 0; it < TK_ITERS; ++it) {
        const uint64_t j = c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x;
        if (c0 + (uint64_t)it * TK_VEC >= a.ld) break;     // uniform
        float vv[4] = {0.f, 0.f, 0.f, 0.f};
        if (j < a.ld) {
            const float4 v = *reinterpret_cast<const float4*>(dr + j);
            vv[0] = v.x; vv[1] = v.y; vv[2] = v.z; vv[3] = v.w;
        }
        bool sel[4];
        uint32_t neq = 0;
        bool iseq[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool live = (j + c < a.N);
            const uint32_t key = key_of(vv[c]);
            sel[c] = live && key > tau;
            iseq[c] = live && key == tau;
            neq += iseq[c];
        }
        if (ties) {                                         // uniform per chunk
            uint32_t tot;
            uint32_t rank = run_eq + block_exclusive_scan(neq, wave_sums, &tot);
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (iseq[c]) { sel[c] = rank < r_tie; ++rank; }
            run_eq += tot;
        }
        const uint32_t nsel = (uint32_t)sel[0] + sel[1] + sel[2] + sel[3];
        uint32_t tot;
        uint32_t pos = run_out + block_exclusive_scan(nsel, wave_sums, &tot);
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (sel[c]) {
                if (pos < a.k) out[pos] = make_uint2((uint32_t)(j + c), __float_as_uint(vv[c]));
                ++pos;
                dr[j + c] = 0.f;                            // v - C[v] = v - v
            }
        run_out += tot;
    }
}

// ---- gossip on the sparse messages (Algorithm 1, line 9) ----------------------------------------
// One workgroup per (row, chunk): the neighbours' pairs that fall into the chunk are contiguous in
// their messages (out_off), so they are accumulated in ascending neighbour order into an LDS copy
// of the chunk and then applied once per touched column.
__global__ void __launch_bounds__(TK_THREADS) topk_gossip(TopkArgs a, const uint32_t* __restrict__ out_off, uint32_t nchunks) {
    __shared__ float acc[TK_CHUNK];
    __shared__ uint32_t taken[TK_CHUNK / 32];
    const int row = blockIdx.y;
    const uint32_t c = blockIdx.x;
    const uint64_t c0 = (uint64_t)c * TK_CHUNK;
    const int e0 = a.rowptr[row], e1 = a.rowptr[row + 1];
    bool any = false;
    for (int e = e0; e < e1; ++e) {
        const uint32_t* off = out_off + (size_t)a.col[e] * (nchunks + 1) + c;
        any |= (off[0] != off[1]);
    }
    if (!any) return;                                       // uniform
    for (int q = threadIdx.x; q < TK_CHUNK; q += TK_THREADS) acc[q] = 0.f;
    for (int q = threadIdx.x; q < TK_CHUNK / 32; q += TK_THREADS) taken[q] = 0u;
    __syncthreads();
    for (int e = e0; e < e1; ++e) {
        const int nb = a.col[e];
        const float w = a.coef[e];
        const uint32_t* off = out_off + (size_t)nb * (nchunks + 1) + c;
        const uint2* in = reinterpret_cast<const uint2*>(a.msg + (uint64_t)nb * a.k * 8);
        for (uint32_t p = off[0] + threadIdx.x; p < off[1]; p += TK_THREADS) {
            const uint2 pr = in[p];
            const uint32_t q = (uint32_t)((uint64_t)pr.x - c0);
            if (q < (uint32_t)TK_CHUNK) acc[q] = fmaf(w, __uint_as_float(pr.y), acc[q]);
        }
        __syncthreads();
    }
    float* xr = a.x + (uint64_t)row * a.ld;
    for (int e = e0; e < e1; ++e) {
        const int nb = a.col[e];
        const uint32_t* off = out_off + (size_t)nb * (nchunks + 1) + c;
        const uint2* in = reinterpret_cast<const uint2*>(a.msg + (uint64_t)nb * a.k * 8);
        for (uint32_t p = off[0] + threadIdx.x; p < off[1]; p += TK_THREADS) {
            const uint32_t jj = in[p].x;
            const uint32_t q = (uint32_t)((uint64_t)jj - c0);
            if (q >= (uint32_t)TK_CHUNK || jj >= a.N) continue;
            const uint32_t bit = 1u << (q & 31);
            const uint32_t old = atomicOr(&taken[q >> 5], bit);
            if (!(old & bit)) xr[jj] = fmaf(a.eta, acc[q], xr[jj]);
        }
    }
}

}  // namespace

struct TopkState {
    uint32_t nchunks = 0;
    int n = 0;
    uint32_t* hist = nullptr;
    TopkRow* rows = nullptr;
    uint32_t* cnt_gt = nullptr;
    uint32_t* cnt_eq = nullptr;
    uint32_t* eq_before = nullptr;
    uint32_t* out_off = nullptr;
};

void topk_destroy(TopkState* s) {
    if (!s) return;
    void* ptrs[] = {s->hist, s->rows, s->cnt_gt, s->cnt_eq, s->eq_before, s->out_off};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    delete s;
}

ds_status topk_create(const ds_config& cfg, uint64_t /*ld*/, TopkState** out, std::string& err) {
    TopkState* s = new TopkState();
    s->n = cfg.n;
    s->nchunks = (uint32_t)((cfg.N + TK_CHUNK - 1) / TK_CHUNK);
    const size_t n = (size_t)cfg.n, nc = s->nchunks;
    bool ok = hipMalloc(&s->hist, n * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s->rows, n * sizeof(TopkRow)) == hipSuccess &&
              hipMalloc(&s->cnt_gt, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s->cnt_eq, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s->eq_before, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s->out_off, n * (nc + 1) * sizeof(uint32_t)) == hipSuccess;
    ok = ok && hipMemset(s->hist, 0, n * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s->rows, 0, n * sizeof(TopkRow)) == hipSuccess && hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        err = "top-k scratch allocation failed";
        topk_destroy(s);
        return DS_ENOMEM;
    }
    *out = s;
    return DS_OK;
}

ds_status topk_step(TopkState* s, const TopkArgs& a, const Graph& /*graph*/, hipStream_t stream, std::string& /*err*/) {
    const dim3 grid(s->nchunks, a.n), block(TK_THREADS);
    const dim3 rows(a.n);
    hipLaunchKernelGGL(topk_form_hist1, grid, block, 0, stream, a, s->hist);
    hipLaunchKernelGGL(topk_select<1>, rows, block, 0, stream, s->hist, s->rows, (uint32_t)a.k);
    hipLaunchKernelGGL(topk_hist_level<2>, grid, block, 0, stream, a.delta, a.ld, a.N, s->rows, s->hist, s->cnt_gt, s->cnt_eq, s->nchunks);
    hipLaunchKernelGGL(topk_select<2>, rows, block, 0, stream, s->hist, s->rows, (uint32_t)a.k);
    hipLaunchKernelGGL(topk_hist_level<3>, grid, block, 0, stream, a.delta, a.ld, a.N, s->rows, s->hist, s->cnt_gt, s->cnt_eq, s->nchunks);
    hipLaunchKernelGGL(topk_select<3>, rows, block, 0, stream, s->hist, s->rows, (uint32_t)a.k);
    hipLaunchKernelGGL(topk_fix_counts, grid, block, 0, stream, a.delta, a.ld, a.N, s->rows, s->cnt_gt, s->cnt_eq, s->nchunks);
    hipLaunchKernelGGL(topk_scan_chunks, rows, block, 0, stream, s->rows, s->cnt_gt, s->cnt_eq, s->eq_before, s->out_off, s->nchunks);
    hipLaunchKernelGGL(topk_write_selected, grid, block, 0, stream, a, s->rows, s->cnt_eq, s->eq_before, s->out_off, s->nchunks);
    hipLaunchKernelGGL(topk_gossip, grid, block, 0, stream, a, s->out_off, s->nchunks);
    return DS_OK;
}

}  // namespace dsq

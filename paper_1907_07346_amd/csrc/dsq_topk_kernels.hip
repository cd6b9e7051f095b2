// Top-k path of libdsq (gfx950): exact magnitude select per worker row, ordered packing of the
// (index, value) message, residual write-back and the sparse gossip update.
//
// DeepSqueeze's Algorithm 1 with C_omega = top-k (one of the operators the paper lists under
// Assumption 1.6): line 5 forms v, line 6 keeps the k largest |v| (ties to the lower index) and
// leaves everything else in delta, lines 7-8 "send" the k pairs, line 9 mixes the neighbours'
// sparse vectors into x.
//
// The select is an MSB-first radix select on key = bits(v) & 0x7fffffff (order preserving for
// finite |v|): 11 + 11 + 9 bits, workgroup histograms in LDS, three tiny per-row select kernels
// that end with the exact threshold key tau and the number r_tie of elements equal to tau that
// still belong to the set.  Ordered output (ascending index: the tie rule and a canonical
// message need it) comes from per-chunk counts, a per-row scan over chunks and an ordered
// compaction inside each chunk.
//
// Two sources feed the select, chosen per row on the device with no host round trip:
//   * candidate mode (the fast path): the pass that forms v also appends every element whose key
//     reaches a per-row guess `tlo` (extrapolated from the previous steps' thresholds, aimed at
//     about 3 k elements) to a small per-chunk slot.  If at least k candidates were collected
//     and no slot overflowed, the whole select runs on the slots (a few % of N) and v is never
//     read again.
//   * full mode (always exact, used on the first step and whenever the guess fails): the same
//     select with histogram passes over v itself.
// Both end in the same tau, r_tie, per-chunk counts and message, so results never depend on the
// guess; only speed does.
//
// The sparse tail of a step is deferred: the first pass writes x = (x - gamma g) + 0 and
// delta = v, which already are the final values of every column nobody sent; the remainder --
// delta = 0 where this worker sent v (line 6) and eta * sum_j a_ij C[v_j] where a neighbour did
// (line 9) -- is folded into the NEXT step's first pass (which streams x and delta anyway), or
// applied by topk_flush before anyone else looks at the state.

#include "dsq_internal.h"

namespace dsq {

namespace {

constexpr int TK_THREADS = 256;
constexpr int TK_VEC = 4 * TK_THREADS;       // elements per workgroup iteration
constexpr int TK_ITERS = 4;
constexpr int TK_CHUNK = TK_VEC * TK_ITERS;  // columns per chunk (one workgroup of the streaming passes)
constexpr int TK_CAP = 512;                  // candidate slots per chunk (12.5 % of the chunk)
constexpr int TK_H1 = 256;                   // level-1 bins the first pass tracks, counted from tlo's bin upwards
constexpr int TK_CPW = 8;                    // chunks per workgroup in topk_fix_cand
constexpr int TK_FPW = 8;                    // chunks per workgroup in the full-mode kernels (few, cheap-to-skip workgroups)
constexpr int TK_HWG = 16;                   // workgroups per row in the candidate-mode histogram passes
constexpr int TK_HTHREADS = 1024;            // threads of those workgroups
constexpr int BINS1 = 2048, SHIFT1 = 20;     // key bits 30..20
constexpr int BINS2 = 2048, SHIFT2 = 9;      // key bits 19..9
constexpr int BINS3 = 512;                   // key bits 8..0
constexpr int HIST_BINS = 2048;

struct TopkRow {
    uint32_t prefix1, need1;   // level-1 bin holding the threshold; how many to take inside it
    uint32_t prefix2, need2;   // 22-bit prefix of the threshold key; how many to take among its matches
    uint32_t tau, r_tie;       // threshold key; number of elements with key == tau to take (lowest indices)
    uint32_t total;            // number of selected elements found by the scan (must equal k)
    uint32_t tlo;              // candidate threshold key for the next first pass (0xffffffff: collect nothing)
    uint32_t cand_mode;        // 1: this step's select runs on the candidate slots
    uint32_t overflow;         // a slot overflowed in this step's first pass
    uint32_t cand_total;       // candidates collected in this step
    uint32_t tlo_used;         // the threshold this step's first pass collected with
    uint32_t tau_prev;         // threshold key of the previous step (0xffffffff: none yet)
    uint32_t pad;
};

typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld4_stream(const float* p) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4_stream(float* p, const float4& v) {
    const f32x4 w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<f32x4*>(p));
}

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

struct Scratch {               // device pointers of the select's scratch (all owned by TopkState)
    uint32_t* hist;            // n x 2048
    TopkRow* rows;             // n
    uint32_t* cnt_gt;          // n x nchunks: keys above the threshold (prefix) in the chunk
    uint32_t* cnt_eq;          // n x nchunks: keys equal to the threshold (prefix) in the chunk
    uint32_t* eq_before;       // n x nchunks: ties in earlier chunks of the row
    uint32_t* out_off;         // n x (nchunks+1): message offset of each chunk
    uint32_t* cand_cnt;        // n x nchunks: candidates stored in the chunk's slot
    uint32_t* slot_val;        // n x nchunks x TK_CAP candidate values (fp32 bits), unordered inside a slot; the select
                               // passes read only these
    uint16_t* slot_idx;        // same shape: the candidates' columns, relative to the start of the chunk
    uint32_t nchunks;
};

// ---- pass 1: pending gossip of the previous step, Algorithm 1 line 5, candidate collection ------
__global__ void __launch_bounds__(TK_THREADS) topk_form_collect(TopkArgs a, Scratch s) {
    __shared__ float acc[TK_CHUNK];
    __shared__ uint32_t own[TK_CHUNK / 32];       // columns this worker itself sent in the previous step
    __shared__ uint32_t h[TK_H1];                              // level-1 digits of the candidates, relative to tlo's
    __shared__ uint32_t cand_count;
    const int row = blockIdx.y;
    const uint32_t chunk = blockIdx.x;
    const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
    if (threadIdx.x == 0) cand_count = 0;
    for (int b = threadIdx.x; b < TK_H1; b += TK_THREADS) h[b] = 0;
    // all dense loads of the chunk go out first (12 x 16 bytes per lane); the sparse tail of the previous
    // step is gathered while they are in flight
    float* xr = a.x + (uint64_t)row * a.ld;
    float* dr = a.delta + (uint64_t)row * a.ld;
    const float* gr = a.g + (uint64_t)row * a.g_ld;
    float4 xin[TK_ITERS], din[TK_ITERS], gin[TK_ITERS];
#pragma unroll
    for (int it = 0; it < TK_ITERS; ++it) {
        const uint64_t j = c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x;
        xin[it] = din[it] = gin[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j < a.ld) {
            xin[it] = ld4_stream(xr + j);
            din[it] = ld4_stream(dr + j);
            if (j + 3 < a.N) {
                gin[it] = ld4_stream(gr + j);
            } else {
                gin[it].x = (j + 0 < a.N) ? gr[j + 0] : 0.f;
                gin[it].y = (j + 1 < a.N) ? gr[j + 1] : 0.f;
                gin[it].z = (j + 2 < a.N) ? gr[j + 2] : 0.f;
                gin[it].w = (j + 3 < a.N) ? gr[j + 3] : 0.f;
            }
        }
    }
    bool patch = false;
    {
        // eta * sum_j a_ij C[v_j] of the previous step for this chunk: the neighbours' pairs that fall
        // into the chunk are contiguous in their messages; accumulate neighbour after neighbour.
        const int e0 = a.rowptr[row], e1 = a.rowptr[row + 1];
        for (int e = e0; e < e1; ++e) {
            const uint32_t* off = s.out_off + (size_t)a.col[e] * (s.nchunks + 1) + chunk;
            patch |= (off[0] != off[1]);
        }
        if (patch) {                                           // uniform
            for (int q = threadIdx.x; q < TK_CHUNK; q += TK_THREADS) acc[q] = 0.f;
            for (int q = threadIdx.x; q < TK_CHUNK / 32; q += TK_THREADS) own[q] = 0u;
            __syncthreads();
            for (int e = e0; e < e1; ++e) {
                const int nb = a.col[e];
                const float w = a.coef[e];
                const uint32_t* off = s.out_off + (size_t)nb * (s.nchunks + 1) + chunk;
                const uint2* in = reinterpret_cast<const uint2*>(a.msg + (uint64_t)nb * a.k * 8);
                for (uint32_t p = off[0] + threadIdx.x; p < off[1]; p += TK_THREADS) {
                    const uint2 pr = in[p];
                    const uint32_t q = (uint32_t)((uint64_t)pr.x - c0);
                    if (q < (uint32_t)TK_CHUNK) {
                        acc[q] = fmaf(w, __uint_as_float(pr.y), acc[q]);
                        if (nb == row) atomicOr(&own[q >> 5], 1u << (q & 31));
                    }
                }
                __syncthreads();
            }
        }
    }
    __syncthreads();
    const uint32_t tlo = s.rows[row].tlo;
    const uint32_t bin0 = tlo >> SHIFT1;                       // (0xfff for "collect nothing")
    bool far = false;                                          // a candidate beyond the tracked bins
    uint32_t* slot_val = s.slot_val + ((size_t)row * s.nchunks + chunk) * TK_CAP;
    uint16_t* slot_idx = s.slot_idx + ((size_t)row * s.nchunks + chunk) * TK_CAP;
#pragma unroll
    for (int it = 0; it < TK_ITERS; ++it) {
        const uint32_t q0 = (uint32_t)it * TK_VEC + 4 * threadIdx.x;
        const uint64_t j = c0 + q0;
        if (j >= a.ld) break;
        float4 xv = xin[it], dv = din[it];
        const float4 gv = gin[it];
        if (patch) {                                // lines 6 and 9 of the previous step
            xv.x = fmaf(a.eta, acc[q0 + 0], xv.x); xv.y = fmaf(a.eta, acc[q0 + 1], xv.y);
            xv.z = fmaf(a.eta, acc[q0 + 2], xv.z); xv.w = fmaf(a.eta, acc[q0 + 3], xv.w);
            const uint32_t sent = own[q0 >> 5] >> (q0 & 31);   // delta = v - C[v] = 0 where v was sent
            if (sent & 1u) dv.x = 0.f;
            if (sent & 2u) dv.y = 0.f;
            if (sent & 4u) dv.z = 0.f;
            if (sent & 8u) dv.w = 0.f;
        }
        float4 xh, v;
        xh.x = fmaf(-a.gamma, gv.x, xv.x); v.x = xh.x + dv.x;
        xh.y = fmaf(-a.gamma, gv.y, xv.y); v.y = xh.y + dv.y;
        xh.z = fmaf(-a.gamma, gv.z, xv.z); v.z = xh.z + dv.z;
        xh.w = fmaf(-a.gamma, gv.w, xv.w); v.w = xh.w + dv.w;
        // x holds xh + eta*0 until the sparse part of line 9 is applied
        xh.x += 0.f; xh.y += 0.f; xh.z += 0.f; xh.w += 0.f;
        st4_stream(xr + j, xh);
        st4_stream(dr + j, v);
        const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (j + c < a.N && key_of(vv[c]) >= tlo) {
                const uint32_t idx = atomicAdd(&cand_count, 1u);
                if (idx < (uint32_t)TK_CAP) { slot_val[idx] = __float_as_uint(vv[c]); slot_idx[idx] = (uint16_t)(q0 + c); }
                const uint32_t rel = (key_of(vv[c]) >> SHIFT1) - bin0;
                if (rel < (uint32_t)TK_H1) atomicAdd(&h[rel], 1u); else far = true;
            }
    }
    __syncthreads();
    // the row histogram is used if the row ends up in candidate mode and wiped by topk_decide otherwise;
    // a candidate beyond the tracked bins (256 bins = 2^32 in magnitude above tlo) sends the row there too
    uint32_t* hrow = s.hist + (size_t)row * HIST_BINS;
    for (int b = threadIdx.x; b < TK_H1; b += TK_THREADS)
        if (h[b]) atomicAdd(&hrow[bin0 + b], h[b]);
    if (far) atomicOr(&s.rows[row].overflow, 1u);
    if (threadIdx.x == 0) {
        const uint32_t c = cand_count;
        s.cand_cnt[(size_t)row * s.nchunks + chunk] = c < (uint32_t)TK_CAP ? c : (uint32_t)TK_CAP;
        if (c > (uint32_t)TK_CAP) atomicOr(&s.rows[row].overflow, 1u);
    }
}

// ---- per row: did the guess work?  (candidates >= k and no slot overflow) ----------------------
__global__ void __launch_bounds__(TK_THREADS) topk_decide(Scratch s, uint32_t k) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.x;
    uint32_t sum = 0;
    for (uint32_t c = threadIdx.x; c < s.nchunks; c += TK_THREADS) sum += s.cand_cnt[(size_t)row * s.nchunks + c];
    const uint32_t total = block_sum(sum, wave_sums);
    const bool cand = total >= k && s.rows[row].overflow == 0;
    if (!cand)                                             // full mode builds its own level-1 histogram
        for (int b = threadIdx.x; b < HIST_BINS; b += TK_THREADS) s.hist[(size_t)row * HIST_BINS + b] = 0;
    __syncthreads();
    if (threadIdx.x == 0) {
        TopkRow& r = s.rows[row];
        r.cand_total = total;
        r.cand_mode = cand ? 1u : 0u;
        r.overflow = 0;
        r.tlo_used = r.tlo;
    }
}

// ---- digit histograms.  LEVEL 1: all keys; 2: keys matching prefix1; 3: keys matching prefix2,
//      plus per-chunk counts of keys above / inside the 22-bit prefix. -------------------------------
template <int LEVEL>
__device__ __forceinline__ void hist_key(uint32_t key, uint32_t prefix, uint32_t* h, uint32_t& gt, uint32_t& eq) {
    if (LEVEL == 1) {
        atomicAdd(&h[key >> SHIFT1], 1u);
    } else if (LEVEL == 2) {
        if ((key >> SHIFT1) == prefix) atomicAdd(&h[(key >> SHIFT2) & (BINS2 - 1)], 1u);
    } else {
        const uint32_t hi = key >> SHIFT2;
        if (hi == prefix) { atomicAdd(&h[key & (BINS3 - 1)], 1u); ++eq; }
        else if (hi > prefix) ++gt;
    }
}

template <int LEVEL>
__global__ void __launch_bounds__(TK_THREADS) topk_hist_full(const float* __restrict__ delta, uint64_t ld, uint64_t N, Scratch s) {
    __shared__ uint32_t h[HIST_BINS];
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.y;
    if (s.rows[row].cand_mode) return;                         // uniform
    constexpr int BINS = (LEVEL == 3) ? BINS3 : HIST_BINS;
    for (int b = threadIdx.x; b < BINS; b += TK_THREADS) h[b] = 0;
    __syncthreads();
    const uint32_t prefix = (LEVEL == 2) ? s.rows[row].prefix1 : (LEVEL == 3) ? s.rows[row].prefix2 : 0u;
    const float* dr = delta + (uint64_t)row * ld;
    for (uint32_t chunk = blockIdx.x * TK_FPW; chunk < (blockIdx.x + 1) * TK_FPW && chunk < s.nchunks; ++chunk) {
        const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
        uint32_t gt = 0, eq = 0;
#pragma unroll 2
        for (int it = 0; it < TK_ITERS; ++it) {
            const uint64_t j = c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x;
            if (j >= ld) break;
            const float4 v = *reinterpret_cast<const float4*>(dr + j);
            const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (j + c < N) hist_key<LEVEL>(key_of(vv[c]), prefix, h, gt, eq);
        }
        if (LEVEL == 3) {
            const uint32_t gts = block_sum(gt, wave_sums);
            const uint32_t eqs = block_sum(eq, wave_sums);
            if (threadIdx.x == 0) {
                s.cnt_gt[(size_t)row * s.nchunks + chunk] = gts;
                s.cnt_eq[(size_t)row * s.nchunks + chunk] = eqs;
            }
        }
    }
    __syncthreads();
    uint32_t* hrow = s.hist + (size_t)row * HIST_BINS;
    for (int b = threadIdx.x; b < BINS; b += TK_THREADS)
        if (h[b]) atomicAdd(&hrow[b], h[b]);
}

// Candidate mode: TK_HWG workgroups of 1024 threads per row, each walking a contiguous range of chunks
// with 32 lanes per chunk (32 chunks side by side) and 8 slot loads in flight per lane.  Few, large
// workgroups keep the number of global histogram atomics down (one flush of <= 2048 bins each).
template <int LEVEL>
__global__ void __launch_bounds__(TK_HTHREADS) topk_hist_cand(Scratch s) {
    __shared__ uint32_t h[HIST_BINS];
    const int row = blockIdx.y;
    if (!s.rows[row].cand_mode) return;                        // uniform
    constexpr int BINS = (LEVEL == 3) ? BINS3 : HIST_BINS;
    for (int b = threadIdx.x; b < BINS; b += TK_HTHREADS) h[b] = 0;
    __syncthreads();
    const uint32_t prefix = (LEVEL == 2) ? s.rows[row].prefix1 : s.rows[row].prefix2;
    constexpr int TPC = 32, SIDE = TK_HTHREADS / TPC;          // lanes per chunk, chunks side by side
    const int sub = threadIdx.x % TPC;
    const uint32_t per_wg = (s.nchunks + TK_HWG - 1) / TK_HWG;
    const uint32_t first = blockIdx.x * per_wg;
    const uint32_t last = (first + per_wg < s.nchunks) ? first + per_wg : s.nchunks;
    for (uint32_t chunk = first + threadIdx.x / TPC; chunk < last; chunk += SIDE) {
        const size_t cidx = (size_t)row * s.nchunks + chunk;
        const uint32_t cnt = s.cand_cnt[cidx];
        const uint32_t* slot = s.slot_val + cidx * TK_CAP;
        uint32_t gt = 0, eq = 0;
        for (uint32_t p0 = sub; p0 < cnt; p0 += 8 * TPC) {
            uint32_t key[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) key[u] = (p0 + u * TPC < cnt) ? (slot[p0 + u * TPC] & 0x7FFFFFFFu) : 0xFFFFFFFFu;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (key[u] != 0xFFFFFFFFu) hist_key<LEVEL>(key[u], prefix, h, gt, eq);
        }
        if (LEVEL == 3) {
            // the 32 lanes of a chunk are half a wave: fold with shuffles inside the half
#pragma unroll
            for (int o = 1; o < TPC; o <<= 1) { gt += __shfl_xor(gt, o); eq += __shfl_xor(eq, o); }
            if (sub == 0) { s.cnt_gt[cidx] = gt; s.cnt_eq[cidx] = eq; }
        }
    }
    __syncthreads();
    uint32_t* hrow = s.hist + (size_t)row * HIST_BINS;
    for (int b = threadIdx.x; b < BINS; b += TK_HTHREADS)
        if (h[b]) atomicAdd(&hrow[b], h[b]);
}

// ---- where to collect candidates in the next step ------------------------------------------------
// Keys are (piecewise) logarithmic in |v|, and near the threshold the number of keys above a level
// falls roughly exponentially with the level.  With d = tau - tlo the distance that caught
// ratio * k candidates this step, the distance that would catch 3 k is d* = d ln 3 / ln ratio.  The
// threshold itself moves from step to step (delta keeps growing early in a run), so the next level
// is aimed at tau + 3/4 drift - d*.  Without usable candidates (full mode) a fixed distance of two
// level-1 bins is taken.  Only speed depends on this guess; a bad one sends the row through the exact full path.
__device__ __forceinline__ uint32_t next_candidate_threshold(const TopkRow& r, uint32_t tau, uint32_t k) {
    const float d0 = 2.f * (float)(1u << SHIFT1);
    float dstar = d0;
    if (r.cand_mode && r.cand_total > k && tau > r.tlo_used) {
        const float ratio = (float)r.cand_total / (float)k;
        const float d = (float)(tau - r.tlo_used);
        dstar = d * (1.0986123f / logf(ratio));
        dstar = fminf(fmaxf(dstar, 1024.f), 4.f * d0);
    }
    float drift = 0.f;
    if (r.tau_prev != 0xFFFFFFFFu && tau > r.tau_prev) drift = fminf((float)(tau - r.tau_prev), 8.f * d0);
    // the drift decays as a run settles: three quarters of the last one is the forecast
    const float t = (float)tau + 0.75f * drift - dstar;
    return t > 0.f ? (uint32_t)t : 0u;
}

// ---- per-row digit select: the bin where the count from the top crosses `need` -----------------
// Level 3 ends with the threshold key and also aims the candidate collection of the next step.
template <int LEVEL>
__global__ void __launch_bounds__(TK_THREADS) topk_select(Scratch s, uint32_t k) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.x;
    constexpr int BINS = (LEVEL == 1) ? BINS1 : (LEVEL == 2) ? BINS2 : BINS3;
    constexpr int PER = HIST_BINS / TK_THREADS;           // 8 consecutive bins per thread
    uint32_t* hrow = s.hist + (size_t)row * HIST_BINS;
    TopkRow& r = s.rows[row];
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
            else {
                const uint32_t tau = (r.prefix2 << SHIFT2) | (uint32_t)b;
                r.tlo = next_candidate_threshold(r, tau, k);
                r.tau_prev = tau;
                r.tau = tau;
                r.r_tie = rem;
            }
        }
        above += mine[q];
        hrow[b] = 0;                                      // leave the histogram clean for the next pass
    }
}

// ---- exact per-chunk counts: only chunks that hold a key with the threshold's 22-bit prefix -----
__global__ void __launch_bounds__(TK_THREADS) topk_fix_full(const float* __restrict__ delta, uint64_t ld, uint64_t N, Scratch s) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.y;
    if (s.rows[row].cand_mode) return;
    const uint32_t tau = s.rows[row].tau;
    const float* dr = delta + (uint64_t)row * ld;
    for (uint32_t chunk = blockIdx.x * TK_FPW; chunk < (blockIdx.x + 1) * TK_FPW && chunk < s.nchunks; ++chunk) {
        const size_t ci = (size_t)row * s.nchunks + chunk;
        if (s.cnt_eq[ci] == 0) continue;                  // uniform: nothing in this chunk can tie or straddle
        const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
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
        if (threadIdx.x == 0) { s.cnt_gt[ci] = gts; s.cnt_eq[ci] = eqs; }
    }
}

__global__ void __launch_bounds__(TK_THREADS) topk_fix_cand(Scratch s) {
    __shared__ uint32_t c_gt[TK_CPW], c_eq[TK_CPW];
    const int row = blockIdx.y;
    if (!s.rows[row].cand_mode) return;
    if (threadIdx.x < TK_CPW) { c_gt[threadIdx.x] = 0; c_eq[threadIdx.x] = 0; }
    __syncthreads();
    const uint32_t tau = s.rows[row].tau;
    constexpr int TPC = TK_THREADS / TK_CPW;
    const int ci = threadIdx.x / TPC, sub = threadIdx.x % TPC;
    const uint32_t chunk = blockIdx.x * TK_CPW + ci;
    if (chunk < s.nchunks) {
        const size_t cidx = (size_t)row * s.nchunks + chunk;
        if (s.cnt_eq[cidx] != 0) {
            const uint32_t cnt = s.cand_cnt[cidx];
            const uint32_t* slot = s.slot_val + cidx * TK_CAP;
            uint32_t gt = 0, eq = 0;
            for (uint32_t p = sub; p < cnt; p += TPC) {
                const uint32_t key = slot[p] & 0x7FFFFFFFu;
                gt += key > tau;
                eq += key == tau;
            }
            if (gt) atomicAdd(&c_gt[ci], gt);
            if (eq) atomicAdd(&c_eq[ci], eq);
        }
    }
    __syncthreads();
    const uint32_t chunk0 = blockIdx.x * TK_CPW;
    if (threadIdx.x < TK_CPW && chunk0 + threadIdx.x < s.nchunks) {
        const size_t cidx = (size_t)row * s.nchunks + chunk0 + threadIdx.x;
        if (s.cnt_eq[cidx] != 0) { s.cnt_gt[cidx] = c_gt[threadIdx.x]; s.cnt_eq[cidx] = c_eq[threadIdx.x]; }
    }
}

// ---- per-row scan over chunks: tie quota and output offset of every chunk -----------------------
__global__ void __launch_bounds__(TK_THREADS) topk_scan_chunks(Scratch s, unsigned long long* t_ptr) {
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicAdd(t_ptr, 1ull);   // one step taken
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.x;
    const uint32_t nchunks = s.nchunks;
    const uint32_t r_tie = s.rows[row].r_tie;
    const uint32_t* gt = s.cnt_gt + (size_t)row * nchunks;
    const uint32_t* eq = s.cnt_eq + (size_t)row * nchunks;
    uint32_t* eqb = s.eq_before + (size_t)row * nchunks;
    uint32_t* off = s.out_off + (size_t)row * (nchunks + 1);
    // each thread owns a run of consecutive chunks, so that two workgroup scans serve the whole row
    const uint32_t per = (nchunks + TK_THREADS - 1) / TK_THREADS;
    const uint32_t lo = (threadIdx.x * per < nchunks) ? threadIdx.x * per : nchunks;
    const uint32_t hi = (lo + per < nchunks) ? lo + per : nchunks;
    uint32_t sum_e = 0;
    for (uint32_t c = lo; c < hi; ++c) sum_e += eq[c];
    uint32_t tot_e, tot_o;
    const uint32_t before0 = block_exclusive_scan(sum_e, wave_sums, &tot_e);   // ties in earlier chunks of the row
    uint32_t before = before0, sum_take = 0;
    for (uint32_t c = lo; c < hi; ++c) {
        const uint32_t e = eq[c];
        const uint32_t quota = (before < r_tie) ? (r_tie - before) : 0u;
        sum_take += gt[c] + (e < quota ? e : quota);
        before += e;
    }
    uint32_t o = block_exclusive_scan(sum_take, wave_sums, &tot_o);
    before = before0;
    for (uint32_t c = lo; c < hi; ++c) {
        const uint32_t e = eq[c];
        const uint32_t quota = (before < r_tie) ? (r_tie - before) : 0u;
        eqb[c] = before;
        off[c] = o;
        o += gt[c] + (e < quota ? e : quota);
        before += e;
    }
    if (threadIdx.x == 0) { off[nchunks] = tot_o; s.rows[row].total = tot_o; }
}

// ---- ordered compaction: message pairs, delta <- 0 on the selected set (Algorithm 1, line 6) ----
__device__ __forceinline__ void write_full_chunk(const TopkArgs& a, const Scratch& s, int row, uint32_t chunk, uint32_t* wave_sums) {
    const uint32_t nchunks = s.nchunks;
    const size_t ci = (size_t)row * nchunks + chunk;
    const uint32_t off0 = s.out_off[(size_t)row * (nchunks + 1) + chunk];
    const uint32_t off1 = s.out_off[(size_t)row * (nchunks + 1) + chunk + 1];
    if (off0 == off1) return;                               // uniform
    const bool ties = s.cnt_eq[ci] != 0;
    const uint32_t tau = s.rows[row].tau, r_tie = s.rows[row].r_tie;
    uint32_t run_eq = s.eq_before[ci], run_out = off0;
    const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
    const float* dr = a.delta + (uint64_t)row * a.ld;
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
            }
        run_out += tot;
    }
}

__global__ void __launch_bounds__(TK_THREADS) topk_write_full(TopkArgs a, Scratch s) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.y;
    if (s.rows[row].cand_mode) return;
    for (uint32_t chunk = blockIdx.x * TK_FPW; chunk < (blockIdx.x + 1) * TK_FPW && chunk < s.nchunks; ++chunk)
        write_full_chunk(a, s, row, chunk, wave_sums);
}

// Candidate mode, one wave per chunk.  A slot is unordered, so order comes from two bitmaps over the
// chunk's columns (selected, tied): the place of a pair in the message is the number of selected
// columns below it, and the ties that belong to the set are the `quota` lowest tied columns.
constexpr int TK_WORDS = TK_CHUNK / 32;                        // bitmap words per chunk
__device__ __forceinline__ void bitmap_prefix(const uint32_t* bits, uint32_t* prefix, int lane) {
    // prefix[w] = number of set bits in words [0, w); 4 consecutive words per lane
    uint32_t c[TK_WORDS / 64], sum = 0;
#pragma unroll
    for (int q = 0; q < TK_WORDS / 64; ++q) { c[q] = __popc(bits[lane * (TK_WORDS / 64) + q]); sum += c[q]; }
    uint32_t inc = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(inc, o);
        if (lane >= o) inc += up;
    }
    uint32_t run = inc - sum;
#pragma unroll
    for (int q = 0; q < TK_WORDS / 64; ++q) { prefix[lane * (TK_WORDS / 64) + q] = run; run += c[q]; }
}
__device__ __forceinline__ uint32_t bitmap_rank(const uint32_t* bits, const uint32_t* prefix, uint32_t q) {
    return prefix[q >> 5] + __popc(bits[q >> 5] & ((1u << (q & 31)) - 1u));
}

__global__ void __launch_bounds__(64) topk_write_cand(TopkArgs a, Scratch s) {
    __shared__ uint32_t sel_bits[TK_WORDS], eq_bits[TK_WORDS], prefix[TK_WORDS];
    const int row = blockIdx.y;
    const int lane = threadIdx.x;
    const uint32_t nchunks = s.nchunks, chunk = blockIdx.x;
    const size_t cidx = (size_t)row * nchunks + chunk;
    const uint32_t* slot_val = s.slot_val + cidx * TK_CAP;
    const uint16_t* slot_idx = s.slot_idx + cidx * TK_CAP;
    // The slot goes into registers, 8 pairs per lane.  The first half is loaded before anything is known
    // about the chunk (the slot's memory exists whatever its fill; what lies behind `cnt` is discarded
    // below), so that these loads do not queue behind the chunk's counters.
    constexpr int EPL = TK_CAP / 64, SPEC = EPL / 2;
    uint2 ent[EPL];
#pragma unroll
    for (int u = 0; u < SPEC; ++u) {
        const uint32_t p = (uint32_t)u * 64 + lane;
        ent[u] = make_uint2(slot_idx[p], slot_val[p]);     // .x: column in the chunk
    }
    const uint32_t cand_mode = s.rows[row].cand_mode;
    const uint32_t tau = s.rows[row].tau, r_tie = s.rows[row].r_tie;
    const uint32_t off0 = s.out_off[(size_t)row * (nchunks + 1) + chunk];
    const uint32_t off1 = s.out_off[(size_t)row * (nchunks + 1) + chunk + 1];
    const uint32_t cnt = s.cand_cnt[cidx];
    const uint32_t eqb = s.eq_before[cidx];
    const uint32_t cnt_eq = s.cnt_eq[cidx];
    if (!cand_mode || off0 == off1) return;                 // uniform
    const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
    const uint32_t quota = (eqb < r_tie) ? (r_tie - eqb) : 0u;   // ties of this chunk that belong to the set
    const bool ties = cnt_eq != 0 && quota != 0;
#pragma unroll
    for (int u = 0; u < EPL; ++u) {
        const uint32_t p = (uint32_t)u * 64 + lane;
        if (u < SPEC) { if (p >= cnt) ent[u] = make_uint2(0xFFFFFFFFu, 0u); }
        else ent[u] = (p < cnt) ? make_uint2(slot_idx[p], slot_val[p]) : make_uint2(0xFFFFFFFFu, 0u);
    }
    for (int w = lane; w < TK_WORDS; w += 64) { sel_bits[w] = 0; eq_bits[w] = 0; }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < EPL; ++u) {
        const uint32_t key = ent[u].y & 0x7FFFFFFFu;
        const uint32_t q = ent[u].x;
        if (q >= (uint32_t)TK_CHUNK) continue;              // the padding pairs
        if (key > tau) atomicOr(&sel_bits[q >> 5], 1u << (q & 31));
        else if (key == tau && ties) atomicOr(&eq_bits[q >> 5], 1u << (q & 31));
    }
    __syncthreads();
    if (ties) {                                             // uniform
        bitmap_prefix(eq_bits, prefix, lane);
        __syncthreads();
        for (int w = lane; w < TK_WORDS; w += 64) {
            // keep the tied columns whose rank among the ties is below the quota
            uint32_t word = eq_bits[w], keep = 0;
            uint32_t rank = prefix[w];
            while (word) {
                const uint32_t bit = word & (0u - word);
                if (rank < quota) keep |= bit;
                ++rank;
                word ^= bit;
            }
            sel_bits[w] |= keep;
        }
        __syncthreads();
    }
    bitmap_prefix(sel_bits, prefix, lane);
    __syncthreads();
    uint2* out = reinterpret_cast<uint2*>(a.msg + (uint64_t)row * a.k * 8);
#pragma unroll
    for (int u = 0; u < EPL; ++u) {
        const uint32_t q = ent[u].x;
        if (q >= (uint32_t)TK_CHUNK) continue;
        if (sel_bits[q >> 5] & (1u << (q & 31))) {
            const uint32_t pos = off0 + bitmap_rank(sel_bits, prefix, q);
            if (pos < a.k && pos < off1) out[pos] = make_uint2((uint32_t)(c0 + q), ent[u].y);
        }
    }
}

// ---- the deferred sparse tail of a step, applied in place (when the state must be complete now) --
// One workgroup per (row, chunk): the neighbours' pairs that fall into the chunk are contiguous in
// their messages (out_off), so they are accumulated in ascending neighbour order into an LDS copy
// of the chunk and then applied once per touched column.
__global__ void __launch_bounds__(TK_THREADS) topk_gossip(TopkArgs a, Scratch s) {
    __shared__ float acc[TK_CHUNK];
    __shared__ uint32_t taken[TK_CHUNK / 32];
    const int row = blockIdx.y;
    const uint32_t c = blockIdx.x;
    const uint32_t nchunks = s.nchunks;
    const uint64_t c0 = (uint64_t)c * TK_CHUNK;
    const int e0 = a.rowptr[row], e1 = a.rowptr[row + 1];
    bool any = false;
    for (int e = e0; e < e1; ++e) {
        const uint32_t* off = s.out_off + (size_t)a.col[e] * (nchunks + 1) + c;
        any |= (off[0] != off[1]);
    }
    if (!any) return;                                       // uniform
    for (int q = threadIdx.x; q < TK_CHUNK; q += TK_THREADS) acc[q] = 0.f;
    for (int q = threadIdx.x; q < TK_CHUNK / 32; q += TK_THREADS) taken[q] = 0u;
    __syncthreads();
    for (int e = e0; e < e1; ++e) {
        const int nb = a.col[e];
        const float w = a.coef[e];
        const uint32_t* off = s.out_off + (size_t)nb * (nchunks + 1) + c;
        const uint2* in = reinterpret_cast<const uint2*>(a.msg + (uint64_t)nb * a.k * 8);
        for (uint32_t p = off[0] + threadIdx.x; p < off[1]; p += TK_THREADS) {
            const uint2 pr = in[p];
            const uint32_t q = (uint32_t)((uint64_t)pr.x - c0);
            if (q < (uint32_t)TK_CHUNK) acc[q] = fmaf(w, __uint_as_float(pr.y), acc[q]);
        }
        __syncthreads();
    }
    float* xr = a.x + (uint64_t)row * a.ld;
    float* dr = a.delta + (uint64_t)row * a.ld;
    for (int e = e0; e < e1; ++e) {
        const int nb = a.col[e];
        const uint32_t* off = s.out_off + (size_t)nb * (nchunks + 1) + c;
        const uint2* in = reinterpret_cast<const uint2*>(a.msg + (uint64_t)nb * a.k * 8);
        for (uint32_t p = off[0] + threadIdx.x; p < off[1]; p += TK_THREADS) {
            const uint32_t jj = in[p].x;
            const uint32_t q = (uint32_t)((uint64_t)jj - c0);
            if (q >= (uint32_t)TK_CHUNK || jj >= a.N) continue;
            if (nb == row) dr[jj] = 0.f;                    // line 6: delta = v - C[v] = 0 where v was sent
            const uint32_t bit = 1u << (q & 31);
            const uint32_t old = atomicOr(&taken[q >> 5], bit);
            if (!(old & bit)) xr[jj] = fmaf(a.eta, acc[q], xr[jj]);
        }
    }
}

__global__ void __launch_bounds__(256) topk_zero_words(uint32_t* p, size_t words) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i + 3 < words) *reinterpret_cast<uint4*>(p + i) = make_uint4(0u, 0u, 0u, 0u);   // the array comes from hipMalloc: 16-byte aligned
    else for (size_t q = i; q < words; ++q) p[q] = 0u;
}

__global__ void topk_init_rows(TopkRow* rows, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        TopkRow r{};
        r.tlo = 0xFFFFFFFFu;                                // no guess yet: the first step runs in full mode
        r.tau_prev = 0xFFFFFFFFu;
        rows[i] = r;
    }
}

}  // namespace

struct TopkState {
    Scratch s{};
    int n = 0;
    bool pending = false;          // a step has been enqueued since the last flush (or may have been, by a
                                   // replayed graph): its sparse tail may not have been applied yet
};

void topk_destroy(TopkState* st) {
    if (!st) return;
    void* ptrs[] = {st->s.hist, st->s.rows, st->s.cnt_gt, st->s.cnt_eq, st->s.eq_before, st->s.out_off, st->s.cand_cnt, st->s.slot_val, st->s.slot_idx};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    delete st;
}

ds_status topk_create(const ds_config& cfg, uint64_t /*ld*/, TopkState** out, std::string& err) {
    TopkState* st = new TopkState();
    st->n = cfg.n;
    Scratch& s = st->s;
    s.nchunks = (uint32_t)((cfg.N + TK_CHUNK - 1) / TK_CHUNK);
    const size_t n = (size_t)cfg.n, nc = s.nchunks;
    bool ok = hipMalloc(&s.hist, n * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.rows, n * sizeof(TopkRow)) == hipSuccess &&
              hipMalloc(&s.cnt_gt, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.cnt_eq, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.eq_before, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.out_off, n * (nc + 1) * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.cand_cnt, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.slot_val, n * nc * TK_CAP * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.slot_idx, n * nc * TK_CAP * sizeof(uint16_t)) == hipSuccess;
    ok = ok && hipMemset(s.hist, 0, n * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s.out_off, 0, n * (nc + 1) * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s.cand_cnt, 0, n * nc * sizeof(uint32_t)) == hipSuccess;
    if (ok) {
        hipLaunchKernelGGL(topk_init_rows, dim3((cfg.n + 63) / 64), dim3(64), 0, 0, s.rows, cfg.n);
        ok = hipDeviceSynchronize() == hipSuccess;
    }
    if (!ok) {
        err = "top-k scratch allocation failed";
        topk_destroy(st);
        return DS_ENOMEM;
    }
    *out = st;
    return DS_OK;
}

ds_status topk_candidate_rows(TopkState* st, hipStream_t stream, uint32_t* count) {
    std::vector<TopkRow> rows(st->n);
    if (hipStreamSynchronize(stream) != hipSuccess) return DS_EHIP;
    if (hipMemcpy(rows.data(), st->s.rows, rows.size() * sizeof(TopkRow), hipMemcpyDeviceToHost) != hipSuccess) return DS_EHIP;
    uint32_t c = 0;
    for (const TopkRow& r : rows) c += r.cand_mode ? 1u : 0u;
    *count = c;
    return DS_OK;
}

ds_status topk_flush(TopkState* st, const TopkArgs& a, hipStream_t stream) {
    if (!st || !st->pending) return DS_OK;
    const dim3 grid(st->s.nchunks, a.n), block(TK_THREADS);
    hipLaunchKernelGGL(topk_gossip, grid, block, 0, stream, a, st->s);
    // the tail is applied: no message offsets, nothing for the next first pass to apply again (a kernel, not a
    // memset: the caller may be capturing the stream)
    const size_t words = (size_t)st->n * (st->s.nchunks + 1);
    hipLaunchKernelGGL(topk_zero_words, dim3((unsigned)((words + 1023) / 1024)), dim3(256), 0, stream, st->s.out_off, words);
    // `pending` stays set: a captured graph of ds_step may be replayed without this code noticing, and a flush
    // with nothing to apply is a grid of workgroups that return at once
    return hipGetLastError() == hipSuccess ? DS_OK : DS_EHIP;
}

ds_status topk_step(TopkState* st, const TopkArgs& a, hipStream_t stream) {
    const Scratch& s = st->s;
    const dim3 grid(s.nchunks, a.n), block(TK_THREADS);
    const dim3 cgrid((s.nchunks + TK_CPW - 1) / TK_CPW, a.n);
    const dim3 fgrid((s.nchunks + TK_FPW - 1) / TK_FPW, a.n);
    const dim3 hgrid(TK_HWG, a.n), hblock(TK_HTHREADS);
    const dim3 rows(a.n);
    const uint32_t k = (uint32_t)a.k;
    // after a flush (and at the start) all message offsets are zero, so the first pass finds no tail to apply
    hipLaunchKernelGGL(topk_form_collect, grid, block, 0, stream, a, s);
    hipLaunchKernelGGL(topk_decide, rows, block, 0, stream, s, k);
    hipLaunchKernelGGL(topk_hist_full<1>, fgrid, block, 0, stream, a.delta, a.ld, a.N, s);
    hipLaunchKernelGGL(topk_select<1>, rows, block, 0, stream, s, k);
    hipLaunchKernelGGL(topk_hist_cand<2>, hgrid, hblock, 0, stream, s);
    hipLaunchKernelGGL(topk_hist_full<2>, fgrid, block, 0, stream, a.delta, a.ld, a.N, s);
    hipLaunchKernelGGL(topk_select<2>, rows, block, 0, stream, s, k);
    hipLaunchKernelGGL(topk_hist_cand<3>, hgrid, hblock, 0, stream, s);
    hipLaunchKernelGGL(topk_hist_full<3>, fgrid, block, 0, stream, a.delta, a.ld, a.N, s);
    hipLaunchKernelGGL(topk_select<3>, rows, block, 0, stream, s, k);
    hipLaunchKernelGGL(topk_fix_cand, cgrid, block, 0, stream, s);
    hipLaunchKernelGGL(topk_fix_full, fgrid, block, 0, stream, a.delta, a.ld, a.N, s);
    hipLaunchKernelGGL(topk_scan_chunks, rows, block, 0, stream, s, a.t_ptr);
    hipLaunchKernelGGL(topk_write_cand, grid, dim3(64), 0, stream, a, s);
    hipLaunchKernelGGL(topk_write_full, fgrid, block, 0, stream, a, s);
    st->pending = true;
    return DS_OK;
}

}  // namespace dsq

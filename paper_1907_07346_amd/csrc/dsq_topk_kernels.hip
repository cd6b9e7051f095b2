// Top-k path of libdsq (gfx950): exact magnitude select per worker row, ordered packing of the
// (index, value) message, residual write-back and the sparse gossip update.
//
// DeepSqueeze's Algorithm 1 with C_omega = top-k (one of the operators the paper lists under
// Assumption 1.6): line 5 forms v, line 6 keeps the k largest |v| (ties to the lower index) and
// leaves everything else in delta, lines 7-8 "send" the k pairs, line 9 mixes the neighbours'
// sparse vectors into x.
//
// Keys: key = bits(v) & 0x7fffffff (order preserving for finite |v|).  The select ends with the exact
// threshold key tau and the number r_tie of elements equal to tau that still belong to the set.  Ordered
// output (ascending index: the tie rule and a canonical message need it) comes from per-chunk counts, a
// per-row scan over chunks and an ordered compaction inside each chunk.
//
// Two sources feed the select, chosen per row on the device with no host round trip:
//   * candidate mode (the fast path): the pass that forms v also appends every element whose key reaches a
//     per-row guess `tlo` (aimed at about 1.6 k elements from the previous step's catch and the drift of the
//     threshold) to a small per-chunk slot, with a level-1 histogram (bins of 2^20 keys) of those keys.  If
//     at least k candidates were collected and no slot overflowed, small kernels finish the step without
//     reading v again:
//       topk_decide_select  per row: the level-1 bin that holds the threshold, and how many to take inside
//       topk_hist_cand2     the slots' level-2 histogram (bins of 512 keys) inside that bin
//       topk_select2_cand   per row: the level-2 bin of the threshold
//       topk_bin_collect    per chunk: candidates above that bin counted; the few inside it listed per row
//       topk_finish         per row: exact tau and r_tie from the list, per-chunk counts, scan over chunks
//       topk_write_cand     per chunk: the ordered message from the slot
//   * full mode (always exact, used on the first step and whenever the guess fails): an MSB-first radix
//     select over v itself, 11 + 11 + 9 bits, workgroup histograms in LDS, every workgroup of a pass
//     working out the previous level's bin for itself.  Its kernels run on a small grid-stride grid and
//     return at once for rows in candidate mode, so a step that needs none of them pays a few microseconds
//     for their launches.
// Both end in the same tau, r_tie, per-chunk counts and message, so results never depend on the
// guess; only speed does.
//
// The sparse tail of a step is deferred: the first pass writes x = (x - gamma g) + 0 and
// delta = v, which already are the final values of every column nobody sent; the remainder --
// delta = 0 where this worker sent v (line 6) and eta * sum_j a_ij C[v_j] where a neighbour did
// (line 9) -- is folded into the NEXT step's first pass (which streams x and delta anyway), or
// applied by topk_flush before anyone else looks at the state.

#include "dsq_internal.h"
#include "dsq_philox.h"

namespace dsq {

namespace {

constexpr int TK_THREADS = 256;
constexpr int TK_VEC = 4 * TK_THREADS;       // elements per workgroup iteration
constexpr int TK_ITERS = 4;
constexpr int TK_CHUNK = TK_VEC * TK_ITERS;  // columns per chunk (one workgroup of the streaming passes)
constexpr int TK_CAP = 512;                  // candidate slots per chunk (12.5 % of the chunk)
constexpr int TK_H1 = 256;                   // level-1 bins the first pass tracks, counted from tlo's bin upwards
constexpr int TK_HWG = 16;                   // workgroups per row in topk_hist_cand2 and topk_bin_collect
constexpr int TK_HTHREADS = 1024;            // threads of those workgroups
constexpr int TK_FWG = 64;                   // full-mode workgroups per row (grid-stride over the row's chunks)
constexpr int TK_WPW = 8;                    // chunks per wave (= workgroup) in topk_write_cand
constexpr int TK_RTHREADS = 1024;            // threads of the per-row kernels
constexpr int BINS1 = 2048, SHIFT1 = 20;     // level 1: key bits 30..20
constexpr int BINS2 = 2048, SHIFT2 = 9;      // level 2: key bits 19..9
constexpr int BINS3 = 512;                   // level 3: key bits 8..0
constexpr int HIST_BINS = 2048;
constexpr uint32_t FINE_SPAN = 1u << SHIFT2; // keys in a level-2 bin
constexpr int TK_HPARTS = 16;                // partial level-1 histograms per row the first pass spreads its atomics over
constexpr uint32_t TK_LIST_CAP = 8192;       // candidates inside the threshold's level-2 bin a row can list
constexpr float TK_TARGET = 1.6f;            // candidates aimed at, in units of k

struct TopkRow {
    uint32_t prefix1, need1;   // full mode: level-1 bin holding the threshold; how many to take inside it
    uint32_t prefix2, need2;   // full mode: 22-bit prefix of the threshold key; how many to take among its matches
    uint32_t tau, r_tie;       // threshold key; number of elements with key == tau to take (lowest indices)
    uint32_t total;            // number of selected elements found by the scan (must equal k)
    uint32_t tlo;              // candidate threshold key for the next first pass (0xffffffff: collect nothing)
    uint32_t cand_mode;        // 1: this step's select runs on the candidate slots
    uint32_t overflow;         // a slot overflowed in this step's first pass
    uint32_t cand_total;       // candidates collected in this step
    uint32_t tlo_used;         // the threshold this step's first pass collected with
    uint32_t tau_prev;         // threshold key of the previous step (0xffffffff: none yet)
    uint32_t bin_lo;           // candidate mode: first key of the histogram bin that holds the threshold
    uint32_t bin_need;         //                 how many elements to take inside that bin
    uint32_t list_count;       //                 elements of that bin listed so far by topk_bin_collect
    float drift_prev;          // last step's movement of |tau| as a float (for the forecast of the next threshold)
    float lambda;              // GSpar: this step's k / sum |v|
    float lambda_hi;           // GSpar: the upper bound the NEXT first pass collects with (0: none)
    uint32_t gs_mode;          // GSpar: 1 = this step's kept elements are among those its first pass collected
    uint32_t gs_need_count;    // GSpar: chunks of the row that must decide from v itself (0: gs_count_dense has nothing to do)
    uint32_t gs_need_write;    // GSpar: chunks that kept more than a slot holds (0: gs_write_dense has nothing to do)
    uint32_t gs_total;         // GSpar: pairs in the row's last message (what a shorter message must clear behind it)
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
    uint32_t* hist;            // n x 2048: level-1 histogram (candidates of the first pass, or all keys in full mode)
    uint32_t* hist_part;       // n x TK_HPARTS x 2048: what the first pass's workgroups add to (chunk mod TK_HPARTS picks the
                               // part: a few hot addresses per row serialise their atomics); folded into hist by topk_decide_select
    uint32_t* hist2;           // n x 2048: level 2
    uint32_t* hist3;           // n x 512:  level 3 (full mode)
    TopkRow* rows;             // n
    uint32_t* cnt_gt;          // n x nchunks: keys above the threshold (prefix) in the chunk
    uint32_t* cnt_eq;          // n x nchunks: keys equal to the threshold (prefix) in the chunk
    uint32_t* eq_before;       // n x nchunks: ties in earlier chunks of the row
    uint32_t* out_off;         // n x (nchunks+1): message offset of each chunk
    uint32_t* cand_cnt;        // n x nchunks: candidates stored in the chunk's slot
    uint32_t* slot_val;        // n x nchunks x TK_CAP candidate values (fp32 bits), unordered inside a slot; the select
                               // passes read only these
    uint16_t* slot_idx;        // same shape: the candidates' columns, relative to the start of the chunk
    uint2* list;               // n x TK_LIST_CAP: (key, chunk) of the candidates inside the threshold's histogram bin
    double* csum;              // GSpar: n x nchunks tree sums of |v| over the chunks
    uint32_t* gs_overflow;     // GSpar: set once a row kept more than its message holds
    uint32_t nchunks;
};

// Scans over the TK_RTHREADS threads of a per-row workgroup.
__device__ __forceinline__ uint32_t row_exclusive_scan(uint32_t v, uint32_t* wave_sums /*[16]*/, uint32_t* total) {
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
    for (int w = 0; w < TK_RTHREADS / 64; ++w) {
        const uint32_t sm = wave_sums[w];
        if (w < wave) base += sm;
        tot += sm;
    }
    *total = tot;
    return base + inc - v;
}

constexpr uint32_t kGsparStreamTag = 0x47535052u;            // GSpar: 4th counter word of the mask's random stream

// The keep decisions of four adjacent columns of worker `row`.
__device__ __forceinline__ uint32_t gs_keep4(const TopkArgs& a, int row, uint64_t j, uint32_t t_lo, float lambda, const float4& v) {
    uint32_t rnd[4];
    philox4x32_10((uint32_t)(j >> 2), (uint32_t)row, t_lo, kGsparStreamTag, a.seed_lo, a.seed_hi, rnd);
    const float vv[4] = {v.x, v.y, v.z, v.w};
    uint32_t keep = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float p = lambda * fabsf(vv[c]);
        const float u = (float)(rnd[c] >> 8) * (1.0f / 16777216.0f);
        if (j + c < a.N && u < p) keep |= 1u << c;
    }
    return keep;
}

// Exclusive prefix sums of four small counts at once (16 bits each, packed; sums stay below 2^16) over the 256
// threads of a workgroup; *total receives the packed sums.
__device__ __forceinline__ unsigned long long block_exclusive_scan4(unsigned long long v, unsigned long long* wave_sums /*[4]*/,
                                                                    unsigned long long* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long up = __shfl_up(inc, o);
        if (lane >= o) inc += up;
    }
    __syncthreads();                       // wave_sums may still be read from a previous call
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    unsigned long long base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < TK_THREADS / 64; ++w) {
        const unsigned long long sm = wave_sums[w];
        if (w < wave) base += sm;
        tot += sm;
    }
    *total = tot;
    return base + inc - v;
}

// The elements of one chunk whose mask bit is set, in column order, into the chunk's slot (the first TK_CAP of
// them); returns their number.  vin: the lane's four float4 of the chunk, keep: their four 4-bit masks.
__device__ __forceinline__ uint32_t gs_collect(const float4 (&vin)[TK_ITERS], const uint32_t (&keep)[TK_ITERS], uint32_t* slot_val,
                                               uint16_t* slot_idx, unsigned long long* wave_sums) {
    unsigned long long packed = 0;
#pragma unroll
    for (int it = 0; it < TK_ITERS; ++it) packed |= (unsigned long long)__popc(keep[it]) << (16 * it);
    unsigned long long tot;
    const unsigned long long before = block_exclusive_scan4(packed, wave_sums, &tot);
    uint32_t run = 0;
#pragma unroll
    for (int it = 0; it < TK_ITERS; ++it) {
        const uint32_t q0 = (uint32_t)it * TK_VEC + 4 * threadIdx.x;
        uint32_t pos = run + (uint32_t)((before >> (16 * it)) & 0xFFFFu);
        const float vv[4] = {vin[it].x, vin[it].y, vin[it].z, vin[it].w};
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (keep[it] & (1u << c)) {
                if (pos < (uint32_t)TK_CAP) { slot_val[pos] = __float_as_uint(vv[c]); slot_idx[pos] = (uint16_t)(q0 + c); }
                ++pos;
            }
        run += (uint32_t)((tot >> (16 * it)) & 0xFFFFu);
    }
    return run;
}
static_assert(TK_ITERS == 4 && TK_THREADS * 4 < 65536, "four 16-bit fields");

__device__ __forceinline__ double wave_tree_sum_f64(double v) {   // adjacent pairs first; every lane gets the sum
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) v += __shfl_xor(v, o);
    return v;
}

// ---- pass 1: pending gossip of the previous step, Algorithm 1 line 5, candidate collection ------
// GS (the GSpar operator shares this pass and the message conventions): no candidates; instead the chunk's sum of
// |v| in double, as the balanced adjacent-pairs tree the operator's lambda is defined with.
template <bool GS>
__global__ void __launch_bounds__(TK_THREADS) topk_form_collect(TopkArgs a, Scratch s) {
    __shared__ float acc[TK_CHUNK];
    [[maybe_unused]] __shared__ double sweep_abs[TK_ITERS * (TK_THREADS / 64)];
    [[maybe_unused]] __shared__ unsigned long long wave_sums4[TK_THREADS / 64];
    [[maybe_unused]] float4 gs_v[TK_ITERS];
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
    // x and delta rows are padded to whole chunks (the pitch is a multiple of the chunk plus a skew), so only g
    // needs care, and only in the row's last chunk: everywhere else the twelve loads go out back to back with
    // nothing between them that could make one wait for another.
    float4 xin[TK_ITERS], din[TK_ITERS], gin[TK_ITERS];
    if (c0 + TK_CHUNK <= a.N) {                                // uniform
#pragma unroll
        for (int it = 0; it < TK_ITERS; ++it) {
            const uint64_t j = c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x;
            xin[it] = ld4_stream(xr + j);
            din[it] = ld4_stream(dr + j);
            gin[it] = ld4_stream(gr + j);
        }
    } else {
#pragma unroll
        for (int it = 0; it < TK_ITERS; ++it) {
            const uint64_t j = c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x;
            xin[it] = ld4_stream(xr + j);
            din[it] = ld4_stream(dr + j);
            gin[it].x = (j + 0 < a.N) ? gr[j + 0] : 0.f;
            gin[it].y = (j + 1 < a.N) ? gr[j + 1] : 0.f;
            gin[it].z = (j + 2 < a.N) ? gr[j + 2] : 0.f;
            gin[it].w = (j + 3 < a.N) ? gr[j + 3] : 0.f;
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
            // Neighbours in ascending order, four at a time: their pair loads go out together (memory operations
            // complete in issue order, so a load issued only after the previous neighbour was accumulated would
            // show its whole latency with nothing else of this workgroup in flight), then they are accumulated one
            // after the other.  A neighbour with more than one pair per thread in this chunk takes the loop below.
            constexpr int EB = 4;
            for (int eb = e0; eb < e1; eb += EB) {
                uint2 pr[EB];
                bool have[EB], wide[EB];
#pragma unroll
                for (int u = 0; u < EB; ++u) {
                    have[u] = wide[u] = false;
                    if (eb + u < e1) {
                        const int nb = a.col[eb + u];
                        const uint32_t* off = s.out_off + (size_t)nb * (s.nchunks + 1) + chunk;
                        const uint32_t p0 = off[0], p1 = off[1];
                        wide[u] = p1 - p0 > (uint32_t)TK_THREADS;                    // uniform
                        if (!wide[u] && p0 + threadIdx.x < p1) {
                            pr[u] = reinterpret_cast<const uint2*>(a.msg + (uint64_t)nb * a.k * 8)[p0 + threadIdx.x];
                            have[u] = true;
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < EB; ++u) {
                    if (eb + u < e1) {                                               // uniform
                        const int nb = a.col[eb + u];
                        const float w = a.coef[eb + u];
                        if (wide[u]) {
                            const uint32_t* off = s.out_off + (size_t)nb * (s.nchunks + 1) + chunk;
                            const uint2* in = reinterpret_cast<const uint2*>(a.msg + (uint64_t)nb * a.k * 8);
                            for (uint32_t p = off[0] + threadIdx.x; p < off[1]; p += TK_THREADS) {
                                const uint2 one = in[p];
                                const uint32_t q = (uint32_t)((uint64_t)one.x - c0);
                                if (q < (uint32_t)TK_CHUNK) {
                                    acc[q] = fmaf(w, __uint_as_float(one.y), acc[q]);
                                    if (nb == row) atomicOr(&own[q >> 5], 1u << (q & 31));
                                }
                            }
                        } else if (have[u]) {
                            const uint32_t q = (uint32_t)((uint64_t)pr[u].x - c0);
                            if (q < (uint32_t)TK_CHUNK) {
                                acc[q] = fmaf(w, __uint_as_float(pr[u].y), acc[q]);
                                if (nb == row) atomicOr(&own[q >> 5], 1u << (q & 31));
                            }
                        }
                        __syncthreads();
                    }
                }
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
        if constexpr (GS) {                                    // padding columns hold v = 0
            const double sw = wave_tree_sum_f64(((double)fabsf(v.x) + (double)fabsf(v.y)) + ((double)fabsf(v.z) + (double)fabsf(v.w)));
            if ((threadIdx.x & 63) == 0) sweep_abs[it * (TK_THREADS / 64) + (threadIdx.x >> 6)] = sw;   // sweep index = column order
            gs_v[it] = v;
            continue;
        }
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
    if constexpr (GS) {
        // With an upper bound of this step's lambda from the last step, the elements that can be kept at all
        // (u < lambda_hi |v|, about 1 % of the chunk) go into the slot now, in column order, and the second pass
        // over v is not needed if the bound holds.
        const float lambda_hi = s.rows[row].lambda_hi;
        if (lambda_hi > 0.f) {                                 // uniform
            const uint32_t t_lo = (uint32_t)*a.t_ptr;
            uint32_t keep[TK_ITERS];
#pragma unroll
            for (int it = 0; it < TK_ITERS; ++it) keep[it] = gs_keep4(a, row, c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x, t_lo, lambda_hi, gs_v[it]);
            const uint32_t n = gs_collect(gs_v, keep, slot_val, slot_idx, wave_sums4);
            if (threadIdx.x == 0) s.cand_cnt[(size_t)row * s.nchunks + chunk] = n;
        }
        if (threadIdx.x == 0) {
            double t[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) t[q] = sweep_abs[q];
#pragma unroll
            for (int len = 16; len > 1; len >>= 1)
#pragma unroll
                for (int q = 0; q < len / 2; ++q) t[q] = t[2 * q] + t[2 * q + 1];
            s.csum[(size_t)row * s.nchunks + chunk] = t[0];
        }
        return;
    }
    // the row histogram is used if the row ends up in candidate mode and wiped by topk_decide_select either way;
    // a candidate beyond the tracked bins (256 bins = 2^32 in magnitude above tlo) sends the row the exact way
    uint32_t* hrow = s.hist_part + ((size_t)row * TK_HPARTS + (chunk & (uint32_t)(TK_HPARTS - 1))) * HIST_BINS;
    for (int b = threadIdx.x; b < TK_H1; b += TK_THREADS)
        if (h[b]) atomicAdd(&hrow[bin0 + b], h[b]);
    if (far) atomicOr(&s.rows[row].overflow, 1u);
    if (threadIdx.x == 0) {
        const uint32_t c = cand_count;
        s.cand_cnt[(size_t)row * s.nchunks + chunk] = c < (uint32_t)TK_CAP ? c : (uint32_t)TK_CAP;
        if (c > (uint32_t)TK_CAP) atomicOr(&s.rows[row].overflow, 1u);
    }
}

// ---- digit select on a row histogram: the bin where the count from the top crosses `need` ----------
// 256 threads, 8 consecutive bins each, largest keys first.  res (LDS): [0] bin, [1] how many to take inside
// it, [2] elements in it, [3] all elements counted.  A crossing exists whenever need <= the total count.
__device__ __forceinline__ void select_digit(const uint32_t* hrow, int bins, uint32_t need, uint32_t* wave_sums, uint32_t* res) {
    constexpr int PER = HIST_BINS / TK_THREADS;
    uint32_t mine[PER], sum = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int b = HIST_BINS - 1 - (threadIdx.x * PER + q);
        mine[q] = (b < bins) ? hrow[b] : 0u;
        sum += mine[q];
    }
    uint32_t total;
    uint32_t above = block_exclusive_scan(sum, wave_sums, &total);     // keys in strictly higher bins
    if (threadIdx.x == 0) { res[0] = 0; res[1] = 0; res[2] = 0; res[3] = total; }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int b = HIST_BINS - 1 - (threadIdx.x * PER + q);
        if (above < need && need <= above + mine[q]) { res[0] = (uint32_t)b; res[1] = need - above; res[2] = mine[q]; }
        above += mine[q];
    }
    __syncthreads();
}

// ---- candidate mode, per row: did the guess work, and which level-1 bin holds the threshold? -----
// The row is in candidate mode if at least k candidates were collected and no slot overflowed.  Leaves all
// three histograms of the row clean.
__global__ void __launch_bounds__(TK_THREADS) topk_decide_select(Scratch s, uint32_t k) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    __shared__ uint32_t res[4];
    const int row = blockIdx.x;
    uint32_t* hrow = s.hist + (size_t)row * HIST_BINS;
    TopkRow& r = s.rows[row];
    // the first pass left its counts in TK_HPARTS partial histograms, in the TK_H1 bins from tlo's upwards
    const uint32_t bin0 = r.tlo >> SHIFT1;
    for (uint32_t b = bin0 + threadIdx.x; b < bin0 + (uint32_t)TK_H1 && b < (uint32_t)HIST_BINS; b += TK_THREADS) {
        uint32_t sum = 0;
#pragma unroll
        for (int q = 0; q < TK_HPARTS; ++q) {
            uint32_t* part = s.hist_part + ((size_t)row * TK_HPARTS + q) * HIST_BINS + b;
            sum += *part;
            *part = 0;
        }
        hrow[b] += sum;
    }
    __syncthreads();
    select_digit(hrow, BINS1, k, wave_sums, res);
    for (int b = threadIdx.x; b < HIST_BINS; b += TK_THREADS) { hrow[b] = 0; s.hist2[(size_t)row * HIST_BINS + b] = 0; }
    for (int b = threadIdx.x; b < BINS3; b += TK_THREADS) s.hist3[(size_t)row * BINS3 + b] = 0;
    if (threadIdx.x == 0) {
        const uint32_t total = res[3];
        const bool cand = total >= k && r.overflow == 0 && r.tlo != 0xFFFFFFFFu;
        if (cand) { r.prefix1 = res[0]; r.need1 = res[1]; }
        r.cand_mode = cand ? 1u : 0u;
        r.cand_total = total;
        r.overflow = 0;
        r.tlo_used = r.tlo;
        r.list_count = 0;
    }
}

// ---- candidate mode: level-2 histogram of the slots' keys inside the threshold's level-1 bin --------
// TK_HWG workgroups of 1024 threads per row, each walking a contiguous range of chunks with 16 lanes per
// chunk (64 chunks side by side) and 8 slot loads in flight per lane.  Few, large workgroups keep the number
// of global histogram atomics down (one flush of <= 2048 bins each).
__global__ void __launch_bounds__(TK_HTHREADS) topk_hist_cand2(Scratch s) {
    __shared__ uint32_t h[HIST_BINS];
    const int row = blockIdx.y;
    if (!s.rows[row].cand_mode) return;                        // uniform
    for (int b = threadIdx.x; b < HIST_BINS; b += TK_HTHREADS) h[b] = 0;
    __syncthreads();
    const uint32_t prefix = s.rows[row].prefix1;
    constexpr int TPC = 16, SIDE = TK_HTHREADS / TPC;          // lanes per chunk, chunks side by side
    const int sub = threadIdx.x % TPC;
    const uint32_t per_wg = (s.nchunks + TK_HWG - 1) / TK_HWG;
    const uint32_t first = blockIdx.x * per_wg;
    const uint32_t last = (first + per_wg < s.nchunks) ? first + per_wg : s.nchunks;
    const uint32_t* cand_cnt = s.cand_cnt + (size_t)row * s.nchunks;
    uint32_t chunk = first + threadIdx.x / TPC;
    uint32_t cnt = chunk < last ? cand_cnt[chunk] : 0u;        // the next chunk's count is asked for one turn ahead
    for (; chunk < last; chunk += SIDE) {
        const uint32_t cnt_next = (chunk + SIDE < last) ? cand_cnt[chunk + SIDE] : 0u;
        const uint32_t* slot = s.slot_val + ((size_t)row * s.nchunks + chunk) * TK_CAP;
        for (uint32_t p0 = sub; p0 < cnt; p0 += 8 * TPC) {
            uint32_t key[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) key[u] = (p0 + u * TPC < cnt) ? (slot[p0 + u * TPC] & 0x7FFFFFFFu) : 0xFFFFFFFFu;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (key[u] != 0xFFFFFFFFu && (key[u] >> SHIFT1) == prefix) atomicAdd(&h[(key[u] >> SHIFT2) & (BINS2 - 1)], 1u);
        }
        cnt = cnt_next;
    }
    __syncthreads();
    uint32_t* hrow = s.hist2 + (size_t)row * HIST_BINS;
    for (int b = threadIdx.x; b < HIST_BINS; b += TK_HTHREADS)
        if (h[b]) atomicAdd(&hrow[b], h[b]);
}

// ---- candidate mode, per row: the level-2 bin of the threshold ------------------------------------
// A bin with more elements than a row can list (many equal or nearly equal keys) sends the row the exact way.
__global__ void __launch_bounds__(TK_THREADS) topk_select2_cand(Scratch s) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    __shared__ uint32_t res[4];
    const int row = blockIdx.x;
    TopkRow& r = s.rows[row];
    if (!r.cand_mode) return;                                  // uniform
    uint32_t* hrow = s.hist2 + (size_t)row * HIST_BINS;
    select_digit(hrow, BINS2, r.need1, wave_sums, res);
    for (int b = threadIdx.x; b < HIST_BINS; b += TK_THREADS) hrow[b] = 0;     // full mode may need it clean
    if (threadIdx.x == 0) {
        if (res[1] == 0 || res[2] > TK_LIST_CAP) {
            r.cand_mode = 0;
        } else {
            r.bin_lo = ((r.prefix1 << (SHIFT1 - SHIFT2)) | res[0]) << SHIFT2;
            r.bin_need = res[1];
        }
    }
}

// ---- full mode: digit histograms over v.  LEVEL 1: all keys; 2: keys matching prefix1; 3: keys matching
//      prefix2, plus per-chunk counts of keys above / inside the 22-bit prefix.  From level 2 on every
//      workgroup first works out the previous level's bin from that level's (complete) histogram. ---------
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
__global__ void __launch_bounds__(TK_THREADS) topk_hist_full(const float* __restrict__ delta, uint64_t ld, uint64_t N, Scratch s, uint32_t k) {
    __shared__ uint32_t h[HIST_BINS];
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    __shared__ uint32_t res[4];
    const int row = blockIdx.y;
    TopkRow& r = s.rows[row];
    if (r.cand_mode) return;                                   // uniform
    constexpr int BINS = (LEVEL == 3) ? BINS3 : HIST_BINS;
    for (int b = threadIdx.x; b < BINS; b += TK_THREADS) h[b] = 0;
    uint32_t prefix = 0;
    if (LEVEL == 2) {
        select_digit(s.hist + (size_t)row * HIST_BINS, BINS1, k, wave_sums, res);
        prefix = res[0];
        if (blockIdx.x == 0 && threadIdx.x == 0) { r.prefix1 = res[0]; r.need1 = res[1]; }
    } else if (LEVEL == 3) {
        select_digit(s.hist2 + (size_t)row * HIST_BINS, BINS2, r.need1, wave_sums, res);
        prefix = (r.prefix1 << (SHIFT1 - SHIFT2)) | res[0];
        if (blockIdx.x == 0 && threadIdx.x == 0) { r.prefix2 = prefix; r.need2 = res[1]; }
    }
    __syncthreads();
    const float* dr = delta + (uint64_t)row * ld;
    for (uint32_t chunk = blockIdx.x; chunk < s.nchunks; chunk += gridDim.x) {
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
    uint32_t* hrow = (LEVEL == 1) ? s.hist + (size_t)row * HIST_BINS : (LEVEL == 2) ? s.hist2 + (size_t)row * HIST_BINS
                                                                                     : s.hist3 + (size_t)row * BINS3;
    for (int b = threadIdx.x; b < BINS; b += TK_THREADS)
        if (h[b]) atomicAdd(&hrow[b], h[b]);
}

// ---- full mode: the threshold key from the level-3 histogram, then exact per-chunk counts for the chunks
//      that hold a key with the threshold's 22-bit prefix ---------------------------------------------------
__global__ void __launch_bounds__(TK_THREADS) topk_fix_full(const float* __restrict__ delta, uint64_t ld, uint64_t N, Scratch s) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    __shared__ uint32_t res[4];
    const int row = blockIdx.y;
    TopkRow& r = s.rows[row];
    if (r.cand_mode) return;
    select_digit(s.hist3 + (size_t)row * BINS3, BINS3, r.need2, wave_sums, res);
    const uint32_t tau = (r.prefix2 << SHIFT2) | res[0];
    if (blockIdx.x == 0 && threadIdx.x == 0) { r.tau = tau; r.r_tie = res[1]; }
    const float* dr = delta + (uint64_t)row * ld;
    for (uint32_t chunk = blockIdx.x; chunk < s.nchunks; chunk += gridDim.x) {
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

// ---- candidate mode, per chunk: candidates above the threshold's bin counted, those inside it listed ----
// The walk of topk_hist_cand2 (16 lanes per chunk, counts asked for one turn ahead).  The bin holds a few
// hundred elements of a whole row (it is 512 keys wide), so the list is short and its appends (one returning
// atomic each) are rare.
__global__ void __launch_bounds__(TK_HTHREADS) topk_bin_collect(Scratch s) {
    const int row = blockIdx.y;
    if (!s.rows[row].cand_mode) return;                   // uniform
    const uint32_t lo = s.rows[row].bin_lo;
    constexpr int TPC = 16, SIDE = TK_HTHREADS / TPC;
    const int sub = threadIdx.x % TPC;
    const uint32_t per_wg = (s.nchunks + TK_HWG - 1) / TK_HWG;
    const uint32_t first = blockIdx.x * per_wg;
    const uint32_t last = (first + per_wg < s.nchunks) ? first + per_wg : s.nchunks;
    const uint32_t* cand_cnt = s.cand_cnt + (size_t)row * s.nchunks;
    uint2* list = s.list + (size_t)row * TK_LIST_CAP;
    uint32_t chunk = first + threadIdx.x / TPC;
    uint32_t cnt = chunk < last ? cand_cnt[chunk] : 0u;
    for (; chunk < last; chunk += SIDE) {                 // the 16 lanes of a chunk leave the loop together
        const uint32_t cnt_next = (chunk + SIDE < last) ? cand_cnt[chunk + SIDE] : 0u;
        const size_t cidx = (size_t)row * s.nchunks + chunk;
        const uint32_t* slot = s.slot_val + cidx * TK_CAP;
        uint32_t gt = 0;
        for (uint32_t p0 = sub; p0 < cnt; p0 += 8 * TPC) {
            uint32_t key[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) key[u] = (p0 + u * TPC < cnt) ? (slot[p0 + u * TPC] & 0x7FFFFFFFu) : 0u;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t rel = key[u] - lo;          // wraps to a huge number below the bin
                if (key[u] >= lo && rel >= FINE_SPAN) ++gt;
                else if (rel < FINE_SPAN && p0 + u * TPC < cnt) {
                    const uint32_t at = atomicAdd(&s.rows[row].list_count, 1u);
                    if (at < TK_LIST_CAP) list[at] = make_uint2(key[u], chunk);
                }
            }
        }
#pragma unroll
        for (int o = 1; o < TPC; o <<= 1) gt += __shfl_xor(gt, o);
        if (sub == 0) { s.cnt_gt[cidx] = gt; s.cnt_eq[cidx] = 0; }
        cnt = cnt_next;
    }
}

// ---- where to collect candidates in the next step ------------------------------------------------
// Near the threshold the number of keys above a level falls roughly exponentially with the level.  With
// d = tau - tlo the distance that caught ratio * k candidates this step, d* = d ln(target) / ln(ratio) would
// have caught target * k; the next level is (forecast of the next tau) - d*.  The forecast is made on |tau|
// as a float (keys are only piecewise linear in the magnitude: the slope halves at every power of two): the
// last movement repeated, or three quarters of it while the movement still changes by more than a quarter
// from step to step (early in a run delta grows fast and then settles).  Without usable candidates (full
// mode) a fixed distance of two million keys (a quarter of a binade) is taken.  Only speed depends on this
// guess; a bad one sends the row through the exact full path.
__device__ __forceinline__ uint32_t next_candidate_threshold(TopkRow& r, uint32_t tau, uint32_t k) {
    const float d0 = 2.f * (float)(1u << SHIFT1);
    float dist = d0;
    if (r.cand_mode && r.cand_total > k && tau > r.tlo_used) {
        const float ratio = (float)r.cand_total / (float)k;
        dist = (float)(tau - r.tlo_used) * (logf(TK_TARGET) / logf(ratio));
        dist = fminf(fmaxf(dist, 65536.f), 4.f * d0);
    }
    const float mag = __uint_as_float(tau);
    float move = 0.f, next = mag;
    if (r.tau_prev != 0xFFFFFFFFu) {
        move = mag - __uint_as_float(r.tau_prev);
        const bool steady = fabsf(move - r.drift_prev) <= 0.25f * fabsf(move);
        next = mag + (steady ? move : 0.75f * move);
        if (!(next > 0.f) || !(next < 3.0e38f)) next = mag;
    }
    r.drift_prev = move;
    const float t = (float)__float_as_uint(next) - dist;
    return t > 0.f ? (uint32_t)t : 0u;
}

// ---- per row: exact threshold (candidate mode), per-chunk counts, scan over chunks -----------------
// Candidate mode: the listed keys of the threshold's bin (512 possible values) are counted in LDS, the
// count from the top gives tau and the tie quota, and the chunks of the listed keys above / equal to tau
// get their counts corrected.  Both modes: the scan over the row's chunks (tie quota and message offset of
// every chunk), the guess for the next step, and the step counter.
__global__ void __launch_bounds__(TK_RTHREADS) topk_finish(Scratch s, uint32_t k, unsigned long long* t_ptr) {
    __shared__ uint32_t wave_sums[TK_RTHREADS / 64];
    __shared__ uint32_t h[FINE_SPAN];
    __shared__ uint32_t sel[2];
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicAdd(t_ptr, 1ull);   // one step taken
    const int row = blockIdx.x;
    const uint32_t nchunks = s.nchunks;
    TopkRow& r = s.rows[row];
    uint32_t* gtw = s.cnt_gt + (size_t)row * nchunks;
    uint32_t* eqw = s.cnt_eq + (size_t)row * nchunks;
    if (r.cand_mode) {                                              // uniform
        const uint32_t lo = r.bin_lo, need = r.bin_need;
        const uint32_t nlist = r.list_count < TK_LIST_CAP ? r.list_count : TK_LIST_CAP;
        const uint2* list = s.list + (size_t)row * TK_LIST_CAP;
        for (uint32_t b = threadIdx.x; b < FINE_SPAN; b += TK_RTHREADS) h[b] = 0;
        if (threadIdx.x == 0) { sel[0] = lo; sel[1] = 0; }
        __syncthreads();
        for (uint32_t e = threadIdx.x; e < nlist; e += TK_RTHREADS) atomicAdd(&h[list[e].x - lo], 1u);
        __syncthreads();
        // one value per thread (the first 512 threads), largest first
        const uint32_t b = (threadIdx.x < FINE_SPAN) ? FINE_SPAN - 1 - threadIdx.x : 0u;
        const uint32_t mine = (threadIdx.x < FINE_SPAN) ? h[b] : 0u;
        uint32_t total;
        const uint32_t above = row_exclusive_scan(mine, wave_sums, &total);
        if (threadIdx.x < FINE_SPAN && above < need && need <= above + mine) { sel[0] = lo + b; sel[1] = need - above; }
        __syncthreads();
        const uint32_t tau = sel[0];
        for (uint32_t e = threadIdx.x; e < nlist; e += TK_RTHREADS) {
            const uint2 en = list[e];
            if (en.x > tau) atomicAdd(&gtw[en.y], 1u);
            else if (en.x == tau) atomicAdd(&eqw[en.y], 1u);
        }
        if (threadIdx.x == 0) { r.tau = tau; r.r_tie = sel[1]; }
        __threadfence();                                            // the corrected counts, before the scan reads them
        __syncthreads();
    } else {
        // full mode: topk_fix_full left tau and the tie quota; the level-1 histogram of all keys must not meet the
        // next first pass's candidates
        for (int b = threadIdx.x; b < HIST_BINS; b += TK_RTHREADS) s.hist[(size_t)row * HIST_BINS + b] = 0;
        if (threadIdx.x == 0) { sel[0] = r.tau; sel[1] = r.r_tie; }
    }
    __syncthreads();
    const uint32_t tau_row = sel[0], r_tie = sel[1];
    uint32_t* eqb = s.eq_before + (size_t)row * nchunks;
    uint32_t* off = s.out_off + (size_t)row * (nchunks + 1);
    // each thread owns a run of consecutive chunks, so that two workgroup scans serve the whole row; the counts
    // are read past the vector cache (atomics above updated them in L2)
    const uint32_t per = (nchunks + TK_RTHREADS - 1) / TK_RTHREADS;
    const uint32_t lo_c = (threadIdx.x * per < nchunks) ? threadIdx.x * per : nchunks;
    const uint32_t hi_c = (lo_c + per < nchunks) ? lo_c + per : nchunks;
    auto load = [](const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
    constexpr uint32_t REG = 8;                              // a thread's run fits in registers up to 8192 chunks a row
    uint32_t e_r[REG], g_r[REG];
#pragma unroll
    for (uint32_t q = 0; q < REG; ++q) {
        const bool in = per <= REG && lo_c + q < hi_c;
        e_r[q] = in ? load(eqw + lo_c + q) : 0u;
        g_r[q] = in ? load(gtw + lo_c + q) : 0u;
    }
    uint32_t sum_e = 0;
    if (per <= REG) {
#pragma unroll
        for (uint32_t q = 0; q < REG; ++q) sum_e += e_r[q];
    } else {
        for (uint32_t c = lo_c; c < hi_c; ++c) sum_e += load(eqw + c);
    }
    uint32_t tot_e, tot_o;
    const uint32_t before0 = row_exclusive_scan(sum_e, wave_sums, &tot_e);     // ties in earlier chunks of the row
    uint32_t before = before0, sum_take = 0;
    if (per <= REG) {
#pragma unroll
        for (uint32_t q = 0; q < REG; ++q) {
            const uint32_t quota = (before < r_tie) ? (r_tie - before) : 0u;
            sum_take += g_r[q] + (e_r[q] < quota ? e_r[q] : quota);
            before += e_r[q];
        }
    } else {
        for (uint32_t c = lo_c; c < hi_c; ++c) {
            const uint32_t e = load(eqw + c);
            const uint32_t quota = (before < r_tie) ? (r_tie - before) : 0u;
            sum_take += load(gtw + c) + (e < quota ? e : quota);
            before += e;
        }
    }
    uint32_t o = row_exclusive_scan(sum_take, wave_sums, &tot_o);
    before = before0;
    if (per <= REG) {
#pragma unroll
        for (uint32_t q = 0; q < REG; ++q) {
            if (lo_c + q < hi_c) {
                const uint32_t quota = (before < r_tie) ? (r_tie - before) : 0u;
                eqb[lo_c + q] = before;
                off[lo_c + q] = o;
                o += g_r[q] + (e_r[q] < quota ? e_r[q] : quota);
                before += e_r[q];
            }
        }
    } else {
        for (uint32_t c = lo_c; c < hi_c; ++c) {
            const uint32_t e = load(eqw + c);
            const uint32_t quota = (before < r_tie) ? (r_tie - before) : 0u;
            eqb[c] = before;
            off[c] = o;
            o += load(gtw + c) + (e < quota ? e : quota);
            before += e;
        }
    }
    if (threadIdx.x == 0) {
        off[nchunks] = tot_o;
        r.total = tot_o;
        r.tlo = next_candidate_threshold(r, tau_row, k);
        r.tau_prev = tau_row;
    }
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
    for (uint32_t chunk = blockIdx.x; chunk < s.nchunks; chunk += gridDim.x)
        write_full_chunk(a, s, row, chunk, wave_sums);
}

// Candidate mode: 16 lanes per chunk, so a wave (= a workgroup) writes four chunks side by side, TK_WPW / 4
// times in a row.  A slot is unordered, so order comes from two bitmaps over the chunk's columns (selected,
// tied): the place of a pair in the message is the number of selected columns below it, and the ties that
// belong to the set are the `quota` lowest tied columns.
constexpr int TK_WORDS = TK_CHUNK / 32;                        // bitmap words per chunk
constexpr int TK_GL = 16;                                      // lanes per chunk
constexpr int TK_WPL = TK_WORDS / TK_GL;                       // bitmap words per lane (consecutive)
// prefix[w] = number of set bits in words [0, w) of one chunk's bitmap; the TK_GL lanes of the chunk call together
__device__ __forceinline__ void bitmap_prefix(const uint32_t* bits, uint32_t* prefix, int sub) {
    uint32_t c[TK_WPL], sum = 0;
#pragma unroll
    for (int q = 0; q < TK_WPL; ++q) { c[q] = __popc(bits[sub * TK_WPL + q]); sum += c[q]; }
    uint32_t inc = sum;
#pragma unroll
    for (int o = 1; o < TK_GL; o <<= 1) {
        const uint32_t up = __shfl_up(inc, o, TK_GL);
        if (sub >= o) inc += up;
    }
    uint32_t run = inc - sum;
#pragma unroll
    for (int q = 0; q < TK_WPL; ++q) { prefix[sub * TK_WPL + q] = run; run += c[q]; }
}
__device__ __forceinline__ uint32_t bitmap_rank(const uint32_t* bits, const uint32_t* prefix, uint32_t q) {
    return prefix[q >> 5] + __popc(bits[q >> 5] & ((1u << (q & 31)) - 1u));
}

__global__ void __launch_bounds__(64) topk_write_cand(TopkArgs a, Scratch s) {
    constexpr int GROUPS = 64 / TK_GL;                         // chunks side by side in the wave
    constexpr int TURNS = TK_WPW / GROUPS;
    constexpr int SPEC = 8;                                    // slot entries per lane held in registers: 128 per chunk
    __shared__ uint32_t sel_all[GROUPS][TK_WORDS], eq_all[GROUPS][TK_WORDS], prefix_all[GROUPS][TK_WORDS];
    const int row = blockIdx.y;
    if (!s.rows[row].cand_mode) return;                     // uniform
    const int lane = threadIdx.x, grp = lane / TK_GL, sub = lane % TK_GL;
    uint32_t* sel_bits = sel_all[grp];
    uint32_t* eq_bits = eq_all[grp];
    uint32_t* prefix = prefix_all[grp];
    const uint32_t nchunks = s.nchunks;
    const uint32_t tau = s.rows[row].tau, r_tie = s.rows[row].r_tie;
    uint2* out = reinterpret_cast<uint2*>(a.msg + (uint64_t)row * a.k * 8);
    // All loads of the wave's chunks go out first: the slots' first 128 entries (what a slot normally holds; the
    // slot's memory exists whatever its fill, what lies behind `cnt` is discarded below) and the chunks' counters.
    uint2 ent[TURNS][SPEC];
    uint32_t cnt[TURNS], off0[TURNS], off1[TURNS], eqb[TURNS], ceq[TURNS];
#pragma unroll
    for (int tn = 0; tn < TURNS; ++tn) {
        const uint32_t want = blockIdx.x * TK_WPW + tn * GROUPS + grp;
        const uint32_t chunk = want < nchunks ? want : nchunks - 1;              // a clamped chunk is skipped below
        const size_t cidx = (size_t)row * nchunks + chunk;
#pragma unroll
        for (int u = 0; u < SPEC; ++u) {
            const uint32_t p = (uint32_t)u * TK_GL + sub;
            ent[tn][u] = make_uint2(s.slot_idx[cidx * TK_CAP + p], s.slot_val[cidx * TK_CAP + p]);   // .x: column in the chunk
        }
        cnt[tn] = s.cand_cnt[cidx];
        off0[tn] = s.out_off[(size_t)row * (nchunks + 1) + chunk];
        off1[tn] = s.out_off[(size_t)row * (nchunks + 1) + chunk + 1];
        eqb[tn] = s.eq_before[cidx];
        ceq[tn] = s.cnt_eq[cidx];
    }
#pragma unroll
    for (int tn = 0; tn < TURNS; ++tn) {
        // every lane walks through all barriers of a turn (one wave: they only order its LDS accesses); a group
        // with nothing to write idles through them
        const uint32_t chunk = blockIdx.x * TK_WPW + tn * GROUPS + grp;
        const bool active = chunk < nchunks && off0[tn] != off1[tn];
        const size_t cidx = (size_t)row * nchunks + (chunk < nchunks ? chunk : 0u);
        const uint32_t* slot_val = s.slot_val + cidx * TK_CAP;
        const uint16_t* slot_idx = s.slot_idx + cidx * TK_CAP;
        const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
        const uint32_t quota = (eqb[tn] < r_tie) ? (r_tie - eqb[tn]) : 0u;        // ties of this chunk that belong to the set
        const bool ties = active && ceq[tn] != 0 && quota != 0;
        const uint32_t n_ent = active ? cnt[tn] : 0u;
#pragma unroll
        for (int q = 0; q < TK_WPL; ++q) { sel_bits[sub * TK_WPL + q] = 0; eq_bits[sub * TK_WPL + q] = 0; }
        __syncthreads();
        auto mark = [&](uint32_t q, uint32_t bits) {
            const uint32_t key = bits & 0x7FFFFFFFu;
            if (key > tau) atomicOr(&sel_bits[q >> 5], 1u << (q & 31));
            else if (key == tau && ties) atomicOr(&eq_bits[q >> 5], 1u << (q & 31));
        };
#pragma unroll
        for (int u = 0; u < SPEC; ++u)
            if ((uint32_t)u * TK_GL + sub < n_ent) mark(ent[tn][u].x, ent[tn][u].y);
        for (uint32_t p = SPEC * TK_GL + sub; p < n_ent; p += TK_GL) mark(slot_idx[p], slot_val[p]);   // a fuller slot than usual
        __syncthreads();
        if (ties) bitmap_prefix(eq_bits, prefix, sub);          // all lanes of the group together
        __syncthreads();
        if (ties) {
#pragma unroll
            for (int q = 0; q < TK_WPL; ++q) {
                // keep the tied columns whose rank among the ties is below the quota
                const int w = sub * TK_WPL + q;
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
        }
        __syncthreads();
        bitmap_prefix(sel_bits, prefix, sub);
        __syncthreads();
        auto emit = [&](uint32_t q, uint32_t bits) {
            if (sel_bits[q >> 5] & (1u << (q & 31))) {
                const uint32_t pos = off0[tn] + bitmap_rank(sel_bits, prefix, q);
                if (pos < a.k && pos < off1[tn]) out[pos] = make_uint2((uint32_t)(c0 + q), bits);
            }
        };
#pragma unroll
        for (int u = 0; u < SPEC; ++u)
            if ((uint32_t)u * TK_GL + sub < n_ent) emit(ent[tn][u].x, ent[tn][u].y);
        for (uint32_t p = SPEC * TK_GL + sub; p < n_ent; p += TK_GL) emit(slot_idx[p], slot_val[p]);
        __syncthreads();                                    // the bitmaps are reused by the next turn
    }
}

// ---- GSpar: the magnitude-proportional sparsifier on the message conventions of the top-k path ------------
// A row's message is [count, 0][pairs ...]: the header takes the place of pair 0, so the message offsets of the
// chunks (out_off) start at 1 and the first pass / the flush apply the tail exactly as for top-k.
static_assert(TK_ITERS * (TK_THREADS / 64) == 16, "the chunk trees are written for 16 sweeps");

// Per row: S = sum |v| (the tree continued over the chunk sums, padded with zeros to a power of two), lambda = k / S.
__global__ void __launch_bounds__(TK_RTHREADS) gs_row_lambda(Scratch s, double k_expected) {
    __shared__ double wsum[TK_RTHREADS / 64];
    const int row = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t nchunks = s.nchunks;
    uint32_t per = 1;                                         // leaves per thread: a power of two
    while ((uint64_t)per * TK_RTHREADS < nchunks) per <<= 1;
    const double* leaf = s.csum + (size_t)row * nchunks;
    double stack[32];                                         // adjacent-pairs tree over this thread's leaves: a binary counter
    int sp = 0;
    const uint64_t first = (uint64_t)threadIdx.x * per;
    for (uint32_t e = 0; e < per; ++e) {
        const uint64_t c = first + e;
        double val = (c < nchunks) ? leaf[c] : 0.0;
        for (uint32_t bit = e; bit & 1u; bit >>= 1) val = stack[--sp] + val;
        stack[sp++] = val;
    }
    const double sum = wave_tree_sum_f64(stack[0]);           // per is a power of two: one entry is left
    if (lane == 0) wsum[wave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) t[q] = wsum[q];
#pragma unroll
        for (int len = 16; len > 1; len >>= 1)
#pragma unroll
            for (int q = 0; q < len / 2; ++q) t[q] = t[2 * q] + t[2 * q + 1];
        const float lambda = (t[0] > 0.0) ? (float)(k_expected / t[0]) : 0.f;
        const float used = s.rows[row].lambda_hi;              // what this step's first pass collected with (0: nothing)
        s.rows[row].lambda = lambda;
        const uint32_t mode = (used > 0.f && lambda <= used) ? 1u : 0u;
        s.rows[row].gs_mode = mode;
        s.rows[row].gs_need_count = mode ? 0u : s.nchunks;     // gs_sift adds the chunks whose slot overflowed
        s.rows[row].gs_need_write = 0u;                        // gs_count_dense adds the chunks that keep more than a slot
        // sum |v| of 10^5 .. 10^8 elements moves by a fraction of a per cent per step: 5 % of room costs 5 % more
        // slot entries to sift and is missed only when the state is replaced from outside
        s.rows[row].lambda_hi = (lambda > 0.f && lambda < 1.0e30f) ? lambda * 1.05f : 0.f;
    }
}
static_assert(TK_RTHREADS / 64 == 16, "the wave tree above is written for 16 waves");

// Per chunk, one wave each: a row whose first pass collected with an upper bound of lambda that held (gs_mode)
// only sifts what that pass left in the slot -- the elements with u < lambda_hi |v|, a superset of the kept ones
// in column order -- and closes the gaps in place.  Chunks with more of them than a slot holds, and rows without a
// bound that held, are left to gs_count_dense.
constexpr int GS_WAVES = 4;                                   // chunks per workgroup
__device__ __forceinline__ bool gs_chunk_is_sifted(const Scratch& s, int row, size_t slot) {
    return s.rows[row].gs_mode && s.cand_cnt[slot] <= (uint32_t)TK_CAP;
}
__global__ void __launch_bounds__(GS_WAVES * 64) gs_sift(TopkArgs a, Scratch s) {
    const int row = blockIdx.y;
    const uint32_t chunk = blockIdx.x * GS_WAVES + (threadIdx.x >> 6);
    if (chunk >= s.nchunks) return;
    const size_t slot = (size_t)row * s.nchunks + chunk;
    const int lane = threadIdx.x & 63;
    if (!gs_chunk_is_sifted(s, row, slot)) {                   // uniform over the wave
        if (s.rows[row].gs_mode && lane == 0) atomicAdd(&s.rows[row].gs_need_count, 1u);
        return;
    }
    const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
    const float lambda = s.rows[row].lambda;
    const uint32_t t_lo = (uint32_t)*a.t_ptr;
    uint32_t* slot_val = s.slot_val + slot * TK_CAP;
    uint16_t* slot_idx = s.slot_idx + slot * TK_CAP;
    const uint32_t have = s.cand_cnt[slot];
    const unsigned long long below = (1ull << lane) - 1ull;
    uint32_t kept = 0;
    for (uint32_t p0 = 0; p0 < have; p0 += 64) {               // a kept entry moves to a place at or before its own,
        const uint32_t p = p0 + lane;                          // which this or an earlier round has already read
        uint32_t val = 0;
        uint16_t idx = 0;
        bool keep = false;
        if (p < have) {
            val = slot_val[p];
            idx = slot_idx[p];
            const uint64_t j = c0 + idx;
            uint32_t rnd[4];
            philox4x32_10((uint32_t)(j >> 2), (uint32_t)row, t_lo, kGsparStreamTag, a.seed_lo, a.seed_hi, rnd);
            const uint32_t word = (j & 3) == 0 ? rnd[0] : (j & 3) == 1 ? rnd[1] : (j & 3) == 2 ? rnd[2] : rnd[3];
            keep = (float)(word >> 8) * (1.0f / 16777216.0f) < lambda * fabsf(__uint_as_float(val));
        }
        const unsigned long long m = __ballot(keep);
        if (keep) {
            const uint32_t pos = kept + (uint32_t)__popcll(m & below);
            slot_val[pos] = val;
            slot_idx[pos] = idx;
        }
        kept += (uint32_t)__popcll(m);
    }
    if (lane == 0) s.cnt_gt[slot] = kept;
}

// The chunks gs_sift left out: decisions from v itself, the kept elements in column order into the slot (the first
// TK_CAP of them), their number.  A fixed number of workgroups per row walks the chunks, so that a step in which
// every chunk was sifted pays little for the launch.
__global__ void __launch_bounds__(TK_THREADS) gs_count_dense(TopkArgs a, Scratch s) {
    __shared__ unsigned long long wave_sums4[TK_THREADS / 64];
    const int row = blockIdx.y;
    if (s.rows[row].gs_need_count == 0u) return;              // every chunk of the row was sifted
    const float lambda = s.rows[row].lambda;
    const uint32_t t_lo = (uint32_t)*a.t_ptr;
    const float* dr = a.delta + (uint64_t)row * a.ld;         // holds v
    for (uint32_t chunk = blockIdx.x; chunk < s.nchunks; chunk += gridDim.x) {
        const size_t slot = (size_t)row * s.nchunks + chunk;
        if (gs_chunk_is_sifted(s, row, slot)) continue;        // uniform
        const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
        float4 vin[TK_ITERS];
        uint32_t keep[TK_ITERS];
#pragma unroll
        for (int it = 0; it < TK_ITERS; ++it) vin[it] = ld4_stream(dr + c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x);   // rows are padded to whole chunks
#pragma unroll
        for (int it = 0; it < TK_ITERS; ++it) keep[it] = gs_keep4(a, row, c0 + (uint64_t)it * TK_VEC + 4 * threadIdx.x, t_lo, lambda, vin[it]);
        const uint32_t n = gs_collect(vin, keep, s.slot_val + slot * TK_CAP, s.slot_idx + slot * TK_CAP, wave_sums4);
        if (threadIdx.x == 0) {
            s.cnt_gt[slot] = n;
            if (n > (uint32_t)TK_CAP) atomicAdd(&s.rows[row].gs_need_write, 1u);
        }
    }
}

// Per row: where each chunk's pairs go in the message (offsets in pairs from the start of the row, the header
// being pair 0), the header, zeros behind a message shorter than the last one, the overflow flag.
__global__ void __launch_bounds__(TK_RTHREADS) gs_scan(TopkArgs a, Scratch s) {
    __shared__ uint32_t wave_sums[TK_RTHREADS / 64];
    const int row = blockIdx.x;
    const uint32_t nchunks = s.nchunks;
    const uint32_t cap = (uint32_t)a.k - 1u;                  // pairs the message has room for
    const uint32_t* cnt = s.cnt_gt + (size_t)row * nchunks;
    uint32_t* off = s.out_off + (size_t)row * (nchunks + 1);
    uint32_t base = 0;
    for (uint32_t b0 = 0; b0 < nchunks; b0 += TK_RTHREADS) {
        const uint32_t c = b0 + threadIdx.x;
        const uint32_t mine = (c < nchunks) ? cnt[c] : 0u;
        uint32_t tot;
        const uint32_t before = base + row_exclusive_scan(mine, wave_sums, &tot);
        if (c < nchunks) off[c] = 1u + (before < cap ? before : cap);       // never past the row's last pair
        base += tot;
    }
    const uint32_t count = base < cap ? base : cap;
    uint2* mrow = reinterpret_cast<uint2*>(a.msg + (uint64_t)row * a.k * 8);
    const uint32_t last = s.rows[row].gs_total;
    for (uint32_t p = count + threadIdx.x; p < last; p += TK_RTHREADS) mrow[1 + p] = make_uint2(0u, 0u);
    __syncthreads();                                          // every thread has read gs_total
    if (threadIdx.x == 0) {
        off[nchunks] = 1u + count;
        mrow[0] = make_uint2(count, 0u);
        s.rows[row].gs_total = count;
        if (base > cap) atomicOr(s.gs_overflow, 1u);
    }
}

// Per chunk, one wave each: the slot's pairs to their place in the message.  Chunks that kept more than a slot
// holds are left to gs_write_dense.
__global__ void __launch_bounds__(GS_WAVES * 64) gs_write(TopkArgs a, Scratch s) {
    const int row = blockIdx.y;
    const uint32_t chunk = blockIdx.x * GS_WAVES + (threadIdx.x >> 6);
    if (chunk >= s.nchunks) return;
    const size_t slot = (size_t)row * s.nchunks + chunk;
    const uint32_t cnt = s.cnt_gt[slot];
    if (cnt > (uint32_t)TK_CAP) return;                        // uniform over the wave
    const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
    const uint32_t limit = (uint32_t)a.k;                     // pair positions of the row: [1, limit)
    const uint32_t base = s.out_off[(size_t)row * (s.nchunks + 1) + chunk];
    uint2* mrow = reinterpret_cast<uint2*>(a.msg + (uint64_t)row * a.k * 8);
    const uint32_t* slot_val = s.slot_val + slot * TK_CAP;
    const uint16_t* slot_idx = s.slot_idx + slot * TK_CAP;
    for (uint32_t p = threadIdx.x & 63; p < cnt; p += 64)
        if (base + p < limit) mrow[base + p] = make_uint2((uint32_t)(c0 + slot_idx[p]), slot_val[p]);
}

// The chunks that kept more than a slot holds decide again from v and write their pairs directly.
__global__ void __launch_bounds__(TK_THREADS) gs_write_dense(TopkArgs a, Scratch s) {
    __shared__ uint32_t wave_sums[TK_THREADS / 64];
    const int row = blockIdx.y;
    if (s.rows[row].gs_need_write == 0u) return;              // no chunk of the row kept more than its slot holds
    const uint32_t limit = (uint32_t)a.k;
    uint2* mrow = reinterpret_cast<uint2*>(a.msg + (uint64_t)row * a.k * 8);
    const float lambda = s.rows[row].lambda;
    const uint32_t t_lo = (uint32_t)*a.t_ptr;                 // the step's counter: advanced only after this kernel
    const float* dr = a.delta + (uint64_t)row * a.ld;
    for (uint32_t chunk = blockIdx.x; chunk < s.nchunks; chunk += gridDim.x) {
        if (s.cnt_gt[(size_t)row * s.nchunks + chunk] <= (uint32_t)TK_CAP) continue;    // uniform
        const uint64_t c0 = (uint64_t)chunk * TK_CHUNK;
        uint32_t run = s.out_off[(size_t)row * (s.nchunks + 1) + chunk];
        for (int it = 0; it < TK_ITERS; ++it) {
            const uint32_t q0 = (uint32_t)it * TK_VEC + 4 * threadIdx.x;
            const float4 v = ld4_stream(dr + c0 + q0);
            const uint32_t keep = gs_keep4(a, row, c0 + q0, t_lo, lambda, v);
            uint32_t tot;
            uint32_t pos = run + block_exclusive_scan(__popc(keep), wave_sums, &tot);
            const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (keep & (1u << c)) {
                    if (pos < limit) mrow[pos] = make_uint2((uint32_t)(c0 + q0 + c), __float_as_uint(vv[c]));
                    ++pos;
                }
            run += tot;
        }
    }
}

__global__ void gs_close(unsigned long long* t_ptr) { atomicAdd(t_ptr, 1ull); }      // one step taken

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
    bool gspar = false;            // the GSpar operator runs on this state (its own select-free chain of kernels)
    bool pending = false;          // a step has been enqueued since the last flush (or may have been, by a
                                   // replayed graph): its sparse tail may not have been applied yet
};

void topk_destroy(TopkState* st) {
    if (!st) return;
    void* ptrs[] = {st->s.hist, st->s.hist_part, st->s.hist2, st->s.hist3, st->s.rows, st->s.cnt_gt, st->s.cnt_eq, st->s.eq_before, st->s.out_off, st->s.cand_cnt, st->s.slot_val, st->s.slot_idx,
                    st->s.list, st->s.csum, st->s.gs_overflow};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    delete st;
}

ds_status topk_create(const ds_config& cfg, uint64_t ld, TopkState** out, std::string& err) {
    TopkState* st = new TopkState();
    st->n = cfg.n;
    st->gspar = cfg.comp.kind == DS_COMP_GSPAR;
    Scratch& s = st->s;
    s.nchunks = (uint32_t)((cfg.N + TK_CHUNK - 1) / TK_CHUNK);
    // the first pass reads and writes whole chunks of x and delta
    if ((uint64_t)s.nchunks * TK_CHUNK > ld) { err = "internal: row pitch smaller than the chunked row"; delete st; return DS_EINVAL; }
    const size_t n = (size_t)cfg.n, nc = s.nchunks;
    bool ok = hipMalloc(&s.hist, n * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.hist_part, n * TK_HPARTS * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.hist2, n * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.hist3, n * BINS3 * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.rows, n * sizeof(TopkRow)) == hipSuccess &&
              hipMalloc(&s.cnt_gt, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.cnt_eq, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.eq_before, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.out_off, n * (nc + 1) * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.cand_cnt, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.slot_val, n * nc * TK_CAP * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.slot_idx, n * nc * TK_CAP * sizeof(uint16_t)) == hipSuccess &&
              hipMalloc(&s.list, n * TK_LIST_CAP * sizeof(uint2)) == hipSuccess &&
              hipMalloc(&s.csum, (st->gspar ? n * nc : 1) * sizeof(double)) == hipSuccess &&
              hipMalloc(&s.gs_overflow, sizeof(uint32_t)) == hipSuccess;
    ok = ok && hipMemset(s.hist, 0, n * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s.hist_part, 0, n * TK_HPARTS * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s.hist2, 0, n * HIST_BINS * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s.hist3, 0, n * BINS3 * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s.out_off, 0, n * (nc + 1) * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s.cand_cnt, 0, n * nc * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s.gs_overflow, 0, sizeof(uint32_t)) == hipSuccess;
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
    for (const TopkRow& r : rows) c += (st->gspar ? r.gs_mode : r.cand_mode) ? 1u : 0u;
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

ds_status gspar_overflowed(TopkState* st, hipStream_t stream, bool* overflowed) {
    uint32_t flag = 0;
    if (hipStreamSynchronize(stream) != hipSuccess) return DS_EHIP;
    if (hipMemcpy(&flag, st->s.gs_overflow, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess) return DS_EHIP;
    *overflowed = flag != 0;
    return DS_OK;
}

ds_status topk_step(TopkState* st, const TopkArgs& a, hipStream_t stream) {
    const Scratch& s = st->s;
    const dim3 grid(s.nchunks, a.n), block(TK_THREADS), rblock(TK_RTHREADS);
    if (st->gspar) {
        // form (tail of the last step, line 5, sums of |v|, what can be kept at all) -> lambda -> kept elements and
        // their number per chunk -> offsets -> pairs
        hipLaunchKernelGGL(topk_form_collect<true>, grid, block, 0, stream, a, s);
        hipLaunchKernelGGL(gs_row_lambda, dim3(a.n), rblock, 0, stream, s, (double)a.k_expected);
        const dim3 wgrid((s.nchunks + GS_WAVES - 1) / GS_WAVES, a.n), wblock(GS_WAVES * 64);
        const dim3 dgrid(s.nchunks < (uint32_t)TK_FWG ? s.nchunks : (uint32_t)TK_FWG, a.n);
        hipLaunchKernelGGL(gs_sift, wgrid, wblock, 0, stream, a, s);
        hipLaunchKernelGGL(gs_count_dense, dgrid, block, 0, stream, a, s);
        hipLaunchKernelGGL(gs_scan, dim3(a.n), rblock, 0, stream, a, s);
        hipLaunchKernelGGL(gs_write, wgrid, wblock, 0, stream, a, s);
        hipLaunchKernelGGL(gs_write_dense, dgrid, block, 0, stream, a, s);
        hipLaunchKernelGGL(gs_close, dim3(1), dim3(1), 0, stream, a.t_ptr);
        st->pending = true;
        return hipGetLastError() == hipSuccess ? DS_OK : DS_EHIP;
    }
    const dim3 wgrid((s.nchunks + TK_WPW - 1) / TK_WPW, a.n);
    // full mode walks a row's chunks with a fixed number of workgroups, so that a step in which no row needs it
    // pays little for the launches
    const dim3 fgrid(s.nchunks < (uint32_t)TK_FWG ? s.nchunks : (uint32_t)TK_FWG, a.n);
    const dim3 hgrid(TK_HWG, a.n), hblock(TK_HTHREADS);
    const dim3 rows(a.n);
    const uint32_t k = (uint32_t)a.k;
    // after a flush (and at the start) all message offsets are zero, so the first pass finds no tail to apply
    hipLaunchKernelGGL(topk_form_collect<false>, grid, block, 0, stream, a, s);
    hipLaunchKernelGGL(topk_decide_select, rows, block, 0, stream, s, k);
    hipLaunchKernelGGL(topk_hist_cand2, hgrid, hblock, 0, stream, s);
    hipLaunchKernelGGL(topk_select2_cand, rows, block, 0, stream, s);
    hipLaunchKernelGGL(topk_bin_collect, hgrid, hblock, 0, stream, s);
    hipLaunchKernelGGL(topk_hist_full<1>, fgrid, block, 0, stream, a.delta, a.ld, a.N, s, k);
    hipLaunchKernelGGL(topk_hist_full<2>, fgrid, block, 0, stream, a.delta, a.ld, a.N, s, k);
    hipLaunchKernelGGL(topk_hist_full<3>, fgrid, block, 0, stream, a.delta, a.ld, a.N, s, k);
    hipLaunchKernelGGL(topk_fix_full, fgrid, block, 0, stream, a.delta, a.ld, a.N, s);
    hipLaunchKernelGGL(topk_finish, rows, rblock, 0, stream, s, k, a.t_ptr);
    hipLaunchKernelGGL(topk_write_cand, wgrid, dim3(64), 0, stream, a, s);
    hipLaunchKernelGGL(topk_write_full, fgrid, block, 0, stream, a, s);
    st->pending = true;
    return DS_OK;
}

}  // namespace dsq

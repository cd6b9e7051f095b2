// Norm-rescaled b-bit path of libdsq (gfx950): the compression the paper's experiments describe
// (section "Experimental Setup", paragraph "Compression"): every element of a worker's vector is
// sent as a b-bit code together with ONE number, the Euclidean norm of the vector, and the
// receiver scales what it decodes to that norm.
//
//   s    = max_j |v_j|                       (range of the 2^b level grid; not sent)
//   q_j  = rint(clamp(fma(v_j, (L/2)/s, L/2), 0, L)),  L = 2^b - 1   (nearest level, ties to even)
//   y_j  = 2 q_j - L                         (odd integer in [-L, L])
//   nrm  = fp32(sqrt(S2)),  S2 = sum_j v_j^2 in double, balanced adjacent-pairs tree over the
//          zero-padded vector (the square of a float is exact in double)
//   C[v] = y * unit,  unit = fp32(nrm / sqrt(sum_j y_j^2))   (double arithmetic, one rounding)
//
// Both the range and the decode scale are properties of the whole vector, so Algorithm 1's
// lines 5-9 cannot be one pass: the codes need s, and delta = v - C[v] and the gossip sum need
// unit.  A step is therefore
//   form      (dense)  [tail of the previous step] ; xh = x - gamma g -> x ; v = xh + delta -> delta ;
//                      per-chunk max|v| and tree sums of v^2
//   row_scale (tiny)   s, nrm per row
//   quantize  (dense)  read v, write the codes into the message, per-chunk sum of y^2
//   row_unit  (tiny)   unit per row, the norm into the message header, step counter
// and the step's tail -- delta = v - C[v] (line 6) and x = xh + eta sum_j a_ij C[v_j] (line 9), both
// functions of the codes and the n units only -- is folded into the NEXT step's `form` pass, which
// streams x and delta anyway, or applied by l2q_flush before anyone else looks at the state.
// Traffic per element and step: form 12 B read + 8 B written (+ (deg+1) b/8 B of codes, mostly
// L2 hits), quantize 4 B read + b/8 B written: 24 B + codes against the 20 B + b/8 B any
// implementation must move.

#include "dsq_internal.h"

namespace dsq {

namespace {

constexpr int LQ_THREADS = 256;
constexpr int LQ_ITERS = 4;
constexpr int LQ_CHUNK = 4 * LQ_THREADS * LQ_ITERS;       // 4096 columns per workgroup
constexpr int LQ_ROW_THREADS = 1024;                      // threads of the per-row kernels

struct L2Row {
    float s;          // max |v| of the row
    float inv;        // (L/2) / s, or 0 for an all-zero row
    float nrm;        // the Euclidean norm that is sent
    float unit;       // decode scale nrm / ||y||
};

struct L2Scratch {
    L2Row* rows;                  // n
    float* cmax;                  // n x nchunks: max |v| of the chunk
    double* csq;                  // n x nchunks: tree sum of v^2 over the chunk
    uint32_t* csy2;               // n x nchunks: sum of y^2 over the chunk (< 2^32: 4096 * 255^2)
    uint32_t* pending;            // 1: the last step's tail has not been applied to x and delta yet
    uint32_t nchunks;
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

// The four b-bit codes of columns col..col+3 of one worker's message (col a multiple of 4).
template <int BITS>
__device__ __forceinline__ uint32_t load_codes4(const uint8_t* msg_row, uint64_t col) {
    if constexpr (BITS == 2) return msg_row[4 + (col >> 2)];
    else if constexpr (BITS == 4) return *reinterpret_cast<const uint16_t*>(msg_row + 4 + (col >> 1));
    else return *reinterpret_cast<const uint32_t*>(msg_row + 4 + col);
}

// Lines 6 (second half) and 9 of Algorithm 1 for four adjacent columns of worker `row`, from the
// codes in the message buffer: d holds v and becomes delta, xh becomes x.
template <int BITS>
__device__ __forceinline__ void apply_tail4(const L2Args& a, const L2Scratch& s, int row, uint64_t col,
                                            float4& xh, float4& d) {
    constexpr int L = (1 << BITS) - 1;
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    float* xp = reinterpret_cast<float*>(&xh);
    float* dp = reinterpret_cast<float*>(&d);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    float own[4] = {0.f, 0.f, 0.f, 0.f};
    const int e0 = a.rowptr[row], e1 = a.rowptr[row + 1];
    for (int e = e0; e < e1; ++e) {                       // ascending neighbour index, own index included
        const int nb = a.col[e];
        const float coef = a.coef[e];
        const float unit = s.rows[nb].unit;
        const uint32_t codes = load_codes4<BITS>(a.msg + (uint64_t)nb * a.msg_row_bytes, col);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int y = 2 * (int)((codes >> (BITS * c)) & MASK) - L;
            const float cv = (float)y * unit;
            acc[c] = fmaf(coef, cv, acc[c]);
            if (nb == row) own[c] = cv;
        }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (col + c < a.N) {                              // padding columns stay zero
            dp[c] = dp[c] - own[c];
            xp[c] = fmaf(a.eta, acc[c], xp[c]);
        }
    }
}

__device__ __forceinline__ double wave_tree_sum(double v) {   // adjacent pairs first; every lane gets the sum
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) v += __shfl_xor(v, o);
    return v;
}

// First pass of a step: the previous step's tail (if pending), then line 5.
template <int BITS>
__global__ void __launch_bounds__(LQ_THREADS) l2q_form(L2Args a, L2Scratch s) {
    __shared__ double sweep_sq[LQ_ITERS * (LQ_THREADS / 64)];
    __shared__ float wave_max[LQ_THREADS / 64];
    const int row = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t col0 = (uint64_t)blockIdx.x * LQ_CHUNK;
    const bool tail = *s.pending != 0u;
    float* xr = a.x + (uint64_t)row * a.ld;
    float* dr = a.delta + (uint64_t)row * a.ld;
    const float* gr = a.g + (uint64_t)row * a.g_ld;
    float vmax = 0.f;
#pragma unroll
    for (int it = 0; it < LQ_ITERS; ++it) {
        const uint64_t col = col0 + (uint64_t)it * (4 * LQ_THREADS) + 4u * threadIdx.x;   // < ld: ld is a multiple of the chunk
        float4 x4 = ld4_stream(xr + col), d4 = ld4_stream(dr + col);
        float4 g4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (col < a.N) {                                  // g_ld >= N and a multiple of 4: the float4 is inside the row
            g4 = ld4_stream(gr + col);
            if (col + 3 >= a.N) {                         // whatever lies behind column N-1 is not a gradient
                if (col + 1 >= a.N) g4.y = 0.f;
                if (col + 2 >= a.N) g4.z = 0.f;
                g4.w = 0.f;
            }
            if (tail) apply_tail4<BITS>(a, s, row, col, x4, d4);
        }
        float4 xh, v;
        xh.x = fmaf(-a.gamma, g4.x, x4.x); xh.y = fmaf(-a.gamma, g4.y, x4.y);
        xh.z = fmaf(-a.gamma, g4.z, x4.z); xh.w = fmaf(-a.gamma, g4.w, x4.w);
        v.x = xh.x + d4.x; v.y = xh.y + d4.y; v.z = xh.z + d4.z; v.w = xh.w + d4.w;
        st4_stream(xr + col, xh);
        st4_stream(dr + col, v);
        vmax = fmaxf(vmax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
        const double q0 = (double)v.x * (double)v.x, q1 = (double)v.y * (double)v.y;
        const double q2 = (double)v.z * (double)v.z, q3 = (double)v.w * (double)v.w;
        const double sw = wave_tree_sum((q0 + q1) + (q2 + q3));
        if (lane == 0) sweep_sq[it * (LQ_THREADS / 64) + wave] = sw;      // sweep index = column order
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, o));
    if (lane == 0) wave_max[wave] = vmax;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) t[k] = sweep_sq[k];
#pragma unroll
        for (int len = 16; len > 1; len >>= 1)
#pragma unroll
            for (int p = 0; p < len / 2; ++p) t[p] = t[2 * p] + t[2 * p + 1];
        const size_t slot = (size_t)row * s.nchunks + blockIdx.x;
        s.csq[slot] = t[0];
        s.cmax[slot] = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
    }
}
static_assert(LQ_ITERS * (LQ_THREADS / 64) == 16, "the chunk tree below is written for 16 sweeps");

// Per row: s = max of the chunk maxima; S2 = the tree continued over the chunks (padded with
// zeros to a power of two); nrm = fp32(sqrt(S2)).
__global__ void __launch_bounds__(LQ_ROW_THREADS) l2q_row_scale(L2Scratch s, float half_levels) {
    __shared__ double wsum[LQ_ROW_THREADS / 64];
    __shared__ float wmax[LQ_ROW_THREADS / 64];
    const int row = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t nchunks = s.nchunks;
    uint32_t per = 1;                                     // leaves per thread: a power of two
    while ((uint64_t)per * LQ_ROW_THREADS < nchunks) per <<= 1;
    const double* sq = s.csq + (size_t)row * nchunks;
    const float* mx = s.cmax + (size_t)row * nchunks;
    // adjacent-pairs tree over this thread's `per` leaves: a binary counter of partial sums
    double stack[32];
    int sp = 0;
    float vmax = 0.f;
    const uint64_t first = (uint64_t)threadIdx.x * per;
    for (uint32_t e = 0; e < per; ++e) {
        const uint64_t c = first + e;
        double val = 0.0;
        if (c < nchunks) { val = sq[c]; vmax = fmaxf(vmax, mx[c]); }
        for (uint32_t bit = e; bit & 1u; bit >>= 1) val = stack[--sp] + val;
        stack[sp++] = val;
    }
    double sum = wave_tree_sum(stack[0]);                 // per is a power of two: one entry is left
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, o));
    if (lane == 0) { wsum[wave] = sum; wmax[wave] = vmax; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t[16];
        float m = 0.f;
#pragma unroll
        for (int k = 0; k < 16; ++k) { t[k] = wsum[k]; m = fmaxf(m, wmax[k]); }
#pragma unroll
        for (int len = 16; len > 1; len >>= 1)
#pragma unroll
            for (int p = 0; p < len / 2; ++p) t[p] = t[2 * p] + t[2 * p + 1];
        L2Row r = s.rows[row];
        r.s = m;
        r.inv = (m > 0.f) ? half_levels / m : 0.f;
        r.nrm = (float)sqrt(t[0]);
        s.rows[row] = r;
    }
}
static_assert(LQ_ROW_THREADS / 64 == 16, "the wave tree above is written for 16 waves");

// Second pass: the codes of v (which `form` left in delta), and sum y^2 per chunk.
template <int BITS>
__global__ void __launch_bounds__(LQ_THREADS) l2q_quantize(L2Args a, L2Scratch s) {
    constexpr int L = (1 << BITS) - 1;
    __shared__ uint32_t wave_sy2[LQ_THREADS / 64];
    const int row = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t col0 = (uint64_t)blockIdx.x * LQ_CHUNK;
    const float inv = s.rows[row].inv;
    const bool zero_row = !(s.rows[row].s > 0.f);
    const float hl = 0.5f * (float)L;
    const float* dr = a.delta + (uint64_t)row * a.ld;
    uint8_t* mrow = a.msg + (uint64_t)row * a.msg_row_bytes;
    const uint64_t code_bytes = a.msg_row_bytes - 4;      // whole 32-bit words
    uint32_t sy2 = 0;
#pragma unroll
    for (int it = 0; it < LQ_ITERS; ++it) {
        const uint64_t col = col0 + (uint64_t)it * (4 * LQ_THREADS) + 4u * threadIdx.x;
        const uint64_t byte = col * BITS / 8;
        if (byte >= code_bytes) continue;                 // behind the last code word of the row
        const float4 v4 = ld4_stream(dr + col);
        const float* vp = reinterpret_cast<const float*>(&v4);
        uint32_t packed = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (col + c < a.N) {                          // padding codes are 0 and do not count
                int q = 0;
                if (!zero_row) {
                    float t = fmaf(vp[c], inv, hl);
                    t = (t > 0.f) ? t : 0.f;              // also sends NaN to 0
                    t = (t < (float)L) ? t : (float)L;
                    q = (int)rintf(t);                    // nearest, ties to even
                }
                const int y = 2 * q - L;
                sy2 += (uint32_t)(y * y);
                packed |= (uint32_t)q << (BITS * c);
            }
        }
        if constexpr (BITS == 2) mrow[4 + byte] = (uint8_t)packed;
        else if constexpr (BITS == 4) *reinterpret_cast<uint16_t*>(mrow + 4 + byte) = (uint16_t)packed;
        else *reinterpret_cast<uint32_t*>(mrow + 4 + byte) = packed;
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) sy2 += __shfl_xor(sy2, o);
    if (lane == 0) wave_sy2[wave] = sy2;
    __syncthreads();
    if (threadIdx.x == 0)
        s.csy2[(size_t)row * s.nchunks + blockIdx.x] = wave_sy2[0] + wave_sy2[1] + wave_sy2[2] + wave_sy2[3];
}

// Per row: sum y^2 (an integer, any order), the decode scale, the message header; the step is
// complete up to its tail, which is now pending.
__global__ void __launch_bounds__(LQ_ROW_THREADS) l2q_row_unit(L2Args a, L2Scratch s) {
    __shared__ unsigned long long wsum[LQ_ROW_THREADS / 64];
    const int row = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t* sy = s.csy2 + (size_t)row * s.nchunks;
    unsigned long long sum = 0;
    for (uint32_t c = threadIdx.x; c < s.nchunks; c += LQ_ROW_THREADS) sum += sy[c];
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) wsum[wave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long total = 0;
#pragma unroll
        for (int k = 0; k < LQ_ROW_THREADS / 64; ++k) total += wsum[k];
        L2Row r = s.rows[row];
        r.unit = (float)((double)r.nrm / sqrt((double)total));           // total >= N >= 1
        s.rows[row] = r;
        *reinterpret_cast<float*>(a.msg + (uint64_t)row * a.msg_row_bytes) = r.nrm;
        if (row == 0) {
            *s.pending = 1u;
            atomicAdd(a.t_ptr, 1ull);                                    // one step taken
        }
    }
}

// The tail on its own (l2q_flush): delta = v - C[v], x = xh + eta sum_j a_ij C[v_j].
template <int BITS>
__global__ void __launch_bounds__(LQ_THREADS) l2q_tail(L2Args a, L2Scratch s) {
    if (*s.pending == 0u) return;
    const int row = blockIdx.y;
    const uint64_t col0 = (uint64_t)blockIdx.x * LQ_CHUNK;
    float* xr = a.x + (uint64_t)row * a.ld;
    float* dr = a.delta + (uint64_t)row * a.ld;
#pragma unroll
    for (int it = 0; it < LQ_ITERS; ++it) {
        const uint64_t col = col0 + (uint64_t)it * (4 * LQ_THREADS) + 4u * threadIdx.x;
        if (col >= a.N) continue;
        float4 x4 = ld4_stream(xr + col), d4 = ld4_stream(dr + col);
        apply_tail4<BITS>(a, s, row, col, x4, d4);
        st4_stream(xr + col, x4);
        st4_stream(dr + col, d4);
    }
}

__global__ void l2q_clear_pending(L2Scratch s) { *s.pending = 0u; }

}  // namespace

struct L2State {
    L2Scratch s{};
    int n = 0, bits = 0;
    bool stepped = false;          // a step has been enqueued (or may have been, by a replayed graph)
};

void l2q_destroy(L2State* st) {
    if (!st) return;
    L2Scratch& s = st->s;
    void* ptrs[] = {s.rows, s.cmax, s.csq, s.csy2, s.pending};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    delete st;
}

ds_status l2q_create(const ds_config& cfg, uint64_t ld, L2State** out, std::string& err) {
    L2State* st = new (std::nothrow) L2State();
    if (!st) { err = "out of host memory"; return DS_ENOMEM; }
    st->n = cfg.n;
    st->bits = cfg.comp.bits;
    L2Scratch& s = st->s;
    s.nchunks = (uint32_t)((cfg.N + LQ_CHUNK - 1) / LQ_CHUNK);
    if ((uint64_t)s.nchunks * LQ_CHUNK > ld) { err = "internal: row pitch smaller than the chunked row"; l2q_destroy(st); return DS_EINVAL; }
    const size_t n = (size_t)cfg.n, nc = s.nchunks;
    bool ok = hipMalloc(&s.rows, n * sizeof(L2Row)) == hipSuccess &&
              hipMalloc(&s.cmax, n * nc * sizeof(float)) == hipSuccess &&
              hipMalloc(&s.csq, n * nc * sizeof(double)) == hipSuccess &&
              hipMalloc(&s.csy2, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.pending, sizeof(uint32_t)) == hipSuccess;
    ok = ok && hipMemset(s.rows, 0, n * sizeof(L2Row)) == hipSuccess &&
         hipMemset(s.pending, 0, sizeof(uint32_t)) == hipSuccess && hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        err = "scratch allocation for the norm-rescaled compressor failed";
        l2q_destroy(st);
        return DS_ENOMEM;
    }
    *out = st;
    return DS_OK;
}

ds_status l2q_step(L2State* st, const L2Args& a, hipStream_t stream) {
    const L2Scratch& s = st->s;
    const dim3 grid(s.nchunks, a.n), block(LQ_THREADS), rows(a.n), rblock(LQ_ROW_THREADS);
    const float hl = 0.5f * (float)((1 << st->bits) - 1);
    // All rows go through `form` before any row's codes are replaced: the tail that `form` applies reads the
    // previous step's codes of the neighbours.  (Splitting the rows into groups that run form -> quantize
    // back to back, hoping that v is still in the memory-side cache, was measured slower at every group size.)
    if (st->bits == 2)      hipLaunchKernelGGL(l2q_form<2>, grid, block, 0, stream, a, s);
    else if (st->bits == 4) hipLaunchKernelGGL(l2q_form<4>, grid, block, 0, stream, a, s);
    else                    hipLaunchKernelGGL(l2q_form<8>, grid, block, 0, stream, a, s);
    hipLaunchKernelGGL(l2q_row_scale, rows, rblock, 0, stream, s, hl);
    if (st->bits == 2)      hipLaunchKernelGGL(l2q_quantize<2>, grid, block, 0, stream, a, s);
    else if (st->bits == 4) hipLaunchKernelGGL(l2q_quantize<4>, grid, block, 0, stream, a, s);
    else                    hipLaunchKernelGGL(l2q_quantize<8>, grid, block, 0, stream, a, s);
    hipLaunchKernelGGL(l2q_row_unit, rows, rblock, 0, stream, a, s);
    st->stepped = true;
    return hipGetLastError() == hipSuccess ? DS_OK : DS_EHIP;
}

ds_status l2q_flush(L2State* st, const L2Args& a, hipStream_t stream) {
    if (!st || !st->stepped) return DS_OK;
    const L2Scratch& s = st->s;
    const dim3 grid(s.nchunks, a.n), block(LQ_THREADS);
    // the kernels look at the device's pending flag themselves: a replayed graph of ds_step sets it
    // without this code noticing
    if (st->bits == 2)      hipLaunchKernelGGL(l2q_tail<2>, grid, block, 0, stream, a, s);
    else if (st->bits == 4) hipLaunchKernelGGL(l2q_tail<4>, grid, block, 0, stream, a, s);
    else                    hipLaunchKernelGGL(l2q_tail<8>, grid, block, 0, stream, a, s);
    hipLaunchKernelGGL(l2q_clear_pending, dim3(1), dim3(1), 0, stream, s);
    return hipGetLastError() == hipSuccess ? DS_OK : DS_EHIP;
}

}  // namespace dsq

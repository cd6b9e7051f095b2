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
//
// Speculative codes (what makes the second dense pass unnecessary in steady state).  The code of an
// element depends on the row's range s only through inv = (L/2)/s, and is monotone in it.  `form`
// therefore takes a band [s_lo, s_hi] guessed from the previous steps, computes every element's code
// for both ends, and writes the code straight into the message where the two agree (then it is the
// code for every s inside the band).  The few elements whose two codes differ (those next to a level
// boundary, ~1 % at 2 bits and a band of +-20 %) go into a per-chunk slot with their value.  Once
// row_scale knows s: if it lies inside the band and no slot overflowed, the second-pass kernel only
// settles the slotted elements of each chunk (an xor on their bits of the message word, a correction
// of the chunk's sum of y^2); otherwise it is the exact second pass over v as before.
// The results never depend on the guess.  Because `form` now writes codes while other workgroups
// still read the previous step's codes for the tail, the messages alternate between two buffers;
// cell 4 of the step cells names the one the last completed step wrote.

#include "dsq_internal.h"

namespace dsq {

namespace {

constexpr int LQ_THREADS = 256;
constexpr int LQ_ITERS = 4;
constexpr int LQ_CHUNK = 4 * LQ_THREADS * LQ_ITERS;       // 4096 columns per workgroup
constexpr int LQ_ROW_THREADS = 1024;                      // threads of the per-row kernels

constexpr uint32_t LQ_UCAP = 256;                         // slotted (undecided) elements a chunk has room for

struct L2Row {
    float s;          // max |v| of the row
    float inv;        // (L/2) / s, or 0 for an all-zero row
    float nrm;        // the Euclidean norm that is sent
    float unit;       // decode scale nrm / ||y||
    // speculation: the band the NEXT form pass assumes for s (s_hi = 0: none), as the two values of inv
    float s_lo, s_hi, inv_lo_s, inv_hi_s;   // inv_lo_s = (L/2)/s_lo (the larger one), inv_hi_s = (L/2)/s_hi
    float s_prev;     // s of the step before (0: none)
    float drift;      // recent relative movement of s from step to step (decaying maximum)
    uint32_t mode;    // this step: 1 = the codes `form` wrote stand (once the undecided ones are settled), 0 = exact second pass
    uint32_t overflowed;   // this step: a chunk had more undecided elements than its slot holds
    uint32_t streak;  // consecutive speculating steps that overflowed
    uint32_t wait;    // steps to sit out before the next guess (backs off when the slots keep overflowing)
};

struct L2Scratch {
    L2Row* rows;                  // n
    float* cmax;                  // n x nchunks: max |v| of the chunk
    double* csq;                  // n x nchunks: tree sum of v^2 over the chunk
    uint32_t* csy2;               // n x nchunks: sum of y^2 over the chunk (< 2^32: 4096 * 255^2)
    uint32_t* pending;            // 1: the last step's tail has not been applied to x and delta yet
    uint32_t* ucount;             // n x nchunks: undecided elements `form` slotted for the chunk
    uint2* uslot;                 // n x nchunks x LQ_UCAP: (column offset in the chunk | placeholder code << 16, bits of v)
    uint32_t* row_flags;          // n: bit 0 = a slot of the row overflowed in this step's form pass
    uint32_t nchunks;
};

// Code of one element for a given inv = (L/2)/s: nearest level, ties to even; NaN goes to level 0.
template <int BITS>
__device__ __forceinline__ int code_of(float v, float inv) {
    constexpr int L = (1 << BITS) - 1;
    float t = fmaf(v, inv, 0.5f * (float)L);
    t = (t > 0.f) ? t : 0.f;
    t = (t < (float)L) ? t : (float)L;
    return (int)rintf(t);
}

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
__device__ __forceinline__ void apply_tail4(const L2Args& a, const L2Scratch& s, const uint8_t* msg, int row, uint64_t col,
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
        const uint32_t codes = load_codes4<BITS>(msg + (uint64_t)nb * a.msg_row_bytes, col);
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

// Which of the two message buffers the last completed step wrote (cell 4 of the step cells).
__device__ __forceinline__ uint32_t last_half(const L2Args& a) { return (uint32_t)(a.t_ptr[4] & 1ull); }

// First pass of a step: the previous step's tail (if pending), then line 5, and -- when the row has a
// guess of its range -- the codes that do not depend on where in the guessed band the range falls.
template <int BITS>
__global__ void __launch_bounds__(LQ_THREADS) l2q_form(L2Args a, L2Scratch s) {
    constexpr int L = (1 << BITS) - 1;
    __shared__ double sweep_sq[LQ_ITERS * (LQ_THREADS / 64)];
    __shared__ float wave_max[LQ_THREADS / 64];
    __shared__ uint32_t wave_sy2[LQ_THREADS / 64];
    __shared__ uint32_t slot_fill;
    const int row = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t col0 = (uint64_t)blockIdx.x * LQ_CHUNK;
    const bool tail = *s.pending != 0u;
    const uint32_t prev = last_half(a);
    const uint8_t* msg_prev = a.msg + (uint64_t)prev * a.msg_half;          // the codes the tail decodes
    uint8_t* mrow = a.msg + (uint64_t)(prev ^ 1u) * a.msg_half + (uint64_t)row * a.msg_row_bytes;   // this step's message
    const uint64_t code_bytes = a.msg_row_bytes - 4;      // whole 32-bit words
    const L2Row guess = s.rows[row];
    const bool spec = guess.s_hi > 0.f;                   // uniform over the workgroup
    const size_t chunk = (size_t)row * s.nchunks + blockIdx.x;
    uint2* slot = s.uslot + chunk * LQ_UCAP;
    if (threadIdx.x == 0) slot_fill = 0u;
    __syncthreads();
    float* xr = a.x + (uint64_t)row * a.ld;
    float* dr = a.delta + (uint64_t)row * a.ld;
    const float* gr = a.g + (uint64_t)row * a.g_ld;
    float vmax = 0.f;
    uint32_t sy2 = 0;
    // all twelve 16-byte loads of the lane go out before the first store: x and delta are updated in place, so the
    // compiler must otherwise keep every later load behind the stores of the iteration before
    float4 xs[LQ_ITERS], ds[LQ_ITERS], gs[LQ_ITERS];
#pragma unroll
    for (int it = 0; it < LQ_ITERS; ++it) {
        const uint64_t col = col0 + (uint64_t)it * (4 * LQ_THREADS) + 4u * threadIdx.x;   // < ld: ld is a multiple of the chunk
        xs[it] = ld4_stream(xr + col);
        ds[it] = ld4_stream(dr + col);
        gs[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (col < a.N) gs[it] = ld4_stream(gr + col);     // g_ld >= N and a multiple of 4: the float4 is inside the row
    }
#pragma unroll
    for (int it = 0; it < LQ_ITERS; ++it) {
        const uint32_t off = (uint32_t)it * (4 * LQ_THREADS) + 4u * threadIdx.x;          // column inside the chunk
        const uint64_t col = col0 + off;
        float4 x4 = xs[it], d4 = ds[it], g4 = gs[it];
        if (col < a.N) {
            if (col + 3 >= a.N) {                         // whatever lies behind column N-1 is not a gradient
                if (col + 1 >= a.N) g4.y = 0.f;
                if (col + 2 >= a.N) g4.z = 0.f;
                g4.w = 0.f;
            }
            if (tail) apply_tail4<BITS>(a, s, msg_prev, row, col, x4, d4);
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
        const uint64_t byte = col * BITS / 8;
        if (spec && byte < code_bytes) {
            const float* vp = reinterpret_cast<const float*>(&v);
            uint32_t packed = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (col + c < a.N) {                      // padding codes are 0 and do not count
                    const int qa = code_of<BITS>(vp[c], guess.inv_lo_s);
                    const int qb = code_of<BITS>(vp[c], guess.inv_hi_s);
                    if (qa != qb) {                       // undecided until s is known: slot it, qb stands in
                        const uint32_t k = atomicAdd(&slot_fill, 1u);
                        if (k < LQ_UCAP) slot[k] = make_uint2((off + (uint32_t)c) | ((uint32_t)qb << 16), __float_as_uint(vp[c]));
                    }
                    const int y = 2 * qb - L;
                    sy2 += (uint32_t)(y * y);
                    packed |= (uint32_t)qb << (BITS * c);
                }
            }
            if constexpr (BITS == 2) mrow[4 + byte] = (uint8_t)packed;
            else if constexpr (BITS == 4) *reinterpret_cast<uint16_t*>(mrow + 4 + byte) = (uint16_t)packed;
            else *reinterpret_cast<uint32_t*>(mrow + 4 + byte) = packed;
        }
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { vmax = fmaxf(vmax, __shfl_xor(vmax, o)); sy2 += __shfl_xor(sy2, o); }
    if (lane == 0) { wave_max[wave] = vmax; wave_sy2[wave] = sy2; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) t[k] = sweep_sq[k];
#pragma unroll
        for (int len = 16; len > 1; len >>= 1)
#pragma unroll
            for (int p = 0; p < len / 2; ++p) t[p] = t[2 * p] + t[2 * p + 1];
        s.csq[chunk] = t[0];
        s.cmax[chunk] = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
        if (spec) {
            const uint32_t fill = slot_fill;
            s.csy2[chunk] = wave_sy2[0] + wave_sy2[1] + wave_sy2[2] + wave_sy2[3];
            s.ucount[chunk] = fill < LQ_UCAP ? fill : LQ_UCAP;
            if (fill > LQ_UCAP) atomicOr(&s.row_flags[row], 1u);
        }
    }
}
static_assert(LQ_ITERS * (LQ_THREADS / 64) == 16, "the chunk tree below is written for 16 sweeps");
static_assert(LQ_CHUNK <= 65536, "a slot entry keeps the column offset inside the chunk in 16 bits");

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
        // did the form pass speculate for this row, and does its band hold the range?  (division is monotone,
        // so s_lo <= s <= s_hi puts inv between the two values the codes were computed for)
        r.overflowed = s.row_flags[row] & 1u;
        s.row_flags[row] = 0u;
        r.mode = (r.s_hi > 0.f && m >= r.s_lo && m <= r.s_hi && !r.overflowed) ? 1u : 0u;
        s.rows[row] = r;
    }
}
static_assert(LQ_ROW_THREADS / 64 == 16, "the wave tree above is written for 16 waves");

// Second pass, one workgroup per chunk.  Rows whose speculative codes stand: the chunk's undecided elements get
// their exact code now that s is known (one slot entry per thread: an xor on the element's bits of the message
// word, a correction of the chunk's sum of y^2).  Other rows: the codes of v (which `form` left in delta) and the
// sum of y^2 per chunk, from scratch.
static_assert(LQ_UCAP <= LQ_THREADS, "one slot entry per thread");
template <int BITS>
__global__ void __launch_bounds__(LQ_THREADS) l2q_quantize(L2Args a, L2Scratch s) {
    constexpr int L = (1 << BITS) - 1;
    __shared__ uint32_t wave_sy2[LQ_THREADS / 64];
    const int row = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t col0 = (uint64_t)blockIdx.x * LQ_CHUNK;
    if (s.rows[row].mode) {                                // uniform over the workgroup
        const size_t chunk = (size_t)row * s.nchunks + blockIdx.x;
        if (threadIdx.x >= s.ucount[chunk]) return;        // <= LQ_UCAP entries
        const uint2 e = s.uslot[chunk * LQ_UCAP + threadIdx.x];
        const int qb = (int)(e.x >> 16);
        const int q = code_of<BITS>(__uint_as_float(e.y), s.rows[row].inv);
        if (q != qb) {
            uint32_t* words = reinterpret_cast<uint32_t*>(a.msg + (uint64_t)(last_half(a) ^ 1u) * a.msg_half + (uint64_t)row * a.msg_row_bytes + 4);
            const uint64_t bit = (col0 + (e.x & 0xFFFFu)) * BITS;                         // position in the row's code stream
            atomicXor(&words[bit >> 5], (uint32_t)(q ^ qb) << (bit & 31u));                // several threads may share a word
            const int y = 2 * q - L, yb = 2 * qb - L;
            atomicAdd(&s.csy2[chunk], (uint32_t)(y * y) - (uint32_t)(yb * yb));            // modulo 2^32: the sum itself fits
        }
        return;
    }
    const float inv = s.rows[row].inv;
    const bool zero_row = !(s.rows[row].s > 0.f);
    const float* dr = a.delta + (uint64_t)row * a.ld;
    uint8_t* mrow = a.msg + (uint64_t)(last_half(a) ^ 1u) * a.msg_half + (uint64_t)row * a.msg_row_bytes;
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
                const int q = zero_row ? 0 : code_of<BITS>(vp[c], inv);
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

// Per row: sum y^2 (an integer, any order), the decode scale, the message header, and the band the next form
// pass may assume for s.  The last row to finish closes the step: its tail is now pending, the message buffers
// change roles, the step counter moves.
__global__ void __launch_bounds__(LQ_ROW_THREADS) l2q_row_unit(L2Args a, L2Scratch s, float half_levels) {
    __shared__ unsigned long long wsum[LQ_ROW_THREADS / 64];
    const int row = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t* sy = s.csy2 + (size_t)row * s.nchunks;
    const uint32_t written = last_half(a) ^ 1u;           // read before this workgroup counts itself finished
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
        // The band for the next step: centred on this step's s, as wide as s has been moving lately.  A band
        // too wide to be worth it (many undecided elements), an all-zero row, or slots that keep overflowing
        // (many levels: the boundaries are dense) leave the next step to the exact second pass.
        const bool tried = r.s_hi > 0.f;
        if (tried && r.overflowed) { r.streak = r.streak < 6u ? r.streak + 1u : 6u; r.wait = 1u << r.streak; }
        else if (r.mode) r.streak = 0u;
        const float rel = (r.s_prev > 0.f) ? fabsf(r.s - r.s_prev) / r.s_prev : 0.2f;      // first step: wait for a second look
        r.drift = fmaxf(rel, 0.7f * r.drift);
        r.s_prev = r.s;
        const float h = 1.5f * r.drift + 0.02f;
        r.s_lo = r.s_hi = r.inv_lo_s = r.inv_hi_s = 0.f;
        if (r.wait > 0u) {
            r.wait -= 1u;
        } else if (r.s > 0.f && h <= 0.3f) {
            r.s_lo = r.s * (1.f - h);
            r.s_hi = r.s * (1.f + h);
            r.inv_lo_s = half_levels / r.s_lo;
            r.inv_hi_s = half_levels / r.s_hi;
            if (!(r.s_lo > 0.f) || !(r.inv_lo_s < 3.0e38f)) r.s_lo = r.s_hi = r.inv_lo_s = r.inv_hi_s = 0.f;   // denormal ranges: no guess
        }
        s.rows[row] = r;
        *reinterpret_cast<float*>(a.msg + (uint64_t)written * a.msg_half + (uint64_t)row * a.msg_row_bytes) = r.nrm;
        // every workgroup has read cell 4 by the time it counts itself; the last one flips it
        unsigned long long* done = a.t_ptr + 5;
        if (__hip_atomic_fetch_add(done, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned long long)gridDim.x - 1ull) {
            __hip_atomic_store(done, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(a.t_ptr + 4, (unsigned long long)written, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
    const uint8_t* msg_last = a.msg + (uint64_t)last_half(a) * a.msg_half;
    float* xr = a.x + (uint64_t)row * a.ld;
    float* dr = a.delta + (uint64_t)row * a.ld;
#pragma unroll
    for (int it = 0; it < LQ_ITERS; ++it) {
        const uint64_t col = col0 + (uint64_t)it * (4 * LQ_THREADS) + 4u * threadIdx.x;
        if (col >= a.N) continue;
        float4 x4 = ld4_stream(xr + col), d4 = ld4_stream(dr + col);
        apply_tail4<BITS>(a, s, msg_last, row, col, x4, d4);
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
    void* ptrs[] = {s.rows, s.cmax, s.csq, s.csy2, s.pending, s.ucount, s.uslot, s.row_flags};
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
              hipMalloc(&s.pending, sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.ucount, n * nc * sizeof(uint32_t)) == hipSuccess &&
              hipMalloc(&s.uslot, n * nc * LQ_UCAP * sizeof(uint2)) == hipSuccess &&
              hipMalloc(&s.row_flags, n * sizeof(uint32_t)) == hipSuccess;
    // rows start with no guess (s_hi = 0): the first two steps are exact (the first has no s_prev and counts as a
    // movement of 20 %, too wide a band), speculation starts with the third if s moved little between them
    ok = ok && hipMemset(s.rows, 0, n * sizeof(L2Row)) == hipSuccess &&
         hipMemset(s.ucount, 0, n * nc * sizeof(uint32_t)) == hipSuccess &&
         hipMemset(s.row_flags, 0, n * sizeof(uint32_t)) == hipSuccess &&
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
    hipLaunchKernelGGL(l2q_row_unit, rows, rblock, 0, stream, a, s, hl);
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

ds_status l2q_speculated_rows(L2State* st, hipStream_t stream, uint32_t* count) {
    *count = 0;
    if (hipStreamSynchronize(stream) != hipSuccess) return DS_EHIP;
    std::vector<L2Row> rows((size_t)st->n);
    if (hipMemcpy(rows.data(), st->s.rows, rows.size() * sizeof(L2Row), hipMemcpyDeviceToHost) != hipSuccess) return DS_EHIP;
    for (const L2Row& r : rows) *count += r.mode ? 1u : 0u;
    return DS_OK;
}

}  // namespace dsq

// DeepSqueeze reference step on the CPU -- TEST INFRASTRUCTURE, not product code.
//
// A plain, slow, one-loop-per-sentence implementation of one iteration of
// DeepSqueeze (Tang et al., arXiv:1907.07346, Algorithm 1) for n simulated
// workers.  It exists only so that tests, the smoke check and the benchmark's
// CPU-baseline leg have something independent to compare the GPU library with.
// It shares no code, header, table or constant generator with the HIP path.
//
// State is held as in the paper's matrix notation (Section "Mathematical
// formulation"), transposed: row i of X, G, Delta is worker i's vector of N
// parameters.  One call performs, for every worker i,
//
//   line 5   v_i      = x_i - gamma * g_i + delta_i
//   line 6   C[v_i]   = compress(v_i);   delta_i = v_i - C[v_i]
//   line 7-8 the packed message of C[v_i] is "sent" (written to `msg`)
//   line 9   x_i      = x_i - gamma * g_i + eta * sum_{j in N(i)} (W_ij - I_ij) C[v_j]
//
// with i in N(i) (the note in line 8), so the worker's own term enters through
// its *compressed* value with coefficient W_ii - 1.
//
// The paper leaves C_omega generic (Assumption 1.6 only asks for a bounded
// signal-to-noise factor).  The seven operators implemented here, and the exact
// floating-point evaluation order used for `real = float`, are this
// repository's readings; every one is stated next to the code that does it.
//
// After the DeepSqueeze step come the two compressed decentralized methods the
// paper compares it with (DCD-PSGD, CHOCO-SGD), as this repository reads them
// from the paper's unrolled forms; see the note above step_dcd.
//
// Every function below is pinned by tests/test_oracle_pins.py against what the
// paper and plain mathematics fix.  What nothing available can fix is the CHOICE
// of the operators' grids, rounding and tie rules where the paper is silent
// (against the authors' unpublished code that choice is "parity unpinned").
//
// Everything is templated on `real`: double is used to check the algebraic
// identities the paper states, float (same expression order as the GPU
// kernels, contraction off, explicit fma) is used for bit-level parity.
//
// Build: g++ -O2 -ffp-contract=off -shared -fPIC ds_oracle.cpp -o libds_oracle.so
// The loops over workers carry `#pragma omp parallel for`: without -fopenmp (the build every test uses) the
// pragmas are ignored and the code is the sequential program it reads as; with -fopenmp (a second library,
// built only for the benchmark's all-cores baseline) workers are spread over the host's cores.  No iteration
// of those loops reads what another one writes, so both builds give the same bits.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
// as 1, 2, 3", SC'11).  Counter-based: out = f(counter, key), no state.
// ---------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;   // round multipliers
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;   // key schedule (Weyl) increments
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = M0 * c0;                     // 32x32 -> 64
        const uint64_t p1 = M1 * c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n1 = lo1;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        const uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The random word that decides the stochastic rounding of element j of worker
// i at iteration t.  Reading (the paper draws no random numbers itself):
// counter = (floor(j/4), i, t mod 2^32, 'QUNT'), key = (seed low, seed high),
// element j takes output word j mod 4.
const uint32_t kQuantTag = 0x51554E54u;

uint32_t rounding_word(uint64_t seed, uint64_t t, uint32_t i, uint64_t j) {
    const uint32_t ctr[4] = {(uint32_t)(j / 4), i, (uint32_t)t, kQuantTag};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    philox4x32_10(ctr, key, out);
    return out[j % 4];
}

// The random word that decides whether element j of worker i is kept by the random sparsifier at
// iteration t: the same addressing as the rounding words, in a stream of its own ('SPAR').
const uint32_t kSparseTag = 0x53504152u;

uint32_t keep_word(uint64_t seed, uint64_t t, uint32_t i, uint64_t j) {
    const uint32_t ctr[4] = {(uint32_t)(j / 4), i, (uint32_t)t, kSparseTag};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    philox4x32_10(ctr, key, out);
    return out[j % 4];
}

// ... and by the magnitude-proportional sparsifier (operator 6), in a third stream ('GSPR').
const uint32_t kGsparTag = 0x47535052u;

uint32_t gspar_word(uint64_t seed, uint64_t t, uint32_t i, uint64_t j) {
    const uint32_t ctr[4] = {(uint32_t)(j / 4), i, (uint32_t)t, kGsparTag};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    philox4x32_10(ctr, key, out);
    return out[j % 4];
}

enum Kind { IDENTITY = 0, QUANT_MAXABS = 1, SIGN_MEANABS = 2, TOPK = 3, QUANT_L2NORM = 4, RAND_SPARSE = 5, GSPAR = 6 };

template <typename real> real fma_(real a, real b, real c);
template <> float  fma_<float>(float a, float b, float c)    { return std::fmaf(a, b, c); }
template <> double fma_<double>(double a, double b, double c) { return std::fma(a, b, c); }

template <typename real> struct Msg {           // append-only byte sink of one worker, may be disabled
    std::vector<uint8_t>* bytes;
    void put(const void* p, size_t nbytes) {
        if (!bytes) return;
        const uint8_t* b = static_cast<const uint8_t*>(p);
        bytes->insert(bytes->end(), b, b + nbytes);
    }
    void put_u32(uint32_t w) { put(&w, 4); }
    void put_f32(real s)     { float f = (float)s; put(&f, 4); }
};

// ---------------------------------------------------------------------------
// C_omega, operator 1: stochastic b-bit uniform quantisation of one block with
// a max-abs scale.  Grid: L+1 = 2^b equally spaced levels from -s to +s (no
// zero level); v is mapped to t = (v/s + 1) * L/2 in [0, L], rounded down or up
// at random so that E[q] = t, and decoded as (2q - L) * (s/L).
// Message: [f32 s][ceil(m*b/32) u32 words], code of element e in bits
// [b*(e mod 32/b), +b) of word floor(e*b/32).
// ---------------------------------------------------------------------------
template <typename real>
void compress_block_quant(const real* v, real* cv, uint64_t m, int bits,
                          uint64_t seed, uint64_t t, uint32_t i, uint64_t j0, Msg<real>& msg) {
    const int L = (1 << bits) - 1;
    real s = 0;
    for (uint64_t e = 0; e < m; ++e) s = std::max(s, (real)std::fabs(v[e]));
    const uint64_t nwords = (m * bits + 31) / 32;
    std::vector<uint32_t> words(nwords, 0u);
    const real hl = (real)0.5 * (real)L;
    const real unit = s / (real)L;
    const real inv = (s > 0) ? hl / s : (real)0;
    for (uint64_t e = 0; e < m; ++e) {
        int q = 0;
        if (s > 0) {
            real tt = fma_<real>(v[e], inv, hl);
            tt = (tt > (real)0) ? tt : (real)0;          // also sends NaN to 0
            tt = (tt < (real)L) ? tt : (real)L;
            const real q0 = std::floor(tt);
            const real fr = tt - q0;                     // exact
            const real u = (real)(rounding_word(seed, t, i, j0 + e) >> 8) * (real)(1.0 / 16777216.0);
            q = (int)q0 + ((u < fr) ? 1 : 0);
            q = std::min(q, L);
        }
        cv[e] = (real)(2 * q - L) * unit;                // all-zero block: -L * 0 = -0
        const uint64_t bitpos = e * (uint64_t)bits;
        words[bitpos / 32] |= (uint32_t)q << (bitpos % 32);
    }
    msg.put_f32(s);
    for (uint64_t w = 0; w < nwords; ++w) msg.put_u32(words[w]);
}

// ---------------------------------------------------------------------------
// C_omega, operator 2: one sign bit per element and the block's mean absolute
// value as scale (the 1-bit SGD family the paper's related-work section names).
// The mean is sum/m with m the number of real elements; the sum is taken by a
// balanced binary tree over the block padded with +0 to `block` entries
// (adjacent pairs first), so that the float result does not depend on who
// computes it.  A set bit means "negative" (the IEEE sign bit, so -0 counts as
// negative).  Message: [f32 s][ceil(m/32) u32 words].
// ---------------------------------------------------------------------------
template <typename real>
void compress_block_sign(const real* v, real* cv, uint64_t m, uint64_t block, Msg<real>& msg) {
    std::vector<real> a(block, (real)0);
    for (uint64_t e = 0; e < m; ++e) a[e] = std::fabs(v[e]);
    for (uint64_t len = block; len > 1; len /= 2)
        for (uint64_t p = 0; p < len / 2; ++p) a[p] = a[2 * p] + a[2 * p + 1];
    const real s = a[0] / (real)m;
    const uint64_t nwords = (m + 31) / 32;
    std::vector<uint32_t> words(nwords, 0u);
    for (uint64_t e = 0; e < m; ++e) {
        const bool neg = std::signbit(v[e]);
        cv[e] = neg ? -s : s;
        if (neg) words[e / 32] |= 1u << (e % 32);
    }
    msg.put_f32(s);
    for (uint64_t w = 0; w < nwords; ++w) msg.put_u32(words[w]);
}

// ---------------------------------------------------------------------------
// C_omega, operator 3: top-k by magnitude over the whole vector of one worker.
// Order: larger |v| first, equal |v| -> lower index first; the first k are
// kept with their exact value, all others become +0.
// Message: k pairs (u32 index, f32 value), ascending index.
// ---------------------------------------------------------------------------
template <typename real>
void compress_row_topk(const real* v, real* cv, uint64_t N, uint64_t k, Msg<real>& msg) {
    std::vector<uint64_t> order(N);
    for (uint64_t j = 0; j < N; ++j) order[j] = j;
    auto before = [v](uint64_t a, uint64_t b) {
        const real fa = std::fabs(v[a]), fb = std::fabs(v[b]);
        if (fa != fb) return fa > fb;
        return a < b;
    };
    if (k < N) std::nth_element(order.begin(), order.begin() + k, order.end(), before);
    std::vector<uint8_t> keep(N, 0);
    for (uint64_t r = 0; r < k && r < N; ++r) keep[order[r]] = 1;
    for (uint64_t j = 0; j < N; ++j) {
        cv[j] = keep[j] ? v[j] : (real)0;
        if (keep[j]) { msg.put_u32((uint32_t)j); msg.put_f32(v[j]); }
    }
}

// ---------------------------------------------------------------------------
// Sum of squares of a vector by a balanced binary tree in double precision:
// the vector is padded with zeros to a power of two, adjacent pairs are added
// first, then adjacent results, and so on.  (A pinned order, so that the
// result is one well-defined number; the square of a float is exact in double.)
// ---------------------------------------------------------------------------
template <typename real>
double sum_squares_tree(const real* v, uint64_t N) {
    uint64_t P = 1;
    while (P < N) P *= 2;
    std::vector<double> a(P, 0.0);
    for (uint64_t j = 0; j < N; ++j) a[j] = (double)v[j] * (double)v[j];
    for (uint64_t len = P; len > 1; len /= 2)
        for (uint64_t p = 0; p < len / 2; ++p) a[p] = a[2 * p] + a[2 * p + 1];
    return a[0];
}

// ---------------------------------------------------------------------------
// C_omega, operator 4: the compression of the paper's experiments (Section
// "Experimental Setup", paragraph "Compression"): every element of a worker's
// tensor becomes a b-bit code, and one number, the Euclidean norm of the
// original tensor, travels with the codes; the receiver scales the decoded
// tensor so that its Euclidean norm equals that number.
// The paper gives neither grid nor rounding.  Reading: the grid is that of
// operator 1 with the whole vector as one block (2^b equally spaced levels
// from -s to +s, s = max|v|, which is not sent); v is rounded to the NEAREST
// level (ties: to the even code), because the paragraph names no randomness
// and Assumption 1.6 needs a signal-to-noise factor alpha < 1, which unbiased
// random rounding to 4 levels does not give.  The code q stands for the odd
// integer y = 2q - L, and the receiver returns
//     C[v] = y * (nrm / ||y||_2),   nrm = ||v||_2 as sent (fp32),
// with ||y||_2^2 = sum y_j^2 an exact integer (>= N, so never zero).
// nrm^2 is the tree sum above; the scalar arithmetic is done in double and
// rounded once:  nrm = (real) sqrt(S2),  unit = (real)(nrm / sqrt(sum y^2)).
// Message: [f32 nrm][ceil(N*b/32) u32 words], codes packed as in operator 1.
// ---------------------------------------------------------------------------
template <typename real>
void compress_row_quant_l2norm(const real* v, real* cv, uint64_t N, int bits, Msg<real>& msg) {
    const int L = (1 << bits) - 1;
    real s = 0;
    for (uint64_t j = 0; j < N; ++j) s = std::max(s, (real)std::fabs(v[j]));
    const real nrm = (real)std::sqrt(sum_squares_tree<real>(v, N));
    const uint64_t nwords = (N * bits + 31) / 32;
    std::vector<uint32_t> words(nwords, 0u);
    std::vector<int> y(N);
    const real hl = (real)0.5 * (real)L;
    const real inv = (s > 0) ? hl / s : (real)0;
    uint64_t sum_y2 = 0;
    for (uint64_t j = 0; j < N; ++j) {
        int q = 0;
        if (s > 0) {
            real tt = fma_<real>(v[j], inv, hl);         // (v/s + 1) * L/2 in [0, L]
            tt = (tt > (real)0) ? tt : (real)0;          // also sends NaN to 0
            tt = (tt < (real)L) ? tt : (real)L;
            q = (int)std::nearbyint(tt);                 // round to nearest, ties to even (default rounding mode)
        }
        y[j] = 2 * q - L;
        sum_y2 += (uint64_t)(y[j] * y[j]);
        const uint64_t bitpos = j * (uint64_t)bits;
        words[bitpos / 32] |= (uint32_t)q << (bitpos % 32);
    }
    const real unit = (real)((double)nrm / std::sqrt((double)sum_y2));
    for (uint64_t j = 0; j < N; ++j) cv[j] = (real)y[j] * unit;
    msg.put_f32(nrm);
    for (uint64_t w = 0; w < nwords; ++w) msg.put_u32(words[w]);
}

// ---------------------------------------------------------------------------
// C_omega, operator 5: random sparsification (named with GSpar, top-k and
// random quantisation among the operators that satisfy Assumption 1.6): every
// element is kept with the same probability p, independently, and the others
// become +0.  Reading: no rescaling by 1/p -- the unbiased variant has
// E|C[v] - v|^2 = (1/p - 1)|v|^2, outside Assumption 1.6 for p < 1/2, whereas
// the plain mask gives exactly alpha^2 = 1 - p.  p is given through k, the
// expected number of kept elements per worker: element j is kept iff the top
// 24 bits of its random word are below T = floor(k 2^24 / N) (an integer test,
// so every implementation takes the same decision); k = N keeps everything.
// The receiver regenerates the mask from the shared seed, so only the kept
// values travel.  Message per worker: [u32 count][count f32 values, ascending
// index], zero-padded to a fixed capacity of `cap` values; a worker that keeps
// more than `cap` values (8 standard deviations above k) is reported as an error.
// ---------------------------------------------------------------------------
uint64_t rand_sparse_capacity(uint64_t N, uint64_t k) {
    uint64_t root = 0;
    while (root * root < k) ++root;                       // ceil(sqrt(k))
    const uint64_t cap = k + 8 * root + 64;
    return cap < N ? cap : N;
}

template <typename real>
bool compress_row_rand_sparse(const real* v, real* cv, uint64_t N, uint64_t k,
                              uint64_t seed, uint64_t t, uint32_t i, Msg<real>& msg) {
    const uint64_t T = (k << 24) / N;                     // k <= N < 2^32: no overflow
    const uint64_t cap = rand_sparse_capacity(N, k);
    std::vector<real> kept;
    for (uint64_t j = 0; j < N; ++j) {
        const bool keep = (uint64_t)(keep_word(seed, t, i, j) >> 8) < T;
        cv[j] = keep ? v[j] : (real)0;
        if (keep) kept.push_back(v[j]);
    }
    const bool overflow = kept.size() > cap;
    msg.put_u32((uint32_t)(overflow ? cap : kept.size()));
    for (uint64_t r = 0; r < cap; ++r) msg.put_f32(r < kept.size() ? kept[r] : (real)0);
    return !overflow;
}

// ---------------------------------------------------------------------------
// C_omega, operator 6: GSpar, named next to random sparsification, top-k and
// random quantisation as satisfying Assumption 1.6 (section "Theoretical
// analysis", the paragraph after Theorem 1).  The paper says no more about it.
// Reading: the magnitude-proportional sparsifier that name stands for --
// element j is kept with probability p_j = min(1, lambda |v_j|), independently,
// with lambda chosen so that the expected number of kept elements is k when no
// probability is cut off at 1:  lambda = k / sum_j |v_j|  (one shot: where some
// p_j are cut off the expected count is below k; no second round redistributes
// it).  As for operator 5 the kept values are NOT divided by p_j: the unbiased
// variant has E||C[v] - v||^2 = sum v_j^2 (1/p_j - 1), unbounded against
// ||v||^2, while the plain mask gives sum v_j^2 (1 - p_j) < ||v||^2, inside
// the assumption.  sum |v| is taken in double by the balanced adjacent-pairs
// tree over the zero-padded vector (|v_j| is exact in double), lambda and
// p_j = lambda * |v_j| are single roundings in `real`; element j is kept iff
// u_j < p_j with u_j = (word >> 8) / 2^24 from the stream 'GSPR' (so p_j >= 1
// always keeps).  The mask depends on v, so the receiver cannot rebuild it and
// the message carries the columns:
//   [u32 count][u32 0][count (u32 column, f32 value) pairs, ascending column],
// zero-padded to the capacity of operator 5 (pairs instead of values).
// Returns false if more elements were kept than the message has room for.
// ---------------------------------------------------------------------------
template <typename real>
double sum_abs_tree(const real* v, uint64_t N) {
    uint64_t P = 1;
    while (P < N) P *= 2;
    std::vector<double> a(P, 0.0);
    for (uint64_t j = 0; j < N; ++j) a[j] = std::fabs((double)v[j]);
    for (uint64_t len = P; len > 1; len /= 2)
        for (uint64_t p = 0; p < len / 2; ++p) a[p] = a[2 * p] + a[2 * p + 1];
    return a[0];
}

template <typename real>
bool compress_row_gspar(const real* v, real* cv, uint64_t N, uint64_t k,
                        uint64_t seed, uint64_t t, uint32_t i, Msg<real>& msg) {
    const double total = sum_abs_tree<real>(v, N);
    const real lambda = (total > 0) ? (real)((double)k / total) : (real)0;
    const uint64_t cap = rand_sparse_capacity(N, k);
    std::vector<uint64_t> cols;
    for (uint64_t j = 0; j < N; ++j) {
        const real p = lambda * (real)std::fabs(v[j]);
        const real u = (real)(gspar_word(seed, t, i, j) >> 8) * (real)(1.0 / 16777216.0);
        const bool keep = u < p;
        cv[j] = keep ? v[j] : (real)0;
        if (keep) cols.push_back(j);
    }
    const bool overflow = cols.size() > cap;
    msg.put_u32((uint32_t)(overflow ? cap : cols.size()));
    msg.put_u32(0u);
    for (uint64_t r = 0; r < cap; ++r) {
        if (r < cols.size()) { msg.put_u32((uint32_t)cols[r]); msg.put_f32(v[cols[r]]); }
        else { msg.put_u32(0u); msg.put_u32(0u); }
    }
    return !overflow;
}

// Argument and CSR sanity shared by the update rules below: 0 if fine.
template <typename real>
int check_arguments(int n, uint64_t N, const int32_t* rowptr, const int32_t* col, const real* wval,
                    int kind, int bits, uint64_t block, uint64_t k, const real* x, const real* state2, const real* g) {
    if (n < 1 || N < 1 || !rowptr || !col || !wval || !x || !state2 || !g) return 1;
    if ((kind == QUANT_MAXABS || kind == SIGN_MEANABS) && (block < 1 || (block & (block - 1)))) return 1;
    if ((kind == QUANT_MAXABS || kind == QUANT_L2NORM) && (bits < 1 || bits > 8 || 32 % bits)) return 1;
    if ((kind == TOPK || kind == RAND_SPARSE || kind == GSPAR) && (k < 1 || k > N)) return 1;
    if ((kind == RAND_SPARSE || kind == GSPAR) && N > 0xFFFFFFFFull) return 1;
    for (int i = 0; i < n; ++i) {                         // CSR sanity: sorted, has diagonal
        bool diag = false;
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            if (col[e] < 0 || col[e] >= n) return 1;
            if (e > rowptr[i] && col[e] <= col[e - 1]) return 1;
            diag |= (col[e] == i);
        }
        if (!diag) return 1;
    }
    return 0;
}

// C_omega applied to every worker's vector (rows of v -> rows of cv), and what each worker sends written to
// msg_buf in worker order.  Every worker appends to a sink of its own; the sinks are joined afterwards (so
// workers may be processed side by side).  Returns 0, 1 (unknown operator), 2 (msg_buf too small) or 3 (a
// random-sparsification message outgrew its capacity).
template <typename real>
int compress_workers(int n, uint64_t N, const real* v, real* cv, int kind, int bits, uint64_t block, uint64_t k,
                     uint64_t seed, uint64_t t, uint64_t col0, uint8_t* msg_buf, uint64_t msg_cap, uint64_t* msg_bytes) {
    bool sparse_overflow = false;
    std::vector<std::vector<uint8_t>> sent(msg_buf ? n : 0);
    bool bad_kind = false;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        const real* vi = &v[(uint64_t)i * N];
        real* ci = &cv[(uint64_t)i * N];
        if (msg_buf) sent[i].reserve(msg_cap / n + 16);
        Msg<real> msg{msg_buf ? &sent[i] : nullptr};
        if (kind == IDENTITY) {
            for (uint64_t j = 0; j < N; ++j) { ci[j] = vi[j]; msg.put_f32(vi[j]); }
        } else if (kind == QUANT_MAXABS || kind == SIGN_MEANABS) {
            for (uint64_t j0 = 0; j0 < N; j0 += block) {
                const uint64_t m = std::min<uint64_t>(block, N - j0);
                if (kind == QUANT_MAXABS)
                    compress_block_quant<real>(vi + j0, ci + j0, m, bits, seed, t, (uint32_t)i, col0 + j0, msg);
                else
                    compress_block_sign<real>(vi + j0, ci + j0, m, block, msg);
            }
        } else if (kind == TOPK) {
            compress_row_topk<real>(vi, ci, N, k, msg);
        } else if (kind == QUANT_L2NORM) {
            compress_row_quant_l2norm<real>(vi, ci, N, bits, msg);
        } else if (kind == RAND_SPARSE) {
            if (!compress_row_rand_sparse<real>(vi, ci, N, k, seed, t, (uint32_t)i, msg)) {
#pragma omp atomic write
                sparse_overflow = true;
            }
        } else if (kind == GSPAR) {
            if (!compress_row_gspar<real>(vi, ci, N, k, seed, t, (uint32_t)i, msg)) {
#pragma omp atomic write
                sparse_overflow = true;
            }
        } else {
#pragma omp atomic write
            bad_kind = true;
        }
    }
    if (bad_kind) return 1;
    uint64_t msg_used = 0;
    bool msg_overflow = false;
    for (int i = 0; msg_buf && i < n; ++i) {
        if (msg_used + sent[i].size() > msg_cap) { msg_overflow = true; break; }
        std::memcpy(msg_buf + msg_used, sent[i].data(), sent[i].size());
        msg_used += sent[i].size();
    }
    if (msg_bytes) *msg_bytes = msg_used;
    if (sparse_overflow) return 3;
    return msg_overflow ? 2 : 0;
}

// out_i = sum_{j in N(i)} (W_ij - I_ij) src_j for every worker: neighbours in ascending index order (own index
// included), accumulated by a chain of fused multiply-adds starting from zero.
template <typename real>
void mix_minus_identity(int n, uint64_t N, const int32_t* rowptr, const int32_t* col, const real* wval,
                        const real* src, real* out) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i)
        for (uint64_t j = 0; j < N; ++j) {
            real acc = 0;
            for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                const int nb = col[e];
                const real a = (nb == i) ? (wval[e] - (real)1) : wval[e];
                acc = fma_<real>(a, src[(uint64_t)nb * N + j], acc);
            }
            out[(uint64_t)i * N + j] = acc;
        }
}

// ---------------------------------------------------------------------------
// One iteration for all workers.  Dense n x N row-major arrays throughout.
// W comes as CSR (rowptr, col, val) *including* the diagonal entry of every
// row, columns ascending; the mixing coefficient of line 9 is
// a_ij = W_ij - I_ij, formed once in `real`.
// ---------------------------------------------------------------------------
template <typename real>
int step(int n, uint64_t N, const int32_t* rowptr, const int32_t* col, const real* wval,
         int kind, int bits, uint64_t block, uint64_t k,
         real gamma, real eta, uint64_t seed, uint64_t t,
         real* x, real* delta, const real* g,
         real* cv_out, uint8_t* msg_buf, uint64_t msg_cap, uint64_t* msg_bytes, uint64_t col0 = 0) {
    if (check_arguments<real>(n, N, rowptr, col, wval, kind, bits, block, k, x, delta, g)) return 1;

    const uint64_t total = (uint64_t)n * N;
    std::vector<real> xh(total), v(total), mixed(total), cv_local;
    real* cv = cv_out;
    if (!cv) { cv_local.resize(total); cv = cv_local.data(); }

    // Algorithm 1, line 5: the error-compensated variable, evaluated as
    // (x - gamma g) + delta with the product fused into the first sum.
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i)
        for (uint64_t j = 0; j < N; ++j) {
            const uint64_t p = (uint64_t)i * N + j;
            xh[p] = fma_<real>(-gamma, g[p], x[p]);
            v[p] = xh[p] + delta[p];
        }

    // Line 6, first half, and lines 7-8: compress, and write what is sent.
    const int rc = compress_workers<real>(n, N, v.data(), cv, kind, bits, block, k, seed, t, col0, msg_buf, msg_cap, msg_bytes);
    if (rc == 1) return 1;

    // Line 6, second half: what compression lost is carried to the next step.
#pragma omp parallel for schedule(static)
    for (uint64_t p = 0; p < total; ++p) delta[p] = v[p] - cv[p];

    // Line 9: gossip on the compressed values.
    mix_minus_identity<real>(n, N, rowptr, col, wval, cv, mixed.data());
#pragma omp parallel for schedule(static)
    for (uint64_t p = 0; p < total; ++p) x[p] = fma_<real>(eta, mixed[p], xh[p]);
    return rc;
}

// ---------------------------------------------------------------------------
// The two compressed decentralized methods the paper measures DeepSqueeze against (section "Why DeepSqueeze is
// better", the DCD-PSGD and CHOCO-SGD items; section "Related Work", "Compressed Communication Distributed
// Learning").  The paper gives no update rule for them, only unrolled forms of X_t and two statements: with no
// compression error every method is the paper's D-PSGD, X+ = (X - gamma G) W_eff; and the error of one step
// reaches X through a power of W_eff alone (DCD-PSGD), or through (W_eff - I) times such a power (CHOCO-SGD).
// The rules below are this repository's reading: the simplest per-worker rules with exactly those two
// properties, written in the notation of Algorithm 1 and with the same C_omega, message format and mixing
// coefficients W_ij - I_ij as the step above.  Their unrolled forms (derived by induction, pinned over six steps
// in tests/test_oracle_pins.py) differ from the printed ones in the exponent of W_eff, a stray factor eta and,
// for DCD-PSGD, the last term of the sum, the same kind of slip the printed DeepSqueeze form has.  Against
// the cited papers themselves they are "parity unpinned": neither is available here.
// ---------------------------------------------------------------------------

// DCD-PSGD ("use the difference of the model updates as the shared information"): every worker compresses
// the move the uncompressed method would make, and applies the compressed move; so does everyone who keeps
// a copy of its model, which is why the copies stay exact and X itself can stand for them.
//   xh_i = x_i - gamma g_i
//   z_i  = xh_i + eta sum_{j in N(i)} (W_ij - I_ij) xh_j - x_i        (the D-PSGD target minus the model)
//   x_i  = x_i + C[z_i];     the message is the packed C[z_i]
// Matrix form: X+ = (X - gamma G) W_eff - Delta_t, Delta_t = Z_t - C[Z_t].
// Unrolled, X_0 = 0:  X_t = -gamma sum_{s<t} G_s W_eff^{t-s} - sum_{s<t} Delta_s W_eff^{t-1-s}.
// No state besides x: `delta` is left untouched.
template <typename real>
int step_dcd(int n, uint64_t N, const int32_t* rowptr, const int32_t* col, const real* wval,
             int kind, int bits, uint64_t block, uint64_t k, real gamma, real eta, uint64_t seed, uint64_t t,
             real* x, real* delta_unused, const real* g, real* cv_out, uint8_t* msg_buf, uint64_t msg_cap, uint64_t* msg_bytes) {
    if (check_arguments<real>(n, N, rowptr, col, wval, kind, bits, block, k, x, delta_unused, g)) return 1;
    const uint64_t total = (uint64_t)n * N;
    std::vector<real> xh(total), mixed(total), z(total), cv_local;
    real* cv = cv_out;
    if (!cv) { cv_local.resize(total); cv = cv_local.data(); }
#pragma omp parallel for schedule(static)
    for (uint64_t p = 0; p < total; ++p) xh[p] = fma_<real>(-gamma, g[p], x[p]);
    mix_minus_identity<real>(n, N, rowptr, col, wval, xh.data(), mixed.data());
#pragma omp parallel for schedule(static)
    for (uint64_t p = 0; p < total; ++p) z[p] = fma_<real>(eta, mixed[p], xh[p]) - x[p];
    const int rc = compress_workers<real>(n, N, z.data(), cv, kind, bits, block, k, seed, t, 0, msg_buf, msg_cap, msg_bytes);
    if (rc == 1) return 1;
#pragma omp parallel for schedule(static)
    for (uint64_t p = 0; p < total; ++p) x[p] = x[p] + cv[p];
    return rc;
}

// CHOCO-SGD ("sharing the difference of the model difference"): every worker i has a public copy xhat_i of its
// model, known to its neighbours, which moves only by compressed differences; the gossip step runs on the copies.
//   xh_i   = x_i - gamma g_i
//   q_i    = C[xh_i - xhat_i];       the message is the packed q_i
//   xhat_i = xhat_i + q_i
//   x_i    = xh_i + eta sum_{j in N(i)} (W_ij - I_ij) xhat_j        (the copies after their update)
// Matrix form: X+ = (X - gamma G) W_eff - Delta_t (W_eff - I), Delta_t = (X - gamma G) - Xhat+  (what the copy
// still misses; equal to the compression error of this step's difference).
// Unrolled, X_0 = Xhat_0 = 0:  X_t = -gamma sum_{s<t} G_s W_eff^{t-s} - sum_{s<t} Delta_s (W_eff - I) W_eff^{t-1-s}.
// `xhat` takes the place of delta in the state.
template <typename real>
int step_choco(int n, uint64_t N, const int32_t* rowptr, const int32_t* col, const real* wval,
               int kind, int bits, uint64_t block, uint64_t k, real gamma, real eta, uint64_t seed, uint64_t t,
               real* x, real* xhat, const real* g, real* cv_out, uint8_t* msg_buf, uint64_t msg_cap, uint64_t* msg_bytes) {
    if (check_arguments<real>(n, N, rowptr, col, wval, kind, bits, block, k, x, xhat, g)) return 1;
    const uint64_t total = (uint64_t)n * N;
    std::vector<real> xh(total), d(total), mixed(total), cv_local;
    real* q = cv_out;
    if (!q) { cv_local.resize(total); q = cv_local.data(); }
#pragma omp parallel for schedule(static)
    for (uint64_t p = 0; p < total; ++p) {
        xh[p] = fma_<real>(-gamma, g[p], x[p]);
        d[p] = xh[p] - xhat[p];
    }
    const int rc = compress_workers<real>(n, N, d.data(), q, kind, bits, block, k, seed, t, 0, msg_buf, msg_cap, msg_bytes);
    if (rc == 1) return 1;
#pragma omp parallel for schedule(static)
    for (uint64_t p = 0; p < total; ++p) xhat[p] = xhat[p] + q[p];
    mix_minus_identity<real>(n, N, rowptr, col, wval, xhat, mixed.data());
#pragma omp parallel for schedule(static)
    for (uint64_t p = 0; p < total; ++p) x[p] = fma_<real>(eta, mixed[p], xh[p]);
    return rc;
}

}  // namespace

extern "C" {

void dso_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    philox4x32_10(ctr, key, out);
}

uint32_t dso_rounding_word(uint64_t seed, uint64_t t, uint32_t i, uint64_t j) {
    return rounding_word(seed, t, i, j);
}

uint32_t dso_keep_word(uint64_t seed, uint64_t t, uint32_t i, uint64_t j) { return keep_word(seed, t, i, j); }

uint32_t dso_gspar_word(uint64_t seed, uint64_t t, uint32_t i, uint64_t j) { return gspar_word(seed, t, i, j); }

double dso_sum_abs_tree_f32(const float* v, uint64_t N) { return sum_abs_tree<float>(v, N); }

uint64_t dso_rand_sparse_capacity(uint64_t N, uint64_t k) { return rand_sparse_capacity(N, k); }

// Threads the loops over workers are spread over: 1 unless built with -fopenmp.
int dso_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

double dso_sum_squares_tree_f32(const float* v, uint64_t N) { return sum_squares_tree<float>(v, N); }

int dso_step_f32(int n, uint64_t N, const int32_t* rowptr, const int32_t* col, const float* wval,
                 int kind, int bits, uint64_t block, uint64_t k, float gamma, float eta,
                 uint64_t seed, uint64_t t, float* x, float* delta, const float* g,
                 float* cv, uint8_t* msg, uint64_t msg_cap, uint64_t* msg_bytes) {
    return step<float>(n, N, rowptr, col, wval, kind, bits, block, k, gamma, eta, seed, t,
                       x, delta, g, cv, msg, msg_cap, msg_bytes);
}

// The same step on a window of columns [col0, col0 + N) of a wider problem: only the addresses of
// the random rounding words know about col0.  For the per-block operators (col0 a multiple of the
// block size) and the identity the result equals the corresponding columns of the wide problem's.
int dso_step_window_f32(int n, uint64_t N, uint64_t col0, const int32_t* rowptr, const int32_t* col, const float* wval,
                        int kind, int bits, uint64_t block, float gamma, float eta,
                        uint64_t seed, uint64_t t, float* x, float* delta, const float* g,
                        uint8_t* msg, uint64_t msg_cap, uint64_t* msg_bytes) {
    if (kind == TOPK || kind == QUANT_L2NORM || kind == RAND_SPARSE || kind == GSPAR) return 1;   // whole-vector operators and messages have no windows
    if ((kind == QUANT_MAXABS || kind == SIGN_MEANABS) && block && col0 % block) return 1;
    return step<float>(n, N, rowptr, col, wval, kind, bits, block, 0, gamma, eta, seed, t,
                       x, delta, g, nullptr, msg, msg_cap, msg_bytes, col0);
}

int dso_step_f64(int n, uint64_t N, const int32_t* rowptr, const int32_t* col, const double* wval,
                 int kind, int bits, uint64_t block, uint64_t k, double gamma, double eta,
                 uint64_t seed, uint64_t t, double* x, double* delta, const double* g,
                 double* cv, uint8_t* msg, uint64_t msg_cap, uint64_t* msg_bytes) {
    return step<double>(n, N, rowptr, col, wval, kind, bits, block, k, gamma, eta, seed, t,
                        x, delta, g, cv, msg, msg_cap, msg_bytes);
}

// The comparison updates: algo 1 = DCD-PSGD (state2 is not used), algo 2 = CHOCO-SGD (state2 = xhat).
int dso_compare_step_f32(int algo, int n, uint64_t N, const int32_t* rowptr, const int32_t* col, const float* wval,
                         int kind, int bits, uint64_t block, uint64_t k, float gamma, float eta,
                         uint64_t seed, uint64_t t, float* x, float* state2, const float* g,
                         float* cv, uint8_t* msg, uint64_t msg_cap, uint64_t* msg_bytes) {
    if (algo == 1) return step_dcd<float>(n, N, rowptr, col, wval, kind, bits, block, k, gamma, eta, seed, t, x, state2, g, cv, msg, msg_cap, msg_bytes);
    if (algo == 2) return step_choco<float>(n, N, rowptr, col, wval, kind, bits, block, k, gamma, eta, seed, t, x, state2, g, cv, msg, msg_cap, msg_bytes);
    return 1;
}

int dso_compare_step_f64(int algo, int n, uint64_t N, const int32_t* rowptr, const int32_t* col, const double* wval,
                         int kind, int bits, uint64_t block, uint64_t k, double gamma, double eta,
                         uint64_t seed, uint64_t t, double* x, double* state2, const double* g,
                         double* cv, uint8_t* msg, uint64_t msg_cap, uint64_t* msg_bytes) {
    if (algo == 1) return step_dcd<double>(n, N, rowptr, col, wval, kind, bits, block, k, gamma, eta, seed, t, x, state2, g, cv, msg, msg_cap, msg_bytes);
    if (algo == 2) return step_choco<double>(n, N, rowptr, col, wval, kind, bits, block, k, gamma, eta, seed, t, x, state2, g, cv, msg, msg_cap, msg_bytes);
    return 1;
}

}  // extern "C"

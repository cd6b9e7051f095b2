/*
 * dsq.h -- C ABI of libdsq: the per-iteration hot path of DeepSqueeze
 * (Tang, Lian, Qiu, Yuan, Zhang, Zhang, Liu: "DeepSqueeze: Decentralization
 * meets error-compensated compression", arXiv:1907.07346) on one AMD MI355X.
 *
 * The library simulates the n workers of the paper's Equation (1) as the rows
 * of an n x N fp32 state on a single GPU.  One ds_step() call is one pass of
 * the loop body of Algorithm 1 (lines 5-9) for all workers:
 *
 *   v_i     = x_i - gamma g_i + delta_i                              (line 5)
 *   C[v_i]  = C_omega(v_i),   delta_i = v_i - C[v_i]                 (line 6)
 *   message_i = packed C[v_i]  ("send"/"receive" = written to HBM)   (lines 7-8)
 *   x_i     = x_i - gamma g_i + eta sum_{j in N(i)} (W_ij - I_ij) C[v_j],
 *             N(i) containing i itself                               (line 9)
 *
 * All pointers named *_dev are device pointers of the current HIP device; all
 * others are host pointers.  No torch types, no C++ types.  Every function
 * returns a ds_status (or a plain value), never throws and never aborts.
 * A handle is not thread-safe; calls on one handle must not overlap.
 */
#ifndef DSQ_H
#define DSQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ds_handle ds_handle;   /* opaque; owned by the library, freed by ds_destroy */

typedef enum {
    DS_OK = 0,
    DS_EINVAL = 1,   /* bad argument or unsupported configuration; see ds_last_error */
    DS_ENOMEM = 2,   /* device or host allocation failed */
    DS_EHIP = 3,     /* a HIP runtime call failed */
    DS_ESTATE = 4    /* call not valid in the handle's current state (e.g. no step taken yet) */
} ds_status;

/* Communication graph.  W is the symmetric doubly stochastic mixing matrix of
 * the paper's Algorithm section and Assumption 1.2. */
typedef enum {
    DS_TOPO_RING = 0,     /* W_ii = W_i,i+1 = W_i,i-1 = 1/3 (indices mod n), n >= 3            */
    DS_TOPO_TORUS2D = 1,  /* node r*cols+c; self and the 4 wrap-around neighbours weigh 1/5;   */
                          /* torus_rows, torus_cols >= 3, torus_rows*torus_cols == n           */
    DS_TOPO_CSR = 2       /* W given by the caller in CSR form                                 */
} ds_topology;

/* Compression operator C_omega (the paper leaves it generic, Assumption 1.6). */
typedef enum {
    DS_COMP_IDENTITY = 0,     /* C[v] = v: the step is plain D-PSGD; message = v in fp32        */
    DS_COMP_QUANT_MAXABS = 1, /* stochastic `bits`-bit uniform quantisation per block of `block` */
                              /* elements, scale = max |v| of the block; bits in {2, 4, 8}       */
    DS_COMP_SIGN_MEANABS = 2, /* sign bit per element, scale = mean |v| of the block            */
    DS_COMP_TOPK = 3,         /* the k largest |v| of each worker's whole vector, ties to the   */
                              /* lower index; message = k (u32 index, f32 value) pairs          */
    DS_COMP_QUANT_L2NORM = 4, /* the compression of the paper's experiments (section             */
                              /* "Experimental Setup", paragraph "Compression"): a `bits`-bit     */
                              /* code per element of the worker's whole vector plus ONE number,   */
                              /* its Euclidean norm, to which the receiver rescales what it       */
                              /* decodes.  Grid: 2^bits levels from -max|v| to +max|v|, nearest   */
                              /* level (ties to the even code); code q stands for y = 2q - L,     */
                              /* C[v] = y * (norm / ||y||_2).  Message per worker:                */
                              /* [f32 norm][ceil(N*bits/32) u32 words]; bits in {2, 4, 8}         */
    DS_COMP_RAND_SPARSE = 5,  /* random sparsification (named next to top-k under Assumption 1.6): */
                              /* every element is kept independently with probability k/N (floor   */
                              /* to a multiple of 2^-24) and not rescaled; the mask comes from the  */
                              /* shared seed, so the message carries values only:                  */
                              /* [u32 count][count f32, ascending column], zero-padded to          */
                              /* min(N, k + 8 ceil(sqrt k) + 64) values per worker                  */
    DS_COMP_GSPAR = 6         /* GSpar (named next to random sparsification under Assumption 1.6), read as the */
                              /* magnitude-proportional sparsifier: element j is kept with probability          */
                              /* p_j = min(1, k |v_j| / sum_j |v_j|) (one shot: no second round where some p_j  */
                              /* are cut off at 1) and, like DS_COMP_RAND_SPARSE, not rescaled; the mask depends */
                              /* on v, so the message carries the columns: [u32 count][u32 0][count (u32 column, */
                              /* f32 value) pairs, ascending column], zero-padded to min(N, k + 8 ceil(sqrt k)   */
                              /* + 64) pairs                                                                     */
} ds_comp_kind;

typedef struct {
    int32_t  kind;    /* ds_comp_kind */
    int32_t  bits;    /* QUANT_MAXABS, QUANT_L2NORM: 2, 4 or 8; otherwise ignored               */
    int32_t  block;   /* QUANT_MAXABS, SIGN_MEANABS: power of two, 64 <= block <= 2048 (the fused  */
                      /* kernel holds a whole block in one wave's registers)                    */
    int32_t  reserved;
    uint64_t k;       /* TOPK: 1 <= k <= N; RAND_SPARSE, GSPAR: expected kept elements per      */
                      /* worker, 1 <= k <= N; otherwise ignored                                 */
} ds_comp;

/* Update rule of a step.  DS_ALGO_DEEPSQUEEZE is Algorithm 1.  The other two are the compressed decentralized
 * methods the paper measures DeepSqueeze against (section "Why DeepSqueeze is better", the DCD-PSGD and
 * CHOCO-SGD items; section "Experiments").  The paper states no update rule for them, only unrolled forms of X_t
 * and two properties: without compression error each is the paper's D-PSGD, X+ = (X - gamma G) W_eff, and one
 * step's error reaches X through powers of W_eff alone (DCD-PSGD) or through (W_eff - I) times such powers
 * (CHOCO-SGD).  The rules below are the simplest per-worker rules with those properties, in Algorithm 1's
 * notation, with the same C_omega, message layout and coefficients W_ij - I_ij (xh_i = x_i - gamma g_i):
 *   DS_ALGO_DCD_PSGD   z_i = xh_i + eta sum_{j in N(i)} (W_ij - I_ij) xh_j - x_i;   x_i = x_i + C[z_i];
 *                      message_i = packed C[z_i].  No second state array: delta is not touched.
 *   DS_ALGO_CHOCO_SGD  q_i = C[xh_i - xhat_i];   xhat_i = xhat_i + q_i;   message_i = packed q_i;
 *                      x_i = xh_i + eta sum_{j in N(i)} (W_ij - I_ij) xhat_j  (the copies after their update).
 *                      The workers' public copies xhat_i take the place of delta_i in the state: wherever this
 *                      header says delta (ds_read_state, ds_write_state, ds_state_ptrs, ds_diagnostics out[1]
 *                      and out[2]) read xhat.
 * Both are served for DS_COMP_QUANT_MAXABS and DS_COMP_SIGN_MEANABS by a fused tile kernel that keeps n rows
 * of one tile in LDS as fp32: n * max(block, 256) * 4 bytes must fit in 160 KB. */
typedef enum { DS_ALGO_DEEPSQUEEZE = 0, DS_ALGO_DCD_PSGD = 1, DS_ALGO_CHOCO_SGD = 2 } ds_algorithm;

typedef struct {
    int32_t  n;               /* number of workers (rows), >= 1                                  */
    int32_t  topo;            /* ds_topology                                                     */
    uint64_t N;               /* parameters per worker (columns), >= 1                           */
    int32_t  torus_rows;      /* DS_TOPO_TORUS2D only                                            */
    int32_t  torus_cols;
    /* DS_TOPO_CSR only (host pointers, copied by ds_init): CSR of W, n rows, every row holding
     * its diagonal entry (possibly 0), columns strictly ascending.  ds_init checks W >= 0,
     * symmetry and row sums == 1 within 1e-6.  Must be NULL for RING / TORUS2D.               */
    const int32_t* W_rowptr;
    const int32_t* W_col;
    const float*   W_val;
    ds_comp  comp;
    float    gamma;           /* learning rate                                                   */
    float    eta;             /* averaging rate; the paper's Theorem 1 wants eta <= 1/2: a larger */
                              /* value is accepted and noted in ds_last_error                    */
    uint64_t seed;            /* key of the random streams (stochastic rounding, sparsifier mask) */
    int32_t  algo;            /* ds_algorithm; 0 = DeepSqueeze                                    */
    int32_t  reserved;        /* must be 0                                                        */
} ds_config;

/* ---- host-only helpers (no GPU needed) ------------------------------------------------------ */

/* Checks a configuration the way ds_init does.  On failure writes a message of at most
 * errbuf_len-1 characters into errbuf (if non-NULL) and returns DS_EINVAL. */
ds_status ds_validate_config(const ds_config* cfg, char* errbuf, uint64_t errbuf_len);

/* Writes the CSR of W for a ring or torus configuration (the matrix ds_init would use).
 * rowptr: n+1 entries; col, val: capacity `cap` entries; *nnz receives the count.
 * Returns DS_EINVAL if the topology is invalid or cap is too small. */
ds_status ds_build_topology(const ds_config* cfg, int32_t* rowptr, int32_t* col, float* val,
                            uint64_t cap, uint64_t* nnz);

/* Bytes of all n workers' packed messages of one step (row i's message starts at
 * i * ds_message_bytes(cfg) / n).  Layout per worker:
 *   QUANT / SIGN: for each block, in column order: [f32 scale][ceil(m*b/32) u32 words], m = number
 *                 of elements in the block (the last one may be ragged), b = bits (1 for SIGN);
 *                 the code of element e of the block sits in bits [b*(e mod 32/b), +b) of word
 *                 floor(e*b/32); QUANT code q in [0, 2^b-1] decodes to (2q - (2^b-1)) * scale/(2^b-1);
 *                 SIGN bit 1 means negative and decodes to -scale; unused high bits are 0.
 *   TOPK:         k pairs (u32 index, f32 value) in ascending index order.
 *   IDENTITY:     N fp32 values.
 *   QUANT_L2NORM: [f32 norm][ceil(N*b/32) u32 words], codes packed as for QUANT; code q stands for the odd
 *                 integer y = 2q - (2^b-1) and the receiver returns y * (norm / sqrt(sum of y^2)).
 *   RAND_SPARSE:  [u32 count][count f32 values in ascending column order], zero-padded to the fixed capacity
 *                 min(N, k + 8 ceil(sqrt k) + 64) values; which columns were kept follows from the seed
 *                 (Philox4x32-10, counter (floor(j/4), i, t, 'SPAR'), word j mod 4, kept iff
 *                 (word >> 8) < floor(k 2^24 / N)).
 *   GSPAR:        [u32 count][u32 0][count pairs (u32 column, f32 value) in ascending column order], zero-padded
 *                 to the same capacity in pairs.  Element j is kept iff u < p_j, u = (word >> 8) / 2^24 with the
 *                 Philox word of counter (floor(j/4), i, t, 'GSPR'), word j mod 4, and p_j = fp32(k / S) * |v_j| in
 *                 fp32, S = sum_j |v_j| in double (balanced adjacent-pairs tree over the zero-padded vector).
 * Returns 0 for an invalid configuration. */
uint64_t ds_message_bytes(const ds_config* cfg);

/* Identifies the sources the library was built from (a hash the build script computes over the kernel and
 * host sources, this header and the compiler flags); reports print it next to their measurements. */
const char* ds_build_id(void);

/* ---- the hot path --------------------------------------------------------------------------- */

/* Creates the state on the current HIP device: x = 0, delta = 0, t = 0 (Algorithm 1, line 1;
 * Assumption 1.4).  Allocates x, delta (n rows with an internal pitch), the message buffer and
 * scratch with hipMalloc.  *out is NULL on failure; ds_init_ex also says why.
 * For large problems (n*N >= 32 Mi) of the block compressors the call times the candidate launch
 * shapes and row pitches of the fused kernel on the (still zero) state and keeps the fastest; the
 * choice is reported by ds_plan_name and can be pinned through ds_init_ex. */
ds_status ds_init(const ds_config* cfg, ds_handle** out);

/* ds_init with a say in the kernel plan and with the reason of a failure.  `plan` may be NULL (everything
 * automatic, what ds_init does).  errbuf (may be NULL) receives the reason of a failure, or the note ds_init
 * leaves in ds_last_error (eta > 1/2). */
typedef struct {
    int32_t variant;      /* 0: automatic; 1: the row-streaming variant of the block compressors (every wave   */
                          /*    takes one row of a tile, no LDS exchange; what serves more workers than the     */
                          /*    fused kernel's LDS holds is chosen automatically anyway)                        */
    int32_t tile_plan;    /* -1: automatic; i >= 0 pins the i-th candidate launch shape of the fused kernel      */
                          /*    (an index past the last candidate leaves the choice automatic)                   */
    int64_t pitch_skew;   /* -1: automatic; else floats added to the padded row length of x and delta:          */
                          /*    a multiple of 4, at most 12288                                                   */
    int32_t autotune;     /* 1: time the candidates at init (large problems only); 0: first candidate, default   */
                          /*    pitch (reproducible launches, a few per cent slower)                             */
    int32_t reserved;
} ds_plan_request;
ds_status ds_init_ex(const ds_config* cfg, const ds_plan_request* plan, char* errbuf, uint64_t errbuf_len, ds_handle** out);

/* One iteration of Algorithm 1 (lines 5-9) for all n workers with the gradients g_dev.
 * g_dev: caller-owned DEVICE pointer, n rows of fp32, row pitch g_ld >= N elements, g_ld a multiple
 * of 4, base 16-byte aligned; read-only.  Work is enqueued on hip_stream (a hipStream_t, NULL = the
 * default stream) and the call returns without synchronising; g_dev must stay valid until that
 * work has finished, and the stream until the handle's next call that synchronises (those calls
 * enqueue on, and wait for, the stream of the last ds_step).  Advances the step counter t by 1.  DS_ESTATE if the current HIP device is not
 * the one ds_init ran on.
 * The call only launches kernels: it makes no allocation, copy, memset or synchronisation, and the
 * step counter that selects the random rounding words lives in device memory and is advanced by
 * the enqueued work itself.  A stream capture of the call therefore gives a HIP graph whose every
 * replay is the next iteration (the gradients are read from the captured g_dev at replay time).
 * Such a graph stays valid until ds_destroy, or a ds_set_mixing that changes the number of stored
 * entries of W. */
ds_status ds_step(ds_handle* h, const float* g_dev, uint64_t g_ld, void* hip_stream);

/* ds_step for callers that cannot allocate device memory or keep a handle (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): one iteration of Algorithm 1 (lines 5-9) on arrays the caller
 * owns, with nothing allocated, copied or synchronised.  What ds_step keeps in the handle's scratch memory -- the
 * step counter with the tile kernel's finished-workgroup counters, and W - I in CSR form, built here by a small
 * kernel -- lives in a static device array of 61,700 bytes inside the library (one copy per GPU, held until the
 * process ends), which bounds the problem: n <= 1024 workers, DS_TOPO_RING or DS_TOPO_TORUS2D, and the
 * compressors of the fused tile kernel (DS_COMP_QUANT_MAXABS, DS_COMP_SIGN_MEANABS, DS_COMP_IDENTITY) with n
 * small enough for it (the codes of all n rows of a tile must fit in LDS); anything else is DS_EINVAL.
 *   x_dev, delta_dev: n rows of pitch ld floats, ld a multiple of 4 and at least N rounded up to a multiple of
 *                     4096, 16-byte aligned, columns >= N zero (they stay zero); updated in place.
 *   g_dev, g_ld:      as for ds_step.        msg_dev: ds_message_bytes(cfg) bytes, 4-byte aligned; receives the
 *   packed messages.  t: the iteration number (selects the random rounding words, as the handle's counter does).
 * The result is bit for bit what ds_init + ds_write_state(x, delta, t) + ds_step gives.  Work is enqueued on
 * hip_stream.  All calls on one GPU share the one static array: calls that overlap on a GPU (two streams, two
 * threads) race; calls on one stream are safe back to back.  errbuf (may be NULL) receives the reason of a
 * failure, or the eta > 1/2 note. */
ds_status ds_step_static(const ds_config* cfg, float* x_dev, float* delta_dev, uint64_t ld, const float* g_dev, uint64_t g_ld,
                         void* msg_dev, uint64_t t, void* hip_stream, char* errbuf, uint64_t errbuf_len);

/* Replaces the mixing matrix W for the following steps (time-varying communication graphs; the
 * paper's Algorithm 1 holds for any symmetric doubly stochastic W, and its related-work section
 * cites time-varying topologies).  CSR of W as for DS_TOPO_CSR (host pointers, copied): n rows, every
 * row with its diagonal entry, columns strictly ascending; checked like in ds_init (W >= 0,
 * symmetric, rows summing to 1 within 1e-6).  The step counter, x and delta are untouched.  The call
 * synchronises with the stream of the last ds_step.  DS_EINVAL leaves the old W in place.  A W with
 * as many stored entries as the current one is written over it in place (device addresses, and HIP
 * graphs captured from ds_step, stay valid); any other W moves to a new allocation. */
ds_status ds_set_mixing(ds_handle* h, const int32_t* W_rowptr, const int32_t* W_col, const float* W_val);

/* Replaces the step length gamma and the consensus step eta for the following steps (the paper's
 * experiments decay the learning rate during a run, section "Convergence Efficiency"; Algorithm 1
 * itself is stated for constants).  Both must be finite; eta > 1/2 is accepted with the note
 * ds_init gives.  A deferred tail of the last step is applied first, with the old eta.  A HIP
 * graph captured from ds_step keeps the values it was captured with.  Synchronises nothing. */
ds_status ds_set_rates(ds_handle* h, float gamma, float eta);

/* Copies the state -- the workers' models x_i and carried compression errors delta_i of Algorithm 1 (rows of
 * X and Delta in the paper's matrix notation, section "Mathematical formulation") -- to dense host arrays of
 * n*N fp32 each (delta_host may be NULL).  Synchronises with the stream of the last ds_step. */
ds_status ds_read_state(ds_handle* h, float* x_host, float* delta_host);

/* Overwrites x and delta (Algorithm 1's per-worker state; line 1 starts them at zero) from dense host
 * arrays (n*N fp32 each; NULL leaves that array unchanged) and sets the step counter.  With the
 * counter-based random stream this makes a run restartable: read_state at step t, write_state into a
 * fresh handle, and the continuation is bit-identical. */
ds_status ds_write_state(ds_handle* h, const float* x_host, const float* delta_host, uint64_t t);

/* Copies the packed messages of the last ds_step -- what Algorithm 1's lines 7-8 send and receive,
 * C_omega[v_i] of every worker in its wire format (layout: ds_message_bytes) -- into host_buf of
 * capacity cap; *bytes receives the size.  DS_ESTATE before the first step, DS_EINVAL if cap is
 * too small.  Synchronises like ds_read_state. */
ds_status ds_read_messages(ds_handle* h, void* host_buf, uint64_t cap, uint64_t* bytes);

/* Borrows the device arrays of x and delta (Algorithm 1's state, as for ds_read_state): row i of x starts
 * at x_dev + i*ld.  Ownership stays with the
 * handle; columns >= N of each row are padding the caller must leave zero.  The contents are
 * complete once the work enqueued so far on the stream of the last ds_step has finished (top-k,
 * the norm-rescaled codes and the row-streaming plans leave the last part of a step's update of x
 * and delta to the next step's first pass: this call enqueues it on that stream instead); call it
 * again after later steps before reading x. */
ds_status ds_state_ptrs(ds_handle* h, float** x_dev, float** delta_dev, uint64_t* ld);

/* Borrows the device buffer that holds the messages of the last ds_step (ds_message_bytes bytes, layout as
 * above).  Some launch plans alternate between two buffers, so ask again after every step; then the call
 * synchronises with the stream of the last ds_step. */
ds_status ds_message_ptr(ds_handle* h, void** msg_dev, uint64_t* bytes);

/* The quantities the paper's analysis tracks, computed on the device in fp64 (off the hot path,
 * synchronises):
 *   out[0] = ||X (I - A_n)||_F^2 = sum_i |x_i - mean_i x_i|^2   (consensus distance, squared)
 *   out[1] = ||Delta||_F^2                                       (compression error carried over)
 *   out[2] = ||Delta (W_eff - I)||_F^2, W_eff - I = eta (W - I)  (the part of it that reaches x)
 *   out[3] = bytes of one step's packed messages (= ds_message_bytes) */
ds_status ds_diagnostics(ds_handle* h, double* out4);

/* Diagnostics for DS_COMP_TOPK, DS_COMP_GSPAR and DS_COMP_QUANT_L2NORM: the number of workers whose last ds_step took the
 * path that needs no second pass over v.  Top-k: the k largest were found among the candidates collected while
 * forming v, instead of re-reading v (the exact fallback taken on the first step and whenever the threshold
 * guess of the previous step was too high or a candidate slot overflowed).  Norm-rescaled codes: the codes written
 * while forming v under a guessed band for max|v| stood (the band held the real maximum and no slot of undecided
 * elements overflowed), instead of the exact second pass.  GSpar: everything that was kept was among the elements
 * collected while forming v under an upper bound of lambda taken from the step before.  Results are identical
 * either way.  Synchronises; 0
 * for other compressors; DS_ESTATE before the first step. */
ds_status ds_topk_candidate_rows(ds_handle* h, uint32_t* count);

/* Step counter t: the number of iterations executed since init (graph replays included), or since
 * the value set by ds_write_state.  Read from the device; synchronises with the stream of the last
 * ds_step call. */
uint64_t ds_step_count(const ds_handle* h);

/* Name of the kernel plan ds_step uses for this handle (static string, for reports). */
const char* ds_plan_name(const ds_handle* h);

/* Text of the last error or warning on this handle ("" if none).  Valid until the next call. */
const char* ds_last_error(const ds_handle* h);

/* Harness aid, not part of the method: synthetic stochastic gradients made on the device, bit-identical to
 * the host generator paper_1907_07346_amd/detgen.py (Philox4x32-10 -> Box-Muller in double with fixed
 * polynomials for ln, sin and cos), so that long free runs need no host-device traffic.
 *   DS_GRAD_NORMAL      g = scale * N(0,1), independent per (step, worker, column)
 *   DS_GRAD_STUDENT_T3  g = scale * Z / sqrt((Z1^2 + Z2^2 + Z3^2) / 3): heavy tails, 3 degrees of freedom
 *   DS_GRAD_QUADRATIC   g = (x - c) + scale * xi for f_i(x) = 1/2 |x - c_i|^2, c_i ~ N(0,1) fixed by the seed;
 *                       x_dev: the current iterate, n rows of pitch x_ld (e.g. from ds_state_ptrs)
 * g_dev: n rows of pitch g_ld >= N, columns N .. g_ld-1 are written as zeros.  x_dev is ignored (may be NULL)
 * for the first two kinds.  Enqueued on hip_stream; no synchronisation. */
typedef enum { DS_GRAD_NORMAL = 0, DS_GRAD_STUDENT_T3 = 1, DS_GRAD_QUADRATIC = 2 } ds_grad_kind;
typedef struct {
    int32_t  n;       /* workers */
    int32_t  kind;    /* ds_grad_kind */
    uint64_t N;       /* parameters per worker */
    float    scale;   /* noise level (fp32) */
    float    reserved;
    uint64_t seed;
} ds_workload;
ds_status ds_workload_gradient(const ds_workload* w, uint64_t t, const float* x_dev, uint64_t x_ld, float* g_dev,
                               uint64_t g_ld, void* hip_stream);

/* Measurement aid, not part of the method: a plain streaming copy of `bytes` (a multiple of 16,
 * both pointers 16-byte aligned, device memory) enqueued on hip_stream.  Benchmarks use it to
 * report the HBM bandwidth a trivial kernel reaches on the same GPU, and profiles use it to
 * calibrate the hardware traffic counters against a known byte count.  DS_EINVAL for bytes >= 64 GiB. */
ds_status ds_bench_copy(void* dst_dev, const void* src_dev, uint64_t bytes, void* hip_stream);

/* Measurement aid, not part of the method: the access mix of ds_step without its arithmetic -- per 16 bytes
 * three streaming loads (x, delta, g) and two stores (x += g, delta += g, in place) -- over three device arrays of
 * `bytes` each (a multiple of 16, 16-byte aligned), enqueued on hip_stream.  5 * bytes move per call.
 * delta_dev == NULL: the mix of the DCD-PSGD step instead, two loads (x, g) and one store (x += g), 3 * bytes per call.
 * DS_EINVAL for bytes >= 64 GiB. */
ds_status ds_bench_stream(void* x_dev, void* delta_dev, const void* g_dev, uint64_t bytes, void* hip_stream);

/* Frees everything the handle owns (synchronises first).  NULL is a no-op. */
void ds_destroy(ds_handle* h);

#ifdef __cplusplus
}
#endif
#endif /* DSQ_H */

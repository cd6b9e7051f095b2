// Internal declarations shared by the host side and the kernel launchers of libdsq.
// Nothing here is part of the C ABI (that is include/dsq.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "dsq.h"

namespace dsq {

constexpr int kWave = 64;                 // gfx950 wavefront
constexpr int kSweep = 4 * kWave;         // columns one wave covers with one float4 per lane
constexpr uint64_t kPitchAlign = 4096;    // x / delta row pitch: N rounded up to this many floats ...
constexpr uint64_t kPitchSkew = 2560;     // ... plus 10 KB, so that rows do not sit a power of two apart: with all rows
                                          // of a column tile in flight at once, HBM channel hashing made a 16 MiB pitch
                                          // 12 % slower than this one on MI355X (measured, 64 rows x 4 Mi columns)
constexpr int kMinBlock = 64, kMaxBlock = 2048;
constexpr size_t kStepCells = 32 * 65;    // 64-bit cells behind the step counter (see TileArgs::t_ptr)

// Host-side description of W - I in CSR form (diagonal always present, columns ascending).
struct Graph {
    std::vector<int32_t> rowptr, col;
    std::vector<float> w;      // W_ij as given / built
    std::vector<float> coef;   // a_ij = W_ij - I_ij in fp32 (the coefficients of Algorithm 1, line 9)
    int max_degree = 0;        // entries per row, diagonal included
};

// Validation and topology construction (pure host code, usable without a GPU).
ds_status validate_config(const ds_config* cfg, std::string& err, std::string* warn);
ds_status build_graph(const ds_config* cfg, Graph& g, std::string& err);
uint64_t message_row_bytes(const ds_config* cfg);

// Arguments of the fused tile kernels (block quantiser / sign / identity).
struct TileArgs {
    float* x;                  // n x ld
    float* delta;              // n x ld
    const float* g;            // n x g_ld
    uint8_t* msg;              // n x msg_row_bytes
    const int32_t* rowptr;     // device CSR of W - I: rowptr (n+1), col (nnz) and coef (nnz, fp32 bits)
    const int32_t* col;        // are ONE contiguous array in that order (the tile kernel copies it whole)
    const float* coef;
    uint64_t ld, g_ld, N, msg_row_bytes;
    int n, nnz;                // workers; stored entries of W - I
    float gamma, eta;
    uint32_t seed_lo, seed_hi;
    // row-streaming variant only:
    const uint8_t* msg_prev;           // the previous step's messages: set by the kernels themselves (msg holds two
    uint64_t msg_half;                 // buffers of msg_half bytes; step t writes half t & 1 and reads the other)
    uint32_t* pending;                 // 1: the previous step's gossip sum has not been added to x yet
    // random sparsifier only:
    const uint32_t* keep_off;          // n x nsweeps: kept values before each 256-column sweep inside its group of 16
    const uint32_t* keep_group_off;    // n x ngroups: values the row's message holds before each group
    uint32_t* keep_raw;                // 2 x n x nsweeps: kept elements per sweep; half [t & 1] belongs to step t
    uint64_t nsweeps, ngroups;         // ceil(N / 256), ceil(nsweeps / 16)
    uint32_t keep_thr;                 // an element is kept iff the top 24 bits of its random word are below this
    uint32_t msg_cap;                  // values a row's message has room for
    unsigned long long* t_ptr;         // kStepCells 64-bit cells in device memory.  [0]: the step counter t, read by
                                       // the kernel and advanced by its last workgroup to finish, so that a captured
                                       // HIP graph of ds_step keeps moving along the random stream on replay.
                                       // [1]: finished first-level cells; [2]: random sparsifier: the step whose keep
                                       // counts are in keep_raw (~0 if none); [3]: row-streaming variant: a gossip sum is
                                       // pending; [4]: row-streaming variant: the message buffer (0 / 1) the last step
                                       // wrote; [16]: tile queue of the kernels whose workgroups walk over tiles (next tile
                                       // to hand out, counted from the grid size); [32 (1+c)], c < 64: finished
                                       // workgroups with blockIdx % 64 == c.
                                       // Cells [1], [16] and [32 (1+c)] are zero between launches.
};

// A compiled variant of the fused tile kernel, chosen once at init.
struct TilePlan {
    const char* name = "";
    void (*launch)(const TileArgs&, int rows_per_wave, hipStream_t) = nullptr;
    int tile_cols = 0;         // columns per workgroup
    int waves = 0;             // waves per workgroup
    int rows_per_wave = 0;     // rows each wave owns (held in registers when the variant says so)
    int sweeps = 0;            // 256-column sweeps per tile
    // Row-streaming variant (no LDS exchange, so no limit on n): a step leaves x = x - gamma g and its gossip sum
    // to the next step's pass, which decodes the neighbours' codes from the previous messages; `flush` adds a
    // pending sum now.
    bool streaming = false;
    void (*flush)(const TileArgs&, hipStream_t) = nullptr;
};

// Random sparsifier: makes sure the kept-element counts of this step's 256-column sweeps are in keep_raw (the tile
// kernel of the previous step normally left them there; otherwise they are recounted from the random words) and
// turns them into message offsets: local_off (n x nsweeps, = TileArgs::keep_off of the tile launch that follows)
// inside groups of 16 sweeps, group_tot (n x ngroups, = TileArgs::keep_group_off) across the groups.  Writes
// the per-row count into the message header (prev_count, n words, remembers it so that stale values behind a
// shorter message are cleared) and raises *overflow if a row keeps more than msg_cap values.
void launch_keep_offsets(const TileArgs& a, uint32_t* local_off, uint32_t* group_tot, uint32_t* prev_count, uint32_t* overflow,
                         hipStream_t stream);
uint64_t rand_sparse_capacity(uint64_t N, uint64_t k);

// The row-streaming plan of a block compressor (quantiser or sign); false if the compressor has none.
bool stream_plan(const ds_config& cfg, TilePlan& plan);

// Lists the variants that fit (n, compressor), best guess first; returns false with `err` set if none does.
bool choose_tile_plans(const ds_config& cfg, int nnz, std::vector<TilePlan>& plans, std::string& err);

// ---- top-k path ---------------------------------------------------------------------------------
struct TopkArgs {
    float* x;
    float* delta;
    const float* g;
    uint8_t* msg;              // n x k pairs (u32 index, f32 value)
    const int32_t* rowptr;
    const int32_t* col;
    const float* coef;
    uint64_t ld, g_ld, N, k;   // k: pairs from one row's message to the next (top-k: the k of the operator; GSpar: the
                               // capacity plus the header pair)
    int n;
    float gamma, eta;
    unsigned long long* t_ptr;  // step counter in device memory (advanced once per step)
    // GSpar only:
    uint64_t k_expected;       // the operator's k (expected kept elements)
    uint32_t seed_lo, seed_hi; // key of the mask's random stream
};

struct TopkState;              // device scratch of the radix select (histograms, per-chunk counts)
ds_status topk_create(const ds_config& cfg, uint64_t ld, TopkState** out, std::string& err);
void topk_destroy(TopkState* s);
ds_status topk_step(TopkState* s, const TopkArgs& a, hipStream_t stream);
// topk_step leaves the sparse part of the gossip update of x to the next step's first pass;
// topk_flush applies it now (no-op if nothing is pending).  Call before x is read or replaced, with the
// buffers, mixing matrix and eta the last step ran with (a.g is not used).
ds_status topk_flush(TopkState* s, const TopkArgs& a, hipStream_t stream);
// Number of rows whose last step selected from the candidate slots (the fast path).
ds_status topk_candidate_rows(TopkState* s, hipStream_t stream, uint32_t* count);
// GSpar: true if a row has kept more elements than its message has room for in some step since the handle was made.
ds_status gspar_overflowed(TopkState* s, hipStream_t stream, bool* overflowed);

// ---- norm-rescaled b-bit path (DS_COMP_QUANT_L2NORM) ----------------------------------------------
struct L2Args {
    float* x;
    float* delta;
    const float* g;
    uint8_t* msg;              // n rows of [f32 norm][code words]
    const int32_t* rowptr;
    const int32_t* col;
    const float* coef;
    uint64_t ld, g_ld, N, msg_row_bytes;
    uint64_t msg_half;         // msg holds two buffers of this many bytes; a step writes the one the last step did not
    int n;
    float gamma, eta;
    unsigned long long* t_ptr;  // step cells in device memory: [0] the step counter (advanced once per step), [4] the
                                // message buffer (0 / 1) the last completed step wrote, [5] rows finished in the
                                // step's last kernel (zero between launches)
};

struct L2State;                // device scratch: per-row scales, per-chunk partial reductions
ds_status l2q_create(const ds_config& cfg, uint64_t ld, L2State** out, std::string& err);
void l2q_destroy(L2State* s);
ds_status l2q_step(L2State* s, const L2Args& a, hipStream_t stream);
// l2q_step leaves delta = v - C[v] and the gossip update of x to the next step's first pass;
// l2q_flush applies them now (no-op if nothing is pending).  Call before the state is read or replaced, with
// the buffers, mixing matrix and eta the last step ran with (a.g is not used).
ds_status l2q_flush(L2State* s, const L2Args& a, hipStream_t stream);
// Number of rows whose last step kept the codes its first pass wrote speculatively (no second dense pass).
ds_status l2q_speculated_rows(L2State* s, hipStream_t stream, uint32_t* count);

// Device twin of the deterministic host gradient generator (harness aid).
ds_status launch_workload_gradient(const ds_workload& w, uint64_t t, const float* x, uint64_t x_ld, float* g, uint64_t g_ld,
                                   hipStream_t stream);

}  // namespace dsq

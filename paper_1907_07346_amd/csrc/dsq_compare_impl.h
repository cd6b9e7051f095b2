// Tile kernels for the two compressed decentralized methods the DeepSqueeze paper measures itself against
// (section "Why DeepSqueeze is better": the DCD-PSGD and CHOCO-SGD items; the paper prints only unrolled forms,
// the per-worker rules below are the reading include/dsq.h states under ds_algorithm).  Same tile shape as the
// DeepSqueeze kernel (dsq_tile_impl.h): one workgroup owns TC columns of ALL n workers, one pass over HBM, the
// rows meet through LDS.  What differs is what the rows exchange: both methods gossip on fp32 vectors (the public
// copies, or the models after their local step), not on decoded codes, so LDS holds n rows of TC floats.
//
//   CHOCO-SGD  phase 1 (per row)  xh = x - gamma g,  d = xh - xhat,  q = C[d] (scales, codes, message -> HBM),
//                                 xhat = xhat + q -> HBM and LDS
//              barrier
//              phase 2 (per row)  x = xh + eta sum_j (W_ij - I_ij) xhat_j from LDS              -> HBM
//              traffic per worker-parameter: 12 B read (x, g, xhat), 8 B written (x, xhat) + the message
//
//   DCD-PSGD   phase 1 (per row)  xh = x - gamma g -> LDS (x and xh stay in registers)
//              barrier
//              phase 2 (per row)  z = (xh + eta sum_j (W_ij - I_ij) xh_j) - x,  C[z] (scales, codes, message -> HBM),
//                                 x = x + C[z]                                                   -> HBM
//              traffic per worker-parameter: 8 B read (x, g), 4 B written (x) + the message
//
// The compression itself (block scales by wave reductions, stochastic rounding words, message layout) is the
// DeepSqueeze tile's encode_row, called with what the row keeps switched from v - C[v] to base + C[v].

#pragma once

#include "dsq_tile_impl.h"

namespace dsq {
namespace {

constexpr int kAlgoDcd = 1, kAlgoChoco = 2;     // = DS_ALGO_DCD_PSGD, DS_ALGO_CHOCO_SGD

template <int KIND, int BITS, int B, int SW, int NW>
struct CompareTile {
    using T = Tile<KIND, BITS, B, SW, NW>;
    static constexpr int TC = T::TC;
    static constexpr int ROW_BYTES = SW * kWave * 16;        // one float4 per lane and sweep

    // LDS: [fp32 values of all rows of the tile][rowptr n+1][col nnz][coef nnz]
    static __host__ __device__ constexpr size_t lds_bytes(int n, int nnz) {
        return (size_t)n * ROW_BYTES + (size_t)(n + 1 + 2 * nnz) * 4;
    }

    template <bool FULL>
    static __device__ __forceinline__ void load_x_g(const TileArgs& a, int i, uint64_t col0, int lane, float4 (&xv)[SW], float4 (&gv)[SW]) {
        const float* xr = a.x + (uint64_t)i * a.ld + col0 + 4 * lane;
        const float* gr = a.g + (uint64_t)i * a.g_ld + col0 + 4 * lane;
#pragma unroll
        for (int s = 0; s < SW; ++s) {
            xv[s] = ld4(xr + s * kSweep);
            if (FULL) {
                gv[s] = ld4(gr + s * kSweep);
            } else {                                                 // the caller's g has no padding to rely on
                const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                gv[s].x = (j + 0 < a.N) ? gr[s * kSweep + 0] : 0.f;
                gv[s].y = (j + 1 < a.N) ? gr[s * kSweep + 1] : 0.f;
                gv[s].z = (j + 2 < a.N) ? gr[s * kSweep + 2] : 0.f;
                gv[s].w = (j + 3 < a.N) ? gr[s * kSweep + 3] : 0.f;
            }
        }
    }

    static __device__ __forceinline__ void local_step(const TileArgs& a, const float4 (&xv)[SW], const float4 (&gv)[SW], float4 (&xh)[SW]) {
#pragma unroll
        for (int s = 0; s < SW; ++s) {
            xh[s].x = fmaf(-a.gamma, gv[s].x, xv[s].x); xh[s].y = fmaf(-a.gamma, gv[s].y, xv[s].y);
            xh[s].z = fmaf(-a.gamma, gv[s].z, xv[s].z); xh[s].w = fmaf(-a.gamma, gv[s].w, xv[s].w);
        }
    }

    // sum_j (W_ij - I_ij) row_j over the fp32 rows in LDS: neighbours in ascending index order (own index
    // included), one chain of fused multiply-adds per element starting from zero.
    static __device__ __forceinline__ void mix_row(const TileArgs& a, int i, int lane, const uint8_t* lds_vals,
                                                   const int32_t* lds_graph, float (&acc)[SW][4]) {
        const int32_t* g_col = lds_graph + a.n + 1;
        const float* g_coef = reinterpret_cast<const float*>(g_col + a.nnz);
        const int e0 = __builtin_amdgcn_readfirstlane(lds_graph[i]);
        const int e1 = __builtin_amdgcn_readfirstlane(lds_graph[i + 1]);
#pragma unroll
        for (int s = 0; s < SW; ++s) acc[s][0] = acc[s][1] = acc[s][2] = acc[s][3] = 0.f;
        auto edge = [&](int e) {
            const int nb = __builtin_amdgcn_readfirstlane(g_col[e]);
            const float w = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(g_coef[e])));
            const float4* nrow = reinterpret_cast<const float4*>(lds_vals + (size_t)nb * ROW_BYTES);
#pragma unroll
            for (int s = 0; s < SW; ++s) {
                const float4 r = nrow[s * kWave + lane];
                acc[s][0] = fmaf(w, r.x, acc[s][0]); acc[s][1] = fmaf(w, r.y, acc[s][1]);
                acc[s][2] = fmaf(w, r.z, acc[s][2]); acc[s][3] = fmaf(w, r.w, acc[s][3]);
            }
        };
        const int deg = e1 - e0;
        if (deg == 3) {                                   // ring
            edge(e0); edge(e0 + 1); edge(e0 + 2);
        } else if (deg == 5) {                            // 2-D torus
            edge(e0); edge(e0 + 1); edge(e0 + 2); edge(e0 + 3); edge(e0 + 4);
        } else {
            for (int e = e0; e < e1; ++e) edge(e);
        }
    }

    // ---- CHOCO-SGD --------------------------------------------------------------------------------------------
    template <bool FULL>
    static __device__ __forceinline__ void choco_phase1(const TileArgs& a, int i, uint64_t col0, int lane, uint8_t* lds_vals, float4 (&xh)[SW]) {
        float4 xv[SW], gv[SW], hv[SW], d[SW];
        float* hr = a.delta + (uint64_t)i * a.ld + col0 + 4 * lane;          // the public copies live where delta does
#pragma unroll
        for (int s = 0; s < SW; ++s) hv[s] = ld4(hr + s * kSweep);
        load_x_g<FULL>(a, i, col0, lane, xv, gv);
        local_step(a, xv, gv, xh);
#pragma unroll
        for (int s = 0; s < SW; ++s) {
            d[s].x = xh[s].x - hv[s].x; d[s].y = xh[s].y - hv[s].y; d[s].z = xh[s].z - hv[s].z; d[s].w = xh[s].w - hv[s].w;
        }
        // q = C[d]; xhat + q goes to HBM (through hr) and, as fp32, to this row's LDS slot
        T::template encode_row<FULL, 1>(a, i, i, col0, lane, d, hv, lds_vals + (size_t)i * ROW_BYTES, nullptr, hr);
    }

    template <bool FULL>
    static __device__ __forceinline__ void choco_phase2(const TileArgs& a, int i, uint64_t col0, int lane, const uint8_t* lds_vals,
                                                        const int32_t* lds_graph, const float4 (&xh)[SW]) {
        float acc[SW][4];
        mix_row(a, i, lane, lds_vals, lds_graph, acc);
        float* xout = a.x + (uint64_t)i * a.ld + col0 + 4 * lane;
#pragma unroll
        for (int s = 0; s < SW; ++s) {
            float4 xn;
            xn.x = fmaf(a.eta, acc[s][0], xh[s].x); xn.y = fmaf(a.eta, acc[s][1], xh[s].y);
            xn.z = fmaf(a.eta, acc[s][2], xh[s].z); xn.w = fmaf(a.eta, acc[s][3], xh[s].w);
            if (!FULL) {                                             // keep the pitch padding at zero
                const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                if (!(j + 0 < a.N)) xn.x = 0.f;
                if (!(j + 1 < a.N)) xn.y = 0.f;
                if (!(j + 2 < a.N)) xn.z = 0.f;
                if (!(j + 3 < a.N)) xn.w = 0.f;
            }
            st4(xout + s * kSweep, xn);
        }
    }

    // ---- DCD-PSGD ---------------------------------------------------------------------------------------------
    template <bool FULL>
    static __device__ __forceinline__ void dcd_phase1(const TileArgs& a, int i, uint64_t col0, int lane, uint8_t* lds_vals,
                                                      float4 (&xv)[SW], float4 (&xh)[SW]) {
        float4 gv[SW];
        load_x_g<FULL>(a, i, col0, lane, xv, gv);
        local_step(a, xv, gv, xh);
        float4* row = reinterpret_cast<float4*>(lds_vals + (size_t)i * ROW_BYTES);
#pragma unroll
        for (int s = 0; s < SW; ++s) row[s * kWave + lane] = xh[s];
    }

    // XH_LDS: the row's own xh is read from its LDS slot (where phase 1 put it) when it is needed, not passed in.
    template <bool FULL, bool XH_LDS = false>
    static __device__ __forceinline__ void dcd_phase2(const TileArgs& a, int i, uint64_t col0, int lane, const uint8_t* lds_vals,
                                                      const int32_t* lds_graph, const float4 (&xv)[SW], const float4 (&xh)[SW]) {
        float acc[SW][4];
        mix_row(a, i, lane, lds_vals, lds_graph, acc);
        float4 z[SW];
        const float4* own = reinterpret_cast<const float4*>(lds_vals + (size_t)i * ROW_BYTES);
#pragma unroll
        for (int s = 0; s < SW; ++s) {                               // the uncompressed method's target minus the model
            const float4 h = XH_LDS ? own[s * kWave + lane] : xh[s];
            z[s].x = fmaf(a.eta, acc[s][0], h.x) - xv[s].x; z[s].y = fmaf(a.eta, acc[s][1], h.y) - xv[s].y;
            z[s].z = fmaf(a.eta, acc[s][2], h.z) - xv[s].z; z[s].w = fmaf(a.eta, acc[s][3], h.w) - xv[s].w;
        }
        float* xout = a.x + (uint64_t)i * a.ld + col0 + 4 * lane;
        T::template encode_row<FULL, 2>(a, i, i, col0, lane, z, xv, nullptr, nullptr, xout);     // x = x + C[z]
    }

    // RPW > 0: every wave holds its rows' registers across the barrier.  RPW == 0: rows_per_wave rows per wave,
    // re-formed from HBM (mostly cache) in phase 2.
    template <int ALGO, int RPW, bool FULL>
    static __device__ __forceinline__ void run(const TileArgs& a, int rpw_runtime, uint64_t col0, uint8_t* lds) {
        const int lane = threadIdx.x & (kWave - 1);
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        uint8_t* lds_vals = lds;
        int32_t* lds_graph = reinterpret_cast<int32_t*>(lds + (size_t)a.n * ROW_BYTES);
        const int gtotal = a.n + 1 + 2 * a.nnz;                      // rowptr | col | coef, contiguous in device memory
        for (int q = threadIdx.x; q < gtotal; q += NW * kWave) lds_graph[q] = a.rowptr[q];
        if constexpr (RPW > 0) {
            float4 xh[RPW][SW];
            [[maybe_unused]] float4 xv[ALGO == kAlgoDcd ? RPW : 1][SW];
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                const int i = wave + r * NW;
                if (i < a.n) {
                    if constexpr (ALGO == kAlgoChoco) choco_phase1<FULL>(a, i, col0, lane, lds_vals, xh[r]);
                    else dcd_phase1<FULL>(a, i, col0, lane, lds_vals, xv[r], xh[r]);
                }
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                const int i = wave + r * NW;
                if (i < a.n) {
                    if constexpr (ALGO == kAlgoChoco) choco_phase2<FULL>(a, i, col0, lane, lds_vals, lds_graph, xh[r]);
                    else dcd_phase2<FULL>(a, i, col0, lane, lds_vals, lds_graph, xv[r], xh[r]);
                }
            }
        } else {
            float4 xh[SW], xv[SW], gv[SW];
            for (int r = 0; r < rpw_runtime; ++r) {
                const int i = wave + r * NW;
                if (i < a.n) {
                    if constexpr (ALGO == kAlgoChoco) choco_phase1<FULL>(a, i, col0, lane, lds_vals, xh);
                    else dcd_phase1<FULL>(a, i, col0, lane, lds_vals, xv, xh);
                }
            }
            __syncthreads();
            for (int r = 0; r < rpw_runtime; ++r) {
                const int i = wave + r * NW;
                if (i < a.n) {
                    load_x_g<FULL>(a, i, col0, lane, xv, gv);       // x is still the old model: phase 1 did not write it
                    local_step(a, xv, gv, xh);
                    if constexpr (ALGO == kAlgoChoco) choco_phase2<FULL>(a, i, col0, lane, lds_vals, lds_graph, xh);
                    else dcd_phase2<FULL>(a, i, col0, lane, lds_vals, lds_graph, xv, xh);
                }
            }
        }
    }
};

template <int KIND, int BITS, int B, int SW, int NW, int RPW, int ALGO>
__global__ void __launch_bounds__(NW* kWave) compare_tile_kernel(TileArgs a, int rpw_runtime) {
    using C = CompareTile<KIND, BITS, B, SW, NW>;
    extern __shared__ __align__(16) uint8_t lds[];
    const uint64_t tile = (uint64_t)blockIdx.y * gridDim.x + blockIdx.x;
    const uint64_t col0 = tile * C::TC;
    if (col0 + C::TC <= a.N) C::template run<ALGO, RPW, true>(a, rpw_runtime, col0, lds);
    else if (col0 < a.N)     C::template run<ALGO, RPW, false>(a, rpw_runtime, col0, lds);
    // The step counter (read by the rounding words of phase 1 / phase 2) is advanced by the last workgroup to
    // finish; every wave of this workgroup must be done with it first.
    __syncthreads();
    step_counter_bump<KIND, BITS, B, SW, NW>(a, tile, (unsigned long long)gridDim.x * gridDim.y, false);
}

template <int KIND, int BITS, int B, int SW, int NW, int RPW, int ALGO>
void launch_compare(const TileArgs& a, int rpw_runtime, hipStream_t stream) {
    using C = CompareTile<KIND, BITS, B, SW, NW>;
    const uint64_t tiles = (a.N + C::TC - 1) / C::TC;
    const uint64_t max_x = 0xFFFFFFFFull / (NW * kWave);
    const unsigned gx = (unsigned)(tiles < max_x ? tiles : max_x);
    const unsigned gy = (unsigned)((tiles + gx - 1) / gx);
    const size_t lds = C::lds_bytes(a.n, a.nnz);
    auto kern = compare_tile_kernel<KIND, BITS, B, SW, NW, RPW, ALGO>;
    static unsigned long long attr_devices = 0;                       // as for the DeepSqueeze tile: once per kernel and device
    if (lds > 48 * 1024) {
        int dev = 0;
        (void)hipGetDevice(&dev);
        const unsigned long long bit = 1ull << (dev & 63);
        if (!(attr_devices & bit)) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            attr_devices |= bit;
        }
    }
    hipLaunchKernelGGL(kern, dim3(gx, gy), dim3(NW * kWave), lds, stream, a, rpw_runtime);
}

template <int KIND, int BITS, int B, int SW, int NW, int RPW, int ALGO>
void add_compare_plan(int n, const char* name, std::vector<TilePlan>& plans) {
    // registers: CHOCO-SGD holds xh of its rows across the barrier, DCD-PSGD x and xh (float4 each per sweep).
    // A 16-wave workgroup caps a wave at 128 VGPRs, an 8-wave one at 256; DCD-PSGD has nothing else to hold
    // while its loads are in flight, so its 8-wave shapes may keep up to 32 float4.
    constexpr int held = (ALGO == kAlgoDcd ? 2 : 1) * RPW * SW;
    constexpr int room = NW > 8 ? 8 : (ALGO == kAlgoDcd && SW <= 4 ? 32 : 16);   // 8 sweeps: the encoder's own registers grow too
    if constexpr (held <= room && (NW <= 8 || SW <= 4)) {
        if (n > NW * RPW) return;
        if (RPW > 1 && n <= NW * (RPW / 2)) return;
        TilePlan p;
        p.name = name;
        p.launch = &launch_compare<KIND, BITS, B, SW, NW, RPW, ALGO>;
        p.tile_cols = SW * kSweep;
        p.waves = NW;
        p.rows_per_wave = RPW;
        p.sweeps = SW;
        plans.push_back(p);
    }
}

// DCD-PSGD with the next tile's streams requested ahead.  The kernel above has all loads of a workgroup before its
// barrier and all arithmetic and stores behind it, and LDS (n rows of a tile in fp32) leaves room for one or two
// workgroups per CU, so nothing is in flight while a workgroup encodes.  Here a workgroup walks over tiles
// (the first one is blockIdx.x, the following ones are drawn from a counter in device memory, so that a workgroup
// on a slow CU takes fewer): after the barrier that publishes xh of tile T it requests x and g of its
// next tile into a second set of registers and then mixes, encodes and stores tile T (SPARE).  Where the registers
// do not allow a second set (many rows per wave), the request for row r of the next tile goes out as soon as row r
// of tile T is stored, into the registers that row has just given up: all but the last row's loads then overlap the
// encoding of the rows behind it.  Whole tiles only; the ragged last tile, if there is one, is taken by one
// workgroup with the plain routine at the end.  A row's own xh is read back from its LDS slot in phase 2 (the same
// fp32 values) rather than held in registers across the barrier: measured equal or faster, and 50 VGPRs fewer.
template <int KIND, int BITS, int B, int SW, int NW, int RPW, bool SPARE>
__global__ void __launch_bounds__(NW* kWave) dcd_ahead_kernel(TileArgs a) {
    using C = CompareTile<KIND, BITS, B, SW, NW>;
    extern __shared__ __align__(16) uint8_t lds[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint8_t* lds_vals = lds;
    int32_t* lds_graph = reinterpret_cast<int32_t*>(lds + (size_t)a.n * C::ROW_BYTES);
    const int gtotal = a.n + 1 + 2 * a.nnz;
    for (int q = threadIdx.x; q < gtotal; q += NW * kWave) lds_graph[q] = a.rowptr[q];
    const uint64_t whole = a.N / C::TC;                              // tiles without a ragged end
    constexpr int RS = SPARE ? RPW : 1;
    float4 xv[RPW][SW], gv[RPW][SW], xh[SW];
    [[maybe_unused]] float4 xn[RS][SW], gn[RS][SW];
    // tile queue: thread 0 draws the tile after next while the current one is in work and hands it to the others
    // through LDS at the first barrier
    // (32-bit numbers: a row of 2^32 tiles would be a terabyte)
    __shared__ unsigned s_next;
    unsigned long long* queue = a.t_ptr + 16;
    unsigned* queue32 = reinterpret_cast<unsigned*>(queue);
    const unsigned none = 0xFFFFFFFFu;
    unsigned upcoming = none;
    auto draw = [&]() {
        const unsigned q = gridDim.x + __hip_atomic_fetch_add(queue32, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return q < whole ? q : none;
    };
    if (threadIdx.x == 0) upcoming = draw();
    uint64_t tile = blockIdx.x;
    if (tile < whole) {
#pragma unroll
        for (int r = 0; r < RPW; ++r)
            if (wave + r * NW < a.n) C::template load_x_g<true>(a, wave + r * NW, tile * C::TC, lane, xv[r], gv[r]);
    }
    while (tile < whole) {
        const uint64_t col0 = tile * C::TC;
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int i = wave + r * NW;
            if (i < a.n) {
                C::local_step(a, xv[r], gv[r], xh);
                float4* row = reinterpret_cast<float4*>(lds_vals + (size_t)i * C::ROW_BYTES);
#pragma unroll
                for (int s = 0; s < SW; ++s) row[s * kWave + lane] = xh[s];
            }
        }
        if (threadIdx.x == 0) s_next = upcoming;
        __syncthreads();                                             // xh of all rows of tile T (and the graph) are in LDS
        const unsigned nx = (unsigned)__builtin_amdgcn_readfirstlane((int)s_next);
        const uint64_t next = nx != none ? (uint64_t)nx : whole;
        if (threadIdx.x == 0 && nx != none) upcoming = draw();
        if constexpr (SPARE) {
            if (next < whole) {                                      // uniform
#pragma unroll
                for (int r = 0; r < RPW; ++r)
                    if (wave + r * NW < a.n) C::template load_x_g<true>(a, wave + r * NW, next * C::TC, lane, xn[r], gn[r]);
            }
        }
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int i = wave + r * NW;
            if (i < a.n) {
                C::template dcd_phase2<true, true>(a, i, col0, lane, lds_vals, lds_graph, xv[r], xh);
                if constexpr (!SPARE) {
                    if (next < whole) C::template load_x_g<true>(a, i, next * C::TC, lane, xv[r], gv[r]);
                }
            }
        }
        __syncthreads();                                             // every wave is done with tile T's rows in LDS
        if constexpr (SPARE) {
#pragma unroll
            for (int r = 0; r < RPW; ++r)
#pragma unroll
                for (int s = 0; s < SW; ++s) { xv[r][s] = xn[r][s]; gv[r][s] = gn[r][s]; }
        }
        tile = next;
    }
    if (whole * C::TC < a.N && blockIdx.x == (unsigned)(whole % gridDim.x))            // uniform over the workgroup
        C::template run<kAlgoDcd, RPW, false>(a, 0, whole * C::TC, lds);
    __syncthreads();                                                 // every wave has read the step counter for the last time
    step_counter_bump<KIND, BITS, B, SW, NW>(a, blockIdx.x, gridDim.x, false, queue);
}

template <int KIND, int BITS, int B, int SW, int NW, int RPW, bool SPARE>
void launch_dcd_ahead(const TileArgs& a, int, hipStream_t stream) {
    using C = CompareTile<KIND, BITS, B, SW, NW>;
    const size_t lds = C::lds_bytes(a.n, a.nnz);
    auto kern = dcd_ahead_kernel<KIND, BITS, B, SW, NW, RPW, SPARE>;
    // as many workgroups as the device holds at once (asked once per kernel, device and LDS size)
    static int resident[64] = {0};
    static size_t resident_lds[64] = {0};
    int dev = 0;
    (void)hipGetDevice(&dev);
    dev &= 63;
    if (resident[dev] == 0 || resident_lds[dev] != lds) {
        if (lds > 48 * 1024) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, NW * kWave, lds) != hipSuccess || per_cu < 1) per_cu = 1;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        resident[dev] = per_cu * cus;
        resident_lds[dev] = lds;
        (void)hipGetLastError();
    }
    const uint64_t whole = a.N / C::TC;
    const uint64_t want = whole ? whole : 1;
    const unsigned grid = (unsigned)(want < (uint64_t)resident[dev] ? want : (uint64_t)resident[dev]);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * kWave), lds, stream, a);
}

template <int KIND, int BITS, int B, int SW, int NW, int RPW, bool SPARE>
void add_dcd_ahead_plan(int n, int nnz, const char* name, std::vector<TilePlan>& plans) {
    // registers, counted as x and the encoder's copy of a row of the tile in work and, with SPARE, x, g of the next
    // one, in float4 per lane
    constexpr int held = (SPARE ? 4 : 2) * RPW * SW;
    constexpr int room = SPARE ? (NW > 8 ? 16 : (SW <= 2 ? 64 : 32))
                               : (NW > 8 ? (SW <= 2 ? 16 : 8) : 32);          // beyond these the compiler spills
    if constexpr (held <= room && (NW <= 8 || SW <= 4)) {
        if (n > NW * RPW) return;
        if (RPW > 1 && n <= NW * (RPW / 2)) return;
        if (CompareTile<KIND, BITS, B, SW, NW>::lds_bytes(n, nnz) + 64 > kMaxLds) return;   // the kernel's own queue word
        TilePlan p;
        p.name = name;
        p.launch = &launch_dcd_ahead<KIND, BITS, B, SW, NW, RPW, SPARE>;
        p.tile_cols = SW * kSweep;
        p.waves = NW;
        p.rows_per_wave = RPW;
        p.sweeps = SW;
        plans.push_back(p);
    }
}

template <int KIND, int BITS, int B, int ALGO>
bool pick_compare_for_block(int n, int nnz, std::vector<TilePlan>& plans, std::string& err) {
    constexpr int SW = (B <= kSweep) ? 1 : (B / kSweep);
    using C = CompareTile<KIND, BITS, B, SW, 8>;
    if (C::lds_bytes(n, nnz) > kMaxLds) {
        err = "n is too large for the comparison kernels with this block size: n rows of one tile (n * max(block, 256) floats) must fit in 160 KB of LDS";
        return false;
    }
    add_compare_plan<KIND, BITS, B, SW, 8, 1, ALGO>(n, "8w/1row", plans);
    add_compare_plan<KIND, BITS, B, SW, 8, 2, ALGO>(n, "8w/2rows", plans);
    add_compare_plan<KIND, BITS, B, SW, 8, 4, ALGO>(n, "8w/4rows", plans);
    add_compare_plan<KIND, BITS, B, SW, 8, 8, ALGO>(n, "8w/8rows", plans);
    add_compare_plan<KIND, BITS, B, SW, 16, 1, ALGO>(n, "16w/1row", plans);
    add_compare_plan<KIND, BITS, B, SW, 16, 2, ALGO>(n, "16w/2rows", plans);
    add_compare_plan<KIND, BITS, B, SW, 16, 4, ALGO>(n, "16w/4rows", plans);
    if constexpr (ALGO == kAlgoDcd) {                               // after the plain shapes: small problems take the first candidate
        add_dcd_ahead_plan<KIND, BITS, B, SW, 16, 1, true>(n, nnz, "16w/1row/ahead", plans);
        add_dcd_ahead_plan<KIND, BITS, B, SW, 8, 1, true>(n, nnz, "8w/1row/ahead", plans);
        add_dcd_ahead_plan<KIND, BITS, B, SW, 8, 2, true>(n, nnz, "8w/2rows/ahead", plans);
        add_dcd_ahead_plan<KIND, BITS, B, SW, 8, 4, true>(n, nnz, "8w/4rows/ahead", plans);
        add_dcd_ahead_plan<KIND, BITS, B, SW, 8, 8, true>(n, nnz, "8w/8rows/ahead", plans);
        add_dcd_ahead_plan<KIND, BITS, B, SW, 8, 4, false>(n, nnz, "8w/4rows/ahead-in-turn", plans);
        add_dcd_ahead_plan<KIND, BITS, B, SW, 8, 8, false>(n, nnz, "8w/8rows/ahead-in-turn", plans);
        add_dcd_ahead_plan<KIND, BITS, B, SW, 16, 2, false>(n, nnz, "16w/2rows/ahead-in-turn", plans);
        add_dcd_ahead_plan<KIND, BITS, B, SW, 16, 4, false>(n, nnz, "16w/4rows/ahead-in-turn", plans);
    }
    if (plans.empty()) {
        constexpr int LW = SW >= 8 ? 8 : 16;                        // waves of the looped fallback
        TilePlan p;
        p.name = SW >= 8 ? "8w/looped" : "16w/looped";
        p.launch = &launch_compare<KIND, BITS, B, SW, LW, 0, ALGO>;
        p.tile_cols = SW * kSweep;
        p.waves = LW;
        p.rows_per_wave = (n + LW - 1) / LW;
        p.sweeps = SW;
        plans.push_back(p);
    }
    return true;
}

template <int KIND, int BITS, int ALGO>
bool pick_compare_for_kind(int block, int n, int nnz, std::vector<TilePlan>& plans, std::string& err) {
    switch (block) {
        case 64:   return pick_compare_for_block<KIND, BITS, 64, ALGO>(n, nnz, plans, err);
        case 128:  return pick_compare_for_block<KIND, BITS, 128, ALGO>(n, nnz, plans, err);
        case 256:  return pick_compare_for_block<KIND, BITS, 256, ALGO>(n, nnz, plans, err);
        case 512:  return pick_compare_for_block<KIND, BITS, 512, ALGO>(n, nnz, plans, err);
        case 1024: return pick_compare_for_block<KIND, BITS, 1024, ALGO>(n, nnz, plans, err);
        case 2048: return pick_compare_for_block<KIND, BITS, 2048, ALGO>(n, nnz, plans, err);
        default: err = "block must be a power of two between 64 and 2048"; return false;
    }
}

}  // namespace
}  // namespace dsq

// Fused compress-and-gossip tile kernels for the block compressors of libdsq (gfx950): the templates.
// Included by the dsq_tile_*.hip translation units, which instantiate them per compressor (side by side
// at build time).
//
// One workgroup owns a tile of TC consecutive parameter columns for ALL n workers.
// Because every scale block is column-local and the mixing matrix W only couples
// different workers at the same column, the whole loop body of DeepSqueeze's
// Algorithm 1 (lines 5-9) can be finished for the tile in one pass over HBM:
//
//   phase 1 (per worker row, one wave per row at a time)
//     line 5   xh = x - gamma g,  v = xh + delta            (float4 streams, registers)
//     line 6   per block: scale by a wave64 reduction, codes, C[v], delta = v - C[v] -> HBM
//     line 7   packed message -> HBM, and the codes + decode units -> LDS
//   barrier    ("receive": every row's codes of this tile are now in LDS)
//   phase 2    line 9: x = xh + eta * sum_j (W_ij - I_ij) C[v_j], decoding the neighbours'
//              codes from LDS, with xh still in registers                      -> HBM
//
// Traffic per worker-parameter: 12 B read (x, g, delta), 8 B written (x, delta) plus the
// packed message.  The floating-point expression order below is fixed (contraction off,
// explicit fmaf) so that codes, scales and messages are reproducible bit for bit.

#pragma once

#include "dsq_internal.h"
#include "dsq_philox.h"

namespace dsq {
namespace {

constexpr uint32_t kQuantStreamTag = 0x51554E54u;   // 4th counter word of the rounding stream
constexpr uint32_t kSparseStreamTag = 0x53504152u;  // ... and of the stream that draws the random sparsifier's mask

// 16-byte streaming accesses.  x, g and delta are touched exactly once per step, so they are
// marked non-temporal: on gfx950 that keeps the streams from displacing each other in L2 / MALL.
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld4(const float* p) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4(float* p, const float4& v) {
    const f32x4 w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<f32x4*>(p));
}

// ---- wave64 reductions on the DPP cross-lane path (no LDS traffic); the result is wave-uniform ----
// row_shr:1,2,4,8 fold each row of 16 lanes into its lane 15, row_bcast15 folds row r into row r+1
// (rows 1 and 3), row_bcast31 folds lane 31 into lane 63.  Lanes without a source keep `old`.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float old, float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_move<0x111, 0xF>(v, v));
    v = fmaxf(v, dpp_move<0x112, 0xF>(v, v));
    v = fmaxf(v, dpp_move<0x114, 0xF>(v, v));
    v = fmaxf(v, dpp_move<0x118, 0xF>(v, v));
    v = fmaxf(v, dpp_move<0x142, 0xA>(v, v));
    v = fmaxf(v, dpp_move<0x143, 0xC>(v, v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// Pairwise tree in lane order: level k adds the sums of adjacent groups of 2^k lanes (the order of the
// two operands of an addition does not matter), which is the balanced tree the scale definition asks for.
__device__ __forceinline__ float wave_sum_tree(float v) {
    v = v + dpp_move<0x111, 0xF>(0.f, v);
    v = v + dpp_move<0x112, 0xF>(0.f, v);
    v = v + dpp_move<0x114, 0xF>(0.f, v);
    v = v + dpp_move<0x118, 0xF>(0.f, v);
    v = v + dpp_move<0x142, 0xA>(0.f, v);
    v = v + dpp_move<0x143, 0xC>(0.f, v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Blocks narrower than a sweep (64 or 128 columns = 16 or 32 lanes): butterfly inside the group of lanes that
// holds the block; every lane of the group ends with the result.  For the sum this is again the balanced
// adjacent-pairs tree (the two partners of a level add the same two numbers).
template <int G>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
    for (int o = 1; o < G; o <<= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
template <int G>
__device__ __forceinline__ float group_sum_tree(float v) {
#pragma unroll
    for (int o = 1; o < G; o <<= 1) v = v + __shfl_xor(v, o);
    return v;
}

template <int KIND, int BITS> struct CodeTraits;
template <> struct CodeTraits<DS_COMP_QUANT_MAXABS, 8> { using lane_t = uint32_t; static constexpr int row_bytes_per_sweep = 256; };
template <> struct CodeTraits<DS_COMP_QUANT_MAXABS, 4> { using lane_t = uint16_t; static constexpr int row_bytes_per_sweep = 128; };
template <> struct CodeTraits<DS_COMP_QUANT_MAXABS, 2> { using lane_t = uint8_t;  static constexpr int row_bytes_per_sweep = 64; };
template <> struct CodeTraits<DS_COMP_SIGN_MEANABS, 1> { using lane_t = uint32_t; static constexpr int row_bytes_per_sweep = 32; };
template <> struct CodeTraits<DS_COMP_IDENTITY, 32>    { using lane_t = float4;   static constexpr int row_bytes_per_sweep = 1024; };
template <> struct CodeTraits<DS_COMP_RAND_SPARSE, 32> { using lane_t = float4;   static constexpr int row_bytes_per_sweep = 1024; };

__device__ __forceinline__ float comp(const float4& v, int c) { return c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w; }
__device__ __forceinline__ void set_comp(float4& v, int c, float f) { if (c == 0) v.x = f; else if (c == 1) v.y = f; else if (c == 2) v.z = f; else v.w = f; }

template <int KIND, int BITS, int B, int SW, int NW>
struct Tile {
    static constexpr int TC = SW * kSweep;                 // columns per tile
    static constexpr bool SUB = B < kSweep;                // several scale blocks share one sweep
    static constexpr int BPS = SUB ? kSweep / B : 1;       // scale blocks per sweep (SUB)
    static constexpr int G = SUB ? B / 4 : kWave;          // lanes that hold one block of a sweep
    static constexpr int SPB = SUB ? 1 : B / kSweep;       // sweeps per scale block
    static constexpr int BPT = SUB ? SW * BPS : SW / SPB;  // scale blocks per tile
    static constexpr int L = BITS < 31 ? (1 << (BITS & 15)) - 1 : 0;   // top quantisation level
    using CT = CodeTraits<KIND, BITS>;
    static constexpr int ROW_CODE_BYTES = SW * CT::row_bytes_per_sweep;
    static constexpr int MSG_BLOCK_BYTES = 4 + B * (BITS & 15) / 8;   // [scale][codes] of a full block
    static_assert((SUB ? kSweep % B == 0 : B % kSweep == 0) && SW % SPB == 0, "tile must hold whole blocks");

    // LDS: [codes of all rows][decode units of all rows][rowptr n+1][col nnz][coef nnz]
    static __host__ __device__ constexpr size_t lds_bytes(int n, int nnz) {
        return (size_t)n * ROW_CODE_BYTES + (size_t)n * BPT * sizeof(float) + (size_t)(n + 1 + 2 * nnz) * 4;
    }

    // ---- line 9 of the PREVIOUS step for one row of a tile, decoding the neighbours' codes from that step's
    //      messages in HBM (row-streaming variant: nothing is shared through LDS): x = xh + eta sum_j a_ij C[v_j]
    template <bool FULL>
    static __device__ __forceinline__ void gossip_from_messages(const TileArgs& a, int i, uint64_t col0, int lane, float4 (&x)[SW]) {
        static_assert(KIND == DS_COMP_QUANT_MAXABS || KIND == DS_COMP_SIGN_MEANABS || KIND == DS_COMP_IDENTITY,
                      "messages of this operator cannot be decoded per column");
        float acc[SW][4];
#pragma unroll
        for (int s = 0; s < SW; ++s) acc[s][0] = acc[s][1] = acc[s][2] = acc[s][3] = 0.f;
        const int e0 = a.rowptr[i], e1 = a.rowptr[i + 1];
        for (int e = e0; e < e1; ++e) {                         // ascending neighbour index, own index included
            const int nb = a.col[e];
            const float w = a.coef[e];
            const uint8_t* nrow = a.msg_prev + (uint64_t)nb * a.msg_row_bytes;
#pragma unroll
            for (int s = 0; s < SW; ++s) {
                const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                if (!FULL && j >= a.N) continue;                // no message bytes exist for these columns
                if constexpr (KIND == DS_COMP_IDENTITY) {       // the message is v itself
                    const float* vrow = reinterpret_cast<const float*>(nrow);
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float cv = (FULL || j + c < a.N) ? vrow[j + c] : 0.f;
                        acc[s][c] = fmaf(w, cv, acc[s][c]);
                    }
                    continue;
                }
                const uint64_t bcol0 = SUB ? col0 + (uint64_t)s * kSweep + (uint64_t)(lane / G) * B
                                           : col0 + (uint64_t)(s / SPB) * B;
                const uint8_t* blk = nrow + (bcol0 / B) * MSG_BLOCK_BYTES;
                const float scale = *reinterpret_cast<const float*>(blk);
                const int slot = SUB ? lane % G : (s % SPB) * kWave + lane;     // lane-slot inside the block
                if constexpr (KIND == DS_COMP_QUANT_MAXABS) {
                    using lane_t = typename CT::lane_t;
                    const float unit = scale / (float)L;
                    const uint32_t codes = reinterpret_cast<const lane_t*>(blk + 4)[slot];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int q = (int)((codes >> (BITS * c)) & (uint32_t)L);
                        float cv = (float)(2 * q - L) * unit;
                        if (!FULL && !(j + c < a.N)) cv = 0.f;
                        acc[s][c] = fmaf(w, cv, acc[s][c]);
                    }
                } else {
                    const uint32_t word = reinterpret_cast<const uint32_t*>(blk + 4)[slot >> 3];
                    const uint32_t nib = word >> (4 * (lane & 7));
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        float cv = ((nib >> c) & 1u) ? -scale : scale;
                        if (!FULL && !(j + c < a.N)) cv = 0.f;
                        acc[s][c] = fmaf(w, cv, acc[s][c]);
                    }
                }
            }
        }
#pragma unroll
        for (int s = 0; s < SW; ++s) {
            x[s].x = fmaf(a.eta, acc[s][0], x[s].x); x[s].y = fmaf(a.eta, acc[s][1], x[s].y);
            x[s].z = fmaf(a.eta, acc[s][2], x[s].z); x[s].w = fmaf(a.eta, acc[s][3], x[s].w);
            if (!FULL) {                                        // keep the pitch padding at zero
                const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                if (!(j + 0 < a.N)) x[s].x = 0.f;
                if (!(j + 1 < a.N)) x[s].y = 0.f;
                if (!(j + 2 < a.N)) x[s].z = 0.f;
                if (!(j + 3 < a.N)) x[s].w = 0.f;
            }
        }
    }

    // ---- lines 6-7 for blocks of 64 or 128 columns: G = B/4 lanes hold one block of a sweep --------
    // What a row keeps of an element after C[v] is known.  MODE 0, Algorithm 1 line 6: the residual v - C[v].
    // MODE 1 and 2 serve the comparison updates (dsq_compare_impl.h): `base` + C[v], where base is the worker's
    // public copy (MODE 1, the new copy also goes to LDS as fp32 for the gossip phase) or its model (MODE 2).
    template <int MODE>
    static __device__ __forceinline__ float kept(float vc, float cv, float base) {
        if constexpr (MODE == 0) return vc - cv;                     // line 6: delta = v - C[v]
        else return base + cv;
    }

    template <bool FULL, int MODE = 0>
    static __device__ __forceinline__ void compress_sub_blocks(const TileArgs& a, int i, int li, uint64_t col0, int lane, const float4 (&v)[SW],
                                                               const float4 (&base)[SW], uint8_t* msg_row, uint8_t* lds_row, float* lds_units, float* dout) {
        const int grp = lane / G, in_blk = lane % G;                  // block of the sweep, lane-slot inside the block
        [[maybe_unused]] uint32_t t_lo = 0;
        if constexpr (KIND == DS_COMP_QUANT_MAXABS) t_lo = (uint32_t)*a.t_ptr;
#pragma unroll
        for (int s = 0; s < SW; ++s) {
            const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
            const uint64_t bcol0 = col0 + (uint64_t)s * kSweep + (uint64_t)grp * B;
            const bool block_live = FULL || (bcol0 < a.N);
            const uint64_t m = FULL ? (uint64_t)B : (block_live ? (a.N - bcol0 < (uint64_t)B ? a.N - bcol0 : (uint64_t)B) : 0);
            const uint32_t nwords = (uint32_t)((m * BITS + 31) / 32);
            uint8_t* msg_blk = msg_row + (bcol0 / B) * MSG_BLOCK_BYTES;
            if constexpr (KIND == DS_COMP_QUANT_MAXABS) {
                const float mx = fmaxf(fmaxf(fabsf(v[s].x), fabsf(v[s].y)), fmaxf(fabsf(v[s].z), fabsf(v[s].w)));
                const float scale = group_max<G>(mx);
                const float hl = 0.5f * (float)L;
                const float unit = scale / (float)L;
                const float inv = (scale > 0.f) ? hl / scale : 0.f;
                if (in_blk == 0) {
                    if constexpr (MODE == 0) lds_units[li * BPT + s * BPS + grp] = unit;
                    if (block_live) *reinterpret_cast<float*>(msg_blk) = scale;
                }
                uint32_t rnd[4];
                philox4x32_10((uint32_t)(j >> 2), (uint32_t)i, t_lo, kQuantStreamTag, a.seed_lo, a.seed_hi, rnd);
                uint32_t codes = 0;
                float4 dnew;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float vc = comp(v[s], c);
                    float tt = fmaf(vc, inv, hl);
                    tt = (tt > 0.f) ? tt : 0.f;
                    tt = (tt < (float)L) ? tt : (float)L;
                    const float q0 = floorf(tt);
                    const float fr = tt - q0;
                    const float u = (float)(rnd[c] >> 8) * (1.0f / 16777216.0f);
                    int q = (int)q0 + ((u < fr) ? 1 : 0);
                    q = q < L ? q : L;
                    if (!(scale > 0.f)) q = 0;
                    float cv = (float)(2 * q - L) * unit;
                    if (!FULL && !(j + c < a.N)) { q = 0; cv = 0.f; }
                    codes |= (uint32_t)q << (BITS * c);
                    set_comp(dnew, c, kept<MODE>(vc, cv, comp(base[s], c)));
                }
                st4(dout + s * kSweep, dnew);
                using lane_t = typename CT::lane_t;
                if constexpr (MODE == 0) reinterpret_cast<lane_t*>(lds_row)[s * kWave + lane] = (lane_t)codes;
                if constexpr (MODE == 1) reinterpret_cast<float4*>(lds_row)[s * kWave + lane] = dnew;
                const uint32_t word = (uint32_t)in_blk * (uint32_t)sizeof(lane_t) / 4u;
                if (FULL || word < nwords) reinterpret_cast<lane_t*>(msg_blk + 4)[in_blk] = (lane_t)codes;
            } else if constexpr (KIND == DS_COMP_SIGN_MEANABS) {
                const float sum = group_sum_tree<G>((fabsf(v[s].x) + fabsf(v[s].y)) + (fabsf(v[s].z) + fabsf(v[s].w)));
                const float scale = block_live ? sum / (float)m : 0.f;
                if (in_blk == 0) {
                    if constexpr (MODE == 0) lds_units[li * BPT + s * BPS + grp] = scale;
                    if (block_live) *reinterpret_cast<float*>(msg_blk) = scale;
                }
                uint32_t nib = 0;
                float4 dnew;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float vc = comp(v[s], c);
                    uint32_t neg = __float_as_uint(vc) >> 31;
                    float cv = neg ? -scale : scale;
                    if (!FULL && !(j + c < a.N)) { neg = 0; cv = 0.f; }
                    nib |= neg << c;
                    set_comp(dnew, c, kept<MODE>(vc, cv, comp(base[s], c)));
                }
                st4(dout + s * kSweep, dnew);
                if constexpr (MODE == 1) reinterpret_cast<float4*>(lds_row)[s * kWave + lane] = dnew;
                uint32_t word = nib << (4 * (lane & 7));              // 8 lanes share one 32-bit word
                word |= __shfl_xor(word, 1);
                word |= __shfl_xor(word, 2);
                word |= __shfl_xor(word, 4);
                if ((lane & 7) == 0) {
                    if constexpr (MODE == 0) reinterpret_cast<uint32_t*>(lds_row)[s * 8 + (lane >> 3)] = word;
                    const uint32_t widx = (uint32_t)in_blk >> 3;
                    if (FULL || widx < nwords) reinterpret_cast<uint32_t*>(msg_blk + 4)[widx] = word;
                }
            }
        }
    }

    // ---- phase 1 for one row: returns xh (x - gamma g) in registers ---------------------------
    // `li` is the slot of the row in the LDS arrays (the row itself in the fused kernel).  TAIL: x holds the
    // previous step's x - gamma g and that step's gossip sum is still due (row-streaming variant).
    template <bool FULL, bool TAIL = false>
    static __device__ __forceinline__ void compress_row(const TileArgs& a, int i, int li, uint64_t col0, int lane,
                                                        uint8_t* lds_codes, float* lds_units, float4 (&xh)[SW]) {
        float4 xv[SW], gv[SW], dv[SW];
        const float* xr = a.x + (uint64_t)i * a.ld + col0 + 4 * lane;
        const float* dr = a.delta + (uint64_t)i * a.ld + col0 + 4 * lane;
        const float* gr = a.g + (uint64_t)i * a.g_ld + col0 + 4 * lane;
#pragma unroll
        for (int s = 0; s < SW; ++s) {
            xv[s] = ld4(xr + s * kSweep);
            dv[s] = ld4(dr + s * kSweep);
            if (FULL) {
                gv[s] = ld4(gr + s * kSweep);
            } else {
                const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                gv[s].x = (j + 0 < a.N) ? gr[s * kSweep + 0] : 0.f;
                gv[s].y = (j + 1 < a.N) ? gr[s * kSweep + 1] : 0.f;
                gv[s].z = (j + 2 < a.N) ? gr[s * kSweep + 2] : 0.f;
                gv[s].w = (j + 3 < a.N) ? gr[s * kSweep + 3] : 0.f;
            }
        }
        if constexpr (TAIL) {
            if (*a.pending != 0u) gossip_from_messages<FULL>(a, i, col0, lane, xv);
        }
        float4 v[SW];
#pragma unroll
        for (int s = 0; s < SW; ++s) {                      // Algorithm 1, line 5
            xh[s].x = fmaf(-a.gamma, gv[s].x, xv[s].x);  v[s].x = xh[s].x + dv[s].x;
            xh[s].y = fmaf(-a.gamma, gv[s].y, xv[s].y);  v[s].y = xh[s].y + dv[s].y;
            xh[s].z = fmaf(-a.gamma, gv[s].z, xv[s].z);  v[s].z = xh[s].z + dv[s].z;
            xh[s].w = fmaf(-a.gamma, gv[s].w, xv[s].w);  v[s].w = xh[s].w + dv[s].w;
        }

        uint8_t* lds_row = lds_codes + (size_t)li * ROW_CODE_BYTES;
        float* dout = a.delta + (uint64_t)i * a.ld + col0 + 4 * lane;
        encode_row<FULL, 0>(a, i, li, col0, lane, v, v, lds_row, lds_units, dout);
    }

    // ---- line 6 and line 7 for one row of a tile whose v is in registers: scales, codes, the packed message,
    //      and what the row keeps (see `kept`) stored through dout.  lds_row: the row's slot of the LDS exchange.
    template <bool FULL, int MODE>
    static __device__ __forceinline__ void encode_row(const TileArgs& a, int i, int li, uint64_t col0, int lane, const float4 (&v)[SW],
                                                      const float4 (&base)[SW], uint8_t* lds_row, float* lds_units, float* dout) {
        static_assert(MODE == 0 || KIND == DS_COMP_QUANT_MAXABS || KIND == DS_COMP_SIGN_MEANABS,
                      "the comparison updates are built for the block compressors");
        uint8_t* msg_row = a.msg + (uint64_t)i * a.msg_row_bytes;
        if constexpr (SUB) {
            compress_sub_blocks<FULL, MODE>(a, i, li, col0, lane, v, base, msg_row, lds_row, lds_units, dout);
            return;
        }
#pragma unroll
        for (int b = 0; b < (SUB ? 0 : BPT); ++b) {
            const uint64_t bcol0 = col0 + (uint64_t)b * B;            // first column of the block
            const bool block_live = FULL || (bcol0 < a.N);
            const uint64_t m = FULL ? (uint64_t)B : (block_live ? (a.N - bcol0 < (uint64_t)B ? a.N - bcol0 : (uint64_t)B) : 0);
            const uint32_t nwords = (uint32_t)((m * BITS + 31) / 32);
            uint8_t* msg_blk = msg_row + (bcol0 / B) * MSG_BLOCK_BYTES;

            if constexpr (KIND == DS_COMP_QUANT_MAXABS) {
                const uint32_t t_lo = (uint32_t)*a.t_ptr;            // step counter, low word (Philox counter word 2)
                float mx = 0.f;
#pragma unroll
                for (int s = b * SPB; s < (b + 1) * SPB; ++s)
                    mx = fmaxf(fmaxf(fmaxf(mx, fabsf(v[s].x)), fmaxf(fabsf(v[s].y), fabsf(v[s].z))), fabsf(v[s].w));
                const float scale = wave_max(mx);
                const float hl = 0.5f * (float)L;
                const float unit = scale / (float)L;
                const float inv = (scale > 0.f) ? hl / scale : 0.f;
                if (lane == 0) {
                    if constexpr (MODE == 0) lds_units[li * BPT + b] = unit;
                    if (block_live) *reinterpret_cast<float*>(msg_blk) = scale;
                }
#pragma unroll
                for (int s = b * SPB; s < (b + 1) * SPB; ++s) {
                    const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                    uint32_t rnd[4];
                    philox4x32_10((uint32_t)(j >> 2), (uint32_t)i, t_lo, kQuantStreamTag, a.seed_lo, a.seed_hi, rnd);
                    uint32_t codes = 0;
                    float4 dnew;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float vc = comp(v[s], c);
                        float tt = fmaf(vc, inv, hl);
                        tt = (tt > 0.f) ? tt : 0.f;
                        tt = (tt < (float)L) ? tt : (float)L;
                        const float q0 = floorf(tt);
                        const float fr = tt - q0;
                        const float u = (float)(rnd[c] >> 8) * (1.0f / 16777216.0f);
                        int q = (int)q0 + ((u < fr) ? 1 : 0);
                        q = q < L ? q : L;
                        if (!(scale > 0.f)) q = 0;
                        float cv = (float)(2 * q - L) * unit;
                        if (!FULL && !(j + c < a.N)) { q = 0; cv = 0.f; }
                        codes |= (uint32_t)q << (BITS * c);
                        set_comp(dnew, c, kept<MODE>(vc, cv, comp(base[s], c)));
                    }
                    st4(dout + s * kSweep, dnew);
                    using lane_t = typename CT::lane_t;
                    if constexpr (MODE == 0) reinterpret_cast<lane_t*>(lds_row)[s * kWave + lane] = (lane_t)codes;
                    if constexpr (MODE == 1) reinterpret_cast<float4*>(lds_row)[s * kWave + lane] = dnew;
                    const int in_blk = (s - b * SPB) * kWave + lane;  // lane-slot inside the block
                    const uint32_t word = (uint32_t)in_blk * (uint32_t)sizeof(lane_t) / 4u;
                    if (FULL || word < nwords)
                        reinterpret_cast<lane_t*>(msg_blk + 4)[in_blk] = (lane_t)codes;
                }
            } else if constexpr (KIND == DS_COMP_SIGN_MEANABS) {
                // balanced pairwise tree over the block: inside the lane, across lanes, across sweeps
                float part[SPB];
#pragma unroll
                for (int s = 0; s < SPB; ++s) {
                    const float4& q = v[b * SPB + s];
                    part[s] = wave_sum_tree((fabsf(q.x) + fabsf(q.y)) + (fabsf(q.z) + fabsf(q.w)));
                }
#pragma unroll
                for (int w = 1; w < SPB; w <<= 1)
#pragma unroll
                    for (int s = 0; s + w < SPB; s += 2 * w) part[s] = part[s] + part[s + w];
                const float scale = block_live ? part[0] / (float)m : 0.f;
                if (lane == 0) {
                    if constexpr (MODE == 0) lds_units[li * BPT + b] = scale;
                    if (block_live) *reinterpret_cast<float*>(msg_blk) = scale;
                }
#pragma unroll
                for (int s = b * SPB; s < (b + 1) * SPB; ++s) {
                    const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                    uint32_t nib = 0;
                    float4 dnew;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float vc = comp(v[s], c);
                        uint32_t neg = __float_as_uint(vc) >> 31;
                        float cv = neg ? -scale : scale;
                        if (!FULL && !(j + c < a.N)) { neg = 0; cv = 0.f; }
                        nib |= neg << c;
                        set_comp(dnew, c, kept<MODE>(vc, cv, comp(base[s], c)));
                    }
                    st4(dout + s * kSweep, dnew);
                    if constexpr (MODE == 1) reinterpret_cast<float4*>(lds_row)[s * kWave + lane] = dnew;
                    uint32_t word = nib << (4 * (lane & 7));          // 8 lanes share one 32-bit word
                    word |= __shfl_xor(word, 1);
                    word |= __shfl_xor(word, 2);
                    word |= __shfl_xor(word, 4);
                    if ((lane & 7) == 0) {
                        if constexpr (MODE == 0) reinterpret_cast<uint32_t*>(lds_row)[s * 8 + (lane >> 3)] = word;
                        const uint32_t widx = (uint32_t)(s - b * SPB) * 8u + (uint32_t)(lane >> 3);
                        if (FULL || widx < nwords) reinterpret_cast<uint32_t*>(msg_blk + 4)[widx] = word;
                    }
                }
            } else if constexpr (KIND == DS_COMP_RAND_SPARSE) {
                // C[v] = v on a random mask (kept iff the top 24 bits of the element's Philox word are below
                // the threshold), +0 elsewhere; the message is the kept values in column order, written at
                // the sweep's offset (counted beforehand from the same words) plus the rank inside the sweep.
                const uint32_t t_lo = (uint32_t)*a.t_ptr;
                float* vals = reinterpret_cast<float*>(msg_row + 4);
#pragma unroll
                for (int s = b * SPB; s < (b + 1) * SPB; ++s) {
                    const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                    uint32_t rnd[4];
                    philox4x32_10((uint32_t)(j >> 2), (uint32_t)i, t_lo, kSparseStreamTag, a.seed_lo, a.seed_hi, rnd);
                    uint32_t keep = 0;
                    float4 cv, dnew;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float vc = comp(v[s], c);
                        const bool k = ((rnd[c] >> 8) < a.keep_thr) && (FULL || j + c < a.N);
                        keep |= (k ? 1u : 0u) << c;
                        const float cc = k ? vc : 0.f;
                        set_comp(cv, c, cc);
                        set_comp(dnew, c, vc - cc);                  // line 6: delta = v - C[v]
                    }
                    st4(dout + s * kSweep, dnew);
                    reinterpret_cast<float4*>(lds_row)[s * kWave + lane] = cv;
                    const uint32_t mine = __popc(keep);
                    uint32_t inc = mine;                             // inclusive prefix over the lanes
#pragma unroll
                    for (int o = 1; o < kWave; o <<= 1) {
                        const uint32_t up = __shfl_up(inc, o);
                        if (lane >= o) inc += up;
                    }
                    const uint64_t sweep = (col0 >> 8) + (uint64_t)s;
                    // While the streams are in flight: how many elements of this sweep step t+1 will keep (its
                    // message offsets are needed before its tile kernel starts; counted here, the integer work
                    // hides behind the memory traffic instead of taking a pass of its own).
                    philox4x32_10((uint32_t)(j >> 2), (uint32_t)i, t_lo + 1u, kSparseStreamTag, a.seed_lo, a.seed_hi, rnd);
                    uint32_t next = 0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) next += (((rnd[c] >> 8) < a.keep_thr) && (FULL || j + c < a.N)) ? 1u : 0u;
#pragma unroll
                    for (int o = 1; o < kWave; o <<= 1) next += __shfl_xor(next, o);
                    if (lane == 0 && (FULL || sweep < a.nsweeps))
                        a.keep_raw[(uint64_t)((t_lo + 1u) & 1u) * a.n * a.nsweeps + (uint64_t)i * a.nsweeps + sweep] = next;
                    if (FULL || sweep < a.nsweeps) {
                        uint32_t pos = a.keep_group_off[(uint64_t)i * a.ngroups + (sweep >> 4)] +
                                       a.keep_off[(uint64_t)i * a.nsweeps + sweep] + inc - mine;
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (keep & (1u << c)) {
                                if (pos < a.msg_cap) vals[pos] = comp(v[s], c);
                                ++pos;
                            }
                    }
                }
            } else {   // DS_COMP_IDENTITY: C[v] = v, delta = 0, the message is v itself
#pragma unroll
                for (int s = b * SPB; s < (b + 1) * SPB; ++s) {
                    const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                    float4 dnew;
                    dnew.x = v[s].x - v[s].x; dnew.y = v[s].y - v[s].y; dnew.z = v[s].z - v[s].z; dnew.w = v[s].w - v[s].w;
                    st4(dout + s * kSweep, dnew);
                    reinterpret_cast<float4*>(lds_row)[s * kWave + lane] = v[s];
                    float* mrow = reinterpret_cast<float*>(msg_row);
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (FULL || j + c < a.N) mrow[j + c] = comp(v[s], c);
                }
            }
        }
    }

    // ---- phase 2 for one row: gossip on the decoded neighbours (Algorithm 1, line 9) ----------
    // acc[s][c] accumulates one neighbour after the other (CSR order), all sweeps at once, so the LDS
    // reads of one neighbour are in flight together.
    static __device__ __forceinline__ void gossip_accumulate(int nb, float w, int lane, const uint8_t* lds_codes,
                                                             const float* lds_units, float (&acc)[SW][4]) {
        const uint8_t* nrow = lds_codes + (size_t)nb * ROW_CODE_BYTES;
        if constexpr (KIND == DS_COMP_QUANT_MAXABS) {
            using lane_t = typename CT::lane_t;
            uint32_t codes[SW];
            float unit[SW];                                          // of the block this lane's columns are in
#pragma unroll
            for (int s = 0; s < SW; ++s) codes[s] = reinterpret_cast<const lane_t*>(nrow)[s * kWave + lane];
#pragma unroll
            for (int s = 0; s < SW; ++s) unit[s] = lds_units[nb * BPT + (SUB ? s * BPS + lane / G : s / SPB)];
#pragma unroll
            for (int s = 0; s < SW; ++s)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int q = (int)((codes[s] >> (BITS * c)) & (uint32_t)L);
                    acc[s][c] = fmaf(w, (float)(2 * q - L) * unit[s], acc[s][c]);
                }
        } else if constexpr (KIND == DS_COMP_SIGN_MEANABS) {
            uint32_t word[SW];
            float scale[SW];
#pragma unroll
            for (int s = 0; s < SW; ++s) word[s] = reinterpret_cast<const uint32_t*>(nrow)[s * 8 + (lane >> 3)];
#pragma unroll
            for (int s = 0; s < SW; ++s) scale[s] = lds_units[nb * BPT + (SUB ? s * BPS + lane / G : s / SPB)];
#pragma unroll
            for (int s = 0; s < SW; ++s) {
                const uint32_t nib = word[s] >> (4 * (lane & 7));
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    acc[s][c] = fmaf(w, ((nib >> c) & 1u) ? -scale[s] : scale[s], acc[s][c]);
            }
        } else {
#pragma unroll
            for (int s = 0; s < SW; ++s) {
                const float4 cv = reinterpret_cast<const float4*>(nrow)[s * kWave + lane];
                acc[s][0] = fmaf(w, cv.x, acc[s][0]); acc[s][1] = fmaf(w, cv.y, acc[s][1]);
                acc[s][2] = fmaf(w, cv.z, acc[s][2]); acc[s][3] = fmaf(w, cv.w, acc[s][3]);
            }
        }
    }

    template <bool FULL>
    static __device__ __forceinline__ void gossip_row(const TileArgs& a, int i, uint64_t col0, int lane,
                                                      const uint8_t* lds_codes, const float* lds_units,
                                                      const int32_t* lds_graph, const float4 (&xh)[SW]) {
        // the graph sits in LDS (copied at kernel start); row i is the same for the whole wave
        const int32_t* g_col = lds_graph + a.n + 1;
        const float* g_coef = reinterpret_cast<const float*>(g_col + a.nnz);
        const int e0 = __builtin_amdgcn_readfirstlane(lds_graph[i]);
        const int e1 = __builtin_amdgcn_readfirstlane(lds_graph[i + 1]);
        float acc[SW][4];
#pragma unroll
        for (int s = 0; s < SW; ++s) acc[s][0] = acc[s][1] = acc[s][2] = acc[s][3] = 0.f;
        auto edge = [&](int e) {
            const int nb = __builtin_amdgcn_readfirstlane(g_col[e]);
            const float w = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(g_coef[e])));
            gossip_accumulate(nb, w, lane, lds_codes, lds_units, acc);
        };
        const int deg = e1 - e0;
        if (deg == 3) {                                   // ring
            edge(e0); edge(e0 + 1); edge(e0 + 2);
        } else if (deg == 5) {                            // 2-D torus
            edge(e0); edge(e0 + 1); edge(e0 + 2); edge(e0 + 3); edge(e0 + 4);
        } else {
            for (int e = e0; e < e1; ++e) edge(e);
        }
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

    // Re-forms xh from x and g (used when a wave owns more rows than it can hold in registers).
    template <bool FULL>
    static __device__ __forceinline__ void reload_xh(const TileArgs& a, int i, uint64_t col0, int lane, float4 (&xh)[SW]) {
        const float* xr = a.x + (uint64_t)i * a.ld + col0 + 4 * lane;
        const float* gr = a.g + (uint64_t)i * a.g_ld + col0 + 4 * lane;
#pragma unroll
        for (int s = 0; s < SW; ++s) {
            const float4 xv = ld4(xr + s * kSweep);
            float4 gv;
            if (FULL) {
                gv = ld4(gr + s * kSweep);
            } else {
                const uint64_t j = col0 + (uint64_t)s * kSweep + 4 * lane;
                gv.x = (j + 0 < a.N) ? gr[s * kSweep + 0] : 0.f;
                gv.y = (j + 1 < a.N) ? gr[s * kSweep + 1] : 0.f;
                gv.z = (j + 2 < a.N) ? gr[s * kSweep + 2] : 0.f;
                gv.w = (j + 3 < a.N) ? gr[s * kSweep + 3] : 0.f;
            }
            xh[s].x = fmaf(-a.gamma, gv.x, xv.x); xh[s].y = fmaf(-a.gamma, gv.y, xv.y);
            xh[s].z = fmaf(-a.gamma, gv.z, xv.z); xh[s].w = fmaf(-a.gamma, gv.w, xv.w);
        }
    }

    template <int RPW, bool FULL>
    static __device__ __forceinline__ void run(const TileArgs& a, int rpw_runtime, uint64_t col0, uint8_t* lds) {
        const int lane = threadIdx.x & (kWave - 1);
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        uint8_t* lds_codes = lds;
        float* lds_units = reinterpret_cast<float*>(lds + (size_t)a.n * ROW_CODE_BYTES);
        int32_t* lds_graph = reinterpret_cast<int32_t*>(lds_units + (size_t)a.n * BPT);
        // W - I in CSR form (rowptr | col | coef, contiguous in device memory) -> LDS.  The loads are
        // issued first and parked in registers; the LDS writes come after phase 1, so their latency
        // hides behind the row streams.  Read only after the barrier.
        constexpr int GPRE = 2;
        const int gtotal = a.n + 1 + 2 * a.nnz;
        int32_t gpre[GPRE];
#pragma unroll
        for (int k = 0; k < GPRE; ++k) {
            const int q = threadIdx.x + k * NW * kWave;
            gpre[k] = (q < gtotal) ? a.rowptr[q] : 0;
        }
        auto park_graph = [&]() {
#pragma unroll
            for (int k = 0; k < GPRE; ++k) {
                const int q = threadIdx.x + k * NW * kWave;
                if (q < gtotal) lds_graph[q] = gpre[k];
            }
            for (int q = threadIdx.x + GPRE * NW * kWave; q < gtotal; q += NW * kWave) lds_graph[q] = a.rowptr[q];
        };
        if constexpr (RPW > 0) {
            float4 xh[RPW][SW];
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                const int i = wave + r * NW;
                if (i < a.n) compress_row<FULL>(a, i, i, col0, lane, lds_codes, lds_units, xh[r]);
            }
            park_graph();
            __syncthreads();
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                const int i = wave + r * NW;
                if (i < a.n) gossip_row<FULL>(a, i, col0, lane, lds_codes, lds_units, lds_graph, xh[r]);
            }
        } else {
            float4 xh[SW];
            for (int r = 0; r < rpw_runtime; ++r) {
                const int i = wave + r * NW;
                if (i < a.n) compress_row<FULL>(a, i, i, col0, lane, lds_codes, lds_units, xh);
            }
            park_graph();
            __syncthreads();
            for (int r = 0; r < rpw_runtime; ++r) {
                const int i = wave + r * NW;
                if (i < a.n) {
                    reload_xh<FULL>(a, i, col0, lane, xh);
                    gossip_row<FULL>(a, i, col0, lane, lds_codes, lds_units, lds_graph, xh);
                }
            }
        }
    }
};

// ---- random sparsifier: where each 256-column sweep's kept values go in the message -----------
// The mask depends on (seed, step, worker, column) only, so the number of kept elements of every
// sweep is known before the state is touched.  Normally the tile kernel of step t-1 has left the
// counts of step t in keep_raw[t & 1] (and t in the tag cell t_ptr[2]); this kernel recounts them
// when that is not so (first step, or the step counter was set from outside): one wave per sweep,
// no memory reads.
constexpr int kKeepGroup = 16;                                        // sweeps per offset group
__global__ void __launch_bounds__(256) keep_count_if_stale_kernel(TileArgs a) {
    const unsigned long long t = a.t_ptr[0];
    if (a.t_ptr[2] == t) return;                                      // uniform: the counts are there
    const int lane = threadIdx.x & (kWave - 1);
    const int i = blockIdx.y;
    uint32_t* raw = a.keep_raw + (uint64_t)(t & 1ull) * a.n * a.nsweeps + (uint64_t)i * a.nsweeps;
    for (uint64_t sweep = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6); sweep < a.nsweeps; sweep += (uint64_t)gridDim.x * 4) {
        const uint64_t j = sweep * kSweep + 4 * lane;
        uint32_t rnd[4];
        philox4x32_10((uint32_t)(j >> 2), (uint32_t)i, (uint32_t)t, kSparseStreamTag, a.seed_lo, a.seed_hi, rnd);
        uint32_t cnt = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) cnt += (((rnd[c] >> 8) < a.keep_thr) && (j + c < a.N)) ? 1u : 0u;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) cnt += __shfl_xor(cnt, o);
        if (lane == 0) raw[sweep] = cnt;
    }
}

// Counts of step t -> each sweep's offset inside its group of 16 sweeps, and the groups' totals.
__global__ void __launch_bounds__(256) keep_local_scan_kernel(TileArgs a, uint32_t* __restrict__ local_off, uint32_t* __restrict__ group_tot) {
    const unsigned long long t = a.t_ptr[0];
    const int i = blockIdx.y;
    const uint64_t sweep = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint32_t* raw = a.keep_raw + (uint64_t)(t & 1ull) * a.n * a.nsweeps + (uint64_t)i * a.nsweeps;
    const uint32_t cnt = (sweep < a.nsweeps) ? raw[sweep] : 0u;
    uint32_t inc = cnt;
    const int sub = threadIdx.x & (kKeepGroup - 1);
#pragma unroll
    for (int o = 1; o < kKeepGroup; o <<= 1) {
        const uint32_t up = __shfl_up(inc, o, kKeepGroup);
        if (sub >= o) inc += up;
    }
    if (sweep < a.nsweeps) local_off[(uint64_t)i * a.nsweeps + sweep] = inc - cnt;
    if (sub == kKeepGroup - 1 && (sweep >> 4) < a.ngroups) group_tot[(uint64_t)i * a.ngroups + (sweep >> 4)] = inc;
}

// Per row: group totals -> exclusive group offsets (in place), the count into the message header,
// stale values behind a shorter message cleared, and a flag if a row keeps more values than its
// message has room for.
__global__ void __launch_bounds__(1024) keep_scan_kernel(TileArgs a, uint32_t* __restrict__ group_tot, uint32_t* __restrict__ prev_count,
                                                         uint32_t* __restrict__ overflow) {
    __shared__ uint32_t wave_tot[16];
    const int i = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    uint32_t* row = group_tot + (uint64_t)i * a.ngroups;
    // each thread owns a run of consecutive groups
    const uint64_t per = (a.ngroups + 1023) / 1024;
    const uint64_t lo = (threadIdx.x * per < a.ngroups) ? threadIdx.x * per : a.ngroups;
    const uint64_t hi = (lo + per < a.ngroups) ? lo + per : a.ngroups;
    uint32_t sum = 0;
    for (uint64_t q = lo; q < hi; ++q) sum += row[q];
    uint32_t inc = sum;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t up = __shfl_up(inc, o);
        if (lane >= o) inc += up;
    }
    if (lane == kWave - 1) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        if (w < wave) base += wave_tot[w];
        total += wave_tot[w];
    }
    uint32_t run = base + inc - sum;
    for (uint64_t q = lo; q < hi; ++q) {
        const uint32_t c = row[q];
        row[q] = run;
        run += c;
    }
    // the message is zero behind its last value: clear what the previous step wrote beyond this step's count
    const uint32_t now = total < a.msg_cap ? total : a.msg_cap;
    const uint32_t before = prev_count[i];
    float* vals = reinterpret_cast<float*>(a.msg + (uint64_t)i * a.msg_row_bytes + 4);
    for (uint32_t q = now + threadIdx.x; q < before; q += 1024) vals[q] = 0.f;
    __syncthreads();
    if (threadIdx.x == 0) {
        *reinterpret_cast<uint32_t*>(a.msg + (uint64_t)i * a.msg_row_bytes) = now;
        prev_count[i] = now;
        if (total > a.msg_cap) atomicOr(overflow, 1u);
    }
}

template <int KIND, int BITS, int B, int SW, int NW, int RPW>
__global__ void __launch_bounds__(NW* kWave) fused_tile_kernel(TileArgs a, int rpw_runtime) {
    using T = Tile<KIND, BITS, B, SW, NW>;
    extern __shared__ __align__(16) uint8_t lds[];
    // tiles are numbered along x first; the grid has a second row only when x alone would pass the
    // 2^32 work-items a launch dimension can hold, and its last row may then have spare workgroups
    const uint64_t tile = (uint64_t)blockIdx.y * gridDim.x + blockIdx.x;
    const uint64_t col0 = tile * T::TC;
    if (col0 + T::TC <= a.N) T::template run<RPW, true>(a, rpw_runtime, col0, lds);
    else if (col0 < a.N)     T::template run<RPW, false>(a, rpw_runtime, col0, lds);
    // Advance the step counter once per launch: the workgroup that finds all others finished does it.
    // Thread 0 is past the barrier that follows phase 1, so every wave of its workgroup has read t (the
    // value has been consumed, so the load has completed) before the workgroup counts itself finished.
    // Two levels of counters, 64 cells a cache line or more apart and one on top, because returning
    // atomics on a single address serialise: with ~10^5 workgroups one shared counter doubled the
    // kernel time on MI355X, 64 cells cost < 0.5 %.  Relaxed atomics on purpose: a release fence
    // would write back the XCD's L2 once per workgroup; the end of the kernel publishes the new t.
    // All cells are zero again when the kernel ends.
    if (threadIdx.x == 0) {
        const unsigned long long blocks = (unsigned long long)gridDim.x * gridDim.y;
        const unsigned cell = (unsigned)(tile & 63u);
        const unsigned long long members = (blocks >> 6) + (cell < (blocks & 63u) ? 1u : 0u);
        unsigned long long* cnt = a.t_ptr + 32ull * (1 + cell);
        if (__hip_atomic_fetch_add(cnt, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == members - 1ull) {
            __hip_atomic_store(cnt, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned long long cells = blocks < 64u ? blocks : 64u;
            unsigned long long* done = a.t_ptr + 1;
            if (__hip_atomic_fetch_add(done, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == cells - 1ull) {
                __hip_atomic_store(done, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const unsigned long long t = __hip_atomic_fetch_add(a.t_ptr, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // random sparsifier: this launch has left the keep counts of step t+1 behind
                if constexpr (KIND == DS_COMP_RAND_SPARSE) __hip_atomic_store(a.t_ptr + 2, t + 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// ---- row-streaming variant: every wave takes one (row, tile) on its own ----------------------------
// Phase 1 of the fused kernel, preceded by the PREVIOUS step's line 9 decoded from that step's messages
// in HBM, and followed by the store of x - gamma g.  No barrier and no LDS exchange, so any number of
// workers fits; the price is reading (degree + 1) code streams per column (mostly cache hits) and a
// deferred gossip sum that readers of x must flush.
template <int KIND, int BITS, int B, int SW, int NW>
__device__ __forceinline__ void step_counter_bump(const TileArgs& a, unsigned long long linear_block, unsigned long long blocks, bool set_pending,
                                                  unsigned long long* also_clear = nullptr) {
    if (threadIdx.x == 0) {
        const unsigned cell = (unsigned)(linear_block & 63u);
        const unsigned long long members = (blocks >> 6) + (cell < (blocks & 63u) ? 1u : 0u);
        unsigned long long* cnt = a.t_ptr + 32ull * (1 + cell);
        if (__hip_atomic_fetch_add(cnt, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == members - 1ull) {
            __hip_atomic_store(cnt, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned long long cells = blocks < 64u ? blocks : 64u;
            unsigned long long* done = a.t_ptr + 1;
            if (__hip_atomic_fetch_add(done, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == cells - 1ull) {
                __hip_atomic_store(done, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const unsigned long long t = __hip_atomic_fetch_add(a.t_ptr, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // a cell the launch used as a work queue: every other workgroup has drawn its last number
                if (also_clear != nullptr) __hip_atomic_store(also_clear, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (set_pending) {
                    __hip_atomic_store(a.pending, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    // which of the two message buffers this step wrote (readers must not infer it from t: the
                    // counter can be set from outside)
                    __hip_atomic_store(a.t_ptr + 4, t & 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
}

template <int KIND, int BITS, int B, int SW, int NW, bool FLUSH>
__global__ void __launch_bounds__(NW* kWave) stream_tile_kernel(TileArgs a) {
    using T = Tile<KIND, BITS, B, SW, NW>;
    extern __shared__ __align__(16) uint8_t lds[];            // what phase 1 leaves for a gossip phase: unused here
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned long long t = a.t_ptr[0];
    a.msg_prev = a.msg + ((t & 1ull) ^ 1ull) * a.msg_half;    // in a flush t has advanced: the same half
    a.msg = a.msg + (t & 1ull) * a.msg_half;
    const uint64_t tile = (uint64_t)blockIdx.y * gridDim.x + blockIdx.x;
    const uint64_t col0 = tile * T::TC;
    const int row = blockIdx.z * NW + wave;
    if (row < a.n && col0 < a.N) {
        const bool full = col0 + T::TC <= a.N;
        float* xr = a.x + (uint64_t)row * a.ld + col0 + 4 * lane;
        float4 xh[SW];
        if constexpr (FLUSH) {
            if (*a.pending != 0u) {
#pragma unroll
                for (int s = 0; s < SW; ++s) xh[s] = ld4(xr + s * kSweep);
                if (full) T::template gossip_from_messages<true>(a, row, col0, lane, xh);
                else      T::template gossip_from_messages<false>(a, row, col0, lane, xh);
#pragma unroll
                for (int s = 0; s < SW; ++s) st4(xr + s * kSweep, xh[s]);
            }
        } else {
            uint8_t* lds_codes = lds;
            float* lds_units = reinterpret_cast<float*>(lds + (size_t)NW * T::ROW_CODE_BYTES);
            if (full) T::template compress_row<true, true>(a, row, wave, col0, lane, lds_codes, lds_units, xh);
            else      T::template compress_row<false, true>(a, row, wave, col0, lane, lds_codes, lds_units, xh);
#pragma unroll
            for (int s = 0; s < SW; ++s) st4(xr + s * kSweep, xh[s]);      // x - gamma g; padding columns come out as zero
        }
    }
    if constexpr (!FLUSH) {
        __syncthreads();                                      // every wave of the workgroup has read t and pending
        const unsigned long long blocks = (unsigned long long)gridDim.x * gridDim.y * gridDim.z;
        step_counter_bump<KIND, BITS, B, SW, NW>(a, ((unsigned long long)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x, blocks, true);
    }
}

__global__ void clear_pending_kernel(uint32_t* pending) { *pending = 0u; }

template <int KIND, int BITS, int B, int SW, int NW, bool FLUSH>
void launch_stream(const TileArgs& a, hipStream_t stream) {
    using T = Tile<KIND, BITS, B, SW, NW>;
    const uint64_t tiles = (a.N + T::TC - 1) / T::TC;
    const uint64_t max_x = 0xFFFFFFFFull / (NW * kWave);
    const unsigned gx = (unsigned)(tiles < max_x ? tiles : max_x);
    const unsigned gy = (unsigned)((tiles + gx - 1) / gx);
    const unsigned gz = (unsigned)((a.n + NW - 1) / NW);
    const size_t lds = FLUSH ? 0 : (size_t)NW * (T::ROW_CODE_BYTES + T::BPT * sizeof(float));
    hipLaunchKernelGGL((stream_tile_kernel<KIND, BITS, B, SW, NW, FLUSH>), dim3(gx, gy, gz), dim3(NW * kWave), lds, stream, a);
    if (FLUSH) hipLaunchKernelGGL(clear_pending_kernel, dim3(1), dim3(1), 0, stream, a.pending);
}

template <int KIND, int BITS, int B>
TilePlan make_stream_plan() {
    constexpr int SW = B <= kSweep ? 1 : B / kSweep, NW = 4;
    TilePlan p;
    p.name = "stream/4w";
    p.launch = [](const TileArgs& a, int, hipStream_t s) { launch_stream<KIND, BITS, B, SW, NW, false>(a, s); };
    p.flush = [](const TileArgs& a, hipStream_t s) { launch_stream<KIND, BITS, B, SW, NW, true>(a, s); };
    p.tile_cols = SW * kSweep;
    p.waves = NW;
    p.rows_per_wave = 1;
    p.sweeps = SW;
    p.streaming = true;
    return p;
}

template <int KIND, int BITS>
bool stream_plan_for_block(int block, TilePlan& plan) {
    switch (block) {
        case 64:   plan = make_stream_plan<KIND, BITS, 64>(); return true;
        case 128:  plan = make_stream_plan<KIND, BITS, 128>(); return true;
        case 256:  plan = make_stream_plan<KIND, BITS, 256>(); return true;
        case 512:  plan = make_stream_plan<KIND, BITS, 512>(); return true;
        case 1024: plan = make_stream_plan<KIND, BITS, 1024>(); return true;
        case 2048: plan = make_stream_plan<KIND, BITS, 2048>(); return true;
        default: return false;
    }
}

template <int KIND, int BITS, int B, int SW, int NW, int RPW>
void launch_tile(const TileArgs& a, int rpw_runtime, hipStream_t stream) {
    using T = Tile<KIND, BITS, B, SW, NW>;
    const uint64_t tiles = (a.N + T::TC - 1) / T::TC;
    // a launch dimension holds fewer than 2^32 work-items: very long vectors get a second grid row
    const uint64_t max_x = 0xFFFFFFFFull / (NW * kWave);
    const unsigned gx = (unsigned)(tiles < max_x ? tiles : max_x);
    const unsigned gy = (unsigned)((tiles + gx - 1) / gx);
    const size_t lds = T::lds_bytes(a.n, a.nnz);
    auto kern = fused_tile_kernel<KIND, BITS, B, SW, NW, RPW>;
    // more than the default dynamic LDS has to be asked for once per kernel and device (handles are
    // bound to one device, but a process may hold handles on several)
    static unsigned long long attr_devices = 0;
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

template <int KIND, int BITS, int B, int SW, int NW, int RPW>
TilePlan make_plan(const char* name) {
    TilePlan p;
    p.name = name;
    p.launch = &launch_tile<KIND, BITS, B, SW, NW, RPW>;
    p.tile_cols = SW * kSweep;
    p.waves = NW;
    p.rows_per_wave = RPW;
    p.sweeps = SW;
    return p;
}

constexpr size_t kMaxLds = 160 * 1024;

// Variant table for one (KIND, BITS, B): every launch shape that fits n, best guess first.
// Measured on MI355X: 8-wave workgroups whose waves each own several rows usually beat 16-wave
// ones (two or more workgroups then share a CU and one's gossip phase overlaps the other's loads),
// but the order changes with the shape and from GPU to GPU, so ds_init times the candidates.
// A wave keeps xh for all its rows in registers, so rows-per-wave * sweeps is capped.
template <int KIND, int BITS, int B, int SW, int NW, int RPW>
void add_plan(int n, const char* name, std::vector<TilePlan>& plans) {
    if constexpr (RPW * SW <= (NW > 8 ? 8 : 16) && (NW <= 8 || SW <= 4)) {   // else the 128-VGPR cap of a 16-wave group spills
        if (n > NW * RPW) return;
        if (RPW > 1 && n <= NW * (RPW / 2)) return;            // a smaller RPW already covers n
        plans.push_back(make_plan<KIND, BITS, B, SW, NW, RPW>(name));
    }
}

template <int KIND, int BITS, int B, int SW>
void add_plans_for_sweeps(int n, std::vector<TilePlan>& plans) {
    add_plan<KIND, BITS, B, SW, 8, 1>(n, "tile/8w/1row", plans);
    add_plan<KIND, BITS, B, SW, 8, 2>(n, "tile/8w/2rows", plans);
    add_plan<KIND, BITS, B, SW, 8, 4>(n, "tile/8w/4rows", plans);
    add_plan<KIND, BITS, B, SW, 8, 8>(n, "tile/8w/8rows", plans);
    add_plan<KIND, BITS, B, SW, 16, 1>(n, "tile/16w/1row", plans);
    add_plan<KIND, BITS, B, SW, 16, 2>(n, "tile/16w/2rows", plans);
    add_plan<KIND, BITS, B, SW, 16, 4>(n, "tile/16w/4rows", plans);
    add_plan<KIND, BITS, B, SW, 4, 2>(n, "tile/4w/2rows", plans);
    add_plan<KIND, BITS, B, SW, 4, 4>(n, "tile/4w/4rows", plans);
}

template <int KIND, int BITS, int B>
bool pick_for_block(int n, int nnz, std::vector<TilePlan>& plans, std::string& err) {
    constexpr int SW = (B <= kSweep) ? 1 : (B / kSweep);
    using T8 = Tile<KIND, BITS, B, (B <= kSweep) ? 2 : SW, 8>;
    if (T8::lds_bytes(n, nnz) > kMaxLds) {
        err = "n is too large for the fused tile kernel: the codes of all n rows of one tile must fit in 160 KB of LDS";
        return false;
    }
    add_plans_for_sweeps<KIND, BITS, B, SW>(n, plans);
    if constexpr (B <= kSweep) {
        // 256-column blocks: also try two blocks per tile
        std::vector<TilePlan> two;
        add_plans_for_sweeps<KIND, BITS, B, 2>(n, two);
        for (TilePlan& p : two) plans.push_back(p);
    }
    if (plans.empty()) {
        TilePlan plan;
        if constexpr (SW >= 8) {
            plan = make_plan<KIND, BITS, B, SW, 8, 0>("tile/8w/looped");
            plan.rows_per_wave = (n + 7) / 8;
        } else {
            plan = make_plan<KIND, BITS, B, SW, 16, 0>("tile/16w/looped");
            plan.rows_per_wave = (n + 15) / 16;
        }
        plans.push_back(plan);
    }
    return true;
}

template <int KIND, int BITS>
bool pick_for_kind(int block, int n, int nnz, std::vector<TilePlan>& plan, std::string& err) {
    switch (block) {
        case 64:   return pick_for_block<KIND, BITS, 64>(n, nnz, plan, err);
        case 128:  return pick_for_block<KIND, BITS, 128>(n, nnz, plan, err);
        case 256:  return pick_for_block<KIND, BITS, 256>(n, nnz, plan, err);
        case 512:  return pick_for_block<KIND, BITS, 512>(n, nnz, plan, err);
        case 1024: return pick_for_block<KIND, BITS, 1024>(n, nnz, plan, err);
        case 2048: return pick_for_block<KIND, BITS, 2048>(n, nnz, plan, err);
        default: err = "block must be a power of two between 64 and 2048"; return false;
    }
}

}  // namespace
}  // namespace dsq

// Host-only part of libdsq: configuration checks, the mixing matrix W of the built-in
// topologies, and message sizes.  No GPU call in this file.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>

#include "dsq_internal.h"

namespace dsq {

static bool is_pow2(uint64_t v) { return v && !(v & (v - 1)); }

ds_status validate_config(const ds_config* cfg, std::string& err, std::string* warn) {
    if (!cfg) { err = "config is NULL"; return DS_EINVAL; }
    if (cfg->n < 1) { err = "n must be >= 1"; return DS_EINVAL; }
    if (cfg->N < 1) { err = "N must be >= 1"; return DS_EINVAL; }
    if (cfg->N > 0xFFFFFFF0ull) { err = "N must fit 32-bit indices"; return DS_EINVAL; }
    if (!std::isfinite(cfg->gamma) || !std::isfinite(cfg->eta)) { err = "gamma and eta must be finite"; return DS_EINVAL; }
    switch (cfg->topo) {
        case DS_TOPO_RING:
            if (cfg->n < 3) { err = "a ring needs n >= 3 (else the two neighbours coincide)"; return DS_EINVAL; }
            if (cfg->W_rowptr || cfg->W_col || cfg->W_val) { err = "W must be NULL for DS_TOPO_RING"; return DS_EINVAL; }
            break;
        case DS_TOPO_TORUS2D:
            if (cfg->torus_rows < 3 || cfg->torus_cols < 3) { err = "torus sides must be >= 3"; return DS_EINVAL; }
            if ((int64_t)cfg->torus_rows * cfg->torus_cols != cfg->n) { err = "torus_rows * torus_cols must equal n"; return DS_EINVAL; }
            if (cfg->W_rowptr || cfg->W_col || cfg->W_val) { err = "W must be NULL for DS_TOPO_TORUS2D"; return DS_EINVAL; }
            break;
        case DS_TOPO_CSR: {
            if (!cfg->W_rowptr || !cfg->W_col || !cfg->W_val) { err = "DS_TOPO_CSR needs W_rowptr, W_col and W_val"; return DS_EINVAL; }
            const int n = cfg->n;
            if (cfg->W_rowptr[0] != 0) { err = "W_rowptr[0] must be 0"; return DS_EINVAL; }
            std::map<std::pair<int, int>, float> entries;
            for (int i = 0; i < n; ++i) {
                if (cfg->W_rowptr[i + 1] < cfg->W_rowptr[i]) { err = "W_rowptr must be non-decreasing"; return DS_EINVAL; }
                bool diag = false;
                double sum = 0.0;
                for (int e = cfg->W_rowptr[i]; e < cfg->W_rowptr[i + 1]; ++e) {
                    const int j = cfg->W_col[e];
                    if (j < 0 || j >= n) { err = "W_col entry out of range"; return DS_EINVAL; }
                    if (e > cfg->W_rowptr[i] && j <= cfg->W_col[e - 1]) { err = "columns of a W row must be strictly ascending"; return DS_EINVAL; }
                    const float w = cfg->W_val[e];
                    if (!(w >= 0.f) || !std::isfinite(w)) { err = "W entries must be finite and >= 0"; return DS_EINVAL; }
                    diag |= (j == i);
                    sum += w;
                    entries[{i, j}] = w;
                }
                if (!diag) { err = "every W row must store its diagonal entry"; return DS_EINVAL; }
                if (std::fabs(sum - 1.0) > 1e-6) { err = "rows of W must sum to 1 (doubly stochastic)"; return DS_EINVAL; }
            }
            for (const auto& kv : entries) {
                auto it = entries.find({kv.first.second, kv.first.first});
                const float wt = (it == entries.end()) ? 0.f : it->second;
                if (std::fabs(wt - kv.second) > 1e-6f) { err = "W must be symmetric"; return DS_EINVAL; }
            }
            break;
        }
        default: err = "unknown topology"; return DS_EINVAL;
    }
    const ds_comp& c = cfg->comp;
    switch (c.kind) {
        case DS_COMP_IDENTITY: break;
        case DS_COMP_QUANT_MAXABS:
            if (c.bits != 2 && c.bits != 4 && c.bits != 8) { err = "bits must be 2, 4 or 8"; return DS_EINVAL; }
            [[fallthrough]];
        case DS_COMP_SIGN_MEANABS:
            if (c.block < kMinBlock || c.block > kMaxBlock || !is_pow2((uint64_t)c.block)) {
                err = "block must be a power of two between 64 and 2048"; return DS_EINVAL;
            }
            break;
        case DS_COMP_TOPK:
            if (c.k < 1 || c.k > cfg->N) { err = "k must be in [1, N]"; return DS_EINVAL; }
            break;
        case DS_COMP_QUANT_L2NORM:
            if (c.bits != 2 && c.bits != 4 && c.bits != 8) { err = "bits must be 2, 4 or 8"; return DS_EINVAL; }
            break;
        case DS_COMP_RAND_SPARSE:
        case DS_COMP_GSPAR:
            if (c.k < 1 || c.k > cfg->N) { err = "k (expected number of kept elements) must be in [1, N]"; return DS_EINVAL; }
            break;
        default: err = "unknown compressor"; return DS_EINVAL;
    }
    if (cfg->algo != DS_ALGO_DEEPSQUEEZE) {
        if (cfg->algo != DS_ALGO_DCD_PSGD && cfg->algo != DS_ALGO_CHOCO_SGD) { err = "unknown update rule (algo)"; return DS_EINVAL; }
        if (c.kind != DS_COMP_QUANT_MAXABS && c.kind != DS_COMP_SIGN_MEANABS) {
            err = "DCD-PSGD and CHOCO-SGD are built for DS_COMP_QUANT_MAXABS and DS_COMP_SIGN_MEANABS only"; return DS_EINVAL;
        }
    }
    if (cfg->reserved != 0) { err = "reserved must be 0"; return DS_EINVAL; }
    if (warn && cfg->eta > 0.5f) *warn = "warning: eta > 1/2, outside the range of the paper's Theorem 1 (W_eff may not be PSD)";
    return DS_OK;
}

ds_status build_graph(const ds_config* cfg, Graph& g, std::string& err) {
    const int n = cfg->n;
    g.rowptr.assign(1, 0);
    g.col.clear(); g.w.clear(); g.coef.clear();
    auto push_row = [&](std::map<int, float>& row) {
        for (auto& kv : row) { g.col.push_back(kv.first); g.w.push_back(kv.second); }
        g.rowptr.push_back((int32_t)g.col.size());
    };
    if (cfg->topo == DS_TOPO_RING) {
        if (n < 3) { err = "a ring needs n >= 3"; return DS_EINVAL; }
        const float w = 1.0f / 3.0f;
        for (int i = 0; i < n; ++i) {
            std::map<int, float> row{{i, w}, {(i + 1) % n, w}, {(i + n - 1) % n, w}};
            push_row(row);
        }
    } else if (cfg->topo == DS_TOPO_TORUS2D) {
        const int R = cfg->torus_rows, C = cfg->torus_cols;
        if (R < 3 || C < 3 || (int64_t)R * C != n) { err = "bad torus shape"; return DS_EINVAL; }
        const float w = 1.0f / 5.0f;
        for (int r = 0; r < R; ++r)
            for (int c = 0; c < C; ++c) {
                std::map<int, float> row{{r * C + c, w},
                                         {((r + 1) % R) * C + c, w}, {((r + R - 1) % R) * C + c, w},
                                         {r * C + (c + 1) % C, w}, {r * C + (c + C - 1) % C, w}};
                push_row(row);
            }
    } else if (cfg->topo == DS_TOPO_CSR) {
        g.rowptr.assign(cfg->W_rowptr, cfg->W_rowptr + n + 1);
        g.col.assign(cfg->W_col, cfg->W_col + g.rowptr[n]);
        g.w.assign(cfg->W_val, cfg->W_val + g.rowptr[n]);
    } else {
        err = "unknown topology";
        return DS_EINVAL;
    }
    g.coef.resize(g.w.size());
    g.max_degree = 0;
    for (int i = 0; i < n; ++i) {
        g.max_degree = std::max(g.max_degree, g.rowptr[i + 1] - g.rowptr[i]);
        for (int e = g.rowptr[i]; e < g.rowptr[i + 1]; ++e)
            g.coef[e] = (g.col[e] == i) ? (g.w[e] - 1.0f) : g.w[e];       // W_ij - I_ij, formed once in fp32
    }
    return DS_OK;
}

// Values a worker's random-sparsification message has room for: the expected count k, eight standard deviations
// of the kept count on top (its variance is below k), and a small constant for tiny k; never more than N.
uint64_t rand_sparse_capacity(uint64_t N, uint64_t k) {
    uint64_t r = (uint64_t)std::sqrt((double)k);          // near floor(sqrt k); the two loops make it exact
    while (r * r > k) --r;
    while ((r + 1) * (r + 1) <= k) ++r;
    const uint64_t sigma_bound = (r * r == k) ? r : r + 1; // ceil(sqrt k)
    return std::min<uint64_t>(N, k + 8 * sigma_bound + 64);
}

uint64_t message_row_bytes(const ds_config* cfg) {
    const ds_comp& c = cfg->comp;
    switch (c.kind) {
        case DS_COMP_IDENTITY: return cfg->N * 4;
        case DS_COMP_TOPK: return c.k * 8;
        case DS_COMP_QUANT_L2NORM: return 4 + 4 * ((cfg->N * (uint64_t)c.bits + 31) / 32);
        case DS_COMP_RAND_SPARSE: return 4 + 4 * rand_sparse_capacity(cfg->N, c.k);
        case DS_COMP_GSPAR: return 8 + 8 * rand_sparse_capacity(cfg->N, c.k);
        case DS_COMP_QUANT_MAXABS:
        case DS_COMP_SIGN_MEANABS: {
            const uint64_t b = (c.kind == DS_COMP_QUANT_MAXABS) ? (uint64_t)c.bits : 1;
            const uint64_t B = (uint64_t)c.block;
            const uint64_t full = cfg->N / B, tail = cfg->N % B;
            uint64_t bytes = full * (4 + 4 * ((B * b + 31) / 32));
            if (tail) bytes += 4 + 4 * ((tail * b + 31) / 32);
            return bytes;
        }
        default: return 0;
    }
}

}  // namespace dsq

extern "C" {

ds_status ds_validate_config(const ds_config* cfg, char* errbuf, uint64_t errbuf_len) {
    std::string err;
    const ds_status st = dsq::validate_config(cfg, err, nullptr);
    if (errbuf && errbuf_len) {
        std::snprintf(errbuf, (size_t)errbuf_len, "%s", err.c_str());
    }
    return st;
}

ds_status ds_build_topology(const ds_config* cfg, int32_t* rowptr, int32_t* col, float* val, uint64_t cap, uint64_t* nnz) {
    if (!cfg || !rowptr || !col || !val) return DS_EINVAL;
    std::string err;
    if (dsq::validate_config(cfg, err, nullptr) != DS_OK) return DS_EINVAL;
    dsq::Graph g;
    if (dsq::build_graph(cfg, g, err) != DS_OK) return DS_EINVAL;
    if (nnz) *nnz = g.col.size();
    if (g.col.size() > cap) return DS_EINVAL;
    std::memcpy(rowptr, g.rowptr.data(), g.rowptr.size() * sizeof(int32_t));
    std::memcpy(col, g.col.data(), g.col.size() * sizeof(int32_t));
    std::memcpy(val, g.w.data(), g.w.size() * sizeof(float));
    return DS_OK;
}

#ifndef DSQ_BUILD_ID
#define DSQ_BUILD_ID "unknown"
#endif
const char* ds_build_id(void) { return DSQ_BUILD_ID; }

uint64_t ds_message_bytes(const ds_config* cfg) {
    std::string err;
    if (dsq::validate_config(cfg, err, nullptr) != DS_OK) return 0;
    return dsq::message_row_bytes(cfg) * (uint64_t)cfg->n;
}

}  // extern "C"

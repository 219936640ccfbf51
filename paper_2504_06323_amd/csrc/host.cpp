// Host-only entry points: version, status names, workspace sizes and the
// projection planner (Algorithm 1's normalize(R_LLM) plus the Projection
// Planner of Section 3.3).  Nothing here touches a device.
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "mosaic_prune.h"

namespace mp {
size_t colsum_workspace_bytes(int64_t n_rows, int64_t n_cols);
size_t score_workspace_bytes(int64_t rows, int64_t cols);
size_t select_workspace_bytes(int64_t rows, int64_t cols);
size_t struct_workspace_bytes(int64_t inter, int64_t hidden);
size_t rank_batch_workspace_bytes();
}  // namespace mp

extern "C" int prune_version(void) { return 100; }

extern "C" const char *prune_status_string(int status) {
    switch (status) {
        case PRUNE_OK: return "ok";
        case PRUNE_ERR_NULL: return "null pointer";
        case PRUNE_ERR_SHAPE: return "bad shape";
        case PRUNE_ERR_DTYPE: return "bad dtype";
        case PRUNE_ERR_ALIGNMENT: return "bad alignment";
        case PRUNE_ERR_WORKSPACE: return "workspace too small";
        case PRUNE_ERR_RANGE: return "argument out of range";
        case PRUNE_ERR_DEVICE: return "device launch failed";
        default: return "unknown status";
    }
}

extern "C" size_t prune_workspace_bytes(int op, int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0) return 0;
    size_t n = 0;
    switch (op) {
        case PRUNE_OP_STATS: n = mp::colsum_workspace_bytes(rows, cols); break;
        case PRUNE_OP_SCORE: n = mp::score_workspace_bytes(rows, cols); break;
        case PRUNE_OP_OUTLIER: return 0;
        case PRUNE_OP_SELECT: n = mp::select_workspace_bytes(rows, cols); break;
        case PRUNE_OP_STRUCT: n = mp::struct_workspace_bytes(rows, cols); break;
        case PRUNE_OP_BATCH: n = mp::rank_batch_workspace_bytes(); break;
        default: return 0;
    }
    return (n + 255) / 256 * 256;
}

namespace {

// s = p + 2 * lambda * (mean(r_hat) - r_hat) over the entries idx[0..n)
void spread(const std::vector<double> &ratio, const std::vector<int> &idx, double p, double lambda, double *out) {
    double lo = ratio[idx[0]], hi = ratio[idx[0]];
    for (int i : idx) {
        lo = fmin(lo, ratio[i]);
        hi = fmax(hi, ratio[i]);
    }
    if (hi == lo) {
        for (int i : idx) out[i] = p;
        return;
    }
    double mean_hat = 0.0;
    for (int i : idx) mean_hat += (ratio[i] - lo) / (hi - lo);
    mean_hat /= static_cast<double>(idx.size());
    for (int i : idx) out[i] = p + 2.0 * lambda * (mean_hat - (ratio[i] - lo) / (hi - lo));
}

}  // namespace

extern "C" int prune_plan_sparsity(const unsigned long long *counts, const unsigned long long *numels,
                                   const int64_t *cols, int n_layers, int n_proj, double p, double lambda, int scope,
                                   double *sparsity_out, uint32_t *zeros_per_row_out, int *clamped_out) {
    if (!counts || !numels || !sparsity_out || (zeros_per_row_out && !cols)) return PRUNE_ERR_NULL;
    if (n_layers <= 0 || n_proj <= 0) return PRUNE_ERR_SHAPE;
    if (!(p >= 0.0 && p < 1.0) || !(lambda >= 0.0)) return PRUNE_ERR_RANGE;
    if (scope != PRUNE_SCOPE_GLOBAL && scope != PRUNE_SCOPE_CATEGORY && scope != PRUNE_SCOPE_LAYER) return PRUNE_ERR_RANGE;
    const int n = n_layers * n_proj;
    std::vector<double> ratio(n);
    for (int i = 0; i < n; ++i) {
        if (numels[i] == 0 || counts[i] > numels[i]) return PRUNE_ERR_RANGE;
        ratio[i] = 100.0 * static_cast<double>(counts[i]) / static_cast<double>(numels[i]);  // R = O / C * 100
    }
    std::vector<int> idx;
    if (scope == PRUNE_SCOPE_GLOBAL) {
        for (int i = 0; i < n; ++i) idx.push_back(i);
        spread(ratio, idx, p, lambda, sparsity_out);
    } else if (scope == PRUNE_SCOPE_CATEGORY) {
        for (int m = 0; m < n_proj; ++m) {
            idx.clear();
            for (int l = 0; l < n_layers; ++l) idx.push_back(l * n_proj + m);
            spread(ratio, idx, p, lambda, sparsity_out);
        }
    } else {
        // one ratio per layer from the layer's pooled counts, held in the slot of its first projection, spread over
        // the layers, then handed to the layer's other projections
        for (int l = 0; l < n_layers; ++l) {
            unsigned long long c = 0, e = 0;
            for (int m = 0; m < n_proj; ++m) {
                c += counts[l * n_proj + m];
                e += numels[l * n_proj + m];
            }
            ratio[l * n_proj] = 100.0 * static_cast<double>(c) / static_cast<double>(e);
            idx.push_back(l * n_proj);
        }
        spread(ratio, idx, p, lambda, sparsity_out);
        for (int i = 0; i < n; ++i) sparsity_out[i] = sparsity_out[i - i % n_proj];
    }
    int clamped = 0;
    if (cols) {
        for (int i = 0; i < n; ++i) {
            if (cols[i] <= 0) return PRUNE_ERR_SHAPE;
            const double hi = 1.0 - 1.0 / static_cast<double>(cols[i]);
            double s = sparsity_out[i];
            if (s < 0.0) s = 0.0;
            if (s > hi) s = hi;
            if (s != sparsity_out[i]) clamped = 1;
            sparsity_out[i] = s;
            if (zeros_per_row_out) zeros_per_row_out[i] = static_cast<uint32_t>(floor(s * static_cast<double>(cols[i])));
        }
    }
    if (clamped_out) *clamped_out = clamped;
    return PRUNE_OK;
}

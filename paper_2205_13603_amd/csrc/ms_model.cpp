// Learned cost model for the search (Section 4 of arXiv 2205.13603, "End-to-end search": the
// evolutionary search proposes many candidates, a cost model trained on the measurements so far
// predicts their running time, and only the most promising ones are measured).
//
// The model is least-squares gradient boosting of small regression trees with exact greedy
// splits (Friedman's algorithm; the paper's implementation uses a tree-boosting library).  It is
// deterministic: rows are visited in a fixed order, sums are accumulated sequentially in double,
// a split must improve on the best so far by a strict inequality, and candidate thresholds are
// the midpoints between consecutive distinct values of a feature.
//
// Features of a variant: what the trace interpreter derived (tile factors, workgroup shape, LDS
// and register footprints, staging and vectorisation decisions), mostly as log2.
// Host only.
#include "ms_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <vector>

using namespace ms;

struct ms_cost_model {
    int32_t n_trees, depth, min_leaf;
    double lr;
    int32_t d = 0;       // features the model was fitted on
    double base = 0;     // mean of the targets
    struct Node {
        int32_t feature; // -1 = leaf
        double threshold;
        int32_t left, right;
        double value;
    };
    std::vector<std::vector<Node>> trees;
};

namespace {

struct Builder {
    const double *X;
    int32_t n, d, max_depth, min_leaf;
    const std::vector<double> *r; // residuals
    std::vector<ms_cost_model::Node> nodes;

    int32_t build(std::vector<int32_t> &rows, int32_t depth)
    {
        ms_cost_model::Node node;
        node.feature = -1;
        node.threshold = 0;
        node.left = node.right = -1;
        double sum = 0;
        for (int32_t i : rows) sum += (*r)[(size_t)i];
        const double cnt = (double)rows.size();
        node.value = sum / cnt;
        int32_t id = (int32_t)nodes.size();
        nodes.push_back(node);
        if (depth >= max_depth || (int32_t)rows.size() < 2 * min_leaf) return id;
        // best split: maximise S_L^2 / n_L + S_R^2 / n_R - S^2 / n
        double best_gain = 0;
        int32_t best_f = -1;
        double best_thr = 0;
        std::vector<int32_t> order(rows.size());
        for (int32_t f = 0; f < d; ++f) {
            order = rows;
            std::stable_sort(order.begin(), order.end(),
                             [&](int32_t a, int32_t b) { return X[(size_t)a * d + f] < X[(size_t)b * d + f]; });
            double sl = 0;
            for (size_t k = 0; k + 1 < order.size(); ++k) {
                sl += (*r)[(size_t)order[k]];
                const double xa = X[(size_t)order[k] * d + f], xb = X[(size_t)order[k + 1] * d + f];
                if (!(xa < xb)) continue; // split only between distinct values
                const int32_t nl = (int32_t)k + 1, nr = (int32_t)order.size() - nl;
                if (nl < min_leaf || nr < min_leaf) continue;
                const double sr = sum - sl;
                const double gain = sl * sl / (double)nl + sr * sr / (double)nr - sum * sum / cnt;
                if (gain > best_gain) {
                    best_gain = gain;
                    best_f = f;
                    best_thr = 0.5 * (xa + xb);
                }
            }
        }
        if (best_f < 0) return id;
        std::vector<int32_t> L, R;
        for (int32_t i : rows) (X[(size_t)i * d + best_f] < best_thr ? L : R).push_back(i);
        if (L.empty() || R.empty()) return id; // a midpoint that rounds onto one of its neighbours
        nodes[(size_t)id].feature = best_f;
        nodes[(size_t)id].threshold = best_thr;
        const int32_t l = build(L, depth + 1);
        nodes[(size_t)id].left = l;
        const int32_t rr = build(R, depth + 1);
        nodes[(size_t)id].right = rr;
        return id;
    }
};

double tree_predict(const std::vector<ms_cost_model::Node> &t, const double *x)
{
    int32_t i = 0;
    while (t[(size_t)i].feature >= 0) i = x[t[(size_t)i].feature] < t[(size_t)i].threshold ? t[(size_t)i].left : t[(size_t)i].right;
    return t[(size_t)i].value;
}

double lg(double v) { return std::log2(v < 1 ? 1.0 : v); }

} // namespace

extern "C" int32_t ms_cost_model_create(int32_t n_trees, int32_t depth, double learning_rate, int32_t min_leaf, ms_cost_model **out)
{
    if (!out) return fail(MS_ERR_BAD_ARG, "ms_cost_model_create: NULL argument");
    *out = nullptr;
    if (n_trees < 0 || n_trees > 4096 || depth < 1 || depth > 12 || !(learning_rate > 0) || learning_rate > 1 || min_leaf < 1)
        return fail(MS_ERR_BAD_ARG, "ms_cost_model_create: bad hyper-parameters");
    ms_cost_model *m = new (std::nothrow) ms_cost_model();
    if (!m) return fail(MS_ERR_NOMEM, "ms_cost_model_create: out of memory");
    m->n_trees = n_trees;
    m->depth = depth;
    m->lr = learning_rate;
    m->min_leaf = min_leaf;
    *out = m;
    return MS_OK;
}

extern "C" void ms_cost_model_destroy(ms_cost_model *m) { delete m; }

extern "C" int32_t ms_cost_model_fit(ms_cost_model *m, const double *X, const double *y, int32_t n, int32_t d)
{
    if (!m || !X || !y) return fail(MS_ERR_BAD_ARG, "ms_cost_model_fit: NULL argument");
    if (n < 1 || d < 1 || d > 1024) return fail(MS_ERR_BAD_ARG, "ms_cost_model_fit: n = %d, d = %d", n, d);
    for (int64_t i = 0; i < (int64_t)n * d; ++i)
        if (!std::isfinite(X[i])) return fail(MS_ERR_BAD_ARG, "ms_cost_model_fit: feature %lld is not finite", (long long)i);
    double sum = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (!std::isfinite(y[i])) return fail(MS_ERR_BAD_ARG, "ms_cost_model_fit: target %d is not finite", i);
        sum += y[i];
    }
    m->d = d;
    m->base = sum / n;
    m->trees.clear();
    std::vector<double> F((size_t)n, m->base), r((size_t)n);
    std::vector<int32_t> rows((size_t)n);
    for (int32_t t = 0; t < m->n_trees; ++t) {
        for (int32_t i = 0; i < n; ++i) r[(size_t)i] = y[i] - F[(size_t)i];
        std::iota(rows.begin(), rows.end(), 0);
        Builder b;
        b.X = X;
        b.n = n;
        b.d = d;
        b.max_depth = m->depth;
        b.min_leaf = m->min_leaf;
        b.r = &r;
        std::vector<int32_t> all = rows;
        b.build(all, 0);
        for (int32_t i = 0; i < n; ++i) F[(size_t)i] += m->lr * tree_predict(b.nodes, X + (size_t)i * d);
        m->trees.push_back(std::move(b.nodes));
    }
    return MS_OK;
}

extern "C" int32_t ms_cost_model_predict(const ms_cost_model *m, const double *X, int32_t n, int32_t d, double *out)
{
    if (!m || !X || !out) return fail(MS_ERR_BAD_ARG, "ms_cost_model_predict: NULL argument");
    if (m->d == 0) return fail(MS_ERR_BAD_ARG, "ms_cost_model_predict: the model has not been fitted");
    if (n < 0 || d != m->d) return fail(MS_ERR_BAD_ARG, "ms_cost_model_predict: %d features, the model was fitted on %d", d, m->d);
    for (int32_t i = 0; i < n; ++i) {
        double f = m->base;
        for (auto &t : m->trees) f += m->lr * tree_predict(t, X + (size_t)i * d);
        out[i] = f;
    }
    return MS_OK;
}

extern "C" int32_t ms_variant_features(const ms_op *op, const ms_variant_params *p, double *out, int32_t cap, int32_t *n_out)
{
    if (!op || !p || !n_out) return fail(MS_ERR_BAD_ARG, "ms_variant_features: NULL argument");
    std::vector<double> f;
    const int32_t *tl[4] = {p->ti, p->tj, p->tc, p->tk};
    for (int l = 0; l < 4; ++l)
        for (int k = 0; k < 4; ++k) f.push_back(lg((double)tl[l][k]));
    f.push_back((double)(p->mfma ? p->tile_unit[0] : 0)); // intrinsic rows (0 = vector ALU)
    f.push_back((double)(p->mfma ? p->tile_unit[2] : 0)); // intrinsic k
    f.push_back(lg((double)p->block_m));
    f.push_back(lg((double)p->block_n));
    f.push_back(lg((double)p->block_k));
    f.push_back(lg((double)p->threads));
    f.push_back((double)p->waves);
    f.push_back(lg((double)p->acc_per_thread));
    f.push_back(lg((double)p->lds_bytes + 1));
    f.push_back(lg((double)p->grid[0] * p->grid[1] * p->grid[2]));
    f.push_back((double)p->cache_read);
    f.push_back(lg((double)p->vec));
    f.push_back(lg((double)p->vec_b));
    f.push_back(lg((double)p->unroll + 1));
    f.push_back(lg((double)p->unroll_k1));
    f.push_back(lg((double)p->unroll_k2));
    f.push_back((double)p->lds_pad);
    f.push_back((double)p->reorder);
    f.push_back((double)p->cache_write);
    f.push_back((double)p->compute_at);
    f.push_back(lg((double)std::max(1, p->rfactor)));
    // derived: register tile of one thread / wavefront, operand traffic per multiply-accumulate of a workgroup tile
    const double rm = (double)std::max(1, p->ti[1]) * std::max(1, p->ti[3]) * std::max(1, p->tile_unit[0]);
    const double rn = (double)std::max(1, p->tj[1]) * std::max(1, p->tj[3]) * std::max(1, p->tile_unit[1]);
    f.push_back(lg(rm));
    f.push_back(lg(rn));
    f.push_back(1.0 / rm + 1.0 / rn);
    f.push_back(1.0 / std::max(1, p->block_m) + 1.0 / std::max(1, p->block_n));
    *n_out = (int32_t)f.size();
    if (out) {
        if (cap < (int32_t)f.size()) return fail(MS_ERR_BAD_ARG, "ms_variant_features: room for %d values, %d needed", cap, (int)f.size());
        memcpy(out, f.data(), f.size() * sizeof(double));
    }
    return MS_OK;
}

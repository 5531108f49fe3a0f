// Boosted-tree predictor of MTNN (Section IV): the runtime evaluator used by Algorithm 2 and
// the offline trainer that turns a table of (m, n, k, label) into a model.
//
// The paper trains CART regression trees under gradient boosting with a library and fixes only
// four settings (depth <= 8, 8 estimators, eta = 1, gamma = 0).  This trainer follows that
// library's documented defaults for the rest: binary logistic objective on y = [label == +1],
// initial margin 0, second-order (gradient / hessian) leaf values -G/(H + lambda) and split gain
// 1/2 [G_L^2/(H_L+lambda) + G_R^2/(H_R+lambda) - G^2/(H+lambda)] - gamma, exact greedy search
// over thresholds halfway between distinct neighbouring feature values, no subsampling.
#include "../../include/mtnn.h"
#include "selector.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <atomic>
#include <mutex>
#include <string>

namespace mtnn {

void selector_features(int m, int n, int k, double* x)
{
    const double dm = m, dn = n, dk = k;
    x[0] = dm;
    x[1] = dn;
    x[2] = dk;
    x[3] = dn * dk;        // elements of B: what the transpose moves
    x[4] = dm * dn;        // elements of C
    x[5] = dm * dk;        // elements of A
    x[6] = dm * dn * dk;   // multiply-adds
}

double model_margin(const Model& model, const double* x)
{
    double margin = 0.0;
    for (const auto& tree : model.trees) {
        int at = 0;
        while (tree[at].feature >= 0)
            at = (x[tree[at].feature] < tree[at].threshold) ? tree[at].left : tree[at].right;
        margin += tree[at].value;
    }
    return margin;
}

namespace {

struct Split {
    bool found = false;
    double gain = 0.0;
    int feature = -1;
    double threshold = 0.0;
};

struct Trainer {
    int nrows, nfeat;
    const double* X;
    TrainParams tp;
    std::vector<double> g, h;

    double at(int row, int f) const { return X[(size_t)row * nfeat + f]; }
    double score(double G, double H) const { return G * G / (H + tp.lambda); }

    // samples arrive in increasing row order and every sum below runs in a fixed order, so a
    // model is a pure function of the table
    Split best_split(const std::vector<int>& rows) const
    {
        double G = 0.0, H = 0.0;
        for (int r : rows) { G += g[r]; H += h[r]; }
        const double parent = score(G, H);
        Split best;
        std::vector<int> order(rows);
        for (int f = 0; f < nfeat; ++f) {
            order = rows;
            std::sort(order.begin(), order.end(), [&](int a, int b) {
                const double va = at(a, f), vb = at(b, f);
                return va < vb || (va == vb && a < b);
            });
            double GL = 0.0, HL = 0.0;
            for (size_t pos = 0; pos + 1 < order.size(); ++pos) {
                const int r = order[pos];
                GL += g[r];
                HL += h[r];
                const double v = at(r, f), vnext = at(order[pos + 1], f);
                if (v == vnext) continue;
                const double GR = G - GL, HR = H - HL;
                if (HL < tp.min_child_weight || HR < tp.min_child_weight) continue;
                const double gain = 0.5 * (score(GL, HL) + score(GR, HR) - parent) - tp.gamma;
                // strict improvement only: equal gains keep the lowest feature, then threshold
                if (gain > 0.0 && (!best.found || gain > best.gain)) {
                    best.found = true;
                    best.gain = gain;
                    best.feature = f;
                    best.threshold = 0.5 * (v + vnext);
                }
            }
        }
        return best;
    }

    int grow(std::vector<TreeNode>& tree, const std::vector<int>& rows, int depth) const
    {
        const int me = (int)tree.size();
        tree.push_back(TreeNode{-1, 0.0, -1, -1, 0.0});
        Split sp;
        if (depth < tp.max_depth) sp = best_split(rows);
        if (!sp.found) {
            double G = 0.0, H = 0.0;
            for (int r : rows) { G += g[r]; H += h[r]; }
            tree[me].value = -G / (H + tp.lambda) * tp.eta;
            return me;
        }
        std::vector<int> lrows, rrows;
        for (int r : rows) (at(r, sp.feature) < sp.threshold ? lrows : rrows).push_back(r);
        tree[me].feature = sp.feature;
        tree[me].threshold = sp.threshold;
        const int l = grow(tree, lrows, depth + 1);
        const int r = grow(tree, rrows, depth + 1);
        tree[me].left = l;
        tree[me].right = r;
        return me;
    }
};

double tree_value(const std::vector<TreeNode>& tree, const double* x)
{
    int at = 0;
    while (tree[at].feature >= 0)
        at = (x[tree[at].feature] < tree[at].threshold) ? tree[at].left : tree[at].right;
    return tree[at].value;
}

}  // namespace

Model train_gbdt(int nrows, int nfeat, const double* X, const int* labels, const TrainParams& tp)
{
    Trainer tr;
    tr.nrows = nrows;
    tr.nfeat = nfeat;
    tr.X = X;
    tr.tp = tp;
    tr.g.assign(nrows, 0.0);
    tr.h.assign(nrows, 0.0);
    std::vector<double> margin(nrows, 0.0);
    std::vector<int> all(nrows);
    for (int i = 0; i < nrows; ++i) all[i] = i;

    Model model;
    model.num_features = nfeat;
    for (int round = 0; round < tp.num_trees; ++round) {
        for (int i = 0; i < nrows; ++i) {
            const double p = 1.0 / (1.0 + std::exp(-margin[i]));
            const double y = labels[i] == 1 ? 1.0 : 0.0;
            tr.g[i] = p - y;
            tr.h[i] = p * (1.0 - p);
        }
        std::vector<TreeNode> tree;
        tr.grow(tree, all, 0);
        for (int i = 0; i < nrows; ++i) margin[i] += tree_value(tree, X + (size_t)i * nfeat);
        model.trees.push_back(std::move(tree));
    }
    return model;
}

// ---- model files: a small text format, doubles written as C99 hex floats so they round-trip

bool save_model(const Model& model, const char* path)
{
    FILE* f = std::fopen(path, "w");
    if (!f) return false;
    std::fprintf(f, "mtnn-gbdt 1\nfeatures %d\ntrees %d\n", model.num_features, (int)model.trees.size());
    for (size_t t = 0; t < model.trees.size(); ++t) {
        std::fprintf(f, "tree %d nodes %d\n", (int)t, (int)model.trees[t].size());
        for (const TreeNode& nd : model.trees[t])
            std::fprintf(f, "%d %a %d %d %a\n", nd.feature, nd.threshold, nd.left, nd.right, nd.value);
    }
    const bool ok = std::ferror(f) == 0;
    return std::fclose(f) == 0 && ok;
}

bool load_model(const char* path, Model& out)
{
    FILE* f = std::fopen(path, "r");
    if (!f) return false;
    Model m;
    int version = 0, ntrees = 0;
    bool ok = std::fscanf(f, " mtnn-gbdt %d features %d trees %d", &version, &m.num_features, &ntrees) == 3 &&
              version == 1 && m.num_features > 0 && m.num_features <= 64 && ntrees >= 0 && ntrees <= 1024;
    for (int t = 0; ok && t < ntrees; ++t) {
        int id = -1, nnodes = 0;
        ok = std::fscanf(f, " tree %d nodes %d", &id, &nnodes) == 2 && id == t && nnodes >= 1 && nnodes <= (1 << 20);
        std::vector<TreeNode> tree;
        for (int i = 0; ok && i < nnodes; ++i) {
            TreeNode nd;
            char thr[64], val[64];
            ok = std::fscanf(f, " %d %63s %d %d %63s", &nd.feature, thr, &nd.left, &nd.right, val) == 5;
            if (!ok) break;
            char* end = nullptr;
            nd.threshold = std::strtod(thr, &end);
            ok = end && *end == '\0';
            nd.value = std::strtod(val, &end);
            ok = ok && end && *end == '\0';
            tree.push_back(nd);
        }
        // structure check: children in range and strictly after their parent (so every walk ends)
        for (int i = 0; ok && i < (int)tree.size(); ++i) {
            const TreeNode& nd = tree[i];
            if (nd.feature < 0) continue;
            ok = nd.feature < m.num_features && nd.left > i && nd.right > i &&
                 nd.left < (int)tree.size() && nd.right < (int)tree.size() && std::isfinite(nd.threshold);
        }
        if (ok) m.trees.push_back(std::move(tree));
    }
    std::fclose(f);
    if (ok) out = std::move(m);
    return ok;
}

// ---- the current predictor -----------------------------------------------------------------------

namespace {
std::mutex g_model_mutex;
std::shared_ptr<const Model> g_model;   // null = no model: always NT
// Counts every change of the current predictor.  Memoised answers carry the count they were made
// under: an address would not do, since a new model can be allocated where a freed one was.
std::atomic<unsigned long long> g_model_generation{1};

// first use: a model named by the environment variable MTNN_MODEL is loaded if nothing else has
// been installed; a missing or malformed file leaves "always NT" in place
std::once_flag g_env_once;
void load_from_env()
{
    const char* path = std::getenv("MTNN_MODEL");
    if (!path || !*path) return;
    Model m;
    if (!load_model(path, m)) return;
    auto p = std::make_shared<const Model>(std::move(m));
    std::lock_guard<std::mutex> lock(g_model_mutex);
    if (!g_model) {
        g_model = std::move(p);
        g_model_generation.fetch_add(1, std::memory_order_release);
    }
}

std::shared_ptr<const Model> current()
{
    std::call_once(g_env_once, load_from_env);
    std::lock_guard<std::mutex> lock(g_model_mutex);
    return g_model;
}
void install(Model&& m)
{
    auto p = std::make_shared<const Model>(std::move(m));
    std::lock_guard<std::mutex> lock(g_model_mutex);
    g_model = std::move(p);
    g_model_generation.fetch_add(1, std::memory_order_release);
}
}  // namespace

}  // namespace mtnn

extern "C" {

int mtnn_num_features(void) { return mtnn::kSelectorFeatures; }

int mtnn_features(int m, int n, int k, double* x)
{
    if (!x) return MTNN_ERR_NULL;
    if (m <= 0 || n <= 0 || k <= 0) return MTNN_ERR_DIM;
    mtnn::selector_features(m, n, k, x);
    return MTNN_OK;
}

int mtnn_select(int m, int n, int k)
{
    if (m <= 0 || n <= 0 || k <= 0) return 0;
    // a one-entry memo: training loops repeat the same few shapes, and the hit path is four compares.
    // The generation is read before the model: an answer stored under an older count than the model
    // it was computed from is at worst recomputed, never served for a newer model.
    struct Memo { int m, n, k, label; unsigned long long generation; };
    static thread_local Memo memo = {0, 0, 0, 0, 0};
    std::call_once(mtnn::g_env_once, mtnn::load_from_env);
    const unsigned long long gen = mtnn::g_model_generation.load(std::memory_order_acquire);
    if (memo.generation == gen && memo.m == m && memo.n == n && memo.k == k) return memo.label;
    auto model = mtnn::current();
    if (!model || model->num_features != mtnn::kSelectorFeatures) return 1;
    double x[mtnn::kSelectorFeatures];
    mtnn::selector_features(m, n, k, x);
    const int label = mtnn::model_margin(*model, x) >= 0.0 ? 1 : -1;
    memo = Memo{m, n, k, label, gen};
    return label;
}

int mtnn_select_batch(int count, const int* mnk, int* labels)
{
    if (count < 0) return MTNN_ERR_DIM;
    if (count == 0) return MTNN_OK;
    if (!mnk || !labels) return MTNN_ERR_NULL;
    auto model = mtnn::current();
    const bool usable = model && model->num_features == mtnn::kSelectorFeatures;
    for (int i = 0; i < count; ++i) {
        const int m = mnk[3 * i], n = mnk[3 * i + 1], k = mnk[3 * i + 2];
        if (m <= 0 || n <= 0 || k <= 0) { labels[i] = 0; continue; }
        if (!usable) { labels[i] = 1; continue; }
        double x[mtnn::kSelectorFeatures];
        mtnn::selector_features(m, n, k, x);
        labels[i] = mtnn::model_margin(*model, x) >= 0.0 ? 1 : -1;
    }
    return MTNN_OK;
}

int mtnn_load_model(const char* path)
{
    if (!path) return MTNN_ERR_NULL;
    mtnn::Model m;
    if (!mtnn::load_model(path, m)) return MTNN_ERR_MODEL;
    mtnn::install(std::move(m));
    return MTNN_OK;
}

int mtnn_save_model(const char* path)
{
    if (!path) return MTNN_ERR_NULL;
    auto model = mtnn::current();
    if (!model) return MTNN_ERR_MODEL;
    return mtnn::save_model(*model, path) ? MTNN_OK : MTNN_ERR_MODEL;
}

void mtnn_unload_model(void)
{
    std::lock_guard<std::mutex> lock(mtnn::g_model_mutex);
    mtnn::g_model.reset();
    mtnn::g_model_generation.fetch_add(1, std::memory_order_release);
}

int mtnn_gbdt_train(int nrows, int nfeat, const double* X, const int* labels, int num_trees, int max_depth,
                    double eta, double gamma, double lambda, double min_child_weight)
{
    if (nrows <= 0 || nfeat <= 0 || nfeat > 64 || num_trees < 0 || num_trees > 1024 || max_depth < 0 || max_depth > 30)
        return MTNN_ERR_ARG;
    if (!X || !labels) return MTNN_ERR_NULL;
    for (int i = 0; i < nrows; ++i)
        if (labels[i] != 1 && labels[i] != -1) return MTNN_ERR_ARG;
    for (size_t i = 0; i < (size_t)nrows * nfeat; ++i)
        if (!std::isfinite(X[i])) return MTNN_ERR_ARG;
    mtnn::TrainParams tp;
    tp.num_trees = num_trees;
    tp.max_depth = max_depth;
    tp.eta = eta;
    tp.gamma = gamma;
    tp.lambda = lambda;
    tp.min_child_weight = min_child_weight;
    mtnn::install(mtnn::train_gbdt(nrows, nfeat, X, labels, tp));
    return MTNN_OK;
}

int mtnn_train_selector(int nrows, const int* mnk, const int* labels)
{
    if (nrows <= 0) return MTNN_ERR_ARG;
    if (!mnk || !labels) return MTNN_ERR_NULL;
    std::vector<double> X((size_t)nrows * mtnn::kSelectorFeatures);
    for (int i = 0; i < nrows; ++i) {
        if (mnk[3 * i] <= 0 || mnk[3 * i + 1] <= 0 || mnk[3 * i + 2] <= 0) return MTNN_ERR_DIM;
        mtnn::selector_features(mnk[3 * i], mnk[3 * i + 1], mnk[3 * i + 2], &X[(size_t)i * mtnn::kSelectorFeatures]);
    }
    const mtnn::TrainParams tp;   // the paper's configuration
    return mtnn_gbdt_train(nrows, mtnn::kSelectorFeatures, X.data(), labels, tp.num_trees, tp.max_depth, tp.eta,
                           tp.gamma, tp.lambda, tp.min_child_weight);
}

int mtnn_model_num_trees(void)
{
    auto m = mtnn::current();
    return m ? (int)m->trees.size() : 0;
}

int mtnn_model_num_features(void)
{
    auto m = mtnn::current();
    return m ? m->num_features : 0;
}

int mtnn_model_tree_size(int tree)
{
    auto m = mtnn::current();
    if (!m || tree < 0 || tree >= (int)m->trees.size()) return -1;
    return (int)m->trees[tree].size();
}

int mtnn_model_node(int tree, int idx, int* feature, double* threshold, int* left, int* right, double* value)
{
    auto m = mtnn::current();
    if (!m || tree < 0 || tree >= (int)m->trees.size()) return MTNN_ERR_ARG;
    if (idx < 0 || idx >= (int)m->trees[tree].size()) return MTNN_ERR_ARG;
    const mtnn::TreeNode& nd = m->trees[tree][idx];
    if (feature) *feature = nd.feature;
    if (threshold) *threshold = nd.threshold;
    if (left) *left = nd.left;
    if (right) *right = nd.right;
    if (value) *value = nd.value;
    return MTNN_OK;
}

int mtnn_model_margin(const double* x, int nfeat, double* margin)
{
    if (!x || !margin) return MTNN_ERR_NULL;
    auto m = mtnn::current();
    if (!m || nfeat != m->num_features) return MTNN_ERR_MODEL;
    *margin = mtnn::model_margin(*m, x);
    return MTNN_OK;
}

}  // extern "C"

// Boosted-tree predictor of MTNN (Section IV of the paper): model storage, evaluation,
// training and the text format of model files.  Host-only code.
#pragma once
#include <vector>

namespace mtnn {

constexpr int kSelectorFeatures = 7;

struct TreeNode {
    int feature;        // -1 for a leaf
    double threshold;   // x[feature] < threshold goes left
    int left, right;    // indices in the tree's node array (pre-order)
    double value;       // leaf value (already scaled by eta)
};

struct Model {
    int num_features = 0;
    std::vector<std::vector<TreeNode>> trees;
};

struct TrainParams {
    int num_trees = 8;             // Section IV-B: 8 estimators
    int max_depth = 8;             //               depth at most 8
    double eta = 1.0;              //               step size shrinkage 1
    double gamma = 0.0;            //               minimum loss reduction 0
    double lambda = 1.0;           // leaf L2 penalty (library default; the paper is silent)
    double min_child_weight = 1.0; // minimum hessian weight of a child (library default)
};

void selector_features(int m, int n, int k, double* x);
double model_margin(const Model& model, const double* x);
Model train_gbdt(int nrows, int nfeat, const double* X, const int* labels, const TrainParams& tp);
bool save_model(const Model& model, const char* path);
bool load_model(const char* path, Model& out);

}  // namespace mtnn

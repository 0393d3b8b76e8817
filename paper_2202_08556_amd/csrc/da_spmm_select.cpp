// da_spmm_select: data-aware choice among the 8 algorithms (paper Sec. 5.1).  The paper trains a
// gradient-boosted tree classifier on input characteristics (Table 2); here the trained trees are
// compiled into the library as tables and walked on the host.  Pure function, no device work.
#include "da_spmm.h"

#include <cmath>

namespace {

struct SelNode {
    int feature;      // index into the feature vector, < 0 for a leaf
    double threshold; // go left when x[feature] <= threshold
    int left;         // child index, or row of kLeafScores for a leaf
    int right;
};

#include "selector_model.inc"

constexpr int kNumSelFeatures = 7;

inline double lg(double x) { return std::log2(x < 1.0 ? 1.0 : x); }

}  // namespace

extern "C" int da_spmm_select(const da_features* f)
{
    if (!f) return -DA_ERR_INVALID_ARG;
    if (f->rows < 0 || f->nnz < 0 || f->N < 0) return -DA_ERR_INVALID_ARG;
    if (!(f->row_nnz_mean >= 0.0) || !(f->row_nnz_std >= 0.0) || !(f->row_nnz_max >= 0.0))
        return -DA_ERR_INVALID_ARG;                      // also rejects NaN
    if (std::isinf(f->row_nnz_mean) || std::isinf(f->row_nnz_std) || std::isinf(f->row_nnz_max))
        return -DA_ERR_INVALID_ARG;
    // feature vector: sizes on a log scale, dispersion as coefficient of variation
    const double mean = f->row_nnz_mean;
    double x[kNumSelFeatures];
    x[0] = lg((double)f->rows);
    x[1] = lg((double)f->nnz);
    x[2] = std::log2(mean + 1.0);
    x[3] = mean > 0.0 ? f->row_nnz_std / mean : 0.0;
    x[4] = std::log2(f->row_nnz_max + 1.0);
    x[5] = lg((double)f->N);
    x[6] = mean > 0.0 ? std::log2(f->row_nnz_max / mean + 1.0) : 0.0;

    double score[DA_NUM_ALGOS] = {0};
    for (int t = 0; t < kNumTrees; ++t) {
        int i = kTreeRoot[t];
        while (kNodes[i].feature >= 0)
            i = (x[kNodes[i].feature] <= kNodes[i].threshold) ? kNodes[i].left : kNodes[i].right;
        const float* leaf = kLeafScores[kNodes[i].left];
        for (int a = 0; a < DA_NUM_ALGOS; ++a) score[a] += (double)leaf[a];
    }
    int best = 0;
    for (int a = 1; a < DA_NUM_ALGOS; ++a)
        if (score[a] > score[best]) best = a;
    return best;
}

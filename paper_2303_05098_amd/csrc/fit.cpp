// Offline training stage on the host: CART trees and random forests over the ten features (Section V; the
// hyper-parameters are those of Table III: estimators, bootstrap, max depth, min samples per leaf, min samples
// before a split, max features per split, criterion).
//
// Fixed choices (the paper names scikit-learn's classifiers and gives no listing):
//   * every random number is hash(seed, stream, index), a counter-based 64-bit mixer, so a forest is a pure function
//     of (data, options) and trees can be fitted in any order;
//   * tree t with bootstrap trains on n draws with replacement, row = hash(seed, 2t, i) mod n;
//   * nodes are numbered depth first, left before right, so a child always follows its parent in the arrays;
//   * with max_features < 10 the features of a node are tried in a random order (Fisher-Yates driven by
//     hash(seed, 2t+1, 16*node + k)) until max_features were tried and an admissible cut is known;
//   * a cut lies between two distinct neighbouring values a < b with at least min_samples_leaf rows on each side;
//     threshold = (a + b) / 2 (or a, should that round up to b); rows with value <= threshold go left;
//   * gini costs are compared as exact fractions in 128-bit integers, entropy costs as doubles summed in class order;
//     equal costs: lower feature index, then lower threshold;
//   * a leaf predicts its most frequent class, ties to the lowest id.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <memory>
#include <new>
#include <utility>
#include <vector>

#include "mo.h"
#include "model.hpp"

namespace {

constexpr int F = MO_NUM_FEATURES;
constexpr int NC = MO_NUM_FORMATS;
constexpr int64_t kMaxSamples = 1 << 20;   // keeps the 128-bit cross products of the gini comparison exact

inline uint64_t mix(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

inline uint64_t hash3(uint64_t seed, uint64_t stream, uint64_t idx)
{
    const uint64_t key = mix(mix(seed) ^ stream);
    return mix(mix(idx ^ key));
}

// Cost of a cut as a fraction num / den (den > 0); smaller is better.  Entropy uses dnum with den = 1.
struct Cost {
    __int128 num = 0, den = 1;
    double dnum = 0.0;
    bool exact = true;
};

inline bool less(const Cost &a, const Cost &b) { return a.exact ? a.num * b.den < b.num * a.den : a.dnum < b.dnum; }

struct Cut {
    Cost cost;
    int feature = -1;
    double threshold = 0.0;
    bool valid = false;
};

inline bool better(const Cut &a, const Cut &b)
{
    if (less(a.cost, b.cost)) return true;
    if (less(b.cost, a.cost)) return false;
    if (a.feature != b.feature) return a.feature < b.feature;
    return a.threshold < b.threshold;
}

inline double entropy_cost(const int64_t *c)
{
    int64_t tot = 0;
    for (int k = 0; k < NC; ++k) tot += c[k];
    double e = 0.0;
    for (int k = 0; k < NC; ++k)
        if (c[k] > 0) e += (double)c[k] * (std::log((double)tot) - std::log((double)c[k]));
    return e;
}

struct Trainer {
    const double *X;
    const int32_t *y;
    int64_t n;
    mo_fit_opts o;
    std::vector<int32_t> rows, tmp;                       // sample of the current tree, partitioned in place
    std::vector<std::pair<double, int32_t>> sorted;       // (value, class) of one node and one feature

    Cut best_cut(int64_t lo, int64_t hi, int f)
    {
        const int64_t nn = hi - lo;
        sorted.resize((size_t)nn);
        int64_t total[NC] = {0}, left[NC] = {0};
        for (int64_t p = 0; p < nn; ++p) {
            const int32_t r = rows[lo + p];
            sorted[p] = {X[(int64_t)r * F + f], y[r]};
            total[y[r]]++;
        }
        std::sort(sorted.begin(), sorted.end());
        Cut best;
        for (int64_t p = 0; p + 1 < nn; ++p) {
            left[sorted[p].second]++;
            const double a = sorted[p].first, b = sorted[p + 1].first;
            const int64_t nl = p + 1, nr = nn - p - 1;
            if (!(a < b) || nl < o.min_samples_leaf || nr < o.min_samples_leaf) continue;
            Cost c;
            if (o.criterion == MO_GINI) {
                __int128 sl = 0, sr = 0;
                for (int k = 0; k < NC; ++k) {
                    sl += (__int128)left[k] * left[k];
                    sr += (__int128)(total[k] - left[k]) * (total[k] - left[k]);
                }
                c.num = -(sl * nr + sr * nl);
                c.den = (__int128)nl * nr;
            } else {
                int64_t right[NC];
                for (int k = 0; k < NC; ++k) right[k] = total[k] - left[k];
                c.exact = false;
                c.dnum = entropy_cost(left) + entropy_cost(right);
            }
            if (!best.valid || less(c, best.cost)) {
                double thr = (a + b) / 2;
                if (thr >= b) thr = a;
                best.cost = c; best.feature = f; best.threshold = thr; best.valid = true;
            }
        }
        return best;
    }

    // Appends tree t to the model.  Explicit stack: the left child is pushed last, so it and its whole subtree are
    // numbered before the right child (same numbering as a depth-first recursion, without its stack depth).
    void fit_tree(int32_t t, mo_model *m)
    {
        rows.resize((size_t)n);
        tmp.resize((size_t)n);
        for (int64_t i = 0; i < n; ++i)
            rows[i] = o.bootstrap ? (int32_t)(hash3(o.seed, 2ull * t, (uint64_t)i) % (uint64_t)n) : (int32_t)i;
        struct Item { int64_t lo, hi; int32_t depth, parent, side; };
        std::vector<Item> stack{{0, n, 0, -1, 0}};
        const int32_t base = m->tree_off.back();
        int32_t next = 0;
        while (!stack.empty()) {
            const Item it = stack.back();
            stack.pop_back();
            const int32_t me = next++;
            if (it.parent >= 0) (it.side ? m->right : m->left)[base + it.parent] = me;
            int64_t cnt[NC] = {0};
            for (int64_t p = it.lo; p < it.hi; ++p) cnt[y[rows[p]]]++;
            int major = 0, present = 0;
            for (int k = 0; k < NC; ++k) {
                if (cnt[k] > cnt[major]) major = k;
                present += cnt[k] > 0;
            }
            m->feature.push_back(-1); m->threshold.push_back(0.0); m->left.push_back(-1); m->right.push_back(-1);
            m->klass.push_back(major);
            const int64_t nn = it.hi - it.lo;
            if ((o.max_depth >= 0 && it.depth >= o.max_depth) || present <= 1 || nn < o.min_samples_split ||
                nn < 2 * (int64_t)o.min_samples_leaf)
                continue;
            int order[F];
            for (int k = 0; k < F; ++k) order[k] = k;
            if (o.max_features < F)
                for (int k = 0; k + 1 < F; ++k) {
                    const int j = k + (int)(hash3(o.seed, 2ull * t + 1, 16ull * (uint64_t)me + k) % (uint64_t)(F - k));
                    std::swap(order[k], order[j]);
                }
            Cut best;
            for (int k = 0; k < F; ++k) {
                const Cut c = best_cut(it.lo, it.hi, order[k]);
                if (c.valid && (!best.valid || better(c, best))) best = c;
                if (k + 1 >= o.max_features && best.valid) break;
            }
            if (!best.valid) continue;
            m->feature[base + me] = best.feature;
            m->threshold[base + me] = best.threshold;
            m->klass[base + me] = -1;
            // stable partition of rows[lo, hi): <= threshold first
            int64_t nl = 0, nr = 0;
            for (int64_t p = it.lo; p < it.hi; ++p) {
                const int32_t r = rows[p];
                if (X[(int64_t)r * F + best.feature] <= best.threshold) rows[it.lo + nl++] = r;
                else tmp[nr++] = r;
            }
            std::copy(tmp.begin(), tmp.begin() + nr, rows.begin() + it.lo + nl);
            stack.push_back({it.lo + nl, it.hi, it.depth + 1, me, 1});
            stack.push_back({it.lo, it.lo + nl, it.depth + 1, me, 0});
        }
        m->tree_off.push_back(base + next);
        m->n_trees++;
    }
};

}  // namespace

extern "C" {

void mo_default_fit_opts(mo_fit_opts *o)
{
    if (!o) return;
    o->n_estimators = 100;
    o->bootstrap = 1;
    o->max_depth = -1;
    o->min_samples_leaf = 1;
    o->min_samples_split = 2;
    o->max_features = MO_NUM_FEATURES;
    o->criterion = MO_GINI;
    o->seed = 0;
}

mo_status mo_model_fit(const double *features, const int32_t *labels, int64_t n, const mo_fit_opts *opts, mo_model **out)
{
    if (!out) return MO_E_NULL;
    *out = nullptr;
    if (!features || !labels) return MO_E_NULL;
    if (n < 1 || n > kMaxSamples) return MO_E_SHAPE;
    mo_fit_opts o;
    if (opts) o = *opts; else mo_default_fit_opts(&o);
    if (o.n_estimators < 1 || o.n_estimators > (1 << 16) || o.min_samples_leaf < 1 || o.min_samples_split < 2 ||
        o.max_features < 1 || o.max_features > MO_NUM_FEATURES || (o.criterion != MO_GINI && o.criterion != MO_ENTROPY) ||
        (o.bootstrap != 0 && o.bootstrap != 1))
        return MO_E_PARAM;
    for (int64_t i = 0; i < n; ++i)
        if (labels[i] < 0 || labels[i] >= MO_NUM_FORMATS) return MO_E_PARAM;
    for (int64_t i = 0; i < n * F; ++i)
        if (features[i] != features[i]) return MO_E_PARAM;            // NaN has no place on either side of a cut
    try {
        std::unique_ptr<mo_model> m(new mo_model());
        m->tree_off.push_back(0);
        Trainer tr{features, labels, n, o, {}, {}, {}};
        for (int32_t t = 0; t < o.n_estimators; ++t) {
            if ((int64_t)m->tree_off.back() + 2 * n > (1 << 24)) return MO_E_SHAPE;   // node limit of the model file
            tr.fit_tree(t, m.get());
        }
        *out = m.release();
    } catch (const std::bad_alloc &) {
        return MO_E_ALLOC;
    }
    return MO_OK;
}

}  // extern "C"

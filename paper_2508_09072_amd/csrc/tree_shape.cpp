// Tree-shape selection on the host (Appendix E; Theorem 1 of Section 3.3): prune the seed tree leaf by
// leaf in order of acceptance frequency and pick the pruning level with the best modelled throughput
//     sum_i alpha_i / (sum_{i >= 1} t_i + T_V(|T|)),
// with T_V taken from a table measured on the machine (the verification time of a tree of k nodes).
// Plain C++ on host memory; no GPU involved.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <functional>
#include <new>
#include <queue>
#include <vector>

#include "reader.h"

namespace {

bool tree_ok(const int32_t *parents, int32_t T) {
    if (!parents || T < 1 || parents[0] != -1) return false;
    for (int32_t i = 1; i < T; ++i)
        if (parents[i] < 0 || parents[i] >= i) return false;
    return true;
}

// Removal order of Appendix E: repeatedly the leaf with the lowest alpha (equal: the highest id).
// A heap of the current leaves; removing a node may turn its parent into a leaf.
void removal_order(const int32_t *parents, const float *alpha, int32_t T, std::vector<int32_t> &order) {
    std::vector<int32_t> n_children(T, 0);
    for (int32_t i = 1; i < T; ++i) ++n_children[parents[i]];
    auto worse = [&](int32_t a, int32_t b) {       // true if a should come out after b
        if (alpha[a] != alpha[b]) return alpha[a] > alpha[b];
        return a < b;
    };
    std::priority_queue<int32_t, std::vector<int32_t>, decltype(worse)> leaves(worse);
    for (int32_t i = 1; i < T; ++i)
        if (n_children[i] == 0) leaves.push(i);
    order.clear();
    order.reserve(T > 0 ? T - 1 : 0);
    while (!leaves.empty()) {
        const int32_t v = leaves.top();
        leaves.pop();
        order.push_back(v);
        const int32_t par = parents[v];
        if (par > 0 && --n_children[par] == 0) leaves.push(par);
    }
}

}  // namespace

extern "C" int32_t reader_tree_prune_order(const int32_t *parents, const float *alpha, int32_t T, int32_t *order) {
    if (!tree_ok(parents, T) || !alpha || (T > 1 && !order)) return -1;
    for (int32_t i = 0; i < T; ++i)
        if (!(alpha[i] >= 0.f)) return -1;          // (also refuses NaN)
    try {
        std::vector<int32_t> ord;
        removal_order(parents, alpha, T, ord);
        std::copy(ord.begin(), ord.end(), order);
        return (int32_t)ord.size();
    } catch (const std::bad_alloc &) {
        return -1;
    }
}

extern "C" int32_t reader_tree_select(const int32_t *parents, const float *alpha, const float *t_draft,
                                      const float *tv, int32_t T, int32_t exhaustive, int32_t *keep,
                                      double *throughput, int32_t *evaluations) {
    if (!tree_ok(parents, T) || !alpha || !t_draft || !tv || !keep) return -1;
    for (int32_t i = 0; i < T; ++i)
        if (!(alpha[i] >= 0.f) || !(t_draft[i] >= 0.f) || !(tv[i] > 0.f)) return -1;
    try {
        std::vector<int32_t> order;
        removal_order(parents, alpha, T, order);
        // gain[n], cost[n]: sum of alpha / of drafting times of T_n (the seed tree without the first n of the order)
        std::vector<double> gain(T), cost(T);
        double g = 0.0, c = 0.0;
        for (int32_t i = 0; i < T; ++i) { g += alpha[i]; if (i > 0) c += t_draft[i]; }
        gain[0] = g; cost[0] = c;
        for (int32_t n = 1; n < T; ++n) {
            g -= alpha[order[n - 1]];
            c -= t_draft[order[n - 1]];
            gain[n] = g;
            cost[n] = c < 0.0 ? 0.0 : c;
        }
        int32_t evals = 0;
        auto score = [&](int32_t n) {
            ++evals;
            return gain[n] / (cost[n] + (double)tv[T - n - 1]);
        };
        int32_t best = 0;
        double best_score = 0.0;
        if (exhaustive || T <= 4) {
            best_score = score(0);
            for (int32_t n = 1; n < T; ++n) {
                const double s = score(n);
                if (s > best_score) { best_score = s; best = n; }
            }
        } else {
            // Golden-section search on the integer interval [lo, hi] for a curve that rises and then falls
            // (Appendix E: the response in n is close to unimodal).  Two interior points are kept; each
            // step drops the part of the interval beyond the worse one and scores one new point.
            const double inv_phi = 0.6180339887498949;
            int32_t lo = 0, hi = T - 1;
            int32_t x1 = hi - (int32_t)std::lround((hi - lo) * inv_phi), x2 = lo + (int32_t)std::lround((hi - lo) * inv_phi);
            double f1 = score(x1), f2 = score(x2);
            while (hi - lo > 3) {
                if (f1 >= f2) {              // the peak is not to the right of x2 (equal: the larger tree wins)
                    hi = x2; x2 = x1; f2 = f1;
                    x1 = hi - (int32_t)std::lround((hi - lo) * inv_phi);
                    if (x1 >= x2) x1 = x2 - 1;
                    if (x1 < lo) x1 = lo;
                    f1 = score(x1);
                } else {
                    lo = x1; x1 = x2; f1 = f2;
                    x2 = lo + (int32_t)std::lround((hi - lo) * inv_phi);
                    if (x2 <= x1) x2 = x1 + 1;
                    if (x2 > hi) x2 = hi;
                    f2 = score(x2);
                }
            }
            best = lo;
            best_score = score(lo);
            for (int32_t n = lo + 1; n <= hi; ++n) {
                const double s = score(n);
                if (s > best_score) { best_score = s; best = n; }
            }
        }
        for (int32_t i = 0; i < T; ++i) keep[i] = 1;
        for (int32_t n = 0; n < best; ++n) keep[order[n]] = 0;
        if (throughput) *throughput = best_score;
        if (evaluations) *evaluations = evals;
        return best;
    } catch (const std::bad_alloc &) {
        return -1;
    }
}

// Mixed-scheme selection (Section 4.1 eq. (3); fusion-aware form Section 4.2 eq. (4) with its
// constraints (C1), (C2)) as a multiple-choice knapsack, solved on the host by dynamic
// programming over a discretised cost axis.  No device code.
//
// A "class" is a set of mutually exclusive options of which exactly one is taken.  For plain
// mixed-scheme quantization a class is a layer and an option a quantizer.  For the fusion-aware
// problem a class is a cluster of layers that share their input ({q,k,v}, {o}, {gate,up}, {down}
// of one block) and an option is one way of splitting the cluster into fused groups together
// with one quantizer per group; (C1) - every layer in exactly one active group - then holds by
// construction, the option's loss is the sum of its layers' loss terms and its cost the sum of
// its groups' profiled costs, and (C2) is the knapsack constraint.
#include <cmath>
#include <cstdlib>
#include <limits>
#include <vector>

#include "qp_internal.h"

extern "C" qp_status qp_msq_solve(int32_t n_classes, const int32_t *begin, const double *loss, const double *cost,
                                  double budget, int32_t resolution, int32_t *choice, double *total_loss,
                                  double *total_cost) {
    if (!begin || !loss || !cost || !choice) return QP_ERR_NULL;
    if (n_classes < 1 || resolution < 1 || resolution > (1 << 22) || !(budget >= 0.0) || !std::isfinite(budget))
        return QP_ERR_SHAPE;
    if (begin[0] != 0) return QP_ERR_SHAPE;
    for (int c = 0; c < n_classes; ++c)
        if (begin[c + 1] <= begin[c]) return QP_ERR_SHAPE;            // a class without options
    const int n_opt = begin[n_classes];
    for (int o = 0; o < n_opt; ++o)
        if (!(cost[o] >= 0.0) || !std::isfinite(cost[o]) || !std::isfinite(loss[o])) return QP_ERR_SHAPE;
    if ((int64_t)n_classes * (resolution + 1) > ((int64_t)1 << 31)) return QP_ERR_SHAPE;

    // Cost axis: R + 1 cells of width q = budget / R; an option's cost is rounded UP to whole
    // cells, so whatever the table calls feasible is feasible for the true costs.
    const int R = resolution;
    const double q = (budget > 0.0) ? budget / R : 1.0;
    std::vector<int> w(n_opt);
    for (int o = 0; o < n_opt; ++o) {
        double cells = (budget > 0.0) ? std::ceil(cost[o] / q - 1e-9) : (cost[o] > 0.0 ? R + 1.0 : 0.0);
        w[o] = cells > R ? R + 1 : (int)cells;
    }
    const double INF = std::numeric_limits<double>::infinity();
    // best[k] after the first c classes: least loss with rounded cost exactly k
    std::vector<double> best(R + 1, INF), next(R + 1);
    std::vector<int32_t> pick((size_t)n_classes * (R + 1), -1);
    best[0] = 0.0;
    for (int c = 0; c < n_classes; ++c) {
        std::fill(next.begin(), next.end(), INF);
        int32_t *pc = &pick[(size_t)c * (R + 1)];
        for (int o = begin[c]; o < begin[c + 1]; ++o) {
            if (w[o] > R) continue;
            for (int k = 0; k + w[o] <= R; ++k) {
                if (best[k] == INF) continue;
                const double v = best[k] + loss[o];
                if (v < next[k + w[o]]) {   // strict: ties keep the option with the lower index
                    next[k + w[o]] = v;
                    pc[k + w[o]] = o;
                }
            }
        }
        best.swap(next);
    }
    int kbest = -1;
    for (int k = 0; k <= R; ++k)
        if (best[k] < INF && (kbest < 0 || best[k] < best[kbest])) kbest = k;
    if (kbest < 0) return QP_ERR_UNSUPPORTED;   // no selection fits the budget
    double tl = 0.0, tc = 0.0;
    int k = kbest;
    for (int c = n_classes - 1; c >= 0; --c) {
        const int o = pick[(size_t)c * (R + 1) + k];
        choice[c] = o - begin[c];
        tl += loss[o];
        tc += cost[o];
        k -= w[o];
    }
    if (total_loss) *total_loss = tl;
    if (total_cost) *total_cost = tc;
    return QP_OK;
}

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
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <limits>
#include <vector>

#include "qp_internal.h"

// The dynamic programme.  Throws std::bad_alloc when the tables do not fit the host's memory (the
// exported entry points catch it).
static qp_status msq_solve(int32_t n_classes, const int32_t *begin, const double *loss, const double *cost,
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
    // cells, so whatever the table calls feasible is feasible for the true costs.  A cost that is a
    // whole number of cells must not be pushed into the next cell by the rounding of the division:
    // the smaller count is taken when it still covers the cost (cells * q >= cost as computed, i.e.
    // within one rounding of the true product).
    const int R = resolution;
    const double q = (budget > 0.0) ? budget / R : 1.0;
    std::vector<int> w(n_opt);
    for (int o = 0; o < n_opt; ++o) {
        double cells;
        if (budget > 0.0) {
            cells = std::ceil(cost[o] / q);
            if (cells >= 1.0 && (cells - 1.0) * q >= cost[o]) cells -= 1.0;
        } else {
            cells = cost[o] > 0.0 ? R + 1.0 : 0.0;
        }
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

extern "C" qp_status qp_msq_solve(int32_t n_classes, const int32_t *begin, const double *loss, const double *cost,
                                  double budget, int32_t resolution, int32_t *choice, double *total_loss,
                                  double *total_cost) {
    try {
        return msq_solve(n_classes, begin, loss, cost, budget, resolution, choice, total_loss, total_cost);
    } catch (...) {
        return QP_ERR_MEMORY;   // the tables did not fit: nothing crosses the C boundary as an exception
    }
}

// ------------------------------------------------------------------ fusion-aware form, eq. (4)
// Layers of a block in the order q, k, v, o, u, g, d; the twelve fusible groups of Section 4.2 in the
// order {q} {k} {v} {q,k} {q,v} {k,v} {q,k,v} {o} {u} {g} {u,g} {d}.  Layers that share their input form
// a cluster ({q,k,v}, {o}, {u,g}, {d}); a selection that satisfies (C1) splits every cluster into
// groups - one of the partitions below - and gives every group one quantizer.
namespace {
constexpr int kLayers = 7, kGroups = 12, kClusters = 4;
const int kGroupLayers[kGroups][3] = {{0, -1, -1}, {1, -1, -1}, {2, -1, -1}, {0, 1, -1}, {0, 2, -1}, {1, 2, -1},
                                      {0, 1, 2},   {3, -1, -1}, {4, -1, -1}, {5, -1, -1}, {4, 5, -1}, {6, -1, -1}};
struct Partition { int n; int g[3]; };
const Partition kQkv[5] = {{3, {0, 1, 2}}, {2, {3, 2, -1}}, {2, {4, 1, -1}}, {2, {5, 0, -1}}, {1, {6, -1, -1}}};
const Partition kO[1] = {{1, {7, -1, -1}}};
const Partition kUg[2] = {{2, {8, 9, -1}}, {1, {10, -1, -1}}};
const Partition kD[1] = {{1, {11, -1, -1}}};
const Partition *const kParts[kClusters] = {kQkv, kO, kUg, kD};
const int kNParts[kClusters] = {5, 1, 2, 1};

struct Option {
    double loss, cost;
    int8_t part;     // partition of the cluster
    int8_t q[3];     // quantizer of each of its groups
};
}  // namespace

extern "C" qp_status qp_msq_solve_fused(int32_t n_blocks, int32_t n_quant, const double *loss, const double *cost,
                                        double budget, int32_t resolution, int32_t fusion, int32_t *assign,
                                        double *total_loss, double *total_cost) {
    if (!loss || !cost || !assign) return QP_ERR_NULL;
    if (n_blocks < 1 || n_blocks > 4096 || n_quant < 1 || n_quant > 16) return QP_ERR_SHAPE;
    try {
        std::vector<std::vector<Option>> classes;   // one per (block, cluster), pruned
        classes.reserve((size_t)n_blocks * kClusters);
        for (int b = 0; b < n_blocks; ++b) {
            const double *lb = loss + (size_t)b * kLayers * n_quant;
            const double *cb = cost + (size_t)b * kGroups * n_quant;
            for (int cl = 0; cl < kClusters; ++cl) {
                std::vector<Option> opts;
                for (int p = 0; p < kNParts[cl]; ++p) {
                    const Partition &P = kParts[cl][p];
                    bool fused = false;
                    for (int i = 0; i < P.n; ++i) fused = fused || kGroupLayers[P.g[i]][1] >= 0;
                    if (!fusion && fused) continue;     // per-layer selection, eq. (3): single-layer groups only
                    int total = 1;
                    for (int i = 0; i < P.n; ++i) total *= n_quant;
                    for (int code = 0; code < total; ++code) {
                        Option o{0.0, 0.0, (int8_t)p, {-1, -1, -1}};
                        int rest = code;
                        for (int i = 0; i < P.n; ++i) {
                            const int q = rest % n_quant;
                            rest /= n_quant;
                            o.q[i] = (int8_t)q;
                            o.cost += cb[P.g[i] * n_quant + q];
                            for (int m = 0; m < 3; ++m) {
                                const int layer = kGroupLayers[P.g[i]][m];
                                if (layer >= 0) o.loss += lb[layer * n_quant + q];
                            }
                        }
                        if (!std::isfinite(o.loss) || !std::isfinite(o.cost) || !(o.cost >= 0.0)) return QP_ERR_SHAPE;
                        opts.push_back(o);
                    }
                }
                // an option that another one beats or equals in both loss and cost can never be needed
                std::stable_sort(opts.begin(), opts.end(), [](const Option &a, const Option &c) {
                    return a.cost < c.cost || (a.cost == c.cost && a.loss < c.loss);
                });
                std::vector<Option> kept;
                double best = std::numeric_limits<double>::infinity();
                for (const Option &o : opts)
                    if (o.loss < best) {
                        kept.push_back(o);
                        best = o.loss;
                    }
                classes.push_back(std::move(kept));
            }
        }
        const int n_classes = (int)classes.size();
        std::vector<int32_t> begin(n_classes + 1, 0), choice(n_classes);
        for (int c = 0; c < n_classes; ++c) begin[c + 1] = begin[c] + (int32_t)classes[c].size();
        std::vector<double> fl(begin[n_classes]), fc(begin[n_classes]);
        for (int c = 0; c < n_classes; ++c)
            for (size_t o = 0; o < classes[c].size(); ++o) {
                fl[begin[c] + o] = classes[c][o].loss;
                fc[begin[c] + o] = classes[c][o].cost;
            }
        const qp_status s = msq_solve(n_classes, begin.data(), fl.data(), fc.data(), budget, resolution, choice.data(),
                                      total_loss, total_cost);
        if (s != QP_OK) return s;
        for (int i = 0; i < n_blocks * kGroups; ++i) assign[i] = -1;
        for (int c = 0; c < n_classes; ++c) {
            const Option &o = classes[c][choice[c]];
            const Partition &P = kParts[c % kClusters][o.part];
            for (int i = 0; i < P.n; ++i) assign[(c / kClusters) * kGroups + P.g[i]] = o.q[i];
        }
        return QP_OK;
    } catch (...) {
        return QP_ERR_MEMORY;
    }
}

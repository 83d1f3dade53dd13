// Heterogeneity-aware optimal pipeline partition (paper sections 3.2-3.3).
//
// The paper's recurrence (Eq. 3) is over states (layers done, devices used,
// device of the next stage).  Here the same state space is solved backwards:
//
//   g(i, S, u) = smallest achievable largest period for layers i..L-1 when the
//                devices in S are spent and u (not in S) runs the stage that
//                starts at layer i
//              = min over the stage end j in (i, L] that fits u's memory of
//                  j == L :  T_comp(i..L-1, u)
//                  j <  L :  min over v not in S+{u} of
//                            max(T_comp(i..j-1, u), P_{j-1} / b_{u,v}, g(j, S+{u}, v))
//   T_opt      = min_u g(0, {}, u).
//
// (Eq. 1 gives the communication term, Eq. 2 the period of a stage; the last
// stage sends nothing.)  Every value is one of the candidate periods, combined
// only by max/min, so T_opt is reproduced bit for bit by any other exact
// solver that sums T_comp in the same order (first layer of the stage to last).
//
// The backward form makes the unique answer cheap to construct: walking
// forward from layer 0 and always taking the smallest device id, then the
// smallest stage end, for which g still reaches T_opt yields the
// lexicographically smallest optimal sequence (dev_0, last_0, dev_1, ...).
//
// Work is O(2^D L^2 D^2) in the worst case as in section 3.3; stages whose
// compute time alone exceeds a cheap upper bound on T_opt (the best single
// device that fits, else +inf) are cut off, which is exact because periods
// only grow along a stage.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <limits>
#include <new>
#include <vector>

#include "edgepipe.h"
#include "ep_error.h"

namespace {

struct Problem {
    int L, D;
    const double *t_comp, *layer_mem, *dev_mem, *xfer, *bw;
    double comm(int u, int v, int last_layer) const
    {
        const double b = bw[(size_t)u * D + v];
        if (!(b > 0.0)) return std::numeric_limits<double>::infinity();
        return xfer[last_layer] / b;
    }
};

inline int popcount64(uint64_t x) { return __builtin_popcountll(x); }

}  // namespace

extern "C" ep_status ep_partition(int32_t L, int32_t D, const double *t_comp,
                                  const double *layer_mem, const double *dev_mem,
                                  const double *xfer_bytes, const double *bw, double *t_opt,
                                  int32_t *n_stages, int32_t *stage_dev, int32_t *stage_first,
                                  int32_t *stage_last)
{
    if (L < 1 || D < 1 || D > 20)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_partition: need L >= 1 and 1 <= D <= 20 (L=%d, D=%d)", L, D);
    if (!t_comp || !layer_mem || !dev_mem || !xfer_bytes || !bw || !t_opt || !n_stages ||
        !stage_dev || !stage_first || !stage_last)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_partition: null pointer argument");
    for (int64_t k = 0; k < (int64_t)L * D; ++k)
        if (!(t_comp[k] >= 0.0) || std::isinf(t_comp[k]))
            return ep_fail(EP_ERR_INVALID_ARG, "ep_partition: t_comp[%lld] must be finite and >= 0", (long long)k);
    for (int l = 0; l < L; ++l)
        if (!(layer_mem[l] >= 0.0) || !(xfer_bytes[l] >= 0.0))
            return ep_fail(EP_ERR_INVALID_ARG, "ep_partition: layer_mem and xfer_bytes must be >= 0");
    for (int64_t k = 0; k < (int64_t)D * D; ++k)
        if (std::isnan(bw[k]))
            return ep_fail(EP_ERR_INVALID_ARG, "ep_partition: bw[%lld] is NaN", (long long)k);

    const Problem P{L, D, t_comp, layer_mem, dev_mem, xfer_bytes, bw};
    const double INF = std::numeric_limits<double>::infinity();

    // Upper bound: best single device that holds the whole model.
    double ub = INF;
    for (int u = 0; u < D; ++u) {
        double mem = 0.0, comp = 0.0;
        bool fits = true;
        for (int l = 0; l < L && fits; ++l) {
            mem += layer_mem[l];
            if (mem > dev_mem[u]) fits = false;
            comp += t_comp[(size_t)l * D + u];
        }
        if (fits && comp < ub) ub = comp;
    }

    const uint64_t nS = 1ull << D;
    const size_t n_states = (size_t)L * nS * D;     // i in [0, L)
    double *g = new (std::nothrow) double[n_states];
    if (!g) return ep_fail(EP_ERR_OOM, "ep_partition: cannot allocate %zu table entries", n_states);
    auto at = [&](int i, uint64_t S, int u) -> double & { return g[((size_t)i * nS + S) * D + u]; };

    // Backward sweep.  A state (i, S, u) can only arise with |S| <= i stages
    // before it (each stage has at least one layer) and |S| >= 1 unless i == 0.
    for (int i = L - 1; i >= 0; --i) {
        for (uint64_t S = 0; S < nS; ++S) {
            const int used = popcount64(S);
            if (used > i || (i > 0 && used == 0) || (i == 0 && used != 0)) continue;
            for (int u = 0; u < D; ++u) {
                if (S >> u & 1) continue;
                const uint64_t S2 = S | (1ull << u);
                double best = INF, mem = 0.0, comp = 0.0;
                for (int j = i + 1; j <= L; ++j) {       // stage = layers i..j-1
                    mem += layer_mem[j - 1];
                    if (mem > dev_mem[u]) break;
                    comp += t_comp[(size_t)(j - 1) * D + u];
                    if (comp > ub || comp >= best) break;  // periods only grow with j
                    if (j == L) {
                        if (comp < best) best = comp;
                    } else {
                        for (int v = 0; v < D; ++v) {
                            if (S2 >> v & 1) continue;
                            double c = P.comm(u, v, j - 1);
                            if (c < comp) c = comp;
                            const double rest = at(j, S2, v);
                            if (rest > c) c = rest;
                            if (c < best) best = c;
                        }
                    }
                }
                at(i, S, u) = best;
            }
        }
    }

    double topt = INF;
    for (int u = 0; u < D; ++u)
        if (at(0, 0, u) < topt) topt = at(0, 0, u);
    if (topt == INF) {
        delete[] g;
        return ep_fail(EP_ERR_INFEASIBLE, "ep_partition: no strategy satisfies the memory limits");
    }

    // Forward construction of the lexicographically smallest optimal strategy.
    std::vector<int32_t> dev, first, last;
    int i = 0, u = -1;
    uint64_t S = 0;
    for (int c = 0; c < D; ++c)
        if (at(0, 0, c) <= topt) { u = c; break; }
    while (true) {
        const uint64_t S2 = S | (1ull << u);
        double mem = 0.0, comp = 0.0;
        int chosen_j = -1, chosen_v = -1;
        for (int j = i + 1; j <= L && chosen_j < 0; ++j) {
            mem += layer_mem[j - 1];
            if (mem > dev_mem[u]) break;
            comp += t_comp[(size_t)(j - 1) * D + u];
            if (comp > topt) break;
            if (j == L) { chosen_j = j; break; }
            for (int v = 0; v < D; ++v) {
                if (S2 >> v & 1) continue;
                if (P.comm(u, v, j - 1) <= topt && at(j, S2, v) <= topt) {
                    chosen_j = j; chosen_v = v; break;
                }
            }
        }
        if (chosen_j < 0) {   // cannot happen: g(i,S,u) <= T_opt guarantees a continuation
            delete[] g;
            return ep_fail(EP_ERR_INVALID_ARG, "ep_partition: internal error while building the strategy");
        }
        dev.push_back(u); first.push_back(i); last.push_back(chosen_j - 1);
        if (chosen_j == L) break;
        S = S2; i = chosen_j; u = chosen_v;
    }
    delete[] g;

    *t_opt = topt;
    *n_stages = (int32_t)dev.size();
    for (size_t s = 0; s < dev.size(); ++s) {
        stage_dev[s] = dev[s]; stage_first[s] = first[s]; stage_last[s] = last[s];
    }
    return EP_OK;
}

// Optimal pipeline partition with identical devices collapsed into categories
// (paper section 3.3, the paragraph after Algorithm 1: with N categories of
// n_1 .. n_N identical devices the search state shrinks from 2^D subsets to
// prod (n_c + 1) count vectors).
//
// Two devices are identical when they have the same execution time for every
// layer, the same memory, the same bandwidth to and from every third device and
// the same bandwidth between each other in both directions; that relation is an
// equivalence, and inside a class every pair then has one common bandwidth.  The
// classes are found here from the per-device inputs, so the call takes exactly
// what ep_partition takes.
//
// The recurrence is the one of ep_partition.cpp with the used-device set S
// replaced by the vector k of used devices per category:
//
//   g(i, k, c) = smallest achievable largest period for layers i..L-1 when k_c'
//                devices of each category c' are spent and a device of category c
//                (k_c < n_c) runs the stage that starts at layer i
//
// with the same candidate periods (Eq. 1, Eq. 2), the same order of summation
// and the same cut-offs, so T_opt is bit for bit the value ep_partition returns.
// The strategy is built forward in the same way (smallest device id, then
// smallest stage end, that still reaches T_opt); since identical devices have
// identical g, looking only at the lowest unused id of each category finds the
// same lexicographically smallest optimal strategy.
#include <cmath>
#include <cstdint>
#include <limits>
#include <new>
#include <vector>

#include "edgepipe.h"
#include "ep_error.h"

namespace {

struct Input {
    int L, D;
    const double *t_comp, *layer_mem, *dev_mem, *xfer, *bw;
};

bool identical(const Input &P, int u, int v)
{
    if (P.dev_mem[u] != P.dev_mem[v]) return false;
    for (int l = 0; l < P.L; ++l)
        if (P.t_comp[(size_t)l * P.D + u] != P.t_comp[(size_t)l * P.D + v]) return false;
    if (P.bw[(size_t)u * P.D + v] != P.bw[(size_t)v * P.D + u]) return false;
    for (int w = 0; w < P.D; ++w) {
        if (w == u || w == v) continue;
        if (P.bw[(size_t)u * P.D + w] != P.bw[(size_t)v * P.D + w]) return false;
        if (P.bw[(size_t)w * P.D + u] != P.bw[(size_t)w * P.D + v]) return false;
    }
    return true;
}

}  // namespace

extern "C" ep_status ep_partition_categories(int32_t L, int32_t D, const double *t_comp,
                                             const double *layer_mem, const double *dev_mem,
                                             const double *xfer_bytes, const double *bw, double *t_opt,
                                             int32_t *n_stages, int32_t *stage_dev, int32_t *stage_first,
                                             int32_t *stage_last, int32_t *n_categories)
{
    if (L < 1 || D < 1 || D > 64)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_partition_categories: need L >= 1 and 1 <= D <= 64 (L=%d, D=%d)", L, D);
    if (!t_comp || !layer_mem || !dev_mem || !xfer_bytes || !bw || !t_opt || !n_stages || !stage_dev ||
        !stage_first || !stage_last)
        return ep_fail(EP_ERR_INVALID_ARG, "ep_partition_categories: null pointer argument");
    for (int64_t k = 0; k < (int64_t)L * D; ++k)
        if (!(t_comp[k] >= 0.0) || std::isinf(t_comp[k]))
            return ep_fail(EP_ERR_INVALID_ARG, "ep_partition_categories: t_comp[%lld] must be finite and >= 0", (long long)k);
    for (int l = 0; l < L; ++l)
        if (!(layer_mem[l] >= 0.0) || !(xfer_bytes[l] >= 0.0))
            return ep_fail(EP_ERR_INVALID_ARG, "ep_partition_categories: layer_mem and xfer_bytes must be >= 0");
    for (int64_t k = 0; k < (int64_t)D * D; ++k)
        if (std::isnan(bw[k])) return ep_fail(EP_ERR_INVALID_ARG, "ep_partition_categories: bw[%lld] is NaN", (long long)k);

    const Input P{L, D, t_comp, layer_mem, dev_mem, xfer_bytes, bw};
    const double INF = std::numeric_limits<double>::infinity();

    // ---- categories: members in increasing device id, categories in order of their first member
    std::vector<int> cat_of(D, -1);
    std::vector<std::vector<int>> members;
    for (int u = 0; u < D; ++u) {
        for (size_t c = 0; c < members.size() && cat_of[u] < 0; ++c)
            if (identical(P, members[c][0], u)) cat_of[u] = (int)c;
        if (cat_of[u] < 0) {
            cat_of[u] = (int)members.size();
            members.push_back({});
        }
        members[cat_of[u]].push_back(u);
    }
    const int N = (int)members.size();
    if (n_categories) *n_categories = N;
    std::vector<int> rep(N), cnt(N);
    std::vector<size_t> stride(N);
    size_t n_vec = 1;
    for (int c = 0; c < N; ++c) {
        rep[c] = members[c][0];
        cnt[c] = (int)members[c].size();
        stride[c] = n_vec;
        if (n_vec > (size_t)1 << 40) return ep_fail(EP_ERR_OOM, "ep_partition_categories: state space too large");
        n_vec *= (size_t)cnt[c] + 1;
    }
    const size_t n_states = (size_t)L * n_vec * N;
    if (n_vec > ((size_t)1 << 31) || n_states > ((size_t)1 << 31))
        return ep_fail(EP_ERR_OOM, "ep_partition_categories: %zu table entries are too many", n_states);
    // bandwidth from a device of category a to a (different) device of category b
    auto cat_bw = [&](int a, int b) -> double {
        if (a != b) return bw[(size_t)rep[a] * D + rep[b]];
        return cnt[a] >= 2 ? bw[(size_t)members[a][0] * D + members[a][1]] : 0.0;
    };
    auto comm = [&](int a, int b, int last_layer) -> double {
        const double bb = cat_bw(a, b);
        if (!(bb > 0.0)) return INF;
        return xfer_bytes[last_layer] / bb;
    };

    // Upper bound: best single device that holds the whole model.
    double ub = INF;
    for (int c = 0; c < N; ++c) {
        const int u = rep[c];
        double mem = 0.0, comp = 0.0;
        bool fits = true;
        for (int l = 0; l < L && fits; ++l) {
            mem += layer_mem[l];
            if (mem > dev_mem[u]) fits = false;
            comp += t_comp[(size_t)l * D + u];
        }
        if (fits && comp < ub) ub = comp;
    }

    double *g = new (std::nothrow) double[n_states];
    if (!g) return ep_fail(EP_ERR_OOM, "ep_partition_categories: cannot allocate %zu table entries", n_states);
    auto at = [&](int i, size_t kv, int c) -> double & { return g[((size_t)i * n_vec + kv) * N + c]; };

    // Backward sweep over count vectors.  k is kept as digits next to its index kv.
    std::vector<int> k(N);
    for (int i = L - 1; i >= 0; --i) {
        std::fill(k.begin(), k.end(), 0);
        for (size_t kv = 0; kv < n_vec; ++kv) {
            int used = 0;
            for (int c = 0; c < N; ++c) used += k[c];
            if (!(used > i || (i > 0 && used == 0) || (i == 0 && used != 0))) {
                for (int c = 0; c < N; ++c) {
                    if (k[c] >= cnt[c]) continue;
                    const int u = rep[c];
                    const size_t kv2 = kv + stride[c];
                    double best = INF, mem = 0.0, comp = 0.0;
                    for (int j = i + 1; j <= L; ++j) {       // stage = layers i..j-1
                        mem += layer_mem[j - 1];
                        if (mem > dev_mem[u]) break;
                        comp += t_comp[(size_t)(j - 1) * D + u];
                        if (comp > ub || comp >= best) break;  // periods only grow with j
                        if (j == L) {
                            if (comp < best) best = comp;
                        } else {
                            for (int v = 0; v < N; ++v) {
                                if (k[v] + (v == c ? 1 : 0) >= cnt[v]) continue;
                                double cc = comm(c, v, j - 1);
                                if (cc < comp) cc = comp;
                                const double rest = at(j, kv2, v);
                                if (rest > cc) cc = rest;
                                if (cc < best) best = cc;
                            }
                        }
                    }
                    at(i, kv, c) = best;
                }
            }
            for (int c = 0; c < N; ++c) {        // next count vector
                if (++k[c] <= cnt[c]) break;
                k[c] = 0;
            }
        }
    }

    double topt = INF;
    for (int c = 0; c < N; ++c)
        if (at(0, 0, c) < topt) topt = at(0, 0, c);
    if (topt == INF) {
        delete[] g;
        return ep_fail(EP_ERR_INFEASIBLE, "ep_partition_categories: no strategy satisfies the memory limits");
    }

    // Forward construction: devices in increasing id (an unused device stands for its category).
    std::vector<int32_t> dev, first, last;
    std::vector<char> spent(D, 0);
    std::fill(k.begin(), k.end(), 0);
    size_t kv = 0;
    int i = 0, u = -1;
    for (int d = 0; d < D; ++d)
        if (at(0, 0, cat_of[d]) <= topt) { u = d; break; }
    while (true) {
        const int c = cat_of[u];
        const size_t kv2 = kv + stride[c];
        spent[u] = 1;
        double mem = 0.0, comp = 0.0;
        int chosen_j = -1, chosen_v = -1;
        for (int j = i + 1; j <= L && chosen_j < 0; ++j) {
            mem += layer_mem[j - 1];
            if (mem > dev_mem[u]) break;
            comp += t_comp[(size_t)(j - 1) * D + u];
            if (comp > topt) break;
            if (j == L) { chosen_j = j; break; }
            for (int v = 0; v < D; ++v) {
                if (spent[v]) continue;
                const int cv = cat_of[v];
                if (comm(c, cv, j - 1) <= topt && at(j, kv2, cv) <= topt) {
                    chosen_j = j; chosen_v = v; break;
                }
            }
        }
        if (chosen_j < 0) {   // cannot happen: g(i,k,c) <= T_opt guarantees a continuation
            delete[] g;
            return ep_fail(EP_ERR_INVALID_ARG, "ep_partition_categories: internal error while building the strategy");
        }
        dev.push_back(u); first.push_back(i); last.push_back(chosen_j - 1);
        if (chosen_j == L) break;
        kv = kv2; ++k[c]; i = chosen_j; u = chosen_v;
    }
    delete[] g;

    *t_opt = topt;
    *n_stages = (int32_t)dev.size();
    for (size_t s = 0; s < dev.size(); ++s) {
        stage_dev[s] = dev[s]; stage_first[s] = first[s]; stage_last[s] = last[s];
    }
    return EP_OK;
}

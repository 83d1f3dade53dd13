/*
 * Full-size cross-check of the pipeline partition (paper section 3.2-3.3):
 * the recurrence of Eq. 3 evaluated set by set, written from the equation,
 * not from the printed listing.
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT: on small instances this solver and the
 * library's planner are both checked against exhaustive enumeration
 * (partition.py); at 16 devices x 32 layers, where enumeration is out of reach,
 * the library's T_opt is compared with this one.  It shares no source with the
 * library.
 *
 * State.  f(j, S, u), u in S: the smallest achievable largest period over all
 * ways to run layers 0 .. j-1 on exactly the devices of S, one stage each, with
 * u running the last of these stages.  Counted are the compute time of every
 * one of the stages (Eq. 1: T_comp of a stage on its device) and the transfer
 * time of every stage but the last (Eq. 2: a stage's period is the larger of
 * its compute and its transfer to the next device) - what the last stage sends
 * depends on who receives it and is added when the next stage is attached.
 *   one stage:   f(j, {u}, u) = T_comp(0 .. j-1, u)                 if it fits u
 *   otherwise:   f(j, S, u)   = min over i < j, w in S \ {u} of
 *                   max( f(i, S \ {u}, w), P_{i-1} / b(w, u), T_comp(i .. j-1, u) )
 *                                                      if layers i .. j-1 fit u
 *   T_opt = min over S, u of f(L, S, u): the last stage sends nothing.
 * This is Eq. 3 with the state indexed by the device that ran the last stage
 * instead of the one that runs the next (the two index the same transitions);
 * the minimum is taken per state over its predecessors, sets in increasing
 * numeric order (S \ {u} < S), so every predecessor is final when it is read.
 * Readings of the paper where it cannot be taken literally: any device may run
 * the first stage; the transfer term belongs to the pair (sender, receiver);
 * a device's memory holds exactly the layers of its stage; T_comp of a run of
 * layers is the sum of the per-layer times, added first layer to last.
 * For the strategy each state keeps the (i, w) that gave its minimum (the first
 * one found among equals, so only T_opt and the validity of the strategy are
 * comparable with other solvers).
 *
 * Layers are 0-based; a stage covers layers i .. j-1; what it sends is
 * xfer_bytes[j-1].  Returns 0 ok, 1 infeasible, 2 out of memory, 3 bad argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

int epo_partition_dp(int32_t L, int32_t D, const double *t_comp /* [L*D] */,
                     const double *layer_mem /* [L] */, const double *dev_mem /* [D] */,
                     const double *xfer_bytes /* [L] */, const double *bw /* [D*D] */,
                     double *t_opt, int32_t *n_stages, int32_t *stage_dev,
                     int32_t *stage_first, int32_t *stage_last)
{
    if (L < 1 || D < 1 || D > 20) return 3;
    const int64_t n_sets = (int64_t)1 << D;
    const int64_t row = (int64_t)L + 1;                    /* f(., S, u) for j = 0 .. L */
    const int64_t n = n_sets * D * row;
#define AT(S, u, j) (((int64_t)(S) * D + (u)) * row + (j))
    double *f = (double *)malloc(sizeof(double) * (size_t)n);
    int32_t *from = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);   /* i * 32 + w, or -1: first stage */
    if (!f || !from) { free(f); free(from); return 2; }
    for (int64_t k = 0; k < n; ++k) { f[k] = INFINITY; from[k] = -1; }

    for (int64_t S = 1; S < n_sets; ++S) {
        for (int32_t u = 0; u < D; ++u) {
            if (!(S >> u & 1)) continue;
            const int64_t rest = S & ~((int64_t)1 << u);
            double *fu = f + AT(S, u, 0);
            int32_t *gu = from + AT(S, u, 0);
            if (rest == 0) {
                /* a single stage from layer 0 */
                double mem = 0.0, comp = 0.0;
                for (int32_t j = 1; j <= L; ++j) {
                    mem += layer_mem[j - 1];
                    if (mem > dev_mem[u]) break;
                    comp += t_comp[(int64_t)(j - 1) * D + u];
                    fu[j] = comp;
                }
                continue;
            }
            for (int32_t w = 0; w < D; ++w) {
                if (!(rest >> w & 1)) continue;
                const double *fw = f + AT(rest, w, 0);
                for (int32_t i = 1; i < L; ++i) {
                    if (fw[i] == INFINITY) continue;       /* no way to end a stage on w at layer i with this set */
                    const double send = xfer_bytes[i - 1] / bw[(int64_t)w * D + u];
                    const double before = fw[i] > send ? fw[i] : send;
                    double mem = 0.0, comp = 0.0;
                    for (int32_t j = i + 1; j <= L; ++j) {
                        mem += layer_mem[j - 1];
                        if (mem > dev_mem[u]) break;
                        comp += t_comp[(int64_t)(j - 1) * D + u];
                        const double cand = before > comp ? before : comp;
                        if (cand < fu[j]) { fu[j] = cand; gu[j] = i * 32 + w; }
                    }
                }
            }
        }
    }

    double best = INFINITY;
    int64_t best_S = 0;
    int32_t best_u = -1;
    for (int64_t S = 1; S < n_sets; ++S)
        for (int32_t u = 0; u < D; ++u)
            if ((S >> u & 1) && f[AT(S, u, L)] < best) { best = f[AT(S, u, L)]; best_S = S; best_u = u; }
    if (best_u < 0) { free(f); free(from); return 1; }
    *t_opt = best;

    /* the strategy, last stage first */
    int32_t dev_r[32], first_r[32], last_r[32], cnt = 0;
    int64_t S = best_S;
    int32_t u = best_u, j = L;
    for (;;) {
        const int32_t g = from[AT(S, u, j)];
        const int32_t i = g < 0 ? 0 : g / 32;
        dev_r[cnt] = u; first_r[cnt] = i; last_r[cnt] = j - 1; ++cnt;
        if (g < 0) break;
        S &= ~((int64_t)1 << u);
        u = g % 32;
        j = i;
    }
    *n_stages = cnt;
    for (int32_t s = 0; s < cnt; ++s) {
        stage_dev[s] = dev_r[cnt - 1 - s];
        stage_first[s] = first_r[cnt - 1 - s];
        stage_last[s] = last_r[cnt - 1 - s];
    }
    free(f); free(from);
    return 0;
#undef AT
}

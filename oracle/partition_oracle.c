/*
 * The paper's three-dimensional dynamic program for the pipeline partition
 * (section 3.3, Eq. 3 and Algorithm 1), rendered directly: state h(i, S, u) =
 * smallest achievable largest period for the first i layers using the device
 * set S, with u the device that runs the next stage; transitions are pushed
 * forward from each state in the order i, S, u, j, v; a precursor table gives
 * the strategy by back-tracing.
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT: it is the full-size cross-check of
 * the library's planner (on small instances both are checked against
 * exhaustive enumeration in partition.py).  It shares no source with the
 * library.
 *
 * Readings where the printed algorithm cannot be taken literally:
 *  - any device may run the first stage: h(0, {}, u) = 0 for every u (the text
 *    initialises only h(0, {}, none), which no loop reads);
 *  - the communication term depends on the receiver v, so the candidate value
 *    is formed inside the loop over v; the last stage (j = L) sends nothing;
 *  - the memory test covers exactly the layers i+1..j placed on u;
 *  - the final state keeps its start layer so that the back-trace can begin;
 *  - T_comp of a run of layers is the running sum of per-layer times.
 * Ties keep the first candidate found (strict <), as printed.
 *
 * Layers are 0-based here: a stage covers layers i..j-1 for the paper's
 * (i, j]; P of a stage is xfer_bytes[j-1].
 * Returns 0 ok, 1 infeasible, 2 out of memory, 3 bad argument.
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
    const int64_t nS = (int64_t)1 << D;
    const int64_t n = (int64_t)(L + 1) * nS * D;
#define IDX(i, S, u) ((((int64_t)(i)) * nS + (S)) * D + (u))
    double *h = (double *)malloc(sizeof(double) * (size_t)n);
    int32_t *pre = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);   /* i * 32 + u */
    if (!h || !pre) { free(h); free(pre); return 2; }
    for (int64_t k = 0; k < n; ++k) { h[k] = INFINITY; pre[k] = -1; }
    for (int32_t u = 0; u < D; ++u) h[IDX(0, 0, u)] = 0.0;

    double answer = INFINITY;
    int32_t ans_i = -1, ans_u = -1;
    int64_t ans_S = 0;

    for (int32_t i = 0; i < L; ++i) {
        for (int64_t S = 0; S < nS; ++S) {
            for (int32_t u = 0; u < D; ++u) {
                if (S & ((int64_t)1 << u)) continue;
                const double hv = h[IDX(i, S, u)];
                if (hv == INFINITY) continue;          /* unreachable state */
                double mem = 0.0, comp = 0.0;
                for (int32_t j = i + 1; j <= L; ++j) {
                    mem += layer_mem[j - 1];
                    if (mem > dev_mem[u]) break;
                    comp += t_comp[(int64_t)(j - 1) * D + u];
                    if (j == L) {
                        double Cv = hv > comp ? hv : comp;
                        if (Cv < answer) { answer = Cv; ans_i = i; ans_u = u; ans_S = S; }
                    } else {
                        const int64_t S2 = S | ((int64_t)1 << u);
                        for (int32_t v = 0; v < D; ++v) {
                            if (S2 & ((int64_t)1 << v)) continue;
                            double comm = xfer_bytes[j - 1] / bw[(int64_t)u * D + v];
                            double Cv = hv > comp ? hv : comp;
                            if (comm > Cv) Cv = comm;
                            if (Cv < h[IDX(j, S2, v)]) {
                                h[IDX(j, S2, v)] = Cv;
                                pre[IDX(j, S2, v)] = i * 32 + u;
                            }
                        }
                    }
                }
            }
        }
    }
    if (answer == INFINITY) { free(h); free(pre); return 1; }
    *t_opt = answer;

    /* back-trace: stages are found last to first */
    int32_t cnt = 0, end = L, i = ans_i, u = ans_u;
    int64_t S = ans_S;
    int32_t rdev[32], rfirst[32], rlast[32];
    for (;;) {
        rdev[cnt] = u; rfirst[cnt] = i; rlast[cnt] = end - 1; ++cnt;
        if (i == 0) break;
        int32_t p = pre[IDX(i, S, u)];
        int32_t pi = p / 32, pu = p % 32;
        end = i;
        S &= ~((int64_t)1 << pu);
        i = pi; u = pu;
    }
    *n_stages = cnt;
    for (int32_t s = 0; s < cnt; ++s) {
        stage_dev[s] = rdev[cnt - 1 - s];
        stage_first[s] = rfirst[cnt - 1 - s];
        stage_last[s] = rlast[cnt - 1 - s];
    }
    free(h); free(pre);
    return 0;
#undef IDX
}

/*
 * CPU oracle for the sequential planner of Algorithm 1: TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the CPU-baseline leg of the benchmark may call this
 * file.  It shares no code with the HIP library and the library never calls it.
 *
 * What it computes (Algorithm 1, "Link Load Balancing w. Iterative Approximation"): link loads
 * L_e and link costs c_e start at zero and every pair (s, d) starts with its whole workload as
 * remainder r.  While any remainder is left, the pairs are swept in order; a pair with r > 0
 *   1. scans its candidate paths in list order (direct, one relay, NIC paths: the order of the
 *      candidate CSR) for the lowest bottleneck cost  c(P) = max_{e in P} c_e,  strict `<`, so
 *      ties keep the earlier candidate;
 *   2. routes  f = r              if r < chi            (the residual),
 *              f = chi * floor(r * phi / chi)   otherwise  (a multiple of the chunk chi);
 *   3. if f > 0: adds f to the flow of that path, L_e += f and c_e = F(L_e) on its links, and
 *      subtracts f from r.
 * The update is immediate (Gauss-Seidel): the next pair of the same sweep already sees it.
 * Outputs: the flow in bytes routed on every candidate path (the per-pair path and flow lists
 * of the algorithm, summed per path), lambda = max_e L_e / cap_e, and the number of sweeps.
 *
 * Readings, where the listing is silent:
 *   - F(L_e) = L_e / cap_e (capacity-normalized load; the text only says that F penalises
 *     loaded links), evaluated as L_e * (1 / cap_e);
 *   - the listing calls the routed fraction lambda and the chunk epsilon; here they are phi
 *     and chi, because lambda and eps name the congestion and the step elsewhere;
 *   - when r >= chi but r * phi < chi the listed rule routes nothing and the loop would never
 *     end: such a pair routes one chunk, f = chi;
 *   - max_sweeps bounds the loop (returns 2 when it is hit).
 *
 * Every floating-point statement is one IEEE-754 binary64 operation (-ffp-contract=off).
 *
 * Pins (tests/test_alg1_pins.py): a four-sweep example worked by hand, conservation and chunk
 * multiples, the Gauss-Seidel schedule on two identical pairs, bottleneck (not additive) path
 * cost, phi = 1, the single-chunk rule, zero traffic, and brute-force agreement with a
 * line-by-line Python transcription of the steps above on tiny random inputs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

int nimble_oracle_alg1(int32_t n_links, const double *cap, int32_t n_comm,
                       const int32_t *comm_path_ptr, int32_t n_paths,
                       const int32_t *path_link_ptr, const int32_t *path_links,
                       const double *demand, double phi, double chi, int32_t max_sweeps,
                       double *flows, double *lambda_out, int32_t *sweeps_out, double *load_out)
{
    if (n_links < 1 || n_comm < 0 || n_paths < 0 || !(phi > 0.0) || !(phi <= 1.0) ||
        !(chi > 0.0) || max_sweeps < 1)
        return 1;
    double *L = (double *)calloc((size_t)n_links, sizeof(double));
    double *c = (double *)calloc((size_t)n_links, sizeof(double));
    double *invcap = (double *)malloc((size_t)n_links * sizeof(double));
    double *r = (double *)malloc((size_t)(n_comm > 0 ? n_comm : 1) * sizeof(double));
    if (!L || !c || !invcap || !r) {
        free(L); free(c); free(invcap); free(r);
        return 3;
    }
    for (int32_t e = 0; e < n_links; ++e) invcap[e] = 1.0 / cap[e];
    for (int32_t k = 0; k < n_comm; ++k) r[k] = demand[k];
    for (int32_t p = 0; p < n_paths; ++p) flows[p] = 0.0;
    int32_t sweeps = 0;
    int rc = 0;
    for (;;) {
        int any = 0;
        for (int32_t k = 0; k < n_comm; ++k)
            if (r[k] > 0.0) any = 1;
        if (!any) break;
        if (sweeps == max_sweeps) {
            rc = 2;
            break;
        }
        sweeps += 1;
        for (int32_t k = 0; k < n_comm; ++k) {
            if (!(r[k] > 0.0)) continue;
            double c_best = INFINITY;
            int32_t p_best = -1;
            for (int32_t p = comm_path_ptr[k]; p < comm_path_ptr[k + 1]; ++p) {
                double cp = 0.0;                       /* costs are >= 0: max starts at 0 */
                for (int32_t i = path_link_ptr[p]; i < path_link_ptr[p + 1]; ++i) {
                    const double ce = c[path_links[i]];
                    if (ce > cp) cp = ce;
                }
                if (cp < c_best) {
                    c_best = cp;
                    p_best = p;
                }
            }
            if (p_best < 0) continue;                  /* a pair without candidates */
            double f;
            if (r[k] < chi) {
                f = r[k];
            } else {
                const double want = r[k] * phi;
                const double chunks = floor(want / chi);
                f = chunks * chi;
                if (!(f > 0.0)) f = chi;
            }
            flows[p_best] = flows[p_best] + f;
            for (int32_t i = path_link_ptr[p_best]; i < path_link_ptr[p_best + 1]; ++i) {
                const int32_t e = path_links[i];
                L[e] = L[e] + f;
                c[e] = L[e] * invcap[e];
            }
            r[k] = r[k] - f;
        }
    }
    double lam = 0.0;
    for (int32_t e = 0; e < n_links; ++e) {
        const double u = L[e] * invcap[e];
        if (u > lam) lam = u;
        if (load_out) load_out[e] = L[e];
    }
    *lambda_out = lam;
    *sweeps_out = sweeps;
    free(L); free(c); free(invcap); free(r);
    return rc;
}

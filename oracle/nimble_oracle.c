/*
 * CPU oracle for the execution-time planner: TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the CPU-baseline leg of the benchmark may call this
 * file.  It shares no code with the HIP library and the library never calls it.
 *
 * What it computes.  The planner's problem is the minimum-congestion routing of Eq. (1)-(5)
 * (Sec. IV-B), read in its fractional, path-based, capacity-normalized form (the abstract and
 * Sec. III-C call the objective "capacity-normalized"): links e with capacity cap_e,
 * commodities k with demand d_k and a fixed list of candidate paths, find split fractions
 * minimising  lambda = max_e (1/cap_e) * sum_{paths p through e} d_k(p) x_p.
 * The method is the multiplicative-weights scheme the section cites (Garg-Koenemann):
 * route on the currently cheapest candidate, then raise the cost of loaded links.  The
 * candidate scan uses strict `<` in list order, as Algorithm 1 does, so ties go to the
 * lowest path index.  Link loads accumulate as in Algorithm 1 (L_e <- L_e + f).
 *
 * Schedule and cost function (the paper gives no formula for F(L_e)):
 *   - Jacobi: every commodity of an iteration is routed against the same link lengths.
 *   - length update  len_e <- len_e * (1 + eps * u_e / rho),  u_e = load_e / cap_e,
 *     rho = max_e (sum of demands of commodities that can reach e) / cap_e, so the
 *     normalised load u_e / rho lies in [0, 1].
 *   - price_e = len_e / cap_e; path cost = sum of prices (flag 0) or, as in Sec. IV-B's
 *     bottleneck rule, price_e = len_e and path cost = max of prices (flag 1).
 *   - outputs: splits_p = (times p was chosen) / iters, lambda = max_e (sum_t u_e^t) / iters.
 *
 * Every floating-point statement below is one IEEE-754 binary64 operation (compile with
 * -ffp-contract=off); the loops are the definition written out, with no blocking or
 * reordering.  OpenMP is used only over commodities in the cheapest-path scan, where the
 * iterations are independent, so results do not depend on the thread count.
 *
 * Pins (tests/test_oracle_pins.py): equal and unequal parallel links (closed forms), uniform
 * traffic on a full mesh, single-path topologies (static congestion), single hot pair on a
 * mesh / on rails, invariants, power-of-two scaling and link relabelling, an exact LP optimum
 * from a dense simplex on tiny inputs, the weak-duality lower bound, and a hand-worked
 * bottleneck-mode trajectory on two links of unequal capacity (price = len, initially too).
 * tests/test_oracle_mutations.py alters one statement at a time in a copy of this file and
 * checks that the pins notice.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_COST_MAX 1u

int nimble_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void nimble_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * Returns 0 on success, 1 on invalid arguments, 2 on allocation failure.
 * Optional outputs (may be NULL): count_out[n_paths] times each path was chosen;
 * sumload_out[n_links] = sum over iterations of u_e; lb_out[iters] = weak-duality lower
 * bound on the LP optimum after each iteration's routing step (sum cost only).
 */
/*
 * len_io (may be NULL): link lengths to start from and, on return, the lengths after the last
 * iteration.  NULL starts from len = 1, the plain method.  Starting a solve from the lengths a
 * previous solve ended with continues that solve's price trajectory: the "hysteresis" policy of
 * Sec. I (path selection must not oscillate between consecutive plans) read as a warm start.
 */
int nimble_oracle_solve_warm(int32_t n_links, const double *cap,
                             int32_t n_comm, const int32_t *comm_path_ptr,
                             int32_t n_paths, const int32_t *path_link_ptr,
                             const int32_t *path_links,
                             const double *demand, double eps, int32_t iters, uint32_t flags,
                             double *len_io, double *splits, double *lambda,
                             uint32_t *count_out, double *sumload_out, double *lb_out);

int nimble_oracle_solve(int32_t n_links, const double *cap,
                        int32_t n_comm, const int32_t *comm_path_ptr,
                        int32_t n_paths, const int32_t *path_link_ptr,
                        const int32_t *path_links,
                        const double *demand, double eps, int32_t iters, uint32_t flags,
                        double *splits, double *lambda,
                        uint32_t *count_out, double *sumload_out, double *lb_out)
{
    return nimble_oracle_solve_warm(n_links, cap, n_comm, comm_path_ptr, n_paths, path_link_ptr,
                                    path_links, demand, eps, iters, flags, NULL, splits, lambda,
                                    count_out, sumload_out, lb_out);
}

int nimble_oracle_solve_warm(int32_t n_links, const double *cap,
                             int32_t n_comm, const int32_t *comm_path_ptr,
                             int32_t n_paths, const int32_t *path_link_ptr,
                             const int32_t *path_links,
                             const double *demand, double eps, int32_t iters, uint32_t flags,
                             double *len_io, double *splits, double *lambda,
                             uint32_t *count_out, double *sumload_out, double *lb_out)
{
    if (n_links < 1 || n_comm < 1 || n_paths < 1 || iters < 1 || !(eps > 0.0) || !cap ||
        !comm_path_ptr || !path_link_ptr || !path_links || !demand || !splits || !lambda)
        return 1;
    const int use_max = (flags & ORACLE_COST_MAX) != 0;
    const int E = n_links, K = n_comm, P = n_paths;

    double *invcap = malloc(sizeof(double) * E);
    double *reach = malloc(sizeof(double) * E);   /* demand that can reach e */
    double *len = malloc(sizeof(double) * E);
    double *price = malloc(sizeof(double) * E);
    double *S = malloc(sizeof(double) * E);
    double *load = malloc(sizeof(double) * E);
    double *best = malloc(sizeof(double) * K);
    int32_t *choice = malloc(sizeof(int32_t) * K);
    int32_t *stamp = malloc(sizeof(int32_t) * E);
    uint32_t *count = calloc(P, sizeof(uint32_t));
    if (!invcap || !reach || !len || !price || !S || !load || !best || !choice || !stamp ||
        !count) {
        free(invcap); free(reach); free(len); free(price); free(S); free(load); free(best);
        free(choice); free(stamp); free(count);
        return 2;
    }

    for (int e = 0; e < E; ++e) {
        invcap[e] = 1.0 / cap[e];
        reach[e] = 0.0;
        stamp[e] = -1;
    }
    /* width rho: each commodity counted once per link it can use, commodities ascending */
    for (int k = 0; k < K; ++k)
        for (int p = comm_path_ptr[k]; p < comm_path_ptr[k + 1]; ++p)
            for (int i = path_link_ptr[p]; i < path_link_ptr[p + 1]; ++i) {
                int e = path_links[i];
                if (stamp[e] != k) {
                    stamp[e] = k;
                    reach[e] = reach[e] + demand[k];
                }
            }
    double rho = 0.0;
    for (int e = 0; e < E; ++e) {
        double w = reach[e] * invcap[e];
        if (w > rho) rho = w;
    }
    const double invrho = (rho > 0.0) ? 1.0 / rho : 0.0;

    for (int e = 0; e < E; ++e) {
        len[e] = len_io ? len_io[e] : 1.0;
        price[e] = use_max ? len[e] : len[e] * invcap[e];
        S[e] = 0.0;
    }

    for (int t = 0; t < iters; ++t) {
        /* cheapest candidate of every commodity under the same prices (Jacobi) */
#pragma omp parallel for schedule(static)
        for (int k = 0; k < K; ++k) {
            double cbest = INFINITY;
            int jbest = 0;
            const int p0 = comm_path_ptr[k];
            const int np = comm_path_ptr[k + 1] - p0;
            for (int j = 0; j < np; ++j) {
                const int p = p0 + j;
                double c = 0.0;
                for (int i = path_link_ptr[p]; i < path_link_ptr[p + 1]; ++i) {
                    double pe = price[path_links[i]];
                    if (use_max) {
                        if (pe > c) c = pe;
                    } else {
                        c = c + pe;
                    }
                }
                if (c < cbest) {
                    cbest = c;
                    jbest = j;
                }
            }
            choice[k] = jbest;
            best[k] = cbest;
            count[p0 + jbest] += 1u;
        }

        if (lb_out) {
            /* sum_k d_k * dist_k / sum_e len_e  <=  LP optimum (sum cost, price = len/cap) */
            double num = 0.0, den = 0.0;
            for (int k = 0; k < K; ++k) num += demand[k] * best[k];
            for (int e = 0; e < E; ++e) den += len[e];
            lb_out[t] = use_max ? 0.0 : num / den;
        }

        /* link loads: commodities in ascending order add their demand along the chosen path */
        for (int e = 0; e < E; ++e) load[e] = 0.0;
        for (int k = 0; k < K; ++k) {
            const int p = comm_path_ptr[k] + choice[k];
            for (int i = path_link_ptr[p]; i < path_link_ptr[p + 1]; ++i) {
                int e = path_links[i];
                load[e] = load[e] + demand[k];
            }
        }

        /* congestion bookkeeping and multiplicative length update */
        for (int e = 0; e < E; ++e) {
            double u = load[e] * invcap[e];
            S[e] = S[e] + u;
            double g = u * invrho;
            double t1 = eps * g;
            double t2 = 1.0 + t1;
            len[e] = len[e] * t2;
            price[e] = use_max ? len[e] : len[e] * invcap[e];
        }
    }

    const double T = (double)iters;
    for (int p = 0; p < P; ++p) splits[p] = (double)count[p] / T;
    double smax = 0.0;
    for (int e = 0; e < E; ++e)
        if (S[e] > smax) smax = S[e];
    *lambda = smax / T;

    if (len_io) memcpy(len_io, len, sizeof(double) * E);
    if (count_out) memcpy(count_out, count, sizeof(uint32_t) * P);
    if (sumload_out) memcpy(sumload_out, S, sizeof(double) * E);

    free(invcap); free(reach); free(len); free(price); free(S); free(load); free(best);
    free(choice); free(stamp); free(count);
    return 0;
}

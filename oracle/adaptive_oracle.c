/*
 * CPU oracle for the adaptive-step variant of the planner: TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the CPU-baseline leg of the benchmark may call this
 * file.  It shares no code with the HIP library and the library never calls it.
 *
 * What it computes.  The same problem and the same Jacobi candidate scan as nimble_oracle.c
 * (minimum-congestion routing of Sec. IV-B by the multiplicative-weights scheme of Garg and
 * Koenemann that the section cites), with the two refinements of that scheme that make it stop
 * as soon as the plan is good enough:
 *
 *   adaptive step    sigma_t = 1 / max_e u_e^t  (u_e^t = load_e^t / cap_e): the most loaded
 *                    link of every iteration grows by the full factor 1 + eps,
 *                      len_e <- len_e * (1 + eps * (u_e^t * sigma_t));
 *                    the plan is the sigma-weighted average of the iterations' routings:
 *                      S_e += sigma_t * u_e^t,  W += sigma_t,
 *                      splits_p = (sum of sigma_t over the iterations that chose p) / W,
 *                      lambda   = max_e S_e / W.
 *   early stop       every check_every iterations the weak-duality bound
 *                      LB_t = alpha_t / D_t,  alpha_t = sum_k d_k * (cost of k's cheapest
 *                      candidate under the prices of iteration t),  D_t = sum_e len_e,
 *                    (sum cost, price = len / cap: D is the price-weighted capacity) is a lower
 *                    bound on the optimum; the solve stops once
 *                      lambda_t <= (1 + eps)^2 * max_{checks so far} LB.
 *
 * alpha and D are sums of many terms; so that a parallel machine can reproduce them bit for
 * bit their association is fixed: terms in index order (commodities, links by id), summed
 * sequentially inside chunks of 256 consecutive terms, the chunk sums then added sequentially.
 * Every other statement is one IEEE binary64 operation as in nimble_oracle.c
 * (-ffp-contract=off).  A solve with all-zero traffic ends at once with lambda = 0.
 *
 * Readings: the paper cites the scheme and fixes neither the step nor a stopping rule; this is
 * the textbook variable-step form (step = 1 / largest normalised load, weighted average,
 * duality gap as the certificate).  Bottleneck-cost mode (flag 1) has no such bound: there
 * the solve runs max_iters iterations.
 *
 * Pins (tests/test_adaptive_pins.py): the switch iteration on two parallel links worked by
 * hand, LB <= LP optimum <= lambda on tiny instances (exact simplex), the stopping guarantee,
 * splits summing to 1, fewer iterations than the fixed-step method for the same gap, zero
 * traffic, the chunked sum against math.fsum, the bottleneck-mode price (hand-worked, unequal
 * capacities), and the stop iteration under a plain sequential sum
 * (tests/test_oracle_mutations.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ADAPTIVE_CHUNK 256

/* sum of x[0..n): sequential inside chunks of ADAPTIVE_CHUNK terms, chunk sums sequential */
static double chunked_sum(const double *x, int64_t n)
{
    double total = 0.0;
    for (int64_t c = 0; c < n; c += ADAPTIVE_CHUNK) {
        const int64_t end = c + ADAPTIVE_CHUNK < n ? c + ADAPTIVE_CHUNK : n;
        double s = 0.0;
        for (int64_t i = c; i < end; ++i) s = s + x[i];
        total = total + s;
    }
    return total;
}

double nimble_oracle_chunked_sum(const double *x, int64_t n) { return chunked_sum(x, n); }

/*
 * Returns 0 on success, 1 on invalid arguments, 2 on allocation failure.
 * iters_out: iterations made.  lb_out: best lower bound seen (0 if never checked).
 * Optional (may be NULL): weight_out[n_paths] the sigma sums per path, sigma_out[max_iters].
 */
int nimble_oracle_solve_adaptive(int32_t n_links, const double *cap, int32_t n_comm,
                                 const int32_t *comm_path_ptr, int32_t n_paths,
                                 const int32_t *path_link_ptr, const int32_t *path_links,
                                 const double *demand, double eps, int32_t max_iters,
                                 int32_t check_every, uint32_t flags, double *splits,
                                 double *lambda, int32_t *iters_out, double *lb_out,
                                 double *weight_out, double *sigma_out)
{
    if (n_links < 1 || n_comm < 1 || n_paths < 1 || max_iters < 1 || check_every < 1 ||
        !(eps > 0.0) || !cap || !comm_path_ptr || !path_link_ptr || !path_links || !demand ||
        !splits || !lambda || !iters_out || !lb_out)
        return 1;
    const int use_max = (flags & 1u) != 0;
    const int E = n_links, K = n_comm, P = n_paths;
    double *invcap = malloc(sizeof(double) * E);
    double *len = malloc(sizeof(double) * E);
    double *price = malloc(sizeof(double) * E);
    double *S = calloc(E, sizeof(double));
    double *load = malloc(sizeof(double) * E);
    double *u = malloc(sizeof(double) * E);
    double *best = malloc(sizeof(double) * K);
    double *term = malloc(sizeof(double) * K);
    int32_t *choice = malloc(sizeof(int32_t) * K);
    double *weight = calloc(P, sizeof(double));
    if (!invcap || !len || !price || !S || !load || !u || !best || !term || !choice || !weight) {
        free(invcap); free(len); free(price); free(S); free(load); free(u); free(best);
        free(term); free(choice); free(weight);
        return 2;
    }
    for (int e = 0; e < E; ++e) {
        invcap[e] = 1.0 / cap[e];
        len[e] = 1.0;
        price[e] = use_max ? 1.0 : invcap[e];
    }
    double W = 0.0, lb_best = 0.0, lam = 0.0;
    int32_t t = 0;
    const double gap = (1.0 + eps) * (1.0 + eps);
    while (t < max_iters) {
        /* cheapest candidate of every commodity under the same prices (Jacobi); the
           commodities are independent, so the threads change nothing */
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
                    const double pe = price[path_links[i]];
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
        }
        /* lower bound under the prices the choices were made with */
        const int check = ((t + 1) % check_every) == 0 && !use_max;
        double lb_t = 0.0;
        if (check) {
            for (int k = 0; k < K; ++k) term[k] = demand[k] * best[k];
            const double alpha = chunked_sum(term, K);
            const double D = chunked_sum(len, E);
            lb_t = alpha / D;
        }
        /* link loads and normalised loads */
        for (int e = 0; e < E; ++e) load[e] = 0.0;
        for (int k = 0; k < K; ++k) {
            const int p = comm_path_ptr[k] + choice[k];
            for (int i = path_link_ptr[p]; i < path_link_ptr[p + 1]; ++i) {
                const int e = path_links[i];
                load[e] = load[e] + demand[k];
            }
        }
        double umax = 0.0;
        for (int e = 0; e < E; ++e) {
            u[e] = load[e] * invcap[e];
            if (u[e] > umax) umax = u[e];
        }
        if (!(umax > 0.0)) break;                    /* no traffic at all */
        const double sigma = 1.0 / umax;
        if (sigma_out) sigma_out[t] = sigma;
        for (int k = 0; k < K; ++k) {
            const int p = comm_path_ptr[k] + choice[k];
            weight[p] = weight[p] + sigma;
        }
        W = W + sigma;
        double smax = 0.0;
        for (int e = 0; e < E; ++e) {
            const double su = sigma * u[e];
            S[e] = S[e] + su;
            if (S[e] > smax) smax = S[e];
            const double t1 = eps * su;
            const double t2 = 1.0 + t1;
            len[e] = len[e] * t2;
            price[e] = use_max ? len[e] : len[e] * invcap[e];
        }
        lam = smax / W;
        t += 1;
        if (check) {
            if (lb_t > lb_best) lb_best = lb_t;
            const double bound = gap * lb_best;
            if (lam <= bound) break;
        }
    }
    for (int p = 0; p < P; ++p) splits[p] = W > 0.0 ? weight[p] / W : 0.0;
    if (!(W > 0.0)) {
        /* no traffic: every commodity stays on its first candidate */
        for (int k = 0; k < K; ++k)
            if (comm_path_ptr[k + 1] > comm_path_ptr[k]) splits[comm_path_ptr[k]] = 1.0;
    }
    *lambda = lam;
    *iters_out = t;
    *lb_out = lb_best;
    if (weight_out) memcpy(weight_out, weight, sizeof(double) * P);
    free(invcap); free(len); free(price); free(S); free(load); free(u); free(best);
    free(term); free(choice); free(weight);
    return 0;
}

/*
 * nimble_plan.h -- C ABI of the MI355X execution-time planner.
 *
 * The planner solves the minimum-congestion routing problem of Eq. (1)-(5) (Sec. IV-B,
 * "Hop-Adaptive MCF load balancing") in its fractional, path-based, capacity-normalized form
 * with a Jacobi multiplicative-weights iteration (the Garg-Koenemann scheme the section
 * cites): every iteration routes each commodity on its currently cheapest candidate path
 * (strict `<` in list order, as the candidate scan of Algorithm 1), accumulates link loads
 * (Algorithm 1, L_e <- L_e + f), and multiplies the length of every link by
 * (1 + eps * u_e / rho), u_e = load_e / cap_e.  Outputs are the fraction of iterations each
 * candidate was chosen and the maximum link congestion lambda of that split.
 *
 * All arithmetic is IEEE binary64 without fused multiply-add.  Index arrays are int32.
 * "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory on the
 * GPU that was current when the topology was created.  The library never frees or keeps a
 * pointer the caller passed; nimble_topo_create copies what it needs.
 *
 * Threading: a nimble_topo_t owns one workspace, so at most ONE solve may be in flight per
 * topology at a time (enqueue the next solve on the same stream, or synchronise first).
 * nimble_last_error() is thread-local.
 */
#ifndef NIMBLE_PLAN_H
#define NIMBLE_PLAN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nimble_topo nimble_topo_t; /* opaque, owned by the library */

typedef enum {
    NIMBLE_OK = 0,
    NIMBLE_ERR_INVALID = 1, /* bad argument: null pointer, malformed CSR, eps/iters out of domain */
    NIMBLE_ERR_ALLOC = 2,   /* host or device allocation failed */
    NIMBLE_ERR_HIP = 3,     /* a HIP runtime call failed (message in nimble_last_error) */
    NIMBLE_ERR_RANGE = 4    /* valid input beyond a documented limit of this build */
} nimble_status_t;

/* flags of nimble_topo_create */
enum {
    NIMBLE_COST_SUM = 0u, /* path cost = sum of link prices, price = len/cap (default) */
    NIMBLE_COST_MAX = 1u, /* path cost = max of link prices, price = len: the bottleneck
                             rule of Sec. IV-B (intra-node 2-hop and inter-node path costs) */
    NIMBLE_LAYOUT_BATCH = 2u /* the topology will mostly solve batches of plans in the streaming
                             regime (nimble_topo_reserve_batch): lay the reverse CSR out for
                             launches that cover many plans (tuned for batches of about 16),
                             at the price of slower single plans on mid-size fabrics.
                             Results do not depend on it. */
};

/* kernel regimes, for nimble_topo_set_regime (testing and benchmarking) */
enum {
    NIMBLE_REGIME_AUTO = 0,     /* chosen from the problem size and the number of plans: resident
                                   when the per-plan state fits in LDS, unless so few plans of a
                                   fabric with long reverse rows are asked for that streaming
                                   them one after the other is faster */
    NIMBLE_REGIME_RESIDENT = 1, /* one workgroup per plan, whole iteration loop in one kernel,
                                   state in LDS */
    NIMBLE_REGIME_STREAM = 2,   /* one kernel per phase: two or three launches per iteration
                                   streaming the repacked CSRs */
    NIMBLE_REGIME_PERSISTENT = 3 /* one persistent kernel per solve with grid-wide barriers */
};

/*
 * Build a topology: links with capacities and, per commodity, the ordered list of candidate
 * paths as a two-level CSR (the sets E, K and the candidate paths of Sec. IV-B / Algorithm 1).
 *
 *   n_links        number of directed links, >= 1
 *   cap            host [n_links], bytes/s, finite and > 0
 *   n_comm         number of commodities (source-destination pairs), 1 <= n_comm < 2^24 - 1
 *   comm_path_ptr  host [n_comm+1], comm_path_ptr[0] = 0, strictly increasing,
 *                  comm_path_ptr[n_comm] = n_paths; commodity k owns candidate paths
 *                  comm_path_ptr[k] .. comm_path_ptr[k+1]-1, in tie-break order; at most 127
 *                  candidates per commodity
 *   n_paths        total number of candidate paths
 *   path_link_ptr  host [n_paths+1], path_link_ptr[0] = 0, strictly increasing
 *   path_links     host [path_link_ptr[n_paths]], link ids in [0, n_links), no link twice in
 *                  one path; the order inside a path is the order costs are added in
 *   flags          NIMBLE_COST_SUM or NIMBLE_COST_MAX, optionally | NIMBLE_LAYOUT_BATCH
 *   out            receives the handle; release it with nimble_topo_destroy
 *
 * Validation happens here, on the host, before any device call: malformed input returns
 * NIMBLE_ERR_INVALID, sizes beyond the limits above NIMBLE_ERR_RANGE.  The reverse
 * link -> (commodity, path) CSR is built here (stable counting sort, ascending
 * (commodity, path) inside every link) and uploaded with the forward CSR.
 */
nimble_status_t nimble_topo_create(int32_t n_links, const double *cap,
                                   int32_t n_comm, const int32_t *comm_path_ptr,
                                   int32_t n_paths, const int32_t *path_link_ptr,
                                   const int32_t *path_links,
                                   uint32_t flags, nimble_topo_t **out);

/* Frees device and host memory of the topology.  NULL is ignored.  The caller must make sure
 * no solve on this topology is still running. */
void nimble_topo_destroy(nimble_topo_t *topo);

/*
 * One plan: split fractions and maximum congestion for one demand vector (the All-to-Allv
 * byte matrix of Sec. III-A flattened to commodity order).
 *
 *   d_traffic   device [n_comm], bytes, finite and >= 0 (not checked: checking would need a
 *               host synchronisation).  Results are bit-identical to the sequential
 *               definition when demands are integer-valued with total < 2^53; otherwise they
 *               are still identical from run to run, with loads summed in a fixed tree order.
 *   eps         step size, 0 < eps <= 0.5
 *   iters       number of Jacobi iterations, >= 1, iters * log1p(eps) <= 700 (else lengths
 *               could overflow: NIMBLE_ERR_RANGE)
 *   d_splits    device [n_paths] out: times chosen / iters; sums to 1 per commodity
 *   d_lambda    device [1] out: max_e (1/cap_e) * sum_p d_k(p) splits_p, in seconds
 *               (NaN if the persistent regime abandoned the solve, see
 *               nimble_debug_set_spin_limit)
 *   hip_stream  hipStream_t (NULL = default stream).  The call only enqueues work; outputs are
 *               valid after the stream is synchronised.  No host synchronisation inside.
 * Nothing is allocated or freed here, so a caller may capture the call into a HIP graph on its
 * own stream.  The streaming regime records the choices of every iteration in the topology's
 * choice log when that holds `iters` rows (see nimble_topo_reserve) and counts the split
 * fractions from it once at the end; with a shorter log every iteration bumps a per-path
 * counter instead (same results, slower on large fabrics).
 */
nimble_status_t nimble_plan_solve(nimble_topo_t *topo, const double *d_traffic, double eps,
                                  int32_t iters, double *d_splits, double *d_lambda,
                                  void *hip_stream);

/*
 * Sizes the topology's choice log for streaming-regime solves of up to `iters` iterations
 * (one byte per commodity, rounded up to 512, and iteration).  nimble_topo_create reserves 1024
 * iterations by itself when that takes at most 64 MiB; larger fabrics or longer solves call
 * this once, outside the solve loop: it may free and allocate device memory, which
 * synchronises the device.  A log never shrinks.  NIMBLE_ERR_RANGE beyond 1 GiB,
 * NIMBLE_ERR_ALLOC when the memory cannot be had (the topology keeps working, with per-path
 * counters).
 */
nimble_status_t nimble_topo_reserve(nimble_topo_t *topo, int32_t iters);

/*
 * Makes room for `plans` plans of a batch to run side by side in the streaming regime: one
 * state block per plan (demand copies, lengths, prices, congestion sums, choices, counts,
 * partial sums) and a choice log of plans * iters rows.  nimble_plan_solve_batch then covers
 * that many plans with every kernel launch (a batch larger than the reservation is solved in
 * groups of that size; a topology starts with room for one plan).  Call it outside the solve
 * loop: it may free and allocate device memory.  NIMBLE_ERR_RANGE beyond 4 GiB of state or
 * 1 GiB of log, NIMBLE_ERR_ALLOC when the memory cannot be had.  Batches in the resident regime
 * need none of this.
 */
nimble_status_t nimble_topo_reserve_batch(nimble_topo_t *topo, int32_t plans, int32_t iters);

/*
 * nimble_plan_solve for callers that cannot allocate device memory and cannot let the library
 * do it either: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same results, always the streaming regime; the per-iteration
 * choice log lives in a buffer of nimble_static_scratch_bytes() bytes (32 MiB) that is part
 * of the library's device image -- every GPU the library runs on holds one until the process
 * ends -- instead of the topology's own log.  The call allocates and frees nothing and does
 * not synchronise.
 *   limit   (n_comm + 8 rounded up to 512) * iters <= nimble_static_scratch_bytes(), else
 *           NIMBLE_ERR_RANGE (1000 iterations of 16 256 commodities fit, of 261 632 do not)
 *   sharing all topologies on one GPU share the buffer: calls that overlap on one GPU (two
 *           streams, two threads) race on it; calls on one stream, one after the other, do not
 */
nimble_status_t nimble_plan_solve_static(nimble_topo_t *topo, const double *d_traffic, double eps,
                                         int32_t iters, double *d_splits, double *d_lambda,
                                         void *hip_stream);
int64_t nimble_static_scratch_bytes(void);

/*
 * `batch` independent plans on the same topology (one per MoE layer x micro-batch), solved
 * concurrently.  d_traffic is device [batch][n_comm], d_splits device [batch][n_paths],
 * d_lambda device [batch]; the rest as nimble_plan_solve.  batch >= 1.  Topologies whose
 * per-plan state does not fit in LDS run the streaming regime: as many plans share every
 * kernel launch as nimble_topo_reserve_batch has made room for (one after the other without
 * it).
 */
nimble_status_t nimble_plan_solve_batch(nimble_topo_t *topo, int32_t batch,
                                        const double *d_traffic, double eps, int32_t iters,
                                        double *d_splits, double *d_lambda, void *hip_stream);

/*
 * The sequential planner of Algorithm 1 ("Link Load Balancing w. Iterative Approximation",
 * Sec. IV-B), for `batch` independent problems on the same topology.  Per problem: link loads
 * and costs start at 0 and every pair's remainder at its demand; while any remainder is left
 * the pairs are swept in order, and a pair with remainder r > 0 takes the candidate with the
 * lowest bottleneck cost max_e F(L_e) (strict `<` in candidate order), routes f = r if r < chi,
 * else the largest multiple of chi that is <= r * phi (one chunk when that is 0), and adds f to
 * the loads of that candidate's links at once (the next pair sees it).  F(L_e) = L_e / cap_e.
 * A group of lanes (one per candidate of the current pair) runs one problem; topologies with
 * more than 64 candidates per pair, paths of more than 8 links, or tables beyond 64 KB of LDS
 * run one thread per problem.
 *
 *   d_traffic   device [batch][n_comm], bytes >= 0
 *   phi         routed fraction of the remainder per visit, 0 < phi <= 1
 *   chi         chunk granularity in bytes, > 0
 *   max_sweeps  bound on the sweeps of a problem, >= 1
 *   d_flows     device [batch][n_paths] out: bytes routed on every candidate path (the
 *               algorithm's per-pair path and flow lists, summed per path); the flows of a
 *               pair add up to its demand
 *   d_lambda    device [batch] out: max_e L_e / cap_e; NaN for a problem that still had
 *               traffic left after max_sweeps sweeps
 *   d_sweeps    device int32 [batch] out: sweeps made
 *   hip_stream  as for nimble_plan_solve: the call only enqueues work.
 * Errors: NIMBLE_ERR_INVALID for bad arguments; NIMBLE_ERR_RANGE when the topology fits neither
 * kernel: 8 x (n_links + n_comm) doubles exceed 150 KB (the per-problem state lives in LDS).
 * Results are bit-identical to the plain CPU definition for any demands.
 */
nimble_status_t nimble_alg1_solve_batch(nimble_topo_t *topo, int32_t batch,
                                        const double *d_traffic, double phi, double chi,
                                        int32_t max_sweeps, double *d_flows, double *d_lambda,
                                        int32_t *d_sweeps, void *hip_stream);

/*
 * nimble_plan_solve started from given link lengths (warm start) instead of len = 1, and
 * returning the lengths after the last iteration.  Consecutive plans of a changing workload
 * that hand the lengths on keep the price trajectory: links that were loaded stay expensive,
 * so path selection does not flip back at every new plan (the hysteresis policy named in
 * Sec. I, read as a warm start).  T1 iterations followed by T2 iterations from the returned
 * lengths make exactly the choices of one solve of T1 + T2 iterations.
 *
 *   d_len   device [n_links], by link id, in and out; every entry finite and > 0 (1.0
 *           everywhere is the cold start).  Lengths grow by at most (1 + eps) per iteration:
 *           the caller rescales them (e.g. by a power of two, which changes nothing else)
 *           before they can overflow.
 * The other arguments as for nimble_plan_solve.  Always runs the streaming regime; like
 * nimble_plan_solve it only enqueues work.
 */
nimble_status_t nimble_plan_solve_warm(nimble_topo_t *topo, const double *d_traffic, double eps,
                                       int32_t iters, double *d_len, double *d_splits,
                                       double *d_lambda, void *hip_stream);

/*
 * The adaptive-step variant of the method (the multiplicative-weights scheme Sec. IV-B cites,
 * in its variable-step form), which stops as soon as the plan is provably good enough:
 *   step        sigma_t = 1 / max_e u_e^t: the most loaded link of an iteration grows by the
 *               full factor 1 + eps;  len_e *= 1 + eps * sigma_t * u_e^t
 *   plan        the sigma-weighted average of the iterations' routings: splits_p = (sum of
 *               sigma_t over the iterations that chose p) / sum_t sigma_t, lambda likewise
 *   early stop  every check_every iterations the weak-duality bound
 *               LB = (sum_k d_k * cheapest cost of k) / (sum_e len_e)  <=  optimum  is taken
 *               (both sums in index order, sequential inside chunks of 256 terms, the chunk
 *               sums sequential); the solve stops once lambda <= (1 + eps)^2 * best LB.
 *               Bottleneck-cost topologies (NIMBLE_COST_MAX) have no such bound and run
 *               max_iters iterations.
 *
 *   max_iters    >= 1, max_iters * log1p(eps) <= 700
 *   check_every  >= 1
 *   d_splits, d_lambda   device outputs as for nimble_plan_solve
 *   iters_done   host out: iterations made (0 for all-zero traffic: every pair then stays on
 *                its first candidate)
 *   lower_bound  host out: best LB seen (0 if no check was made)
 * The stop decision is taken on the device; the host enqueues ahead and follows the device's
 * progress through two words of pinned memory, so the stream is never synchronised during the
 * solve (kernels enqueued after the stop return at once).  Unlike nimble_plan_solve the call
 * waits for the stream before it returns, because iters_done and lower_bound are host outputs,
 * and it cannot be captured into a graph.  Always runs the streaming regime; needs the per-iteration choice log of
 * max_iters rows and grows it when it is shorter (NIMBLE_ERR_ALLOC if it cannot be allocated,
 * NIMBLE_ERR_RANGE beyond 1 GiB), as well as a workspace of its own on the first call.
 * Bit-identical to the plain CPU definition for integer-valued demands.
 */
nimble_status_t nimble_plan_solve_adaptive(nimble_topo_t *topo, const double *d_traffic,
                                           double eps, int32_t max_iters, int32_t check_every,
                                           double *d_splits, double *d_lambda,
                                           int32_t *iters_done, double *lower_bound,
                                           void *hip_stream);

/*
 * Post-processing of a plan into what a dataplane consumes: bytes per candidate path in whole
 * chunks (the Paths / Flows lists of Algorithm 1), with the practical policies of Sec. I and
 * Sec. V-A: no fragmentation below the chunk granularity and no multi-hop forwarding of small
 * messages (1 MB or less in the paper).  Per pair with demand d and counts c_j = splits_j * iters:
 *   d <= small_threshold: everything on the pair's first candidate;
 *   otherwise N = floor(d / chi) whole chunks are apportioned by largest remainder (quota
 *   floor(N * c_j / iters); the chunks left over go to the largest remainders N * c_j mod iters,
 *   ties to the lower index) and the residual d - N * chi joins the candidate with the largest
 *   count (ties to the lower index).
 *
 *   d_traffic        device [n_comm], the demands the plan was solved for
 *   d_splits         device [n_paths], the output of nimble_plan_solve with the same iters
 *   iters            >= 1
 *   chi              chunk in bytes, 1 <= chi <= 2^40
 *   small_threshold  bytes, >= 0 (0: no pair is treated as small unless its demand is 0)
 *   d_flows          device [n_paths] out: bytes per candidate path; the flows of a pair add up
 *                    to its demand exactly (integer demands below 2^53).  A pair with
 *                    d / chi >= 2^31 gets NaN flows.
 * One batch entry per call; only enqueues work on hip_stream.  Bit-identical to the plain CPU
 * definition.
 */
nimble_status_t nimble_plan_quantize(nimble_topo_t *topo, const double *d_traffic,
                                     const double *d_splits, int32_t iters, int64_t chi,
                                     double small_threshold, double *d_flows, void *hip_stream);

/* Last error message of the calling thread ("" if none). Never NULL. */
const char *nimble_last_error(void);

/* Size queries. */
int32_t nimble_topo_num_links(const nimble_topo_t *topo);
int32_t nimble_topo_num_comm(const nimble_topo_t *topo);
int32_t nimble_topo_num_paths(const nimble_topo_t *topo);
int64_t nimble_topo_nnz(const nimble_topo_t *topo);

/* Bytes of the stored (device) representation that one iteration has to read or write:
 * forward CSR, reverse CSR, and the per-link / per-commodity state.  This is the numerator
 * of the bandwidth figure the benchmark reports. */
int64_t nimble_topo_bytes_per_iter(const nimble_topo_t *topo);

/* The same figure for one phase of the streaming regime (0: path-cost gather + argmin over
 * the forward CSR, 1: link-load reduce over the reverse CSR, 2: length update).  On topologies
 * whose reduce and update run as one kernel, phase 1 covers both and phase 2 is 0.  Phase 3 is
 * not memory traffic: the bytes the path-cost kernel reads from LDS per launch (one 8-byte
 * price per candidate step, or nine per four candidates that share their first and last
 * links pairwise), 0 for the kernels that do not keep the prices of a record in LDS lane by
 * lane. */
int64_t nimble_topo_phase_bytes(const nimble_topo_t *topo, int32_t phase);

/* Force a kernel regime (NIMBLE_REGIME_*) for later solves; NIMBLE_ERR_RANGE if the topology
 * does not fit that regime.  The regime actually used is returned by nimble_topo_regime. */
nimble_status_t nimble_topo_set_regime(nimble_topo_t *topo, int32_t regime);
int32_t nimble_topo_regime(const nimble_topo_t *topo);

#ifdef __cplusplus
}
#endif
#endif /* NIMBLE_PLAN_H */

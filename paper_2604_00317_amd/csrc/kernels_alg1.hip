// The sequential planner of Algorithm 1 ("Link Load Balancing w. Iterative Approximation"),
// batched: one thread per problem, all problems on the same topology.
//
// The algorithm is a Gauss-Seidel sweep -- every routed chunk changes the link costs the next
// pair sees -- so one problem offers no parallelism beyond its candidate scan; a batch of
// problems does.  A thread keeps the link loads L_e and the remainders r_k of its problem in
// LDS (entry-major, one column per thread: conflict-free; 64 problems per workgroup, fewer when
// the topology is larger), reads the candidate CSR through
// wave-uniform loads (all threads walk the same pairs, candidates and links), and follows
// the steps of the listing: bottleneck cost max_e c_e with c_e = F(L_e) = L_e / cap_e, strict
// `<` in candidate order, f = r if r < chi else chi * floor(r * phi / chi) (one chunk when that
// is zero), immediate update of L_e, until no remainder is left.  Every floating-point
// statement is one IEEE binary64 operation.
#include <hip/hip_runtime.h>

#include "kernels.hpp"
#include "wave_ops.hpp"

namespace nimble {

namespace {

constexpr int kAlg1Threads = 64;          // most problems per workgroup
constexpr int kAlg1MinThreads = 8;        // fewest: larger topologies leave less LDS per problem
constexpr size_t kAlg1LdsBudget = 150 * 1024;

__global__ __launch_bounds__(kAlg1Threads) void k_alg1(int E, int K, int P, int batch,
                                                        const int32_t *__restrict__ cp,
                                                        const int32_t *__restrict__ lp,
                                                        const int32_t *__restrict__ pl,
                                                        const double *__restrict__ invcap,
                                                        const double *__restrict__ demand,
                                                        double phi, double chi, int max_sweeps,
                                                        double *__restrict__ flows,
                                                        double *__restrict__ lambda,
                                                        int32_t *__restrict__ sweeps_out)
{
    extern __shared__ double s_state[];              // L[E][T], then r[K][T], T = blockDim.x
    const int t = threadIdx.x;
    const int T = blockDim.x;
    const int b = blockIdx.x * T + t;
    const bool live = b < batch;
    double *L = s_state + t;
    double *r = s_state + size_t(E) * T + t;
    for (int e = 0; e < E; ++e) L[e * T] = 0.0;
    for (int k = 0; k < K; ++k) r[k * T] = live ? demand[size_t(b) * K + k] : 0.0;
    double *my_flows = flows + size_t(live ? b : 0) * P;
    if (live)
        for (int p = 0; p < P; ++p) my_flows[p] = 0.0;
    int sweeps = 0;
    bool gave_up = false;
    for (;;) {
        bool any = false;
        for (int k = 0; k < K; ++k) any = any || r[k * T] > 0.0;
        if (!any) break;
        if (sweeps == max_sweeps) {
            gave_up = true;
            break;
        }
        sweeps += 1;
        for (int k = 0; k < K; ++k) {                // the same pair in every thread
            const double rk = r[k * T];
            if (!(rk > 0.0)) continue;
            double c_best = __builtin_inf();
            int p_best = -1;
            const int pa = cp[k], pb = cp[k + 1];
            for (int p = pa; p < pb; ++p) {
                double c_path = 0.0;                 // costs are >= 0: the max starts at 0
                const int la = lp[p], lb = lp[p + 1];
                for (int i = la; i < lb; ++i) {
                    const int e = pl[i];
                    const double ce = L[e * T] * invcap[e];
                    if (ce > c_path) c_path = ce;
                }
                if (c_path < c_best) {
                    c_best = c_path;
                    p_best = p;
                }
            }
            if (p_best < 0) continue;                // a pair without candidates
            double f;
            if (rk < chi) {
                f = rk;
            } else {
                const double want = rk * phi;
                const double chunks = floor(want / chi);
                f = chunks * chi;
                if (!(f > 0.0)) f = chi;
            }
            my_flows[p_best] = my_flows[p_best] + f;
            const int la = lp[p_best], lb = lp[p_best + 1];
            for (int i = la; i < lb; ++i) {
                const int e = pl[i];
                L[e * T] = L[e * T] + f;
            }
            r[k * T] = rk - f;
        }
    }
    if (live) {
        double lam = 0.0;
        for (int e = 0; e < E; ++e) {
            const double u = L[e * T] * invcap[e];
            if (u > lam) lam = u;
        }
        lambda[b] = gave_up ? __builtin_nan("") : lam;
        sweeps_out[b] = sweeps;
    }
}

}  // namespace

// Problems per workgroup: the most (a power of two, at most 64) whose state fits the budget.
int alg1_threads(const DeviceTopo &t)
{
    const size_t per_problem = sizeof(double) * (static_cast<size_t>(t.E) + static_cast<size_t>(t.K));
    int threads = kAlg1Threads;
    while (threads > kAlg1MinThreads && per_problem * threads > kAlg1LdsBudget) threads >>= 1;
    return threads;
}

size_t alg1_lds_bytes(const DeviceTopo &t)
{
    return sizeof(double) * alg1_threads(t) * (static_cast<size_t>(t.E) + static_cast<size_t>(t.K));
}

bool alg1_fits(const DeviceTopo &t) { return alg1_lds_bytes(t) <= kAlg1LdsBudget; }

hipError_t launch_alg1(const DeviceTopo &t, int32_t batch, const double *demand, double phi,
                       double chi, int32_t max_sweeps, double *flows, double *lambda,
                       int32_t *sweeps, hipStream_t s)
{
    const size_t lds = alg1_lds_bytes(t);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_alg1),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(lds));
    if (e != hipSuccess) return e;
    const int threads = alg1_threads(t);
    const int grid = (batch + threads - 1) / threads;
    hipLaunchKernelGGL(k_alg1, dim3(grid), dim3(threads), lds, s, t.E, t.K, t.P, batch,
                       t.comm_ptr, t.path_ptr, t.path_links, t.invcap, demand, phi, chi,
                       max_sweeps, flows, lambda, sweeps);
    return hipGetLastError();
}

}  // namespace nimble

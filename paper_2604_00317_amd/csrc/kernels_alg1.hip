// The sequential planner of Algorithm 1 ("Link Load Balancing w. Iterative Approximation"),
// batched, all problems on the same topology.  Two kernels compute the same numbers: a group of
// G lanes per problem whose lanes cost the candidates of a pair side by side (k_alg1_group, up
// to 64 candidates per pair), and one thread per problem (k_alg1) for anything else.
//
// The algorithm is a Gauss-Seidel sweep -- every routed chunk changes the link costs the next
// pair sees -- so one problem offers no parallelism beyond its candidate scan; a batch of
// problems does.  A thread keeps the link loads L_e and the remainders r_k of its problem in
// LDS (entry-major, one column per thread: conflict-free; 64 problems per workgroup, fewer when
// the topology is larger), reads the candidate CSR through
// wave-uniform loads (all threads walk the same pairs, candidates and links), and sweeps the
// pairs as Algorithm 1 does: bottleneck cost max_e c_e with c_e = F(L_e) = L_e / cap_e, strict
// `<` in candidate order, f = r if r < chi else chi * floor(r * phi / chi) (one chunk when that
// is zero), immediate update of L_e, until no remainder is left.  Every floating-point
// statement is one IEEE binary64 operation.  Both kernels are tested against the hand-worked
// examples of the algorithm directly (tests/test_gpu_alg1.py), not only against the CPU oracle.
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


// G lanes per problem (G a power of two >= the most candidates of any pair, at most 64), 64 / G
// problems per wave.  The sweep over the pairs stays sequential -- every routed chunk changes
// the costs the next pair sees -- but lane j costs candidate j of the pair, the group takes the
// (cost, index) minimum by DPP (the lowest index among equal costs: the strict `<` of the
// sequential scan), and the winning lane routes the chunk.  A problem lives inside one wave, so
// its lanes are ordered by the wave's in-order LDS operations; workgroups never synchronise
// after the set-up (a workgroup is one wave).  LDS: the candidate table of the topology (per
// pair and lane, LM link ids padded with E, whose load and 1/capacity are 0) and 1/capacity
// once per workgroup, then L[E+1], r[K] and the flows f[P] per problem -- nothing in the sweep
// touches global memory.  All lanes walk all pairs, so a wave sweeps until the last of its
// problems is done.
template <int G, int LM>
__global__ __launch_bounds__(kWave) void k_alg1_group(int E, int K, int P, int batch,
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
    extern __shared__ __align__(16) double s_mem[];
    constexpr int kPerBlock = kWave / G;                      // problems of this wave
    const size_t per_problem = size_t(E) + 1 + K + P;
    double *s_ic = s_mem;                                     // [E + 1]
    double *s_state = s_ic + (E + 1);                         // per problem: L[E+1], r[K], f[P]
    int32_t *s_cp = reinterpret_cast<int32_t *>(s_state + kPerBlock * per_problem);   // [K + 1]
    int32_t *s_tab = s_cp + (K + 1);                          // [K][G][LM]
    for (int e = threadIdx.x; e <= E; e += kWave) s_ic[e] = e < E ? invcap[e] : 0.0;
    for (int k = threadIdx.x; k <= K; k += kWave) s_cp[k] = cp[k];
    for (int idx = threadIdx.x; idx < K * G; idx += kWave) {
        const int k = idx / G, jj = idx % G;
        const int p = cp[k] + jj;
        int la = 0, lb = 0;
        if (p < cp[k + 1]) {
            la = lp[p];
            lb = lp[p + 1];
        }
        for (int i = 0; i < LM; ++i) s_tab[size_t(idx) * LM + i] = la + i < lb ? pl[la + i] : E;
    }
    const int lane = threadIdx.x;
    const int j = lane % G;
    const int slot = lane / G;
    const int b = blockIdx.x * kPerBlock + slot;
    const bool live = b < batch;
    double *L = s_state + size_t(slot) * per_problem;
    double *r = L + (E + 1);
    double *fl = r + K;
    for (int e = j; e <= E; e += G) L[e] = 0.0;
    for (int k = j; k < K; k += G) r[k] = live ? demand[size_t(b) * K + k] : 0.0;
    for (int p = j; p < P; p += G) fl[p] = 0.0;
    __syncthreads();                                 // one wave: orders the set-up
    // lanes of this problem inside the wave
    const unsigned long long gmask = (G == 64 ? ~0ull : ((1ull << G) - 1ull)) << (lane - j);
    int sweeps = 0;
    bool gave_up = false, done = false;
    // the first pair's share of the topology
    int n_pa = s_cp[0], n_np = s_cp[1] - s_cp[0];
    int n_e[LM];
    double n_ic[LM];
#pragma unroll
    for (int i = 0; i < LM; ++i) {
        n_e[i] = s_tab[size_t(j) * LM + i];
        n_ic[i] = s_ic[n_e[i]];
    }
    for (;;) {
        bool mine = false;
        for (int k = j; k < K; k += G) mine = mine || r[k] > 0.0;
        const bool any = (__ballot(mine) & gmask) != 0ull;
        if (!done) {
            if (!any) done = true;
            else if (sweeps == max_sweeps) {
                gave_up = true;
                done = true;
            } else sweeps += 1;
        }
        if (__all(done)) break;                      // wave-uniform
        for (int k = 0; k < K; ++k) {                // the same pair in every lane
            // this pair's share of the topology was requested during the previous pair; the
            // next pair's (the first pair of the next sweep after the last) is requested now,
            // so that only the loads L_e -- which the previous pair may have changed -- are
            // waited for on the way to the argmin
            const int pa = n_pa, np = n_np;
            int e[LM];
            double ice[LM];
#pragma unroll
            for (int i = 0; i < LM; ++i) {
                e[i] = n_e[i];
                ice[i] = n_ic[i];
            }
            {
                const int kn = k + 1 < K ? k + 1 : 0;
                n_pa = s_cp[kn];
                n_np = s_cp[kn + 1] - n_pa;
                const int32_t *tab = s_tab + (size_t(kn) * G + j) * LM;
#pragma unroll
                for (int i = 0; i < LM; ++i) n_e[i] = tab[i];
#pragma unroll
                for (int i = 0; i < LM; ++i) n_ic[i] = s_ic[n_e[i]];
            }
            const double rk = r[k];
            double Lv[LM];
#pragma unroll
            for (int i = 0; i < LM; ++i) Lv[i] = L[e[i]];
            // the amount depends on the remainder only: every lane works it out while the
            // loads arrive and the argmin runs (the division is the longest chain of the step)
            double f = rk;
            {
                const double want = rk * phi;
                const double chunks = floor(want / chi);
                double fc = chunks * chi;
                if (!(fc > 0.0)) fc = chi;
                if (!(rk < chi)) f = fc;
            }
            double c = 0.0;                          // costs are >= 0: the max starts at 0
#pragma unroll
            for (int i = 0; i < LM; ++i) {           // padding steps cost 0 * 0
                const double ce = Lv[i] * ice[i];
                if (ce > c) c = ce;
            }
            if (j >= np) c = __builtin_inf();
            const int bj = group_argmin_two_pass<G>(c, j);
            if (!done && rk > 0.0 && np > 0 && j == bj) {
                fl[pa + bj] = fl[pa + bj] + f;
#pragma unroll
                for (int i = 0; i < LM; ++i)
                    if (e[i] < E) L[e[i]] = Lv[i] + f;
                r[k] = rk - f;
            }
            // the next pair sees the loads this one left
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
    if (live) {
        double *out = flows + size_t(b) * P;
        for (int p = j; p < P; p += G) out[p] = fl[p];
    }
    double lam = 0.0;
    for (int e = j; e < E; e += G) {
        const double u = L[e] * s_ic[e];
        if (u > lam) lam = u;
    }
    if constexpr (G > 1) lam = fmax(lam, partner_f64<1>(lam));
    if constexpr (G > 2) lam = fmax(lam, partner_f64<2>(lam));
    if constexpr (G > 4) lam = fmax(lam, partner_f64<4>(lam));
    if constexpr (G > 8) lam = fmax(lam, partner_f64<8>(lam));
    if constexpr (G > 16) lam = fmax(lam, partner_f64<16>(lam));
    if constexpr (G > 32) lam = fmax(lam, partner_f64<32>(lam));
    if (live && j == 0) {
        lambda[b] = gave_up ? __builtin_nan("") : lam;
        sweeps_out[b] = sweeps;
    }
}

constexpr size_t kAlg1GroupLds = 64 * 1024;      // no opt-in needed below this

// link ids per candidate in the table of k_alg1_group: 2 or 8
int alg1_group_steps(const DeviceTopo &t) { return t.lmax <= 2 ? 2 : 8; }

// lanes per problem of k_alg1_group, or 0 if the topology does not fit it
int alg1_group_lanes(const DeviceTopo &t, size_t &lds)
{
    if (t.alg1_thread_per_problem || t.pmax > kWave || t.pmax < 1 || t.lmax > 8 || t.K < 1)
        return 0;
    const int G = lanes_per_commodity(t.pmax);
    const size_t per_block = kWave / G;
    lds = sizeof(double) * (t.E + 1) +
          sizeof(double) * per_block * (static_cast<size_t>(t.E) + 1 + t.K + t.P) +
          sizeof(int32_t) * (t.K + 1) +
          sizeof(int32_t) * static_cast<size_t>(t.K) * G * alg1_group_steps(t);
    return lds <= kAlg1GroupLds ? G : 0;
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

bool alg1_fits(const DeviceTopo &t)
{
    size_t lds = 0;
    return alg1_group_lanes(t, lds) > 0 || alg1_lds_bytes(t) <= kAlg1LdsBudget;
}

hipError_t launch_alg1(const DeviceTopo &t, int32_t batch, const double *demand, double phi,
                       double chi, int32_t max_sweeps, double *flows, double *lambda,
                       int32_t *sweeps, hipStream_t s)
{
    size_t glds = 0;
    const int G = alg1_group_lanes(t, glds);
    if (G > 0) {
        const int per_block = kWave / G;
        const int ggrid = (batch + per_block - 1) / per_block;
        const bool two = alg1_group_steps(t) == 2;
#define NIMBLE_ALG1_ARGS                                                                       \
    dim3(ggrid), dim3(kWave), glds, s, t.E, t.K, t.P, batch, t.comm_ptr, t.path_ptr,           \
        t.path_links, t.invcap, demand, phi, chi, max_sweeps, flows, lambda, sweeps
#define NIMBLE_ALG1_LAUNCH(GG)                                                                 \
    case GG:                                                                                   \
        if (two) hipLaunchKernelGGL((k_alg1_group<GG, 2>), NIMBLE_ALG1_ARGS);                  \
        else hipLaunchKernelGGL((k_alg1_group<GG, 8>), NIMBLE_ALG1_ARGS);                      \
        return hipGetLastError();
        switch (G) {
            NIMBLE_ALG1_LAUNCH(1)
            NIMBLE_ALG1_LAUNCH(2)
            NIMBLE_ALG1_LAUNCH(4)
            NIMBLE_ALG1_LAUNCH(8)
            NIMBLE_ALG1_LAUNCH(16)
            NIMBLE_ALG1_LAUNCH(32)
            NIMBLE_ALG1_LAUNCH(64)
        }
#undef NIMBLE_ALG1_LAUNCH
#undef NIMBLE_ALG1_ARGS
    }
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

// Resident regime: one group of NT threads per plan, the whole Jacobi loop inside one kernel,
// per-plan state (prices, lengths, congestion sums, demands, choices, counts) in LDS.  Several
// plans share a workgroup and, when it fits, one LDS copy of the topology.  This is the path of
// the batched solve (one plan per MoE layer x micro-batch) and of small single plans.
//
// Per iteration: each thread scans the candidates of its commodities in list order with a
// strict `<` (Algorithm 1's scan), then each thread walks the reverse rows of its links in
// ascending (commodity, path) order -- the sequential order of Algorithm 1's L_e += f -- and
// applies the multiplicative length update.  Reverse rows hold (commodity, window | mask) pairs,
// ascending by commodity, of which at most one per commodity can hit.  Two workgroup barriers per iteration.
#include "host_topo.hpp"
#include "kernels.hpp"
#include "wave_ops.hpp"

namespace nimble {

namespace {

constexpr size_t kLdsBudget = 64 * 1024;   // static + dynamic LDS a kernel may use without opt-in
constexpr int kMaxPlansPerBlock = 4;

struct ResidentLayout {
    // offsets in bytes from the start of dynamic LDS; per-plan block first, topology last
    size_t price, len, S, demand, count, choice, plan_bytes;
    size_t topo_bytes;
};

__host__ __device__ inline size_t align8(size_t x) { return (x + 7) & ~size_t(7); }

__host__ __device__ inline ResidentLayout make_layout(int E, int K, int P, int64_t nnz,
                                                      int64_t rev_len /* pairs */)
{
    ResidentLayout l;
    size_t o = 0;
    l.price = o;  o += sizeof(double) * E;
    l.len = o;    o += sizeof(double) * E;
    l.S = o;      o += sizeof(double) * E;
    l.demand = o; o += sizeof(double) * K;
    l.count = o;  o += align8(sizeof(uint32_t) * P);
    l.choice = o; o += align8(K + 1);
    l.plan_bytes = o;
    l.topo_bytes = align8(sizeof(int32_t) * (K + 1)) + align8(sizeof(int32_t) * (P + 1)) +
                   align8(sizeof(int32_t) * nnz) + align8(sizeof(int32_t) * (E + 1)) +
                   align8(sizeof(uint32_t) * 2 * rev_len) + sizeof(double) * E;
    return l;
}

template <bool MAXC, bool TOPO_LDS>
__global__ __launch_bounds__(1024) void k_resident(
    int E, int K, int P, int nnz, int rev_len, int batch, int nt, int plans_per_block,
    double eps, int iters,
    const int32_t *__restrict__ g_cp, const int32_t *__restrict__ g_lp,
    const int32_t *__restrict__ g_pl, const int32_t *__restrict__ g_rp,
    const uint32_t *__restrict__ g_rev, const double *__restrict__ g_invcap,
    const double *__restrict__ demand_all, double *__restrict__ splits_all,
    double *__restrict__ lambda_all)
{
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ double red[16];
    __shared__ double s_invrho[kMaxPlansPerBlock];

    const ResidentLayout lay = make_layout(E, K, P, nnz, rev_len);
    const int slot = threadIdx.x / nt;            // plan slot inside the workgroup
    const int t = threadIdx.x - slot * nt;        // thread inside the plan group
    const int plan = blockIdx.x * plans_per_block + slot;
    const bool live = plan < batch;

    unsigned char *mine = lds + lay.plan_bytes * slot;
    double *price = reinterpret_cast<double *>(mine + lay.price);
    double *len = reinterpret_cast<double *>(mine + lay.len);
    double *S = reinterpret_cast<double *>(mine + lay.S);
    double *demand = reinterpret_cast<double *>(mine + lay.demand);
    uint32_t *count = reinterpret_cast<uint32_t *>(mine + lay.count);
    uint8_t *choice = mine + lay.choice;

    const int32_t *cp = g_cp, *lp = g_lp, *pl = g_pl, *rp = g_rp;
    const uint32_t *rev = g_rev;
    const double *invcap = g_invcap;
    if constexpr (TOPO_LDS) {
        unsigned char *tb = lds + lay.plan_bytes * plans_per_block;
        int32_t *s_cp = reinterpret_cast<int32_t *>(tb);
        tb += align8(sizeof(int32_t) * (K + 1));
        int32_t *s_lp = reinterpret_cast<int32_t *>(tb);
        tb += align8(sizeof(int32_t) * (P + 1));
        int32_t *s_pl = reinterpret_cast<int32_t *>(tb);
        tb += align8(sizeof(int32_t) * nnz);
        int32_t *s_rp = reinterpret_cast<int32_t *>(tb);
        tb += align8(sizeof(int32_t) * (E + 1));
        uint32_t *s_rev = reinterpret_cast<uint32_t *>(tb);
        tb += align8(sizeof(uint32_t) * 2 * rev_len);
        double *s_ic = reinterpret_cast<double *>(tb);
        for (int i = threadIdx.x; i <= K; i += blockDim.x) s_cp[i] = g_cp[i];
        for (int i = threadIdx.x; i <= P; i += blockDim.x) s_lp[i] = g_lp[i];
        for (int i = threadIdx.x; i < nnz; i += blockDim.x) s_pl[i] = g_pl[i];
        for (int i = threadIdx.x; i <= E; i += blockDim.x) s_rp[i] = g_rp[i];
        for (int i = threadIdx.x; i < 2 * rev_len; i += blockDim.x) s_rev[i] = g_rev[i];
        for (int i = threadIdx.x; i < E; i += blockDim.x) s_ic[i] = g_invcap[i];
        cp = s_cp; lp = s_lp; pl = s_pl; rp = s_rp; rev = s_rev; invcap = s_ic;
    }

    const double *d_in = demand_all + static_cast<size_t>(live ? plan : 0) * K;
    for (int k = t; k < K; k += nt) demand[k] = d_in[k];
    for (int p = t; p < P; p += nt) count[p] = 0u;
    if (t == 0) choice[K] = 0u;   // slot K is read (never used) by padding pairs
    __syncthreads();

    // width rho: every commodity that can reach a link counts once (first-of-commodity flag)
    double wmax = 0.0;
    for (int e = t; e < E; e += nt) {
        double reach = 0.0;
        for (int i = rp[e]; i < rp[e + 1]; ++i) {
            const uint32_t wa = rev[2 * i];
            if (wa & kFirstFlag) reach = reach + demand[wa & kCommMask];
        }
        const double ic = invcap[e];
        wmax = fmax(wmax, reach * ic);
        len[e] = 1.0;
        price[e] = MAXC ? 1.0 : ic;
        S[e] = 0.0;
    }
    // per-plan max: reduce inside the plan group through LDS (nt is a multiple of 64)
    {
        const double wm = wave_max(wmax);
        __syncthreads();
        if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x >> 6] = wm;
        __syncthreads();
        if (t == 0) {
            double m = 0.0;
            const int w0 = (slot * nt) >> 6, nw = nt >> 6;
            for (int w = 0; w < nw; ++w) m = fmax(m, red[w0 + w]);
            s_invrho[slot] = (m > 0.0) ? 1.0 / m : 0.0;
        }
        __syncthreads();
    }
    const double invrho = s_invrho[slot];

    for (int it = 0; it < iters; ++it) {
        for (int k = t; k < K; k += nt) {
            const int p0 = cp[k];
            const int np = cp[k + 1] - p0;
            double best = __builtin_inf();
            int bj = 0;
            int a = lp[p0];
            for (int j = 0; j < np; ++j) {
                const int b = lp[p0 + j + 1];
                double c = 0.0;
                for (int i = a; i < b; ++i) {
                    const double pe = price[pl[i]];
                    if constexpr (MAXC) c = (pe > c) ? pe : c;
                    else c = c + pe;
                }
                if (c < best) {
                    best = c;
                    bj = j;
                }
                a = b;
            }
            choice[k] = static_cast<uint8_t>(bj);
            count[p0 + bj] += 1u;
        }
        __syncthreads();
        for (int e = t; e < E; e += nt) {
            double load = 0.0;
            for (int i = rp[e]; i < rp[e + 1]; ++i) {
                const uint32_t wa = rev[2 * i], wb = rev[2 * i + 1];
                const uint32_t k = wa & kCommMask;
                const uint32_t ch = choice[k];
                if ((ch >> 5) == ((wa >> kWindowShift) & 3u) && ((wb >> (ch & 31u)) & 1u))
                    load = load + demand[k];
            }
            const double ic = invcap[e];
            const double u = load * ic;
            S[e] = S[e] + u;
            const double g = u * invrho;
            const double t1 = eps * g;
            const double t2 = 1.0 + t1;
            const double l = len[e] * t2;
            len[e] = l;
            price[e] = MAXC ? l : l * ic;
        }
        __syncthreads();
    }

    const double T = static_cast<double>(iters);
    if (live) {
        double *out = splits_all + static_cast<size_t>(plan) * P;
        for (int p = t; p < P; p += nt) out[p] = static_cast<double>(count[p]) / T;
    }
    double smax = 0.0;
    for (int e = t; e < E; e += nt) smax = fmax(smax, S[e]);
    const double sm = wave_max(smax);
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x >> 6] = sm;
    __syncthreads();
    if (t == 0 && live) {
        double m = 0.0;
        const int w0 = (slot * nt) >> 6, nw = nt >> 6;
        for (int w = 0; w < nw; ++w) m = fmax(m, red[w0 + w]);
        lambda_all[plan] = m / T;
    }
}

struct ResidentPlan {
    int nt, plans_per_block;
    bool topo_lds;
    size_t lds_bytes;
};

bool plan_resident(const DeviceTopo &t, int batch, ResidentPlan &rp)
{
    const ResidentLayout lay = make_layout(t.E, t.K, t.P, t.nnz, t.rev_pairs);
    if (lay.plan_bytes + 256 > kLdsBudget) return false;
    int need = t.K > t.E ? t.K : t.E;
    int nt = kWave;
    while (nt < need && nt < 1024) nt <<= 1;
    rp.nt = nt;
    int ppb = 1;
    if (batch > 1) {
        ppb = 1024 / nt;
        if (ppb > kMaxPlansPerBlock) ppb = kMaxPlansPerBlock;
        if (ppb > batch) ppb = batch;
        while (ppb > 1 && lay.plan_bytes * ppb + 256 > kLdsBudget) --ppb;
    }
    rp.plans_per_block = ppb;
    rp.topo_lds = lay.plan_bytes * ppb + lay.topo_bytes + 256 <= kLdsBudget;
    rp.lds_bytes = lay.plan_bytes * ppb + (rp.topo_lds ? lay.topo_bytes : 0);
    return true;
}

}  // namespace

size_t resident_state_bytes(const DeviceTopo &t)
{
    return make_layout(t.E, t.K, t.P, t.nnz, t.rev_pairs).plan_bytes;
}

size_t resident_topo_bytes(const DeviceTopo &t)
{
    return make_layout(t.E, t.K, t.P, t.nnz, t.rev_pairs).topo_bytes;
}

bool resident_fits(const DeviceTopo &t)
{
    ResidentPlan rp;
    return plan_resident(t, 1, rp);
}

hipError_t launch_resident(const DeviceTopo &t, int32_t batch, const double *demand, double eps,
                           int32_t iters, double *splits, double *lambda, hipStream_t s)
{
    ResidentPlan rp;
    if (!plan_resident(t, batch, rp)) return hipErrorInvalidValue;
    const int grid = (batch + rp.plans_per_block - 1) / rp.plans_per_block;
    const int block = rp.nt * rp.plans_per_block;
#define NIMBLE_RES_LAUNCH(MAXC, TL)                                                            \
    hipLaunchKernelGGL((k_resident<MAXC, TL>), dim3(grid), dim3(block), rp.lds_bytes, s, t.E,  \
                       t.K, t.P, static_cast<int>(t.nnz), static_cast<int>(t.rev_pairs), batch,  \
                       rp.nt, rp.plans_per_block, eps, iters, t.comm_ptr, t.path_ptr,          \
                       t.path_links, t.rev_ptr, t.rev_pair, t.invcap, demand, splits, lambda)
    if (t.cost_max) {
        if (rp.topo_lds) NIMBLE_RES_LAUNCH(true, true);
        else NIMBLE_RES_LAUNCH(true, false);
    } else {
        if (rp.topo_lds) NIMBLE_RES_LAUNCH(false, true);
        else NIMBLE_RES_LAUNCH(false, false);
    }
#undef NIMBLE_RES_LAUNCH
    return hipGetLastError();
}

}  // namespace nimble

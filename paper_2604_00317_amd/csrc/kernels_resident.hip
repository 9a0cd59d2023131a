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
//
// One plan, or a few, leave most of such a group idle and its busy threads with long loops.
// The kernel therefore has a cooperative form (CL > 0) for them: the plan gets all 1024 threads,
// CL lanes share a commodity (one candidate each, the (cost, index) minimum by DPP: lowest index
// among equal costs, the strict `<` of the sequential scan) and 16 lanes share a link's reverse
// row (pairs l, l + 16, ... each, the 16 partial sums added by a fixed butterfly).  Path costs
// are the same sums as before; link loads are added in that fixed tree instead of the
// sequential order, which is the same number for demands on a power-of-two grid (byte counts).
#include "host_topo.hpp"
#include "kernels.hpp"
#include "wave_ops.hpp"

namespace nimble {

namespace {

constexpr size_t kLdsBudget = 64 * 1024;   // static + dynamic LDS a kernel may use without opt-in
constexpr size_t kLdsBudgetMax = 150 * 1024;   // with opt-in, for the LDS copy of the topology
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

template <bool MAXC, bool TOPO_LDS, int CL>
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
        if constexpr (CL > 0) {
            // CL lanes per commodity, one candidate each
            const int j = t % CL, per = nt / CL;
            for (int k0 = 0; k0 < K; k0 += per) {                     // uniform over the group
                const int k = k0 + t / CL;
                double c = __builtin_inf();
                int cand = 0x7FFFFFFF, p0 = 0;
                if (k < K) {
                    p0 = cp[k];
                    if (j < cp[k + 1] - p0) {
                        cand = j;
                        c = 0.0;
                        const int b = lp[p0 + j + 1];
                        for (int i = lp[p0 + j]; i < b; ++i) {
                            const double pe = price[pl[i]];
                            if constexpr (MAXC) c = (pe > c) ? pe : c;
                            else c = c + pe;
                        }
                    }
                }
                const int bj = group_argmin_two_pass<(CL > 0 ? CL : 1)>(c, cand);
                if (k < K && j == 0) {
                    choice[k] = static_cast<uint8_t>(bj);
                    count[p0 + bj] += 1u;
                }
            }
            __syncthreads();
            // 16 lanes per link
            const int l = t & 15, rows = nt >> 4;
            for (int e0 = 0; e0 < E; e0 += rows) {                    // uniform over the group
                const int e = e0 + (t >> 4);
                double load = 0.0;
                if (e < E) {
                    const int end = rp[e + 1];
                    for (int i = rp[e] + l; i < end; i += 16) {
                        const uint32_t wa = rev[2 * i], wb = rev[2 * i + 1];
                        const uint32_t k = wa & kCommMask;
                        const uint32_t ch = choice[k];
                        if ((ch >> 5) == ((wa >> kWindowShift) & 3u) && ((wb >> (ch & 31u)) & 1u))
                            load = load + demand[k];
                    }
                }
                load = load + partner_f64<1>(load);
                load = load + partner_f64<2>(load);
                load = load + partner_f64<4>(load);
                load = load + partner_f64<8>(load);
                if (e < E && l == 0) {
                    const double ic = invcap[e];
                    const double u = load * ic;
                    S[e] = S[e] + u;
                    const double g = u * invrho;
                    const double t1 = eps * g;
                    const double t2 = 1.0 + t1;
                    const double ln = len[e] * t2;
                    len[e] = ln;
                    price[e] = MAXC ? ln : ln * ic;
                }
            }
            __syncthreads();
            continue;
        }
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


// ---- one plan per workgroup, lanes sharing commodities and links, lists in registers ----------
// The cooperative form above for fabrics small enough that a thread can keep its share of the
// lists in registers for the whole solve (as k_resident_reg does for a single node): CL lanes
// per commodity, lane j holding the LDS addresses of the prices of candidate j's steps (at most
// kCoopSteps; short paths point at a +0.0 slot, absent candidates at a +inf slot) for up to
// kCoopRounds commodities; 16 lanes per link, lane l holding the pairs l, l + 16, l + 32, l + 48
// of the row for up to kCoopRounds links.  LDS then carries only what threads exchange --
// prices, choices -- and the demands, lengths, congestion sums and counts.  Same additions in
// the same order as the cooperative form of k_resident, hence the same bits.
constexpr int kCoopRounds = 4;     // commodities per lane group, links per 16-lane row
constexpr int kCoopSteps = 5;      // longest path
constexpr int kCoopPairs = 4;      // pairs per lane: rows of at most 64 pairs

struct CoopLayout {
    size_t price, len, S, invcap, demand, count, choice, bytes;
};

__host__ __device__ inline CoopLayout coop_layout(int E, int K, int P)
{
    CoopLayout l;
    size_t o = 0;
    l.price = o;  o += sizeof(double) * (E + 2);      // [E] = +0.0, [E + 1] = +inf
    l.len = o;    o += sizeof(double) * E;
    l.S = o;      o += sizeof(double) * E;
    l.invcap = o; o += sizeof(double) * E;
    l.demand = o; o += sizeof(double) * (K + 1);      // [K] = 0.0: the pair that is not there
    l.count = o;  o += align8(sizeof(uint32_t) * P);
    l.choice = o; o += align8(K + 1);
    l.bytes = o;
    return l;
}

template <bool MAXC, int CL>
__global__ __launch_bounds__(1024) void k_resident_coop(
    int E, int K, int P, int batch, double eps, int iters, const int32_t *__restrict__ g_cp,
    const int32_t *__restrict__ g_lp, const int32_t *__restrict__ g_pl,
    const int32_t *__restrict__ g_rp, const uint32_t *__restrict__ g_rev,
    const double *__restrict__ g_invcap, const double *__restrict__ demand_all,
    double *__restrict__ splits_all, double *__restrict__ lambda_all)
{
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ double red[16];
    __shared__ double s_invrho;
    constexpr int NT = 1024;
    const CoopLayout lay = coop_layout(E, K, P);
    double *price = reinterpret_cast<double *>(lds + lay.price);
    double *len = reinterpret_cast<double *>(lds + lay.len);
    double *S = reinterpret_cast<double *>(lds + lay.S);
    double *invcap = reinterpret_cast<double *>(lds + lay.invcap);
    double *demand = reinterpret_cast<double *>(lds + lay.demand);
    uint32_t *count = reinterpret_cast<uint32_t *>(lds + lay.count);
    uint8_t *choice = lds + lay.choice;
    const int t = threadIdx.x;
    const int plan = blockIdx.x;                  // grid = batch

    const double *d_in = demand_all + static_cast<size_t>(plan) * K;
    for (int k = t; k < K; k += NT) demand[k] = d_in[k];
    for (int p = t; p < P; p += NT) count[p] = 0u;
    for (int e = t; e < E; e += NT) invcap[e] = g_invcap[e];
    if (t == 0) {
        demand[K] = 0.0;
        choice[K] = 0u;
        price[E] = 0.0;
        price[E + 1] = __builtin_inf();
    }
    __syncthreads();

    // width rho: every commodity that can reach a link counts once (first-of-commodity flag)
    double wmax = 0.0;
    for (int e = t; e < E; e += NT) {
        double reach = 0.0;
        for (int i = g_rp[e]; i < g_rp[e + 1]; ++i) {
            const uint32_t wa = g_rev[2 * i];
            if (wa & kFirstFlag) reach = reach + demand[wa & kCommMask];
        }
        const double ic = invcap[e];
        wmax = fmax(wmax, reach * ic);
        len[e] = 1.0;
        price[e] = MAXC ? 1.0 : ic;
        S[e] = 0.0;
    }
    {
        const double wm = wave_max(wmax);
        if ((t & (kWave - 1)) == 0) red[t >> 6] = wm;
        __syncthreads();
        if (t == 0) {
            double m = 0.0;
            for (int w = 0; w < NT / kWave; ++w) m = fmax(m, red[w]);
            s_invrho = (m > 0.0) ? 1.0 / m : 0.0;
        }
        __syncthreads();
    }
    const double invrho = s_invrho;

    // this lane's share of the lists, for the whole solve
    const int j = t % CL, per = NT / CL;
    int addr[kCoopRounds][kCoopSteps];            // price slots of candidate j of commodity r
    int cand[kCoopRounds], first_path[kCoopRounds];
#pragma unroll
    for (int r = 0; r < kCoopRounds; ++r) {
        const int k = r * per + t / CL;
        cand[r] = 0x7FFFFFFF;
        first_path[r] = 0;
        addr[r][0] = E + 1;
#pragma unroll
        for (int i = 1; i < kCoopSteps; ++i) addr[r][i] = E;
        if (k < K) {
            const int p0 = g_cp[k];
            first_path[r] = p0;
            if (j < g_cp[k + 1] - p0) {
                cand[r] = j;
                const int a = g_lp[p0 + j], n = g_lp[p0 + j + 1] - a;
#pragma unroll
                for (int i = 0; i < kCoopSteps; ++i) addr[r][i] = i < n ? g_pl[a + i] : E;
            }
        }
    }
    const int l = t & 15, rows = NT >> 4;
    uint32_t pair_k[kCoopRounds][kCoopPairs];     // commodity | window << 24, K: no pair
    uint32_t pair_m[kCoopRounds][kCoopPairs];     // candidate mask of the window
#pragma unroll
    for (int r = 0; r < kCoopRounds; ++r) {
        const int e = r * rows + (t >> 4);
#pragma unroll
        for (int q = 0; q < kCoopPairs; ++q) {
            pair_k[r][q] = static_cast<uint32_t>(K);
            pair_m[r][q] = 0u;
            if (e < E) {
                const int i = g_rp[e] + l + 16 * q;
                if (i < g_rp[e + 1]) {
                    const uint32_t wa = g_rev[2 * i];
                    pair_k[r][q] = (wa & kCommMask) | (((wa >> kWindowShift) & 3u) << 24);
                    pair_m[r][q] = g_rev[2 * i + 1];
                }
            }
        }
    }

    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < kCoopRounds; ++r) {
            if (r * per >= K) break;                                  // uniform
            double c = price[addr[r][0]];
#pragma unroll
            for (int i = 1; i < kCoopSteps; ++i) {
                const double pe = price[addr[r][i]];
                if constexpr (MAXC) c = (pe > c) ? pe : c;
                else c = c + pe;
            }
            const int bj = group_argmin_two_pass<CL>(c, cand[r]);
            const int k = r * per + t / CL;
            if (k < K && j == 0) {
                choice[k] = static_cast<uint8_t>(bj);
                count[first_path[r] + bj] += 1u;
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kCoopRounds; ++r) {
            if (r * rows >= E) break;                                 // uniform
            const int e = r * rows + (t >> 4);
            double load = 0.0;
#pragma unroll
            for (int q = 0; q < kCoopPairs; ++q) {
                const uint32_t k = pair_k[r][q] & kCommMask;
                const uint32_t ch = choice[k];
                const bool hit = (ch >> 5) == (pair_k[r][q] >> 24) &&
                                 ((pair_m[r][q] >> (ch & 31u)) & 1u) != 0u;
                const double d = demand[k];
                load = load + (hit ? d : 0.0);
            }
            load = load + partner_f64<1>(load);
            load = load + partner_f64<2>(load);
            load = load + partner_f64<4>(load);
            load = load + partner_f64<8>(load);
            if (e < E && l == 0) {
                const double ic = invcap[e];
                const double u = load * ic;
                S[e] = S[e] + u;
                const double g = u * invrho;
                const double t1 = eps * g;
                const double t2 = 1.0 + t1;
                const double ln = len[e] * t2;
                len[e] = ln;
                price[e] = MAXC ? ln : ln * ic;
            }
        }
        __syncthreads();
    }

    const double T = static_cast<double>(iters);
    double *out = splits_all + static_cast<size_t>(plan) * P;
    for (int p = t; p < P; p += NT) out[p] = static_cast<double>(count[p]) / T;
    double smax = 0.0;
    for (int e = t; e < E; e += NT) smax = fmax(smax, S[e]);
    const double sm = wave_max(smax);
    __syncthreads();
    if ((t & (kWave - 1)) == 0) red[t >> 6] = sm;
    __syncthreads();
    if (t == 0) {
        double m = 0.0;
        for (int w = 0; w < NT / kWave; ++w) m = fmax(m, red[w]);
        lambda_all[plan] = m / T;
    }
}

__host__ __device__ inline size_t reg_plan_bytes(int E, int K, int nt, int maxp)
{
    return sizeof(double) * (E + 2) + align8(K + 1) + sizeof(uint32_t) * maxp * nt;
}

// Register-resident variant for small dense fabrics (one modeled node): every thread owns one
// commodity and one link for the whole solve, so what never changes between iterations lives in
// registers -- the link ids of the commodity's MAXP x MAXL candidate steps, its choice counts,
// the link's MAXROW reverse pairs with the demands they can add, and the link's length,
// congestion sum and 1/capacity.  LDS holds only what threads exchange: the prices and the
// choices.  Short paths are padded with the price slot E (+0.0, neutral for the sum and for the
// maximum of positive prices), absent candidates start at slot E + 1 (+inf: never below the
// best), absent pairs have an empty mask.  The additions are those of the generic kernel in the
// same order (0 + p is p; adding +0.0 changes nothing), so the results are the same bits.
template <bool MAXC, bool ONEWAVE, int MAXP, int MAXL, int MAXROW>
__global__ __launch_bounds__(1024) void k_resident_reg(
    int E, int K, int P, int batch, int nt, int plans_per_block, double eps, int iters,
    const int32_t *__restrict__ g_cp, const int32_t *__restrict__ g_lp,
    const int32_t *__restrict__ g_pl, const int32_t *__restrict__ g_rp,
    const uint32_t *__restrict__ g_rev, const double *__restrict__ g_invcap,
    const double *__restrict__ demand_all, double *__restrict__ splits_all,
    double *__restrict__ lambda_all)
{
    static_assert(MAXP <= 8, "a choice is a bit of one mask byte; eight 8-bit counters per word");
    static_assert(MAXROW % 4 == 0, "four mask bytes per register");
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ double red[16];
    __shared__ double s_invrho[kMaxPlansPerBlock];

    const int slot = threadIdx.x / nt;            // plan slot inside the workgroup
    const int t = threadIdx.x - slot * nt;        // thread inside the plan group
    const int plan = blockIdx.x * plans_per_block + slot;
    const bool live = plan < batch;
    const size_t plan_bytes = reg_plan_bytes(E, K, nt, MAXP);
    double *price = reinterpret_cast<double *>(lds + plan_bytes * slot);
    uint8_t *choice = reinterpret_cast<uint8_t *>(price + E + 2);
    // choice counts of this thread's commodity, candidate j at [j * nt + t]
    uint32_t *count = reinterpret_cast<uint32_t *>(choice + align8(K + 1)) + t;
    const double *d_in = demand_all + static_cast<size_t>(live ? plan : 0) * K;
    // a plan that is one wave needs no workgroup barrier: a wave's LDS operations execute in
    // issue order
    auto plan_sync = [] {
        if constexpr (ONEWAVE) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
            __syncthreads();
        }
    };

    // the commodity of this thread: where the price of every candidate step lives
    const bool has_k = t < K;
    const double *pp[MAXP][MAXL];
    int p0 = 0, np = 0;
    if (has_k) {
        p0 = g_cp[t];
        np = g_cp[t + 1] - p0;
    }
#pragma unroll
    for (int j = 0; j < MAXP; ++j) {
        count[j * nt] = 0u;
        int a = 0, b = 0;
        if (j < np) {
            a = g_lp[p0 + j];
            b = g_lp[p0 + j + 1];
        }
#pragma unroll
        for (int i = 0; i < MAXL; ++i) {
            int e = (i == 0 && j >= np) ? E + 1 : E;
            if (a + i < b) e = g_pl[a + i];
            pp[j][i] = price + e;
        }
    }
    // the link of this thread: for every reverse pair where the commodity's choice lives, the
    // candidates that use the link, and the demand they add
    const bool has_e = t < E;
    const uint8_t *cptr[MAXROW];
    uint32_t wb4[MAXROW / 4];      // the 8-bit candidate masks of four pairs per register
    double dm[MAXROW];
    double ic = 0.0, len = 1.0, S = 0.0, reach = 0.0;
    {
        int r0 = 0, rn = 0;
        if (has_e) {
            r0 = g_rp[t];
            rn = g_rp[t + 1] - r0;
            ic = g_invcap[t];
        }
#pragma unroll
        for (int i = 0; i < MAXROW / 4; ++i) wb4[i] = 0u;
#pragma unroll
        for (int i = 0; i < MAXROW; ++i) {
            cptr[i] = choice + K;                  // padding: the spare choice, empty mask
            dm[i] = 0.0;
            if (i < rn) {
                const uint32_t wa = g_rev[2 * (r0 + i)];
                const uint32_t k = wa & kCommMask;
                if (k < static_cast<uint32_t>(K)) {
                    cptr[i] = choice + k;
                    wb4[i / 4] |= (g_rev[2 * (r0 + i) + 1] & 0xFFu) << (8 * (i % 4));
                    dm[i] = d_in[k];
                }
                // width rho: every commodity that can reach the link counts once
                if (wa & kFirstFlag) reach = reach + dm[i];
            }
        }
    }
    if (has_e) price[t] = MAXC ? 1.0 : ic;
    if (t == 0) {
        price[E] = 0.0;
        price[E + 1] = __builtin_inf();
        choice[K] = 0u;                            // read (never used) by padding pairs
    }
    // per-plan width: reduce inside the plan group through LDS (nt is a multiple of 64)
    {
        const double wm = wave_max(has_e ? reach * ic : 0.0);
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

    // eight 8-bit counters in one 64-bit word, emptied into the LDS counts before any can wrap
    unsigned long long tally = 0ull;
    auto flush = [&] {
#pragma unroll
        for (int j = 0; j < MAXP; ++j)
            count[j * nt] += static_cast<uint32_t>(tally >> (8 * j)) & 0xFFu;
        tally = 0ull;
    };
    for (int it = 0; it < iters; ++it) {
        if (has_k) {
            // the prices of four candidates are requested before the first is used
            constexpr int kBatch = MAXP < 4 ? MAXP : 4;
            double c[MAXP];
#pragma unroll
            for (int j0 = 0; j0 < MAXP; j0 += kBatch) {
                double pv[kBatch][MAXL];
#pragma unroll
                for (int j = 0; j < kBatch; ++j)
#pragma unroll
                    for (int i = 0; i < MAXL; ++i) pv[j][i] = *pp[j0 + j][i];
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    double cj = pv[j][0];                    // 0 + p is p
#pragma unroll
                    for (int i = 1; i < MAXL; ++i) {
                        if constexpr (MAXC) cj = (pv[j][i] > cj) ? pv[j][i] : cj;
                        else cj = cj + pv[j][i];
                    }
                    c[j0 + j] = cj;
                }
            }
            // the minimum, then the lowest candidate that holds it: what the strict `<` scan
            // in candidate order picks (all +inf, a commodity without traffic-bearing
            // candidates, resolves to candidate 0 either way)
            double best = c[0];
#pragma unroll
            for (int j = 1; j < MAXP; ++j) best = fast_min_f64(best, c[j]);
            int bj = MAXP - 1;
#pragma unroll
            for (int j = MAXP - 2; j >= 0; --j) bj = (c[j] == best) ? j : bj;
            choice[t] = static_cast<uint8_t>(bj);
            tally += 1ull << (8 * bj);
            if ((it & 127) == 127) flush();
        }
        plan_sync();
        if (has_e) {
            // the choices of all pairs are requested before the first is used
            uint32_t ch[MAXROW];
#pragma unroll
            for (int i = 0; i < MAXROW; ++i) ch[i] = *cptr[i];
            double load = 0.0;
#pragma unroll
            for (int i = 0; i < MAXROW; ++i) {
                // 1 where the commodity's choice uses the link (a choice is below 8, so it
                // stays inside its mask byte); fma(d, 1.0, load) rounds like load + d, and
                // fma(d, 0.0, load) leaves the sum as it is (demands are finite)
                const uint32_t h = ((wb4[i / 4] >> ch[i]) >> (8 * (i % 4))) & 1u;
                load = __builtin_fma(dm[i], static_cast<double>(h), load);
            }
            const double u = load * ic;
            S = S + u;
            const double g = u * invrho;
            const double t1 = eps * g;
            const double t2 = 1.0 + t1;
            len = len * t2;
            price[t] = MAXC ? len : len * ic;
        }
        plan_sync();
    }

    const double T = static_cast<double>(iters);
    if (has_k) flush();
    if (live && has_k) {
        double *out = splits_all + static_cast<size_t>(plan) * P + p0;
#pragma unroll
        for (int j = 0; j < MAXP; ++j)
            if (j < np) out[j] = static_cast<double>(count[j * nt]) / T;
    }
    const double sm = wave_max(has_e ? S : 0.0);
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

constexpr int kRegMaxPaths = 8, kRegMaxLen = 2, kRegMaxRow = 16;

struct ResidentPlan {
    int nt, plans_per_block;
    bool topo_lds;
    bool in_registers;     // k_resident_reg: one commodity and one link per thread
    int coop_lanes;        // > 0: the cooperative form of k_resident, that many lanes per commodity
    bool coop_registers;   // k_resident_coop: that form with the lists in registers
    size_t lds_bytes;
};

constexpr int kCoopMaxPlans = 256;   // beyond that many plans a thread per commodity serves better

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
    // the topology copy may take the LDS beyond 64 KB (the launch opts in)
    rp.topo_lds = lay.plan_bytes * ppb + lay.topo_bytes + 256 <= kLdsBudgetMax;
    rp.lds_bytes = lay.plan_bytes * ppb + (rp.topo_lds ? lay.topo_bytes : 0);
    // the register kernel gives every thread exactly one commodity and one link (no striding):
    // a plan with more of either than its threads keeps to the LDS kernel, which strides
    rp.in_registers = !t.resident_generic && t.pmax <= kRegMaxPaths && t.lmax <= kRegMaxLen &&
                      t.rev_row_max <= kRegMaxRow && need <= nt;
    if (rp.in_registers) rp.lds_bytes = reg_plan_bytes(t.E, t.K, nt, kRegMaxPaths) * ppb;
    // a few plans: all 1024 threads of a workgroup for each, lanes sharing commodities and links
    rp.coop_lanes = 0;
    rp.coop_registers = false;
    if (!rp.in_registers && !t.resident_generic && batch <= kCoopMaxPlans && t.pmax <= kWave) {
        int cl = 2;
        while (cl < t.pmax) cl <<= 1;
        rp.coop_lanes = cl;
        rp.nt = 1024;
        rp.plans_per_block = 1;
        rp.topo_lds = lay.plan_bytes + lay.topo_bytes + 256 <= kLdsBudgetMax;
        rp.lds_bytes = lay.plan_bytes + (rp.topo_lds ? lay.topo_bytes : 0);
        // lists in registers: at most kCoopRounds commodities per lane group and links per row
        // of 16 lanes, paths of at most kCoopSteps links, rows of at most 16 x kCoopPairs pairs
        // (rows are padded to an even number of pairs)
        const int row_padded = (t.rev_row_max + 1) & ~1;
        const CoopLayout cl_lay = coop_layout(t.E, t.K, t.P);
        rp.coop_registers = t.lmax <= kCoopSteps && t.K <= kCoopRounds * (1024 / cl) &&
                            t.E <= kCoopRounds * (1024 / 16) &&
                            row_padded <= 16 * kCoopPairs && cl_lay.bytes + 256 <= kLdsBudget;
        if (rp.coop_registers) rp.lds_bytes = cl_lay.bytes;
    }
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

bool resident_in_registers(const DeviceTopo &t)
{
    ResidentPlan rp;
    return plan_resident(t, 1, rp) && rp.in_registers;
}

int resident_kernel_kind(const DeviceTopo &t, int batch)
{
    ResidentPlan rp;
    if (!plan_resident(t, batch, rp)) return 0;
    if (rp.in_registers) return 2;
    if (rp.coop_registers) return 4;
    if (rp.coop_lanes > 0) return 3;
    return 1;
}

double resident_iteration_us(const DeviceTopo &t, int batch)
{
    // measured on the two-node fabric (240 commodities of up to 16 candidates, 152 links, rows
    // of up to 64 pairs): 18.6 us per iteration with a thread per commodity and per link (one
    // dependent LDS access after the other, about 0.04 us each), 5.0 us with lanes sharing
    // them, 2.7 us with the lists in registers; the kernels with a thread per commodity run
    // 256 plans side by side for that price, the others one plan per workgroup
    ResidentPlan rp;
    if (!plan_resident(t, batch, rp)) return 1e30;
    const double rounds = (batch + 255) / 256;
    if (rp.coop_registers) return 2.7 * rounds;
    if (rp.coop_lanes > 0) {
        const double fwd = ((static_cast<double>(t.K) * rp.coop_lanes + 1023) / 1024) * (4 + 2 * t.lmax);
        const double rev = ((t.E + 63) / 64) * (2 + 3 * ((t.rev_row_max + 15) / 16));
        return 0.05 * (fwd + rev) * rounds;
    }
    return 0.04 * (2.0 * t.pmax * t.lmax + 3.0 * t.rev_row_max) * rounds;
}

hipError_t launch_resident(const DeviceTopo &t, int32_t batch, const double *demand, double eps,
                           int32_t iters, double *splits, double *lambda, hipStream_t s)
{
    ResidentPlan rp;
    if (!plan_resident(t, batch, rp)) return hipErrorInvalidValue;
    const int grid = (batch + rp.plans_per_block - 1) / rp.plans_per_block;
    const int block = rp.nt * rp.plans_per_block;
#define NIMBLE_RES_LAUNCH_CL(MAXC, TL, CLN)                                                    \
    do {                                                                                       \
        if (rp.lds_bytes + 256 > kLdsBudget) {                                                 \
            hipError_t ea = hipFuncSetAttribute(                                               \
                reinterpret_cast<const void *>(&k_resident<MAXC, TL, CLN>),                    \
                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(rp.lds_bytes));   \
            if (ea != hipSuccess) return ea;                                                   \
        }                                                                                      \
        hipLaunchKernelGGL((k_resident<MAXC, TL, CLN>), dim3(grid), dim3(block), rp.lds_bytes, \
                           s, t.E, t.K, t.P, static_cast<int>(t.nnz),                          \
                           static_cast<int>(t.rev_pairs), batch, rp.nt, rp.plans_per_block,    \
                           eps, iters, t.comm_ptr, t.path_ptr, t.path_links, t.rev_ptr,        \
                           t.rev_pair, t.invcap, demand, splits, lambda);                      \
    } while (0)
#define NIMBLE_RES_LAUNCH(MAXC, TL)                                                            \
    do {                                                                                       \
        switch (rp.coop_lanes) {                                                               \
        case 2: NIMBLE_RES_LAUNCH_CL(MAXC, TL, 2); break;                                      \
        case 4: NIMBLE_RES_LAUNCH_CL(MAXC, TL, 4); break;                                      \
        case 8: NIMBLE_RES_LAUNCH_CL(MAXC, TL, 8); break;                                      \
        case 16: NIMBLE_RES_LAUNCH_CL(MAXC, TL, 16); break;                                    \
        case 32: NIMBLE_RES_LAUNCH_CL(MAXC, TL, 32); break;                                    \
        case 64: NIMBLE_RES_LAUNCH_CL(MAXC, TL, 64); break;                                    \
        default: NIMBLE_RES_LAUNCH_CL(MAXC, TL, 0); break;                                     \
        }                                                                                      \
    } while (0)
    if (rp.in_registers) {
#define NIMBLE_REG_LAUNCH(MAXC, ONEW)                                                          \
    hipLaunchKernelGGL((k_resident_reg<MAXC, ONEW, kRegMaxPaths, kRegMaxLen, kRegMaxRow>),     \
                       dim3(grid), dim3(block), rp.lds_bytes, s, t.E, t.K, t.P, batch, rp.nt,  \
                       rp.plans_per_block, eps, iters, t.comm_ptr, t.path_ptr, t.path_links,   \
                       t.rev_ptr, t.rev_pair, t.invcap, demand, splits, lambda)
        const bool one_wave = rp.nt == kWave;
        if (t.cost_max) {
            if (one_wave) NIMBLE_REG_LAUNCH(true, true);
            else NIMBLE_REG_LAUNCH(true, false);
        } else {
            if (one_wave) NIMBLE_REG_LAUNCH(false, true);
            else NIMBLE_REG_LAUNCH(false, false);
        }
#undef NIMBLE_REG_LAUNCH
        return hipGetLastError();
    }
    if (rp.coop_registers) {
#define NIMBLE_COOP_LAUNCH(MAXC, CLN)                                                          \
    hipLaunchKernelGGL((k_resident_coop<MAXC, CLN>), dim3(batch), dim3(1024), rp.lds_bytes, s, \
                       t.E, t.K, t.P, batch, eps, iters, t.comm_ptr, t.path_ptr, t.path_links, \
                       t.rev_ptr, t.rev_pair, t.invcap, demand, splits, lambda)
#define NIMBLE_COOP_LANES(MAXC)                                                                \
    switch (rp.coop_lanes) {                                                                   \
    case 2: NIMBLE_COOP_LAUNCH(MAXC, 2); break;                                                \
    case 4: NIMBLE_COOP_LAUNCH(MAXC, 4); break;                                                \
    case 8: NIMBLE_COOP_LAUNCH(MAXC, 8); break;                                                \
    case 16: NIMBLE_COOP_LAUNCH(MAXC, 16); break;                                              \
    case 32: NIMBLE_COOP_LAUNCH(MAXC, 32); break;                                              \
    default: NIMBLE_COOP_LAUNCH(MAXC, 64); break;                                              \
    }
        if (t.cost_max) {
            NIMBLE_COOP_LANES(true)
        } else {
            NIMBLE_COOP_LANES(false)
        }
#undef NIMBLE_COOP_LANES
#undef NIMBLE_COOP_LAUNCH
        return hipGetLastError();
    }
    if (t.cost_max) {
        if (rp.topo_lds) NIMBLE_RES_LAUNCH(true, true);
        else NIMBLE_RES_LAUNCH(true, false);
    } else {
        if (rp.topo_lds) NIMBLE_RES_LAUNCH(false, true);
        else NIMBLE_RES_LAUNCH(false, false);
    }
#undef NIMBLE_RES_LAUNCH
#undef NIMBLE_RES_LAUNCH_CL
    return hipGetLastError();
}

}  // namespace nimble

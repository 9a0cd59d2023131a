// Device code of the three per-iteration phases, shared by the streaming kernels (one launch
// per phase) and the persistent kernel (one launch per solve, grid barriers between phases).
// All arithmetic is binary64, one IEEE operation per statement.
#pragma once
#include <hip/hip_runtime.h>

#include "host_topo.hpp"
#include "wave_ops.hpp"

namespace nimble {

// Loads that are consumed once per iteration (CSR streams) bypass cache retention so that the
// gathered tables (prices, choices, demands) keep their place in L2.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <typename T>
__device__ __forceinline__ T stream_load(const T *p)
{
#ifdef NIMBLE_NO_NT
    return *p;
#else
    return __builtin_nontemporal_load(p);
#endif
}

// Forward-CSR loads: neighbouring lanes and the next unrolled load touch the same cache lines,
// so these stay ordinary cached loads.
template <typename T>
__device__ __forceinline__ T csr_load(const T *p)
{
    return *p;
}

// ---- phase A: path-cost gather over the path->link CSR + per-commodity argmin -------------
// L lanes cooperate on one commodity (lane j takes candidates j, j+L, ...); the first LMAX links
// of a path are loaded before any is used so that their latencies overlap.  Costs are added
// left to right in CSR order; the candidate scan keeps the lowest index among equal costs
// (strict `<`, Algorithm 1).  `wave`/`n_waves` enumerate the waves that share the work; the
// loop bounds are wave-uniform, so all 64 lanes reach the cross-lane reduction.
template <int L, int LMAX, bool MAXC>
__device__ __forceinline__ void argmin_phase(int K, const int32_t *__restrict__ cp,
                                             const int32_t *__restrict__ lp,
                                             const int32_t *__restrict__ pl,
                                             const double *__restrict__ price,
                                             uint8_t *__restrict__ choice,
                                             uint32_t *__restrict__ count, int wave,
                                             int n_waves, int lane)
{
    constexpr int kPerWave = kWave / L;
    const int sub = lane / L;
    const int j0 = lane % L;
    for (int base = wave * kPerWave; base < K; base += n_waves * kPerWave) {
        const int k = base + sub;
        double best = __builtin_inf();
        int bj = 0x7FFFFFFF;
        int p0 = 0;
        if (k < K) {
            p0 = cp[k];
            const int np = cp[k + 1] - p0;
            if (j0 < np) bj = j0;   // an all-infinite commodity still resolves to candidate 0
            for (int j = j0; j < np; j += L) {
                const int a = csr_load(lp + p0 + j), b = csr_load(lp + p0 + j + 1);
                int idx[LMAX];
#pragma unroll
                for (int i = 0; i < LMAX; ++i) idx[i] = (a + i < b) ? csr_load(pl + a + i) : -1;
                double pr[LMAX];
#pragma unroll
                for (int i = 0; i < LMAX; ++i) pr[i] = (idx[i] >= 0) ? price[idx[i]] : 0.0;
                double c = 0.0;
                // absent links contribute +0.0, which leaves a sum (or a max of positive
                // prices) unchanged bit for bit
#pragma unroll
                for (int i = 0; i < LMAX; ++i) {
                    if constexpr (MAXC) c = (pr[i] > c) ? pr[i] : c;
                    else c = c + pr[i];
                }
                for (int i = a + LMAX; i < b; ++i) {
                    const double pe = price[csr_load(pl + i)];
                    if constexpr (MAXC) c = (pe > c) ? pe : c;
                    else c = c + pe;
                }
                if (c < best) {
                    best = c;
                    bj = j;
                }
            }
        }
        group_argmin<L>(best, bj);
        if (k < K && j0 == 0) {
            choice[k] = static_cast<uint8_t>(bj);
            count[p0 + bj] += 1u;
        }
    }
}

// ---- phase B: link loads over the reverse link->(commodity, path set) CSR ------------------
// A reverse row holds one 8-byte pair per (commodity, window of 32 candidates) with a bit mask
// of the candidates that use the link.  Rows are cut into chunks of 16*PPL pairs; one 16-lane
// DPP row reduces one chunk: every lane loads its PPL/2 16-byte groups first, then gathers the
// choices, then the demands of the (few) hits, adds them in pair order, and the 16 lane sums
// are combined by a fixed butterfly.  No floating-point atomics; the same tree on every run.
// MODE 0: hit = chosen candidate of the commodity is in the pair's window and mask.
// MODE 1 (width rho): hit = first pair of the commodity in the row, so every commodity that
// can reach the link counts once.
constexpr int kRowLanes = 16;
constexpr int kRowsPerWave = kWave / kRowLanes;

template <int MODE, int PPL>
__device__ __forceinline__ void reduce_phase(int n_chunks, const int32_t *__restrict__ chunk_begin,
                                             const int32_t *__restrict__ chunk_end,
                                             const uint32_t *__restrict__ rev, uint32_t pad_comm,
                                             const uint8_t *__restrict__ choice,
                                             const double *__restrict__ demand,
                                             double *__restrict__ partial, int wave, int n_waves,
                                             int lane)
{
    const int row = lane / kRowLanes;
    const int l = lane % kRowLanes;
    for (int cbase = wave * kRowsPerWave; cbase < n_chunks; cbase += n_waves * kRowsPerWave) {
        const int c = cbase + row;
        int b = 0, e = 0;
        if (c < n_chunks) {
            b = stream_load(chunk_begin + c);
            e = stream_load(chunk_end + c);
        }
        uint32_t wa[PPL], wb[PPL];
#pragma unroll
        for (int it = 0; it < PPL / 2; ++it) {
            const int i = b + it * (kRowLanes * 2) + l * 2;      // pair index
            u32x4 v = {pad_comm, 0u, pad_comm, 0u};
            if (i < e) v = stream_load(reinterpret_cast<const u32x4 *>(rev + 2 * size_t(i)));
            wa[it * 2 + 0] = v.x;
            wb[it * 2 + 0] = v.y;
            wa[it * 2 + 1] = v.z;
            wb[it * 2 + 1] = v.w;
        }
        // gathers are issued in batches before anything waits on them: PPL choice bytes, then
        // the demands of the hits; absent demands are +0.0, which adds exactly
        uint32_t ch[PPL];
#pragma unroll
        for (int q = 0; q < PPL; ++q)
            if constexpr (MODE == 0) ch[q] = choice[wa[q] & kCommMask];
        double dq[PPL];
#pragma unroll
        for (int q = 0; q < PPL; ++q) {
            bool hit;
            if constexpr (MODE == 0)
                hit = ((ch[q] >> 5) == ((wa[q] >> kWindowShift) & 3u)) &&
                      (((wb[q] >> (ch[q] & 31u)) & 1u) != 0u);
            else
                hit = (wa[q] & kFirstFlag) != 0u;
            dq[q] = 0.0;
            if (hit) dq[q] = demand[wa[q] & kCommMask];
        }
        double acc = 0.0;
#pragma unroll
        for (int q = 0; q < PPL; ++q) acc = acc + dq[q];
        acc = acc + partner_f64<1>(acc);
        acc = acc + partner_f64<2>(acc);
        acc = acc + partner_f64<4>(acc);
        acc = acc + partner_f64<8>(acc);
        if (c < n_chunks && l == 0) partial[c] = acc;
    }
}

// ---- phase C: chunk partials -> load, congestion sum, multiplicative length update ---------
// One 16-lane DPP row per link: the lanes fetch the link's chunk partials side by side (16 per
// step), add their own in ascending chunk order, and a fixed butterfly combines the 16 lane
// sums; lane 0 of the row then applies  S_e += u_e,  len_e *= 1 + eps*u_e/rho,  price_e.
// Returns, in lane 0 of every row, the new S_e (0 elsewhere) for the lambda max-reduce.
__device__ __forceinline__ double row_partial_sum(int c0, int c1, int l,
                                                  const double *__restrict__ partial)
{
    double acc = 0.0;
    for (int c = c0 + l; c < c1; c += kRowLanes) acc = acc + partial[c];
    acc = acc + partner_f64<1>(acc);
    acc = acc + partner_f64<2>(acc);
    acc = acc + partner_f64<4>(acc);
    acc = acc + partner_f64<8>(acc);
    return acc;
}

template <bool MAXC>
__device__ __forceinline__ double update_phase(int E, double eps, double invrho,
                                               const int32_t *__restrict__ link_chunk_ptr,
                                               const double *__restrict__ partial,
                                               const double *__restrict__ invcap,
                                               double *__restrict__ len,
                                               double *__restrict__ price, double *__restrict__ S,
                                               int wave, int n_waves, int lane)
{
    const int row = lane / kRowLanes;
    const int l = lane % kRowLanes;
    double smax = 0.0;
    for (int ebase = wave * kRowsPerWave; ebase < E; ebase += n_waves * kRowsPerWave) {
        const int e = ebase + row;
        int c0 = 0, c1 = 0;
        if (e < E) {
            c0 = link_chunk_ptr[e];
            c1 = link_chunk_ptr[e + 1];
        }
        const double load = row_partial_sum(c0, c1, l, partial);
        if (e < E && l == 0) {
            const double ic = invcap[e];
            const double u = load * ic;
            const double s_new = S[e] + u;
            S[e] = s_new;
            const double g = u * invrho;
            const double t1 = eps * g;
            const double t2 = 1.0 + t1;
            const double ln = len[e] * t2;
            len[e] = ln;
            price[e] = MAXC ? ln : ln * ic;
            smax = fmax(smax, s_new);
        }
    }
    return smax;
}

// max over this wave's links of (demand that can reach the link) / capacity: terms of rho
__device__ __forceinline__ double width_phase(int E, const int32_t *__restrict__ link_chunk_ptr,
                                              const double *__restrict__ partial,
                                              const double *__restrict__ invcap, int wave,
                                              int n_waves, int lane)
{
    const int row = lane / kRowLanes;
    const int l = lane % kRowLanes;
    double m = 0.0;
    for (int ebase = wave * kRowsPerWave; ebase < E; ebase += n_waves * kRowsPerWave) {
        const int e = ebase + row;
        int c0 = 0, c1 = 0;
        if (e < E) {
            c0 = link_chunk_ptr[e];
            c1 = link_chunk_ptr[e + 1];
        }
        const double reach = row_partial_sum(c0, c1, l, partial);
        if (e < E) m = fmax(m, reach * invcap[e]);
    }
    return m;
}

}  // namespace nimble

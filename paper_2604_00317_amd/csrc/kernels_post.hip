// Plan post-processing: split fractions -> bytes per candidate path in whole chunks.
//
// The dataplane consumes, per pair, a list of paths with a byte amount each (the Paths / Flows
// lists of Algorithm 1); messages must not be fragmented below the chunk granularity and small
// messages stay off the multi-hop paths (Sec. V-A switches forwarding off for messages of 1 MB
// or less).  A pair at or below the threshold keeps everything on its first candidate;
// otherwise its N = floor(d / chi) whole chunks are apportioned to the candidates by largest
// remainder (quota floor(N * c_j / T), the left-over chunks to the largest remainders
// N * c_j mod T, ties to the lower index) and the residual d - N * chi joins the candidate with
// the largest count.  Chunk numbers are exact 64-bit integers.  Two kernels compute the same
// numbers: a group of L lanes per pair, one candidate per lane (pairs of up to 64 candidates:
// coalesced reads and writes, one division per candidate, ranks by rotating the remainders
// round the group), and one thread per pair for anything wider.
#include <hip/hip_runtime.h>

#include "kernels.hpp"
#include "wave_ops.hpp"

namespace nimble {

namespace {

constexpr int kPostBlock = 256;

__global__ __launch_bounds__(kPostBlock) void k_quantize(int K, const int32_t *__restrict__ cp,
                                                         const double *__restrict__ demand,
                                                         const double *__restrict__ splits,
                                                         int iters, long long chi, double theta,
                                                         double *__restrict__ flows)
{
    const int k = blockIdx.x * kPostBlock + threadIdx.x;
    if (k >= K) return;
    const int a = cp[k], n = cp[k + 1] - a;
    if (n == 0) return;
    const double dk = demand[k];
    if (dk <= theta) {                                   // small message: first candidate only
        flows[a] = dk;
        for (int j = 1; j < n; ++j) flows[a + j] = 0.0;
        return;
    }
    const double T = static_cast<double>(iters);
    const double chi_d = static_cast<double>(chi);
    const double whole = floor(dk / chi_d);
    if (!(whole < 2147483648.0)) {                       // N * c_j would leave 64 bits
        for (int j = 0; j < n; ++j) flows[a + j] = __builtin_nan("");
        return;
    }
    const long long N = static_cast<long long>(whole);
    const double res = dk - static_cast<double>(N * chi);
    long long sum_q = 0, c_max = -1;
    int j_max = 0;
    for (int j = 0; j < n; ++j) {
        const long long c = llrint(splits[a + j] * T);
        sum_q += (N * c) / iters;
        if (c > c_max) {
            c_max = c;
            j_max = j;
        }
    }
    const long long R = N - sum_q;                       // chunks left over, fewer than n
    for (int j = 0; j < n; ++j) {
        const long long c = llrint(splits[a + j] * T);
        const long long q = (N * c) / iters;
        const long long rem = (N * c) % iters;
        long long rank = 0;                              // candidates ahead of j for a left-over
        for (int i = 0; i < n; ++i) {
            const long long ci = llrint(splits[a + i] * T);
            const long long ri = (N * ci) % iters;
            rank += (ri > rem || (ri == rem && i < j)) ? 1 : 0;
        }
        double f = static_cast<double>(chi * (q + (rank < R ? 1 : 0)));
        if (j == j_max) f = f + res;
        flows[a + j] = f;
    }
}

template <int L>
__device__ __forceinline__ int group_sum_i32(int v)
{
    if constexpr (L > 1) v += partner_i32<1>(v);
    if constexpr (L > 2) v += partner_i32<2>(v);
    if constexpr (L > 4) v += partner_i32<4>(v);
    if constexpr (L > 8) v += partner_i32<8>(v);
    if constexpr (L > 16) v += partner_i32<16>(v);
    if constexpr (L > 32) v += partner_i32<32>(v);
    return v;
}

template <int L>
__device__ __forceinline__ int group_max_i32(int v)
{
    if constexpr (L > 1) v = max(v, partner_i32<1>(v));
    if constexpr (L > 2) v = max(v, partner_i32<2>(v));
    if constexpr (L > 4) v = max(v, partner_i32<4>(v));
    if constexpr (L > 8) v = max(v, partner_i32<8>(v));
    if constexpr (L > 16) v = max(v, partner_i32<16>(v));
    if constexpr (L > 32) v = max(v, partner_i32<32>(v));
    return v;
}

// One comparison of the rank count.  Every candidate carries a key that orders the claims on
// the left-over chunks: the remainder in the high bits and 63 - lane below, so a larger key is
// a larger remainder, or the same remainder at a lower index (lanes of a group are in index
// order).  Groups narrower than a DPP row also see keys of their neighbours in the row, which
// do not count.
template <int L>
__device__ __forceinline__ void rank_one(long long ko, int il, long long key, int lane, int &rank)
{
    bool ahead = ko > key;
    if constexpr (L < 16) ahead = ahead && (((il ^ lane) & ~(L - 1)) == 0);
    rank += ahead ? 1 : 0;
}
template <int L>
__device__ __forceinline__ void rank_one(int ko, int il, int key, int lane, int &rank)
{
    bool ahead = ko > key;
    if constexpr (L < 16) ahead = ahead && (((il ^ lane) & ~(L - 1)) == 0);
    rank += ahead ? 1 : 0;
}

template <int CTRL>
__device__ __forceinline__ long long dpp_key(long long v)
{
    const int lo = dpp_i32<CTRL>(static_cast<int>(v));
    const int hi = dpp_i32<CTRL>(static_cast<int>(v >> 32));
    return (static_cast<long long>(hi) << 32) | static_cast<unsigned int>(lo);
}
template <int CTRL>
__device__ __forceinline__ int dpp_key(int v)
{
    return dpp_i32<CTRL>(v);
}

// The same against the keys of a 16-lane row rotated by 1..S lanes (DPP row_ror: lane p of a
// row receives from lane (p - S) mod 16 of the same row).
template <int L, int S>
struct RankRow {
    template <typename KEY>
    static __device__ __forceinline__ void add(KEY v, int row_lane0, KEY key, int lane, int &rank)
    {
        RankRow<L, S - 1>::add(v, row_lane0, key, lane, rank);
        const int il = row_lane0 | ((lane - S) & 15);
        rank_one<L>(dpp_key<0x120 + S>(v), il, key, lane, rank);
    }
};
template <int L>
struct RankRow<L, 0> {
    template <typename KEY>
    static __device__ __forceinline__ void add(KEY, int, KEY, int, int &) {}
};

template <int L, typename KEY>
__device__ __forceinline__ int group_rank(KEY key, int lane)
{
    int rank = 0;
    RankRow<L, 15>::add(key, lane & ~15, key, lane, rank);
    if constexpr (L > 16) {
        const KEY k1 = __shfl_xor(key, 16, kWave);
        rank_one<L>(k1, lane ^ 16, key, lane, rank);
        RankRow<L, 15>::add(k1, (lane ^ 16) & ~15, key, lane, rank);
    }
    if constexpr (L > 32) {
        const KEY k2 = __shfl_xor(key, 32, kWave);
        rank_one<L>(k2, lane ^ 32, key, lane, rank);
        RankRow<L, 15>::add(k2, (lane ^ 32) & ~15, key, lane, rank);
        const KEY k3 = __shfl_xor(key, 48, kWave);
        rank_one<L>(k3, lane ^ 48, key, lane, rank);
        RankRow<L, 15>::add(k3, (lane ^ 48) & ~15, key, lane, rank);
    }
    return rank;
}

// L lanes per pair (L a power of two, every pair has at most L candidates); the lanes of a
// group take the same branches, so the cross-lane steps are reached by whole groups.
template <int L>
__global__ __launch_bounds__(kPostBlock) void k_quantize_group(int K,
                                                               const int32_t *__restrict__ cp,
                                                               const double *__restrict__ demand,
                                                               const double *__restrict__ splits,
                                                               int iters, long long chi,
                                                               double theta,
                                                               double *__restrict__ flows)
{
    const long long tid = static_cast<long long>(blockIdx.x) * kPostBlock + threadIdx.x;
    const long long kk = tid / L;
    const int j = static_cast<int>(tid % L);
    const int k = kk < K ? static_cast<int>(kk) : K;
    const int lane = threadIdx.x & (kWave - 1);
    const bool pair_ok = k < K;
    int a = 0, n = 0;
    double dk = 0.0;
    if (pair_ok) {
        a = cp[k];
        n = cp[k + 1] - a;
        dk = demand[k];
    }
    const bool mine = j < n;
    const double T = static_cast<double>(iters);
    const double chi_d = static_cast<double>(chi);
    const double whole = floor(dk / chi_d);
    const bool small = dk <= theta;
    const bool wide = !(whole < 2147483648.0);           // N * c_j would leave 64 bits
    const long long N = (small || wide) ? 0 : static_cast<long long>(whole);
    const double res = dk - static_cast<double>(N * chi);
    long long c = -1, q = 0;
    int rem = -1;                                        // absent candidates rank behind all
    if (mine) {
        c = llrint(splits[a + j] * T);
        // floor(N * c / T): the quotient is below 2^31, so the double quotient is within one
        // of it and one exact correction step either way settles it
        const long long nc = N * c;
        q = static_cast<long long>(static_cast<double>(nc) / T);
        long long r = nc - q * iters;
        if (r < 0) {
            q -= 1;
            r += iters;
        } else if (r >= iters) {
            q += 1;
            r -= iters;
        }
        rem = static_cast<int>(r);
    }
    // left-over chunks of the pair: fewer than n (every quota is below 2^31, and so is the sum)
    const int R = static_cast<int>(N) - group_sum_i32<L>(static_cast<int>(q));
    // the candidate with the largest count, the lowest index among equals
    const int ci = static_cast<int>(c);                  // c <= iters < 2^31
    const int c_max = group_max_i32<L>(ci);
    int j_max = (ci == c_max) ? j : 0x7FFFFFFF;
    if constexpr (L > 1) j_max = min(j_max, partner_i32<1>(j_max));
    if constexpr (L > 2) j_max = min(j_max, partner_i32<2>(j_max));
    if constexpr (L > 4) j_max = min(j_max, partner_i32<4>(j_max));
    if constexpr (L > 8) j_max = min(j_max, partner_i32<8>(j_max));
    if constexpr (L > 16) j_max = min(j_max, partner_i32<16>(j_max));
    if constexpr (L > 32) j_max = min(j_max, partner_i32<32>(j_max));
    // candidates ahead of j for a left-over chunk; the key fits 32 bits unless the iteration
    // count is huge (wave-uniform choice)
    int rank;
    if (iters < (1 << 24)) {
        const int key = mine ? ((rem << 6) | (63 - lane)) : -1;
        rank = group_rank<L, int>(key, lane);
    } else {
        const long long key = mine ? ((static_cast<long long>(rem) << 6) | (63 - lane)) : -1;
        rank = group_rank<L, long long>(key, lane);
    }
    if (!mine) return;
    double f;
    if (small) f = (j == 0) ? dk : 0.0;                  // small message: first candidate only
    else if (wide) f = __builtin_nan("");
    else {
        f = static_cast<double>(chi * (q + (rank < R ? 1 : 0)));
        if (j == j_max) f = f + res;
    }
    flows[a + j] = f;
}

}  // namespace

hipError_t launch_quantize(const DeviceTopo &t, const double *demand, const double *splits,
                           int32_t iters, int64_t chi, double theta, double *flows,
                           hipStream_t s)
{
    if (t.pmax <= kWave) {
        const int L = lanes_per_commodity(t.pmax);
        const int64_t threads = static_cast<int64_t>(t.K) * L;
        const int g = static_cast<int>((threads + kPostBlock - 1) / kPostBlock);
#define NIMBLE_QUANT_LAUNCH(LL)                                                                \
    case LL:                                                                                   \
        hipLaunchKernelGGL(k_quantize_group<LL>, dim3(g), dim3(kPostBlock), 0, s, t.K,         \
                           t.comm_ptr, demand, splits, iters, static_cast<long long>(chi),     \
                           theta, flows);                                                      \
        return hipGetLastError();
        switch (L) {
            NIMBLE_QUANT_LAUNCH(1)
            NIMBLE_QUANT_LAUNCH(2)
            NIMBLE_QUANT_LAUNCH(4)
            NIMBLE_QUANT_LAUNCH(8)
            NIMBLE_QUANT_LAUNCH(16)
            NIMBLE_QUANT_LAUNCH(32)
            NIMBLE_QUANT_LAUNCH(64)
        }
#undef NIMBLE_QUANT_LAUNCH
    }
    const int grid = (t.K + kPostBlock - 1) / kPostBlock;
    hipLaunchKernelGGL(k_quantize, dim3(grid), dim3(kPostBlock), 0, s, t.K, t.comm_ptr, demand,
                       splits, iters, static_cast<long long>(chi), theta, flows);
    return hipGetLastError();
}

}  // namespace nimble

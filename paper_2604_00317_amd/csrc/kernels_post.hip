// Plan post-processing: split fractions -> bytes per candidate path in whole chunks.
//
// The dataplane consumes, per pair, a list of paths with a byte amount each (the Paths / Flows
// lists of Algorithm 1); messages must not be fragmented below the chunk granularity and small
// messages stay off the multi-hop paths (Sec. V-A switches forwarding off for messages of 1 MB
// or less).  One thread per pair: a pair at or below the threshold keeps everything on its first
// candidate; otherwise its N = floor(d / chi) whole chunks are apportioned to the candidates
// by largest remainder (quota floor(N * c_j / T), the left-over chunks to the largest
// remainders N * c_j mod T, ties to the lower index) and the residual d - N * chi joins the
// candidate with the largest count.  Chunk numbers are exact 64-bit integers.
#include <hip/hip_runtime.h>

#include "kernels.hpp"

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

}  // namespace

hipError_t launch_quantize(const DeviceTopo &t, const double *demand, const double *splits,
                           int32_t iters, int64_t chi, double theta, double *flows,
                           hipStream_t s)
{
    const int grid = (t.K + kPostBlock - 1) / kPostBlock;
    hipLaunchKernelGGL(k_quantize, dim3(grid), dim3(kPostBlock), 0, s, t.K, t.comm_ptr, demand,
                       splits, iters, static_cast<long long>(chi), theta, flows);
    return hipGetLastError();
}

}  // namespace nimble

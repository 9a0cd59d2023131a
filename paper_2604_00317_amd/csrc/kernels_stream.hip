// Streaming regime: three kernels per Jacobi iteration.
//   argmin       path-cost gather over the path->link CSR + per-commodity argmin
//                (lowest index wins ties, the strict `<` scan of Algorithm 1)
//   load_reduce  link loads over the reverse link->(commodity,path) CSR in fixed-size chunks,
//                fixed reduction tree, no floating-point atomics (Algorithm 1: L_e += f)
//   update       chunk partials -> load, congestion sum S_e, multiplicative length update
//                len_e *= 1 + eps*u_e/rho, new price, per-block max of S (lambda)
// All arithmetic is binary64 with one IEEE operation per statement (no contraction).
#include "host_topo.hpp"
#include "kernels.hpp"
#include "wave_ops.hpp"

namespace nimble {

namespace {

constexpr int kBlock = 256;

__global__ __launch_bounds__(kBlock) void k_init(int E, int K, int P, bool cost_max,
                                                 const double *__restrict__ invcap,
                                                 double *__restrict__ len,
                                                 double *__restrict__ price,
                                                 double *__restrict__ S,
                                                 uint8_t *__restrict__ choice,
                                                 uint32_t *__restrict__ count)
{
    const int stride = gridDim.x * blockDim.x;
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    for (int e = tid; e < E; e += stride) {
        len[e] = 1.0;
        price[e] = cost_max ? 1.0 : invcap[e];
        S[e] = 0.0;
    }
    for (int p = tid; p < P; p += stride) count[p] = 0u;
    if (tid == 0) choice[K] = 0xFFu;
}

// L lanes cooperate on one commodity: lane j evaluates candidates j, j+L, ...
template <int L, bool MAXC>
__global__ __launch_bounds__(kBlock) void k_argmin(int K, const int32_t *__restrict__ cp,
                                                   const int32_t *__restrict__ lp,
                                                   const int32_t *__restrict__ pl,
                                                   const double *__restrict__ price,
                                                   uint8_t *__restrict__ choice,
                                                   uint32_t *__restrict__ count)
{
    constexpr int kPerWave = kWave / L;
    const int lane = threadIdx.x & (kWave - 1);
    const int sub = lane / L;          // commodity slot inside the wave
    const int j0 = lane % L;           // first candidate of this lane
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    // wave-uniform loop so that every lane reaches the cross-lane reduction
    for (int base = wave * kPerWave; base < K; base += n_waves * kPerWave) {
        const int k = base + sub;
        double best = __builtin_inf();
        int bj = 0x7FFFFFFF;
        int p0 = 0;
        if (k < K) {
            p0 = cp[k];
            const int np = cp[k + 1] - p0;
            if (j0 < np) bj = j0;      // an all-infinite commodity still resolves to candidate 0
            for (int j = j0; j < np; j += L) {
                const int a = lp[p0 + j], b = lp[p0 + j + 1];
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
            }
        }
        group_argmin<L>(best, bj);
        if (k < K && j0 == 0) {
            choice[k] = static_cast<uint8_t>(bj);
            count[p0 + bj] += 1u;
        }
    }
}

// One wave per chunk of the reverse CSR.  MODE 0: an entry contributes d_k when candidate j is
// the chosen one.  MODE 1 (width rho): an entry contributes when it is the first of its
// commodity in the row, i.e. every commodity that can reach the link counts once.
template <int MODE>
__global__ __launch_bounds__(kBlock) void k_load_reduce(int n_chunks,
                                                        const int32_t *__restrict__ chunk_begin,
                                                        const int32_t *__restrict__ chunk_end,
                                                        const uint32_t *__restrict__ rev,
                                                        const uint8_t *__restrict__ choice,
                                                        const double *__restrict__ demand,
                                                        double *__restrict__ partial)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    for (int c = wave; c < n_chunks; c += n_waves) {
        const int b = chunk_begin[c], e = chunk_end[c];
        double acc = 0.0;
        for (int i = b + lane * 4; i < e; i += kWave * 4) {
            const uint4 v = *reinterpret_cast<const uint4 *>(rev + i);
            const uint32_t ent[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t k = (ent[q] >> kPathBits) & kCommMask;
                bool hit;
                if constexpr (MODE == 0) hit = choice[k] == (ent[q] & kPathMask);
                else hit = (ent[q] & kFirstFlag) != 0u;
                if (hit) acc = acc + demand[k];
            }
        }
        acc = wave_sum(acc);
        if (lane == 0) partial[c] = acc;
    }
}

// reach_e = sum of chunk partials, rho = max_e reach_e / cap_e, scalars[0] = 1/rho (0 if rho=0)
__global__ __launch_bounds__(1024) void k_width(int E, const int32_t *__restrict__ link_chunk_ptr,
                                                const double *__restrict__ partial,
                                                const double *__restrict__ invcap,
                                                double *__restrict__ scalars)
{
    __shared__ double red[16];
    double m = 0.0;
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        double reach = 0.0;
        for (int c = link_chunk_ptr[e]; c < link_chunk_ptr[e + 1]; ++c) reach = reach + partial[c];
        const double w = reach * invcap[e];
        m = fmax(m, w);
    }
    m = block_max(m, red);
    if (threadIdx.x == 0) scalars[0] = (m > 0.0) ? 1.0 / m : 0.0;
}

template <bool MAXC>
__global__ __launch_bounds__(kBlock) void k_update(int E, double eps,
                                                   const int32_t *__restrict__ link_chunk_ptr,
                                                   const double *__restrict__ partial,
                                                   const double *__restrict__ invcap,
                                                   double *__restrict__ len,
                                                   double *__restrict__ price,
                                                   double *__restrict__ S,
                                                   double *__restrict__ scalars)
{
    __shared__ double red[16];
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    double s_new = 0.0;
    if (e < E) {
        const double invrho = scalars[0];
        double load = 0.0;
        for (int c = link_chunk_ptr[e]; c < link_chunk_ptr[e + 1]; ++c) load = load + partial[c];
        const double ic = invcap[e];
        const double u = load * ic;
        s_new = S[e] + u;
        S[e] = s_new;
        const double g = u * invrho;
        const double t1 = eps * g;
        const double t2 = 1.0 + t1;
        const double l = len[e] * t2;
        len[e] = l;
        price[e] = MAXC ? l : l * ic;
    }
    const double m = block_max(s_new, red);
    if (threadIdx.x == 0) scalars[1 + blockIdx.x] = m;
}

__global__ __launch_bounds__(kBlock) void k_epilogue(int P, int iters, int n_update_blocks,
                                                     const uint32_t *__restrict__ count,
                                                     const double *__restrict__ scalars,
                                                     double *__restrict__ splits,
                                                     double *__restrict__ lambda)
{
    __shared__ double red[16];
    const double T = static_cast<double>(iters);
    const int stride = gridDim.x * blockDim.x;
    for (int p = blockIdx.x * blockDim.x + threadIdx.x; p < P; p += stride)
        splits[p] = static_cast<double>(count[p]) / T;
    if (blockIdx.x == 0) {
        double m = 0.0;
        for (int b = threadIdx.x; b < n_update_blocks; b += blockDim.x)
            m = fmax(m, scalars[1 + b]);
        m = block_max(m, red);
        if (threadIdx.x == 0) lambda[0] = m / T;
    }
}

inline int blocks_for(int64_t threads, int block, int cap)
{
    int64_t b = (threads + block - 1) / block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return static_cast<int>(b);
}

template <bool MAXC>
void launch_argmin_l(const DeviceTopo &t, hipStream_t s)
{
    int L = 1;
    while (L < t.pmax && L < kWave) L <<= 1;
    const int grid = blocks_for(static_cast<int64_t>(t.K) * L, kBlock, 1 << 20);
#define NIMBLE_ARGMIN_CASE(LL)                                                                 \
    case LL:                                                                                   \
        hipLaunchKernelGGL((k_argmin<LL, MAXC>), dim3(grid), dim3(kBlock), 0, s, t.K,          \
                           t.comm_ptr, t.path_ptr, t.path_links, t.price, t.choice, t.count);  \
        break;
    switch (L) {
        NIMBLE_ARGMIN_CASE(1)
        NIMBLE_ARGMIN_CASE(2)
        NIMBLE_ARGMIN_CASE(4)
        NIMBLE_ARGMIN_CASE(8)
        NIMBLE_ARGMIN_CASE(16)
        NIMBLE_ARGMIN_CASE(32)
        NIMBLE_ARGMIN_CASE(64)
    }
#undef NIMBLE_ARGMIN_CASE
}

}  // namespace

void launch_init(const DeviceTopo &t, hipStream_t s)
{
    const int n = t.E > t.P ? t.E : t.P;
    hipLaunchKernelGGL(k_init, dim3(blocks_for(n, kBlock, 4096)), dim3(kBlock), 0, s, t.E, t.K,
                       t.P, t.cost_max, t.invcap, t.len, t.price, t.S, t.choice, t.count);
}

void launch_width(const DeviceTopo &t, const double *demand, hipStream_t s)
{
    if (t.n_chunks > 0)
        hipLaunchKernelGGL(k_load_reduce<1>,
                           dim3(blocks_for(static_cast<int64_t>(t.n_chunks) * kWave, kBlock,
                                           1 << 20)),
                           dim3(kBlock), 0, s, t.n_chunks, t.chunk_begin, t.chunk_end,
                           t.rev_entry, t.choice, demand, t.partial);
    hipLaunchKernelGGL(k_width, dim3(1), dim3(1024), 0, s, t.E, t.link_chunk_ptr, t.partial,
                       t.invcap, t.scalars);
}

void launch_argmin(const DeviceTopo &t, hipStream_t s)
{
    if (t.cost_max) launch_argmin_l<true>(t, s);
    else launch_argmin_l<false>(t, s);
}

void launch_load_reduce(const DeviceTopo &t, const double *demand, hipStream_t s)
{
    hipLaunchKernelGGL(k_load_reduce<0>,
                       dim3(blocks_for(static_cast<int64_t>(t.n_chunks) * kWave, kBlock, 1 << 20)),
                       dim3(kBlock), 0, s, t.n_chunks, t.chunk_begin, t.chunk_end, t.rev_entry,
                       t.choice, demand, t.partial);
}

void launch_update(const DeviceTopo &t, double eps, hipStream_t s)
{
    if (t.cost_max)
        hipLaunchKernelGGL(k_update<true>, dim3(t.n_update_blocks), dim3(kBlock), 0, s, t.E, eps,
                           t.link_chunk_ptr, t.partial, t.invcap, t.len, t.price, t.S, t.scalars);
    else
        hipLaunchKernelGGL(k_update<false>, dim3(t.n_update_blocks), dim3(kBlock), 0, s, t.E, eps,
                           t.link_chunk_ptr, t.partial, t.invcap, t.len, t.price, t.S, t.scalars);
}

void launch_epilogue(const DeviceTopo &t, int32_t iters, double *splits, double *lambda,
                     hipStream_t s)
{
    hipLaunchKernelGGL(k_epilogue, dim3(blocks_for(t.P, kBlock, 4096)), dim3(kBlock), 0, s, t.P,
                       iters, t.n_update_blocks, t.count, t.scalars, splits, lambda);
}

}  // namespace nimble

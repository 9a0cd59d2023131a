// Adaptive-step variant of the streaming regime: step sigma_t = 1 / max_e u_e^t, the plan is the
// sigma-weighted average of the iterations' routings, and every check_every iterations the
// weak-duality bound  LB = (sum_k d_k * cheapest cost_k) / (sum_e len_e)  decides whether the
// solve may stop (lambda <= (1 + eps)^2 * best LB).  The candidate scan and the link-load
// reduce are the streaming regime's kernels; this file holds the small kernels around them.
// The two sums of the bound have a fixed association (sequential inside chunks of 256
// consecutive terms, the chunk sums sequential), which one thread per chunk reproduces.
#include <hip/hip_runtime.h>

#include "kernels.hpp"
#include "phases.hpp"
#include "wave_ops.hpp"

namespace nimble {

namespace {

constexpr int kAdBlock = 256;
constexpr int kAdChunk = 256;

// d_k times the cost of the candidate commodity k has just chosen (= its cheapest: the sum
// is taken link by link in path order, exactly as the scan took it)
template <bool MAXC>
__global__ __launch_bounds__(kAdBlock) void k_ad_terms(int K, const int32_t *__restrict__ cp,
                                                       const int32_t *__restrict__ lp,
                                                       const int32_t *__restrict__ pl,
                                                       const double *__restrict__ price,
                                                       const uint8_t *__restrict__ choice,
                                                       const double *__restrict__ demand,
                                                       const int32_t *__restrict__ flags,
                                                       double *__restrict__ term)
{
    if (flags[0]) return;
    const int k = blockIdx.x * kAdBlock + threadIdx.x;
    if (k >= K) return;
    const int p = cp[k] + choice[k];
    double c = 0.0;
    for (int i = lp[p]; i < lp[p + 1]; ++i) {
        const double pe = price[pl[i]];
        if constexpr (MAXC) c = (pe > c) ? pe : c;
        else c = c + pe;
    }
    term[k] = demand[k] * c;
}

// chunk sums: chunk c is the sum of the terms 256c .. 256c + 255 added in order; `index` (may be
// null) redirects term i to x[index[i]].  A workgroup owns kAdChunksPerBlock chunks: all its
// threads fetch the terms side by side (coalesced) into LDS, a padded row per chunk so that
// the rows start in different banks, and one thread per chunk then adds its row in order.
constexpr int kAdChunksPerBlock = 4;
constexpr int kAdRow = kAdChunk + 1;

// x[0] + x[1] + ... + x[n-1] added strictly in that order by one thread.  The additions form
// one dependent chain whatever is done; what can be avoided is waiting for every term in turn:
// sixteen terms are fetched side by side, then added one after the other.
__device__ __forceinline__ double ordered_sum(const double *x, int n)
{
    double s = 0.0;
    int i = 0;
    for (; i + 16 <= n; i += 16) {
        double v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = x[i + j];
#pragma unroll
        for (int j = 0; j < 16; ++j) s = s + v[j];
    }
    for (; i < n; ++i) s = s + x[i];
    return s;
}

__global__ __launch_bounds__(kAdBlock) void k_ad_chunks(int n, const double *__restrict__ x,
                                                        const int32_t *__restrict__ index,
                                                        const int32_t *__restrict__ flags,
                                                        double *__restrict__ chunk)
{
    __shared__ double s_terms[kAdChunksPerBlock * kAdRow];
    if (flags[0]) return;
    const int c0 = blockIdx.x * kAdChunksPerBlock;
    const int first = c0 * kAdChunk;
    // (all terms of the workgroup are requested before the first is stored)
    constexpr int kPer = kAdChunksPerBlock * kAdChunk / kAdBlock;
    double v[kPer];
#pragma unroll
    for (int r = 0; r < kPer; ++r) {
        const int i = first + r * kAdBlock + static_cast<int>(threadIdx.x);
        v[r] = 0.0;
        if (i < n) v[r] = x[index ? index[i] : i];
    }
#pragma unroll
    for (int r = 0; r < kPer; ++r) {
        const int q = r * kAdBlock + static_cast<int>(threadIdx.x);
        s_terms[(q / kAdChunk) * kAdRow + (q % kAdChunk)] = v[r];
    }
    __syncthreads();
    const int c = c0 + threadIdx.x;
    if (threadIdx.x < kAdChunksPerBlock && c * kAdChunk < n) {
        const int len = n - c * kAdChunk < kAdChunk ? n - c * kAdChunk : kAdChunk;
        chunk[c] = ordered_sum(s_terms + threadIdx.x * kAdRow, len);
    }
}

// ascal: [0] W, [1] bound of this check, [2] best bound, [3] lambda.  The chunk sums are added
// in order by one thread, from LDS.
__global__ __launch_bounds__(kAdBlock) void k_ad_lb(int n_alpha, const double *chunk_alpha,
                                                    int n_d, const double *chunk_d,
                                                    const int32_t *__restrict__ flags,
                                                    double *__restrict__ ascal, bool staged)
{
    extern __shared__ double s_chunks[];
    if (flags[0]) return;
    if (staged) {
        for (int i = threadIdx.x; i < n_alpha; i += kAdBlock) s_chunks[i] = chunk_alpha[i];
        for (int i = threadIdx.x; i < n_d; i += kAdBlock) s_chunks[n_alpha + i] = chunk_d[i];
        __syncthreads();
        chunk_alpha = s_chunks;
        chunk_d = s_chunks + n_alpha;
    }
    // two threads, one sum each
    __shared__ double s_sum[2];
    if (threadIdx.x == 0) s_sum[0] = ordered_sum(chunk_alpha, n_alpha);
    if (threadIdx.x == kWave) s_sum[1] = ordered_sum(chunk_d, n_d);
    __syncthreads();
    if (threadIdx.x == 0) ascal[1] = s_sum[0] / s_sum[1];
}

// normalised loads u = load / cap by position, and the maximum of every block; RL lanes per link
template <int RL>
__global__ __launch_bounds__(kAdBlock) void k_ad_u(int E, const int32_t *__restrict__ pos_slot_ptr,
                                                   const int2 *__restrict__ pos_xslot,
                                                   const double *__restrict__ partial,
                                                   const double *__restrict__ invcap_pos,
                                                   const int32_t *__restrict__ flags,
                                                   double *__restrict__ u_pos,
                                                   double *__restrict__ block_max_u)
{
    __shared__ double red[16];
    if (flags[0]) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int row = lane / RL, l = lane % RL;
    const int i = ((blockIdx.x * kAdBlock + threadIdx.x) >> 6) * (kWave / RL) + row;
    int c0 = 0, c1 = 0, s0 = 0, s1 = 0;
    if (i < E) {
        c0 = pos_slot_ptr[i];
        c1 = pos_slot_ptr[i + 1];
        const int2 xs = pos_xslot[i];
        s0 = xs.x;
        s1 = xs.y;
    }
    const double load =
        row_partial_sum<RL>(c0, c1, l, partial) + row_partial_sum<RL>(s0, s1, l, partial);
    double u = 0.0;
    if (i < E) {
        u = load * invcap_pos[i];
        if (l == 0) u_pos[i] = u;
    }
    const double m = block_max(u, red);
    if (threadIdx.x == 0) block_max_u[blockIdx.x] = m;
}

// sigma = 1 / max u; S += sigma * u; len *= 1 + eps * sigma * u; price; W += sigma
template <bool MAXC>
__global__ __launch_bounds__(kAdBlock) void k_ad_apply(
    int E, double eps, int n_u_blocks, const double *__restrict__ block_max_u,
    const double *__restrict__ u_pos, const double *__restrict__ invcap_pos,
    const int32_t *__restrict__ pos_link, double *__restrict__ len, double *__restrict__ price,
    double *__restrict__ S, int32_t *__restrict__ flags, double *__restrict__ ascal,
    double *__restrict__ sigma_log, double *__restrict__ block_max_s)
{
    __shared__ double red[16];
    // the stop word, the link's own state and the maxima are requested together (threads past
    // the last link re-read it), so that one trip to memory serves all three
    const int32_t stop_now = *static_cast<const volatile int32_t *>(flags);
    const int i = blockIdx.x * kAdBlock + threadIdx.x;
    const int ic = i < E ? i : E - 1;
    const double u_i = u_pos[ic];
    const double s_old = S[ic];
    const double l_old = len[ic];
    const double cap_i = invcap_pos[ic];
    const int e_i = pos_link[ic];
    double m = 0.0;
    for (int b = threadIdx.x; b < n_u_blocks; b += kAdBlock) m = fmax(m, block_max_u[b]);
    if (stop_now != 0) return;
    const double umax = block_max(m, red);
    if (!(umax > 0.0)) {                               // no traffic at all: the solve ends here
        if (blockIdx.x == 0 && threadIdx.x == 0) flags[0] = 1;
        return;
    }
    const double sigma = 1.0 / umax;
    double s_new = 0.0;
    if (i < E) {
        const double su = sigma * u_i;
        s_new = s_old + su;
        S[i] = s_new;
        const double t1 = eps * su;
        const double t2 = 1.0 + t1;
        const double ln = l_old * t2;
        len[i] = ln;
        price[e_i] = MAXC ? ln : ln * cap_i;
    }
    __syncthreads();
    const double sm = block_max(s_new, red);
    if (threadIdx.x == 0) {
        block_max_s[blockIdx.x] = sm;
        if (blockIdx.x == 0) {
            ascal[0] = ascal[0] + sigma;
            sigma_log[flags[1]] = sigma;
            flags[1] = flags[1] + 1;
        }
    }
}

// lambda = max S / W; at a check the best bound is updated and the stop test made
__global__ __launch_bounds__(kAdBlock) void k_ad_lambda(int n_s_blocks,
                                                        const double *__restrict__ block_max_s,
                                                        double gap, int check,
                                                        int32_t *__restrict__ flags,
                                                        double *__restrict__ ascal,
                                                        int32_t *host_words)
{
    __shared__ double red[16];
    // what the host reads while it enqueues ahead: whether the solve has stopped and how many
    // checks have been made (written to pinned host memory at system scope)
    auto publish = [&]() {
        __hip_atomic_store(host_words, flags[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(host_words + 1, check, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    };
    if (flags[0] && check) {                          // already stopped
        if (threadIdx.x == 0) publish();
        return;
    }
    double m = 0.0;
    for (int b = threadIdx.x; b < n_s_blocks; b += kAdBlock) m = fmax(m, block_max_s[b]);
    const double smax = block_max(m, red);
    if (threadIdx.x != 0) return;
    const double W = ascal[0];
    const double lam = W > 0.0 ? smax / W : 0.0;
    ascal[3] = lam;
    if (check) {
        if (ascal[1] > ascal[2]) ascal[2] = ascal[1];
        const double bound = gap * ascal[2];
        if (lam <= bound) flags[0] = 1;
        publish();
    }
}

__global__ void k_ad_reset(int32_t *__restrict__ flags, double *__restrict__ ascal)
{
    if (threadIdx.x == 0) {
        flags[0] = 0;
        flags[1] = 0;
        ascal[0] = 0.0;
        ascal[1] = 0.0;
        ascal[2] = 0.0;
        ascal[3] = 0.0;
    }
}

// sigma-weighted split fractions from the choice log: one lane per commodity adds sigma_t to
// the weight of the candidate chosen in iteration t, t ascending, in LDS
__global__ __launch_bounds__(kWave) void k_ad_histogram(int K, int pmax, size_t stride,
                                                        const uint8_t *__restrict__ log,
                                                        const int32_t *__restrict__ cp,
                                                        const double *__restrict__ sigma_log,
                                                        const int32_t *__restrict__ flags,
                                                        const double *__restrict__ ascal,
                                                        double *__restrict__ splits,
                                                        double *__restrict__ lambda)
{
    extern __shared__ double s_w[];
    const int lane = threadIdx.x;
    const int k = blockIdx.x * kWave + lane;
    const int iters = flags[1];
    const double W = ascal[0];
    const int row = pmax | 1;                      // odd row length: conflict-free columns
    double *mine = s_w + lane * row;
    for (int j = 0; j < pmax; ++j) mine[j] = 0.0;
    if (k < K) {
        const uint8_t *col = log + k;
        for (int t = 0; t < iters; ++t) {
            const int c = col[size_t(t) * stride];
            mine[c] = mine[c] + sigma_log[t];
        }
        const int p0 = cp[k], np = cp[k + 1] - p0;
        for (int j = 0; j < np; ++j)
            splits[p0 + j] = W > 0.0 ? mine[j] / W : (j == 0 ? 1.0 : 0.0);
    }
    if (blockIdx.x == 0 && lane == 0) lambda[0] = ascal[3];
}

}  // namespace

void launch_ad_reset(const AdaptiveState &a, hipStream_t s)
{
    hipLaunchKernelGGL(k_ad_reset, dim3(1), dim3(64), 0, s, a.flags, a.ascal);
}

void launch_ad_bound(const DeviceTopo &t, const AdaptiveState &a, const uint8_t *choice,
                     const double *demand, hipStream_t s)
{
    const int gk = (t.K + kAdBlock - 1) / kAdBlock;
    if (t.cost_max)
        hipLaunchKernelGGL(k_ad_terms<true>, dim3(gk), dim3(kAdBlock), 0, s, t.K, t.comm_ptr,
                           t.path_ptr, t.path_links, t.price, choice, demand, a.flags, a.term);
    else
        hipLaunchKernelGGL(k_ad_terms<false>, dim3(gk), dim3(kAdBlock), 0, s, t.K, t.comm_ptr,
                           t.path_ptr, t.path_links, t.price, choice, demand, a.flags, a.term);
    const int n_alpha = (t.K + kAdChunk - 1) / kAdChunk, n_d = (t.E + kAdChunk - 1) / kAdChunk;
    hipLaunchKernelGGL(k_ad_chunks,
                       dim3((n_alpha + kAdChunksPerBlock - 1) / kAdChunksPerBlock), dim3(kAdBlock),
                       0, s, t.K, a.term, static_cast<const int32_t *>(nullptr), a.flags, a.chunk);
    hipLaunchKernelGGL(k_ad_chunks, dim3((n_d + kAdChunksPerBlock - 1) / kAdChunksPerBlock),
                       dim3(kAdBlock), 0, s, t.E, t.len, a.pos_of_link, a.flags,
                       a.chunk + n_alpha);
    // the chunk sums go through LDS while they fit (32 KB: about a million commodities)
    const size_t lb_lds = sizeof(double) * (static_cast<size_t>(n_alpha) + n_d);
    const bool staged = lb_lds <= 32 * 1024;
    hipLaunchKernelGGL(k_ad_lb, dim3(1), dim3(kAdBlock), staged ? lb_lds : 0, s, n_alpha, a.chunk,
                       n_d, a.chunk + n_alpha, a.flags, a.ascal, staged);
}

void launch_ad_update(const DeviceTopo &t, const AdaptiveState &a, double eps, hipStream_t s)
{
    // 16 or 4 lanes per link in k_ad_u (as in the fixed-step update), one thread per link in
    // k_ad_apply
    const int per_block = kAdBlock / t.update_lanes;
    const int gu = (t.E + per_block - 1) / per_block;
    if (t.update_lanes == 4)
        hipLaunchKernelGGL(k_ad_u<4>, dim3(gu), dim3(kAdBlock), 0, s, t.E, t.pos_slot_ptr,
                           t.pos_xslot, t.partial, t.invcap_pos, a.flags, a.u_pos, a.block_max_u);
    else
        hipLaunchKernelGGL(k_ad_u<16>, dim3(gu), dim3(kAdBlock), 0, s, t.E, t.pos_slot_ptr,
                           t.pos_xslot, t.partial, t.invcap_pos, a.flags, a.u_pos, a.block_max_u);
    launch_ad_apply(t, a, eps, gu, s);
}

void launch_ad_apply(const DeviceTopo &t, const AdaptiveState &a, double eps, int n_u_blocks,
                     hipStream_t s)
{
    const int ga = (t.E + kAdBlock - 1) / kAdBlock;
    if (t.cost_max)
        hipLaunchKernelGGL(k_ad_apply<true>, dim3(ga), dim3(kAdBlock), 0, s, t.E, eps, n_u_blocks,
                           a.block_max_u, a.u_pos, t.invcap_pos, t.pos_link, t.len, t.price, t.S,
                           a.flags, a.ascal, a.sigma_log, a.block_max_s);
    else
        hipLaunchKernelGGL(k_ad_apply<false>, dim3(ga), dim3(kAdBlock), 0, s, t.E, eps, n_u_blocks,
                           a.block_max_u, a.u_pos, t.invcap_pos, t.pos_link, t.len, t.price, t.S,
                           a.flags, a.ascal, a.sigma_log, a.block_max_s);
}

void launch_ad_lambda(const DeviceTopo &t, const AdaptiveState &a, double gap, int check,
                      hipStream_t s)
{
    const int ga = (t.E + kAdBlock - 1) / kAdBlock;
    hipLaunchKernelGGL(k_ad_lambda, dim3(1), dim3(kAdBlock), 0, s, ga, a.block_max_s, gap, check,
                       a.flags, a.ascal, a.host_words);
}

hipError_t launch_ad_histogram(const DeviceTopo &t, const AdaptiveState &a, const uint8_t *log,
                               size_t stride, double *splits, double *lambda, hipStream_t s)
{
    const size_t lds = sizeof(double) * kWave * static_cast<size_t>(t.pmax | 1);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_ad_histogram),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(lds));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_ad_histogram, dim3((t.K + kWave - 1) / kWave), dim3(kWave), lds, s, t.K,
                       t.pmax, stride, log, t.comm_ptr, a.sigma_log, a.flags, a.ascal, splits,
                       lambda);
    return hipGetLastError();
}

}  // namespace nimble

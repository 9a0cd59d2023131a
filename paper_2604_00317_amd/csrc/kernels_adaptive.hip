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

// The two sums of the bound as chunk sums, in one launch.  Chunk c of a sum is its terms
// 256c .. 256c + 255 added in order.  A workgroup owns kAdChunksPerBlock chunks of one sum, a
// thread per term: the first blocks_alpha workgroups those of alpha (term k is d_k times the cost
// of the candidate commodity k has just chosen -- its cheapest; the cost is taken link by link
// in path order, exactly as the scan took it), the others those of D (term i is the length of
// link i).  The terms go to LDS, a padded row per chunk so that the rows start in different
// banks, and one thread per chunk then adds its row in order.
constexpr int kAdChunksPerBlock = 4;
constexpr int kAdSumBlock = kAdChunksPerBlock * kAdChunk;
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

template <bool MAXC>
__global__ __launch_bounds__(kAdSumBlock) void k_ad_bound_sums(
    int K, int E, int blocks_alpha, const int32_t *__restrict__ cp, const int32_t *__restrict__ lp,
    const int32_t *__restrict__ pl, const double *__restrict__ price,
    const uint8_t *__restrict__ choice, const double *__restrict__ demand,
    const double *__restrict__ len, const int32_t *__restrict__ pos_of_link,
    const int32_t *__restrict__ flags, double *__restrict__ chunk_alpha,
    double *__restrict__ chunk_d)
{
    __shared__ double s_terms[kAdChunksPerBlock * kAdRow];
    if (flags[0]) return;
    const int tid = threadIdx.x;
    const bool alpha = static_cast<int>(blockIdx.x) < blocks_alpha;          // block-uniform
    const int blk = alpha ? blockIdx.x : blockIdx.x - blocks_alpha;
    const int n = alpha ? K : E;
    const int i = blk * kAdSumBlock + tid;
    double v = 0.0;
    if (alpha) {
        if (i < K) {
            const int p = cp[i] + choice[i];
            const int q0 = lp[p], q1 = lp[p + 1];
            const double dm = demand[i];
            double c = 0.0;
            // eight links at a time: their ids are requested side by side, then their prices,
            // and only then are the prices added in path order (two trips to memory for a path
            // of up to eight links instead of two per link)
            for (int base = q0; base < q1; base += 8) {
                int id[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) id[j] = pl[base + j < q1 ? base + j : q1 - 1];
                double pe[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) pe[j] = price[id[j]];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (base + j < q1) {
                        if constexpr (MAXC) c = (pe[j] > c) ? pe[j] : c;
                        else c = c + pe[j];
                    }
                }
            }
            v = dm * c;
        }
    } else if (i < E) {
        v = len[pos_of_link[i]];
    }
    s_terms[(tid / kAdChunk) * kAdRow + (tid % kAdChunk)] = v;
    __syncthreads();
    const int c = blk * kAdChunksPerBlock + tid;
    if (tid < kAdChunksPerBlock && c * kAdChunk < n) {
        const int cnt = n - c * kAdChunk < kAdChunk ? n - c * kAdChunk : kAdChunk;
        (alpha ? chunk_alpha : chunk_d)[c] = ordered_sum(s_terms + tid * kAdRow, cnt);
    }
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
__global__ __launch_bounds__(kAdBlock) void k_ad_apply(AdApplyArgs a)
{
    __shared__ double red[16];
    ad_apply_block<MAXC>(a, blockIdx.x, red);
}

// lengths by link id from the lengths by position
__global__ __launch_bounds__(kAdBlock) void k_ad_len_id(int E, const int32_t *__restrict__ pos_link,
                                                        const double *__restrict__ len,
                                                        double *__restrict__ len_id)
{
    const int i = blockIdx.x * kAdBlock + threadIdx.x;
    if (i < E) len_id[pos_link[i]] = len[i];
}

// lambda = max S / W.  At a check, first the bound of this check -- alpha / D, each the sum of
// its chunk sums added in order by one thread (from LDS when `staged`) -- then the best bound
// is updated and the stop test made.  ascal: [0] W, [1] bound of this check, [2] best bound,
// [3] lambda.
__global__ __launch_bounds__(kAdBlock) void k_ad_lambda(int n_s_blocks,
                                                        const double *__restrict__ block_max_s,
                                                        double gap, int check, int n_alpha,
                                                        const double *chunk_alpha, int n_d,
                                                        const double *chunk_d, bool staged,
                                                        int32_t *__restrict__ flags,
                                                        double *__restrict__ ascal,
                                                        int32_t *host_words)
{
    extern __shared__ double s_chunks[];
    __shared__ double red[16];
    __shared__ double s_sum[2];
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
    if (check) {
        if (staged) {
            for (int i = threadIdx.x; i < n_alpha; i += kAdBlock) s_chunks[i] = chunk_alpha[i];
            for (int i = threadIdx.x; i < n_d; i += kAdBlock) s_chunks[n_alpha + i] = chunk_d[i];
            __syncthreads();
            chunk_alpha = s_chunks;
            chunk_d = s_chunks + n_alpha;
        }
        // two threads, one sum each
        if (threadIdx.x == 0) s_sum[0] = ordered_sum(chunk_alpha, n_alpha);
        if (threadIdx.x == kWave) s_sum[1] = ordered_sum(chunk_d, n_d);
    }
    const double smax = block_max(m, red);            // (its barriers also publish s_sum)
    if (threadIdx.x != 0) return;
    const double W = ascal[0];
    const double lam = W > 0.0 ? smax / W : 0.0;
    ascal[3] = lam;
    if (check) {
        const double lb = s_sum[0] / s_sum[1];
        ascal[1] = lb;
        if (lb > ascal[2]) ascal[2] = lb;
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
    // weight j of this lane's commodity is entry j * 64 + lane: whatever the lanes choose, they
    // spread evenly over the banks
    double *mine = s_w + lane;
    for (int j = 0; j < pmax; ++j) mine[j * kWave] = 0.0;
    if (k < K) {
        const uint8_t *col = log + k;
        // the choices of sixteen iterations are requested side by side; the additions stay in
        // iteration order
        int t = 0;
        for (; t + 16 <= iters; t += 16) {
            int c[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) c[j] = col[size_t(t + j) * stride];
#pragma unroll
            for (int j = 0; j < 16; ++j)
                mine[c[j] * kWave] = mine[c[j] * kWave] + sigma_log[t + j];
        }
        for (; t < iters; ++t) {
            const int c = col[size_t(t) * stride];
            mine[c * kWave] = mine[c * kWave] + sigma_log[t];
        }
        const int p0 = cp[k], np = cp[k + 1] - p0;
        for (int j = 0; j < np; ++j)
            splits[p0 + j] = W > 0.0 ? mine[j * kWave] / W : (j == 0 ? 1.0 : 0.0);
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
    const int n_alpha = (t.K + kAdChunk - 1) / kAdChunk;
    const int ba = (t.K + kAdSumBlock - 1) / kAdSumBlock, bd = (t.E + kAdSumBlock - 1) / kAdSumBlock;
    if (t.cost_max)
        hipLaunchKernelGGL(k_ad_bound_sums<true>, dim3(ba + bd), dim3(kAdSumBlock), 0, s, t.K, t.E,
                           ba, t.comm_ptr, t.path_ptr, t.path_links, t.price, choice, demand,
                           t.len, a.pos_of_link, a.flags, a.chunk, a.chunk + n_alpha);
    else
        hipLaunchKernelGGL(k_ad_bound_sums<false>, dim3(ba + bd), dim3(kAdSumBlock), 0, s, t.K, t.E,
                           ba, t.comm_ptr, t.path_ptr, t.path_links, t.price, choice, demand,
                           t.len, a.pos_of_link, a.flags, a.chunk, a.chunk + n_alpha);
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
    launch_ad_apply(t, a, eps, gu, a.len_id[0], s);   // (no record kernel reads these here)
}

AdApplyArgs ad_apply_args(const DeviceTopo &t, const AdaptiveState &a, double eps, int n_u_blocks,
                          double *len_id_new)
{
    AdApplyArgs p;
    p.E = t.E;
    p.eps = eps;
    p.n_u_blocks = n_u_blocks;
    p.block_max_u = a.block_max_u;
    p.u_pos = a.u_pos;
    p.invcap_pos = t.invcap_pos;
    p.pos_link = t.pos_link;
    p.len = t.len;
    p.price = t.price;
    p.S = t.S;
    p.flags = a.flags;
    p.ascal = a.ascal;
    p.sigma_log = a.sigma_log;
    p.block_max_s = a.block_max_s;
    p.len_id_new = len_id_new;
    return p;
}

void launch_ad_apply(const DeviceTopo &t, const AdaptiveState &a, double eps, int n_u_blocks,
                     double *len_id_new, hipStream_t s)
{
    const int ga = (t.E + kAdBlock - 1) / kAdBlock;
    const AdApplyArgs p = ad_apply_args(t, a, eps, n_u_blocks, len_id_new);
    if (t.cost_max) hipLaunchKernelGGL(k_ad_apply<true>, dim3(ga), dim3(kAdBlock), 0, s, p);
    else hipLaunchKernelGGL(k_ad_apply<false>, dim3(ga), dim3(kAdBlock), 0, s, p);
}

void launch_ad_len_id(const DeviceTopo &t, double *len_id, hipStream_t s)
{
    hipLaunchKernelGGL(k_ad_len_id, dim3((t.E + kAdBlock - 1) / kAdBlock), dim3(kAdBlock), 0, s,
                       t.E, t.pos_link, t.len, len_id);
}

void launch_ad_lambda(const DeviceTopo &t, const AdaptiveState &a, double gap, int check,
                      hipStream_t s)
{
    const int ga = (t.E + kAdBlock - 1) / kAdBlock;
    const int n_alpha = (t.K + kAdChunk - 1) / kAdChunk, n_d = (t.E + kAdChunk - 1) / kAdChunk;
    // the chunk sums of a check go through LDS while they fit (32 KB: about a million
    // commodities)
    const size_t lb_lds = sizeof(double) * (static_cast<size_t>(n_alpha) + n_d);
    const bool staged = check != 0 && lb_lds <= 32 * 1024;
    hipLaunchKernelGGL(k_ad_lambda, dim3(1), dim3(kAdBlock), staged ? lb_lds : 0, s, ga,
                       a.block_max_s, gap, check, n_alpha, a.chunk, n_d, a.chunk + n_alpha, staged,
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

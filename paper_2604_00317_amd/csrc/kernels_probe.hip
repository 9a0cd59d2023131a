// Probe of grid-wide barriers: what one costs on this part, and whether data written before it
// is seen after it, for the barrier designs a persistent planner kernel could use.  Nothing of
// the plan runs here; the benchmark reports the figures next to the kernel boundaries they
// would replace.
//
// The kernel is launched cooperatively (the runtime refuses a grid that is not co-resident) and
// every wait is bounded: when a wait expires the workgroup raises the abort word, every other
// workgroup sees it at its next poll, and all leave the kernel normally.
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace nimble {

namespace {

constexpr int kMaxXcd = 16;
constexpr int kLine = 32;      // uint32 words per 128-byte line: one counter per line

constexpr int kMaxFlagBlocks = 2048;

struct ProbeWords {
    unsigned int flags[kMaxFlagBlocks];         // kind 4: the round every workgroup has reached
    unsigned int xcd_arrive[kMaxXcd * kLine];   // arrivals of the workgroups of XCD x at [32 x]
    unsigned int xcd_gen[kMaxXcd * kLine];      // generation released to XCD x at [32 x]
    unsigned int global_arrive[kLine];
    unsigned int gen[kLine];
    unsigned int abort[kLine];
};

__global__ void k_probe_clear(unsigned int *w, int n_words, unsigned int *data, int n_data,
                              int *out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_words) w[i] = 0u;
    if (i < n_data) data[i] = 0u;
    if (i < 32) out[i] = 0;
}

__device__ __forceinline__ unsigned int ld_agent(const unsigned int *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ int xcc_id()
{
    // hardware register 20 (XCC_ID), bits 3:0
    return static_cast<int>(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11))) & (kMaxXcd - 1);
}

// Bounded wait until *p (read at agent scope, or at workgroup scope when `local`) reaches
// `target`; false when the solve must be abandoned.
template <bool LOCAL>
__device__ __forceinline__ bool wait_for(const unsigned int *p, unsigned int target,
                                         ProbeWords *w, unsigned int spin_limit)
{
    unsigned int polls = 0;
    for (;;) {
        const unsigned int v = LOCAL ? __hip_atomic_load(p, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_WORKGROUP)
                                     : ld_agent(p);
        if (static_cast<int>(v - target) >= 0) return true;
        if (ld_agent(w->abort) != 0u) return false;
        if (++polls > spin_limit) {
            __hip_atomic_store(w->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}

// One grid-wide barrier, executed by thread 0 of every workgroup between two workgroup
// barriers.  `round` counts the barriers made so far (the same in all workgroups).
//   kind 0  one arrival counter, relaxed agent-scope atomics, no cache maintenance: data that
//           crosses the barrier must itself be written and read at agent scope
//   kind 1  the same counter between two agent-scope fences (release before, acquire after):
//           ordinary stores and loads may cross the barrier
//   kind 2  two levels: the workgroups of an XCD arrive on their XCD's counter, the last of them
//           on the global one, the last of those publishes the generation; all poll that word
//   kind 5  as 2, followed by an acquire fence at agent scope: data stored at agent scope before
//           the barrier may be read with ordinary (cached) loads after it
//   kind 3  two levels with a local release: only the XCD's last arriver polls the global
//           generation, the others poll a word of their own XCD at workgroup scope (it is
//           written and read through that XCD's L2)
// kind 4: no read-modify-write at all.  Every workgroup stores the round it has reached into
// its own word of a flag array and its first wave then reads the whole array (16 bytes per lane
// and load) until every word has reached that round.  All 64 lanes of the wave call this.
__device__ __forceinline__ bool flag_barrier(ProbeWords *w, unsigned int round,
                                             unsigned int n_blocks, unsigned int spin_limit)
{
    const int lane = threadIdx.x & 63;
    const unsigned int target = round + 1u;
    if (lane == 0)
        __hip_atomic_store(&w->flags[blockIdx.x], target, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    unsigned int polls = 0;
    for (;;) {
        bool all = true;
        for (unsigned int base = 0; base < n_blocks; base += 256u) {       // wave-uniform
            const unsigned int i = base + 4u * lane;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // words beyond the grid are not waited for
                const unsigned int v = (i + q < n_blocks) ? ld_agent(&w->flags[i + q]) : target;
                all = all && static_cast<int>(v - target) >= 0;
            }
        }
        if (__ballot(!all) == 0ull) return true;
        if (ld_agent(w->abort) != 0u) return false;
        if (++polls > spin_limit) {
            if (lane == 0)
                __hip_atomic_store(w->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}

template <int KIND>
__device__ __forceinline__ bool probe_barrier(ProbeWords *w, unsigned int round,
                                              unsigned int n_blocks, unsigned int n_xcd_blocks,
                                              unsigned int n_xcd, int xcd,
                                              unsigned int spin_limit)
{
    if constexpr (KIND == 0 || KIND == 1 || KIND == 4) {
        if constexpr (KIND == 1) __threadfence();
        __hip_atomic_fetch_add(w->global_arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool ok = wait_for<false>(w->global_arrive, (round + 1u) * n_blocks, w, spin_limit);
        if constexpr (KIND == 1) __threadfence();
        return ok;
    } else {
        const unsigned int old = __hip_atomic_fetch_add(&w->xcd_arrive[kLine * xcd], 1u,
                                                        __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last_of_xcd = old + 1u == (round + 1u) * n_xcd_blocks;
        if (last_of_xcd) {
            const unsigned int g = __hip_atomic_fetch_add(w->global_arrive, 1u, __ATOMIC_RELAXED,
                                                          __HIP_MEMORY_SCOPE_AGENT);
            if (g + 1u == (round + 1u) * n_xcd)
                __hip_atomic_store(w->gen, round + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if constexpr (KIND == 2) {
            return wait_for<false>(w->gen, round + 1u, w, spin_limit);
        } else if constexpr (KIND == 5) {
            // as 2, then an acquire fence at agent scope (it invalidates what the caches of this
            // XCD hold of other XCDs' data; nothing is written back): data stored at agent scope
            // before the barrier may be read with ordinary loads after it
            const bool ok = wait_for<false>(w->gen, round + 1u, w, spin_limit);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            return ok;
        } else {
            if (last_of_xcd) {
                const bool ok = wait_for<false>(w->gen, round + 1u, w, spin_limit);
                __hip_atomic_store(&w->xcd_gen[kLine * xcd], round + 1u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
                return ok;
            }
            return wait_for<true>(&w->xcd_gen[kLine * xcd], round + 1u, w, spin_limit);
        }
    }
}

struct ProbeArgs {
    ProbeWords *w;
    unsigned int *data;       // one word per workgroup, a line apart
    int *out;                 // [0] values that arrived late or wrong, [1] abandoned,
                              // [2..17] workgroups per XCC id, [18] rounds completed
    int rounds;
    unsigned int spin_limit;
    int n_xcd;                // XCDs the launch assumes (kinds 2, 3)
};

// Every round: each workgroup publishes the round number in its own word, barrier, reads the
// word of a workgroup far away (which must hold this round's number), barrier.
template <int KIND>
__global__ void k_barrier_probe(ProbeArgs a)
{
    __shared__ int s_ok;
    __shared__ int s_xcd;
    const unsigned int nb = gridDim.x;
    if (threadIdx.x == 0) {
        s_xcd = xcc_id();
        atomicAdd(&a.out[2 + s_xcd], 1);
    }
    __syncthreads();
    const int xcd = s_xcd;
    // workgroups are dealt to the XCDs in turn, so every XCD holds the same number when the grid
    // is a multiple of their number (the launcher makes it so); the probe itself checks it
    const unsigned int n_xcd_blocks = nb / static_cast<unsigned int>(a.n_xcd);
    const unsigned int peer = (blockIdx.x + nb / 2u + 3u) % nb;
    int bad = 0;
    unsigned int round = 0;
    int r = 0;
    for (; r < a.rounds; ++r) {
        if (threadIdx.x == 0) {
            if constexpr (KIND == 1) a.data[kLine * blockIdx.x] = static_cast<unsigned int>(r + 1);
            else __hip_atomic_store(&a.data[kLine * blockIdx.x], static_cast<unsigned int>(r + 1),
                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();       // (its release at workgroup scope waits for the store)
        if constexpr (KIND == 4) {
            if (threadIdx.x < 64) {
                const bool ok = flag_barrier(a.w, round, nb, a.spin_limit);
                if (threadIdx.x == 0) s_ok = ok;
            }
        } else if (threadIdx.x == 0) {
            s_ok = probe_barrier<KIND>(a.w, round, nb, n_xcd_blocks, a.n_xcd, xcd, a.spin_limit);
        }
        __syncthreads();
        if (!s_ok) break;
        round += 1u;
        if (threadIdx.x == 0) {
            unsigned int v;
            if constexpr (KIND == 1 || KIND == 5) v = a.data[kLine * peer];
            else v = ld_agent(&a.data[kLine * peer]);
            if (v != static_cast<unsigned int>(r + 1)) bad += 1;
        }
        __syncthreads();
        if constexpr (KIND == 4) {
            if (threadIdx.x < 64) {
                const bool ok = flag_barrier(a.w, round, nb, a.spin_limit);
                if (threadIdx.x == 0) s_ok = ok;
            }
        } else if (threadIdx.x == 0) {
            s_ok = probe_barrier<KIND>(a.w, round, nb, n_xcd_blocks, a.n_xcd, xcd, a.spin_limit);
        }
        __syncthreads();
        if (!s_ok) break;
        round += 1u;
    }
    if (threadIdx.x == 0) {
        if (bad) atomicAdd(&a.out[0], bad);
        if (r < a.rounds) a.out[1] = 1;
        if (blockIdx.x == 0) a.out[18] = r;
    }
}

}  // namespace

size_t barrier_probe_bytes(int max_blocks)
{
    return sizeof(ProbeWords) + sizeof(unsigned int) * kLine * static_cast<size_t>(max_blocks);
}

hipError_t launch_barrier_probe(int kind, int blocks, int threads, int rounds,
                                unsigned int spin_limit, int n_xcd, void *work, int *out,
                                hipStream_t s)
{
    ProbeArgs a;
    a.w = static_cast<ProbeWords *>(work);
    a.data = reinterpret_cast<unsigned int *>(static_cast<unsigned char *>(work) +
                                              sizeof(ProbeWords));
    a.out = out;
    a.rounds = rounds;
    a.spin_limit = spin_limit;
    a.n_xcd = n_xcd;
    const int n_words = static_cast<int>(sizeof(ProbeWords) / 4);
    const int n_data = kLine * blocks;
    const int n_clear = n_words > n_data ? n_words : n_data;
    hipLaunchKernelGGL(k_probe_clear, dim3((n_clear + 255) / 256), dim3(256), 0, s,
                       reinterpret_cast<unsigned int *>(a.w), n_words, a.data, n_data, out);
    void *args[] = {&a};
    const void *fn = nullptr;
    switch (kind) {
    case 0: fn = reinterpret_cast<const void *>(&k_barrier_probe<0>); break;
    case 1: fn = reinterpret_cast<const void *>(&k_barrier_probe<1>); break;
    case 2: fn = reinterpret_cast<const void *>(&k_barrier_probe<2>); break;
    case 3: fn = reinterpret_cast<const void *>(&k_barrier_probe<3>); break;
    case 5: fn = reinterpret_cast<const void *>(&k_barrier_probe<5>); break;
    case 4:
        if (blocks > kMaxFlagBlocks) return hipErrorInvalidValue;
        fn = reinterpret_cast<const void *>(&k_barrier_probe<4>);
        break;
    default: return hipErrorInvalidValue;
    }
    // cooperative launch: the runtime checks that the whole grid is resident at once
    return hipLaunchCooperativeKernel(fn, dim3(blocks), dim3(threads), args, 0, s);
}

}  // namespace nimble

// Persistent regime: the whole solve in ONE kernel.  The grid is sized to be co-resident
// (blocks per CU from the occupancy query times the CU count) and the three phases of every
// iteration are separated by grid-wide barriers instead of kernel boundaries.
//
// Barrier: one monotonically increasing arrival counter in device memory.  Thread 0 of every
// block publishes the block's writes (agent-scope release fence), adds 1, and waits until the
// counter reaches the next multiple of the grid size, then an acquire fence makes the other
// blocks' writes visible.  The wait is bounded: after `spin_limit` polls a block raises the
// abort word, every block sees it at its next poll and leaves the kernel, and the epilogue is
// skipped (lambda is set to NaN by the block that gave up), so no wave can wait forever.
#include "host_topo.hpp"
#include "kernels.hpp"
#include "phases.hpp"
#include "wave_ops.hpp"

namespace nimble {

namespace {

constexpr int kPBlock = 1024;

struct SyncWords {
    unsigned int arrivals;   // barrier counter
    unsigned int abort;      // set when a bounded wait expired
    unsigned long long rho_bits;    // max_e reach_e/cap_e as an ordered bit pattern (values >= 0)
    unsigned long long smax_bits;   // max_e S_e likewise
};

__global__ void k_sync_reset(SyncWords *w)
{
    if (threadIdx.x == 0) {
        w->arrivals = 0u;
        w->abort = 0u;
        w->rho_bits = 0ull;
        w->smax_bits = 0ull;
    }
}

// Returns false when the solve must be abandoned (bounded wait expired somewhere).
__device__ __forceinline__ bool grid_barrier(SyncWords *w, unsigned int n_blocks,
                                             unsigned int spin_limit, int *s_flag)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        const unsigned int old = __hip_atomic_fetch_add(&w->arrivals, 1u, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
        const unsigned int target = (old / n_blocks + 1u) * n_blocks;
        int ok = 1;
        unsigned int polls = 0;
        while (__hip_atomic_load(&w->arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <
               target) {
            if (__hip_atomic_load(&w->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                ok = 0;
                break;
            }
            if (++polls > spin_limit) {
                __hip_atomic_store(&w->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        __threadfence();
        *s_flag = ok;
    }
    __syncthreads();
    return *s_flag != 0;
}

struct PersistentArgs {
    int E, K, P, n_passes, n_schunks, n_tile_items;
    uint32_t pad_comm;
    const int32_t *tile_desc;
    const uint32_t *tile_mask;
    const uint8_t *tile_pres;
    double *demand1n, *demand1t, *demand2t;
    int n_strip_items;
    const uint32_t *strip_base, *strip_mask;
    const uint64_t *strip_pres;
    const int32_t *strip_slot;
    const int32_t *cp, *lp, *pl;
    const int32_t *pass_first_slot;
    const uint32_t *oct_base, *oct_mask;
    const int32_t *schunk_begin, *schunk_end, *schunk_slot;
    const uint32_t *single_pair;
    const int32_t *pos_link, *pos_slot_ptr;
    const int2 *pos_xslot;
    const int32_t *sigma;
    uint8_t *choice2;
    double *demand2;
    const double *invcap, *invcap_pos;
    double *len, *price, *S;
    uint8_t *choice;
    uint32_t *count;
    double *partial;
    SyncWords *sync;
    const double *demand;
    double eps;
    int iters;
    double *splits, *lambda;
    unsigned int spin_limit;
};

template <int MODE>
__device__ __forceinline__ void reduce_both(const PersistentArgs &a, int wave, int n_waves,
                                            int lane)
{
    reduce_tile_phase<MODE>(a.n_tile_items, a.tile_desc, a.tile_mask, a.tile_pres, a.choice,
                                a.demand1t,
                            a.choice2, a.demand2t, a.partial, wave, n_waves, lane);
    reduce_strip_phase<MODE>(a.n_strip_items, a.strip_base, a.strip_pres, a.strip_mask,
                             a.strip_slot, a.choice, a.demand1n, a.choice2, a.demand2, a.partial,
                             wave, n_waves, lane);
    reduce_flat_phase<MODE>(0, a.n_passes, a.pass_first_slot, a.oct_base, a.oct_mask, a.choice,
                            a.demand1n, a.choice2, a.demand2, a.partial, 0, wave, n_waves, lane);
    reduce_phase<MODE, kSinglesPerLane>(a.n_schunks, a.schunk_begin, a.schunk_end, a.schunk_slot,
                                        a.single_pair, a.pad_comm, a.choice, a.demand, a.partial,
                                        n_waves - 1 - wave, n_waves, lane);
}

__device__ __forceinline__ void atomic_max_bits(unsigned long long *addr, double v)
{
    // v >= 0: the IEEE bit pattern is monotone in the value, so an integer max is exact
    __hip_atomic_fetch_max(addr, static_cast<unsigned long long>(__double_as_longlong(v)),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int L, int LMAX, bool MAXC>
__global__ __launch_bounds__(kPBlock) void k_persistent(PersistentArgs a)
{
    __shared__ double red[16];
    __shared__ int s_flag;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    const int n_threads = gridDim.x * blockDim.x;
    const unsigned int nb = gridDim.x;

    // prologue: state and the width rho
    for (int e = tid; e < a.E; e += n_threads) {
        a.len[e] = 1.0;
        a.price[e] = MAXC ? 1.0 : a.invcap[e];
        a.S[e] = 0.0;
    }
    for (int p = tid; p < a.P; p += n_threads) a.count[p] = 0u;
    for (int k = tid; k < a.K; k += n_threads) {
        const double dk = a.demand[k];
        a.demand1n[k] = dk;
        a.demand1t[tile_demand_index(k)] = dk;
        const int sg = a.sigma[k];
        if (sg >= 0) {
            a.demand2[sg] = dk;
            a.demand2t[tile_demand_index(sg)] = dk;
        }
    }
    if (!grid_barrier(a.sync, nb, a.spin_limit, &s_flag)) goto abandoned;
    reduce_both<1>(a, wave, n_waves, lane);
    if (!grid_barrier(a.sync, nb, a.spin_limit, &s_flag)) goto abandoned;
    {
        double m = width_phase(a.E, a.pos_slot_ptr, a.pos_xslot, a.partial, a.invcap_pos, wave,
                               n_waves, lane);
        m = block_max(m, red);
        if (threadIdx.x == 0) atomic_max_bits(&a.sync->rho_bits, m);
    }
    if (!grid_barrier(a.sync, nb, a.spin_limit, &s_flag)) goto abandoned;
    {
        const double rho = __longlong_as_double(static_cast<long long>(__hip_atomic_load(
            &a.sync->rho_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
        const double invrho = (rho > 0.0) ? 1.0 / rho : 0.0;

        for (int it = 0; it < a.iters; ++it) {
            argmin_phase<L, LMAX, MAXC>(a.K, a.cp, a.lp, a.pl, a.price, a.choice, a.count, a.sigma,
                                        a.choice2, wave, n_waves, lane);
            if (!grid_barrier(a.sync, nb, a.spin_limit, &s_flag)) goto abandoned;
            reduce_both<0>(a, wave, n_waves, lane);
            if (!grid_barrier(a.sync, nb, a.spin_limit, &s_flag)) goto abandoned;
            update_phase<MAXC>(a.E, a.eps, invrho, a.pos_link, a.pos_slot_ptr, a.pos_xslot, a.partial,
                               a.invcap_pos, a.len, a.price, a.S, wave, n_waves, lane);
            if (!grid_barrier(a.sync, nb, a.spin_limit, &s_flag)) goto abandoned;
        }
    }
    // epilogue: split fractions and lambda = max_e S_e / iters
    {
        const double T = static_cast<double>(a.iters);
        for (int p = tid; p < a.P; p += n_threads)
            a.splits[p] = static_cast<double>(a.count[p]) / T;
        double m = 0.0;
        for (int e = tid; e < a.E; e += n_threads) m = fmax(m, a.S[e]);
        m = block_max(m, red);
        if (threadIdx.x == 0) atomic_max_bits(&a.sync->smax_bits, m);
        if (!grid_barrier(a.sync, nb, a.spin_limit, &s_flag)) goto abandoned;
        if (tid == 0) {
            const double smax = __longlong_as_double(static_cast<long long>(__hip_atomic_load(
                &a.sync->smax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
            a.lambda[0] = smax / T;
        }
    }
    return;
abandoned:
    if (tid == 0) a.lambda[0] = __builtin_nan("");
}

template <int L, int LMAX, bool MAXC>
hipError_t launch_one(const PersistentArgs &a, int n_cu, hipStream_t s, int *grid_out)
{
    int per_cu = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(
        &per_cu, reinterpret_cast<const void *>(&k_persistent<L, LMAX, MAXC>), kPBlock, 0);
    if (e != hipSuccess) return e;
    if (per_cu < 1) return hipErrorLaunchOutOfResources;
    // One 1024-thread workgroup per CU, launched cooperatively: the runtime then checks that the
    // whole grid is resident at once (with this kernel's real register and LDS needs) and
    // refuses the launch otherwise, instead of leaving the grid barrier to find out.  A plain
    // launch gives no such promise: with two workgroups per CU, as the occupancy query allows,
    // the barrier's bounded wait has expired on this part.
    const int grid = n_cu;
    if (grid_out) *grid_out = grid;
    PersistentArgs copy = a;
    void *params[] = {&copy};
    return hipLaunchCooperativeKernel(reinterpret_cast<const void *>(&k_persistent<L, LMAX, MAXC>),
                                      dim3(grid), dim3(kPBlock), params, 0, s);
}

template <int L, bool MAXC>
hipError_t launch_lmax(const PersistentArgs &a, int lmax, int n_cu, hipStream_t s, int *grid_out)
{
    if (lmax <= 2) return launch_one<L, 2, MAXC>(a, n_cu, s, grid_out);
    if (lmax <= 4) return launch_one<L, 4, MAXC>(a, n_cu, s, grid_out);
    return launch_one<L, 8, MAXC>(a, n_cu, s, grid_out);
}

template <bool MAXC>
hipError_t launch_l(const PersistentArgs &a, int L, int lmax, int n_cu, hipStream_t s,
                    int *grid_out)
{
    switch (L) {
    case 1: return launch_lmax<1, MAXC>(a, lmax, n_cu, s, grid_out);
    case 2: return launch_lmax<2, MAXC>(a, lmax, n_cu, s, grid_out);
    case 4: return launch_lmax<4, MAXC>(a, lmax, n_cu, s, grid_out);
    case 8: return launch_lmax<8, MAXC>(a, lmax, n_cu, s, grid_out);
    case 16: return launch_lmax<16, MAXC>(a, lmax, n_cu, s, grid_out);
    case 32: return launch_lmax<32, MAXC>(a, lmax, n_cu, s, grid_out);
    default: return launch_lmax<64, MAXC>(a, lmax, n_cu, s, grid_out);
    }
}

}  // namespace

size_t persistent_sync_bytes() { return sizeof(SyncWords); }

hipError_t launch_persistent(const DeviceTopo &t, void *sync_words, int n_cu,
                             unsigned int spin_limit, const double *demand, double eps,
                             int32_t iters, double *splits, double *lambda, hipStream_t s)
{
    PersistentArgs a;
    a.E = t.E;
    a.K = t.K;
    a.P = t.P;
    a.n_passes = t.n_passes;
    a.n_schunks = t.n_schunks;
    a.n_tile_items = t.n_tile_items;
    a.tile_desc = t.tile_desc;
    a.tile_mask = t.tile_mask;
    a.tile_pres = t.tile_pres;
    a.demand1n = t.demand1n;
    a.demand1t = t.demand1t;
    a.demand2t = t.demand2t;
    a.n_strip_items = t.n_strip_items;
    a.strip_base = t.strip_base;
    a.strip_pres = t.strip_pres;
    a.strip_mask = t.strip_mask;
    a.strip_slot = t.strip_slot;
    a.pad_comm = static_cast<uint32_t>(t.K);
    a.cp = t.comm_ptr;
    a.lp = t.path_ptr;
    a.pl = t.path_links;
    a.pass_first_slot = t.pass_first_slot;
    a.oct_base = t.oct_base;
    a.oct_mask = t.oct_mask;
    a.schunk_begin = t.schunk_begin;
    a.schunk_end = t.schunk_end;
    a.schunk_slot = t.schunk_slot;
    a.single_pair = t.single_pair;
    a.pos_link = t.pos_link;
    a.pos_slot_ptr = t.pos_slot_ptr;
    a.pos_xslot = t.pos_xslot;
    a.sigma = t.sigma;
    a.choice2 = t.choice2;
    a.demand2 = t.demand2;
    a.invcap = t.invcap;
    a.invcap_pos = t.invcap_pos;
    a.len = t.len;
    a.price = t.price;
    a.S = t.S;
    a.choice = t.choice;
    a.count = t.count;
    a.partial = t.partial;
    a.sync = static_cast<SyncWords *>(sync_words);
    a.demand = demand;
    a.eps = eps;
    a.iters = iters;
    a.splits = splits;
    a.lambda = lambda;
    a.spin_limit = spin_limit;
    hipLaunchKernelGGL(k_sync_reset, dim3(1), dim3(64), 0, s, a.sync);
    const int L = lanes_per_commodity(t.pmax);
    if (t.cost_max) return launch_l<true>(a, L, t.lmax, n_cu, s, nullptr);
    return launch_l<false>(a, L, t.lmax, n_cu, s, nullptr);
}

}  // namespace nimble

// C ABI of the planner library: argument checking, device memory ownership, regime choice and
// kernel sequencing.  Every step of the plan runs in the HIP kernels; there is no CPU
// fallback -- without a usable GPU the device calls fail and the status says so.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <climits>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/nimble_plan.h"
#include "../../include/nimble_plan_debug.h"
#include "host_topo.hpp"
#include "kernels.hpp"

#ifndef NIMBLE_STATIC_SCRATCH_BYTES
#define NIMBLE_STATIC_SCRATCH_BYTES (32u << 20)
#endif


// Scratch of nimble_plan_solve_static: the per-iteration choice log of one streaming-regime
// solve.  Every GPU the library runs on holds its own copy of this array until the process
// ends.  Host code never uses the array's name as an address: the address on a device comes
// from hipGetSymbolAddress (static_scratch_of) and is what kernels are given.
constexpr size_t kStaticScratchBytes = static_cast<size_t>(NIMBLE_STATIC_SCRATCH_BYTES);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local std::string g_last_error;

nimble_status_t fail(nimble_status_t st, const std::string &msg)
{
    g_last_error = msg;
    return st;
}

nimble_status_t fail_hip(hipError_t e, const char *what)
{
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
    return NIMBLE_ERR_HIP;
}

// Every device allocation of the library goes through these two, so that a test can make the
// n-th one fail (nimble_debug_fail_allocation) and can count what is still allocated.
std::atomic<int32_t> g_fail_alloc_in{-1};     // allocations until one fails; -1: none does
std::atomic<int64_t> g_live_allocs{0};
std::atomic<int32_t> g_fail_host_alloc{0};    // the next topology build throws std::bad_alloc

hipError_t dev_malloc(void **p, size_t bytes)
{
    int32_t left = g_fail_alloc_in.load();
    while (left >= 0 && !g_fail_alloc_in.compare_exchange_weak(left, left - 1)) {
    }
    if (left == 0) {
        *p = nullptr;
        return hipErrorOutOfMemory;
    }
    const hipError_t e = hipMalloc(p, bytes);
    if (e == hipSuccess) g_live_allocs.fetch_add(1);
    return e;
}

void dev_free(void *p)
{
    if (!p) return;
    (void)hipFree(p);
    g_live_allocs.fetch_sub(1);
}

// Device address of `scratch` on every device, resolved once per device with that device
// current (every GPU holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

hipError_t static_scratch_of(int device, unsigned char **out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return e;
        if (cur != device) return hipErrorInvalidDevice;
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = static_cast<unsigned char *>(g_scratch_ptr[device]);
    return hipSuccess;
}

}  // namespace

struct nimble_topo {
    nimble::DeviceTopo d{};
    std::vector<void *> allocs;
    int device = -1;
    int32_t forced_regime = NIMBLE_REGIME_AUTO;
    int32_t last_regime = NIMBLE_REGIME_AUTO;
    int64_t bytes_per_iter = 0, bytes_argmin = 0, bytes_reduce = 0, bytes_update = 0;
    int64_t bytes_lds_argmin = 0;   // LDS bytes the lane-major record kernels read per launch
    bool state_ready = false;   // a stream-regime solve has initialised the workspace
    uint8_t *state_log = nullptr;   // the log that solve wrote its choices to (null: counters)
    // per-iteration choice log of the streaming regime (rows of log_stride bytes); grows on
    // demand, so the first solve with more iterations than any before allocates
    uint8_t *choice_log = nullptr;
    int64_t log_rows = 0;
    size_t log_stride = 0;
    bool no_choice_log = false;  // tuning switch read at create: keep per-path counters instead
    int ad_fold = -1;            // tuning switch read at create: 0 the adaptive solve applies
                                 // every step in a launch of its own, 1 inside the next record
                                 // kernel whenever that kernel can, -1 where that is faster
    // workspace of the adaptive-step variant; the sigma log grows with max_iters
    nimble::AdaptiveState ad{};
    bool ad_ready = false;
    int64_t ad_sigma_rows = 0;
    void *sync_words = nullptr; // barrier counter and reductions of the persistent kernel
    // per-plan state: state_plans blocks of d.state_stride bytes in one allocation; the state
    // pointers of `d` are those of block 0
    unsigned char *state = nullptr;
    int32_t state_plans = 0;
    int n_cu = 0;
    unsigned int spin_limit = 1u << 22;   // barrier polls before a solve is abandoned
};

namespace {

template <typename T>
hipError_t upload(nimble_topo *t, const T *host, size_t n, const T **dev)
{
    void *p = nullptr;
    hipError_t e = dev_malloc(&p, (n ? n : 1) * sizeof(T));
    if (e != hipSuccess) return e;
    t->allocs.push_back(p);
    if (n) {
        e = hipMemcpy(p, host, n * sizeof(T), hipMemcpyHostToDevice);
        if (e != hipSuccess) return e;
    }
    *dev = static_cast<const T *>(p);
    return hipSuccess;
}

template <typename T>
hipError_t allocate(nimble_topo *t, size_t n, T **dev)
{
    void *p = nullptr;
    hipError_t e = dev_malloc(&p, (n ? n : 1) * sizeof(T));
    if (e != hipSuccess) return e;
    t->allocs.push_back(p);
    *dev = static_cast<T *>(p);
    return hipSuccess;
}

void release(nimble_topo *t)
{
    for (void *p : t->allocs) dev_free(p);
    t->allocs.clear();
    if (t->choice_log) dev_free(t->choice_log);
    t->choice_log = nullptr;
    t->log_rows = 0;
    if (t->state) dev_free(t->state);
    t->state = nullptr;
    t->state_plans = 0;
    if (t->ad.host_words_host) (void)hipHostFree(t->ad.host_words_host);
    t->ad.host_words_host = nullptr;
    t->ad.host_words = nullptr;
    if (t->ad.sigma_log) dev_free(t->ad.sigma_log);
    t->ad.sigma_log = nullptr;
    t->ad_sigma_rows = 0;
}

// Bytes of one row of a choice log: whole windows of choices (the tile phase reads them 512 at
// a time), with room for the 8 spare entries an octet may touch.
size_t choice_log_stride(const nimble_topo *t)
{
    return (static_cast<size_t>(t->d.K) + 8 + 511) & ~static_cast<size_t>(511);
}

constexpr size_t kChoiceLogCap = static_cast<size_t>(1) << 30;       // most a topology reserves
constexpr size_t kStateCap = static_cast<size_t>(4) << 30;           // and for its plan states
constexpr size_t kChoiceLogAtCreate = static_cast<size_t>(64) << 20; // reserved without being asked
constexpr int32_t kDefaultLogRows = 1024;

// Makes the choice log hold `iters` rows; may free and allocate (both synchronise the device).
// Only nimble_topo_create, nimble_topo_reserve and the adaptive solve call this -- never
// nimble_plan_solve, which uses the log it finds or keeps per-path counters.
nimble_status_t grow_choice_log(nimble_topo *t, int32_t iters)
{
    if (t->log_rows >= iters) return NIMBLE_OK;
    const size_t stride = choice_log_stride(t);
    const size_t bytes = stride * static_cast<size_t>(iters);
    if (bytes > kChoiceLogCap)
        return fail(NIMBLE_ERR_RANGE, "the choice log of that many iterations exceeds 1 GiB");
    if (t->choice_log) dev_free(t->choice_log);      // waits for work that still uses it
    t->choice_log = nullptr;
    t->log_rows = 0;
    void *p = nullptr;
    if (dev_malloc(&p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(NIMBLE_ERR_ALLOC, "the choice log cannot be allocated");
    }
    t->choice_log = static_cast<uint8_t *>(p);
    t->log_rows = iters;
    t->log_stride = stride;
    return NIMBLE_OK;
}

// Per-plan state of the streaming and persistent regimes: every array a solve writes, laid out
// in one block (each array 256-byte aligned), so that a batch is `plans` such blocks at a fixed
// distance.  Entries that only pad an array must read as zero (demand copies, sigma-ordered
// choices), so a new allocation is cleared once.
struct StateLayout {
    size_t demand1n, demand1t, demand2t, choice2, demand2, len, price, S, choice, count, partial,
        scalars, bytes;
};

StateLayout state_layout(const nimble::DeviceTopo &d)
{
    StateLayout L{};
    size_t at = 0;
    auto take = [&](size_t bytes) {
        const size_t here = at;
        at = (at + bytes + 255) & ~static_cast<size_t>(255);
        return here;
    };
    const size_t k_pad = (static_cast<size_t>(d.K) + 511) & ~static_cast<size_t>(511);
    const size_t sg = static_cast<size_t>(d.sigma_size);
    // 8 spare entries: an octet may start at the last multiple of 4 below K
    L.demand1n = take(sizeof(double) * (k_pad + 8));
    L.demand1t = take(sizeof(double) * k_pad);
    L.demand2t = take(sizeof(double) * sg);
    L.choice2 = take(sg);
    L.demand2 = take(sizeof(double) * sg);
    L.len = take(sizeof(double) * static_cast<size_t>(d.E));
    L.price = take(sizeof(double) * static_cast<size_t>(d.E));
    L.S = take(sizeof(double) * static_cast<size_t>(d.E));
    L.choice = take(k_pad + 8);
    L.count = take(sizeof(uint32_t) * static_cast<size_t>(d.P));
    L.partial = take(sizeof(double) * static_cast<size_t>(d.n_slots));
    // [0] = 1/rho, then one maximum of S per update block, or per wave of the link blocks
    L.scalars = take(sizeof(double) *
                     (static_cast<size_t>(std::max({d.n_update_blocks, 4 * d.n_blocks,
                                                    16 * d.n_gblocks})) + 1));
    L.bytes = at;
    return L;
}

// Makes room for the state of `plans` plans; may free and allocate (both synchronise).
hipError_t ensure_state_plans(nimble_topo *t, int32_t plans)
{
    if (plans <= t->state_plans) return hipSuccess;
    nimble::DeviceTopo &d = t->d;
    const StateLayout L = state_layout(d);
    void *p = nullptr;
    hipError_t e = dev_malloc(&p, L.bytes * static_cast<size_t>(plans));
    if (e != hipSuccess) return e;
    e = hipMemset(p, 0, L.bytes * static_cast<size_t>(plans));
    if (e != hipSuccess) {
        dev_free(p);
        return e;
    }
    if (t->state) dev_free(t->state);       // waits for work that still uses it
    unsigned char *b = static_cast<unsigned char *>(p);
    t->state = b;
    t->state_plans = plans;
    d.state_stride = L.bytes;
    d.demand1n = reinterpret_cast<double *>(b + L.demand1n);
    d.demand1t = reinterpret_cast<double *>(b + L.demand1t);
    d.demand2t = reinterpret_cast<double *>(b + L.demand2t);
    d.choice2 = reinterpret_cast<uint8_t *>(b + L.choice2);
    d.demand2 = reinterpret_cast<double *>(b + L.demand2);
    d.len = reinterpret_cast<double *>(b + L.len);
    d.price = reinterpret_cast<double *>(b + L.price);
    d.S = reinterpret_cast<double *>(b + L.S);
    d.choice = reinterpret_cast<uint8_t *>(b + L.choice);
    d.count = reinterpret_cast<uint32_t *>(b + L.count);
    d.partial = reinterpret_cast<double *>(b + L.partial);
    d.scalars = reinterpret_cast<double *>(b + L.scalars);
    t->state_ready = false;
    return hipSuccess;
}

nimble_status_t check_solve_args(const nimble_topo *topo, const double *d_traffic, double eps,
                                 int32_t iters, const double *d_splits, const double *d_lambda)
{
    if (!topo) return fail(NIMBLE_ERR_INVALID, "topology handle is NULL");
    if (!d_traffic || !d_splits || !d_lambda)
        return fail(NIMBLE_ERR_INVALID, "traffic, splits and lambda pointers must not be NULL");
    if (!(eps > 0.0) || !(eps <= 0.5)) return fail(NIMBLE_ERR_INVALID, "eps must be in (0, 0.5]");
    if (iters < 1) return fail(NIMBLE_ERR_INVALID, "iters must be >= 1");
    if (static_cast<double>(iters) * std::log1p(eps) > 700.0)
        return fail(NIMBLE_ERR_RANGE, "iters * log1p(eps) > 700: link lengths could overflow");
    return NIMBLE_OK;
}

nimble_status_t check_device(const nimble_topo *topo)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev != topo->device)
        return fail(NIMBLE_ERR_INVALID, "current device differs from the topology's device");
    return NIMBLE_OK;
}

// The regime of a solve of `batch` plans.  The resident regime runs the plans side by side for
// the price of one -- how long that is depends on the kernel the fabric and the batch allow
// (resident_iteration_us) -- while a streaming-regime iteration costs about two short kernels
// (6.5 us) per plan however wide the rows are.
int32_t pick_regime(const nimble_topo *topo, int32_t batch)
{
    if (topo->forced_regime != NIMBLE_REGIME_AUTO) return topo->forced_regime;
    const nimble::DeviceTopo &d = topo->d;
    if (!nimble::resident_fits(d)) return NIMBLE_REGIME_STREAM;
    if (nimble::resident_in_registers(d)) return NIMBLE_REGIME_RESIDENT;
    const double resident_us = nimble::resident_iteration_us(d, batch);
    const double stream_us = 6.5 * batch;
    return resident_us < stream_us ? NIMBLE_REGIME_RESIDENT : NIMBLE_REGIME_STREAM;
}

// One streaming-regime solve.  Only enqueues kernels: nothing is allocated, freed or
// synchronised here.  `log` (rows of `log_stride` bytes, at least `iters` of them) receives the
// choices of every iteration and the split fractions are counted from it once at the end; with
// log == nullptr every iteration bumps a per-path counter instead.
// `plans` > 1 runs that many plans side by side in every launch (grid.y): their traffic, splits
// and lambda follow each other in the caller's arrays, their state blocks in the topology's
// (ensure_state_plans must have made room), and plan b logs into rows b * iters ... of `log`.
nimble_status_t solve_stream(nimble_topo *topo, const double *d_traffic, double eps,
                             int32_t iters, double *d_splits, double *d_lambda, hipStream_t s,
                             uint8_t *log, size_t log_stride, double *d_len = nullptr,
                             int32_t plans = 1)
{
    nimble::DeviceTopo d = topo->d;
    const bool logged = log != nullptr;
    d.batch = plans;
    d.row_stride = logged ? log_stride * static_cast<size_t>(iters) : d.state_stride;
    nimble::launch_init(d, d_traffic, d_len, s);
    nimble::launch_width(d, d_traffic, s);
    for (int32_t it = 0; it < iters; ++it) {
        uint8_t *row = logged ? log + log_stride * static_cast<size_t>(it) : d.choice;
        nimble::launch_argmin(d, row, logged ? nullptr : d.count, s);
        if (d.n_blocks > 0) {
            nimble::launch_reduce_update(d, row, d_traffic, eps, s);
        } else if (d.n_gblocks > 0) {
            nimble::launch_group_reduce_update(d, row, eps, s);
        } else {
            nimble::launch_load_reduce(d, row, d_traffic, s);
            nimble::launch_update(d, eps, s);
        }
    }
    nimble::launch_epilogue(d, iters, logged ? nullptr : d.count, d_splits, d_lambda, s);
    if (logged) nimble::launch_histogram(d, log, log_stride, iters, d_splits, s);
    if (d_len) nimble::launch_export_len(d, d_len, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "kernel launch (streaming regime)");
    topo->state_ready = true;
    topo->state_log = logged ? log : nullptr;
    return NIMBLE_OK;
}

// The topology's own choice log when it holds `iters` rows, else none (per-path counters).
uint8_t *own_log(const nimble_topo *topo, int32_t iters, int32_t plans = 1)
{
    return (!topo->no_choice_log &&
            topo->log_rows >= static_cast<int64_t>(iters) * plans) ? topo->choice_log : nullptr;
}

nimble_status_t solve_persistent(nimble_topo *topo, const double *d_traffic, double eps,
                                 int32_t iters, double *d_splits, double *d_lambda,
                                 hipStream_t s)
{
    hipError_t e = nimble::launch_persistent(topo->d, topo->sync_words, topo->n_cu,
                                             topo->spin_limit, d_traffic, eps, iters, d_splits,
                                             d_lambda, s);
    if (e != hipSuccess) return fail_hip(e, "kernel launch (persistent regime)");
    return NIMBLE_OK;
}

}  // namespace

// whether nimble_plan_solve_adaptive applies a step inside the next iteration's record kernel
static bool adaptive_folds(const nimble_topo_t *t)
{
    if (t->ad_fold == 0 || (t->d.n_blocks <= 0 && t->d.n_gblocks <= 0)) return false;
    return nimble::record_kernel_folds(t->d, t->ad_fold == 1);
}

extern "C" {

const char *nimble_last_error(void) { return g_last_error.c_str(); }

nimble_status_t nimble_topo_create(int32_t n_links, const double *cap, int32_t n_comm,
                                   const int32_t *comm_path_ptr, int32_t n_paths,
                                   const int32_t *path_link_ptr, const int32_t *path_links,
                                   uint32_t flags, nimble_topo_t **out)
{
    g_last_error.clear();
    if (!out) return fail(NIMBLE_ERR_INVALID, "out is NULL");
    *out = nullptr;
    if (!cap) return fail(NIMBLE_ERR_INVALID, "cap is NULL");
    if (flags & ~static_cast<uint32_t>(NIMBLE_COST_MAX | NIMBLE_LAYOUT_BATCH))
        return fail(NIMBLE_ERR_INVALID, "unknown flag bits");
    std::string why;
    nimble_status_t st = nimble::validate_csr(n_links, cap, n_comm, comm_path_ptr, n_paths,
                                              path_link_ptr, path_links, why);
    if (st != NIMBLE_OK) return fail(st, why);
    const int64_t nnz = path_link_ptr[n_paths];
    if (nnz + 3LL * n_links >= (1LL << 31))
        return fail(NIMBLE_ERR_RANGE, "padded reverse CSR exceeds 2^31 entries");

    nimble_topo *t = nullptr;
    nimble::HostTopo h;
    try {
        t = new nimble_topo();
        // a topology meant for batches takes the tiled reverse layout whatever its size: its
        // choices and demands are fetched window by window, which is what bounds a launch that
        // covers many plans (a single plan of a mid-size fabric is faster with link blocks)
        // (and few, large blocks of link groups: 16 blocks x 16 plans put one workgroup of the
        // fused reduce + update kernel on every compute unit; pieces from 64 commodities on)
        if (flags & NIMBLE_LAYOUT_BATCH) {
            h.tiles = 1;
            h.grp_target = 16;
            h.tile_min_items = 64;
        }
        if (g_fail_host_alloc.exchange(0) != 0) throw std::bad_alloc();      // test hook
        nimble::read_layout_options(h);
        nimble::build_host_topo(n_links, cap, n_comm, comm_path_ptr, n_paths, path_link_ptr,
                                path_links, h);
    } catch (const std::bad_alloc &) {
        delete t;
        return fail(NIMBLE_ERR_ALLOC, "host allocation failed");
    }

    hipError_t e = hipGetDevice(&t->device);
    if (e != hipSuccess) {
        delete t;
        return fail_hip(e, "hipGetDevice (is a GPU visible?)");
    }

    nimble::DeviceTopo &d = t->d;
    d.E = h.E;
    d.K = h.K;
    d.P = h.P;
    d.nnz = h.nnz;
    d.rev_pairs = static_cast<int64_t>(h.rev_pair.size() / 2);
    d.rev_row_max = 0;
    for (int32_t len : h.rev_rowlen) d.rev_row_max = std::max(d.rev_row_max, len);
    t->no_choice_log = std::getenv("NIMBLE_TUNE_NO_CHOICE_LOG") != nullptr;
    if (const char *v = std::getenv("NIMBLE_TUNE_ADAPTIVE_FOLD")) t->ad_fold = std::atoi(v) != 0;
    d.resident_generic = std::getenv("NIMBLE_TUNE_RESIDENT_GENERIC") ? 1 : 0;
    d.alg1_thread_per_problem = std::getenv("NIMBLE_TUNE_ALG1_THREAD_PER_PROBLEM") ? 1 : 0;
    d.n_records = h.n_records;
    d.rec_stride = h.rec_stride;
    d.rec_max_links = h.rec_max_links;
    d.rec_lanes = h.rec_lanes;
    d.rec_per_wave = 0;
    if (const char *env = std::getenv("NIMBLE_TUNE_RECORDS_PER_WAVE"))
        if (std::atoi(env) >= 1 && std::atoi(env) <= 64) d.rec_per_wave = std::atoi(env);
    d.rec_lane_major = h.rec_lane_major;
    d.rec_table16 = h.rec_table16;
    d.rec_dict = h.rec_dict;
    d.n_bodies = h.n_bodies;
    d.rec_around_l2 = -1;
    if (const char *env = std::getenv("NIMBLE_TUNE_RECORD_AROUND_L2"))
        d.rec_around_l2 = std::atoi(env) != 0 ? 1 : 0;
    // (a lane-major layout has its lanes per commodity built in)
    if (const char *env = std::getenv("NIMBLE_TUNE_RECORD_LANES")) {
        const int v = std::atoi(env);
        if (!d.rec_lane_major &&
            (v == 1 || v == 2 || v == 4 || v == 8 || v == 16 || v == 32 || v == 64))
            d.rec_lanes = v;
    }
    if (std::getenv("NIMBLE_TUNE_NO_RECORDS")) d.n_records = 0;
    d.pmax = h.pmax;
    d.lmax = h.lmax;
    d.n_passes = static_cast<int32_t>(h.oct_base.size() / 64);
    d.n_schunks = static_cast<int32_t>(h.schunk_begin.size());
    d.n_slots = h.n_slots;
    d.cost_max = (flags & NIMBLE_COST_MAX) != 0u;
    // 256-thread blocks; a link gets 16 lanes for its slot partials, or 4 when links have few
    // slots (tiled layouts)
    d.update_lanes = (static_cast<int64_t>(h.n_slots) <= 6LL * h.E) ? 4 : 16;
    if (const char *v = std::getenv("NIMBLE_TUNE_UPDATE_LANES")) {
        const int x = std::atoi(v);
        if (x == 4 || x == 16) d.update_lanes = x;
    }
    d.n_update_blocks = (h.E + 256 / d.update_lanes - 1) / (256 / d.update_lanes);
    d.n_blocks = std::getenv("NIMBLE_TUNE_NO_LINK_BLOCKS") ? 0 : h.n_blocks;
    // blocks of link groups: a workgroup of 4, 8 or 16 waves, about two tasks per wave in the
    // largest block
    d.n_gblocks = h.n_gblocks;
    d.gblk_max_slots = h.gblk_max_slots;
    d.gblk_waves = 4;
    while (d.gblk_waves < 16 && 2 * d.gblk_waves < h.gblk_max_tasks) d.gblk_waves *= 2;
    if (const char *v = std::getenv("NIMBLE_TUNE_GROUP_WAVES")) {
        const int x = std::atoi(v);
        if (x == 4 || x == 8 || x == 16) d.gblk_waves = x;
    }

#define NIMBLE_TRY(call, what)                        \
    do {                                              \
        e = (call);                                   \
        if (e != hipSuccess) {                        \
            release(t);                               \
            delete t;                                 \
            return e == hipErrorOutOfMemory           \
                       ? fail(NIMBLE_ERR_ALLOC, what) \
                       : fail_hip(e, what);           \
        }                                             \
    } while (0)

    NIMBLE_TRY(upload(t, comm_path_ptr, static_cast<size_t>(h.K) + 1, &d.comm_ptr), "comm_ptr");
    NIMBLE_TRY(upload(t, path_link_ptr, static_cast<size_t>(h.P) + 1, &d.path_ptr), "path_ptr");
    NIMBLE_TRY(upload(t, path_links, static_cast<size_t>(h.nnz), &d.path_links), "path_links");
    NIMBLE_TRY(upload(t, h.rev_ptr.data(), h.rev_ptr.size(), &d.rev_ptr), "rev_ptr");
    NIMBLE_TRY(upload(t, h.rev_pair.data(), h.rev_pair.size(), &d.rev_pair), "rev_pair");
    if (d.n_records > 0)
        NIMBLE_TRY(upload(t, h.records.data(), h.records.size(), &d.records), "records");
    NIMBLE_TRY(upload(t, h.oct_base.data(), h.oct_base.size(), &d.oct_base), "oct_base");
    NIMBLE_TRY(upload(t, h.oct_mask.data(), h.oct_mask.size(), &d.oct_mask), "oct_mask");
    NIMBLE_TRY(upload(t, h.single_pair.data(), h.single_pair.size(), &d.single_pair),
               "single_pair");
    NIMBLE_TRY(upload(t, h.pass_first_slot.data(), h.pass_first_slot.size(), &d.pass_first_slot),
               "pass_first_slot");
    {
        const int2 *px = nullptr;
        NIMBLE_TRY(upload(t, reinterpret_cast<const int2 *>(h.pos_xslot.data()),
                          h.pos_xslot.size() / 2, &px),
                   "pos_xslot");
        d.pos_xslot = px;
    }
    NIMBLE_TRY(upload(t, h.schunk_begin.data(), h.schunk_begin.size(), &d.schunk_begin), "schunk");
    NIMBLE_TRY(upload(t, h.schunk_end.data(), h.schunk_end.size(), &d.schunk_end), "schunk");
    NIMBLE_TRY(upload(t, h.schunk_slot.data(), h.schunk_slot.size(), &d.schunk_slot), "schunk");
    NIMBLE_TRY(upload(t, h.pos_link.data(), h.pos_link.size(), &d.pos_link), "pos_link");
    {
        std::vector<int32_t> pos_of_link(h.pos_link.size());
        for (size_t i = 0; i < h.pos_link.size(); ++i) pos_of_link[h.pos_link[i]] = static_cast<int32_t>(i);
        NIMBLE_TRY(upload(t, pos_of_link.data(), pos_of_link.size(), &t->ad.pos_of_link),
                   "pos_of_link");
    }
    NIMBLE_TRY(upload(t, h.pos_slot_ptr.data(), h.pos_slot_ptr.size(), &d.pos_slot_ptr),
               "pos_slot_ptr");
    NIMBLE_TRY(upload(t, h.blk_desc.data(), h.blk_desc.size(), &d.blk_desc), "blk_desc");
    NIMBLE_TRY(upload(t, h.gblk_desc.data(), h.gblk_desc.size(), &d.gblk_desc), "gblk_desc");
    NIMBLE_TRY(upload(t, h.tile_desc.data(), h.tile_desc.size(), &d.tile_desc), "tile_desc");
    NIMBLE_TRY(upload(t, h.tile_mask.data(), h.tile_mask.size(), &d.tile_mask), "tile_mask");
    NIMBLE_TRY(upload(t, h.tile_pres.data(), h.tile_pres.size(), &d.tile_pres), "tile_pres");
    NIMBLE_TRY(upload(t, h.strip_base.data(), h.strip_base.size(), &d.strip_base), "strip_base");
    NIMBLE_TRY(upload(t, h.strip_pres.data(), h.strip_pres.size(), &d.strip_pres), "strip_pres");
    NIMBLE_TRY(upload(t, h.strip_mask.data(), h.strip_mask.size(), &d.strip_mask), "strip_mask");
    NIMBLE_TRY(upload(t, h.strip_slot.data(), h.strip_slot.size(), &d.strip_slot), "strip_slot");
    d.n_strip_items = h.n_strip_items;
    d.n_tile_items = h.n_tile_items;
    d.tile_item_cost = 1;
    if (const char *env = std::getenv("NIMBLE_TUNE_TILE_ITEM_COST"))
        if (std::atoi(env) >= 1 && std::atoi(env) <= 64) d.tile_item_cost = std::atoi(env);
    NIMBLE_TRY(upload(t, h.sigma.data(), h.sigma.size(), &d.sigma), "sigma");
    d.sigma_size = h.sigma_size;
    NIMBLE_TRY(upload(t, h.invcap.data(), h.invcap.size(), &d.invcap), "invcap");
    NIMBLE_TRY(upload(t, h.invcap_pos.data(), h.invcap_pos.size(), &d.invcap_pos), "invcap_pos");
    // the state of one plan in flight (a block of its own per plan of a batch)
    d.batch = 1;
    d.batch_kernel = 0;
    if (const char *env = std::getenv("NIMBLE_TUNE_BATCH_KERNEL"))
        if (std::atoi(env) >= 0 && std::atoi(env) <= 1) d.batch_kernel = std::atoi(env);
    NIMBLE_TRY(ensure_state_plans(t, 1), "plan state");
    {
        unsigned char *sw = nullptr;
        NIMBLE_TRY(allocate(t, nimble::persistent_sync_bytes(), &sw), "sync words");
        t->sync_words = sw;
        NIMBLE_TRY(hipDeviceGetAttribute(&t->n_cu, hipDeviceAttributeMultiprocessorCount,
                                         t->device),
                   "hipDeviceGetAttribute");
        // the reduce kernel takes 114 VGPRs: four of its four-wave workgroups per compute unit
        // are resident at once, and a grid of exactly those measured best (22.2 ms per plan on
        // the 64-node fabric against 22.4 to 23.0 with three, five, six or eight)
        int per_cu = 4;
        if (const char *env = std::getenv("NIMBLE_TUNE_REDUCE_BLOCKS_PER_CU"))
            if (std::atoi(env) > 0) per_cu = std::atoi(env);
        d.reduce_blocks = t->n_cu * per_cu;
        // the record kernel with inline bodies: 78 VGPRs, so six of its four-wave workgroups
        // per compute unit; the dictionary kernel says itself how many fit (its grid must be
        // resident at once: a workgroup that starts late finishes late)
        int rec_per_cu = 6;
        d.cost_max = (flags & NIMBLE_COST_MAX) != 0u;
        if (const int occ = nimble::record_kernel_blocks_per_cu(d)) rec_per_cu = occ;
        if (const char *env = std::getenv("NIMBLE_TUNE_RECORD_BLOCKS_PER_CU"))
            if (std::atoi(env) > 0) rec_per_cu = std::atoi(env);
        d.rec_blocks = t->n_cu * rec_per_cu;
    }
    if (d.rec_dict && d.n_records > 0) {
        // Runs of records for the waves of the record kernel: a run holds records of one body
        // (the wave fetches that body once), and the runs are as short as the number of waves
        // that are resident at once allows, so that the grid still fills the chip once.
        const int64_t max_waves = 4LL * d.rec_blocks;
        std::vector<int32_t> run_begin;      // first record of every body's range
        for (int32_t i = 0; i < d.n_records; ++i)
            if (i == 0 || h.rec_body[i] != h.rec_body[i - 1]) run_begin.push_back(i);
        run_begin.push_back(d.n_records);
        int32_t per = 1;
        if (const char *env = std::getenv("NIMBLE_TUNE_RECORDS_PER_WAVE"))
            if (std::atoi(env) >= 1 && std::atoi(env) <= 64) per = std::atoi(env);
        for (;; ++per) {
            int64_t n = 0;
            for (size_t b = 0; b + 1 < run_begin.size(); ++b)
                n += (run_begin[b + 1] - run_begin[b] + per - 1) / per;
            if (n <= max_waves || d.rec_per_wave > 0) break;
        }
        std::vector<int32_t> chunks;
        for (size_t b = 0; b + 1 < run_begin.size(); ++b) {
            // the records of a body are dealt as evenly as its number of runs allows
            const int32_t n_rec = run_begin[b + 1] - run_begin[b];
            const int32_t n_runs = (n_rec + per - 1) / per;
            int32_t at = run_begin[b];
            for (int32_t r = 0; r < n_runs; ++r) {
                const int32_t cnt = n_rec / n_runs + (r < n_rec % n_runs ? 1 : 0);
                chunks.push_back(at);
                chunks.push_back(cnt);
                chunks.push_back(h.rec_body[at]);
                chunks.push_back(0);
                at += cnt;
            }
        }
        d.n_rec_chunks = static_cast<int32_t>(chunks.size() / 4);
        const int4 *pc = nullptr;
        NIMBLE_TRY(upload(t, reinterpret_cast<const int4 *>(chunks.data()), chunks.size() / 4, &pc),
                   "record runs");
        d.rec_chunks = pc;
        NIMBLE_TRY(upload(t, h.rec_dict_words.data(), h.rec_dict_words.size(), &d.rec_dict_words),
                   "record bodies");
    }

    {
        // the address of the static scratch on this device (nimble_plan_solve_static)
        unsigned char *sp = nullptr;
        NIMBLE_TRY(static_scratch_of(t->device, &sp), "hipGetSymbolAddress (static scratch)");
    }
#undef NIMBLE_TRY
    // a choice log for solves of up to kDefaultLogRows iterations, when that is small; larger
    // ones are the caller's decision (nimble_topo_reserve)
    if (!t->no_choice_log &&
        choice_log_stride(t) * static_cast<size_t>(kDefaultLogRows) <= kChoiceLogAtCreate) {
        nimble_status_t st_log = grow_choice_log(t, kDefaultLogRows);
        if (st_log != NIMBLE_OK) {
            release(t);
            delete t;
            return st_log;
        }
    }

    // stored bytes one iteration streams, phase by phase
    if (d.n_records > 0)
        // (a dictionary of bodies is counted once: it stays in the L2)
        t->bytes_argmin = static_cast<int64_t>(h.rec_bytes) * d.n_records + 2LL * h.K +
                          (d.rec_dict ? 4LL * static_cast<int64_t>(h.rec_dict_words.size()) +
                                            16LL * d.n_rec_chunks
                                      : 0LL);
    else
        t->bytes_argmin = 4LL * (h.K + 1) + 4LL * (h.P + 1) + 4LL * h.nnz + 14LL * h.K;
    t->bytes_reduce = 36LL * static_cast<int64_t>(h.oct_base.size()) + 4LL * d.n_passes +
                      4LL * static_cast<int64_t>(h.single_pair.size()) + 12LL * d.n_schunks +
                      8LL * d.n_slots;
    t->bytes_update = 8LL * d.n_slots + 8LL * (h.E + 1) + 56LL * h.E;
    // tile items: 2 KiB per piece, the descriptor, the window's choices and demands, one slot
    // per piece
    t->bytes_reduce += 2048LL * (h.n_pieces - h.n_pieces_uniform) + 8LL * h.n_pieces +
                       (128LL + 512 + 4096) * h.n_tile_items +
                       64LL * static_cast<int64_t>(h.tile_pres.size() / 64 - 1) +
                       // strip items: base, presence, masks and slots per lane (20 B), one line
                       // of choices and one of demands per column, a partial per unit and row
                       64LL * (20 + 8 + 64 + 8) * h.n_strip_items;
    if (d.n_blocks > 0) {
        // one kernel: the slot partials stay in LDS; per block two table entries and one maximum
        t->bytes_reduce = 36LL * static_cast<int64_t>(h.oct_base.size()) + 4LL * d.n_passes +
                          8LL * h.E + 56LL * h.E + 64LL * d.n_blocks;
        t->bytes_update = 0;
    }
    if (d.n_gblocks > 0) {
        // one kernel: the slot partials stay in LDS; the links' tables and state, a descriptor
        // and sixteen maxima per block
        t->bytes_reduce += -8LL * d.n_slots + 16LL * h.E + 56LL * h.E + 192LL * d.n_gblocks;
        t->bytes_update = 0;
    }
    t->bytes_per_iter = t->bytes_argmin + t->bytes_reduce + t->bytes_update;
    // lane-major record kernels: every lane reads 8-byte prices from LDS, per record one for
    // every step of the 8 candidates of its two quads (padding steps included), or 9 for a
    // quad in the product shape
    if (d.n_records > 0 && d.rec_lane_major) t->bytes_lds_argmin = 64 * 8 * h.rec_price_reads;
    *out = t;
    return NIMBLE_OK;
}

void nimble_topo_destroy(nimble_topo_t *topo)
{
    if (!topo) return;
    release(topo);
    delete topo;
}

int32_t nimble_topo_num_links(const nimble_topo_t *t) { return t ? t->d.E : -1; }
int32_t nimble_topo_num_comm(const nimble_topo_t *t) { return t ? t->d.K : -1; }
int32_t nimble_topo_num_paths(const nimble_topo_t *t) { return t ? t->d.P : -1; }
int64_t nimble_topo_nnz(const nimble_topo_t *t) { return t ? t->d.nnz : -1; }
int64_t nimble_topo_bytes_per_iter(const nimble_topo_t *t) { return t ? t->bytes_per_iter : -1; }
int32_t nimble_topo_regime(const nimble_topo_t *t) { return t ? t->last_regime : -1; }
int32_t nimble_topo_adaptive_folds(const nimble_topo_t *t)
{
    return t ? (adaptive_folds(t) ? 1 : 0) : -1;
}

int32_t nimble_topo_resident_in_registers(const nimble_topo_t *t)
{
    return t ? (nimble::resident_in_registers(t->d) ? 1 : 0) : -1;
}

int64_t nimble_topo_phase_bytes(const nimble_topo_t *t, int32_t phase)
{
    if (!t) return -1;
    switch (phase) {
    case 0: return t->bytes_argmin;
    case 1: return t->bytes_reduce;
    case 2: return t->bytes_update;
    case 3: return t->bytes_lds_argmin;
    default: return -1;
    }
}

nimble_status_t nimble_topo_set_regime(nimble_topo_t *topo, int32_t regime)
{
    g_last_error.clear();
    if (!topo) return fail(NIMBLE_ERR_INVALID, "topology handle is NULL");
    switch (regime) {
    case NIMBLE_REGIME_AUTO:
    case NIMBLE_REGIME_STREAM:
    case NIMBLE_REGIME_PERSISTENT:
        break;
    case NIMBLE_REGIME_RESIDENT:
        if (!nimble::resident_fits(topo->d))
            return fail(NIMBLE_ERR_RANGE, "per-plan state does not fit in LDS");
        break;
    default:
        return fail(NIMBLE_ERR_INVALID, "unknown regime");
    }
    topo->forced_regime = regime;
    return NIMBLE_OK;
}

nimble_status_t nimble_plan_solve(nimble_topo_t *topo, const double *d_traffic, double eps,
                                  int32_t iters, double *d_splits, double *d_lambda,
                                  void *hip_stream)
{
    g_last_error.clear();
    nimble_status_t st = check_solve_args(topo, d_traffic, eps, iters, d_splits, d_lambda);
    if (st != NIMBLE_OK) return st;
    st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int32_t regime = pick_regime(topo, 1);
    topo->last_regime = regime;
    if (regime == NIMBLE_REGIME_RESIDENT) {
        hipError_t e = nimble::launch_resident(topo->d, 1, d_traffic, eps, iters, d_splits,
                                               d_lambda, s);
        if (e != hipSuccess) return fail_hip(e, "kernel launch (resident regime)");
        return NIMBLE_OK;
    }
    if (regime == NIMBLE_REGIME_PERSISTENT)
        return solve_persistent(topo, d_traffic, eps, iters, d_splits, d_lambda, s);
    return solve_stream(topo, d_traffic, eps, iters, d_splits, d_lambda, s, own_log(topo, iters),
                        topo->log_stride);
}

nimble_status_t nimble_plan_solve_batch(nimble_topo_t *topo, int32_t batch,
                                        const double *d_traffic, double eps, int32_t iters,
                                        double *d_splits, double *d_lambda, void *hip_stream)
{
    g_last_error.clear();
    nimble_status_t st = check_solve_args(topo, d_traffic, eps, iters, d_splits, d_lambda);
    if (st != NIMBLE_OK) return st;
    if (batch < 1) return fail(NIMBLE_ERR_INVALID, "batch must be >= 1");
    st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int32_t regime = pick_regime(topo, batch);
    topo->last_regime = regime;
    if (regime == NIMBLE_REGIME_RESIDENT) {
        hipError_t e = nimble::launch_resident(topo->d, batch, d_traffic, eps, iters, d_splits,
                                               d_lambda, s);
        if (e != hipSuccess) return fail_hip(e, "kernel launch (resident regime)");
        return NIMBLE_OK;
    }
    if (regime == NIMBLE_REGIME_PERSISTENT) {
        for (int32_t b = 0; b < batch; ++b) {
            st = solve_persistent(topo, d_traffic + static_cast<size_t>(b) * topo->d.K, eps, iters,
                                  d_splits + static_cast<size_t>(b) * topo->d.P, d_lambda + b, s);
            if (st != NIMBLE_OK) return st;
        }
        return NIMBLE_OK;
    }
    // streaming regime: the plans share every launch, as many at a time as the state reserved
    // for them holds (nimble_topo_reserve_batch; a topology starts with room for one)
    const int32_t group = std::min(batch, topo->state_plans);
    for (int32_t b = 0; b < batch; b += group) {
        const int32_t n = std::min(group, batch - b);
        st = solve_stream(topo, d_traffic + static_cast<size_t>(b) * topo->d.K, eps, iters,
                          d_splits + static_cast<size_t>(b) * topo->d.P, d_lambda + b, s,
                          own_log(topo, iters, n), topo->log_stride, nullptr, n);
        if (st != NIMBLE_OK) return st;
    }
    return NIMBLE_OK;
}

nimble_status_t nimble_topo_reserve(nimble_topo_t *topo, int32_t iters)
{
    g_last_error.clear();
    if (!topo) return fail(NIMBLE_ERR_INVALID, "topology handle is NULL");
    if (iters < 1) return fail(NIMBLE_ERR_INVALID, "iters must be >= 1");
    nimble_status_t st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    if (topo->no_choice_log) return NIMBLE_OK;
    return grow_choice_log(topo, iters);
}

nimble_status_t nimble_topo_reserve_batch(nimble_topo_t *topo, int32_t plans, int32_t iters)
{
    g_last_error.clear();
    if (!topo) return fail(NIMBLE_ERR_INVALID, "topology handle is NULL");
    if (plans < 1 || iters < 1) return fail(NIMBLE_ERR_INVALID, "plans and iters must be >= 1");
    nimble_status_t st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    const StateLayout L = state_layout(topo->d);
    if (L.bytes * static_cast<size_t>(plans) > kStateCap)
        return fail(NIMBLE_ERR_RANGE, "the state of that many plans exceeds 4 GiB");
    hipError_t e = ensure_state_plans(topo, plans);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return e == hipErrorOutOfMemory ? fail(NIMBLE_ERR_ALLOC, "plan state")
                                        : fail_hip(e, "plan state");
    }
    if (topo->no_choice_log) return NIMBLE_OK;
    if (static_cast<int64_t>(plans) * iters > INT32_MAX)
        return fail(NIMBLE_ERR_RANGE, "plans * iters exceeds 2^31");
    return grow_choice_log(topo, plans * iters);
}

int64_t nimble_static_scratch_bytes(void) { return static_cast<int64_t>(kStaticScratchBytes); }

nimble_status_t nimble_plan_solve_static(nimble_topo_t *topo, const double *d_traffic, double eps,
                                         int32_t iters, double *d_splits, double *d_lambda,
                                         void *hip_stream)
{
    g_last_error.clear();
    nimble_status_t st = check_solve_args(topo, d_traffic, eps, iters, d_splits, d_lambda);
    if (st != NIMBLE_OK) return st;
    st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    const size_t stride = choice_log_stride(topo);
    if (stride * static_cast<size_t>(iters) > kStaticScratchBytes)
        return fail(NIMBLE_ERR_RANGE,
                    "choice log (commodities rounded up to 512, times iters) exceeds the static "
                    "scratch of " + std::to_string(kStaticScratchBytes) + " bytes");
    // resolved at nimble_topo_create on this device; this lookup only reads the table
    unsigned char *log = nullptr;
    hipError_t e = static_scratch_of(topo->device, &log);
    if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress (static scratch)");
    topo->last_regime = NIMBLE_REGIME_STREAM;
    // every row of the log is written (entries 0..K-1) before it is read and nothing has to
    // start at zero, so what the previous call left behind does no harm
    return solve_stream(topo, d_traffic, eps, iters, d_splits, d_lambda,
                        static_cast<hipStream_t>(hip_stream), log, stride);
}

nimble_status_t nimble_host_resident_kernel(int32_t n_links, int32_t n_comm,
                                            const int32_t *comm_path_ptr, int32_t n_paths,
                                            const int32_t *path_link_ptr,
                                            const int32_t *path_links, int32_t *kernel_out)
{
    g_last_error.clear();
    if (!kernel_out) return fail(NIMBLE_ERR_INVALID, "kernel_out is NULL");
    std::vector<double> cap(n_links > 0 ? static_cast<size_t>(n_links) : 0, 1.0);
    std::string why;
    nimble_status_t st = nimble::validate_csr(n_links, cap.data(), n_comm, comm_path_ptr, n_paths,
                                              path_link_ptr, path_links, why);
    if (st != NIMBLE_OK) return fail(st, why);
    nimble::HostTopo h;
    try {
        nimble::read_layout_options(h);
        nimble::build_host_topo(n_links, cap.data(), n_comm, comm_path_ptr, n_paths,
                                path_link_ptr, path_links, h);
    } catch (const std::bad_alloc &) {
        return fail(NIMBLE_ERR_ALLOC, "host allocation failed");
    }
    nimble::DeviceTopo d{};
    d.E = h.E;
    d.K = h.K;
    d.P = h.P;
    d.nnz = h.nnz;
    d.pmax = h.pmax;
    d.lmax = h.lmax;
    d.rev_pairs = static_cast<int64_t>(h.rev_pair.size() / 2);
    for (int32_t len : h.rev_rowlen) d.rev_row_max = std::max(d.rev_row_max, len);
    d.resident_generic = std::getenv("NIMBLE_TUNE_RESIDENT_GENERIC") ? 1 : 0;
    *kernel_out = nimble::resident_kernel_kind(d, 1);
    return NIMBLE_OK;
}

nimble_status_t nimble_alg1_solve_batch(nimble_topo_t *topo, int32_t batch,
                                        const double *d_traffic, double phi, double chi,
                                        int32_t max_sweeps, double *d_flows, double *d_lambda,
                                        int32_t *d_sweeps, void *hip_stream)
{
    g_last_error.clear();
    if (!topo) return fail(NIMBLE_ERR_INVALID, "topology handle is NULL");
    if (!d_traffic || !d_flows || !d_lambda || !d_sweeps)
        return fail(NIMBLE_ERR_INVALID,
                    "traffic, flows, lambda and sweeps pointers must not be NULL");
    if (batch < 1) return fail(NIMBLE_ERR_INVALID, "batch must be >= 1");
    if (!(phi > 0.0) || !(phi <= 1.0)) return fail(NIMBLE_ERR_INVALID, "phi must be in (0, 1]");
    if (!(chi > 0.0) || !std::isfinite(chi))
        return fail(NIMBLE_ERR_INVALID, "chi must be positive and finite");
    if (max_sweeps < 1) return fail(NIMBLE_ERR_INVALID, "max_sweeps must be >= 1");
    if (!nimble::alg1_fits(topo->d))
        return fail(NIMBLE_ERR_RANGE,
                    "the per-problem state does not fit in the LDS of a compute unit");
    nimble_status_t st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    hipError_t e = nimble::launch_alg1(topo->d, batch, d_traffic, phi, chi, max_sweeps, d_flows,
                                       d_lambda, d_sweeps, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail_hip(e, "kernel launch (Algorithm 1)");
    return NIMBLE_OK;
}

nimble_status_t nimble_plan_solve_warm(nimble_topo_t *topo, const double *d_traffic, double eps,
                                       int32_t iters, double *d_len, double *d_splits,
                                       double *d_lambda, void *hip_stream)
{
    g_last_error.clear();
    nimble_status_t st = check_solve_args(topo, d_traffic, eps, iters, d_splits, d_lambda);
    if (st != NIMBLE_OK) return st;
    if (!d_len) return fail(NIMBLE_ERR_INVALID, "the length pointer must not be NULL");
    st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    topo->last_regime = NIMBLE_REGIME_STREAM;
    return solve_stream(topo, d_traffic, eps, iters, d_splits, d_lambda,
                        static_cast<hipStream_t>(hip_stream), own_log(topo, iters),
                        topo->log_stride, d_len);
}

nimble_status_t nimble_plan_solve_adaptive(nimble_topo_t *topo, const double *d_traffic,
                                           double eps, int32_t max_iters, int32_t check_every,
                                           double *d_splits, double *d_lambda,
                                           int32_t *iters_done, double *lower_bound,
                                           void *hip_stream)
{
    g_last_error.clear();
    nimble_status_t st = check_solve_args(topo, d_traffic, eps, max_iters, d_splits, d_lambda);
    if (st != NIMBLE_OK) return st;
    if (check_every < 1) return fail(NIMBLE_ERR_INVALID, "check_every must be >= 1");
    if (!iters_done || !lower_bound)
        return fail(NIMBLE_ERR_INVALID, "iters_done and lower_bound must not be NULL");
    st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const nimble::DeviceTopo &d = topo->d;
    nimble::AdaptiveState &a = topo->ad;
    hipError_t e = hipSuccess;
    if (!topo->ad_ready) {
        // all or nothing: what a failed attempt did allocate is given back, so that a retry
        // does not pile up buffers
        const size_t n_chunks = (static_cast<size_t>(d.K) + 255) / 256 + (static_cast<size_t>(d.E) + 255) / 256;
        const size_t mark = topo->allocs.size();
        e = allocate(topo, 2, &a.flags);
        if (e == hipSuccess) e = allocate(topo, 4, &a.ascal);
        if (e == hipSuccess) e = allocate(topo, n_chunks, &a.chunk);
        if (e == hipSuccess) e = allocate(topo, static_cast<size_t>(d.E), &a.u_pos);
        if (e == hipSuccess) e = allocate(topo, static_cast<size_t>(d.E), &a.u_id);
        if (e == hipSuccess) e = allocate(topo, static_cast<size_t>(d.E), &a.len_id[0]);
        if (e == hipSuccess) e = allocate(topo, static_cast<size_t>(d.E), &a.len_id[1]);
        if (e == hipSuccess)
            e = allocate(topo, std::max({(static_cast<size_t>(d.E) + 15) / 16,
                                         static_cast<size_t>(4) * static_cast<size_t>(d.n_blocks),
                                         static_cast<size_t>(16) * static_cast<size_t>(d.n_gblocks)}),
                         &a.block_max_u);
        if (e == hipSuccess && !a.host_words_host) {
            // two words of pinned host memory the device writes and the host polls
            void *hp = nullptr;
            e = hipHostMalloc(&hp, 4 * sizeof(int32_t), hipHostMallocMapped);
            if (e == hipSuccess) {
                a.host_words_host = static_cast<int32_t *>(hp);
                void *dp = nullptr;
                e = hipHostGetDevicePointer(&dp, hp, 0);
                a.host_words = static_cast<int32_t *>(dp);
            }
        }
        if (e == hipSuccess) e = allocate(topo, (static_cast<size_t>(d.E) + 255) / 256, &a.block_max_s);
        if (e != hipSuccess) {
            while (topo->allocs.size() > mark) {
                dev_free(topo->allocs.back());
                topo->allocs.pop_back();
            }
            (void)hipGetLastError();
            return e == hipErrorOutOfMemory ? fail(NIMBLE_ERR_ALLOC, "adaptive workspace")
                                            : fail_hip(e, "adaptive workspace");
        }
        topo->ad_ready = true;
    }
    if (topo->ad_sigma_rows < max_iters) {
        if (a.sigma_log) dev_free(a.sigma_log);
        a.sigma_log = nullptr;
        topo->ad_sigma_rows = 0;
        void *p = nullptr;
        if (dev_malloc(&p, sizeof(double) * static_cast<size_t>(max_iters)) != hipSuccess) {
            (void)hipGetLastError();
            return fail(NIMBLE_ERR_ALLOC, "step log of the adaptive solve");
        }
        a.sigma_log = static_cast<double *>(p);
        topo->ad_sigma_rows = max_iters;
    }
    // the weighted split fractions need the choice of every iteration
    if (topo->no_choice_log)
        return fail(NIMBLE_ERR_ALLOC, "the adaptive solve needs the choice log, which is switched off");
    st = grow_choice_log(topo, max_iters);
    if (st != NIMBLE_OK) return st;
    topo->last_regime = NIMBLE_REGIME_STREAM;
    const double gap = (1.0 + eps) * (1.0 + eps);
    // The device takes the stop decision and publishes it, with the number of checks made, in
    // pinned host memory.  The host enqueues ahead without ever synchronising the stream; it
    // only keeps within kAhead checks of the device, so that after the stop little is left in
    // the queue -- and what is left returns at once (every kernel of an iteration looks at the
    // stop word first).
    volatile int32_t *hw = a.host_words_host;
    hw[0] = 0;
    hw[1] = 0;
    nimble::DeviceTopo dd = d;
    dd.stop_flag = a.flags;
    const int32_t ahead = std::max(4, 128 / check_every);
    nimble::launch_ad_reset(a, s);
    nimble::launch_init(dd, d_traffic, nullptr, s);
    // Where the record kernel can, the step of an iteration is applied inside the record kernel
    // of the next one (two launches per iteration instead of three): the scan forms its prices
    // from the lengths before the step (by link id, a.len_id[cur]) while further workgroups of
    // that launch bring the stored state up to date and write the new lengths to the other
    // buffer.  The stop test of an iteration with a check wants lambda after that iteration's
    // step, so it follows the next record kernel (whose scan is then wasted if the solve stops:
    // its row of the choice log lies beyond the iterations made).
    const bool folding = adaptive_folds(topo);
    int cur = 0;                 // a.len_id[cur] holds the lengths of every step applied so far
    bool pending = false;        // the last iteration's step has not been applied yet
    bool lambda_due = false;     // ... and its stop test has not been made yet
    int n_u = 0;
    nimble::FoldArgs fold;
    if (folding) nimble::launch_ad_len_id(dd, a.len_id[0], s);
    int32_t checks = 0;
    bool stalled = false;
    for (int32_t t = 0; t < max_iters; ++t) {
        const bool check = ((t + 1) % check_every) == 0 && !d.cost_max;
        if (check && checks >= ahead) {
            // wait (on the host only) until the device is within `ahead` checks
            const auto t0 = std::chrono::steady_clock::now();
            while (__atomic_load_n(&hw[1], __ATOMIC_ACQUIRE) < checks - ahead + 1 &&
                   __atomic_load_n(&hw[0], __ATOMIC_ACQUIRE) == 0) {
                if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(30)) {
                    stalled = true;
                    break;
                }
                std::this_thread::yield();
            }
            if (stalled) break;
        }
        if (__atomic_load_n(&hw[0], __ATOMIC_ACQUIRE) != 0) break;       // the device has stopped
        uint8_t *row = topo->choice_log + topo->log_stride * static_cast<size_t>(t);
        if (pending) {
            fold.ap = nimble::ad_apply_args(dd, a, eps, n_u, a.len_id[cur ^ 1]);
            fold.len_id = a.len_id[cur];
            fold.u_id = a.u_id;
            fold.invcap = d.invcap;
            fold.apply_blocks = 0;                   // (the launch fills it in)
            dd.fold = &fold;
            nimble::launch_argmin(dd, row, nullptr, s);
            dd.fold = nullptr;
            cur ^= 1;
            pending = false;
        } else {
            nimble::launch_argmin(dd, row, nullptr, s);
        }
        if (lambda_due) nimble::launch_ad_lambda(dd, a, gap, ++checks, s);
        lambda_due = false;
        if (check) nimble::launch_ad_bound(dd, a, row, d_traffic, s);
        if (d.n_blocks > 0 || d.n_gblocks > 0) {
            // link blocks or blocks of link groups: normalised loads in one launch, then the
            // step -- now, or inside the next record kernel
            n_u = d.n_blocks > 0
                      ? nimble::launch_reduce_u(dd, row, a.u_pos, a.u_id, a.block_max_u, s)
                      : nimble::launch_group_reduce_u(dd, row, a.u_pos, a.u_id, a.block_max_u, s);
            if (folding && t + 1 < max_iters) {
                pending = true;
                lambda_due = check;
            } else {
                nimble::launch_ad_apply(dd, a, eps, n_u, a.len_id[cur ^ 1], s);
                cur ^= 1;
                if (check) nimble::launch_ad_lambda(dd, a, gap, ++checks, s);
            }
        } else {
            nimble::launch_load_reduce(dd, row, d_traffic, s);
            nimble::launch_ad_update(dd, a, eps, s);
            if (check) nimble::launch_ad_lambda(dd, a, gap, ++checks, s);
        }
    }
    if (pending) {
        // the loop was left with a step outstanding (the device has stopped, so these return at
        // once, or the host gave up waiting)
        nimble::launch_ad_apply(dd, a, eps, n_u, a.len_id[cur ^ 1], s);
        cur ^= 1;
        if (lambda_due) nimble::launch_ad_lambda(dd, a, gap, ++checks, s);
    }
    if (stalled) {
        (void)hipStreamSynchronize(s);
        return fail(NIMBLE_ERR_HIP, "adaptive solve: the device made no progress for 30 s");
    }
    int32_t flags_host[2] = {0, 0};
    nimble::launch_ad_lambda(d, a, gap, 0, s);
    e = nimble::launch_ad_histogram(d, a, topo->choice_log, topo->log_stride, d_splits, d_lambda, s);
    if (e != hipSuccess) return fail_hip(e, "kernel launch (adaptive regime)");
    double ascal_host[4] = {0, 0, 0, 0};
    e = hipMemcpyAsync(flags_host, a.flags, sizeof(flags_host), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess)
        e = hipMemcpyAsync(ascal_host, a.ascal, sizeof(ascal_host), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail_hip(e, "adaptive solve (results)");
    *iters_done = flags_host[1];
    *lower_bound = ascal_host[2];
    topo->state_ready = true;
    topo->state_log = topo->choice_log;
    return NIMBLE_OK;
}

nimble_status_t nimble_plan_quantize(nimble_topo_t *topo, const double *d_traffic,
                                     const double *d_splits, int32_t iters, int64_t chi,
                                     double small_threshold, double *d_flows, void *hip_stream)
{
    g_last_error.clear();
    if (!topo) return fail(NIMBLE_ERR_INVALID, "topology handle is NULL");
    if (!d_traffic || !d_splits || !d_flows)
        return fail(NIMBLE_ERR_INVALID, "traffic, splits and flows pointers must not be NULL");
    if (iters < 1) return fail(NIMBLE_ERR_INVALID, "iters must be >= 1");
    if (chi < 1 || chi > (1LL << 40))
        return fail(NIMBLE_ERR_INVALID, "chi must be a whole number of bytes in [1, 2^40]");
    if (!(small_threshold >= 0.0))
        return fail(NIMBLE_ERR_INVALID, "small_threshold must be >= 0");
    nimble_status_t st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    hipError_t e = nimble::launch_quantize(topo->d, d_traffic, d_splits, iters, chi,
                                           small_threshold, d_flows,
                                           static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail_hip(e, "kernel launch (plan quantisation)");
    return NIMBLE_OK;
}

nimble_status_t nimble_debug_set_spin_limit(nimble_topo_t *topo, uint32_t polls)
{
    g_last_error.clear();
    if (!topo) return fail(NIMBLE_ERR_INVALID, "topology handle is NULL");
    topo->spin_limit = polls;
    return NIMBLE_OK;
}

nimble_status_t nimble_debug_run_phase(nimble_topo_t *topo, int32_t phase, int32_t reps,
                                       const double *d_traffic, void *hip_stream)
{
    g_last_error.clear();
    if (!topo || !d_traffic) return fail(NIMBLE_ERR_INVALID, "NULL argument");
    if (phase < 0 || phase > 2 || reps < 1) return fail(NIMBLE_ERR_INVALID, "bad phase or reps");
    if (phase == 2 && (topo->d.n_blocks > 0 || topo->d.n_gblocks > 0))
        return fail(NIMBLE_ERR_INVALID, "the length update is part of phase 1 on this topology");
    if (!topo->state_ready)
        return fail(NIMBLE_ERR_INVALID, "run a streaming-regime solve on this topology first");
    nimble_status_t st = check_device(topo);
    if (st != NIMBLE_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    for (int32_t r = 0; r < reps; ++r) {
        uint8_t *row = topo->state_log ? topo->state_log : topo->d.choice;
        if (phase == 0) nimble::launch_argmin(topo->d, row, topo->state_log ? nullptr : topo->d.count, s);
        else if (phase == 1 && topo->d.n_blocks > 0)
            nimble::launch_reduce_update(topo->d, row, d_traffic, 0.0, s);
        else if (phase == 1 && topo->d.n_gblocks > 0)
            nimble::launch_group_reduce_update(topo->d, row, 0.0, s);
        else if (phase == 1) nimble::launch_load_reduce(topo->d, row, d_traffic, s);
        else nimble::launch_update(topo->d, 0.0, s);   // eps 0: lengths stay as they are
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "kernel launch (phase timing)");
    return NIMBLE_OK;
}

nimble_status_t nimble_debug_barrier_probe(int32_t kind, int32_t blocks_per_cu, int32_t threads,
                                           int32_t rounds, uint32_t spin_limit, void *d_work,
                                           int64_t work_bytes, int32_t *d_out, void *hip_stream)
{
    g_last_error.clear();
    if (!d_work || !d_out) return fail(NIMBLE_ERR_INVALID, "NULL argument");
    if (kind < 0 || kind > 5 || blocks_per_cu < 1 || blocks_per_cu > 8 || rounds < 1 ||
        threads < 64 || threads > 1024 || threads % 64)
        return fail(NIMBLE_ERR_INVALID, "kind 0..5, 1..8 blocks per CU, 64..1024 threads");
    int dev = -1, n_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess)
        e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return fail_hip(e, "device query");
    // 8 XCDs on this part; the grid is a multiple of their number
    const int n_xcd = 8;
    const int blocks = n_cu * blocks_per_cu / n_xcd * n_xcd;
    if (blocks < n_xcd) return fail(NIMBLE_ERR_RANGE, "fewer compute units than XCDs");
    if (static_cast<int64_t>(nimble::barrier_probe_bytes(blocks)) > work_bytes)
        return fail(NIMBLE_ERR_INVALID, "d_work is too small for this grid");
    e = nimble::launch_barrier_probe(kind, blocks, threads, rounds, spin_limit, n_xcd, d_work,
                                     d_out, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail_hip(e, "cooperative launch (barrier probe)");
    return NIMBLE_OK;
}

nimble_status_t nimble_debug_fail_allocation(int32_t nth)
{
    g_last_error.clear();
    if (nth < -1) return fail(NIMBLE_ERR_INVALID, "nth must be >= -1");
    g_fail_alloc_in.store(nth);
    return NIMBLE_OK;
}

void nimble_debug_fail_host_allocation(void) { g_fail_host_alloc.store(1); }

int64_t nimble_debug_live_allocations(void) { return g_live_allocs.load(); }

nimble_status_t nimble_debug_stream_read(const void *d_buf, int64_t bytes, int32_t reps,
                                         void *d_sink, void *hip_stream)
{
    g_last_error.clear();
    if (!d_buf || !d_sink) return fail(NIMBLE_ERR_INVALID, "NULL argument");
    if (bytes < 16 || reps < 1) return fail(NIMBLE_ERR_INVALID, "bytes must be >= 16, reps >= 1");
    if ((reinterpret_cast<uintptr_t>(d_buf) | reinterpret_cast<uintptr_t>(d_sink)) & 15u)
        return fail(NIMBLE_ERR_INVALID, "buffers must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    for (int32_t r = 0; r < reps; ++r)
        nimble::launch_stream_read(d_buf, static_cast<size_t>(bytes), d_sink, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "kernel launch (streaming read)");
    return NIMBLE_OK;
}

}  // extern "C"

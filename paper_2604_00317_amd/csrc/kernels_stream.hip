// Streaming regime: one kernel per phase of a Jacobi iteration.  The path-cost gather + argmin
// runs over the forward records (k_argmin_rec) or the plain CSR (k_argmin); the link-load
// reduce and the length update are either one kernel per block of links (k_reduce_update) or
// two (k_load_reduce over tile items, strip items, octet passes and single pairs, then
// k_update).  The reduce phases themselves live in phases.hpp.
#include "host_topo.hpp"
#include "kernels.hpp"
#include "phases.hpp"
#include "wave_ops.hpp"

namespace nimble {

namespace {

constexpr int kBlock = 256;

__global__ __launch_bounds__(kBlock) void k_init(int E, int K, int P, bool cost_max,
                                                 const double *__restrict__ len_in,
                                                 const int32_t *__restrict__ pos_link,
                                                 const double *__restrict__ invcap,
                                                 double *__restrict__ len,
                                                 double *__restrict__ price,
                                                 double *__restrict__ S,
                                                 uint8_t *__restrict__ choice,
                                                 uint32_t *__restrict__ count,
                                                 const int32_t *__restrict__ sigma,
                                                 const double *__restrict__ demand,
                                                 double *__restrict__ demand1n,
                                                 double *__restrict__ demand1t,
                                                 double *__restrict__ demand2,
                                                 double *__restrict__ demand2t, PlanStrides ps)
{
    len = of_plan(len, ps.state);
    price = of_plan(price, ps.state);
    S = of_plan(S, ps.state);
    choice = of_plan(choice, ps.state);
    count = of_plan(count, ps.state);
    demand = of_plan(demand, ps.demand);
    demand1n = of_plan(demand1n, ps.state);
    demand1t = of_plan(demand1t, ps.state);
    demand2 = of_plan(demand2, ps.state);
    demand2t = of_plan(demand2t, ps.state);
    const int stride = gridDim.x * blockDim.x;
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    // the library's own copies of the demands: by id (aligned, padded) and in sigma order for
    // the octets and strips, and by id and by sigma number in the window-transposed order the
    // tile phase reads
    for (int k = tid; k < K; k += stride) {
        const double dk = demand[k];
        demand1n[k] = dk;
        demand1t[tile_demand_index(k)] = dk;
        const int sg = sigma[k];
        if (sg >= 0) {
            demand2[sg] = dk;
            demand2t[tile_demand_index(sg)] = dk;
        }
    }
    // lengths start at 1, or at the caller's values (warm start; given by link id); len and S
    // are kept by position in the flat order of the rows, the price by link id
    for (int e = tid; e < E; e += stride) {
        const double l_e = len_in ? len_in[e] : 1.0;
        price[e] = cost_max ? l_e : l_e * invcap[e];
        len[e] = len_in ? len_in[pos_link[e]] : 1.0;      // here e is a position
        S[e] = 0.0;
    }
    for (int p = tid; p < P; p += stride) count[p] = 0u;
    if (tid == 0) choice[K] = 0u;   // slot K is read (never used) by padding pairs
}

// link lengths after the last iteration, back in link id order
__global__ __launch_bounds__(kBlock) void k_export_len(int E, const int32_t *__restrict__ pos_link,
                                                       const double *__restrict__ len,
                                                       double *__restrict__ len_out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < E) len_out[pos_link[i]] = len[i];
}

template <int L, int LMAX, bool MAXC, bool EXT>
__global__ __launch_bounds__(kBlock) void k_argmin(int K, const int32_t *__restrict__ cp,
                                                   const int32_t *__restrict__ lp,
                                                   const int32_t *__restrict__ pl,
                                                   const double *__restrict__ price,
                                                   uint8_t *__restrict__ choice,
                                                   uint32_t *__restrict__ count,
                                                   const int32_t *__restrict__ sigma,
                                                   uint8_t *__restrict__ choice2, PlanStrides ps)
{
    if constexpr (EXT) {      // a batch (blockIdx.y is the plan) or a solve that may stop early
        if (stopped(ps)) return;
        price = of_plan(price, ps.state);
        choice = of_plan(choice, ps.row);
        count = of_plan(count, ps.state);
        choice2 = of_plan(choice2, ps.state);
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    argmin_phase<L, LMAX, MAXC>(K, cp, lp, pl, price, choice, count, sigma, choice2, wave,
                                n_waves, lane);
}

// Record path-cost gather + argmin: one wave per 4 KiB record of the forward CSR.  The wave
// gathers the prices of the record's link table (the only access that leaves the record)
// into LDS, copies the body of the record into LDS with three 16-byte loads per lane, and
// then L lanes per commodity add S prices per candidate (8-bit table indices) from LDS in CSR
// order -- padding slots read +0.0 -- and reduce (cost, index) across the group.  The sums are the same IEEE operations in
// the same order as in the untiled kernel.
constexpr int kRecWaves = 4;     // independent waves per workgroup

// Orders the LDS accesses of one wave: a wave's LDS operations execute in issue order, so the
// lanes of a wave can exchange data through LDS once the compiler keeps the accesses in order.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Cost of the four candidates of one quad: w[i] holds the table indices of step i of four
// consecutive candidates, one byte each; the prices come from the wave's price slots in LDS
// (short paths read +0.0, absent candidates start at +inf).  Returns the minimum of the quad and
// the lowest candidate that holds it.  The sums are the same IEEE operations in the same order
// as in the untiled kernel (0 + p is p: the sum starts at the first price).
template <int S, bool MAXC>
__device__ __forceinline__ void scan_quad(const double *s_price, const uint32_t *w, double &m4,
                                          int &i4)
{
    double cst[4];
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4) {
        cst[c4] = s_price[(w[0] >> (8 * c4)) & 0xFFu];
#pragma unroll
        for (int i = 1; i < S; ++i) {
            const double pe = s_price[(w[i] >> (8 * c4)) & 0xFFu];
            if constexpr (MAXC) cst[c4] = (pe > cst[c4]) ? pe : cst[c4];
            else cst[c4] = cst[c4] + pe;
        }
    }
    m4 = fast_min_f64(fast_min_f64(cst[0], cst[1]), fast_min_f64(cst[2], cst[3]));
    i4 = cst[0] == m4 ? 0 : (cst[1] == m4 ? 1 : (cst[2] == m4 ? 2 : 3));
}

// The same for a quad in the two-by-two product shape (step 0 and 1: candidates 0, 1 and 2, 3
// read the same slot; step 2: all four; step 3 and 4: candidates 0, 2 and 1, 3): nine prices
// instead of twenty, and the partial sums the candidates share are formed once.  Every
// candidate's cost is still ((((p0 + p1) + p2) + p3) + p4 in that order.
template <bool MAXC>
__device__ __forceinline__ void scan_quad_product(const double *s_price, const uint32_t *w,
                                                  double &m4, int &i4)
{
    auto op = [](double acc, double pe) {
        if constexpr (MAXC) return (pe > acc) ? pe : acc;
        else return acc + pe;
    };
    const double a0 = s_price[w[0] & 0xFFu], a2 = s_price[(w[0] >> 16) & 0xFFu];
    const double b0 = s_price[w[1] & 0xFFu], b2 = s_price[(w[1] >> 16) & 0xFFu];
    const double c = s_price[w[2] & 0xFFu];
    const double d0 = s_price[w[3] & 0xFFu], d1 = s_price[(w[3] >> 8) & 0xFFu];
    const double e0 = s_price[w[4] & 0xFFu], e1 = s_price[(w[4] >> 8) & 0xFFu];
    const double t0 = op(op(a0, b0), c);
    const double t2 = op(op(a2, b2), c);
    double cst[4];
    cst[0] = op(op(t0, d0), e0);
    cst[1] = op(op(t0, d1), e1);
    cst[2] = op(op(t2, d0), e0);
    cst[3] = op(op(t2, d1), e1);
    m4 = fast_min_f64(fast_min_f64(cst[0], cst[1]), fast_min_f64(cst[2], cst[3]));
    i4 = cst[0] == m4 ? 0 : (cst[1] == m4 ? 1 : (cst[2] == m4 ? 2 : 3));
}

template <int L, int S, bool MAXC, bool TWO, bool EXT>
__global__ __launch_bounds__(kWave *kRecWaves) void k_argmin_rec(int n_records,
                                                      const uint8_t *__restrict__ records,
                                                      const double *__restrict__ price,
                                                      uint8_t *__restrict__ choice,
                                                      uint32_t *__restrict__ count,
                                                      uint8_t *__restrict__ choice2,
                                                      PlanStrides ps)
{
    if constexpr (EXT) {      // a batch (blockIdx.y is the plan) or a solve that may stop early
        if (stopped(ps)) return;
        price = of_plan(price, ps.state);
        choice = of_plan(choice, ps.row);
        count = of_plan(count, ps.state);
        choice2 = of_plan(choice2, ps.state);
    }
    // LDS, one private slice per wave: the body of the record (everything after the link
    // table) followed by the price table.  The waves of a workgroup never synchronise with
    // each other.
    constexpr int kBody = kRecBytes - kRecTable;
    __shared__ __align__(16) uint8_t s_all[kRecWaves * (kBody + 8 * kRecPriceSlots)];
    uint8_t *s_rec = s_all + (threadIdx.x >> 6) * (kBody + 8 * kRecPriceSlots);
    double *s_price = reinterpret_cast<double *>(s_rec + kBody);
    constexpr int kGroups = kWave / L;
    constexpr int kLoads = kBody / 1024;
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / L;
    const int j = lane % L;
    const int n_waves = gridDim.x * kRecWaves;
    // the record index is the same in all lanes; in a scalar register the tests on it below
    // are scalar branches
    int rec = __builtin_amdgcn_readfirstlane(blockIdx.x * kRecWaves + (threadIdx.x >> 6));
    if (rec >= n_records) return;
    // Three requests are kept in flight per wave, each issued one record ahead of its use: the
    // link table of the record after the next (one 16-byte load per lane), the prices of the
    // next record's links (four gathers per lane, addressed straight from the table registers:
    // the table is stored so that gather c of lane l is link 64c + l), and the body of the
    // next record.  Past the wave's last record nothing is requested: the records are
    // streamed past the L2, so a redundant request would cost HBM bandwidth like a real one.
    auto table_of = [&](int r) {
        return stream_load(reinterpret_cast<const u32x4 *>(records + size_t(r) * kRecBytes) +
                           lane);
    };
    u32x4 tab = table_of(rec);
    u32x4 body[kLoads];
    double pr[4];
    pr[0] = price[tab.x];
    pr[1] = price[tab.y];
    pr[2] = price[tab.z];
    pr[3] = price[tab.w];
    if (rec + n_waves < n_records) tab = table_of(rec + n_waves);
    {
        const u32x4 *src =
            reinterpret_cast<const u32x4 *>(records + size_t(rec) * kRecBytes + kRecTable);
#pragma unroll
        for (int it = 0; it < kLoads; ++it) body[it] = stream_load(src + it * kWave + lane);
    }
    for (; rec < n_records; rec += n_waves) {           // wave-uniform
        wave_lds_sync();                                // the previous record is done with LDS
#pragma unroll
        for (int it = 0; it < kLoads; ++it)
            reinterpret_cast<u32x4 *>(s_rec)[it * kWave + lane] = body[it];
#pragma unroll
        for (int q = 0; q < 4; ++q) s_price[lane + q * kWave] = pr[q];
        wave_lds_sync();
        const int k0 = *reinterpret_cast<const int32_t *>(s_rec);
        const int p0 = *reinterpret_cast<const int32_t *>(s_rec + 4);
        const uint16_t *h16 = reinterpret_cast<const uint16_t *>(s_rec + 8);
        const int nk = h16[0], nl = h16[2], npad_rec = h16[7];
        const uint16_t *cp16 = reinterpret_cast<const uint16_t *>(s_rec + h16[3]);
        const uint8_t *loc8 = s_rec + h16[4];
        const int32_t *sig = reinterpret_cast<const int32_t *>(s_rec + h16[5]);
        const uint16_t *cq16 = reinterpret_cast<const uint16_t *>(s_rec + h16[6]);
        if (lane == 0) {                             // after the table prices, in LDS order
            s_price[nl] = 0.0;                       // pads short paths
            s_price[nl + 1] = __builtin_inf();       // first step of padding candidates
        }
        // the next record: its prices, its body, and the table of the one after it
        if (rec + n_waves < n_records) {
            pr[0] = price[tab.x];
            pr[1] = price[tab.y];
            pr[2] = price[tab.z];
            pr[3] = price[tab.w];
            if (rec + 2 * n_waves < n_records) tab = table_of(rec + 2 * n_waves);
            const u32x4 *src = reinterpret_cast<const u32x4 *>(
                records + size_t(rec + n_waves) * kRecBytes + kRecTable);
#pragma unroll
            for (int it = 0; it < kLoads; ++it) body[it] = stream_load(src + it * kWave + lane);
        }
        wave_lds_sync();
        const int wstride = npad_rec >> 2;
        const int rounds = (nk + kGroups - 1) / kGroups;
        for (int r = 0; r < rounds; ++r) {        // wave-uniform: all lanes reach the reduction
            const int c = r * kGroups + g;
            double best = __builtin_inf();
            int bj = 0x7FFFFFFF;
            int p_lo = 0, np = 0, q_lo = 0;
            if (c < nk) {
                p_lo = cp16[c];
                np = cp16[c + 1] - p_lo;
                q_lo = cq16[c];
            }
            if constexpr (TWO) {
                // no commodity has more than 8 L candidates: lane j scans the quads j and
                // j + L.  Both are fetched unconditionally (a quad that does not exist re-reads
                // the commodity's first one and is dropped), so the index words and the prices
                // of the two quads are in flight together.
                const int ja = 4 * j, jb = 4 * j + 4 * L;
                const bool va = ja < np, vb = jb < np;
                const uint32_t *lpa =
                    reinterpret_cast<const uint32_t *>(loc8 + q_lo + (va ? ja : 0));
                const uint32_t *lpb =
                    reinterpret_cast<const uint32_t *>(loc8 + q_lo + (vb ? jb : 0));
                uint32_t wa[S], wb[S];
#pragma unroll
                for (int i = 0; i < S; ++i) {
                    wa[i] = lpa[i * wstride];
                    wb[i] = lpb[i * wstride];
                }
                double ma, mb;
                int ia, ib;
                scan_quad<S, MAXC>(s_price, wa, ma, ia);
                scan_quad<S, MAXC>(s_price, wb, mb, ib);
                if (va) bj = ja;
                if (va && ma < best) {
                    best = ma;
                    bj = ja + ia;
                }
                if (vb && mb < best) {
                    best = mb;
                    bj = jb + ib;
                }
            } else {
                if (4 * j < np) bj = 4 * j;
                // lane j scans the quads j, j+L, ... of the commodity
                for (int jq = 4 * j; jq < np; jq += 4 * L) {
                    const uint32_t *lp = reinterpret_cast<const uint32_t *>(loc8 + q_lo + jq);
                    uint32_t w[S];
#pragma unroll
                    for (int i = 0; i < S; ++i) w[i] = lp[i * wstride];
                    double m4;
                    int i4;
                    scan_quad<S, MAXC>(s_price, w, m4, i4);
                    if (m4 < best) {
                        best = m4;
                        bj = jq + i4;
                    }
                }
            }
            bj = group_argmin_two_pass<L>(best, bj);
            if (c < nk && j == 0) {
                choice[k0 + c] = static_cast<uint8_t>(bj);
                const int sg = sig[c];
                if (sg >= 0) choice2[sg] = static_cast<uint8_t>(bj);   // copy in sigma order
                // counts are kept only when the choices are not logged per iteration
                if (count != nullptr) count[p0 + p_lo + bj] += 1u;
            }
        }
    }
}

// FOLD (adaptive step): the step of the iteration before has not been applied to the stored
// state when this launch starts.  The scanning workgroups take, for every link of a record's
// table, the length before that step, the normalised load and 1/capacity (all by link id) and
// form the price with the operations of the step itself, in the same order -- the same bits the
// step writes; the first f.apply_blocks workgroups apply the step to the stored state meanwhile
// (nothing they write is read by this launch).
template <bool FOLD>
struct FoldParam {
    typedef NoFold type;
};
template <>
struct FoldParam<true> {
    typedef FoldArgs type;
};

// the largest normalised load of the fabric from the maxima of the blocks; 0 when there was no
// traffic (the step then ends the solve, and every price stays what it was)
__device__ __forceinline__ double fold_sigma(const AdApplyArgs &ap, int lane)
{
    const double umax = wave_max(max_of_strided<kWave>(ap.block_max_u, ap.n_u_blocks, lane));
    return umax > 0.0 ? 1.0 / umax : 0.0;
}

// what a price is made of: plain, the price itself; folded, length, load and 1/capacity
template <bool FOLD, bool MAXC>
struct PriceTerms {
    double v[4];
    __device__ __forceinline__ void fetch(int q, uint32_t id, const double *price, const NoFold &)
    {
        v[q] = price[id];
    }
    __device__ __forceinline__ double priced(int q, double, double) const { return v[q]; }
};
template <bool MAXC>
struct PriceTerms<true, MAXC> {
    double v[4], u[4], c[4];
    __device__ __forceinline__ void fetch(int q, uint32_t id, const double *, const FoldArgs &f)
    {
        v[q] = f.len_id[id];
        u[q] = f.u_id[id];
        if constexpr (!MAXC) c[q] = f.invcap[id];
    }
    __device__ __forceinline__ double priced(int q, double sigma, double eps) const
    {
        const double su = sigma * u[q];
        const double t1 = eps * su;
        const double t2 = 1.0 + t1;
        const double ln = v[q] * t2;
        if constexpr (MAXC) return ln;
        else return ln * c[q];
    }
};

// The same for records with a lane-major body: the three 16-byte loads of a lane return its own
// twelve words (the table indices of its two quads, five steps each, and two words about its
// commodity and the record), so the body never goes through LDS -- only the prices do.  The
// price slots kRecZeroSlot / kRecInfSlot hold +0.0 / +inf for short paths and absent
// candidates.  One scan round per record: a record has at most 64 / L commodities.
template <int L, int S, bool MAXC, bool T16, bool EXT, bool FOLD = false>
__global__ __launch_bounds__(kWave *kRecWaves) void k_argmin_recl(int n_records, int around_l2,
                                                       const uint8_t *__restrict__ records,
                                                       const double *__restrict__ price,
                                                       uint8_t *__restrict__ choice,
                                                       uint32_t *__restrict__ count,
                                                       uint8_t *__restrict__ choice2,
                                                       PlanStrides ps,
                                                       typename FoldParam<FOLD>::type f)
{
    static_assert(L >= 2 && L <= 16 && S <= kRecLaneSteps,
                  "lane-major records: 2 to 16 lanes per commodity, five steps");
    static_assert(!FOLD || EXT, "the folded step belongs to a solve that may stop early");
    int bx = blockIdx.x, scan_blocks = gridDim.x;
    if constexpr (FOLD) {
        if (bx < f.apply_blocks) {                               // block-uniform
            __shared__ double red[16];
            ad_apply_block<MAXC>(f.ap, bx, red);
            return;
        }
        bx -= f.apply_blocks;
        scan_blocks -= f.apply_blocks;
    }
    int32_t stop_now = 0;
    if constexpr (EXT) {      // a batch (blockIdx.y is the plan) or a solve that may stop early
        stop_now = stop_word(ps);            // tested below, once the first loads are under way
        if constexpr (!FOLD) {               // (a folded step belongs to a single plan)
            price = of_plan(price, ps.state);
            choice = of_plan(choice, ps.row);
            count = of_plan(count, ps.state);
            choice2 = of_plan(choice2, ps.state);
        }
    }
    // T16: the link table is 256 uint16 (8 bytes per lane) and the record 3.5 KiB
    constexpr int kTab = T16 ? kRecTable16 : kRecTable;
    constexpr int kRec = T16 ? kRecBytes16 : kRecBytes;
    __shared__ double s_all[kRecWaves * kRecPriceSlots];
    double *s_price = s_all + (threadIdx.x >> 6) * kRecPriceSlots;
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / L;
    const int j = lane % L;
    const int n_waves = scan_blocks * kRecWaves;
    int rec = __builtin_amdgcn_readfirstlane(bx * kRecWaves + (threadIdx.x >> 6));
    if (rec >= n_records) return;
    // in flight while a record is scanned: the table of the record after the next, the prices
    // and the body of the next one; nothing is requested past the wave's last record
    struct Ids {
        uint32_t a, b, c, d;        // links lane, 64 + lane, 128 + lane, 192 + lane of the table
    };
    // Records that together exceed the L2 are read around it (loads with the sc0 and sc1 bits:
    // a buffer load for the table, global loads for the body; around_l2 is the same for the
    // whole launch): 59 MB per launch on the 64-node fabric
    // would otherwise push out what the reduce and update kernels find there again in the next
    // iteration (their 30 MB fit the L2, the records never will).  A record is one buffer: the
    // hardware drops loads beyond its end.
    constexpr int kAroundL2 = 1 | 16;            // cache policy bits of the buffer loads: sc0, sc1
    auto record = [&](int r) {
        return __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t *>(records + size_t(r) * kRec), 0, kRec, 0x00020000);
    };
    auto table_of = [&](int r) {
        Ids ids;
        if constexpr (T16) {
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            const u32x2 v =
                around_l2 ? __builtin_amdgcn_raw_buffer_load_b64(record(r), lane * 8, 0, kAroundL2)
                          : __builtin_amdgcn_raw_buffer_load_b64(record(r), lane * 8, 0, 0);
            ids.a = v.x & 0xFFFFu;
            ids.b = v.x >> 16;
            ids.c = v.y & 0xFFFFu;
            ids.d = v.y >> 16;
        } else {
            const u32x4 v =
                around_l2
                    ? __builtin_amdgcn_raw_buffer_load_b128(record(r), lane * 16, 0, kAroundL2)
                    : __builtin_amdgcn_raw_buffer_load_b128(record(r), lane * 16, 0, 0);
            ids.a = v.x;
            ids.b = v.y;
            ids.c = v.z;
            ids.d = v.w;
        }
        return ids;
    };
    auto body_of = [&](int r, u32x4 (&buf)[3]) {
        const __amdgpu_buffer_rsrc_t rs = record(r);
        if (around_l2) {
            // the body as pairs of 8-byte relaxed loads at system scope: global loads with the
            // sc0 and sc1 bits (there is no 16-byte load of that kind), 0.8 us per launch faster
            // on the 64-node fabric than buffer loads with the same bits
            const unsigned long long *src = reinterpret_cast<const unsigned long long *>(
                records + size_t(r) * kRec + kTab);
#pragma unroll
            for (int it = 0; it < 3; ++it) {
                const unsigned long long lo = __hip_atomic_load(
                    src + it * 128 + lane * 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                const unsigned long long hi = __hip_atomic_load(
                    src + it * 128 + lane * 2 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                buf[it].x = static_cast<uint32_t>(lo);
                buf[it].y = static_cast<uint32_t>(lo >> 32);
                buf[it].z = static_cast<uint32_t>(hi);
                buf[it].w = static_cast<uint32_t>(hi >> 32);
            }
        } else {
#pragma unroll
            for (int it = 0; it < 3; ++it)
                buf[it] = __builtin_amdgcn_raw_buffer_load_b128(
                    rs, kTab + it * 1024 + lane * 16, 0, 0);
        }
    };
    Ids tab = table_of(rec);
    [[maybe_unused]] double sigma = 0.0, eps = 0.0;
    if constexpr (FOLD) {                    // (the maxima travel together with the table)
        sigma = fold_sigma(f.ap, lane);
        eps = f.ap.eps;
    }
    u32x4 body[3];
    PriceTerms<FOLD, MAXC> pr;
    pr.fetch(0, tab.a, price, f);
    pr.fetch(1, tab.b, price, f);
    pr.fetch(2, tab.c, price, f);
    pr.fetch(3, tab.d, price, f);
    if (rec + n_waves < n_records) tab = table_of(rec + n_waves);
    body_of(rec, body);
    if constexpr (EXT)
        if (stop_now != 0) return;                      // nothing has been written yet
    for (; rec < n_records; rec += n_waves) {           // wave-uniform
        wave_lds_sync();                                // the previous record is done with LDS
#pragma unroll
        for (int q = 0; q < 4; ++q) s_price[lane + q * kWave] = pr.priced(q, sigma, eps);
        if (lane == 0) {                             // after the table prices, in LDS order
            s_price[kRecZeroSlot] = 0.0;             // pads short paths
            s_price[kRecInfSlot] = __builtin_inf();  // first step of absent candidates
        }
        // this lane's words leave the load registers, which take the next record
        const uint32_t w[10] = {body[0].x, body[0].y, body[0].z, body[0].w, body[1].x,
                                body[1].y, body[1].z, body[1].w, body[2].x, body[2].y};
        const uint32_t meta = body[2].z;
        const int32_t own = static_cast<int32_t>(body[2].w);
        if (rec + n_waves < n_records) {
            pr.fetch(0, tab.a, price, f);
            pr.fetch(1, tab.b, price, f);
            pr.fetch(2, tab.c, price, f);
            pr.fetch(3, tab.d, price, f);
            if (rec + 2 * n_waves < n_records) tab = table_of(rec + 2 * n_waves);
            body_of(rec + n_waves, body);
        }
        wave_lds_sync();
        const int np = static_cast<int>(meta & 0xFFu);
        const int p_lo = static_cast<int>(meta >> 8);
        const int ja = 4 * j, jb = 4 * j + 4 * L;
        double ma, mb;
        int ia, ib;
        // which quads of the record have the two-by-two product shape: lane 1 of slot 2
        const uint32_t product =
            S == kRecLaneSteps ? static_cast<uint32_t>(__builtin_amdgcn_readlane(own, 2 * L + 1)) : 0u;
        if (product & 1u) scan_quad_product<MAXC>(s_price, w, ma, ia);            // wave-uniform
        else scan_quad<S, MAXC>(s_price, w, ma, ia);
        if (product & 2u) scan_quad_product<MAXC>(s_price, w + kRecLaneSteps, mb, ib);
        else scan_quad<S, MAXC>(s_price, w + kRecLaneSteps, mb, ib);
        // the strict `<` scan in candidate order: quad A first; absent candidates cost +inf
        double best = __builtin_inf();
        int bj = ja < np ? ja : 0x7FFFFFFF;
        if (ja < np && ma < best) {
            best = ma;
            bj = ja + ia;
        }
        if (jb < np && mb < best) {
            best = mb;
            bj = jb + ib;
        }
        bj = group_argmin_two_pass<L>(best, bj);
        // the record's own words: k0 | nk << 24 in lane 1, p0 in lane L + 1
        const int k0 = __builtin_amdgcn_readlane(own, 1) & 0xFFFFFF;
        if (np > 0 && j == 0) {
            choice[k0 + g] = static_cast<uint8_t>(bj);
            if (own >= 0) choice2[own] = static_cast<uint8_t>(bj);   // copy in sigma order
        }
        // counts are kept only when the choices are not logged per iteration
        if (count != nullptr) {
            const int p0 = __builtin_amdgcn_readlane(own, L + 1);
            if (np > 0 && j == 0) count[p0 + p_lo + bj] += 1u;
        }
    }
}

// The same for records whose bodies live in a dictionary: a wave walks a run of records that
// share one body.  It fetches the body once (three cached 16-byte loads per lane: the few
// bodies of a fabric stay in the L2) and per record only its 16 bytes per lane: four 16-bit
// link table entries, the lane's own word (sigma, or the record's first commodity / first
// candidate) and the body number.  In flight while a record is scanned: the 16 bytes of the
// record after the next and the prices of the next one.
template <int L, int S, bool MAXC, bool EXT, bool FOLD = false>
__global__ __launch_bounds__(kWave *kRecWaves) void k_argmin_recd(int n_chunks, int around_l2,
                                                       const int4 *__restrict__ chunks,
                                                       const uint8_t *__restrict__ records,
                                                       const u32x4 *__restrict__ bodies,
                                                       const double *__restrict__ price,
                                                       uint8_t *__restrict__ choice,
                                                       uint32_t *__restrict__ count,
                                                       uint8_t *__restrict__ choice2,
                                                       PlanStrides ps,
                                                       typename FoldParam<FOLD>::type f)
{
    static_assert(L >= 2 && L <= 16 && S <= kRecLaneSteps,
                  "lane-major records: 2 to 16 lanes per commodity, five steps");
    static_assert(!FOLD || EXT, "the folded step belongs to a solve that may stop early");
    int bx = blockIdx.x;
    if constexpr (FOLD) {
        if (bx < f.apply_blocks) {                               // block-uniform
            __shared__ double red[16];
            ad_apply_block<MAXC>(f.ap, bx, red);
            return;
        }
        bx -= f.apply_blocks;
    }
    int32_t stop_now = 0;
    if constexpr (EXT) {      // a batch (blockIdx.y is the plan) or a solve that may stop early
        stop_now = stop_word(ps);            // tested below, once the first loads are under way
        if constexpr (!FOLD) {               // (a folded step belongs to a single plan)
            price = of_plan(price, ps.state);
            choice = of_plan(choice, ps.row);
            count = of_plan(count, ps.state);
            choice2 = of_plan(choice2, ps.state);
        }
    }
    __shared__ double s_all[kRecWaves * kRecPriceSlots];
    double *s_price = s_all + (threadIdx.x >> 6) * kRecPriceSlots;
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / L;
    const int j = lane % L;
    const int chunk = __builtin_amdgcn_readfirstlane(bx * kRecWaves + (threadIdx.x >> 6));
    if (chunk >= n_chunks) return;
    const int4 ck = chunks[chunk];
    int rec = __builtin_amdgcn_readfirstlane(ck.x);
    const int end = rec + __builtin_amdgcn_readfirstlane(ck.y);
    const int body_id = __builtin_amdgcn_readfirstlane(ck.z);
    constexpr int kAroundL2 = 1 | 16;            // cache policy bits of the buffer loads: sc0, sc1
    auto head_of = [&](int r) {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t *>(records + size_t(r) * kRecBytesDict), 0, kRecBytesDict,
            0x00020000);
        return around_l2 ? __builtin_amdgcn_raw_buffer_load_b128(rs, lane * 16, 0, kAroundL2)
                         : __builtin_amdgcn_raw_buffer_load_b128(rs, lane * 16, 0, 0);
    };
    u32x4 head = head_of(rec);
    // the body of the run: this lane's words 0..10
    const u32x4 *bsrc = bodies + size_t(body_id) * (kRecBodyBytes / 16) + lane;
    const u32x4 b0 = bsrc[0], b1 = bsrc[kWave], b2 = bsrc[2 * kWave];
    const uint32_t w[10] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w, b2.x, b2.y};
    const uint32_t meta = b2.z;
    // which quads of the body have the two-by-two product shape (the same word in all lanes)
    const uint32_t product = S == kRecLaneSteps ? __builtin_amdgcn_readfirstlane(b2.w) : 0u;
    const int np = static_cast<int>(meta & 0xFFu);
    const int p_lo = static_cast<int>(meta >> 8);
    const int ja = 4 * j, jb = 4 * j + 4 * L;
    [[maybe_unused]] double sigma = 0.0, eps = 0.0;
    if constexpr (FOLD) {                    // (the maxima travel together with head and body)
        sigma = fold_sigma(f.ap, lane);
        eps = f.ap.eps;
    }
    PriceTerms<FOLD, MAXC> pr;
    pr.fetch(0, head.x & 0xFFFFu, price, f);
    pr.fetch(1, head.x >> 16, price, f);
    pr.fetch(2, head.y & 0xFFFFu, price, f);
    pr.fetch(3, head.y >> 16, price, f);
    int32_t own_next = static_cast<int32_t>(head.z);
    if (rec + 1 < end) head = head_of(rec + 1);
    if constexpr (EXT)
        if (stop_now != 0) return;                      // nothing has been written yet
    for (; rec < end; ++rec) {                          // wave-uniform
        wave_lds_sync();                                // the previous record is done with LDS
#pragma unroll
        for (int q = 0; q < 4; ++q) s_price[lane + q * kWave] = pr.priced(q, sigma, eps);
        if (lane == 0) {                             // after the table prices, in LDS order
            s_price[kRecZeroSlot] = 0.0;             // pads short paths
            s_price[kRecInfSlot] = __builtin_inf();  // first step of absent candidates
        }
        const int32_t own = own_next;
        if (rec + 1 < end) {
            pr.fetch(0, head.x & 0xFFFFu, price, f);
            pr.fetch(1, head.x >> 16, price, f);
            pr.fetch(2, head.y & 0xFFFFu, price, f);
            pr.fetch(3, head.y >> 16, price, f);
            own_next = static_cast<int32_t>(head.z);
            if (rec + 2 < end) head = head_of(rec + 2);
        }
        wave_lds_sync();
        double ma, mb;
        int ia, ib;
        if (product & 1u) scan_quad_product<MAXC>(s_price, w, ma, ia);            // wave-uniform
        else scan_quad<S, MAXC>(s_price, w, ma, ia);
        if (product & 2u) scan_quad_product<MAXC>(s_price, w + kRecLaneSteps, mb, ib);
        else scan_quad<S, MAXC>(s_price, w + kRecLaneSteps, mb, ib);
        // the strict `<` scan in candidate order: quad A first; absent candidates cost +inf
        double best = __builtin_inf();
        int bj = ja < np ? ja : 0x7FFFFFFF;
        if (ja < np && ma < best) {
            best = ma;
            bj = ja + ia;
        }
        if (jb < np && mb < best) {
            best = mb;
            bj = jb + ib;
        }
        bj = group_argmin_two_pass<L>(best, bj);
        // the record's own words: k0 | nk << 24 in lane 1, p0 in lane L + 1; a slot beyond the
        // record's commodities (the body may hold more than this record does) writes nothing
        const int k0nk = __builtin_amdgcn_readlane(own, 1);
        const int k0 = k0nk & 0xFFFFFF;
        const bool live = np > 0 && g < static_cast<int>(static_cast<uint32_t>(k0nk) >> 24);
        if (live && j == 0) {
            choice[k0 + g] = static_cast<uint8_t>(bj);
            if (own >= 0) choice2[own] = static_cast<uint8_t>(bj);   // copy in sigma order
        }
        // counts are kept only when the choices are not logged per iteration
        if (count != nullptr) {
            const int p0 = __builtin_amdgcn_readlane(own, L + 1);
            if (live && j == 0) count[p0 + p_lo + bj] += 1u;
        }
    }
}

// Split fractions from the per-iteration choice log: one lane per commodity walks its column
// of the log and counts in LDS (a padded row per lane, so lanes hit different banks).
__global__ __launch_bounds__(kWave) void k_histogram(int K, int iters, int pmax, size_t stride,
                                                     const uint8_t *__restrict__ log,
                                                     const int32_t *__restrict__ cp,
                                                     double *__restrict__ splits, PlanStrides ps)
{
    log = of_plan(log, ps.row);
    splits = of_plan(splits, ps.splits);
    extern __shared__ uint32_t s_cnt[];
    const int lane = threadIdx.x;
    const int k = blockIdx.x * kWave + lane;
    // counter j of this lane's commodity is word j * 64 + lane: whatever the lanes choose,
    // lanes l and l + 32 share a bank and nobody else does
    uint32_t *mine = s_cnt + lane;
    for (int j = 0; j < pmax; ++j) mine[j * kWave] = 0u;
    if (k < K) {
        const uint8_t *col = log + k;
        // counts are whole numbers, so their order is free: the choices of sixteen iterations
        // are requested side by side and counted with LDS additions that return nothing (no
        // read-modify-write chain from one iteration to the next)
        auto bump = [&](int c) {
            (void)__hip_atomic_fetch_add(mine + c * kWave, 1u, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_WORKGROUP);
        };
        int t = 0;
        for (; t + 16 <= iters; t += 16) {
            uint8_t c[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) c[u] = col[size_t(t + u) * stride];
#pragma unroll
            for (int u = 0; u < 16; ++u) bump(c[u]);
        }
        for (; t < iters; ++t) bump(col[size_t(t) * stride]);
        const int p0 = cp[k], np = cp[k + 1] - p0;
        const double T = static_cast<double>(iters);
        for (int j = 0; j < np; ++j) splits[p0 + j] = static_cast<double>(mine[j * kWave]) / T;
    }
}

struct ReduceArgs {
    int n_passes, n_schunks, n_tile_items, n_tile_waves, n_strip_items, n_strip_waves;
    const uint32_t *strip_base, *strip_mask;
    const uint64_t *strip_pres;
    const int32_t *strip_slot;
    const double *demand1n;
    const int32_t *tile_desc;
    const uint32_t *tile_mask;
    const uint8_t *tile_pres;
    const double *demand1t, *demand2t;
    const int32_t *pass_first_slot;
    const uint32_t *oct_base, *oct_mask;
    const int32_t *schunk_begin, *schunk_end, *schunk_slot;
    const uint32_t *single_pair;
    uint32_t pad_comm;
    const uint8_t *choice, *choice2;
    const double *demand, *demand2;
    double *partial;
    PlanStrides ps;
};

template <int MODE, bool EXT>
__global__ __launch_bounds__(kBlock) void k_load_reduce(ReduceArgs a)
{
    if constexpr (EXT) {      // a batch (blockIdx.y is the plan) or a solve that may stop early
        if (stopped(a.ps)) return;
        a.demand1n = of_plan(a.demand1n, a.ps.state);
        a.demand1t = of_plan(a.demand1t, a.ps.state);
        a.demand2t = of_plan(a.demand2t, a.ps.state);
        a.demand2 = of_plan(a.demand2, a.ps.state);
        a.choice2 = of_plan(a.choice2, a.ps.state);
        a.partial = of_plan(a.partial, a.ps.state);
        a.choice = of_plan(a.choice, a.ps.row);
        a.demand = of_plan(a.demand, a.ps.demand);
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    // the wave pool is split between the tile items, the strip items and the octet passes in
    // proportion to their numbers
    if (wave < a.n_tile_waves)
        reduce_tile_phase<MODE>(a.n_tile_items, a.tile_desc, a.tile_mask, a.tile_pres, a.choice,
                                a.demand1t, a.choice2, a.demand2t, a.partial, wave, a.n_tile_waves,
                                lane);
    else if (wave < a.n_tile_waves + a.n_strip_waves)
        reduce_strip_phase<MODE>(a.n_strip_items, a.strip_base, a.strip_pres, a.strip_mask,
                                 a.strip_slot, a.choice, a.demand1n, a.choice2, a.demand2,
                                 a.partial, wave - a.n_tile_waves, a.n_strip_waves, lane);
    else
        reduce_flat_phase<MODE>(0, a.n_passes, a.pass_first_slot, a.oct_base, a.oct_mask,
                                a.choice, a.demand1n, a.choice2, a.demand2, a.partial, 0,
                                wave - a.n_tile_waves - a.n_strip_waves,
                                n_waves - a.n_tile_waves - a.n_strip_waves, lane);
    // single pairs (commodities with more than 32 candidates) are walked from the other end of
    // the wave pool
    reduce_phase<MODE, kSinglesPerLane>(a.n_schunks, a.schunk_begin, a.schunk_end, a.schunk_slot,
                                        a.single_pair, a.pad_comm, a.choice, a.demand, a.partial,
                                        wave, n_waves, lane);
}

// Link-load reduce and length update in one kernel, for topologies cut into link blocks: a
// workgroup owns the rows of a block, reduces their octets (a contiguous range of passes) into
// slot partials kept in LDS, and applies  S += u,  len *= 1 + eps*u/rho,  price = len/cap  to
// exactly those links.  len, S and 1/cap are stored by position, so the state of the block's
// links is requested with coalesced loads before the octets are walked and has arrived when
// the partials are complete.  Every wave leaves its maximum of S in scalars[1 + wave id].
struct FusedArgs {
    const int32_t *blk_desc;
    const int32_t *pass_first_slot;
    const uint32_t *oct_base, *oct_mask;
    const int32_t *pos_link, *pos_slot_ptr;
    const uint8_t *choice, *choice2;
    const double *demand1n, *demand2;      // the library's padded copies, by id and by sigma
    const double *invcap_pos;
    double *len, *price, *S, *scalars;
    double eps;
    PlanStrides ps;
    int n_plans;
    double *u_pos, *u_id, *block_max_u;     // adaptive step only (u by position and by id)
};

struct LinkState {
    int e, c0, c1;
    double ic, s, l;
};

// ONLY_U (adaptive step): the update cannot be applied before the largest normalised load of
// the whole fabric is known, so the kernel stops at u = load / cap (by position, to a.u_pos) and
// leaves every wave's maximum of u in a.block_max_u for the kernel that applies the step.
template <bool MAXC, bool ONLY_U, bool EXT>
__global__ __launch_bounds__(kBlock) void k_reduce_update(FusedArgs a)
{
    __shared__ double s_part[kBlkMaxSlots];
    int32_t stop_now = 0;
    if constexpr (EXT) {      // a batch (blockIdx.y is the plan) or a solve that may stop early
        stop_now = stop_word(a.ps);          // tested below, once the first loads are under way
        if constexpr (!ONLY_U) {             // (the adaptive step belongs to a single plan)
            a.choice = of_plan(a.choice, a.ps.row);
            a.choice2 = of_plan(a.choice2, a.ps.state);
            a.demand1n = of_plan(a.demand1n, a.ps.state);
            a.demand2 = of_plan(a.demand2, a.ps.state);
            a.len = of_plan(a.len, a.ps.state);
            a.price = of_plan(a.price, a.ps.state);
            a.S = of_plan(a.S, a.ps.state);
            a.scalars = of_plan(a.scalars, a.ps.state);
        }
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int b = blockIdx.x;
    const int4 d4 = *reinterpret_cast<const int4 *>(a.blk_desc + 8 * b);
    const int i0 = d4.x, i1 = d4.y;             // positions of the block (at least one)
    const int p0 = d4.z, p1 = d4.w;             // its passes
    const int slot0 = a.blk_desc[8 * b + 4];
    const double invrho = a.scalars[0];
    const int row = threadIdx.x / kRowLanes;
    const int l = threadIdx.x % kRowLanes;
    constexpr int kRows = kBlock / kRowLanes;
    // positions past the end re-read the last one (so that every load is unconditional) and
    // are masked out when the update is applied
    auto fetch = [&](int i) {
        const int ic = i < i1 ? i : i1 - 1;
        LinkState st;
        st.e = a.pos_link[ic];
        st.c0 = a.pos_slot_ptr[ic] - slot0;
        st.c1 = a.pos_slot_ptr[ic + 1] - slot0;
        st.ic = a.invcap_pos[ic];
        st.s = a.S[ic];
        st.l = a.len[ic];
        return st;
    };
    double smax = 0.0;
    auto apply = [&](int i, const LinkState &st) {
        const bool valid = i < i1;
        const double load = row_partial_sum(st.c0, valid ? st.c1 : st.c0, l, s_part);
        if (valid && l == 0) {
            const double u = load * st.ic;
            if constexpr (ONLY_U) {
                a.u_pos[i] = u;
                a.u_id[st.e] = u;
                smax = fmax(smax, u);
            } else {
                const double s_new = st.s + u;
                a.S[i] = s_new;
                const double g = u * invrho;
                const double t1 = a.eps * g;
                const double t2 = 1.0 + t1;
                const double ln = st.l * t2;
                a.len[i] = ln;
                a.price[st.e] = MAXC ? ln : ln * st.ic;
                smax = fmax(smax, s_new);
            }
        }
    };
    const LinkState st0 = fetch(i0 + row);
    const LinkState st1 = fetch(i0 + row + kRows);
    if constexpr (EXT)
        if (stop_now != 0) return;           // (the same in every thread; nothing written yet)
    reduce_flat_phase<0>(p0, p1, a.pass_first_slot, a.oct_base, a.oct_mask, a.choice, a.demand1n,
                         a.choice2, a.demand2, s_part, slot0, wave, kBlock / kWave, lane);
    __syncthreads();
    apply(i0 + row, st0);
    apply(i0 + row + kRows, st1);
    for (int ibase = i0 + 2 * kRows; ibase < i1; ibase += kRows)         // block-uniform, rare
        apply(ibase + row, fetch(ibase + row));
    const double m = wave_max(smax);
    if constexpr (ONLY_U) {
        // one maximum per block: the kernel that applies the step folds them all
        __syncthreads();                                // the slots are free again
        if (lane == 0) s_part[wave] = m;
        __syncthreads();
        if (threadIdx.x == 0) {
            double mm = 0.0;
            for (int q = 0; q < kBlock / kWave; ++q) mm = fmax(mm, s_part[q]);
            a.block_max_u[b] = mm;
        }
    } else if (lane == 0) {
        a.scalars[1 + b * (kBlock / kWave) + wave] = m;
    }
}

// The same for tiled layouts whose links are cut into groups: a workgroup owns a block of link
// groups -- its tile items, strip items and octet passes hold rows of the block's links only --
// reduces them into slot partials kept in LDS (a wave takes the block's tasks w, w + waves, ...
// of each kind, the kinds starting at different waves), and then applies the length update of
// exactly those links, RL lanes per link, with the additions of update_phase in the same order.
// len, S and 1/cap are stored by position, so the state of the first round of links is
// requested before the tasks are walked.  Every wave leaves its maximum of S in
// scalars[1 + block * waves + wave].
struct GroupArgs {
    const int32_t *gblk_desc;
    const int32_t *tile_desc;
    const uint32_t *tile_mask;
    const uint8_t *tile_pres;
    const uint32_t *strip_base, *strip_mask;
    const uint64_t *strip_pres;
    const int32_t *strip_slot;
    const int32_t *pass_first_slot;
    const uint32_t *oct_base, *oct_mask;
    const int32_t *pos_link, *pos_slot_ptr;
    const int2 *pos_xslot;
    const uint8_t *choice, *choice2;
    const double *demand1n, *demand2;      // the library's padded copies, by id and by sigma
    const double *demand1t, *demand2t;     // the same, window-transposed
    const double *invcap_pos;
    double *len, *price, *S, *scalars;
    double eps;
    PlanStrides ps;
    double *u_pos, *u_id, *block_max_u;     // adaptive step only (u by position and by id)
};

// ONLY_U (adaptive step): stops at u = load / cap (by position, to a.u_pos) and leaves every
// wave's maximum of u in a.block_max_u, as k_reduce_update does.
template <bool MAXC, int RL, bool EXT, bool ONLY_U = false>
__global__ __launch_bounds__(1024) void k_group_reduce_update(GroupArgs a)
{
    extern __shared__ double s_slots[];
    int32_t stop_now = 0;
    if constexpr (EXT) {      // a batch (blockIdx.y is the plan) or a solve that may stop early
        stop_now = stop_word(a.ps);          // tested below, once the first loads are under way
        if constexpr (!ONLY_U) {             // (the adaptive step belongs to a single plan)
            a.choice = of_plan(a.choice, a.ps.row);
            a.choice2 = of_plan(a.choice2, a.ps.state);
            a.demand1n = of_plan(a.demand1n, a.ps.state);
            a.demand2 = of_plan(a.demand2, a.ps.state);
            a.demand1t = of_plan(a.demand1t, a.ps.state);
            a.demand2t = of_plan(a.demand2t, a.ps.state);
            a.len = of_plan(a.len, a.ps.state);
            a.price = of_plan(a.price, a.ps.state);
            a.S = of_plan(a.S, a.ps.state);
            a.scalars = of_plan(a.scalars, a.ps.state);
        }
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = blockDim.x >> 6;
    const int b = blockIdx.x;
    const int4 *dsc = reinterpret_cast<const int4 *>(a.gblk_desc + 16 * b);
    const int4 d0 = dsc[0], d1 = dsc[1], d2 = dsc[2];
    const int i0 = d0.x, i1 = d0.y;             // positions of the block (at least one)
    const int p0 = d0.z, p1 = d0.w;             // its passes
    const int os0 = d1.x, n_os = d1.y;          // its octet slots: LDS 0 .. n_os - 1
    const int xs0 = d1.z;                       // its other slots: LDS n_os ...
    const int t0 = d2.x, t1 = d2.y;             // its tile items
    const int s0 = d2.z, s1 = d2.w;             // its strip items
    const int xbase = xs0 - n_os;               // other slot s sits at s - xbase
    const double invrho = a.scalars[0];
    const int row = threadIdx.x / RL;
    const int l = threadIdx.x % RL;
    const int rows = blockDim.x / RL;
    struct Link {
        int e, c0, c1, x0, x1;
        double ic, s, l;
    };
    // positions past the end re-read the last one (so that every load is unconditional) and
    // are masked out when the update is applied
    auto fetch = [&](int i) {
        const int ic = i < i1 ? i : i1 - 1;
        Link st;
        st.e = a.pos_link[ic];
        st.c0 = a.pos_slot_ptr[ic] - os0;
        st.c1 = a.pos_slot_ptr[ic + 1] - os0;
        const int2 xs = a.pos_xslot[ic];
        st.x0 = xs.x - xbase;
        st.x1 = xs.y - xbase;
        st.ic = a.invcap_pos[ic];
        st.s = a.S[ic];
        st.l = a.len[ic];
        return st;
    };
    double smax = 0.0;
    auto apply = [&](int i, const Link &st) {
        const bool valid = i < i1;
        const double load = row_partial_sum<RL>(st.c0, valid ? st.c1 : st.c0, l, s_slots) +
                            row_partial_sum<RL>(st.x0, valid ? st.x1 : st.x0, l, s_slots);
        if (valid && l == 0) {
            const double u = load * st.ic;
            if constexpr (ONLY_U) {
                a.u_pos[i] = u;
                a.u_id[st.e] = u;
                smax = fmax(smax, u);
            } else {
                const double s_new = st.s + u;
                a.S[i] = s_new;
                const double g = u * invrho;
                const double t1e = a.eps * g;
                const double t2e = 1.0 + t1e;
                const double ln = st.l * t2e;
                a.len[i] = ln;
                a.price[st.e] = MAXC ? ln : ln * st.ic;
                smax = fmax(smax, s_new);
            }
        }
    };
    const Link first = fetch(i0 + row);
    if constexpr (EXT)
        if (stop_now != 0) return;           // (the same in every thread; nothing written yet)
    // tile items from wave 0 on, strip items where those end, octet passes after them
    const int nt = t1 - t0, ns = s1 - s0;
    int w = wave;
    reduce_tile_phase<0>(nt, a.tile_desc + size_t(t0) * kTileDescInts, a.tile_mask, a.tile_pres,
                         a.choice, a.demand1t, a.choice2, a.demand2t, s_slots, w, n_waves, lane,
                         xbase);
    w = (wave + n_waves - nt % n_waves) % n_waves;
    reduce_strip_phase<0>(ns, a.strip_base + size_t(s0) * kWave, a.strip_pres + size_t(s0) * kWave,
                          a.strip_mask + size_t(s0) * kWave, a.strip_slot + size_t(s0) * kWave,
                          a.choice, a.demand1n, a.choice2, a.demand2, s_slots, w, n_waves, lane,
                          xbase);
    w = (wave + 2 * n_waves - nt % n_waves - ns % n_waves) % n_waves;
    reduce_flat_phase<0>(p0, p1, a.pass_first_slot, a.oct_base, a.oct_mask, a.choice, a.demand1n,
                         a.choice2, a.demand2, s_slots, os0, w, n_waves, lane);
    __syncthreads();
    apply(i0 + row, first);
    for (int ibase = i0 + rows; ibase < i1; ibase += rows)               // block-uniform
        apply(ibase + row, fetch(ibase + row));
    const double m = wave_max(smax);
    if constexpr (ONLY_U) {
        // one maximum per block: the kernel that applies the step folds them all
        __syncthreads();                                // the slots are free again
        if (lane == 0) s_slots[wave] = m;
        __syncthreads();
        if (threadIdx.x == 0) {
            double mm = 0.0;
            for (int q = 0; q < n_waves; ++q) mm = fmax(mm, s_slots[q]);
            a.block_max_u[b] = mm;
        }
    } else if (lane == 0) {
        a.scalars[1 + b * n_waves + wave] = m;
    }
}

// The same for batches, U plans per workgroup: the four waves split the passes of the block as
// in the single-plan kernel, and every wave sums its pass for all U plans at once
// (reduce_flat_phase_multi), so that one trip to memory serves U plans.  A 16-lane row then
// applies the update of a link for the U plans in turn.
template <bool MAXC, int U>
__global__ __launch_bounds__(kBlock) void k_reduce_update_multi(FusedArgs a)
{
    __shared__ double s_part_all[U * kBlkMaxSlots];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const uint8_t *choice[U], *choice2[U];
    const double *demand1n[U], *demand2[U];
    double *s_part[U], *len[U], *price[U], *S[U], *scalars[U];
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int want = static_cast<int>(blockIdx.y) * U + u;
        live[u] = want < a.n_plans;
        const int plan = live[u] ? want : a.n_plans - 1;       // (repeats an existing plan)
        choice[u] = of_plan_at(a.choice, a.ps.row, plan);
        choice2[u] = of_plan_at(a.choice2, a.ps.state, plan);
        demand1n[u] = of_plan_at(a.demand1n, a.ps.state, plan);
        demand2[u] = of_plan_at(a.demand2, a.ps.state, plan);
        len[u] = of_plan_at(a.len, a.ps.state, plan);
        price[u] = of_plan_at(a.price, a.ps.state, plan);
        S[u] = of_plan_at(a.S, a.ps.state, plan);
        scalars[u] = of_plan_at(a.scalars, a.ps.state, plan);
        s_part[u] = s_part_all + u * kBlkMaxSlots;
    }
    const int b = blockIdx.x;
    const int4 d4 = *reinterpret_cast<const int4 *>(a.blk_desc + 8 * b);
    const int i0 = d4.x, i1 = d4.y;             // positions of the block (at least one)
    const int p0 = d4.z, p1 = d4.w;             // its passes
    const int slot0 = a.blk_desc[8 * b + 4];
    const int row = threadIdx.x / kRowLanes;
    const int l = threadIdx.x % kRowLanes;
    constexpr int kRows = kBlock / kRowLanes;
    double invrho[U], smax[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        invrho[u] = scalars[u][0];
        smax[u] = 0.0;
    }
    reduce_flat_phase_multi<U>(p0, p1, a.pass_first_slot, a.oct_base, a.oct_mask, choice, demand1n,
                               choice2, demand2, s_part, slot0, wave, kBlock / kWave, lane);
    __syncthreads();
    for (int ibase = i0; ibase < i1; ibase += kRows) {                  // block-uniform
        const int i = ibase + row;
        const bool valid = i < i1;
        const int ic_i = valid ? i : i1 - 1;
        const int e = a.pos_link[ic_i];
        const int c0 = a.pos_slot_ptr[ic_i] - slot0;
        const int c1 = valid ? a.pos_slot_ptr[ic_i + 1] - slot0 : c0;
        const double ic = a.invcap_pos[ic_i];
        double s_old[U], l_old[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            s_old[u] = S[u][ic_i];
            l_old[u] = len[u][ic_i];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const double load = row_partial_sum(c0, c1, l, s_part[u]);
            if (valid && l == 0 && live[u]) {
                const double uu = load * ic;
                const double s_new = s_old[u] + uu;
                S[u][i] = s_new;
                const double g = uu * invrho[u];
                const double t1 = a.eps * g;
                const double t2 = 1.0 + t1;
                const double ln = l_old[u] * t2;
                len[u][i] = ln;
                price[u][e] = MAXC ? ln : ln * ic;
                smax[u] = fmax(smax[u], s_new);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const double m = wave_max(smax[u]);
        if (lane == 0 && live[u]) scalars[u][1 + b * (kBlock / kWave) + wave] = m;
    }
}

// rho = max_e (demand that can reach e) / cap_e, in two steps: every block leaves the maximum
// over its links in scalars[1 + block], then one block folds those into scalars[0] = 1/rho
// (0 when rho = 0).  A maximum does not depend on the order it is taken in.
__global__ __launch_bounds__(kBlock) void k_width(int E,
                                                  const int32_t *__restrict__ pos_slot_ptr,
                                                  const int2 *__restrict__ pos_xslot,
                                                  const double *__restrict__ partial,
                                                  const double *__restrict__ invcap,
                                                  double *__restrict__ scalars, PlanStrides ps)
{
    __shared__ double red[16];
    partial = of_plan(partial, ps.state);
    scalars = of_plan(scalars, ps.state);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    double m = width_phase(E, pos_slot_ptr, pos_xslot, partial, invcap, wave, n_waves,
                           threadIdx.x & (kWave - 1));
    m = block_max(m, red);
    if (threadIdx.x == 0) scalars[1 + blockIdx.x] = m;
}

__global__ __launch_bounds__(kBlock) void k_width_fold(int n_blocks, double *__restrict__ scalars,
                                                       PlanStrides ps)
{
    __shared__ double red[16];
    scalars = of_plan(scalars, ps.state);
    double m = 0.0;
    for (int b = threadIdx.x; b < n_blocks; b += blockDim.x) m = fmax(m, scalars[1 + b]);
    m = block_max(m, red);
    if (threadIdx.x == 0) scalars[0] = (m > 0.0) ? 1.0 / m : 0.0;
}

// length update fused with the per-block maximum of the congestion sums (lambda = max / iters)
template <bool MAXC, int RL, bool EXT>
__global__ __launch_bounds__(kBlock) void k_update(int E, double eps,
                                                   const int32_t *__restrict__ pos_link,
                                                   const int32_t *__restrict__ pos_slot_ptr,
                                                   const int2 *__restrict__ pos_xslot,
                                                   const double *__restrict__ partial,
                                                   const double *__restrict__ invcap,
                                                   double *__restrict__ len,
                                                   double *__restrict__ price,
                                                   double *__restrict__ S,
                                                   double *__restrict__ scalars, PlanStrides ps)
{
    __shared__ double red[16];
    if constexpr (EXT) {
        partial = of_plan(partial, ps.state);
        len = of_plan(len, ps.state);
        price = of_plan(price, ps.state);
        S = of_plan(S, ps.state);
        scalars = of_plan(scalars, ps.state);
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    const double s_new = update_phase<MAXC, RL>(E, eps, scalars[0], pos_link, pos_slot_ptr,
                                                pos_xslot, partial, invcap, len, price, S, wave,
                                                n_waves, lane);
    const double m = block_max(s_new, red);
    if (threadIdx.x == 0) scalars[1 + blockIdx.x] = m;
}

__global__ __launch_bounds__(kBlock) void k_epilogue(int P, int iters, int n_update_blocks,
                                                     const uint32_t *__restrict__ count,
                                                     const double *__restrict__ scalars,
                                                     double *__restrict__ splits,
                                                     double *__restrict__ lambda, PlanStrides ps)
{
    __shared__ double red[16];
    count = of_plan(count, ps.state);
    scalars = of_plan(scalars, ps.state);
    splits = of_plan(splits, ps.splits);
    lambda = lambda + blockIdx.y;
    const double T = static_cast<double>(iters);
    const int stride = gridDim.x * blockDim.x;
    if (count != nullptr)         // otherwise the splits come from the choice log
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

// Plain streaming read for the empirical bandwidth figure of the benchmark: 16 bytes per lane
// and load, four loads in flight per lane, nothing kept but an xor that is (almost) never
// stored.
__global__ __launch_bounds__(kBlock) void k_stream_read(const u32x4 *__restrict__ p, size_t n16,
                                                        u32x4 *__restrict__ sink)
{
    const size_t stride = size_t(gridDim.x) * blockDim.x;
    size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = stream_load(p + i);
        const u32x4 b = stream_load(p + i + stride);
        const u32x4 c = stream_load(p + i + 2 * stride);
        const u32x4 d = stream_load(p + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n16; i += stride) acc ^= stream_load(p + i);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = acc;   // keeps the loads alive
}

inline int blocks_for(int64_t threads, int block, int cap)
{
    int64_t b = (threads + block - 1) / block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return static_cast<int>(b);
}

// byte distances between the plans of the batch a launch covers (t.batch plans, grid.y)
// whether a launch needs the kernels that know about plans and the stop word; a single plan
// that always runs to the end takes the plain ones, which do not even look
inline bool extended(const DeviceTopo &t) { return t.batch > 1 || t.stop_flag != nullptr; }

inline PlanStrides strides_of(const DeviceTopo &t)
{
    PlanStrides ps;
    ps.state = t.state_stride;
    ps.row = t.row_stride;
    ps.demand = sizeof(double) * static_cast<size_t>(t.K);
    ps.splits = sizeof(double) * static_cast<size_t>(t.P);
    ps.stop = t.stop_flag;
    return ps;
}

// workgroups that apply the pending step (one thread per link position; the first ones of the
// grid, so that they run beside the scan and not after it), and the arguments of a folded launch
static int fold_blocks(const DeviceTopo &t)
{
    return (t.E + kWave * kRecWaves - 1) / (kWave * kRecWaves);
}
static FoldArgs fold_of(const DeviceTopo &t)
{
    FoldArgs f = *t.fold;
    f.apply_blocks = fold_blocks(t);
    return f;
}

template <int L, bool MAXC>
void launch_argmin_lmax(const DeviceTopo &t, int grid, uint8_t *choice, uint32_t *count,
                        hipStream_t s)
{
    if (t.n_records > 0) {
        // one record per wave while the waves fit the chip at once; beyond that the grid is
        // what is resident at once (the same number of workgroups on every compute unit) and a
        // wave walks records rec, rec + n_waves, ..., the next one prefetched while one is
        // scanned
        int rec_grid = (t.n_records + kRecWaves - 1) / kRecWaves;
        // (the plans of a batch share the chip: each gets its part of what is resident)
        int resident = t.rec_blocks / (t.batch > 1 ? t.batch : 1);
        if (resident < 1) resident = 1;
        if (rec_grid > resident) rec_grid = resident;
        if (t.rec_per_wave > 0)
            rec_grid = (t.n_records + kRecWaves * t.rec_per_wave - 1) / (kRecWaves * t.rec_per_wave);
        if constexpr (L >= 2 && L <= 16) {      // (a slot's lanes 1 and L + 1 hold record words)
            if (t.rec_lane_major) {
                // records beyond half of the 32 MB of L2 are read around it
                const int64_t rec_bytes =
                    static_cast<int64_t>(t.n_records) *
                    (t.rec_dict ? kRecBytesDict : (t.rec_table16 ? kRecBytes16 : kRecBytes));
                int around_l2 = rec_bytes > (16LL << 20) ? 1 : 0;
                if (t.rec_around_l2 >= 0) around_l2 = t.rec_around_l2;
                if (t.rec_dict) {
                    const int dgrid = (t.n_rec_chunks + kRecWaves - 1) / kRecWaves;
#define NIMBLE_RECD_LAUNCH(SS)                                                                 \
    case SS:                                                                                   \
        if (t.fold != nullptr)                                                                 \
            hipLaunchKernelGGL((k_argmin_recd<L, SS, MAXC, true, true>),                       \
                               dim3(dgrid + fold_blocks(t)), dim3(kWave * kRecWaves), 0, s,    \
                               t.n_rec_chunks, around_l2, t.rec_chunks, t.records,             \
                               reinterpret_cast<const u32x4 *>(t.rec_dict_words), t.price,     \
                               choice, count, t.choice2, strides_of(t), fold_of(t));           \
        else if (extended(t))                                                                  \
            hipLaunchKernelGGL((k_argmin_recd<L, SS, MAXC, true>), dim3(dgrid, t.batch),       \
                               dim3(kWave * kRecWaves), 0, s, t.n_rec_chunks, around_l2,       \
                               t.rec_chunks, t.records,                                        \
                               reinterpret_cast<const u32x4 *>(t.rec_dict_words), t.price,     \
                               choice, count, t.choice2, strides_of(t), NoFold{0});            \
        else                                                                                   \
            hipLaunchKernelGGL((k_argmin_recd<L, SS, MAXC, false>), dim3(dgrid),               \
                               dim3(kWave * kRecWaves), 0, s, t.n_rec_chunks, around_l2,       \
                               t.rec_chunks, t.records,                                        \
                               reinterpret_cast<const u32x4 *>(t.rec_dict_words), t.price,     \
                               choice, count, t.choice2, strides_of(t), NoFold{0});            \
        return;
                    switch (t.rec_stride) {
                        NIMBLE_RECD_LAUNCH(1)
                        NIMBLE_RECD_LAUNCH(2)
                        NIMBLE_RECD_LAUNCH(3)
                        NIMBLE_RECD_LAUNCH(4)
                        NIMBLE_RECD_LAUNCH(5)
                    }
#undef NIMBLE_RECD_LAUNCH
                }
#define NIMBLE_RECL_LAUNCH(SS)                                                                 \
    case SS:                                                                                   \
        if (t.rec_table16 && t.fold != nullptr)                                                \
            hipLaunchKernelGGL((k_argmin_recl<L, SS, MAXC, true, true, true>),                 \
                               dim3(rec_grid + fold_blocks(t)), dim3(kWave * kRecWaves), 0, s, \
                               t.n_records, around_l2, t.records, t.price, choice, count,      \
                               t.choice2, strides_of(t), fold_of(t));                          \
        else if (t.rec_table16 && extended(t))                                                 \
            hipLaunchKernelGGL((k_argmin_recl<L, SS, MAXC, true, true>),                       \
                               dim3(rec_grid, t.batch), dim3(kWave * kRecWaves), 0, s,         \
                               t.n_records, around_l2, t.records, t.price, choice, count,      \
                               t.choice2, strides_of(t), NoFold{0});                           \
        else if (t.rec_table16)                                                                \
            hipLaunchKernelGGL((k_argmin_recl<L, SS, MAXC, true, false>), dim3(rec_grid),      \
                               dim3(kWave * kRecWaves), 0, s, t.n_records, around_l2,          \
                               t.records, t.price, choice, count, t.choice2, strides_of(t),    \
                               NoFold{0});                                                     \
        else                                                                                   \
            hipLaunchKernelGGL((k_argmin_recl<L, SS, MAXC, false, true>),                      \
                               dim3(rec_grid, t.batch), dim3(kWave * kRecWaves), 0, s,         \
                               t.n_records, around_l2, t.records, t.price, choice, count,      \
                               t.choice2, strides_of(t), NoFold{0});                           \
        return;
                switch (t.rec_stride) {
                    NIMBLE_RECL_LAUNCH(1)
                    NIMBLE_RECL_LAUNCH(2)
                    NIMBLE_RECL_LAUNCH(3)
                    NIMBLE_RECL_LAUNCH(4)
                    NIMBLE_RECL_LAUNCH(5)
                }
#undef NIMBLE_RECL_LAUNCH
            }
        }
        // two quads per lane cover every commodity (the layout's own choice of L does)
        const bool two = (t.pmax + 3) / 4 <= 2 * L;
#define NIMBLE_REC_LAUNCH(SS)                                                                  \
    case SS:                                                                                   \
        if (two)                                                                               \
            hipLaunchKernelGGL((k_argmin_rec<L, SS, MAXC, true, true>), dim3(rec_grid, t.batch), \
                               dim3(kWave * kRecWaves), 0, s, t.n_records, t.records, t.price, \
                               choice, count, t.choice2, strides_of(t));                       \
        else                                                                                   \
            hipLaunchKernelGGL((k_argmin_rec<L, SS, MAXC, false, true>), dim3(rec_grid, t.batch), \
                               dim3(kWave * kRecWaves), 0, s, t.n_records, t.records, t.price, \
                               choice, count, t.choice2, strides_of(t));                       \
        return;
        switch (t.rec_stride) {
            NIMBLE_REC_LAUNCH(1)
            NIMBLE_REC_LAUNCH(2)
            NIMBLE_REC_LAUNCH(3)
            NIMBLE_REC_LAUNCH(4)
            NIMBLE_REC_LAUNCH(5)
            NIMBLE_REC_LAUNCH(6)
            NIMBLE_REC_LAUNCH(7)
            NIMBLE_REC_LAUNCH(8)
        }
#undef NIMBLE_REC_LAUNCH
    }
#define NIMBLE_ARGMIN_LAUNCH(LM)                                                              \
    hipLaunchKernelGGL((k_argmin<L, LM, MAXC, true>), dim3(grid, t.batch), dim3(kBlock), 0, s, t.K, \
                       t.comm_ptr, t.path_ptr, t.path_links, t.price, choice, count, t.sigma, \
                       t.choice2, strides_of(t))
    if (t.lmax <= 2) NIMBLE_ARGMIN_LAUNCH(2);
    else if (t.lmax <= 4) NIMBLE_ARGMIN_LAUNCH(4);
    else NIMBLE_ARGMIN_LAUNCH(8);
#undef NIMBLE_ARGMIN_LAUNCH
}

template <bool MAXC>
void launch_argmin_l(const DeviceTopo &t, uint8_t *choice, uint32_t *count, hipStream_t s)
{
    // untiled kernel: one candidate per lane; record kernel: as many commodities side by side
    // as a record typically holds, each lane scanning several candidates
    int L = lanes_per_commodity(t.pmax);
    if (t.n_records > 0) {
        // record kernel: a lane scans quads of four candidates; the layout builder chose the
        // lanes per commodity together with the record capacity
        const int quads = (t.pmax + 3) / 4;
        L = 1;
        while (2 * L < quads && L < kWave) L <<= 1;
        if (t.rec_lanes > 0) L = t.rec_lanes;
    }
    const int grid = blocks_for(static_cast<int64_t>(t.K) * L, kBlock, 1 << 20);
    switch (L) {
    case 1: launch_argmin_lmax<1, MAXC>(t, grid, choice, count, s); break;
    case 2: launch_argmin_lmax<2, MAXC>(t, grid, choice, count, s); break;
    case 4: launch_argmin_lmax<4, MAXC>(t, grid, choice, count, s); break;
    case 8: launch_argmin_lmax<8, MAXC>(t, grid, choice, count, s); break;
    case 16: launch_argmin_lmax<16, MAXC>(t, grid, choice, count, s); break;
    case 32: launch_argmin_lmax<32, MAXC>(t, grid, choice, count, s); break;
    default: launch_argmin_lmax<64, MAXC>(t, grid, choice, count, s); break;
    }
}

template <int MODE>
void launch_reduce_mode(const DeviceTopo &t, const uint8_t *choice, const double *demand,
                        hipStream_t s)
{
    // a fixed pool of waves, each walking its passes with the loads pipelined
    int64_t waves = static_cast<int64_t>(t.n_passes) + t.n_tile_items + t.n_strip_items;
    if (waves < (t.n_schunks + 3) / 4) waves = (t.n_schunks + 3) / 4;
    const int grid = blocks_for(waves * kWave, kBlock, t.reduce_blocks);
    // every kind of work that exists gets at least one wave and at most one wave per item; an
    // item weighs tile_item_cost octet passes
    const int64_t n_waves = static_cast<int64_t>(grid) * (kBlock / kWave);
    const int64_t w_tile = static_cast<int64_t>(t.n_tile_items) * t.tile_item_cost;
    const int64_t w_strip = static_cast<int64_t>(t.n_strip_items) * t.tile_item_cost;
    const int64_t w_all = w_tile + w_strip + t.n_passes;
    auto share = [&](int64_t w, int64_t items) -> int64_t {
        if (items == 0) return 0;
        int64_t v = (n_waves * w + w_all / 2) / w_all;
        if (v < 1) v = 1;
        return v > items ? items : v;
    };
    int64_t tile_waves = share(w_tile, t.n_tile_items);
    int64_t strip_waves = share(w_strip, t.n_strip_items);
    while (tile_waves + strip_waves > n_waves - 1) {     // the octet passes keep one wave
        if (tile_waves >= strip_waves && tile_waves > 1) tile_waves -= 1;
        else if (strip_waves > 1) strip_waves -= 1;
        else break;
    }
    ReduceArgs a;
    a.n_passes = t.n_passes;
    a.n_schunks = t.n_schunks;
    a.n_tile_items = t.n_tile_items;
    a.n_tile_waves = static_cast<int>(tile_waves);
    a.n_strip_items = t.n_strip_items;
    a.n_strip_waves = static_cast<int>(strip_waves);
    a.strip_base = t.strip_base;
    a.strip_pres = t.strip_pres;
    a.strip_mask = t.strip_mask;
    a.strip_slot = t.strip_slot;
    a.demand1n = t.demand1n;
    a.tile_desc = t.tile_desc;
    a.tile_mask = t.tile_mask;
    a.tile_pres = t.tile_pres;
    a.demand1t = t.demand1t;
    a.demand2t = t.demand2t;
    a.pass_first_slot = t.pass_first_slot;
    a.oct_base = t.oct_base;
    a.oct_mask = t.oct_mask;
    a.schunk_begin = t.schunk_begin;
    a.schunk_end = t.schunk_end;
    a.schunk_slot = t.schunk_slot;
    a.single_pair = t.single_pair;
    a.pad_comm = static_cast<uint32_t>(t.K);
    a.choice = choice;
    a.choice2 = t.choice2;
    a.demand = demand;
    a.demand2 = t.demand2;
    a.partial = t.partial;
    a.ps = strides_of(t);
    if (extended(t) || MODE != 0)
        hipLaunchKernelGGL((k_load_reduce<MODE, true>), dim3(grid, t.batch), dim3(kBlock), 0, s, a);
    else
        hipLaunchKernelGGL((k_load_reduce<0, false>), dim3(grid), dim3(kBlock), 0, s, a);
}

}  // namespace

namespace {

template <int L, bool MAXC>
int recd_blocks_per_cu(int stride)
{
    int n = 0;
    hipError_t e = hipErrorInvalidValue;
#define NIMBLE_RECD_OCC(SS)                                                                    \
    case SS:                                                                                   \
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(                                      \
            &n, reinterpret_cast<const void *>(&k_argmin_recd<L, SS, MAXC, false>),            \
            kWave * kRecWaves,                                                                 \
            0);                                                                                \
        break;
    switch (stride) {
        NIMBLE_RECD_OCC(1)
        NIMBLE_RECD_OCC(2)
        NIMBLE_RECD_OCC(3)
        NIMBLE_RECD_OCC(4)
        NIMBLE_RECD_OCC(5)
    }
#undef NIMBLE_RECD_OCC
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return n;
}

}  // namespace

// Workgroups of the record kernel a compute unit holds at once (from the registers and LDS the
// kernel that would run takes); 0 when unknown.
int record_kernel_blocks_per_cu(const DeviceTopo &t)
{
    if (!(t.n_records > 0 && t.rec_lane_major && t.rec_dict)) return 0;
    const int quads = (t.pmax + 3) / 4;
    int L = 1;
    while (2 * L < quads && L < kWave) L <<= 1;
    if (t.rec_lanes > 0) L = t.rec_lanes;
    switch (L) {
    case 2:
        return t.cost_max ? recd_blocks_per_cu<2, true>(t.rec_stride)
                          : recd_blocks_per_cu<2, false>(t.rec_stride);
    case 4:
        return t.cost_max ? recd_blocks_per_cu<4, true>(t.rec_stride)
                          : recd_blocks_per_cu<4, false>(t.rec_stride);
    case 8:
        return t.cost_max ? recd_blocks_per_cu<8, true>(t.rec_stride)
                          : recd_blocks_per_cu<8, false>(t.rec_stride);
    case 16:
        return t.cost_max ? recd_blocks_per_cu<16, true>(t.rec_stride)
                          : recd_blocks_per_cu<16, false>(t.rec_stride);
    default: return 0;
    }
}

void launch_stream_read(const void *buf, size_t bytes, void *sink, hipStream_t s)
{
    hipLaunchKernelGGL(k_stream_read, dim3(256 * 8), dim3(kBlock), 0, s,
                       static_cast<const u32x4 *>(buf), bytes / 16, static_cast<u32x4 *>(sink));
}

int lanes_per_commodity(int pmax)
{
    int L = 1;
    while (L < pmax && L < kWave) L <<= 1;
    return L;
}

void launch_export_len(const DeviceTopo &t, double *len_out, hipStream_t s)
{
    hipLaunchKernelGGL(k_export_len, dim3((t.E + kBlock - 1) / kBlock), dim3(kBlock), 0, s, t.E,
                       t.pos_link, t.len, len_out);
}

void launch_init(const DeviceTopo &t, const double *demand, const double *len_in, hipStream_t s)
{
    const int n = t.E > t.P ? t.E : t.P;
    hipLaunchKernelGGL(k_init, dim3(blocks_for(n, kBlock, 4096), t.batch), dim3(kBlock), 0, s,
                       t.E, t.K, t.P, t.cost_max, len_in, t.pos_link, t.invcap, t.len, t.price,
                       t.S, t.choice, t.count, t.sigma, demand, t.demand1n, t.demand1t, t.demand2,
                       t.demand2t, strides_of(t));
}

void launch_width(const DeviceTopo &t, const double *demand, hipStream_t s)
{
    launch_reduce_mode<1>(t, t.choice, demand, s);
    hipLaunchKernelGGL(k_width, dim3(t.n_update_blocks, t.batch), dim3(kBlock), 0, s, t.E,
                       t.pos_slot_ptr, t.pos_xslot, t.partial, t.invcap_pos, t.scalars,
                       strides_of(t));
    hipLaunchKernelGGL(k_width_fold, dim3(1, t.batch), dim3(kBlock), 0, s, t.n_update_blocks,
                       t.scalars, strides_of(t));
}

void launch_argmin(const DeviceTopo &t, uint8_t *choice, uint32_t *count, hipStream_t s)
{
    if (t.cost_max) launch_argmin_l<true>(t, choice, count, s);
    else launch_argmin_l<false>(t, choice, count, s);
}

// The kernels that take a folded step are the lane-major record kernels (16-bit tables or a
// dictionary); launch_argmin_l and launch_argmin_lmax choose them under these conditions.
// Folding pays while the scan waits rather than works: three gathers per table entry instead
// of one cost about 0.1 us for every record a compute unit scans, a launch saved about 2 us
// (64-node fabric, 64 records per compute unit: 4 us per iteration slower; 16-node fabric, 3
// records per compute unit: 2 us faster).  Hence only while all records are scanned at once.
bool record_kernel_folds(const DeviceTopo &t, bool whenever_possible)
{
    if (t.n_records <= 0 || !t.rec_lane_major || t.batch > 1) return false;
    if (!whenever_possible && t.n_records > t.rec_blocks * kRecWaves) return false;
    if (!t.rec_dict && !t.rec_table16) return false;
    const int quads = (t.pmax + 3) / 4;
    int L = 1;
    while (2 * L < quads && L < kWave) L <<= 1;
    if (t.rec_lanes > 0) L = t.rec_lanes;
    if (L < 2 || L > 16) return false;
    return t.rec_stride >= 1 && t.rec_stride <= 5;
}

void launch_load_reduce(const DeviceTopo &t, const uint8_t *choice, const double *demand,
                        hipStream_t s)
{
    launch_reduce_mode<0>(t, choice, demand, s);
}

void launch_histogram(const DeviceTopo &t, const uint8_t *log, size_t stride, int32_t iters,
                      double *splits, hipStream_t s)
{
    const size_t lds = sizeof(uint32_t) * kWave * static_cast<size_t>(t.pmax | 1);
    hipLaunchKernelGGL(k_histogram, dim3((t.K + kWave - 1) / kWave, t.batch), dim3(kWave), lds, s,
                       t.K, iters, t.pmax, stride, log, t.comm_ptr, splits, strides_of(t));
}

void launch_update(const DeviceTopo &t, double eps, hipStream_t s)
{
#define NIMBLE_UPDATE_LAUNCH(MC, RL)                                                           \
    do {                                                                                       \
        if (extended(t))                                                                       \
            hipLaunchKernelGGL((k_update<MC, RL, true>), dim3(t.n_update_blocks, t.batch),     \
                               dim3(kBlock), 0, s, t.E, eps, t.pos_link, t.pos_slot_ptr,       \
                               t.pos_xslot, t.partial, t.invcap_pos, t.len, t.price, t.S,      \
                               t.scalars, strides_of(t));                                      \
        else                                                                                   \
            hipLaunchKernelGGL((k_update<MC, RL, false>), dim3(t.n_update_blocks),             \
                               dim3(kBlock), 0, s, t.E, eps, t.pos_link, t.pos_slot_ptr,       \
                               t.pos_xslot, t.partial, t.invcap_pos, t.len, t.price, t.S,      \
                               t.scalars, strides_of(t));                                      \
    } while (0)
    if (t.update_lanes == 4) {
        if (t.cost_max) NIMBLE_UPDATE_LAUNCH(true, 4);
        else NIMBLE_UPDATE_LAUNCH(false, 4);
    } else {
        if (t.cost_max) NIMBLE_UPDATE_LAUNCH(true, 16);
        else NIMBLE_UPDATE_LAUNCH(false, 16);
    }
#undef NIMBLE_UPDATE_LAUNCH
}

static GroupArgs group_args(const DeviceTopo &t, const uint8_t *choice, double eps)
{
    GroupArgs a;
    a.gblk_desc = t.gblk_desc;
    a.tile_desc = t.tile_desc;
    a.tile_mask = t.tile_mask;
    a.tile_pres = t.tile_pres;
    a.strip_base = t.strip_base;
    a.strip_mask = t.strip_mask;
    a.strip_pres = t.strip_pres;
    a.strip_slot = t.strip_slot;
    a.pass_first_slot = t.pass_first_slot;
    a.oct_base = t.oct_base;
    a.oct_mask = t.oct_mask;
    a.pos_link = t.pos_link;
    a.pos_slot_ptr = t.pos_slot_ptr;
    a.pos_xslot = t.pos_xslot;
    a.choice = choice;
    a.choice2 = t.choice2;
    a.demand1n = t.demand1n;
    a.demand2 = t.demand2;
    a.demand1t = t.demand1t;
    a.demand2t = t.demand2t;
    a.invcap_pos = t.invcap_pos;
    a.len = t.len;
    a.price = t.price;
    a.S = t.S;
    a.scalars = t.scalars;
    a.eps = eps;
    a.ps = strides_of(t);
    a.u_pos = nullptr;
    a.u_id = nullptr;
    a.block_max_u = nullptr;
    return a;
}

int launch_group_reduce_u(const DeviceTopo &t, const uint8_t *choice, double *u_pos, double *u_id,
                          double *block_max_u, hipStream_t s)
{
    GroupArgs a = group_args(t, choice, 0.0);
    a.u_pos = u_pos;
    a.u_id = u_id;
    a.block_max_u = block_max_u;
    const dim3 block(kWave * t.gblk_waves);
    const size_t lds = sizeof(double) * static_cast<size_t>(t.gblk_max_slots > 16 ? t.gblk_max_slots : 16);
    if (t.update_lanes == 4)
        hipLaunchKernelGGL((k_group_reduce_update<false, 4, true, true>), dim3(t.n_gblocks), block,
                           lds, s, a);
    else
        hipLaunchKernelGGL((k_group_reduce_update<false, 16, true, true>), dim3(t.n_gblocks),
                           block, lds, s, a);
    return t.n_gblocks;
}

void launch_group_reduce_update(const DeviceTopo &t, const uint8_t *choice, double eps,
                                hipStream_t s)
{
    const GroupArgs a = group_args(t, choice, eps);
    const dim3 block(kWave * t.gblk_waves);
    const size_t lds = sizeof(double) * static_cast<size_t>(t.gblk_max_slots > 0 ? t.gblk_max_slots : 1);
#define NIMBLE_GROUP_LAUNCH(MC, RL)                                                            \
    do {                                                                                       \
        if (extended(t))                                                                       \
            hipLaunchKernelGGL((k_group_reduce_update<MC, RL, true>),                          \
                               dim3(t.n_gblocks, t.batch), block, lds, s, a);                  \
        else                                                                                   \
            hipLaunchKernelGGL((k_group_reduce_update<MC, RL, false>), dim3(t.n_gblocks),      \
                               block, lds, s, a);                                              \
    } while (0)
    if (t.update_lanes == 4) {
        if (t.cost_max) NIMBLE_GROUP_LAUNCH(true, 4);
        else NIMBLE_GROUP_LAUNCH(false, 4);
    } else {
        if (t.cost_max) NIMBLE_GROUP_LAUNCH(true, 16);
        else NIMBLE_GROUP_LAUNCH(false, 16);
    }
#undef NIMBLE_GROUP_LAUNCH
}

void launch_reduce_update(const DeviceTopo &t, const uint8_t *choice, const double *demand,
                          double eps, hipStream_t s)
{
    FusedArgs a;
    a.blk_desc = t.blk_desc;
    a.pass_first_slot = t.pass_first_slot;
    a.oct_base = t.oct_base;
    a.oct_mask = t.oct_mask;
    a.pos_link = t.pos_link;
    a.pos_slot_ptr = t.pos_slot_ptr;
    a.choice = choice;
    a.choice2 = t.choice2;
    a.demand1n = t.demand1n;
    a.demand2 = t.demand2;
    a.invcap_pos = t.invcap_pos;
    a.len = t.len;
    a.price = t.price;
    a.S = t.S;
    a.scalars = t.scalars;
    a.eps = eps;
    a.ps = strides_of(t);
    a.n_plans = t.batch;
    a.u_pos = nullptr;
    a.u_id = nullptr;
    a.block_max_u = nullptr;
    constexpr int kPlansPerBlock = 4;
    if (t.batch >= kPlansPerBlock && t.batch_kernel == 0) {
        // batches: four plans per workgroup, their loads in flight together
        const dim3 grid(t.n_blocks, (t.batch + kPlansPerBlock - 1) / kPlansPerBlock);
        if (t.cost_max)
            hipLaunchKernelGGL((k_reduce_update_multi<true, kPlansPerBlock>), grid, dim3(kBlock), 0,
                               s, a);
        else
            hipLaunchKernelGGL((k_reduce_update_multi<false, kPlansPerBlock>), grid, dim3(kBlock),
                               0, s, a);
        return;
    }
    if (extended(t)) {
        if (t.cost_max)
            hipLaunchKernelGGL((k_reduce_update<true, false, true>), dim3(t.n_blocks, t.batch),
                               dim3(kBlock), 0, s, a);
        else
            hipLaunchKernelGGL((k_reduce_update<false, false, true>), dim3(t.n_blocks, t.batch),
                               dim3(kBlock), 0, s, a);
    } else if (t.cost_max) {
        hipLaunchKernelGGL((k_reduce_update<true, false, false>), dim3(t.n_blocks), dim3(kBlock),
                           0, s, a);
    } else {
        hipLaunchKernelGGL((k_reduce_update<false, false, false>), dim3(t.n_blocks), dim3(kBlock),
                           0, s, a);
    }
}

int launch_reduce_u(const DeviceTopo &t, const uint8_t *choice, double *u_pos, double *u_id,
                    double *block_max_u, hipStream_t s)
{
    FusedArgs a;
    a.blk_desc = t.blk_desc;
    a.pass_first_slot = t.pass_first_slot;
    a.oct_base = t.oct_base;
    a.oct_mask = t.oct_mask;
    a.pos_link = t.pos_link;
    a.pos_slot_ptr = t.pos_slot_ptr;
    a.choice = choice;
    a.choice2 = t.choice2;
    a.demand1n = t.demand1n;
    a.demand2 = t.demand2;
    a.invcap_pos = t.invcap_pos;
    a.len = t.len;
    a.price = t.price;
    a.S = t.S;
    a.scalars = t.scalars;
    a.eps = 0.0;
    a.ps = strides_of(t);
    a.n_plans = 1;
    a.u_pos = u_pos;
    a.u_id = u_id;
    a.block_max_u = block_max_u;
    hipLaunchKernelGGL((k_reduce_update<false, true, true>), dim3(t.n_blocks), dim3(kBlock), 0, s,
                       a);
    return t.n_blocks;
}

void launch_epilogue(const DeviceTopo &t, int32_t iters, const uint32_t *count, double *splits,
                     double *lambda, hipStream_t s)
{
    // the last length update left one maximum of S per wave or block: of the link blocks or the
    // blocks of link groups when a fused kernel ran, of the update blocks otherwise
    const int n_max = t.n_blocks > 0    ? t.n_blocks * (kBlock / kWave)
                      : t.n_gblocks > 0 ? t.n_gblocks * t.gblk_waves
                                        : t.n_update_blocks;
    const int grid = count ? blocks_for(t.P, kBlock, 4096) : 1;
    hipLaunchKernelGGL(k_epilogue, dim3(grid, t.batch), dim3(kBlock), 0, s, t.P, iters, n_max,
                       count, t.scalars, splits, lambda, strides_of(t));
}

}  // namespace nimble

// Device code of the per-iteration phases -- candidate scan over the plain CSR, link-load
// reduce over tile items / strip items / octet passes / single pairs, length update -- shared
// by the streaming kernels (one launch per phase) and the persistent kernel (one launch per
// solve, grid barriers between phases).
// All arithmetic is binary64, one IEEE operation per statement.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "host_topo.hpp"
#include "kernels.hpp"
#include "wave_ops.hpp"

namespace nimble {

// Loads that are consumed once per iteration (CSR streams) bypass cache retention so that the
// gathered tables (prices, choices, demands) keep their place in L2.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <typename T>
__device__ __forceinline__ T stream_load(const T *p)
{
    return __builtin_nontemporal_load(p);
}

// Loads of the reverse layouts (octets, masks, strip words): ordinary cached loads.  A
// non-temporal hint here cost 0.3 to 0.7 us per iteration on the 64-node configuration, whether
// the forward records were read through the L2 or around it.
template <typename T>
__device__ __forceinline__ T layout_load(const T *p)
{
    return *p;
}

// Forward-CSR loads: neighbouring lanes and the next unrolled load touch the same cache lines,
// so these stay ordinary cached loads.
template <typename T>
__device__ __forceinline__ T csr_load(const T *p)
{
    return *p;
}

// ---- batches of plans -----------------------------------------------------------------------
// The streaming kernels run the plans of a batch side by side: blockIdx.y is the plan.  All the
// per-plan state of a topology (demand copies, lengths, prices, congestion sums, choices,
// counts, partials, scalars) lives in one block per plan, so the same byte distance leads from
// any state array of plan 0 to that array of plan b; the caller's arrays and the rows of the
// choice log have distances of their own.
struct PlanStrides {
    size_t state;      // between the state blocks of consecutive plans
    size_t row;        // between the choice rows of one iteration
    size_t demand;     // between the caller's demand vectors
    size_t splits;     // between the caller's split vectors
    // (not a stride: it rides along to every kernel of an iteration) when not null, a word that
    // is non-zero once the solve has stopped; kernels launched after that return at once
    const int32_t *stop;
};

// The stop word itself, requested here and now (a volatile load the compiler leaves in place):
// a kernel that has other loads to issue first tests the value after them, so that the trip to
// memory for this word overlaps with theirs instead of preceding everything.
__device__ __forceinline__ int32_t stop_word(const PlanStrides &ps)
{
    return ps.stop != nullptr ? *static_cast<const volatile int32_t *>(ps.stop) : 0;
}

__device__ __forceinline__ bool stopped(const PlanStrides &ps)
{
    return ps.stop != nullptr && *ps.stop != 0;
}

template <typename T>
__device__ __forceinline__ T *of_plan_at(T *p, size_t stride, int plan)
{
    if (p == nullptr) return p;
    // (byte arithmetic on the pointer itself, not on an integer: the result stays derived from p,
    // so what the compiler knows about p -- __restrict__ above all -- still holds)
    using Byte = std::conditional_t<std::is_const<T>::value, const char, char>;
    return reinterpret_cast<T *>(reinterpret_cast<Byte *>(p) + stride * static_cast<size_t>(plan));
}

template <typename T>
__device__ __forceinline__ T *of_plan(T *p, size_t stride)
{
    return of_plan_at(p, stride, static_cast<int>(blockIdx.y));
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
                                             uint32_t *__restrict__ count,
                                             const int32_t *__restrict__ sigma,
                                             uint8_t *__restrict__ choice2, int wave,
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
            const int sg = sigma[k];
            if (sg >= 0) choice2[sg] = static_cast<uint8_t>(bj);   // copy in sigma order
            if (count != nullptr) count[p0 + bj] += 1u;            // absent: choices are logged
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

template <int PPL>
__device__ __forceinline__ void load_pairs(u32x4 (&v)[PPL / 2], const uint32_t *__restrict__ rev,
                                           int b, int e, int l, uint32_t pad_comm)
{
#pragma unroll
    for (int it = 0; it < PPL / 2; ++it) {
        // every lane always loads (lanes past the end re-read the chunk's first group and
        // discard it): an unconditional load keeps the number of outstanding requests known to
        // the compiler, which is what lets it wait for the older gathers only
        const int i = b + it * (kRowLanes * 2) + l * 2;      // pair index
        const u32x4 pad = {pad_comm, 0u, pad_comm, 0u};
        const u32x4 x = layout_load(reinterpret_cast<const u32x4 *>(rev + 2 * size_t(i < e ? i : b)));
        v[it] = (i < e) ? x : pad;
    }
}

// Software-pipelined over the chunks a DPP row visits: while the choices of the current chunk
// are being gathered, the pairs of the next chunk and the bounds of the one after are already
// requested, and because they are requested AFTER the gathers the in-order return of vector
// loads lets the gathers be consumed while the stream loads are in flight.  The demands of the
// few hits are fetched last, one per loop turn, in pair order.
template <int MODE, int PPL>
__device__ __forceinline__ void reduce_phase(int n_chunks, const int32_t *__restrict__ chunk_begin,
                                             const int32_t *__restrict__ chunk_end,
                                             const int32_t *__restrict__ chunk_slot,
                                             const uint32_t *__restrict__ rev, uint32_t pad_comm,
                                             const uint8_t *__restrict__ choice,
                                             const double *__restrict__ demand,
                                             double *__restrict__ partial, int wave, int n_waves,
                                             int lane)
{
    if (n_chunks <= 0) return;
    const int row = lane / kRowLanes;
    const int l = lane % kRowLanes;
    const int stride = n_waves * kRowsPerWave;
    const int last = n_chunks - 1;
    int c = wave * kRowsPerWave + row;
    int b1, e1;
    u32x4 cur[PPL / 2];
    {
        // bounds of chunks past the end are read from the last chunk and replaced by an empty
        // range, again so that every load is unconditional
        int b0 = chunk_begin[c < last ? c : last], e0 = chunk_end[c < last ? c : last];
        if (c > last) b0 = e0 = 0;
        const int cn = c + stride;
        b1 = chunk_begin[cn < last ? cn : last];
        e1 = chunk_end[cn < last ? cn : last];
        if (cn > last) b1 = e1 = 0;
        load_pairs<PPL>(cur, rev, b0, e0, l, pad_comm);
    }
    for (; c - row < n_chunks; c += stride) {          // wave-uniform bound
        uint32_t wa[PPL], wb[PPL];
#pragma unroll
        for (int it = 0; it < PPL / 2; ++it) {
            wa[it * 2 + 0] = cur[it].x;
            wb[it * 2 + 0] = cur[it].y;
            wa[it * 2 + 1] = cur[it].z;
            wb[it * 2 + 1] = cur[it].w;
        }
        uint32_t ch[PPL];
#pragma unroll
        for (int q = 0; q < PPL; ++q)
            if constexpr (MODE == 0) ch[q] = choice[wa[q] & kCommMask];
        // requests for later chunks, issued after the gathers
        const int c2 = c + 2 * stride;
        const int b2 = chunk_begin[c2 < last ? c2 : last], e2 = chunk_end[c2 < last ? c2 : last];
        const int slot = chunk_slot[c < last ? c : last];
        u32x4 nxt[PPL / 2];
        load_pairs<PPL>(nxt, rev, b1, e1, l, pad_comm);
        uint32_t hits = 0u;
#pragma unroll
        for (int q = 0; q < PPL; ++q) {
            bool hit;
            if constexpr (MODE == 0)
                hit = ((ch[q] >> 5) == ((wa[q] >> kWindowShift) & 3u)) &&
                      (((wb[q] >> (ch[q] & 31u)) & 1u) != 0u);
            else
                hit = (wa[q] & kFirstFlag) != 0u;
            hits |= static_cast<uint32_t>(hit) << q;
        }
        // demands of the hits in pair order
        double acc = 0.0;
        while (hits != 0u) {                 // four hits per turn, their loads side by side
            uint32_t idx[4];
            bool ok[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ok[u] = hits != 0u;
                const int t = ok[u] ? __ffs(hits) - 1 : 0;
                hits &= hits - 1u;           // 0 stays 0
                uint32_t ksel = wa[0];
#pragma unroll
                for (int q = 1; q < PPL; ++q) ksel = (t == q) ? wa[q] : ksel;
                idx[u] = ok[u] ? (ksel & kCommMask) : idx[0];
            }
            double d[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) d[u] = demand[idx[u]];
            // an absent hit re-reads the first one and is masked to +0.0 (masked, not selected:
            // a select would let the compiler move the load under the condition)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int mk = -static_cast<int>(ok[u]);
                acc = acc + __hiloint2double(__double2hiint(d[u]) & mk, __double2loint(d[u]) & mk);
            }
        }
        acc = acc + partner_f64<1>(acc);
        acc = acc + partner_f64<2>(acc);
        acc = acc + partner_f64<4>(acc);
        acc = acc + partner_f64<8>(acc);
        if (c < n_chunks && l == 0) partial[slot] = acc;
#pragma unroll
        for (int it = 0; it < PPL / 2; ++it) cur[it] = nxt[it];
        b1 = (c2 > last) ? 0 : b2;
        e1 = (c2 > last) ? 0 : e2;
    }
}

// ---- phase B, octet part --------------------------------------------------------------------
// An octet is one base commodity id (a multiple of 4) and eight masks for the commodities
// base .. base+7 (0 where the commodity does not use the link); one 8-byte load fetches the
// eight choices.  The octets of all links form one flat array that the waves walk 64 at a time
// (one octet per lane).  Flag bits in the base word: kOctNewSlot = this octet starts a new
// partial-sum slot (first octet of a link's row, or of a pass), kOctSigma = base is in the
// second commodity numbering (choices and demands are read from the sigma-ordered copies).
// A lane fetches the eight choices (one 8-byte load) and the eight demands (four 16-byte loads
// from the library's own padded copies) of its octet together -- both depend on the base word
// only, which was prefetched -- and adds the demands of the hits in slot order (fma(d, 1.0, a)
// for a hit, fma(d, 0.0, a) otherwise: the same sums as plain additions, demands are finite);
// the lanes of one slot are then combined by a segmented inclusive scan (fixed distances
// 1,2,..,32: the same tree on every run) and the last lane of the segment stores the sum.  No
// floating-point atomics.
// MODE 1 (width rho): every commodity with a non-zero mask counts once.
template <int MODE>
__device__ __forceinline__ void reduce_flat_phase(
    int pass_begin, int pass_end, const int32_t *__restrict__ pass_first_slot,
    const uint32_t *__restrict__ oct_base, const uint32_t *__restrict__ oct_mask,
    const uint8_t *__restrict__ choice, const double *__restrict__ demand1n,
    const uint8_t *__restrict__ choice2, const double *__restrict__ demand2,
    double *__restrict__ partial, int slot_base, int wave, int n_waves, int lane)
{
    // passes pass_begin + wave, + n_waves, ... below pass_end; slot s goes to
    // partial[s - slot_base] (global memory, or the LDS of a link block).
    // demand1n / demand2: the demands by id / by sigma number, with 8 spare entries.
    const int first = pass_begin + wave;
    if (first >= pass_end) return;
    const int last = pass_end - 1;
    const u32x4 *masks = reinterpret_cast<const u32x4 *>(oct_mask);
    // While a pass is worked on, the octets of the wave's next pass are in flight.  Every load
    // is unconditional (passes beyond the end re-read the range's last pass), which keeps the
    // number of outstanding requests known to the compiler so that it waits for the oldest only.
    uint32_t bw = layout_load(oct_base + size_t(first) * kWave + lane);
    // masks of a pass: words 0..3 of the 64 octets lane after lane, then words 4..7
    u32x4 m0 = layout_load(masks + size_t(first) * 128 + lane);
    u32x4 m1 = layout_load(masks + size_t(first) * 128 + 64 + lane);
    for (int pass = first; pass < pass_end; pass += n_waves) {     // wave-uniform
        const bool sig = (bw & kOctSigma) != 0u;
        const int base = static_cast<int>(bw & ~3u);
        uint2 ch = make_uint2(0u, 0u);
        if constexpr (MODE == 0)
            ch = *reinterpret_cast<const uint2 *>((sig ? choice2 : choice) + base);
        const u32x4 *dq = reinterpret_cast<const u32x4 *>((sig ? demand2 : demand1n) + base);
        const u32x4 q0 = dq[0], q1 = dq[1], q2 = dq[2], q3 = dq[3];
        const int first_slot = pass_first_slot[pass];
        const uint32_t flagword = bw;
        const uint32_t mk[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
        // the next pass of this wave
        const int np = pass + n_waves < last ? pass + n_waves : last;
        bw = layout_load(oct_base + size_t(np) * kWave + lane);
        m0 = layout_load(masks + size_t(np) * 128 + lane);
        m1 = layout_load(masks + size_t(np) * 128 + 64 + lane);
        const double dm[8] = {
            __hiloint2double(int(q0.y), int(q0.x)), __hiloint2double(int(q0.w), int(q0.z)),
            __hiloint2double(int(q1.y), int(q1.x)), __hiloint2double(int(q1.w), int(q1.z)),
            __hiloint2double(int(q2.y), int(q2.x)), __hiloint2double(int(q2.w), int(q2.z)),
            __hiloint2double(int(q3.y), int(q3.x)), __hiloint2double(int(q3.w), int(q3.z))};
        double acc = 0.0;
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) {
            uint32_t h;
            if constexpr (MODE == 0) {
                // commodities in octets have at most 32 candidates, so the choice is < 32
                const uint32_t c8 = ((sl < 4 ? ch.x : ch.y) >> (8 * (sl & 3))) & 31u;
                h = (mk[sl] >> c8) & 1u;
            } else {
                h = mk[sl] != 0u ? 1u : 0u;
            }
            acc = __builtin_fma(dm[sl], static_cast<double>(h), acc);
        }
        const unsigned long long heads = __ballot((flagword & kOctNewSlot) != 0u);   // bit 0 set
        const unsigned long long upto = heads & (~0ull >> (63 - lane));   // heads at lanes <= lane
        const int start = 63 - __clzll(static_cast<long long>(upto));
        acc = segmented_scan_f64(acc, start, lane);
        const bool tail = lane == kWave - 1 || ((heads >> (lane + 1)) & 1ull) != 0ull;
        if (tail) partial[first_slot - slot_base + __popcll(upto) - 1] = acc;
    }
}

// The octet part for U plans of a batch at once: the octets of a pass (base words, masks, slot
// numbers) are the same for every plan, only the choices and the demands differ.  A lane
// fetches them for all U plans together -- U times the loads in flight for one trip to memory --
// and then sums plan after plan with the arithmetic of reduce_flat_phase (the same additions in
// the same order, so every plan gets the bits it would get alone).  choice, demand1n, choice2,
// demand2 and partial are arrays of U pointers; a plan that does not exist repeats the
// pointers of one that does (its sums are computed and stored twice, which is harmless).
template <int U>
__device__ __forceinline__ void reduce_flat_phase_multi(
    int pass_begin, int pass_end, const int32_t *__restrict__ pass_first_slot,
    const uint32_t *__restrict__ oct_base, const uint32_t *__restrict__ oct_mask,
    const uint8_t *const (&choice)[U], const double *const (&demand1n)[U],
    const uint8_t *const (&choice2)[U], const double *const (&demand2)[U],
    double *const (&partial)[U], int slot_base, int wave, int n_waves, int lane)
{
    const int first = pass_begin + wave;
    if (first >= pass_end) return;
    const int last = pass_end - 1;
    const u32x4 *masks = reinterpret_cast<const u32x4 *>(oct_mask);
    uint32_t bw = layout_load(oct_base + size_t(first) * kWave + lane);
    u32x4 m0 = layout_load(masks + size_t(first) * 128 + lane);
    u32x4 m1 = layout_load(masks + size_t(first) * 128 + 64 + lane);
    for (int pass = first; pass < pass_end; pass += n_waves) {     // wave-uniform
        const bool sig = (bw & kOctSigma) != 0u;
        const int base = static_cast<int>(bw & ~3u);
        uint2 ch[U];
        u32x4 q[U][4];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            ch[u] = *reinterpret_cast<const uint2 *>((sig ? choice2[u] : choice[u]) + base);
            const u32x4 *dq =
                reinterpret_cast<const u32x4 *>((sig ? demand2[u] : demand1n[u]) + base);
            q[u][0] = dq[0];
            q[u][1] = dq[1];
            q[u][2] = dq[2];
            q[u][3] = dq[3];
        }
        const int first_slot = pass_first_slot[pass];
        const uint32_t flagword = bw;
        const uint32_t mk[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
        // the next pass of this wave
        const int np = pass + n_waves < last ? pass + n_waves : last;
        bw = layout_load(oct_base + size_t(np) * kWave + lane);
        m0 = layout_load(masks + size_t(np) * 128 + lane);
        m1 = layout_load(masks + size_t(np) * 128 + 64 + lane);
        const unsigned long long heads = __ballot((flagword & kOctNewSlot) != 0u);
        const unsigned long long upto = heads & (~0ull >> (63 - lane));
        const int start = 63 - __clzll(static_cast<long long>(upto));
        const bool tail = lane == kWave - 1 || ((heads >> (lane + 1)) & 1ull) != 0ull;
        const int slot = first_slot - slot_base + __popcll(upto) - 1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const double dm[8] = {
                __hiloint2double(int(q[u][0].y), int(q[u][0].x)),
                __hiloint2double(int(q[u][0].w), int(q[u][0].z)),
                __hiloint2double(int(q[u][1].y), int(q[u][1].x)),
                __hiloint2double(int(q[u][1].w), int(q[u][1].z)),
                __hiloint2double(int(q[u][2].y), int(q[u][2].x)),
                __hiloint2double(int(q[u][2].w), int(q[u][2].z)),
                __hiloint2double(int(q[u][3].y), int(q[u][3].x)),
                __hiloint2double(int(q[u][3].w), int(q[u][3].z))};
            double acc = 0.0;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) {
                const uint32_t c8 = ((sl < 4 ? ch[u].x : ch[u].y) >> (8 * (sl & 3))) & 31u;
                const uint32_t h = (mk[sl] >> c8) & 1u;
                acc = __builtin_fma(dm[sl], static_cast<double>(h), acc);
            }
            acc = segmented_scan_f64(acc, start, lane);
            if (tail) partial[u][slot] = acc;
        }
    }
}

// ---- phase B, tile part ---------------------------------------------------------------------
// A work item is up to kTileRows pieces of one window: kTileIds consecutive commodity numbers
// (ids, or sigma numbers).  Lane c owns column c, the commodities window + 8c .. + 7: it loads
// their eight choices and eight demands once (coalesced over the wave) and uses them for every
// piece of the item, whose masks arrive as two 16-byte loads per lane and piece.  No per-hit
// gather is left.  Uniform pieces (one mask value plus presence bits) need no mask loads at
// all: the pieces of an item cover the same commodities, so one presence byte per lane serves
// all rows of the item.  The eight
// per-lane row sums are added over the wave by wave_sum8 and lanes 0..7 store one partial each.
// MODE 1 (width rho): every commodity with a non-zero mask counts once.
// Position of commodity number nb in the window-transposed demand copies: inside a window of
// kTileIds numbers the eight demands of a column are 64 entries apart, so that lane c's load of
// demand sl sits next to lane c+1's (eight fully coalesced 8-byte loads per window).
__device__ __forceinline__ int tile_demand_index(int nb)
{
    return (nb & ~(kTileIds - 1)) | ((nb & 7) << 6) | ((nb >> 3) & 63);
}

template <int MODE>
__device__ __forceinline__ void reduce_tile_phase(
    int n_items, const int32_t *__restrict__ tile_desc, const uint32_t *__restrict__ tile_mask,
    const uint8_t *__restrict__ tile_pres,
    const uint8_t *__restrict__ choice, const double *__restrict__ demand1t,
    const uint8_t *__restrict__ choice2, const double *__restrict__ demand2t,
    double *__restrict__ partial, int wave, int n_waves, int lane, int slot_base = 0)
{
    // demand1t / demand2t: the demands by id / by sigma number, window-transposed
    // (tile_demand_index); slot s goes to partial[s - slot_base] (global memory, or the LDS of
    // a block of link groups)
    const u32x4 *masks = reinterpret_cast<const u32x4 *>(tile_mask);
    const int my_row = tile_row_of_lane(lane);
    // the item index lives in a scalar register, so the descriptor words that all lanes share
    // come by scalar loads
    for (int it = __builtin_amdgcn_readfirstlane(wave); it < n_items; it += n_waves) {
        const int32_t *d = tile_desc + size_t(it) * kTileDescInts;
        const int base = __builtin_amdgcn_readfirstlane(d[0]);
        const int flags = __builtin_amdgcn_readfirstlane(d[1]);
        const int n_rows = __builtin_amdgcn_readfirstlane(d[2]);
        const int first = __builtin_amdgcn_readfirstlane(d[3]);
        const int my_slot = d[8 + my_row];
        const bool sig = (flags & 1) != 0;
        const uint8_t *ch_src = sig ? choice2 : choice;
        const double *dm_src = (sig ? demand2t : demand1t) + base + lane;
        uint2 ch = make_uint2(0u, 0u);
        if constexpr (MODE == 0) ch = *reinterpret_cast<const uint2 *>(ch_src + base + 8 * lane);
        double dm[8];
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) dm[sl] = dm_src[sl * 64];
        uint32_t c8[8];
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) c8[sl] = ((sl < 4 ? ch.x : ch.y) >> (8 * (sl & 3))) & 31u;
        double acc[kTileRows];
        if ((flags & 2) != 0) {
            // uniform pieces: one mask per piece (wave-uniform) and one presence byte per
            // lane (the same for every piece of the item).  A hit adds the demand
            // as fma(d, 1.0, a) and a miss as fma(d, 0.0, a): the same sums as plain additions
            // (demands are finite), one instruction per pair less than masking both halves.
            // the rows of an item cover the same commodities (the layout packs them so): the
            // demands of the others are cleared once, and a row only tests its mask
            const uint32_t p0 = tile_pres[size_t(first) * 64 + lane];
            double dz[8];
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) dz[sl] = ((p0 >> sl) & 1u) != 0u ? dm[sl] : 0.0;
#pragma unroll
            for (int r = 0; r < kTileRows; ++r) {
                acc[r] = 0.0;
                if (r >= n_rows) continue;          // wave-uniform: rows past the last piece
                const uint32_t mr =
                    static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(d[16 + r]));
                double a = 0.0;
#pragma unroll
                for (int sl = 0; sl < 8; ++sl) {
                    uint32_t h = 1u;
                    if constexpr (MODE == 0) h = (mr >> c8[sl]) & 1u;
                    else h = mr != 0u ? 1u : 0u;
                    a = __builtin_fma(dz[sl], static_cast<double>(h), a);
                }
                acc[r] = a;
            }
        } else {
            // dense pieces: rows past the last piece re-read it and are not stored
            u32x4 m0[kTileRows], m1[kTileRows];
#pragma unroll
            for (int r = 0; r < kTileRows; ++r) {
                const int pr = first + (r < n_rows ? r : n_rows - 1);
                m0[r] = layout_load(masks + size_t(pr) * 128 + lane);
                m1[r] = layout_load(masks + size_t(pr) * 128 + 64 + lane);
            }
#pragma unroll
            for (int r = 0; r < kTileRows; ++r) {
                const uint32_t mk[8] = {m0[r].x, m0[r].y, m0[r].z, m0[r].w,
                                        m1[r].x, m1[r].y, m1[r].z, m1[r].w};
                double a = 0.0;
#pragma unroll
                for (int sl = 0; sl < 8; ++sl) {
                    // 1 where the commodity routes through the link, else 0
                    uint32_t h;
                    if constexpr (MODE == 0) h = (mk[sl] >> c8[sl]) & 1u;
                    else h = mk[sl] != 0u ? 1u : 0u;
                    a = __builtin_fma(dm[sl], static_cast<double>(h), a);
                }
                acc[r] = a;
            }
        }
        const double total = wave_sum8(acc, lane);
        if (lane < 8 && my_row < n_rows) partial[my_slot - slot_base] = total;
    }
}

// ---- phase B, strip part --------------------------------------------------------------------
// A strip item is 8 units of 8 lanes; a unit is 8 columns (octets) shared by up to 8 links
// whose rows consist of exactly these octets, each row with one mask value.  Lane i of a unit
// gathers the 8 choices and 8 demands of its column once (the demands with four 16-byte loads
// from the library's own aligned copies) and uses them for every row; the row sums are added
// inside the unit's 8 lanes and every lane stores the partial of one row.
// MODE 1 (width rho): every present commodity counts once.
template <int MODE>
__device__ __forceinline__ void reduce_strip_phase(
    int n_items, const uint32_t *__restrict__ strip_base, const uint64_t *__restrict__ strip_pres,
    const uint32_t *__restrict__ strip_mask, const int32_t *__restrict__ strip_slot,
    const uint8_t *__restrict__ choice, const double *__restrict__ demand1n,
    const uint8_t *__restrict__ choice2, const double *__restrict__ demand2,
    double *__restrict__ partial, int wave, int n_waves, int lane, int slot_base = 0)
{
    const int my_row = tile_row_of_lane(lane);
    const int unit0 = lane & ~7;
    for (int it = wave; it < n_items; it += n_waves) {               // wave-uniform
        const size_t at = size_t(it) * kWave;
        const uint32_t bw = layout_load(strip_base + at + lane);
        const uint64_t pres = strip_pres[at + lane];
        const int my_slot = strip_slot[at + unit0 + my_row];
        uint32_t mr[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) mr[r] = strip_mask[at + unit0 + r];
        const bool sig = (bw & kOctSigma) != 0u;
        const int base = static_cast<int>(bw & ~3u);
        uint2 ch = make_uint2(0u, 0u);
        if constexpr (MODE == 0)
            ch = *reinterpret_cast<const uint2 *>((sig ? choice2 : choice) + base);
        const u32x4 *dq = reinterpret_cast<const u32x4 *>((sig ? demand2 : demand1n) + base);
        const u32x4 q0 = dq[0], q1 = dq[1], q2 = dq[2], q3 = dq[3];
        const double dm[8] = {
            __hiloint2double(int(q0.y), int(q0.x)), __hiloint2double(int(q0.w), int(q0.z)),
            __hiloint2double(int(q1.y), int(q1.x)), __hiloint2double(int(q1.w), int(q1.z)),
            __hiloint2double(int(q2.y), int(q2.x)), __hiloint2double(int(q2.w), int(q2.z)),
            __hiloint2double(int(q3.y), int(q3.x)), __hiloint2double(int(q3.w), int(q3.z))};
        uint32_t c8[8];
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) c8[sl] = ((sl < 4 ? ch.x : ch.y) >> (8 * (sl & 3))) & 31u;
        double acc[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint32_t pb = static_cast<uint32_t>(pres >> (8 * r)) & 0xFFu;
            double a = 0.0;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) {
                // a hit adds the demand as fma(d, 1.0, a), a miss as fma(d, 0.0, a): the same
                // sums as plain additions (demands are finite)
                uint32_t h = (pb >> sl) & 1u;
                if constexpr (MODE == 0) h &= mr[r] >> c8[sl];
                a = __builtin_fma(dm[sl], static_cast<double>(h), a);
            }
            acc[r] = a;
        }
        const double total = group8_sum8(acc, lane);
        if (my_slot >= 0) partial[my_slot - slot_base] = total;
    }
}

// ---- phase C: slot partials -> load, congestion sum, multiplicative length update ----------
// One 16-lane DPP row per link: the lanes fetch the link's slot partials side by side (16 per
// step), add their own in ascending slot order, and a fixed butterfly combines the 16 lane
// sums; lane 0 of the row then applies  S_e += u_e,  len_e *= 1 + eps*u_e/rho,  price_e.
// Returns, in lane 0 of every row, the new S_e (0 elsewhere) for the lambda max-reduce.
// Links with few slots (tiled layouts: two or three per link) are better served by 4 lanes
// each, which quarters the threads of the update; RL is the number of lanes per link.
template <int RL = kRowLanes>
__device__ __forceinline__ double row_partial_sum(int c0, int c1, int l,
                                                  const double *__restrict__ partial)
{
    double acc = 0.0;
    for (int c = c0 + l; c < c1; c += RL) acc = acc + partial[c];
    acc = acc + partner_f64<1>(acc);
    acc = acc + partner_f64<2>(acc);
    if constexpr (RL > 4) acc = acc + partner_f64<4>(acc);
    if constexpr (RL > 8) acc = acc + partner_f64<8>(acc);
    return acc;
}

template <bool MAXC, int RL = kRowLanes>
__device__ __forceinline__ double update_phase(int E, double eps, double invrho,
                                               const int32_t *__restrict__ pos_link,
                                               const int32_t *__restrict__ pos_slot_ptr,
                                               const int2 *__restrict__ pos_xslot,
                                               const double *__restrict__ partial,
                                               const double *__restrict__ invcap_pos,
                                               double *__restrict__ len,
                                               double *__restrict__ price, double *__restrict__ S,
                                               int wave, int n_waves, int lane)
{
    // invcap_pos, len and S are stored in the flat order of the rows (by position); only the
    // price array, which the candidate scan gathers from, is indexed by link id
    static_assert(RL == 4 || RL == 16, "4 or 16 lanes per link");
    constexpr int kRows = kWave / RL;
    const int row = lane / RL;
    const int l = lane % RL;
    double smax = 0.0;
    for (int ibase = wave * kRows; ibase < E; ibase += n_waves * kRows) {
        const int i = ibase + row;          // position in the flat order of the rows
        int e = 0, c0 = 0, c1 = 0, s0 = 0, s1 = 0;
        if (i < E) {
            e = pos_link[i];
            c0 = pos_slot_ptr[i];
            c1 = pos_slot_ptr[i + 1];
            const int2 xs = pos_xslot[i];       // the link's piece, strip and single-chunk slots
            s0 = xs.x;
            s1 = xs.y;
        }
        // the link's own state is requested before the partial sums are waited for
        double ic = 0.0, s_old = 0.0, l_old = 0.0;
        if (i < E && l == 0) {
            ic = invcap_pos[i];
            s_old = S[i];
            l_old = len[i];
        }
        // octet slots, then (rarely any) single-pair slots
        const double load = row_partial_sum<RL>(c0, c1, l, partial) + row_partial_sum<RL>(s0, s1, l, partial);
        if (i < E && l == 0) {
            const double u = load * ic;
            const double s_new = s_old + u;
            S[i] = s_new;
            const double g = u * invrho;
            const double t1 = eps * g;
            const double t2 = 1.0 + t1;
            const double ln = l_old * t2;
            len[i] = ln;
            price[e] = MAXC ? ln : ln * ic;
            smax = fmax(smax, s_new);
        }
    }
    return smax;
}

// max over this wave's links of (demand that can reach the link) / capacity: terms of rho
__device__ __forceinline__ double width_phase(int E,
                                              const int32_t *__restrict__ pos_slot_ptr,
                                              const int2 *__restrict__ pos_xslot,
                                              const double *__restrict__ partial,
                                              const double *__restrict__ invcap_pos, int wave,
                                              int n_waves, int lane)
{
    const int row = lane / kRowLanes;
    const int l = lane % kRowLanes;
    double m = 0.0;
    for (int ibase = wave * kRowsPerWave; ibase < E; ibase += n_waves * kRowsPerWave) {
        const int i = ibase + row;
        int c0 = 0, c1 = 0, s0 = 0, s1 = 0;
        if (i < E) {
            c0 = pos_slot_ptr[i];
            c1 = pos_slot_ptr[i + 1];
            const int2 xs = pos_xslot[i];       // the link's piece, strip and single-chunk slots
            s0 = xs.x;
            s1 = xs.y;
        }
        const double reach = row_partial_sum(c0, c1, l, partial) + row_partial_sum(s0, s1, l, partial);
        if (i < E) m = fmax(m, reach * invcap_pos[i]);
    }
    return m;
}

// One workgroup's share of a step of the adaptive solve (Sec. IV-B with the step sigma = 1 /
// max_e u_e): thread i of block `block` owns link position block * 256 + i (workgroups of 256
// threads).  `red` is shared scratch of 16 doubles.  Every block folds all the maxima of u
// itself.
template <bool MAXC>
__device__ __forceinline__ void ad_apply_block(const AdApplyArgs &a, int block, double *red)
{
    // the stop word, the link's own state and the maxima are requested together (threads past
    // the last link re-read it), so that one trip to memory serves all three
    const int32_t stop_now = *static_cast<const volatile int32_t *>(a.flags);
    const int i = block * 256 + static_cast<int>(threadIdx.x);
    const int ic = i < a.E ? i : a.E - 1;
    const double u_i = a.u_pos[ic];
    const double s_old = a.S[ic];
    const double l_old = a.len[ic];
    const double cap_i = a.invcap_pos[ic];
    const int e_i = a.pos_link[ic];
    const double m = max_of_strided<256>(a.block_max_u, a.n_u_blocks, threadIdx.x);
    if (stop_now != 0) return;
    const double umax = block_max(m, red);
    if (!(umax > 0.0)) {                               // no traffic at all: the solve ends here
        if (block == 0 && threadIdx.x == 0) a.flags[0] = 1;
        return;
    }
    const double sigma = 1.0 / umax;
    double s_new = 0.0;
    if (i < a.E) {
        const double su = sigma * u_i;
        s_new = s_old + su;
        a.S[i] = s_new;
        const double t1 = a.eps * su;
        const double t2 = 1.0 + t1;
        const double ln = l_old * t2;
        a.len[i] = ln;
        a.len_id_new[e_i] = ln;
        a.price[e_i] = MAXC ? ln : ln * cap_i;
    }
    __syncthreads();
    const double sm = block_max(s_new, red);
    if (threadIdx.x == 0) {
        a.block_max_s[block] = sm;
        if (block == 0) {
            a.ascal[0] = a.ascal[0] + sigma;
            a.sigma_log[a.flags[1]] = sigma;
            a.flags[1] = a.flags[1] + 1;
        }
    }
}

}  // namespace nimble

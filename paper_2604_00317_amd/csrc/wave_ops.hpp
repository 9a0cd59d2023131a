// Wave64 cross-lane helpers for gfx950: butterfly reductions built from DPP row operations
// (quad_perm, row_half_mirror, row_mirror) for distances below 16 and ds_bpermute for 16/32.
// Every helper must be called with all 64 lanes of the wave active.
#pragma once
#include <hip/hip_runtime.h>

namespace nimble {

constexpr int kWave = 64;

// DPP controls (CDNA ISA): quad_perm [1,0,3,2] / [2,3,0,1], row_half_mirror, row_mirror.
constexpr int kDppXor1 = 0xB1;
constexpr int kDppXor2 = 0x4E;
constexpr int kDppHalfMirror = 0x141;
constexpr int kDppMirror = 0x140;

template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v)
{
    int lo = dpp_i32<CTRL>(__double2loint(v));
    int hi = dpp_i32<CTRL>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}

// Value of the partner lane at butterfly stage STEP (1,2,4,8,16,32).  Stages 4 and 8 use the
// mirror permutations: after stages 1..STEP/2 every aligned group of STEP lanes already holds
// one common value, so any lane of the neighbouring group is a valid partner.
template <int STEP>
__device__ __forceinline__ double partner_f64(double v)
{
    if constexpr (STEP == 1) return dpp_f64<kDppXor1>(v);
    else if constexpr (STEP == 2) return dpp_f64<kDppXor2>(v);
    else if constexpr (STEP == 4) return dpp_f64<kDppHalfMirror>(v);
    else if constexpr (STEP == 8) return dpp_f64<kDppMirror>(v);
    else return __shfl_xor(v, STEP, kWave);
}

template <int STEP>
__device__ __forceinline__ int partner_i32(int v)
{
    if constexpr (STEP == 1) return dpp_i32<kDppXor1>(v);
    else if constexpr (STEP == 2) return dpp_i32<kDppXor2>(v);
    else if constexpr (STEP == 4) return dpp_i32<kDppHalfMirror>(v);
    else if constexpr (STEP == 8) return dpp_i32<kDppMirror>(v);
    else return __shfl_xor(v, STEP, kWave);
}

// (cost, index) argmin over aligned groups of L lanes; ties go to the lower index, so the
// pair order is total and the result does not depend on the reduction tree.  All lanes of a
// group end with the group's result.
template <int STEP>
__device__ __forceinline__ void argmin_stage(double &c, int &j)
{
    double oc = partner_f64<STEP>(c);
    int oj = partner_i32<STEP>(j);
    bool take = (oc < c) || (oc == c && oj < j);
    c = take ? oc : c;
    j = take ? oj : j;
}

template <int L>
__device__ __forceinline__ void group_argmin(double &c, int &j)
{
    if constexpr (L > 1) argmin_stage<1>(c, j);
    if constexpr (L > 2) argmin_stage<2>(c, j);
    if constexpr (L > 4) argmin_stage<4>(c, j);
    if constexpr (L > 8) argmin_stage<8>(c, j);
    if constexpr (L > 16) argmin_stage<16>(c, j);
    if constexpr (L > 32) argmin_stage<32>(c, j);
}

// Minimum of two doubles without the NaN canonicalisation the C library semantics would add
// (costs are never NaN here).
__device__ __forceinline__ double fast_min_f64(double a, double b)
{
    double r;
    asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Argmin over aligned groups of L lanes, every lane holding its own best (cost, index) with
// index = 0x7FFFFFFF when it has no candidate: the costs are min-reduced, then the indices of
// the lanes whose cost equals the minimum are min-reduced, which is the tie rule "lowest
// index".  A group whose costs are all +inf resolves to its lowest candidate index.  Returns
// the winning index in every lane of the group.
template <int L>
__device__ __forceinline__ int group_argmin_two_pass(double c, int j)
{
    double m = c;
    if constexpr (L > 1) m = fast_min_f64(m, partner_f64<1>(m));
    if constexpr (L > 2) m = fast_min_f64(m, partner_f64<2>(m));
    if constexpr (L > 4) m = fast_min_f64(m, partner_f64<4>(m));
    if constexpr (L > 8) m = fast_min_f64(m, partner_f64<8>(m));
    if constexpr (L > 16) m = fast_min_f64(m, partner_f64<16>(m));
    if constexpr (L > 32) m = fast_min_f64(m, partner_f64<32>(m));
    int t = (c == m) ? j : 0x7FFFFFFF;
    if constexpr (L > 1) t = min(t, partner_i32<1>(t));
    if constexpr (L > 2) t = min(t, partner_i32<2>(t));
    if constexpr (L > 4) t = min(t, partner_i32<4>(t));
    if constexpr (L > 8) t = min(t, partner_i32<8>(t));
    if constexpr (L > 16) t = min(t, partner_i32<16>(t));
    if constexpr (L > 32) t = min(t, partner_i32<32>(t));
    return t;
}

// DPP shifts for scans: value of the lane `D` below inside the 16-lane row (0.0 where there is
// none), of lane 15 of the previous row (rows 1 and 3 only), and of lane 31 (rows 2 and 3 only).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_shift_f64(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xF, true);
    return __hiloint2double(hi, lo);
}

// Segmented inclusive scan of `v` over the wave: lanes are grouped into runs that begin at the
// lanes flagged in `heads` (bit 0 must be set); every lane ends with the sum of its run up to
// and including itself, added in a fixed order (row-local shifts 1, 2, 4, 8, then the carry of
// the previous row, then the carry of the lower half).  `start` is the lane at which this
// lane's run begins.
__device__ __forceinline__ double segmented_scan_f64(double v, int start, int lane)
{
    const int l16 = lane & 15;
    const int row_base = lane & ~15;
    // row-local: the source lane must be inside the row and inside the run
    double t = dpp_shift_f64<0x111, 0xF>(v);            // row_shr:1
    if (l16 >= 1 && lane - 1 >= start) v = v + t;
    t = dpp_shift_f64<0x112, 0xF>(v);                   // row_shr:2
    if (l16 >= 2 && lane - 2 >= start) v = v + t;
    t = dpp_shift_f64<0x114, 0xF>(v);                   // row_shr:4
    if (l16 >= 4 && lane - 4 >= start) v = v + t;
    t = dpp_shift_f64<0x118, 0xF>(v);                   // row_shr:8
    if (l16 >= 8 && lane - 8 >= start) v = v + t;
    // carry of the previous row into rows 1 and 3 (their runs may begin in that row)
    t = dpp_shift_f64<0x142, 0xA>(v);                   // row_bcast:15
    if ((lane & 16) != 0 && start < row_base) v = v + t;
    // carry of the lower half into rows 2 and 3
    t = dpp_shift_f64<0x143, 0xC>(v);                   // row_bcast:31
    if (lane >= 32 && start < 32) v = v + t;
    return v;
}

// Sums of eight per-lane values over the 64 lanes, all eight at once: three exchange steps
// inside every group of 8 lanes halve the number of values a lane carries (a lane keeps the
// half its lane bit selects and adds the partner's copy of it), three more steps add the eight
// groups.  Returns the total of value number  4*bit2 + 2*bit0 + bit1  of the lane id (see
// tile_row_of_lane); the order of the additions is the same on every run.
__device__ __forceinline__ double wave_sum8(const double (&a)[8], int lane)
{
    const bool s2 = (lane & 4) != 0;
    double v4[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const double keep = s2 ? a[4 + j] : a[j];
        const double give = s2 ? a[j] : a[4 + j];
        v4[j] = keep + dpp_f64<kDppHalfMirror>(give);     // partner 7 - l: the other bit 2
    }
    const bool s0 = (lane & 1) != 0;
    double v2[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const double keep = s0 ? v4[2 + j] : v4[j];
        const double give = s0 ? v4[j] : v4[2 + j];
        v2[j] = keep + dpp_f64<kDppXor1>(give);
    }
    const bool s1 = (lane & 2) != 0;
    const double keep = s1 ? v2[1] : v2[0];
    const double give = s1 ? v2[0] : v2[1];
    double v = keep + dpp_f64<kDppXor2>(give);
    v = v + dpp_f64<0x128>(v);                            // row_ror:8, lane ^ 8
    v = v + __shfl_xor(v, 16, kWave);
    v = v + __shfl_xor(v, 32, kWave);
    return v;
}

// The first three steps of wave_sum8 alone: sums inside every aligned group of 8 lanes.  Lane l
// ends with the total, over its group, of value number tile_row_of_lane(l).
__device__ __forceinline__ double group8_sum8(const double (&a)[8], int lane)
{
    const bool s2 = (lane & 4) != 0;
    double v4[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const double keep = s2 ? a[4 + j] : a[j];
        const double give = s2 ? a[j] : a[4 + j];
        v4[j] = keep + dpp_f64<kDppHalfMirror>(give);
    }
    const bool s0 = (lane & 1) != 0;
    double v2[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const double keep = s0 ? v4[2 + j] : v4[j];
        const double give = s0 ? v4[j] : v4[2 + j];
        v2[j] = keep + dpp_f64<kDppXor1>(give);
    }
    const bool s1 = (lane & 2) != 0;
    const double keep = s1 ? v2[1] : v2[0];
    const double give = s1 ? v2[0] : v2[1];
    return keep + dpp_f64<kDppXor2>(give);
}

__device__ __forceinline__ int tile_row_of_lane(int lane)
{
    return ((lane >> 2) & 1) * 4 + (lane & 1) * 2 + ((lane >> 1) & 1);
}

__device__ __forceinline__ double wave_max(double v)
{
    v = fmax(v, partner_f64<1>(v));
    v = fmax(v, partner_f64<2>(v));
    v = fmax(v, partner_f64<4>(v));
    v = fmax(v, partner_f64<8>(v));
    v = fmax(v, partner_f64<16>(v));
    v = fmax(v, partner_f64<32>(v));
    return v;
}

// max(x[first], x[first + STRIDE], ...) over the entries below n (0 when there is none; the
// entries are not negative): eight loads are requested side by side, so that the count of trips
// to memory is an eighth of the count of entries.
template <int STRIDE>
__device__ __forceinline__ double max_of_strided(const double *x, int n, int first)
{
    double m = 0.0;
    for (int base = first; base < n; base += 8 * STRIDE) {
        double v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int b = base + q * STRIDE;
            v[q] = x[b < n ? b : n - 1];
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) m = fmax(m, v[q]);
    }
    return m;
}

// Block-wide max for blocks of up to 1024 threads; `red` is shared scratch of >= 16 doubles.
// Returns the maximum in every thread.
__device__ __forceinline__ double block_max(double v, double *red)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wid = threadIdx.x >> 6;
    const int nw = (blockDim.x + kWave - 1) >> 6;
    v = wave_max(v);
    __syncthreads();
    if (lane == 0) red[wid] = v;
    __syncthreads();
    double r = red[0];
    for (int w = 1; w < nw; ++w) r = fmax(r, red[w]);
    return r;
}

}  // namespace nimble

// Launchers of the planner kernels.  Every launcher only enqueues on `stream`.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace nimble {

// Device-side view of one topology plus the workspace of one solve.
struct DeviceTopo {
    int32_t E, K, P;
    int64_t nnz;
    int64_t rev_len;   // padded length of rev_entry
    int32_t pmax, lmax;
    int32_t n_chunks;
    bool cost_max;
    // forward CSR
    const int32_t *comm_ptr;   // [K+1]
    const int32_t *path_ptr;   // [P+1]
    const int32_t *path_links; // [nnz]
    // reverse CSR (rows padded to 4 entries)
    const int32_t *rev_ptr;    // [E+1]
    const uint32_t *rev_entry; // [rev_ptr[E]]
    const int32_t *chunk_begin, *chunk_end; // [n_chunks]
    const int32_t *link_chunk_ptr;          // [E+1]
    const double *invcap;      // [E]
    // state of the plan in flight
    double *len, *price, *S;   // [E]
    uint8_t *choice;           // [K+1], choice[K] = 0xFF (padding sentinel)
    uint32_t *count;           // [P]
    double *partial;           // [n_chunks]
    double *scalars;           // [0] = 1/rho, [1..] = per-block maxima of S
    int32_t n_update_blocks;
};

// ---- streaming regime: one launch per phase ------------------------------------------------
void launch_init(const DeviceTopo &t, hipStream_t s);
void launch_width(const DeviceTopo &t, const double *demand, hipStream_t s);
void launch_argmin(const DeviceTopo &t, hipStream_t s);
void launch_load_reduce(const DeviceTopo &t, const double *demand, hipStream_t s);
void launch_update(const DeviceTopo &t, double eps, hipStream_t s);
void launch_epilogue(const DeviceTopo &t, int32_t iters, double *splits, double *lambda,
                     hipStream_t s);

// ---- resident regime: one workgroup per plan, all iterations in one kernel ------------------
// Bytes of LDS one plan needs (state only) and the bytes of the topology copy.
size_t resident_state_bytes(const DeviceTopo &t);
size_t resident_topo_bytes(const DeviceTopo &t);
bool resident_fits(const DeviceTopo &t);
hipError_t launch_resident(const DeviceTopo &t, int32_t batch, const double *demand, double eps,
                           int32_t iters, double *splits, double *lambda, hipStream_t s);

}  // namespace nimble

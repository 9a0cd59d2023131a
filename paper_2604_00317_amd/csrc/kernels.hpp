// Launchers of the planner kernels.  Every launcher only enqueues on `stream`.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace nimble {

// Device-side view of one topology plus the workspace of one solve.
// One step of the adaptive solve (sigma = 1 / max u; S += sigma u; len *= 1 + eps sigma u; the
// prices; W += sigma), a thread per link position.
struct AdApplyArgs {
    int E;
    double eps;
    int n_u_blocks;                 // maxima in block_max_u
    const double *block_max_u, *u_pos, *invcap_pos;
    const int32_t *pos_link;
    double *len, *price, *S;
    int32_t *flags;
    double *ascal, *sigma_log, *block_max_s;
    double *len_id_new;             // the new lengths once more, by link id
};

// A record kernel that runs while the step of the iteration before is still pending: its
// scanning workgroups compute every price they need from the lengths before that step, the
// normalised loads and the step (all by link id), with the very operations of the step; further
// workgroups of the same launch (its first apply_blocks) apply the step to the stored state.
struct FoldArgs {
    AdApplyArgs ap;
    const double *len_id;           // lengths by link id before the pending step
    const double *u_id;             // normalised loads by link id
    const double *invcap;           // 1 / capacity by link id
    int apply_blocks;               // the first workgroups of the launch apply the step
};
struct NoFold {
    int unused;
};

struct DeviceTopo {
    int32_t E, K, P;
    int64_t nnz;
    int32_t pmax, lmax;
    bool cost_max;
    // forward CSR
    const int32_t *comm_ptr;   // [K+1]
    const int32_t *path_ptr;   // [P+1]
    const int32_t *path_links; // [nnz]
    // forward CSR repacked into self-contained 4 KiB records (n_records = 0: not available)
    int32_t n_records;
    int32_t rec_stride;        // 8-bit link indices per candidate path
    int32_t rec_max_links;     // largest link table of any record
    int32_t rec_lanes;         // lanes per commodity in the record kernel (0: automatic)
    int32_t rec_lane_major;    // 1: record bodies are laid out lane by lane (k_argmin_recl)
    int32_t rec_table16;       // 1: 16-bit link tables, 3.5 KiB records
    int32_t rec_around_l2;     // records read around the L2: 1, 0, or -1 (by their total size)
    int32_t rec_per_wave;      // records a wave walks in the record kernel (0: default)
    const uint8_t *records;
    // dictionary layout of the records (rec_dict = 1): 1 KiB records sorted by body, the bodies
    // once each in rec_dict_words, and the runs of records the waves of the record kernel walk
    int32_t rec_dict;          // 1: records name their body in a dictionary
    int32_t n_bodies;
    const uint32_t *rec_dict_words;   // [n_bodies * 768]
    int32_t n_rec_chunks;      // waves of the record kernel
    const int4 *rec_chunks;    // [n_rec_chunks] first record, records, body, 0: one body per run
    // reverse CSR of 8-byte (commodity, window | mask) pairs, rows padded to 2 pairs
    int64_t rev_pairs;         // padded number of pairs
    int32_t rev_row_max;       // longest reverse row in pairs (without padding)
    int32_t resident_generic;  // 1: the resident regime keeps to its LDS-only kernel
    int32_t alg1_thread_per_problem;   // 1: Algorithm 1 keeps to its thread-per-problem kernel
    const int32_t *rev_ptr;    // [E+1], in pairs
    const uint32_t *rev_pair;  // [2 * rev_pairs]
    // streaming layout of the reverse rows: one flat array of octets (base id | flags, 8
    // masks) walked 64 at a time, plus chunked single pairs for commodities with > 32
    // candidates; every slot of partial[] receives one partial sum
    int32_t n_passes;           // flat octets / 64
    int32_t n_schunks, n_slots;
    const uint32_t *oct_base;   // [64 * n_passes]
    const uint32_t *oct_mask;   // [8 * 64 * n_passes]
    const int32_t *pass_first_slot;   // [n_passes]
    const int32_t *pos_link;          // [E] link whose row comes i-th in the flat array
    const int32_t *pos_slot_ptr;      // [E+1] octet slots of position i
    // link blocks of the fused reduce + update kernel (n_blocks = 0: separate kernels)
    int32_t n_blocks;
    const int32_t *blk_desc;          // [8 * n_blocks]: first position, end position, first
                                      // pass, end pass, first slot, 0, 0, 0
    // blocks of link groups (tiled layouts; n_gblocks = 0: separate reduce and update kernels)
    int32_t n_gblocks;
    const int32_t *gblk_desc;         // [16 * n_gblocks]: positions, passes, octet slots, other
                                      // slots, tile items, strip items (first and end each)
    int32_t gblk_max_slots;           // most partial-sum slots of a block (LDS of the kernel)
    int32_t gblk_waves;               // waves per workgroup of the kernel: 4, 8 or 16
    const uint32_t *single_pair;      // [2 * padded singles]
    const int32_t *schunk_begin, *schunk_end, *schunk_slot;   // [n_schunks], pair units
    const int2 *pos_xslot;            // [E] first and end of the piece, strip and single-chunk
                                      // slots of the link at position i
    // tile work items: up to 8 dense (link, window of 512 commodities) pieces of one window
    int32_t n_tile_items;
    const int32_t *tile_desc;         // [32 * n_tile_items]
    const uint32_t *tile_mask;        // [512 * (dense pieces + 1)]
    const uint8_t *tile_pres;         // [64 * (uniform items + 1)] presence bytes
    int32_t tile_item_cost;           // weight of an item against an octet pass (wave split)
    // strip items: 8 units of 8 octets shared by up to 8 links each
    int32_t n_strip_items;
    const uint32_t *strip_base;       // [64 * (items + 1)] per lane
    const uint64_t *strip_pres;       // [64 * (items + 1)] per lane
    const uint32_t *strip_mask;       // [64 * (items + 1)] per unit and row
    const int32_t *strip_slot;        // [64 * (items + 1)] per unit and row
    double *demand1n;                 // [K rounded up to whole windows] demands by id
    double *demand1t;                 // [K rounded up to whole windows] demands by id, and
    double *demand2t;                 // [sigma_size] by sigma number, both window-transposed
    // second numbering of the commodities for the sigma octets, with sigma-ordered copies of
    // the choices and the demands
    int32_t sigma_size;
    const int32_t *sigma;      // [K], -1 = none
    uint8_t *choice2;          // [sigma_size]
    double *demand2;           // [sigma_size]
    const double *invcap;      // [E] by link id
    const double *invcap_pos;  // [E] by position in the flat order of the rows
    // state of the plan in flight: price by link id (the candidate scan gathers from it);
    // len and S by position in the streaming and persistent regimes
    double *len, *price, *S;   // [E]
    uint8_t *choice;           // [K rounded up to whole windows, + 8] (entries from K on are
                               // only read for empty masks or padding pairs)
    uint32_t *count;           // [P]
    double *partial;           // [n_slots]
    double *scalars;           // [0] = 1/rho, [1..] = per-block maxima of S (update or link blocks)
    // plans a launch of the streaming kernels covers (grid.y) and the byte distances between
    // their state blocks and between their choice rows; 1 and anything for a single plan
    int32_t batch;
    size_t state_stride, row_stride;
    const int32_t *stop_flag;  // adaptive solve: kernels return at once when this word is set
    const FoldArgs *fold;         // adaptive solve: when not null, the record kernel applies the
                                  // step of the iteration before on the fly (see FoldArgs)
    int32_t batch_kernel;      // tuning: 0 four plans per workgroup in the fused reduce + update
                               // of a batch, 1 the single-plan kernel for every plan
    int32_t n_update_blocks;
    int32_t update_lanes;      // lanes per link in the length update: 4 or 16
    int32_t reduce_blocks;     // 256-thread blocks of the link-load reduce (fills the chip once)
    int32_t rec_blocks;        // most workgroups of the record kernel (resident at once)
};

void launch_stream_read(const void *buf, size_t bytes, void *sink, hipStream_t s);
// workgroups of the dictionary record kernel a compute unit holds at once (0: not that kernel)
int record_kernel_blocks_per_cu(const DeviceTopo &t);
int lanes_per_commodity(int pmax);   // power of two >= pmax, at most 64

// ---- streaming regime: one launch per phase ------------------------------------------------
// len_in: link lengths to start from, by link id (null: all 1)
void launch_init(const DeviceTopo &t, const double *demand, const double *len_in, hipStream_t s);
// the lengths after the last iteration, by link id
void launch_export_len(const DeviceTopo &t, double *len_out, hipStream_t s);
void launch_width(const DeviceTopo &t, const double *demand, hipStream_t s);
// `choice` is the row the choices of this iteration are written to / read from (the
// topology's own array, or a row of the per-iteration choice log); `count` may be null when
// the choices are logged.
void launch_argmin(const DeviceTopo &t, uint8_t *choice, uint32_t *count, hipStream_t s);
void launch_load_reduce(const DeviceTopo &t, const uint8_t *choice, const double *demand,
                        hipStream_t s);
void launch_histogram(const DeviceTopo &t, const uint8_t *log, size_t stride, int32_t iters,
                      double *splits, hipStream_t s);
void launch_update(const DeviceTopo &t, double eps, hipStream_t s);
// reduce and update in one launch for tiled layouts cut into blocks of link groups
// (t.n_gblocks > 0): every per-wave maximum of S goes to scalars[1 + block * gblk_waves + wave]
void launch_group_reduce_update(const DeviceTopo &t, const uint8_t *choice, double eps,
                                hipStream_t s);
// the same up to the normalised loads (adaptive step): u by position and one maximum of u per
// wave; returns the number of maxima written
int launch_group_reduce_u(const DeviceTopo &t, const uint8_t *choice, double *u_pos, double *u_id,
                          double *block_max_u, hipStream_t s);
// reduce and update in one launch; only for topologies with link blocks (t.n_blocks > 0)
void launch_reduce_update(const DeviceTopo &t, const uint8_t *choice, const double *demand,
                          double eps, hipStream_t s);
void launch_epilogue(const DeviceTopo &t, int32_t iters, const uint32_t *count, double *splits,
                     double *lambda, hipStream_t s);

// ---- resident regime: one workgroup per plan, all iterations in one kernel ------------------
// Bytes of LDS one plan needs (state only) and the bytes of the topology copy.
size_t resident_state_bytes(const DeviceTopo &t);
size_t resident_topo_bytes(const DeviceTopo &t);
bool resident_fits(const DeviceTopo &t);
bool resident_in_registers(const DeviceTopo &t);   // the resident regime keeps the topology in registers
// which kernel the resident regime runs for `batch` plans: 0 none (does not fit), 1 a thread per
// commodity and per link with the lists in LDS, 2 the same with the lists in registers, 3 lanes
// sharing commodities and links (one plan per workgroup), 4 the same with the lists in registers
int resident_kernel_kind(const DeviceTopo &t, int batch);
// rough time of one iteration of the resident regime for `batch` plans, in microseconds
double resident_iteration_us(const DeviceTopo &t, int batch);
hipError_t launch_resident(const DeviceTopo &t, int32_t batch, const double *demand, double eps,
                           int32_t iters, double *splits, double *lambda, hipStream_t s);

// ---- persistent regime: one kernel per solve, grid barriers between the phases -------------
// `sync_words` is device memory of persistent_sync_bytes() bytes owned by the topology.
// `spin_limit` bounds every barrier wait (polls); when it expires the solve is abandoned and
// lambda is written as NaN.
size_t persistent_sync_bytes();
hipError_t launch_persistent(const DeviceTopo &t, void *sync_words, int n_cu,
                             unsigned int spin_limit, const double *demand, double eps,
                             int32_t iters, double *splits, double *lambda, hipStream_t s);

// ---- probe of grid-wide barriers (benchmark only) -------------------------------------------
// `work` is device memory of barrier_probe_bytes(blocks) bytes; `out` is device int32 [32].
size_t barrier_probe_bytes(int max_blocks);
hipError_t launch_barrier_probe(int kind, int blocks, int threads, int rounds,
                                unsigned int spin_limit, int n_xcd, void *work, int *out,
                                hipStream_t s);

// ---- adaptive-step variant of the streaming regime --------------------------------------------
// Device state of one adaptive solve (owned by the topology, sized for max_iters).
struct AdaptiveState {
    int32_t *flags;            // [0] stop flag, [1] iterations made
    double *ascal;             // [0] W = sum of sigma, [1] bound of this check, [2] best bound,
                               // [3] lambda
    double *chunk;             // [ceil(K/256) + ceil(E/256)] chunk sums of alpha and D
    double *u_pos;             // [E] normalised loads by position
    double *u_id;              // [E] the same by link id
    double *len_id[2];         // [E] each: lengths by link id, written in turn by the steps
    double *block_max_u;       // [ceil(E/16)]
    double *block_max_s;       // [ceil(E/256)]
    double *sigma_log;         // [max_iters]
    const int32_t *pos_of_link;  // [E] position of every link in the flat order
    int32_t *host_words;       // pinned host memory the device writes: [0] stopped, [1] checks
                               // made (the device's address of it)
    int32_t *host_words_host;  // the host's address of the same words
};
void launch_ad_reset(const AdaptiveState &a, hipStream_t s);
// the weak-duality bound under the prices the choices in `choice` were made with
void launch_ad_bound(const DeviceTopo &t, const AdaptiveState &a, const uint8_t *choice,
                     const double *demand, hipStream_t s);
// u, sigma, S, len, price, W from the slot partials of the reduce
void launch_ad_update(const DeviceTopo &t, const AdaptiveState &a, double eps, hipStream_t s);
// link-block fabrics: reduce to normalised loads in one launch (u by position and one maximum
// per wave; returns the number of maxima), then the step from those
int launch_reduce_u(const DeviceTopo &t, const uint8_t *choice, double *u_pos, double *u_id,
                    double *block_max_u, hipStream_t s);
// (the lengths by link id go to len_id_new)
void launch_ad_apply(const DeviceTopo &t, const AdaptiveState &a, double eps, int n_u_blocks,
                     double *len_id_new, hipStream_t s);
// The step applied inside the next iteration's record kernel instead: the arguments of that
// step, and whether this topology's record kernel can take them.
AdApplyArgs ad_apply_args(const DeviceTopo &t, const AdaptiveState &a, double eps, int n_u_blocks,
                          double *len_id_new);
bool record_kernel_folds(const DeviceTopo &t, bool whenever_possible);
// lengths by link id from the lengths by position
void launch_ad_len_id(const DeviceTopo &t, double *len_id, hipStream_t s);
// lambda = max S / W; with `check` (the number of this check, from 1; 0: none) also the best
// bound and the stop test, both published to a.host_words
void launch_ad_lambda(const DeviceTopo &t, const AdaptiveState &a, double gap, int check,
                      hipStream_t s);
hipError_t launch_ad_histogram(const DeviceTopo &t, const AdaptiveState &a, const uint8_t *log,
                               size_t stride, double *splits, double *lambda, hipStream_t s);

// ---- Algorithm 1 (sequential sweep), one thread per problem of a batch -----------------------
// LDS one workgroup (64 problems, down to 8 for larger topologies) needs, and whether it fits
// the LDS of a compute unit.
size_t alg1_lds_bytes(const DeviceTopo &t);
bool alg1_fits(const DeviceTopo &t);
// lambda[b] is NaN when problem b still had traffic left after max_sweeps sweeps.
hipError_t launch_alg1(const DeviceTopo &t, int32_t batch, const double *demand, double phi,
                       double chi, int32_t max_sweeps, double *flows, double *lambda,
                       int32_t *sweeps, hipStream_t s);

// ---- plan post-processing: fractions -> bytes per path in whole chunks ----------------------
hipError_t launch_quantize(const DeviceTopo &t, const double *demand, const double *splits,
                           int32_t iters, int64_t chi, double theta, double *flows,
                           hipStream_t s);

}  // namespace nimble

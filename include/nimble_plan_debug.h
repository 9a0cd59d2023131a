/*
 * nimble_plan_debug.h -- helpers for tests and benchmarks of the planner library.
 *
 * Nothing here is needed to plan: the product ABI is include/nimble_plan.h.  These entry
 * points time single phases, exercise failure paths from the host, and expose the host-side
 * layout builders to tests that run without a GPU.
 */
#ifndef NIMBLE_PLAN_DEBUG_H
#define NIMBLE_PLAN_DEBUG_H

#include "nimble_plan.h"

#ifdef __cplusplus
extern "C" {
#endif

/* 1 if nimble_plan_solve_adaptive applies the step of an iteration inside the record kernel of
 * the next one on this topology (two launches per iteration; the prices of the scan are formed
 * from the lengths before the step, the loads and the step, with the operations of the step
 * itself), 0 if in a launch of its own (three), -1 for a NULL handle.  Both give the same
 * bits. */
int32_t nimble_topo_adaptive_folds(const nimble_topo_t *topo);

/* 1 if the resident regime would run this topology with one commodity and one link per thread,
 * their candidate lists and reverse rows held in registers (at most 8 candidates of at most 2
 * links per commodity, at most 16 (commodity, mask) pairs per link); 0 if it keeps everything
 * in LDS; -1 for a NULL handle.  Both kernels return the same bits. */
int32_t nimble_topo_resident_in_registers(const nimble_topo_t *topo);

/*
 * Benchmark helper: enqueue `reps` back-to-back launches of one phase of the streaming regime
 * on `hip_stream`, without changing the plan state another solve depends on
 * (phase 0: path-cost gather + argmin, 1: link-load reduce, 2: length update with step 0; on
 * topologies whose reduce and update run as one kernel phase 1 is that kernel and phase 2 is
 * refused with NIMBLE_ERR_INVALID).  The state must have been initialised by a previous
 * streaming-regime nimble_plan_solve on this topology with the same d_traffic.  Used to time a
 * kernel's average launch with HIP events.
 */
nimble_status_t nimble_debug_run_phase(nimble_topo_t *topo, int32_t phase, int32_t reps,
                                       const double *d_traffic, void *hip_stream);

/*
 * Benchmark helper: enqueue `reps` back-to-back launches of a plain streaming read of the first
 * `bytes` (rounded down to 16) of d_buf on `hip_stream` -- 16-byte loads, nothing computed.  The
 * benchmark times it to state the read bandwidth this machine reaches next to the published
 * peak.  d_buf and d_sink are device pointers, 16-byte aligned; d_sink is 16 bytes that the
 * kernel may write.  NIMBLE_ERR_INVALID for NULL or misaligned pointers, bytes < 16, reps < 1.
 */
nimble_status_t nimble_debug_stream_read(const void *d_buf, int64_t bytes, int32_t reps,
                                         void *d_sink, void *hip_stream);

/*
 * Benchmark helper: enqueue one cooperative kernel of (compute units x blocks_per_cu, rounded
 * down to a multiple of 8) workgroups of `threads` threads that makes 2 x rounds grid-wide
 * barriers and checks after every other one that a word another workgroup wrote before the
 * barrier has arrived.  kind: 0 one arrival counter, relaxed agent-scope atomics, data
 * exchanged with agent-scope stores and loads; 1 the same counter between agent-scope fences,
 * data exchanged with ordinary stores and loads; 2 one counter per XCD (by the hardware's XCC id)
 * and a global one, all workgroups poll one generation word; 3 as 2, but only the last arriver
 * of an XCD polls the global word and releases the others through a word of their own XCD; 4 no
 * read-modify-write: every workgroup stores its round into its own word of a flag array and
 * its first wave reads the whole array until all words have arrived (at most 2048 workgroups);
 * 5 as 2 followed by an acquire fence at agent scope, the data written at agent scope and read
 * with ordinary loads.
 * Every wait gives up after spin_limit polls.  d_work: device memory of work_bytes >= 16384 +
 * 128 per workgroup.  d_out: device int32 [32] out: [0] words that had not arrived, [1] 1 if a
 * wait expired, [2..17] workgroups that ran on XCC id 0..15, [18] rounds completed.  Timed with
 * HIP events by the caller: duration / (2 x rounds) is the cost of one barrier.
 */
nimble_status_t nimble_debug_barrier_probe(int32_t kind, int32_t blocks_per_cu, int32_t threads,
                                           int32_t rounds, uint32_t spin_limit, void *d_work,
                                           int64_t work_bytes, int32_t *d_out, void *hip_stream);

/*
 * Test helpers for the allocation-failure paths.  nimble_debug_fail_allocation(n): of the
 * device allocations the library makes from now on, the one after the next n fails as if the
 * device were out of memory (n = 0: the very next one; -1 switches the hook off; it switches
 * itself off after it has fired).  nimble_debug_fail_host_allocation(): the next
 * nimble_topo_create fails in its host-side build as if the host were out of memory.
 * nimble_debug_live_allocations(): device allocations of the library that have not been freed.
 * A call that fails this way returns NIMBLE_ERR_ALLOC and leaves nothing allocated that was
 * not allocated before it.
 */
nimble_status_t nimble_debug_fail_allocation(int32_t nth);
void nimble_debug_fail_host_allocation(void);
int64_t nimble_debug_live_allocations(void);

/*
 * Test helper for the persistent regime: every grid-wide barrier of that kernel waits at most
 * `polls` polls of its arrival counter (default 2^22, about a second).  When a wait expires the
 * solve is abandoned -- every workgroup leaves the kernel at its next poll, d_splits is left
 * undefined and d_lambda[0] is written as NaN.  With polls = 0 the first barrier that is not
 * already complete gives up, which lets a test exercise the abandon path without hanging
 * anything.
 */
nimble_status_t nimble_debug_set_spin_limit(nimble_topo_t *topo, uint32_t polls);

/*
 * Host-only helper (no device call): the reverse CSR exactly as nimble_topo_create builds it,
 * unpadded.  rev_ptr is host [n_links+1] out; rev_comm / rev_path are host [nnz] out (the
 * commodity and the candidate index inside that commodity of every incidence).  Returns the
 * same validation codes as nimble_topo_create.
 */
nimble_status_t nimble_host_build_reverse(int32_t n_links, int32_t n_comm,
                                          const int32_t *comm_path_ptr, int32_t n_paths,
                                          const int32_t *path_link_ptr,
                                          const int32_t *path_links, int32_t *rev_ptr,
                                          int32_t *rev_comm, int32_t *rev_path);

/*
 * Host-only helper (no device call): the same reverse CSR, but decoded from the streaming
 * layout the link-load kernel walks (flat octets under the two commodity numberings, slot
 * flags, chunked single pairs), with every row sorted by (commodity, path).  Must equal the
 * output of nimble_host_build_reverse.
 */
nimble_status_t nimble_host_build_reverse_streaming(int32_t n_links, int32_t n_comm,
                                                    const int32_t *comm_path_ptr,
                                                    int32_t n_paths,
                                                    const int32_t *path_link_ptr,
                                                    const int32_t *path_links, int32_t *rev_ptr,
                                                    int32_t *rev_comm, int32_t *rev_path);

/*
 * Host-only helper (no device call): repacks the forward CSR into the self-contained records
 * of 3.5 or 4 KiB (1 KiB plus a dictionary of bodies where many records share their bodies)
 * the path-cost kernel streams (a run of consecutive commodities, the record's
 * own link table, and a fixed number of 8-bit link-table indices per candidate, laid out lane by
 * lane or record-major) exactly as nimble_topo_create does, and reads every incidence back
 * through them.  links_out is host
 * [nnz] out and must equal path_links; path_record is host [n_paths] out, the record of every
 * path (records numbered by their first commodity); n_records_out receives the number of records, or 0 when the topology does not fit
 * records (a path longer than 8 links, padding above 1.5x, more than 254 distinct links or
 * 4 KiB for a single commodity) -- then the untiled kernel is used and the other outputs are
 * not written.
 */
nimble_status_t nimble_host_records_roundtrip(int32_t n_links, int32_t n_comm,
                                            const int32_t *comm_path_ptr, int32_t n_paths,
                                            const int32_t *path_link_ptr,
                                            const int32_t *path_links, int32_t *links_out,
                                              int32_t *path_record, int32_t *n_records_out);

/*
 * Host-only helper (no device call): sizes of the device layout nimble_topo_create would build.
 * out is host int64 [22]: (commodity, window) pairs of the reverse CSR; octets (groups of 8
 * consecutive commodity ids with one mask each); single pairs; octets numbered by the second
 * commodity numbering; single-pair chunks; partial-sum slots; forward records; indices per
 * candidate in a record; link blocks of the fused reduce + update kernel (0: not used); octets
 * including padding; dense (link, window of 512 commodities) pieces; work items of up to 8
 * pieces; pieces stored as one mask plus presence bits; strip items (8 units of 8 octets x up
 * to 8 links that share them); links whose row lives in a strip; 1 if the bodies of the forward
 * records are laid out lane by lane (the record kernel then keeps them in registers), else 0;
 * 1 if those bodies are kept once each in a dictionary (records of 1 KiB that name their body),
 * else 0; the number of distinct bodies in that dictionary; blocks of link groups (tiled layouts
 * whose links can be cut into groups with tile items, strip units and octets of their own: the
 * reduce and the length update of a block then run in one workgroup; 0: none); the most
 * partial-sum slots and the most work items of such a block; the bodies of the dictionary whose
 * quads all have the two-by-two product shape (nine price reads per quad instead of twenty).
 */
nimble_status_t nimble_host_layout_stats(int32_t n_links, int32_t n_comm,
                                         const int32_t *comm_path_ptr, int32_t n_paths,
                                         const int32_t *path_link_ptr,
                                         const int32_t *path_links, int64_t *out);

/*
 * Host-only helper (no device call): which kernel the resident regime would run for one plan
 * of this topology.  kernel_out receives 0 when the per-plan state does not fit the LDS of a
 * compute unit (the resident regime is refused), 1 for the kernel that keeps candidate lists
 * and reverse rows in LDS and lets a thread stride over commodities and links, 2 for the kernel
 * that gives every thread exactly one commodity and one link and keeps their lists in
 * registers (at most 8 candidates of at most 2 links, at most 16 pairs per link, and no more
 * commodities or links than the 1024 threads of a workgroup), 3 for the kernel that gives the
 * plan a whole workgroup whose lanes share commodities (a candidate each) and links (16 lanes
 * per reverse row), 4 for that kernel with the lanes' lists in registers (paths of at most 5
 * links, at most 64 pairs per link, at most 256 links and 4096 / lanes-per-commodity
 * commodities).
 */
nimble_status_t nimble_host_resident_kernel(int32_t n_links, int32_t n_comm,
                                            const int32_t *comm_path_ptr, int32_t n_paths,
                                            const int32_t *path_link_ptr,
                                            const int32_t *path_links, int32_t *kernel_out);

#ifdef __cplusplus
}
#endif
#endif /* NIMBLE_PLAN_DEBUG_H */

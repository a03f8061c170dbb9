/*
 * nezha_sim.h -- C ABI of the MI355X (gfx950) reduction engine of a multi-rail
 * allreduce, after Nezha (arXiv 2405.17870).
 *
 * The message of one allreduce is split across rails (member networks) into
 * contiguous slices, each rail allreduces its slice over the N nodes with a
 * ring, and the arithmetic of that -- the sum of the nodes' gradient buffers --
 * is what this library executes on one GPU, with all N simulated nodes'
 * buffers resident in device memory.  No network transport is involved.
 *
 * Conventions for every entry point
 *   - Return value: nz_status.  Nothing is thrown, the process is never
 *     aborted.  All validation happens before any GPU work is enqueued: on a
 *     status other than NZ_OK nothing was launched and no output was written
 *     (NZ_ERR_HIP excepted: a launch the runtime refuses may follow launches
 *     of the same call that were accepted).
 *   - "host" pointers are ordinary process memory, read (or written) before
 *     the call returns; the caller may free them immediately afterwards.
 *   - "device" pointers are HIP device memory owned by the caller.  The
 *     library never allocates, frees or returns device memory.  Device
 *     buffers must stay alive until `stream` has run past the call's work.
 *   - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *     GPU work is asynchronous with respect to the host.
 *   - Every device buffer base must be aligned to 256 bytes
 *     (NZ_ERR_ALIGNMENT otherwise); together with the 256-byte alignment of
 *     rail boundaries this makes every rail slice start on a 256-byte address.
 *   - Limits: n_nodes <= NZ_MAX_NODES, n_rails <= NZ_MAX_RAILS
 *     (NZ_ERR_UNSUPPORTED beyond them).
 *   - Entry points are re-entrant; concurrent calls must not share output
 *     buffers.  Results are bitwise reproducible.
 *   - Debugging aid: if the environment variable NZ_DEBUG is set to anything
 *     but "" or "0" at the time of a call, an entry point that takes a
 *     stream waits for that stream before it returns and reports a
 *     failure of the execution itself as NZ_ERR_HIP.  Such calls cannot be
 *     captured in a HIP graph.  It is the library's only global setting.
 */
#ifndef NEZHA_SIM_H
#define NEZHA_SIM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NZ_MAX_NODES 128u
#define NZ_MAX_RAILS 8u
#define NZ_RAIL_ALIGN_BYTES 256u

typedef enum {
    NZ_OK = 0,
    NZ_ERR_INVALID_ARG = 1, /* null pointer, zero count, zero weight sum, bad enum, overflow */
    NZ_ERR_ALIGNMENT = 2,   /* a device buffer base is not 256-byte aligned               */
    NZ_ERR_UNSUPPORTED = 3, /* over a limit, or buffers overlap in a way not allowed      */
    NZ_ERR_CAPACITY = 4,    /* a destination buffer is too small                          */
    NZ_ERR_HIP = 5          /* the HIP runtime reported an error (see nz_last_hip_error)  */
} nz_status;

typedef enum { NZ_F32 = 0, NZ_BF16 = 1, NZ_F16 = 2, NZ_I32 = 3 } nz_dtype;

typedef enum { NZ_RING_STEPWISE = 0, NZ_FUSED = 1 } nz_mode;

/* Static text for a status code. */
const char *nz_status_str(nz_status s);

/* Text of the last HIP error seen by the calling thread ("" if none). */
const char *nz_last_hip_error(void);

/* Size in bytes of one element of `dtype`, 0 for an unknown dtype. */
uint32_t nz_dtype_bytes(nz_dtype dtype);

/*
 * Rail partition.  (Sec. 3.4: each network is handed one (ptr, data_length)
 * slice; Sec. 3.5: the Load Balancer derives each rail's pointer from its data
 * volume; Sec. 4.3, under Eq. 5: the proportions sum to one.)
 *
 * Splits [0, n_elems) into n_rails contiguous ranges, in rail order, with
 * lengths proportional to the integer weights ratios[k] (host, n_rails
 * entries, sum > 0).  rail_off (host, caller-owned, n_rails + 1 entries)
 * receives the boundaries in elements: rail k is [rail_off[k], rail_off[k+1]).
 * rail_off[0] = 0, rail_off[n_rails] = n_elems; an interior boundary is the
 * proportional point n_elems * (ratios[0] + .. + ratios[k-1]) / sum, rounded
 * down to a multiple of 256 bytes; a rail of weight zero gets an empty range
 * (a boundary preceded by the whole weight sum is n_elems).  All arithmetic
 * is exact integer arithmetic.  elem_bytes must be 2 or 4.  Pure host
 * function, no GPU involved.
 */
nz_status nz_rail_partition(uint64_t n_elems, uint32_t elem_bytes, const uint32_t *ratios,
                            uint32_t n_rails, uint64_t *rail_off);

/* The same with a caller-chosen alignment (a positive multiple of elem_bytes). */
nz_status nz_rail_partition_ex(uint64_t n_elems, uint32_t elem_bytes, uint32_t align_bytes,
                               const uint32_t *ratios, uint32_t n_rails, uint64_t *rail_off);

/*
 * Ring segments.  (Sec. 2.1.1, Eq. 1: a ring allreduce over N workers handles
 * the message in N pieces of M/N.)
 *
 * Cuts every rail range into n_nodes consecutive segments whose lengths differ
 * by at most one element, longer ones first, with no alignment of their own.
 * rail_off: host, n_rails + 1 non-decreasing entries.  seg_off: host,
 * caller-owned, [n_rails][n_nodes + 1] row-major; segment j of rail k is
 * [seg_off[k][j], seg_off[k][j+1]).  Pure host function.
 */
nz_status nz_segment_map(const uint64_t *rail_off, uint32_t n_rails, uint32_t n_nodes,
                         uint64_t *seg_off);

/*
 * Allreduce (sum) of n_nodes gradient buffers, every rail in the same launch.
 * (Sec. 4.2: the aggregation phase of the allreduce; Sec. 2.1.1, Eq. 1: the
 * ring schedule; Sec. 4.1: rails work on disjoint slices concurrently.)
 *
 * node_bufs: host array of n_nodes device pointers, each n_elems elements of
 * `dtype`: node i's gradients.  out_bufs: host array of n_nodes device
 * pointers receiving node i's result; on completion every out buffer holds,
 * for every element x, the sum over i of node_bufs[i][x].
 *
 * The message is partitioned by nz_rail_partition(ratios) and each rail by
 * nz_segment_map; segment j of a rail is the unit of the ring schedule.
 *   NZ_FUSED: every element is read once from all nodes, summed in fp32
 *     registers (int32: wrapping integer add) in a fixed blocked pairwise
 *     order that depends on n_nodes only, rounded once to `dtype` (nearest
 *     even) and written once to every distinct output buffer.  With fewer
 *     than seven distinct output buffers (fewer than 17 if they span more
 *     than NZ_HBM_REGION_BYTES of addresses, so that they cannot lie in one
 *     memory region: see nz_hbm_place), or while the outputs together
 *     take less than 128 MiB, this is one launch over the whole message
 *     (the sums do not depend on where rails and segments begin; the unit
 *     of work is a 4 KiB tile).  Larger jobs run as a short pipeline of
 *     launches over pieces of at most 24 MiB of the participating rails: launch c sums
 *     piece c into one of the output buffers (the one farthest from the
 *     inputs) and copies piece c - 1 from there (re-read through the L2
 *     caches) to the other output buffers one after the other, because a
 *     single write stream at a time is what HBM sustains best.  The result
 *     is bitwise the same either way.
 *   NZ_RING_STEPWISE: 2 (n_nodes - 1) launches, one per ring step, in stream
 *     order.  Node r sends to node (r+1) mod N; in reduce-scatter step s it
 *     sends segment (r - s) mod N and the receiver stores
 *     dtype(fp32(received) + fp32(own)); in allgather step s it sends segment
 *     (r + 1 - s) mod N and the receiver overwrites its copy.  Partials are
 *     held in `dtype` between steps, as on a wire.
 *
 * Aliasing: out_bufs[i] == node_bufs[i] (in place) is allowed in both modes.
 * In NZ_FUSED, out_bufs entries may repeat (each distinct buffer is written
 * once; all equal = one shared result) and an output buffer may be any node's
 * input buffer, whole: every input of an element is read before any output
 * of that element is written.  Partial overlap of a written buffer with any
 * other buffer, and in NZ_RING_STEPWISE any output that repeats or is another
 * node's input, is NZ_ERR_UNSUPPORTED.  n_elems == 0 returns NZ_OK without
 * launching.
 */
nz_status nz_allreduce_sim(const void *const *node_bufs, uint32_t n_nodes, uint64_t n_elems,
                           const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype, nz_mode mode,
                           void *const *out_bufs, void *stream);

/*
 * How many kernel launches nz_allreduce_sim issues for these arguments (host
 * only; useful to size a HIP graph, and to turn a call's time into time per
 * launch).  n_distinct_outputs: how many different buffers out_bufs names;
 * outputs_span_bytes: from the start of the lowest of them to the end of the
 * highest (0 if not known: taken to lie close together).
 * Same argument checks as nz_allreduce_sim as far as they apply.
 */
nz_status nz_allreduce_launches(uint32_t n_nodes, uint64_t n_elems, const uint32_t *ratios,
                                uint32_t n_rails, nz_dtype dtype, nz_mode mode,
                                uint32_t n_distinct_outputs, uint64_t outputs_span_bytes,
                                uint64_t *launches);

/*
 * The two halves of the allreduce on their own.  (Sec. 2.1.1, Eq. 1: a ring
 * allreduce is N - 1 reduce-scatter steps followed by N - 1 allgather steps,
 * each moving M/N per worker; the same section names the phase decomposition
 * that ZeRO-style training applies to it.)
 *
 * nz_reduce_scatter_sim: same arguments as nz_allreduce_sim.  On completion,
 * for every rail and every segment j, out_bufs[(j - 1) mod N] holds the sum
 * over all nodes of segment j -- node r owns segment (r + 1) mod N, as after
 * the reduce-scatter steps of the ring.  The other elements of the output
 * buffers are unspecified: NZ_FUSED (one launch, each segment read from all
 * nodes and written to its owner only) leaves them untouched, NZ_RING_STEPWISE
 * (N - 1 launches) leaves the ring's partial sums in them.  The summation
 * order, and so every bit of the owned segments, is that of nz_allreduce_sim
 * in the same mode.  Output buffers must be pairwise distinct; out_bufs[i] may
 * alias node_bufs[i] only.
 *
 * nz_allgather_sim: in place on bufs (host array of n_nodes device pointers,
 * pairwise distinct, non-overlapping).  On entry node r's buffer holds valid
 * data in segment (r + 1) mod N of every rail; on exit every buffer holds
 * every segment.  NZ_RING_STEPWISE: N - 1 launches (step s copies segment
 * (r + 1 - s) mod N from node r to node r + 1); NZ_FUSED: each segment read
 * from its owner and stored to the other N - 1 buffers, in one launch for
 * the rails whose segments are at least 16 KiB long -- one destination buffer
 * after the other over pieces of at most 24 MiB of a rail (all passes but the
 * first read the piece from the L2 caches) -- and one more launch, if there
 * are such rails, for those with shorter segments (all destinations from one
 * read).
 * dtype only fixes the element size.
 *
 * nz_reduce_scatter_sim followed by nz_allgather_sim on its outputs gives
 * bitwise the result of nz_allreduce_sim in the same mode.
 */
nz_status nz_reduce_scatter_sim(const void *const *node_bufs, uint32_t n_nodes, uint64_t n_elems,
                                const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype,
                                nz_mode mode, void *const *out_bufs, void *stream);

nz_status nz_allgather_sim(void *const *bufs, uint32_t n_nodes, uint64_t n_elems,
                           const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype, nz_mode mode,
                           void *stream);

/*
 * Ring_Chunked allreduce.  (Evaluation, GPT-3 scalability experiment: the
 * chunked variant of the ring named there.)
 *
 * The ring of NZ_RING_STEPWISE with every segment transfer cut into pieces of
 * at most chunk_elems elements (> 0) that travel as a pipeline: with P =
 * ceil(longest segment / chunk_elems) pieces and the 2 (N - 1) ring steps
 * numbered u = 0 .. 2N - 3, launch number w carries step u = w - c of every
 * piece c that has such a step, so piece c is always one step behind piece
 * c - 1: P + 2 (N - 1) - 1 launches in stream order.  Pieces cover disjoint
 * elements, so the piece-steps inside one launch are independent, and every
 * element goes through the same additions in the same order as in
 * NZ_RING_STEPWISE: the result is bitwise that mode's.
 * Arguments, aliasing rules and errors as nz_allreduce_sim in ring mode.
 */
nz_status nz_allreduce_sim_chunked(const void *const *node_bufs, uint32_t n_nodes, uint64_t n_elems,
                                   const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype,
                                   uint64_t chunk_elems, void *const *out_bufs, void *stream);

/*
 * Fault tolerance.  (Sec. 4.4: when a member network fails, its (ptr,
 * data_length) is handed to the surviving network that was allocated the most
 * data, which runs the allreduce of that slice after its current task.)
 *
 * nz_failover_target: host only.  alive: host, n_rails flags (non-zero =
 * surviving).  *target receives the surviving rail with the longest range in
 * rail_off (lowest index among equals); NZ_ERR_INVALID_ARG if none survives.
 *
 * nz_allreduce_sim_failover: nz_allreduce_sim with rail failed_rail (<
 * n_rails) failing.  The surviving rails' slices are processed first; the
 * failed rail's slice, still cut into the same N segments, follows on the
 * same stream as a second pass (one more launch in NZ_FUSED, 2 (N - 1) more
 * in NZ_RING_STEPWISE).  The result is bitwise that of nz_allreduce_sim.
 * takeover_rail (host, may be NULL) receives nz_failover_target's choice.
 * NZ_ERR_INVALID_ARG if failed_rail is the only rail.
 */
nz_status nz_failover_target(const uint64_t *rail_off, uint32_t n_rails, const uint8_t *alive,
                             uint32_t *target);

nz_status nz_allreduce_sim_failover(const void *const *node_bufs, uint32_t n_nodes, uint64_t n_elems,
                                    const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype,
                                    nz_mode mode, void *const *out_bufs, uint32_t failed_rail,
                                    uint32_t *takeover_rail, void *stream);

/*
 * Data allocation scheme: how to share a message among rails.  (Sec. 4.3.
 * Eq. 4: cold start, all data over the best single rail,
 * T_cold = min_i (T_setup_i + S / B_i).  Eq. 5: hot start with shares alpha
 * summing to one, T_hot = max_i (T_setup_i + alpha_i S / B_i).  Eq. 6: the
 * threshold size at which the two are equal.  Eq. 7, 8: the shares are found
 * by descent on T_hot from latency-derived starting shares.)
 *
 * Host only.  rails: host, n_rails models (startup latency in seconds >= 0,
 * effective bandwidth in bytes per second > 0).  A rail that is given nothing
 * does not take part in Eq. 5.  nz_balance returns the minimiser of Eq. 5
 * directly (the point Eq. 7's descent converges to): the rails that take part
 * all finish at the same time and a rail whose startup latency alone exceeds
 * that time sits out.  If sharing does not beat the best single rail the
 * state is cold and that rail gets everything.
 *   alpha      (host, n_rails doubles, may be NULL): the shares, sum 1;
 *   ratios     (host, n_rails, may be NULL): the shares as integer weights
 *              summing to NZ_RATIO_SCALE, ready for nz_rail_partition;
 *   t_cold, t_hot (may be NULL): Eq. 4 and Eq. 5 for the returned shares;
 *   best_rail  (may be NULL): the rail of Eq. 4;
 *   hot        (may be NULL): 1 in the hot-start state, 0 in cold start.
 * nz_balance_threshold: the message size (bytes) up to which the state is
 * cold (infinity for a single rail).
 *
 * nz_balance_iterate: the shares by the paper's own method, for
 * msg_bytes > 0.  Start: Eq. 8, alpha_i = (T - T_i) / (T (R - 1)) with T_i
 * rail i's latency under a uniform split of the message, T their sum and R
 * the number of rails.  Step (Eq. 7): the derivative of T_hot is S / B_w on
 * the slowest rail w that takes part and zero elsewhere, so a step takes a
 * share from w; the share goes to the rail f that would finish first (a
 * rail holding nothing counts with its startup latency), and the step
 * length is the exact line search along that direction: w and f finish
 * together; if w's startup latency alone reaches that common time, w hands
 * over all it has and sits out.  The iteration ends when no rail would finish
 * before the slowest one, when a step would move less than half a unit of
 * the data-length table (2^-21 of the message), or after max_iterations
 * steps.  T_hot never rises from one step to the next.  alpha, ratios, t_hot
 * as for nz_balance (each may be NULL); iterations (may be NULL) receives the
 * number of steps taken.  No cold/hot decision is made here: compare t_hot
 * with nz_balance's t_cold.
 */
#define NZ_RATIO_SCALE (1u << 20)

typedef struct {
    double setup_s;     /* T_setup: startup latency, seconds */
    double bytes_per_s; /* B: effective bandwidth            */
} nz_rail_model;

nz_status nz_balance(const nz_rail_model *rails, uint32_t n_rails, double msg_bytes, double *alpha,
                     uint32_t *ratios, double *t_cold, double *t_hot, uint32_t *best_rail, int *hot);

nz_status nz_balance_threshold(const nz_rail_model *rails, uint32_t n_rails,
                               double *threshold_bytes);

nz_status nz_balance_iterate(const nz_rail_model *rails, uint32_t n_rails, double msg_bytes,
                             uint32_t max_iterations, double *alpha, uint32_t *ratios,
                             double *t_hot, uint32_t *iterations);

/*
 * Network efficiency and the real-time efficiency ratio.  (Sec. 2.1.2, Eq. 2:
 * delta = T_theoretical / T_actual = 1 / (1 + T_setup / (S / B)).  Sec. 2.2.1,
 * Eq. 3: rho = (S_i delta_i / That_i) / (S_j delta_j / That_j), the quotient
 * of the throughputs of two networks that carry S_i and S_j bytes of one
 * message; data is split across rails only while rho does not exceed the
 * tolerance threshold tau, which the paper sets to 5.)
 *
 * Host only.
 * nz_net_efficiency: *delta receives Eq. 2 for one rail on msg_bytes > 0.
 * nz_efficiency_ratio: rail i carries alpha[i] * msg_bytes (alpha: host,
 * n_rails shares >= 0 with a positive sum, normalised to sum one; NULL = an
 * even split).  *rho receives the largest quotient of Eq. 3 over the pairs of
 * rails that carry something, i.e. the highest throughput over the lowest
 * (>= 1; exactly 1 when fewer than two rails carry data).  Whether to split is
 * the caller's decision: compare *rho with NZ_TOLERANCE_TAU.
 * NZ_ERR_INVALID_ARG: a null pointer, an invalid model, msg_bytes not positive
 * and finite, a negative or non-finite share, all shares zero.
 */
#define NZ_TOLERANCE_TAU 5.0

nz_status nz_net_efficiency(const nz_rail_model *rail, double msg_bytes, double *delta);

nz_status nz_efficiency_ratio(const nz_rail_model *rails, uint32_t n_rails, double msg_bytes,
                              const double *alpha, double *rho);

/*
 * Pack: stage rail segments into contiguous send buffers.  (Sec. 3.2: data
 * moves from the user's UnboundBuffer into a rail's contiguous Buffer.)
 *
 * For every node m, copies segments seg_ids[0..n_segs) of rail `rail` of
 * node_bufs[m] (device) back to back, in list order and without padding, to
 * the start of send_bufs[m] (device).  seg_off: host, the table of
 * nz_segment_map for n_nodes nodes; seg_ids: host, values < n_nodes, may
 * repeat, n_segs <= NZ_MAX_NODES; elem_bytes 2 or 4.  send_capacity_bytes is
 * the size of every send buffer (NZ_ERR_CAPACITY if the packed size exceeds
 * it); packed_bytes (host, may be NULL) receives the packed size per node.
 * One launch for all nodes.  Source and destination must not overlap.
 */
nz_status nz_pack(const void *const *node_bufs, uint32_t n_nodes, const uint64_t *seg_off,
                  uint32_t n_rails, uint32_t rail, const uint32_t *seg_ids, uint32_t n_segs,
                  uint32_t elem_bytes, void *const *send_bufs, uint64_t send_capacity_bytes,
                  uint64_t *packed_bytes, void *stream);

/*
 * Unpack: the inverse of nz_pack.  (Sec. 3.2: results return from the rail's
 * Buffer to the UnboundBuffer.)  Scatters the start of send_bufs[m] back into
 * the listed segments of node_bufs[m]; bytes of node_bufs outside the listed
 * segments are not touched.  seg_ids must not repeat (NZ_ERR_INVALID_ARG).
 */
nz_status nz_unpack(const void *const *send_bufs, uint32_t n_nodes, const uint64_t *seg_off,
                    uint32_t n_rails, uint32_t rail, const uint32_t *seg_ids, uint32_t n_segs,
                    uint32_t elem_bytes, void *const *node_bufs, void *stream);

/*
 * Placement of large buffers in HBM.  (No passage of the paper: a property of
 * the MI355X memory system, for callers that can choose where their buffers
 * live.)
 *
 * The 288 GiB of HBM3E behave as three consecutive regions of
 * NZ_HBM_REGION_BYTES with DRAM banks of their own.  Kernels that stream
 * through many buffers run fastest when the buffers they write are spread
 * over the regions and the buffers they only read are kept together (the
 * fused allreduce of 32 x 670 MB: 82 % of the HBM peak against 75 % with
 * everything in one region).  The library allocates nothing; a caller who
 * wants this layout makes ONE device allocation of arena_bytes as the first
 * large allocation of the process (the driver lays it out from the start of
 * HBM) and asks here where to put its buffers inside it.
 *
 * nz_hbm_place: host only, pure arithmetic.  used: host, NZ_HBM_REGIONS
 * counters owned by the caller, all zero before the first call: the bytes
 * already handed out in each region; updated on success.  Places `count`
 * buffers of bytes_each bytes: with spread != 0 buffer i goes to region
 * (first_region + i) mod NZ_HBM_REGIONS (written buffers), otherwise all go to
 * first_region one after the other (buffers that are only read).  offsets
 * (host, count entries) receives byte offsets into the arena, each a multiple
 * of 2 MiB; a margin of 1 GiB is kept clear on both sides of a region
 * boundary.  NZ_ERR_CAPACITY if a buffer does not fit its region (nothing is
 * changed then); NZ_ERR_INVALID_ARG for a null pointer, first_region out of
 * range or a counter that is not a multiple of 2 MiB.
 */
#define NZ_HBM_REGIONS 3u
#define NZ_HBM_REGION_BYTES (96ull << 30)

nz_status nz_hbm_place(uint64_t arena_bytes, uint64_t *used, uint32_t count, uint64_t bytes_each,
                       int spread, uint32_t first_region, uint64_t *offsets);

#ifdef __cplusplus
}
#endif
#endif /* NEZHA_SIM_H */

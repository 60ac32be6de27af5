/*
 * r2ccl.h -- C ABI of the MI355X-native hot path of a resilient ring all-reduce.
 *
 * One rank's share of a chunked ring all-reduce as described in the R2CCL paper:
 *   (a) partition each chunk over the server's NIC channels in proportion to their
 *       bandwidth, leaving failed channels empty, and partition again whenever the
 *       channel state changes mid-collective (Sec. 2.1 multi-channel partition;
 *       Sec. 5.1 R2CCL-Balance and "Overhead Analysis"; Sec. 4.3 chunk-granular
 *       resume; Sec. 4.2 recovery by re-probing);
 *   (b) the fused reduce-copy that adds the chunk arriving from the ring predecessor
 *       into the local buffer and writes the result into the per-channel send staging
 *       buffers (Sec. 2.1 "persistent GPU kernels over precomputed channels";
 *       Sec. 4.3 Technique II, NIC-registered send buffers);
 *   (c) the ring schedule, reduce-scatter followed by all-gather (Sec. 5.2), run over
 *       R simulated ranks whose buffers all live in one GPU's memory.
 *
 * Conventions
 *   - Every function returns an R2_* code (0 = success); nothing throws or aborts.
 *   - "device" pointers are HIP device memory of the current device, "host" pointers
 *     are ordinary process memory.  The caller owns every buffer.  The library allocates no
 *     device memory.  The only state it keeps for the life of the process, per device: the side
 *     streams and events of r2_split_allreduce_sim / r2_recursive_allreduce_sim, created at their
 *     first call, and two device arrays that are part of its code (see r2_ring_allreduce_sim_static
 *     and r2_partition).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work on it and return; r2_partition alone waits for its result.
 *   - Data buffers (rank buffers, stage buffers) must be 16-byte aligned.
 *   - Argument checks that need no device access happen before any HIP call, so a
 *     bad call returns R2_ERR_INVALID even on a machine without a GPU.
 */
#ifndef R2CCL_H
#define R2CCL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    R2_OK = 0,
    R2_ERR_INVALID = -1,            /* null pointer, zero or too many channels/ranks, bad alignment,
                                       size not a whole number of elements/chunks, bad enum, bad table */
    R2_ERR_NO_HEALTHY_CHANNEL = -2, /* every channel failed or has zero bandwidth (Appendix C: at
                                       least one healthy NIC must remain)                           */
    R2_ERR_OVERFLOW = -3,           /* a size computation does not fit 64 bits                       */
    R2_ERR_CAPACITY = -4,           /* a slice exceeds its stage buffer, the workspace is too small, or
                                       host memory for a call's own bookkeeping ran out              */
    R2_ERR_DEVICE = -5              /* the HIP runtime reported an error                             */
};

#define R2_MAX_CHANNELS 64 /* one wavefront lane and one mask bit per channel */
#define R2_MAX_RANKS 64

typedef enum { R2_F32 = 0, R2_BF16 = 1 } r2_dtype;
enum { R2_OP_SUM = 0, R2_OP_COPY = 1, R2_OP_SUM_FORWARD = 2, R2_OP_SUM_SEND = 3 };
enum { R2_PHASE_RS = 1, R2_PHASE_AG = 2, /* both = all-reduce */
       /* the other collectives R2CCL-Balance serves; each on its own only */
       R2_PHASE_SENDRECV = 4,   /* point-to-point to the ring successor */
       R2_PHASE_BROADCAST = 8,  /* ring broadcast from desc->root       */
       R2_PHASE_REDUCE = 16,    /* ring reduce to desc->root            */
       R2_PHASE_ALLTOALL = 32,  /* pairwise exchange of R blocks        */
       /* a flag for the ring phases (RS, AG or both): every ring link has tables of its own instead of
          one table per transmission for all ranks; see r2_ring_rails_sim */
       R2_PHASE_LINKS = 64 };
enum { R2_SCHED_AUTO = 0, R2_SCHED_STEPS = 1, R2_SCHED_FUSED = 2, R2_SCHED_STEPS_OVERLAP = 3 };

/* Static, human-readable text for a return code. */
const char *r2_strerror(int code);

/* ---------------------------------------------------------------------------------------------
 * (a) Channel partition -- Sec. 5.1, paragraph R2CCL-Balance.
 *
 * A chunk of `bytes` bytes is cut into n_channels consecutive slices, slice c = bytes
 * [offsets[c], offsets[c+1]).  With e[c] = 0 for a failed channel (bit c of fail_mask set) and
 * weights[c] otherwise, P[c] the sum of e before c, W the sum of all e and U = floor(bytes/align):
 *     offsets[c] = align * floor(U * P[c] / W)   while P[c] < W,
 *     offsets[c] = bytes                         once P[c] == W,        offsets[C] = bytes.
 * Hence failed or zero-bandwidth channels get nothing, healthy ones get their proportional share to
 * within one alignment unit, and the sub-unit tail goes to the last healthy channel.  The arithmetic
 * is exact for any uint32 weights and any 64-bit byte count.  align may be any value >= 1 here; the
 * data-moving calls below additionally need tables cut at multiples of 16 bytes.
 * --------------------------------------------------------------------------------------------- */

/* n_problems independent partitions on the device, one wavefront each, asynchronous.
 *   weights   device [n_problems][n_channels]   bandwidth in integer units (e.g. MB/s)
 *   fail_mask device [n_problems]
 *   bytes     device [n_problems]
 *   offsets   device [n_problems][n_channels+1]  out
 *   status    device [n_problems]                out, R2_OK or R2_ERR_NO_HEALTHY_CHANNEL (then the
 *                                                problem's offsets are all zero); may be NULL
 * n_problems == 0 is a no-op. */
int r2_partition_device(const uint32_t *weights, const uint64_t *fail_mask, const uint64_t *bytes,
                        uint32_t n_channels, uint32_t align, uint32_t n_problems,
                        uint64_t *offsets, int32_t *status, void *stream);

/* One partition with HOST pointers: weights[n_channels] in, offsets[n_channels+1] out.  Runs the
 * same device code, on the default stream, and waits for it (so it cannot be captured into a graph).
 * Convenience call; it allocates nothing: the row is written to a small device array inside the
 * library and copied back, and concurrent calls take turns. */
int r2_partition(const uint32_t *weights, uint64_t fail_mask, uint32_t n_channels, uint64_t bytes,
                 uint32_t align, uint64_t *offsets);

/* In-flight failover plan -- Sec. 4.3 (live migration: every NIC is registered on every buffer, and
 * send buffers stay intact until completion, so the unfinished part is retransmitted from where it
 * lies) with the proportional shares of Sec. 5.1.
 *
 * A chunk was staged with table `offsets` while the channels of mask_before were down; during the
 * transmission the channels of mask_after (a superset) are down.  No data moves: for every newly
 * failed channel f, its slice -- bytes [0, len_f) of stage buffer f -- is shared out over the channels
 * still healthy by the partition rule above (weights, mask_after, align), so that healthy NIC c
 * carries bytes [plan[f][c], plan[f][c+1]) of buffer f.  The receiver's layout does not change.
 *   offsets     device [n_problems][n_channels+1]
 *   weights     device [n_problems][n_channels]
 *   mask_before, mask_after  device [n_problems]
 *   plan        device [n_problems][n_channels][n_channels+1] out; rows of channels that did not
 *               newly fail, or whose slice is empty, are all zero
 *   status      device [n_problems], optional; the kernel lowers it to R2_ERR_NO_HEALTHY_CHANNEL if a
 *               non-empty slice has nobody left to carry it (that row is zero).  It never writes
 *               R2_OK: clear it beforehand.
 * One wavefront per (problem, channel); asynchronous; allocates nothing. */
int r2_rollback_plan_device(const uint64_t *offsets, const uint32_t *weights,
                            const uint64_t *mask_before, const uint64_t *mask_after,
                            uint32_t n_channels, uint32_t align, uint32_t n_problems,
                            uint64_t *plan, int32_t *status, void *stream);

/* ---------------------------------------------------------------------------------------------
 * (b) Fused reduce-copy on one chunk -- Sec. 2.1 (collective kernels over channels), Sec. 4.3
 *     Technique II (send/receive staging buffers).
 *
 * `incoming` is the chunk the ring predecessor staged: the concatenation over c of the first
 * in_offsets[c+1]-in_offsets[c] bytes of in_stage[c] (each slice is packed at offset 0 of its
 * channel's buffer).  Then
 *     in_stage == NULL              : v = local                 (copy-send; op is ignored)
 *     op == R2_OP_SUM               : v = incoming + local      (fp32 add; bf16 is widened to fp32,
 *                                                                added, rounded to nearest even)
 *     op == R2_OP_COPY              : v = incoming
 *     in_stage != NULL              : local <- v
 *     out_stage != NULL             : v is cut by out_offsets and slice c written to out_stage[c]+0
 *     op == R2_OP_SUM_FORWARD       : as R2_OP_SUM for local, but the outgoing stage gets `incoming`
 *                                     itself, not the sum (the relay step of the broadcast of
 *                                     Sec. 5.2); needs both stages
 *     op == R2_OP_SUM_SEND          : v = incoming + local goes to the outgoing stage only and local
 *                                     stays as it was (a hop of a Reduce towards its root: a rank
 *                                     that passes the sum on does not keep it); needs both stages
 * in_stage and out_stage may not both be NULL.
 *   local       device, `bytes` bytes (a whole number of elements), 16-byte aligned for full speed;
 *               an address that is only element-aligned is handled one element at a time
 *   in_stage    HOST array of n_channels device pointers (copied at call time), each 16-byte aligned
 *               and `stage_capacity` bytes long; likewise out_stage
 *   in_offsets  DEVICE table of n_channels+1 entries, as written by r2_partition_device; likewise
 *               out_offsets.  The tables are read by the kernel, so they may still be in flight on
 *               `stream` when this is called
 *   status      device int32, optional.  The kernel checks both tables (start at 0, end at `bytes`,
 *               non-decreasing, interior cuts multiples of 16, every slice <= stage_capacity); on a
 *               bad table it moves no data and stores R2_ERR_INVALID or R2_ERR_CAPACITY there.
 *               It never writes R2_OK: clear it beforehand.
 * local, the in_stage buffers and the out_stage buffers must not overlap. */
int r2_reduce_copy(void *local, uint64_t bytes, r2_dtype dtype, int op,
                   const void *const *in_stage, const uint64_t *in_offsets,
                   void *const *out_stage, const uint64_t *out_offsets,
                   uint32_t n_channels, uint64_t stage_capacity, int32_t *status, void *stream);

/* ---------------------------------------------------------------------------------------------
 * (c) Ring all-reduce over R simulated ranks -- Sec. 5.2 (reduce-scatter then all-gather),
 *     Sec. 5.1 (same channel state for the whole server), Sec. 4.3 (chunk-granular progress).
 *
 * Each rank buffer holds n_elems elements = n_slabs slabs of n_ranks ring chunks.  Per slab the
 * ring takes J fused steps (2R-1 for all-reduce, R for a single phase); at step j rank r works on
 * ring chunk (r - j) mod R [all-gather alone: (r + 1 - j) mod R]:
 *     j = 0                     copy-send:        stage <- local
 *     reduce-scatter steps      local <- incoming + local, staged onward
 *     all-gather steps          local <- incoming,         staged onward
 *     j = J-1                   local updated, nothing staged
 * and `incoming` is what rank r-1 staged at step j-1.  A stage write at step j of slab l is
 * transmission t = l*(J-1) + j.  The channel state in force at t is the last epoch with
 * t_start <= t; it decides the partition of that transmission, for all ranks alike, and the reader
 * uses the writer's table.  A failure "at step k" is an epoch with t_start = k; a recovery is a
 * later epoch with the bit cleared.  The result in the rank buffers does not depend on the epochs.
 *
 * R2_PHASE_SENDRECV is the point-to-point case of R2CCL-Balance (Sec. 5.1 applies the redistribution
 * to every collective; Sec. 8 and Appendix E measure it on SendRecv): rank r sends its whole buffer
 * to rank r+1 and receives rank r-1's into a second buffer.  A slab is then one message chunk of
 * n_elems/n_slabs elements, there are J = 2 steps (j = 0: stage <- send buffer; j = 1: receive
 * buffer <- incoming) and one transmission per slab, t = l, so that a channel failing after chunk k
 * re-partitions chunks k, k+1, ...  `rank_bufs` then holds 2R pointers: R send buffers, then R
 * receive buffers (r2_sendrecv_sim takes them apart).  Only the step schedule runs it.
 *
 * The remaining collectives of the table of strategies in Sec. 5 keep their ring schedule as well
 * (Sec. 5.1, "Overhead Analysis": the volume a server must send does not change, only its cut over
 * the healthy NICs).  A slab is one message chunk of n_elems/n_slabs elements; the hop sent at step j
 * of chunk l is transmission t = l*(R-1) + j; one rank is active per step:
 *   R2_PHASE_BROADCAST  J = R steps; at step j rank root+j works: j = 0 stages its chunk, the ranks
 *                       after it take the incoming chunk and stage it onward, the last one only takes
 *                       it.  Afterwards every buffer equals the root's.
 *   R2_PHASE_REDUCE     J = R steps; at step j rank root+1+j works: j = 0 stages its chunk, the ranks
 *                       after it stage incoming + their own chunk onward and keep their own buffer as
 *                       it was (R2_OP_SUM_SEND), at j = R-1 the root adds the incoming sum into its
 *                       buffer: root <- x[root+1] + x[root+2] + ... + x[root], folded in that order,
 *                       rounded to the buffer type after every addition.
 *   R2_PHASE_ALLTOALL   (r2_alltoall_sim) a buffer is R blocks of n_slabs chunks; in round k = 1..R-1
 *                       rank r sends its block r+k to rank r+k and receives rank r-k's block r into
 *                       block r-k of its receive buffer, two steps per chunk as for SENDRECV; chunk l
 *                       of round k is transmission (k-1)*n_slabs + l, for every rank alike.  A rank's
 *                       own block is copied without touching a channel.  The run has (R-1)*n_slabs
 *                       internal slabs: that many rows of tables and that many stage buffers per rank.
 * Only the step schedule runs these.
 *
 * Slabs are independent of each other, and so are the bytes of a chunk.  The run is therefore cut
 * into passes -- groups of whole slabs, or, when one slab is too large, byte ranges of its chunks --
 * such that the stage bytes one step writes (over all ranks) stay within stage_window_bytes and can
 * be read back from the Infinity Cache by the next step.  All J steps of a pass run before the next
 * pass starts; one fused step of one pass, for all ranks, is one kernel launch.
 * --------------------------------------------------------------------------------------------- */

typedef struct {
    uint64_t t_start;        /* first transmission index of this state; epochs[0].t_start == 0,
                                strictly increasing                                             */
    uint64_t fail_mask;      /* bit c set = channel c is down                                   */
    const uint32_t *weights; /* HOST array of n_channels bandwidth weights                      */
} r2_epoch;

typedef struct {
    uint32_t n_ranks;    /* R, 2..R2_MAX_RANKS                                                   */
    uint32_t n_slabs;    /* S >= 1, R*S <= 65535 (R2_PHASE_ALLTOALL: R*(R-1)*S <= 65535)         */
    uint32_t n_channels; /* C, 1..R2_MAX_CHANNELS                                                */
    uint32_t align;      /* partition alignment in bytes, a multiple of 16                       */
    uint64_t n_elems;    /* elements per rank, a multiple of R*S (of S for R2_PHASE_SENDRECV,
                            _BROADCAST and _REDUCE); 0 is allowed: nothing to do                 */
    int32_t dtype;       /* r2_dtype                                                             */
    int32_t phases;      /* R2_PHASE_RS, R2_PHASE_AG, both, or one of the other R2_PHASE_*       */
    uint64_t stage_window_bytes; /* stage bytes one launch may write, summed over ranks; 0 = the
                                    library's default (128 MiB, half the Infinity Cache; 256 MiB
                                    for the two-step exchanges, which use one stage parity).
                                    Only changes how the run is cut into passes, never the
                                    result.                                                    */
    int32_t schedule;    /* R2_SCHED_STEPS: one launch per fused step and pass.
                            R2_SCHED_FUSED: one launch takes every column (1 or 2 KiB of each ring chunk)
                            through all steps between two channel-state changes; needs chunks that
                            are a multiple of 16 bytes.
                            R2_SCHED_AUTO (0): FUSED for launch-bound sizes, else STEPS.
                            R2_SCHED_STEPS_OVERLAP: as STEPS, but the run is cut into at least two
                            passes of half the stage window each, and passes are issued in pairs,
                            step by step alternately on the caller's stream and on a library-owned
                            stream (default priority, created once per device, forked off `stream`
                            after the partition launch and joined to it again with events before
                            the call returns to the caller's order): while one pass's launch ramps
                            up or drains, the other's fills the GPU.  Two passes only run side by
                            side if they cover different slabs, or if one channel state holds for
                            the whole run: byte ranges of one slab share its stage buffers, and a
                            pass that is a step ahead under a newer table would overwrite what the
                            other has not read yet.  So with a state that changes on the way the
                            two streams take the even and the odd slabs, and a run of a single slab
                            takes the plain step schedule.  The result is the same as that of
                            R2_SCHED_STEPS.  Never chosen by AUTO; not with R2_PHASE_LINKS.      */
    int32_t root;        /* R2_PHASE_BROADCAST: the rank whose buffer everybody gets;
                            R2_PHASE_REDUCE: the rank that gets the sum; otherwise 0              */
} r2_sim_desc;

/* Pure host arithmetic on a descriptor (0 if the descriptor is invalid). */
uint32_t r2_sim_num_steps(const r2_sim_desc *desc);         /* J                                  */
uint64_t r2_sim_num_transmissions(const r2_sim_desc *desc); /* rows of the tables: S * (J-1), with S
                                                               the internal slabs ((R-1) * n_slabs for
                                                               all-to-all); R times that with
                                                               R2_PHASE_LINKS (one block per link)    */
uint64_t r2_sim_workspace_bytes(const r2_sim_desc *desc);
uint64_t r2_sim_stage_offset(const r2_sim_desc *desc);      /* byte offset of the stage area      */
uint64_t r2_sim_stage_capacity(const r2_sim_desc *desc);    /* bytes per channel buffer           */

/* Workspace (device, 256-byte aligned, >= r2_sim_workspace_bytes) layout:
 *   [0, ...)                 offsets tables  uint64 [r2_sim_num_transmissions][C+1], row t = transmission t
 *                            (with R2_PHASE_LINKS: R blocks of S*(J-1) rows, block r = the link r -> r+1)
 *   [r2_sim_stage_offset)    stage buffers   [2 parities][R][S][C][r2_sim_stage_capacity bytes];
 *                            the transmission of step j uses parity j & 1
 * Stage memory is never initialised or cleared by the library. */

/* Partition every transmission of the run: fills the tables (and, if not NULL, the device array
 * offsets_log [r2_sim_num_transmissions][C+1]) from the epoch list.  Epoch data travels as kernel arguments, so no
 * host-to-device copy is made.  Returns R2_ERR_NO_HEALTHY_CHANNEL, before any launch, if a state
 * that is in force for some transmission has no healthy channel.  Not for R2_PHASE_LINKS, whose
 * tables r2_ring_rails_sim makes. */
int r2_sim_prepare(const r2_sim_desc *desc, const r2_epoch *epochs, uint32_t n_epochs,
                   void *workspace, uint64_t workspace_bytes, uint64_t *offsets_log, void *stream);

/* Number of passes the run is cut into (0 if the descriptor is invalid). */
uint64_t r2_sim_num_passes(const r2_sim_desc *desc);

/* Fused step j (0 <= j < J) of pass p, for every rank: one launch.  rank_bufs is a HOST array of
 * R device pointers.  Needs the tables of r2_sim_prepare and, for j > 0, the stage that step j-1 of
 * the same pass left. */
int r2_sim_step(const r2_sim_desc *desc, void *const *rank_bufs, uint64_t pass, uint32_t step,
                void *workspace, uint64_t workspace_bytes, void *stream);

/* Fused-column schedule: the steps [step_begin, step_end) of every rank and slab in ONE launch.  A
 * workgroup takes a column (1 KiB, or 2 KiB once that fills the GPU) of the ring chunks of one slab through all these steps, one wave
 * per rank, with a workgroup barrier between steps; columns are independent of each other and
 * drift apart in time.  Only valid if, for every slab, the transmissions t of equal parity with
 * step_begin-1 <= t <= step_end-1 all use one channel state: otherwise a column that is ahead could
 * overwrite stage data that another column has not read yet.  (An epoch starting at step c of a
 * slab therefore needs a launch boundary before step c and one before step c+1;
 * r2_ring_allreduce_sim places them.)  The caller is trusted on this.  Needs the tables of
 * r2_sim_prepare and chunk sizes that are a multiple of 16 bytes (R2_ERR_INVALID otherwise; also for
 * R2_PHASE_LINKS, whose fused launches only r2_ring_rails_sim issues). */
int r2_sim_fused_steps(const r2_sim_desc *desc, void *const *rank_bufs, uint32_t step_begin,
                       uint32_t step_end, void *workspace, uint64_t workspace_bytes, void *stream);

/* Which schedule r2_ring_allreduce_sim will use for this descriptor and epoch list: R2_SCHED_STEPS,
 * R2_SCHED_FUSED or R2_SCHED_STEPS_OVERLAP (desc->schedule itself unless that is R2_SCHED_AUTO, or
 * R2_SCHED_STEPS_OVERLAP for a single slab whose channel state changes on the way, which runs as
 * R2_SCHED_STEPS), or a negative R2_ERR code
 * (R2_ERR_INVALID for R2_PHASE_LINKS: ask r2_rails_resolve_schedule).  Host arithmetic only. */
int r2_sim_resolve_schedule(const r2_sim_desc *desc, const r2_epoch *epochs, uint32_t n_epochs);

/* r2_sim_prepare, then the whole collective that desc->phases names, in place on the rank buffers, by
 * desc->schedule: for every pass the steps 0..J-1, or fused launches cut wherever a channel state
 * changes mid-slab. */
int r2_ring_allreduce_sim(const r2_sim_desc *desc, void *const *rank_bufs,
                          const r2_epoch *epochs, uint32_t n_epochs,
                          void *workspace, uint64_t workspace_bytes,
                          uint64_t *offsets_log, void *stream);

/* The ring run when failures strike while a transmission is in flight -- Sec. 4.3, Technique II (a
 * failure may leave a chunk partially transferred; send buffers stay intact until completion and every
 * NIC is registered on every buffer, so the sender rewinds to the first chunk without a completion and
 * retransmits it over the NICs that are left; completed chunks stay as they are) with the shares of
 * Sec. 5.1.
 *
 * As r2_ring_allreduce_sim, plus in_flight: a HOST array of n_epochs bytes (NULL = all zero).
 * in_flight[i] != 0 says that the failures of epoch i strike DURING transmission k = epochs[i].t_start
 * instead of before it:
 *   - transmission k is staged, and read, with the table of the state before the epoch (epoch i-1):
 *     row k of the tables and of offsets_log is that state's partition; the receiver's layout does not
 *     change and no data moves because of the failure;
 *   - the slices of the channels that newly failed are re-carried by the channels the epoch leaves up:
 *     block i of `plans` is the failover plan of that transmission exactly as r2_rollback_plan_device
 *     defines it (offsets = row k, weights = epoch i's, mask_before = epoch i-1's, mask_after = epoch
 *     i's), made by a launch of the same call in front of the run, without a host synchronisation;
 *   - transmissions after k are cut by epoch i's own state, as for an ordinary epoch.
 * An in-flight epoch may only add failures to the state before it (recoveries are found by re-probing
 * between transmissions, Sec. 4.2, and come as ordinary epochs) and cannot be the first epoch:
 * R2_ERR_INVALID otherwise.  One that starts beyond the run has no effect.
 *   plans  DEVICE [n_epochs][n_channels][n_channels+1], out; every row is written, zero for epochs
 *          that are not in flight or start beyond the run, for channels that did not newly fail and for
 *          empty slices.  May be NULL if no epoch is in flight.
 * The result in the rank buffers is the plain run's.  Asynchronous on `stream`; allocates no device
 * memory (a host copy of the epoch list is made for the duration of the call). */
int r2_ring_allreduce_sim_inflight(const r2_sim_desc *desc, void *const *rank_bufs,
                                   const r2_epoch *epochs, const uint8_t *in_flight, uint32_t n_epochs,
                                   void *workspace, uint64_t workspace_bytes, uint64_t *offsets_log,
                                   uint64_t *plans, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): r2_ring_allreduce_sim without the workspace argument.  The tables and the
 * stage area live in a device array inside the library, R2_STATIC_WORKSPACE_BYTES long, which every GPU
 * the library runs on holds from the moment its code is loaded there until the process ends.  A
 * descriptor whose r2_sim_workspace_bytes exceeds that returns R2_ERR_CAPACITY before anything is
 * launched (72 MiB holds the 8-rank bf16 all-reduce of 4 MiB per rank over 8 channels, the largest of
 * the inference sizes).  Same kernels, same result, same other arguments and errors as
 * r2_ring_allreduce_sim; rank buffers and the optional log are still the caller's.  The call makes no
 * hipMalloc/hipFree and calls nothing that allocates; the first call on a device asks the runtime once
 * for the array's address there.  All calls on one GPU share the one array: it keeps what the last call
 * left (no step ever reads bytes its own run has not written, so nothing is cleared), and calls that
 * overlap in time on one GPU -- different streams, different host threads -- race on it: keep them in
 * order on one stream. */
#define R2_STATIC_WORKSPACE_BYTES (72ull << 20)
int r2_ring_allreduce_sim_static(const r2_sim_desc *desc, void *const *rank_bufs,
                                 const r2_epoch *epochs, uint32_t n_epochs,
                                 uint64_t *offsets_log, void *stream);

/* The same call under the name that fits the phases which are no all-reduce (R2_PHASE_BROADCAST,
 * R2_PHASE_REDUCE, a reduce-scatter or an all-gather alone): identical arguments and behaviour. */
int r2_collective_sim(const r2_sim_desc *desc, void *const *rank_bufs,
                      const r2_epoch *epochs, uint32_t n_epochs,
                      void *workspace, uint64_t workspace_bytes,
                      uint64_t *offsets_log, void *stream);

/* Point-to-point under R2CCL-Balance (Sec. 5.1; measured in Sec. 8 "More results on other
 * collectives" and Appendix E): desc->phases must be R2_PHASE_SENDRECV.  Rank r's send buffer
 * (n_elems elements) goes, chunk by chunk through the partitioned stage buffers, into rank r+1's
 * receive buffer; afterwards recv_bufs[r] equals send_bufs[(r-1) mod R] byte for byte whatever the
 * epochs.  Same workspace, epochs, log and passes as r2_ring_allreduce_sim, which this calls with the
 * two pointer lists joined.  Send buffers are only read. */
int r2_sendrecv_sim(const r2_sim_desc *desc, const void *const *send_bufs, void *const *recv_bufs,
                    const r2_epoch *epochs, uint32_t n_epochs, void *workspace, uint64_t workspace_bytes,
                    uint64_t *offsets_log, void *stream);

/* A ring whose servers each have a channel state of their own -- Sec. 5.1 (R2CCL-Balance acts per
 * server: server i spreads what it must send over its own healthy NICs) and Sec. 6 "Topology-Aware
 * Logical Re-ranking" (when node u loses rail r and its neighbour v loses rail r', what they share drops
 * to the rails that survive at both).  desc->phases must be R2_PHASE_LINKS plus the ring phases.
 * rank_bufs are given in ring order (after any re-ranking, e.g. by r2_bridge_rerank).  Rank r has the
 * epoch list rank_epochs[r] (n_rank_epochs[r] entries, the rules of r2_epoch lists, t = l*(J-1) + j as
 * for the plain ring): which of its channels are down from which transmission on, and how fast each
 * is.  The link r -> r+1 carries transmission t of rank r over the channels that are up at both ends at
 * t, cut in proportion to the slower end's weight per channel; rank r+1 reads with that same table.
 * The tables area of the workspace then holds R blocks of S*(J-1) rows, block r = the link r -> r+1
 * (r2_sim_num_transmissions returns R*S*(J-1)), and offsets_log, if not NULL, receives the same.  The
 * result in the rank buffers is the ring's (all-reduce, reduce-scatter or all-gather), whatever the
 * schedules.  rank_epochs, n_rank_epochs and the weights they point to: HOST memory, read during the
 * call only.  R2_ERR_NO_HEALTHY_CHANNEL, before any launch, if a link is left without a channel at
 * some transmission -- which is what re-ranking is for.  desc->schedule as for the plain ring: one
 * launch per step and pass, or fused columns cut wherever some link's table changes within a slab
 * (R2_SCHED_FUSED is R2_ERR_INVALID where ring chunks are no whole 16-byte vectors or where the R
 * links' table rows of one launch, R * steps * ((C+1)*8 + 24) bytes, exceed 56 KiB of LDS; AUTO then
 * takes the step schedule).  Fused launches cut the chunks themselves when all links' states fit one
 * kernel-argument block (32 states, 640 weights); otherwise one partition launch runs in front.
 * Asynchronous on `stream`; allocates no device memory. */
int r2_ring_rails_sim(const r2_sim_desc *desc, void *const *rank_bufs,
                      const r2_epoch *const *rank_epochs, const uint32_t *n_rank_epochs,
                      void *workspace, uint64_t workspace_bytes, uint64_t *offsets_log, void *stream);

/* Which schedule r2_ring_rails_sim will use for this descriptor and these epoch lists: R2_SCHED_STEPS
 * or R2_SCHED_FUSED, or the negative R2_ERR code that call would return before launching.  Host only. */
int r2_rails_resolve_schedule(const r2_sim_desc *desc, const r2_epoch *const *rank_epochs,
                              const uint32_t *n_rank_epochs);

/* All-to-All under R2CCL-Balance (Sec. 5, table of strategies: point-to-point incl. All-to-All;
 * Sec. 5.1): desc->phases must be R2_PHASE_ALLTOALL.  Afterwards block q of recv_bufs[r] equals
 * block r of send_bufs[q] byte for byte, whatever the epochs (a block is n_elems/R elements).  Same
 * workspace, epochs, log and passes as r2_ring_allreduce_sim, which this calls with the two pointer
 * lists joined (so r2_ring_allreduce_sim, r2_collective_sim and r2_sim_step read 2R pointers from
 * rank_bufs for this phase, as for R2_PHASE_SENDRECV).  Send buffers are only read; no receive buffer
 * may be a send buffer.  (Driven step
 * by step with r2_sim_step, only the exchanged blocks move: the own-block copy is part of this call.) */
int r2_alltoall_sim(const r2_sim_desc *desc, const void *const *send_bufs, void *const *recv_bufs,
                    const r2_epoch *epochs, uint32_t n_epochs, void *workspace, uint64_t workspace_bytes,
                    uint64_t *offsets_log, void *stream);

/* ---------------------------------------------------------------------------------------------
 * R2CCL-AllReduce -- Sec. 5.2 ("Partial AllReduce", "R2CCL-AllReduce", "Data Partition Analysis") and
 * Appendix A.
 *
 * Planner (host arithmetic).  n servers of g GPUs; one server has lost the fraction X (0 < X < 1) of
 * its bandwidth.  With the share Y of the data going through partial all-reduce + broadcast the paper's
 * completion time (B = D = 1) is T(Y) = max(T1, T2) + T3, T1 = a(1-Y)/(1-X), T2 = bY/X, T3 = Y/X,
 * a = 2(ng-1)/(ng), b = 2((n-1)g-1)/((n-1)g).  Appendix A: the plain ring is best while
 * X <= ng/(3ng-2); beyond that T is minimal at Y* = X + X(1-X)/(X + (g(n-1)-1)n).
 *   r2_split_plan   writes Y* to *y_star, the threshold to *threshold and whether to split
 *                   (X > threshold, and at least two healthy GPUs remain) to *use_split; any of the
 *                   three may be NULL.  R2_ERR_INVALID for n < 2, g < 1 or X outside (0, 1).
 *   r2_split_time   T(Y) as above (no argument checks).
 * --------------------------------------------------------------------------------------------- */
int r2_split_plan(uint32_t n_servers, uint32_t gpus_per_server, double lost_fraction,
                  int32_t *use_split, double *y_star, double *threshold);
double r2_split_time(uint32_t n_servers, uint32_t gpus_per_server, double lost_fraction, double y);

/* The tail that goes through partial all-reduce + broadcast when the share y of a buffer of n_elems
 * elements does (HOST arithmetic): floor(y * n_elems) rounded down to a multiple of
 * lcm(n_slabs_global * R, n_slabs_partial * (R-1)) * (16 / element size) elements, so that both rings
 * get chunks of whole 16-byte vectors.  Needs n_elems to be a multiple of
 * n_slabs_global * R * (16 / element size); 0 if it is not, or if an argument is invalid. */
uint64_t r2_split_partial_elems(uint32_t n_ranks, uint32_t n_slabs_global, uint32_t n_slabs_partial,
                                int32_t dtype, uint64_t n_elems, double y);

/* The schedule, over R simulated ranks of which `degraded_rank` d is the one with failed NICs.  Every
 * rank buffer is cut in two: the first n_elems - n_partial elements go through a global ring
 * all-reduce over all R ranks (r2_ring_allreduce_sim, channel state of the degraded server, since the
 * ring passes through it); the last n_partial elements go through
 *   1. a partial ring all-reduce over the R-1 healthy ranks, taken in ring order d+1, d+2, ...
 *      (all channels up), and
 *   2. the tailored broadcast: d stages its own tail; each healthy rank in that order adds it to its
 *      partial result and relays it unchanged (R2_OP_SUM_FORWARD); the last healthy rank sends its
 *      finished result back to d, which copies it.  Transfers to or from d are cut by d's channel
 *      state, transfers between healthy ranks by the full state.
 * Afterwards every rank holds, in the tail, fold(healthy ranks in ring order) + x_d, rounded to the
 * buffer type after every addition, and in the head the plain ring all-reduce.
 * n_partial = 0 is the plain all-reduce.  (n_elems - n_partial) * element size must be a multiple
 * of 16; the head must divide into n_slabs_global * R chunks and the tail into
 * n_slabs_partial * (R-1) chunks.  Head and tail run side by side: the global ring on `stream`, the
 * partial ring and its broadcast on a library-owned stream (default priority, created once per
 * device) that is forked off `stream` and joined to it again with events at the end of the call, so
 * the call stays in order on `stream`. */
typedef struct {
    uint32_t n_ranks;         /* R, 3..R2_MAX_RANKS                          */
    uint32_t degraded_rank;   /* d < R                                       */
    uint32_t n_channels;      /* C                                           */
    uint32_t align;           /* partition alignment, a multiple of 16       */
    uint64_t n_elems;         /* elements per rank                           */
    uint64_t n_partial;       /* elements of the tail (partial all-reduce)   */
    int32_t dtype;            /* r2_dtype                                    */
    int32_t schedule;         /* R2_SCHED_AUTO, _STEPS or _FUSED for the two ring runs (they already run
                                 side by side: no R2_SCHED_STEPS_OVERLAP)    */
    uint32_t n_slabs_global;  /* slabs of the global ring run, >= 1          */
    uint32_t n_slabs_partial; /* slabs of the partial ring run, >= 1         */
} r2_split_desc;

/* Workspace (device, 256-byte aligned): the two ring workspaces, two offsets tables and a
 * double-buffered stage for the broadcast.  0 if the descriptor is invalid. */
uint64_t r2_split_workspace_bytes(const r2_split_desc *desc);

/* weights: HOST array of n_channels bandwidth weights (the same NIC types on every server);
 * degraded_fail_mask: the NICs server d has lost.  Asynchronous on `stream`; allocates nothing. */
int r2_split_allreduce_sim(const r2_split_desc *desc, void *const *rank_bufs, const uint32_t *weights,
                           uint64_t degraded_fail_mask, void *workspace, uint64_t workspace_bytes,
                           void *stream);

/* ---------------------------------------------------------------------------------------------
 * Recursive R2CCL-AllReduce and the strategy selector -- Sec. 6 "Recursive R2CCL-AllReduce", built
 * on the two-ring analysis of Sec. 5.2.
 *
 * With several failures the servers form a spectrum of bandwidths.  A global ring runs at the
 * slowest server's rate; that server is then left out and a faster sub-ring formed from the rest,
 * and so on; each ring reduces a share of the data that matches the bandwidth it adds; all
 * reductions run in parallel and the broadcasts follow (Sec. 6).  The paper gives no pseudo-code:
 * the rules below are this library's reading, chosen so that one degraded server gives back the
 * two-ring schedule of Sec. 5.2 exactly.
 *
 * Plan (HOST, integer and double arithmetic): rank r's own bandwidth is the weight of the channels it
 * still has.  Level 0 holds all ranks.  The next level drops every rank whose own bandwidth is the
 * smallest among the current members, as long as two ranks remain.  A level's ring takes its members in
 * rank order, starting after the highest-numbered rank left out (level 0: from rank 0), re-ranked by
 * r2_bridge_rerank (Sec. 6: re-ranking is applied at every level, since skipping the slower nodes puts
 * nodes side by side that lost different rails); it runs link by link as r2_ring_rails_sim does, a link
 * carrying what both its ends still have, so its bandwidth is its narrowest link's and its increment the
 * gain over the previous level; a peel that gains nothing makes no level and the peeling goes on.
 * Shares minimise the completion time below with alpha = 0: with u_k = share_k / increment_k and
 * f_k = 2(p_k-1)/p_k, p_k = members_k * gpus_per_rank, that time is max_k f_k u_k + max_{k>=1} u_k, and
 * its minimum lies where the rings of the levels up to some j finish together (u_k = tau/f_k) and the
 * levels from j on share one u (= tau/f_j; their shares are then exactly proportional to the bandwidth
 * they add, as Sec. 6 words it); every j is tried, ties go to the smallest.  For two levels this is
 * T1 = T2 of Sec. 5.2.  R2_ERR_NO_HEALTHY_CHANNEL if a link of the global ring is left without a
 * channel even after re-ranking. */
#define R2_MAX_LEVELS 16

typedef struct {
    uint64_t members;   /* bit r: rank r takes part in this level's ring           */
    uint64_t fail_mask; /* channels down at some member (the ring itself runs link by link) */
    uint64_t bandwidth; /* the ring's: that of its narrowest link, in its re-ranked order   */
    uint64_t increment; /* bandwidth minus the previous level's (level 0: itself)  */
    double share;       /* fraction of the data this level reduces                 */
} r2_level;

/* weights: HOST [n_channels]; fail_masks: HOST [n_ranks]; levels: HOST, room for max_levels
 * (1..R2_MAX_LEVELS; the peeling stops there); *n_levels receives the count. */
int r2_recursive_plan(uint32_t n_ranks, uint32_t gpus_per_rank, uint32_t n_channels, const uint32_t *weights,
                      const uint64_t *fail_masks, uint32_t max_levels, r2_level *levels, uint32_t *n_levels);

/* The order in which the ring of a level visits its members (HOST): `members` in rank order starting
 * after the highest-numbered rank that is not a member, re-ranked by r2_bridge_rerank with every rank's
 * surviving channels as its rails.  order: HOST, room for popcount(members) ranks.  fail_masks: HOST
 * [n_ranks].  R2_ERR_INVALID for fewer than two members or members beyond n_ranks. */
int r2_recursive_ring_order(uint32_t n_ranks, uint32_t n_channels, const uint64_t *fail_masks,
                            uint64_t members, uint32_t *order);

/* alpha-beta completion time of a plan (Sec. 6, last paragraph; Sec. 8 "AllReduce performance"):
 *   max_k [ 2(p_k-1) alpha + 2(p_k-1)/p_k * share_k * bytes / (increment_k * beta) ]
 * + max_{k>=1} [ hops_k * alpha + share_k * bytes / (increment_k * beta) ],
 * hops_k = members_k + 2 * (n_ranks - members_k) - 1 (the broadcast chain; relay hops are not counted),
 * beta = bytes per second per unit of weight.  With alpha = 0 and two levels this is T(Y) = max(T1, T2) + T3 of Sec. 5.2;
 * one level is the plain ring at the slowest server's balanced rate (R2CCL-Balance).
 * Negative if an argument is invalid. */
double r2_recursive_time(uint32_t n_ranks, uint32_t gpus_per_rank, const r2_level *levels, uint32_t n_levels,
                         double bytes, double alpha, double beta);

/* The selector: plans every depth 0..D (depth = levels - 1; D = the full peel, at most
 * R2_MAX_LEVELS - 1) and returns in *depth the one with the smallest modelled time, the shallower on a
 * tie.  Depth 0 is R2CCL-Balance, depth 1 with one degraded server is R2CCL-AllReduce.  times
 * (optional, HOST, R2_MAX_LEVELS doubles) receives the modelled time of every depth, *n_depths
 * (optional) their count. */
int r2_select_strategy(uint32_t n_ranks, uint32_t gpus_per_rank, uint32_t n_channels, const uint32_t *weights,
                       const uint64_t *fail_masks, double bytes, double alpha, double beta,
                       uint32_t *depth, double *times, uint32_t *n_depths);

/* The schedule on simulated ranks (a rank stands for a server).  Every rank buffer is cut into
 * n_levels consecutive segments of level_elems[k] elements.  Segment k goes through
 *   1. a ring all-reduce over level k's members in the order r2_recursive_ring_order gives, with a
 *      table per link (r2_ring_rails_sim: a link carries what both its ends still have), and,
 *   2. if the level leaves ranks out, the broadcast chain: the ranks left out, in ascending order, add
 *      their segments up hop by hop; each member, in the ring's order, adds that sum to its ring result
 *      and relays it unchanged (R2_OP_SUM_FORWARD); the last member sends its finished result on, and
 *      the ranks left out copy it and pass it along in ascending order.  The transfer between two ranks
 *      is cut by the union of their failed channels.  Where two consecutive ranks of that walk have no
 *      channel in common (they lost complementary rails), the hop goes through a third rank that has a
 *      channel in common with both and forwards the data untouched, its own segment not involved: the
 *      first such rank among the members in the ring's order, then among the ranks left out in
 *      ascending order; R2_ERR_NO_HEALTHY_CHANNEL, before anything is launched, if there is none.
 * Afterwards every rank holds, in segment k, fold(members in the ring's order) + (running sum of the
 * ranks left out), rounded to the buffer type after every addition.  The levels touch disjoint
 * segments and have workspaces of their own, so they run side by side, as the paper's reductions
 * do: level k on one of a few library-owned streams (default priority, created once per device),
 * forked off `stream` and joined to it again with events before the call returns to the caller's
 * order.  Every segment's byte size must be a multiple of 16 and divide into n_slabs * members_k
 * chunks; level_elems sums to n_elems; a level may be empty. */
typedef struct {
    uint32_t n_ranks;    /* R, 2..R2_MAX_RANKS                      */
    uint32_t n_channels; /* C                                       */
    uint32_t align;      /* partition alignment, a multiple of 16   */
    int32_t dtype;       /* r2_dtype                                */
    int32_t schedule;    /* R2_SCHED_AUTO, _STEPS or _FUSED for the ring runs (no R2_SCHED_STEPS_OVERLAP) */
    uint32_t n_slabs;    /* slabs of every ring run, >= 1           */
    uint32_t n_levels;   /* 1..R2_MAX_LEVELS                        */
    uint32_t reserved;   /* 0                                       */
    uint64_t n_elems;    /* elements per rank                       */
} r2_recursive_desc;

/* Segment sizes that follow the plan's shares as closely as the rings allow (HOST arithmetic): level
 * k >= 1 gets floor(share_k * n_elems) rounded down to a multiple of
 * n_slabs * lcm(members_k, n_ranks) * (16 / element size) elements -- so that its ring chunks are whole
 * 16-byte vectors and what is left for level 0 still divides into the global ring -- and level 0 gets
 * the rest.  Needs n_elems to be a multiple of n_slabs * n_ranks * (16 / element size)
 * (R2_ERR_INVALID otherwise).  Small buffers may leave the upper levels empty.  level_elems: HOST,
 * n_levels entries out. */
int r2_recursive_segments(const r2_recursive_desc *desc, const r2_level *levels, uint64_t *level_elems);

/* Workspace (device, 256-byte aligned): per level, its ring workspace, its broadcast's offsets
 * tables, double-buffered stage and a landing place for relayed data.  0 if an argument is invalid. */
uint64_t r2_recursive_workspace_bytes(const r2_recursive_desc *desc, const r2_level *levels,
                                      const uint64_t *level_elems);

/* levels, level_elems, weights, fail_masks: HOST arrays (n_levels, n_levels, n_channels, n_ranks).
 * Only `members` of a level is read; members must be nested and hold >= 2 ranks.
 * Asynchronous on `stream`; allocates nothing. */
int r2_recursive_allreduce_sim(const r2_recursive_desc *desc, void *const *rank_bufs, const uint32_t *weights,
                               const uint64_t *fail_masks, const r2_level *levels, const uint64_t *level_elems,
                               void *workspace, uint64_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Bridge-based logical re-ranking -- Sec. 6 "Topology-Aware Logical Re-ranking", Appendix D Alg. 1.
 *
 * HOST integer work, no device involved.  `ring` is a permutation of 0..n-1 (the logical ring order);
 * rails[node] is the set of rails (NICs) node still has, as a bit mask.  The capacity of a ring edge is
 * the number of rails its ends share; B_global is the smallest rail count of any node.  Edges with
 * capacity < B_global are repaired, worst gap first (ties in ring order): the first node w (in the
 * ring's current order, other than the pair u, v) with min(|S_u & S_w|, |S_w & S_v|) >= B_global and
 * whose own neighbours x, y satisfy |S_x & S_y| >= B_global is moved to sit right after u.  A pair
 * that is no longer adjacent when its turn comes is skipped.  Writes the new order to out_ring[n] and
 * the number of relocations to *n_relocated (optional).  R2_ERR_INVALID unless ring is a permutation. */
int r2_bridge_rerank(const uint32_t *ring, const uint64_t *rails, uint32_t n, uint32_t *out_ring,
                     uint32_t *n_relocated);

#ifdef __cplusplus
}
#endif
#endif /* R2CCL_H */

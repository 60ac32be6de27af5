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
 * This header is the boundary of the hot path: the partition, the fused reduce-copy, the ring run
 * (also with failures in flight, and with its workspace in a static array).  r2ccl_ext.h declares what
 * is built on top of it: the other collectives, rings with a table per link, R2CCL-AllReduce and its
 * recursive form with their planners, the strategy selector and the bridge re-ranking.
 *
 * Conventions
 *   - Every function returns an R2_* code (0 = success); nothing throws or aborts.
 *   - "device" pointers are HIP device memory of the current device, "host" pointers
 *     are ordinary process memory.  The caller owns every buffer.  The library allocates no
 *     device memory.  The only state it keeps for the life of the process, per device: the side
 *     streams and events of r2_split_allreduce_sim, r2_recursive_allreduce_sim and the
 *     R2_SCHED_STEPS_OVERLAP schedule, created at the first such call, and two device arrays that
 *     are part of its code (see r2_ring_allreduce_sim_static and r2_partition).
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
 * The other R2_PHASE_* values (the other collectives R2CCL-Balance serves, and rings whose links have
 * tables of their own) are described in r2ccl_ext.h; they run through the same calls and kernels.
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
uint64_t r2_sim_stage_capacity(const r2_sim_desc *desc);    /* bytes per channel buffer: the ring
                                                               chunk rounded up to 256, plus, for
                                                               chunks of 1 MiB and more, 128 KiB + 256
                                                               that keep the buffers off power-of-two
                                                               distances (never written)             */

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
 * for the array's address there.  R2_SCHED_STEPS_OVERLAP is R2_ERR_INVALID here: its side stream and
 * events would have to be created at its first use.  All calls on one GPU share the one array: it keeps what the last call
 * left (no step ever reads bytes its own run has not written, so nothing is cleared), and calls that
 * overlap in time on one GPU -- different streams, different host threads -- race on it: keep them in
 * order on one stream. */
#define R2_STATIC_WORKSPACE_BYTES (72ull << 20)
int r2_ring_allreduce_sim_static(const r2_sim_desc *desc, void *const *rank_bufs,
                                 const r2_epoch *epochs, uint32_t n_epochs,
                                 uint64_t *offsets_log, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* R2CCL_H */

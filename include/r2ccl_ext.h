/*
 * r2ccl_ext.h -- what libr2ccl builds on top of the hot path of r2ccl.h, with the same kernels and the
 * same conventions (return codes, device / host pointers, caller-owned buffers, asynchronous calls).
 *
 *   - the other collectives R2CCL-Balance serves (Sec. 5, table of strategies; Sec. 5.1): reduce-scatter
 *     and all-gather alone, send/receive, broadcast, reduce, all-to-all;
 *   - the ring whose servers each have a channel state of their own, a table per link (Sec. 5.1, Sec. 6);
 *   - R2CCL-AllReduce: planner and split schedule (Sec. 5.2, Appendix A);
 *   - its recursive form for several failures, the alpha-beta time and the strategy selector (Sec. 6);
 *   - bridge-based logical re-ranking (Sec. 6, Appendix D Algorithm 1).
 */
#ifndef R2CCL_EXT_H
#define R2CCL_EXT_H

#include "r2ccl.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------------------------------------
 * The other phases of r2_sim_desc (each on its own only; R2_PHASE_LINKS is a flag for the ring phases).
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
 * --------------------------------------------------------------------------------------------- */

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
#endif /* R2CCL_EXT_H */

// R2CCL-AllReduce (R2CCL paper, Sec. 5.2 and Appendix A): when one server has lost a fraction X of
// its bandwidth, a share Y of the data skips it -- the healthy ranks all-reduce that share among
// themselves (partial all-reduce) while everybody all-reduces the rest (global all-reduce) -- and a
// tailored broadcast then brings the degraded rank's own contribution in and the finished result
// back to it.  This file holds the planner arithmetic (closed forms of Appendix A) and the
// schedule, which is built from the ring simulation and the fused reduce-copy of ring.hip.
#include <cmath>

#include "r2_internal.h"

namespace {

constexpr uint64_t kAlign256 = 256;

uint64_t round_up(uint64_t x, uint64_t m) { return (x + m - 1) / m * m; }

struct SplitShape {
    r2_sim_desc global, partial;  // the two ring runs
    uint64_t n_global, n_partial; // elements per rank
    uint64_t elem, part_bytes, cap;
    uint64_t ws_global, ws_partial, tables_off, stage_off, total;
};

int split_shape(const r2_split_desc *d, SplitShape &s)
{
    if (!d) return R2_ERR_INVALID;
    if (d->n_ranks < 3 || d->n_ranks > R2_MAX_RANKS || d->degraded_rank >= d->n_ranks) return R2_ERR_INVALID;
    if (d->n_channels == 0 || d->n_channels > R2_MAX_CHANNELS) return R2_ERR_INVALID;
    if (d->align == 0 || d->align % 16 != 0) return R2_ERR_INVALID;
    if (d->dtype != R2_F32 && d->dtype != R2_BF16) return R2_ERR_INVALID;
    if (d->n_partial > d->n_elems) return R2_ERR_INVALID;
    if (d->n_slabs_global == 0 || d->n_slabs_partial == 0) return R2_ERR_INVALID;
    // the two rings already run side by side on the library's streams: no overlapped passes inside them
    if (d->schedule == R2_SCHED_STEPS_OVERLAP) return R2_ERR_INVALID;
    s.elem = d->dtype == R2_F32 ? 4 : 2;
    s.n_partial = d->n_partial;
    s.n_global = d->n_elems - d->n_partial;
    // the partial part starts on a 16-byte boundary so that every chunk of it does
    if ((s.n_global * s.elem) % 16 != 0) return R2_ERR_INVALID;
    s.global = r2_sim_desc{d->n_ranks, d->n_slabs_global, d->n_channels, d->align, s.n_global, d->dtype,
                           R2_PHASE_RS | R2_PHASE_AG, 0, d->schedule, 0};
    s.partial = r2_sim_desc{d->n_ranks - 1, d->n_slabs_partial, d->n_channels, d->align, s.n_partial,
                            d->dtype, R2_PHASE_RS | R2_PHASE_AG, 0, d->schedule, 0};
    if (r2_sim_num_steps(&s.global) == 0 || r2_sim_num_steps(&s.partial) == 0) return R2_ERR_INVALID;
    s.ws_global = round_up(r2_sim_workspace_bytes(&s.global), kAlign256);
    s.ws_partial = round_up(r2_sim_workspace_bytes(&s.partial), kAlign256);
    s.part_bytes = s.n_partial * s.elem;
    s.cap = round_up(s.part_bytes ? s.part_bytes : 1, kAlign256);
    s.tables_off = s.ws_global + s.ws_partial;
    s.stage_off = s.tables_off + round_up(2 * (uint64_t)(d->n_channels + 1) * 8, kAlign256);
    s.total = s.stage_off + 2 * (uint64_t)d->n_channels * s.cap;
    return R2_OK;
}

}  // namespace

extern "C" int r2_split_plan(uint32_t n_servers, uint32_t gpus_per_server, double lost_fraction,
                             int32_t *use_split, double *y_star, double *threshold)
{
    if (n_servers < 2 || gpus_per_server < 1 || !(lost_fraction > 0.0) || !(lost_fraction < 1.0))
        return R2_ERR_INVALID;
    const double n = n_servers, g = gpus_per_server, X = lost_fraction;
    const double thr = n * g / (3.0 * n * g - 2.0);
    const double y = X + X * (1.0 - X) / (X + (g * (n - 1.0) - 1.0) * n);
    if (threshold) *threshold = thr;
    if (y_star) *y_star = y;
    // a partial all-reduce needs at least two healthy participants
    if (use_split) *use_split = (X > thr && (uint64_t)(n_servers - 1) * gpus_per_server >= 2) ? 1 : 0;
    return R2_OK;
}

extern "C" double r2_split_time(uint32_t n_servers, uint32_t gpus_per_server, double lost_fraction, double y)
{
    const double n = n_servers, g = gpus_per_server, X = lost_fraction;
    const double a = 2.0 * (n * g - 1.0) / (n * g);
    const double b = 2.0 * ((n - 1.0) * g - 1.0) / ((n - 1.0) * g);
    const double t1 = a * (1.0 - y) / (1.0 - X), t2 = b * y / X, t3 = y / X;
    return (t1 > t2 ? t1 : t2) + t3;
}

extern "C" uint64_t r2_split_partial_elems(uint32_t n_ranks, uint32_t n_slabs_global, uint32_t n_slabs_partial,
                                           int32_t dtype, uint64_t n_elems, double y)
{
    if (n_ranks < 3 || n_ranks > R2_MAX_RANKS || n_slabs_global == 0 || n_slabs_partial == 0) return 0;
    if ((dtype != R2_F32 && dtype != R2_BF16) || !(y >= 0.0) || !(y <= 1.0)) return 0;
    const uint64_t per16 = dtype == R2_F32 ? 4 : 8;
    const uint64_t gg = (uint64_t)n_slabs_global * n_ranks, gp = (uint64_t)n_slabs_partial * (n_ranks - 1);
    if (n_elems % (gg * per16) != 0) return 0;
    uint64_t a = gg, b = gp;
    while (b) {
        const uint64_t t = a % b;
        a = b;
        b = t;
    }
    const uint64_t granule = gg / a * gp * per16;
    return (uint64_t)(y * (double)n_elems) / granule * granule;
}

extern "C" uint64_t r2_split_workspace_bytes(const r2_split_desc *desc)
{
    SplitShape s;
    return split_shape(desc, s) == R2_OK ? s.total : 0;
}

extern "C" int r2_split_allreduce_sim(const r2_split_desc *desc, void *const *rank_bufs,
                                      const uint32_t *weights, uint64_t degraded_fail_mask,
                                      void *workspace, uint64_t workspace_bytes, void *stream)
{
    SplitShape s;
    int rc = split_shape(desc, s);
    if (rc) return rc;
    if (!rank_bufs || !weights) return R2_ERR_INVALID;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return R2_ERR_INVALID;
    if (workspace_bytes < s.total) return R2_ERR_CAPACITY;
    const uint32_t R = desc->n_ranks, C = desc->n_channels, d = desc->degraded_rank;
    for (uint32_t r = 0; r < R; ++r) {
        const uint64_t p = reinterpret_cast<uint64_t>(rank_bufs[r]);
        if (desc->n_elems && (!p || (p & 15u))) return R2_ERR_INVALID;
    }
    // the degraded server keeps at least one NIC; the healthy ones have them all
    if (!r2::any_healthy(weights, degraded_fail_mask, C)) return R2_ERR_NO_HEALTHY_CHANNEL;
    if (!r2::any_healthy(weights, 0, C)) return R2_ERR_NO_HEALTHY_CHANNEL;

    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const r2_epoch degraded = {0, degraded_fail_mask, weights};
    const r2_epoch healthy = {0, 0, weights};

    // The head and the tail of the buffers are disjoint and have workspaces of their own, so the two
    // run side by side, as the paper's stage-1 rings do: the global ring on the caller's stream, the
    // partial ring and, behind it, its broadcast on a stream forked off the caller's.
    r2::ForkJoin lanes((hipStream_t)stream);
    if (lanes.rc()) return lanes.rc();
    void *const tail = s.n_global ? (void *)lanes.lane(1) : stream;

    // Stage 1a: global all-reduce of the head of every buffer, over all ranks; the ring passes
    // through the degraded server, so its channel state governs.
    if (s.n_global) {
        rc = r2_ring_allreduce_sim(&s.global, rank_bufs, &degraded, 1, ws, s.ws_global, nullptr, stream);
        if (rc) return rc;
    }
    if (s.n_partial == 0) return R2_OK;

    // Stage 1b: partial all-reduce of the tail among the healthy ranks, in ring order after d.
    void *part[R2_MAX_RANKS];
    uint32_t order[R2_MAX_RANKS];  // order[i] = i-th healthy rank
    for (uint32_t i = 0; i + 1 < R; ++i) {
        order[i] = (d + 1 + i) % R;
        part[i] = static_cast<uint8_t *>(rank_bufs[order[i]]) + s.n_global * s.elem;
    }
    rc = r2_ring_allreduce_sim(&s.partial, part, &healthy, 1, ws + s.ws_global, s.ws_partial, nullptr,
                               tail);
    if (rc) return rc;

    // Stage 2: the tailored broadcast.  d sends its own tail into the healthy ring; every healthy
    // rank adds it to its partial result and passes it on unchanged; the last one sends its
    // finished result back to d.  Links that touch d are cut by d's channel state (table 0), links
    // between healthy ranks by the full state (table 1).
    uint64_t *tables = reinterpret_cast<uint64_t *>(ws + s.tables_off);
    const r2_epoch two[2] = {{0, degraded_fail_mask, weights}, {1, 0, weights}};
    rc = r2::launch_partition_epochs(two, 2, C, desc->align, s.part_bytes, 2, tables, nullptr, (hipStream_t)tail);
    if (rc) return rc;
    const uint64_t *t_deg = tables, *t_ok = tables + (C + 1);
    void *stage[2][R2_MAX_CHANNELS];
    for (uint32_t par = 0; par < 2; ++par)
        for (uint32_t c = 0; c < C; ++c) stage[par][c] = ws + s.stage_off + ((uint64_t)par * C + c) * s.cap;
    void *d_tail = static_cast<uint8_t *>(rank_bufs[d]) + s.n_global * s.elem;
    const r2_dtype dt = (r2_dtype)desc->dtype;

    // step 0: d stages its tail
    rc = r2_reduce_copy(d_tail, s.part_bytes, dt, R2_OP_SUM, nullptr, nullptr, stage[0], t_deg, C, s.cap, nullptr, tail);
    if (rc) return rc;
    for (uint32_t k = 1; k + 1 <= R; ++k) {  // k = 1 .. R-1: the healthy ranks in ring order
        const bool last = k == R - 1;
        const uint64_t *t_in = k == 1 ? t_deg : t_ok;
        const uint64_t *t_out = last ? t_deg : t_ok;
        rc = r2_reduce_copy(part[k - 1], s.part_bytes, dt, last ? R2_OP_SUM : R2_OP_SUM_FORWARD,
                            stage[(k + 1) & 1], t_in, stage[k & 1], t_out, C, s.cap, nullptr, tail);
        if (rc) return rc;
    }
    // step R: d takes the finished result
    rc = r2_reduce_copy(d_tail, s.part_bytes, dt, R2_OP_COPY, stage[(R + 1) & 1], t_deg, nullptr, nullptr, C, s.cap,
                        nullptr, tail);
    if (rc) return rc;
    return lanes.join();
}

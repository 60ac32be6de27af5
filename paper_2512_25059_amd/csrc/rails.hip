// Host side of the ring whose servers each have a channel state of their own: the links' epoch lists,
// the schedule, the fused launches with per-link tables, and the C entry points.  (The step schedule
// of such a ring runs on ring.hip's step kernel, which picks its tables per link.)
//
// R2CCL paper: Sec. 5.1 (R2CCL-Balance acts per server), Sec. 6 "Topology-Aware Logical Re-ranking"
// (neighbours that lost different rails share only the rails surviving at both), Sec. 5.2 (the ring).
#include <new>
#include <vector>

#include "ring_fused_links_device.h"
#include "sim_shape.h"

namespace r2 {
namespace {

// Dynamic LDS of a fused launch over the steps [step_begin, step_end) of a ring with per-link tables:
// the rows of every link plus one ColInfo per row; 0 if that does not fit.
uint32_t links_lds_bytes(const SimShape &s, uint32_t step_begin, uint32_t step_end)
{
    const uint32_t t_first = step_begin ? step_begin - 1 : 0;
    const uint32_t t_end = step_end < s.T_slab ? step_end : s.T_slab;
    if (t_end <= t_first) return 0;
    const uint64_t bytes = (uint64_t)s.R * (t_end - t_first) * ((s.C + 1) * 8 + sizeof(ColInfo));
    return bytes <= kLinksLdsBytes ? (uint32_t)bytes : 0;
}

template <bool BF16, unsigned U>
void launch_links(dim3 grid, dim3 block, uint32_t lds, hipStream_t st, const FusedArgs &a, uint64_t link_rows,
                  const EpochBatch *eb)
{
    if (eb) hipLaunchKernelGGL((ring_fused_links_partition_kernel<BF16, U>), grid, block, lds, st, a, link_rows, *eb);
    else hipLaunchKernelGGL((ring_fused_links_kernel<BF16, U>), grid, block, lds, st, a, link_rows);
}

// One fused launch of a ring with per-link tables.  With `eb` (the links' states on one axis) the
// kernel partitions on its own and records the rows in the workspace and in `log`.
int launch_fused_links(const r2_sim_desc *desc, const SimShape &s, void *const *rank_bufs, uint32_t step_begin,
                       uint32_t step_end, void *workspace, const EpochBatch *eb, uint64_t *log, hipStream_t stream)
{
    FusedArgs a{};
    for (uint32_t r = 0; r < s.R; ++r) a.rank_buf[r] = reinterpret_cast<uint64_t>(rank_bufs[r]);  // checked by the caller
    a.tables = static_cast<const uint64_t *>(workspace);
    a.tables_out = static_cast<uint64_t *>(workspace);
    a.log_out = log;
    a.align = desc->align;
    a.stage = reinterpret_cast<uint64_t>(workspace) + s.stage_off;
    a.chunk_bytes = s.chunk_bytes;
    a.cap = s.cap;
    const unsigned unroll = fused_col_unroll(s);
    const uint64_t col_bytes = (uint64_t)kNarrowColBytes * unroll;
    a.cols_per_chunk = (s.chunk_bytes + col_bytes - 1) / col_bytes;
    a.R = s.R;
    a.S = s.S;
    a.C = s.C;
    a.J = s.J;
    a.T_slab = s.T_slab;
    const int ring_phases = desc->phases & ~R2_PHASE_LINKS;
    a.chunk_start = ring_phases == R2_PHASE_AG ? 1 : 0;
    a.sum_last = ring_phases == R2_PHASE_AG ? 0 : s.R - 1;
    a.j0 = step_begin;
    a.j1 = step_end;
    const uint32_t lds = links_lds_bytes(s, step_begin, step_end);
    if (!lds) return R2_ERR_INVALID;
    const unsigned waves = s.R < kMaxFusedWaves ? s.R : kMaxFusedWaves;
    const dim3 grid((unsigned)(a.cols_per_chunk * s.S)), block(waves * kWave);
    const bool bf16 = desc->dtype == R2_BF16;
    if (unroll == 2) {
        if (bf16) launch_links<true, 2>(grid, block, lds, stream, a, s.tx_per_link, eb);
        else launch_links<false, 2>(grid, block, lds, stream, a, s.tx_per_link, eb);
    } else {
        if (bf16) launch_links<true, 1>(grid, block, lds, stream, a, s.tx_per_link, eb);
        else launch_links<false, 1>(grid, block, lds, stream, a, s.tx_per_link, eb);
    }
    return hip_rc(hipGetLastError());
}

// What r2_ring_rails_sim derives from the ranks' epoch lists before it launches anything.
struct LinkPlan {
    std::vector<uint32_t> speed;  // the weights the link epochs point to
    std::vector<r2_epoch> link;   // the links' epoch lists, strung together on one axis
    bool cut[2 * R2_MAX_RANKS];   // fused launches end before these steps
    bool fused;
};

// The schedule of the link r -> r+1: it changes whenever either end's does; a channel is down if
// either end has it down, and as fast as the slower end.  The links' tables lie one block after the
// other, so their schedules are strung together on one axis (block r starts at row r * tx_per_link)
// and partitioned in one go.  Also decides the schedule, like plan_schedule for the plain ring.
int plan_links(const r2_sim_desc *desc, const SimShape &s, const r2_epoch *const *rank_epochs,
               const uint32_t *n_rank_epochs, LinkPlan &plan)
{
    if (!s.links || !rank_epochs || !n_rank_epochs) return R2_ERR_INVALID;
    for (uint32_t r = 0; r < s.R; ++r) {
        const r2_epoch *e = rank_epochs[r];
        const uint32_t n = n_rank_epochs[r];
        if (!e || n == 0 || e[0].t_start != 0) return R2_ERR_INVALID;
        for (uint32_t i = 0; i < n; ++i)
            if (!e[i].weights || (i && e[i].t_start <= e[i - 1].t_start)) return R2_ERR_INVALID;
    }
    const uint64_t full = s.C == 64 ? ~0ull : ((1ull << s.C) - 1);
    size_t n_all = 0;
    for (uint32_t r = 0; r < s.R; ++r) n_all += (size_t)n_rank_epochs[r] + n_rank_epochs[(r + 1) % s.R];
    plan.speed.assign(n_all * s.C, 0);  // never grows again: the epochs point into it
    plan.link.clear();
    plan.link.reserve(n_all);
    for (uint32_t r = 0; r < s.R; ++r) {
        const r2_epoch *a = rank_epochs[r], *b = rank_epochs[(r + 1) % s.R];
        const uint32_t na = n_rank_epochs[r], nb = n_rank_epochs[(r + 1) % s.R];
        uint32_t ia = 0, ib = 0;
        for (;;) {
            const uint64_t t = a[ia].t_start > b[ib].t_start ? a[ia].t_start : b[ib].t_start;
            if (t >= s.tx_per_link) break;  // never in force (and would run into the next link's block)
            uint32_t *w = plan.speed.data() + plan.link.size() * s.C;
            for (uint32_t c = 0; c < s.C; ++c)
                w[c] = a[ia].weights[c] < b[ib].weights[c] ? a[ia].weights[c] : b[ib].weights[c];
            const uint64_t mask = (a[ia].fail_mask | b[ib].fail_mask) & full;
            if (!any_healthy(w, mask, s.C)) return R2_ERR_NO_HEALTHY_CHANNEL;
            plan.link.push_back(r2_epoch{r * s.tx_per_link + t, mask, w});
            // the next change at either end
            const uint64_t next_a = ia + 1 < na ? a[ia + 1].t_start : ~0ull;
            const uint64_t next_b = ib + 1 < nb ? b[ib + 1].t_start : ~0ull;
            if (next_a == ~0ull && next_b == ~0ull) break;
            if (next_a <= next_b) ++ia;
            if (next_b <= next_a) ++ib;
        }
    }
    // Fused columns, as in the plain ring: a link whose table changes at step c of some slab forces a
    // launch boundary before step c and before step c+1; every launch's rows must fit LDS.
    uint32_t n_cuts = 0;
    for (bool &c : plan.cut) c = false;
    for (const r2_epoch &e : plan.link) {
        const uint32_t c = (uint32_t)(e.t_start % s.tx_per_link % s.T_slab);
        if (c == 0) continue;  // the link's first, or a slab starts here: its stage buffers are its own
        for (uint32_t j = c; j <= c + 1 && j < s.T_slab; ++j)
            if (!plan.cut[j]) {
                plan.cut[j] = true;
                ++n_cuts;
            }
    }
    plan.fused = desc->schedule != R2_SCHED_STEPS && columns_fit(s);
    for (uint32_t j = 1, j0 = 0; j <= s.J && plan.fused; ++j)
        if (j == s.J || plan.cut[j]) {
            plan.fused = links_lds_bytes(s, j0, j) != 0;
            j0 = j;
        }
    if (desc->schedule == R2_SCHED_FUSED && s.chunk_bytes && !plan.fused) return R2_ERR_INVALID;
    if (desc->schedule == R2_SCHED_AUTO)  // launch-bound sizes only, and only if it saves launches
        plan.fused = plan.fused && (uint64_t)s.R * s.S * s.chunk_bytes <= kFusedAutoBytes &&
                     (uint64_t)(n_cuts + 1) * 2 <= s.n_passes * s.J;
    return R2_OK;
}

}  // namespace
}  // namespace r2

using namespace r2;

extern "C" int r2_rails_resolve_schedule(const r2_sim_desc *desc, const r2_epoch *const *rank_epochs,
                                         const uint32_t *n_rank_epochs)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    try {
        LinkPlan plan;
        if ((rc = plan_links(desc, s, rank_epochs, n_rank_epochs, plan))) return rc;
        return plan.fused ? R2_SCHED_FUSED : R2_SCHED_STEPS;
    } catch (const std::bad_alloc &) {  // the merged epoch lists are host allocations; nothing may unwind into C
        return R2_ERR_CAPACITY;
    }
}

extern "C" int r2_ring_rails_sim(const r2_sim_desc *desc, void *const *rank_bufs,
                                 const r2_epoch *const *rank_epochs, const uint32_t *n_rank_epochs,
                                 void *workspace, uint64_t workspace_bytes, uint64_t *offsets_log, void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (!s.links || !rank_bufs) return R2_ERR_INVALID;
    for (uint32_t r = 0; r < s.R; ++r) {
        const uint64_t p = reinterpret_cast<uint64_t>(rank_bufs[r]);
        if (s.chunk_bytes && (!p || (p & 15u))) return R2_ERR_INVALID;
    }
    try {
        LinkPlan plan;
        if ((rc = plan_links(desc, s, rank_epochs, n_rank_epochs, plan))) return rc;
        if ((rc = check_workspace(workspace, workspace_bytes, s))) return rc;

        // The fused kernels cut the chunks themselves when every link's states fit one argument block;
        // otherwise, and for the step schedule, one partition launch makes all tables up front.
        const bool self = plan.fused && plan.link.size() <= epochs_per_batch(s.C);
        if (!self && s.n_tx &&
            (rc = launch_partition_epochs(plan.link.data(), (uint32_t)plan.link.size(), s.C, desc->align, s.chunk_bytes,
                                          s.n_tx, static_cast<uint64_t *>(workspace), offsets_log, (hipStream_t)stream)))
            return rc;
        if (s.chunk_bytes == 0) return R2_OK;
        if (plan.fused) {
            EpochBatch eb;
            if (self) fill_batch(eb, plan.link.data(), 0, (uint32_t)plan.link.size(), s.C);
            uint32_t j0 = 0;
            for (uint32_t j = 1; j <= s.J; ++j)
                if (j == s.J || plan.cut[j]) {
                    if ((rc = launch_fused_links(desc, s, rank_bufs, j0, j, workspace, self ? &eb : nullptr,
                                                 self ? offsets_log : nullptr, (hipStream_t)stream)))
                        return rc;
                    j0 = j;
                }
            return R2_OK;
        }
        for (uint64_t p = 0; p < s.n_passes; ++p)
            for (uint32_t j = 0; j < s.J; ++j)
                if ((rc = r2_sim_step(desc, rank_bufs, p, j, workspace, workspace_bytes, stream))) return rc;
        return R2_OK;
    } catch (const std::bad_alloc &) {
        return R2_ERR_CAPACITY;
    }
}


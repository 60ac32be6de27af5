// Recursive R2CCL-AllReduce (R2CCL paper, Sec. 6, on top of Sec. 5.2): with several failures the
// servers form a spectrum of bandwidths; a global ring runs at the slowest server's rate, the
// slowest is left out and a faster sub-ring formed from the rest, and so on, every ring re-ranked so
// that neighbours share as many rails as the narrowest member has (Sec. 6, "Topology-Aware Logical
// Re-ranking").  This file holds the host planner (the peel, the rings' orders and bandwidths, the
// shares, the alpha-beta time, the choice of depth) and the schedule on simulated ranks, which is built
// from the ring with per-link tables (rails.hip) and the fused reduce-copy of ring.hip.
#include <new>
#include <vector>

#include "r2_internal.h"

namespace {

constexpr uint64_t kAlign256 = 256;

uint64_t round_up(uint64_t x, uint64_t m) { return (x + m - 1) / m * m; }

uint64_t weight_of(const uint32_t *weights, uint64_t fail_mask, uint32_t C)
{
    uint64_t w = 0;
    for (uint32_t c = 0; c < C; ++c)
        if (!((fail_mask >> c) & 1u)) w += weights[c];
    return w;
}

uint64_t union_mask(const uint64_t *fail_masks, uint64_t members, uint32_t R, uint64_t full)
{
    uint64_t u = 0;
    for (uint32_t r = 0; r < R; ++r)
        if ((members >> r) & 1u) u |= fail_masks[r] & full;
    return u;
}

double ring_factor(double p) { return 2.0 * (p - 1.0) / p; }

unsigned popcount64(uint64_t x) { return (unsigned)__builtin_popcountll(x); }

// A level's ring: its members in rank order, starting after the highest-numbered rank that is left
// out (level 0: from rank 0), then re-ranked.  Returns an R2 code; order receives popcount(members) ranks.
int level_ring_order(uint32_t R, uint32_t C, const uint64_t *fail_masks, uint64_t members, uint32_t *order, uint32_t &p)
{
    const uint64_t full = C == 64 ? ~0ull : ((1ull << C) - 1);
    uint32_t base[R2_MAX_RANKS], start = 0;
    for (uint32_t r = 0; r < R; ++r)
        if (!((members >> r) & 1u)) start = r + 1;
    p = 0;
    for (uint32_t i = 0; i < R; ++i) {
        const uint32_t r = (start + i) % R;
        if ((members >> r) & 1u) base[p++] = r;
    }
    // the re-ranking works on nodes 0..p-1: node i is base[i], its rails the channels it still has
    uint32_t ident[R2_MAX_RANKS], moved[R2_MAX_RANKS];
    uint64_t rails[R2_MAX_RANKS];
    for (uint32_t i = 0; i < p; ++i) {
        ident[i] = i;
        rails[i] = ~fail_masks[base[i]] & full;
    }
    const int rc = r2_bridge_rerank(ident, rails, p, moved, nullptr);
    if (rc) return rc;
    for (uint32_t i = 0; i < p; ++i) order[i] = base[moved[i]];
    return R2_OK;
}

// A ring moves data at the rate of its narrowest link; a link carries what both its ends still have.
uint64_t ring_bandwidth(const uint32_t *weights, const uint64_t *fail_masks, const uint32_t *order, uint32_t p,
                        uint32_t C, uint64_t full)
{
    uint64_t lo = ~0ull;
    for (uint32_t i = 0; i < p; ++i) {
        const uint64_t w = weight_of(weights, (fail_masks[order[i]] | fail_masks[order[(i + 1) % p]]) & full, C);
        if (w < lo) lo = w;
    }
    return lo;
}

// Shares that minimise max_k f_k u_k + max_{k>=1} u_k (u_k = share_k / increment_k, f_k the ring
// factor), the completion time with latency ignored: the time is piecewise linear in the shares, so
// the minimum lies where the rings of the levels up to some j finish together (u_k = tau / f_k) and the
// levels from j on have the same u (= tau / f_j): their shares are then exactly proportional to the
// bandwidth they add.  Every j is tried; ties go to the smallest.  Two levels: the point T1 = T2.
void optimal_shares(r2_level *levels, uint32_t L, uint32_t gpus_per_rank)
{
    if (L == 1) {
        levels[0].share = 1.0;
        return;
    }
    double f[R2_MAX_LEVELS], best_t = 0.0;
    for (uint32_t k = 0; k < L; ++k) f[k] = ring_factor((double)popcount64(levels[k].members) * gpus_per_rank);
    for (uint32_t j = 1; j < L; ++j) {
        double work = 0.0;  // sum of increment_k * u_k / tau
        for (uint32_t k = 0; k < L; ++k) work += (double)levels[k].increment / f[k <= j ? k : j];
        const double t = (1.0 + 1.0 / f[j]) / work;
        // Two balance levels can reach the same time exactly (as rationals); in doubles such a tie would go
        // to whichever rounds lower.  A later level must win by more than rounding to replace an earlier one.
        if (j == 1 || t < best_t * (1.0 - 1e-13)) {
            best_t = t;
            for (uint32_t k = 0; k < L; ++k) levels[k].share = (double)levels[k].increment / f[k <= j ? k : j] / work;
        }
    }
}

// The ranks a level's broadcast visits, in order.  The ranks left out add their segments up in
// ascending order (kGather); the sum goes round the ring's members in the ring's order, each adding it to
// its ring result and passing it on unchanged (kMember; the last passes its finished result on); the
// ranks left out take the result in ascending order (kTake).  A hop between two ranks that have no
// channel in common goes through a third that is linked to both and forwards the data untouched
// (kRelay): the first such rank among the ring's members in ring order, then among the ranks left out.
enum Role : uint8_t { kGather, kMember, kTake, kRelay };
struct Visit {
    uint32_t rank;
    Role role;
};
constexpr uint32_t kMaxVisits = 6 * R2_MAX_RANKS;  // 2m + p ranks, and at most one relay per hop

int chain_visits(uint32_t R, uint32_t C, const uint64_t *fail_masks, uint64_t members, const uint32_t *order,
                 uint32_t p, Visit *visits, uint32_t &n)
{
    const uint64_t full = C == 64 ? ~0ull : ((1ull << C) - 1);
    uint32_t excl[R2_MAX_RANKS], m = 0;
    for (uint32_t r = 0; r < R; ++r)
        if (!((members >> r) & 1u)) excl[m++] = r;
    n = 0;
    if (!m) return R2_OK;
    Visit walk[3 * R2_MAX_RANKS];
    uint32_t nw = 0;
    for (uint32_t i = 0; i < m; ++i) walk[nw++] = Visit{excl[i], kGather};
    for (uint32_t i = 0; i < p; ++i) walk[nw++] = Visit{order[i], kMember};
    for (uint32_t i = 0; i < m; ++i) walk[nw++] = Visit{excl[i], kTake};
    auto linked = [&](uint32_t a, uint32_t b) { return ((fail_masks[a] | fail_masks[b]) & full) != full; };
    visits[n++] = walk[0];
    for (uint32_t i = 1; i < nw; ++i) {
        const uint32_t u = visits[n - 1].rank, v = walk[i].rank;
        if (!linked(u, v)) {
            bool found = false;
            for (uint32_t q = 0; q < p + m && !found; ++q) {
                const uint32_t w = q < p ? order[q] : excl[q - p];
                if (w != u && w != v && linked(u, w) && linked(w, v)) {
                    visits[n++] = Visit{w, kRelay};
                    found = true;
                }
            }
            if (!found) return R2_ERR_NO_HEALTHY_CHANNEL;
        }
        visits[n++] = walk[i];
    }
    return R2_OK;
}

struct LevelShape {
    r2_sim_desc ring;
    uint64_t bytes, cap, ws_ring;
    uint64_t ring_off, tables_off, stage_off, relay_off;  // the level's own part of the workspace
    uint32_t m, p, hops;
};

struct RecShape {
    LevelShape lv[R2_MAX_LEVELS];
    uint64_t elem, total;
};

int rec_shape(const r2_recursive_desc *d, const r2_level *levels, const uint64_t *level_elems, RecShape &s)
{
    if (!d || !levels || !level_elems) return R2_ERR_INVALID;
    if (d->n_ranks < 2 || d->n_ranks > R2_MAX_RANKS) return R2_ERR_INVALID;
    if (d->n_channels == 0 || d->n_channels > R2_MAX_CHANNELS) return R2_ERR_INVALID;
    if (d->align == 0 || d->align % 16 != 0) return R2_ERR_INVALID;
    if (d->dtype != R2_F32 && d->dtype != R2_BF16) return R2_ERR_INVALID;
    if (d->n_levels == 0 || d->n_levels > R2_MAX_LEVELS || d->n_slabs == 0 || d->reserved != 0) return R2_ERR_INVALID;
    if (d->schedule == R2_SCHED_STEPS_OVERLAP) return R2_ERR_INVALID;  // the levels already run side by side
    const uint32_t R = d->n_ranks;
    const uint64_t all = R == 64 ? ~0ull : ((1ull << R) - 1);
    s.elem = d->dtype == R2_F32 ? 4 : 2;
    s.total = 0;
    uint64_t sum = 0, prev = all;
    for (uint32_t k = 0; k < d->n_levels; ++k) {
        LevelShape &l = s.lv[k];
        const uint64_t mem = levels[k].members;
        if (k == 0 ? mem != all : ((mem & ~prev) != 0 || mem == prev)) return R2_ERR_INVALID;  // nested, shrinking
        prev = mem;
        l.p = popcount64(mem);
        l.m = R - l.p;
        if (l.p < 2) return R2_ERR_INVALID;
        l.hops = l.m ? l.p + 2 * l.m - 1 : 0;
        const uint64_t n = level_elems[k];
        if (n > d->n_elems - sum) return R2_ERR_INVALID;
        sum += n;
        l.bytes = n * s.elem;
        if (l.bytes % 16 != 0) return R2_ERR_INVALID;
        l.cap = round_up(l.bytes ? l.bytes : 1, kAlign256);
        l.ring = r2_sim_desc{l.p, d->n_slabs, d->n_channels, d->align, n, d->dtype,
                             R2_PHASE_RS | R2_PHASE_AG | R2_PHASE_LINKS, 0, d->schedule, 0};
        l.ws_ring = 0;
        l.ring_off = l.tables_off = l.stage_off = l.relay_off = s.total;
        if (n) {
            if (r2_sim_num_steps(&l.ring) == 0) return R2_ERR_INVALID;
            l.ws_ring = round_up(r2_sim_workspace_bytes(&l.ring), kAlign256);
            if (l.ws_ring == 0) return R2_ERR_INVALID;
            l.tables_off = l.ring_off + l.ws_ring;
            // every hop may need a relay: twice the rows; a relay's landing place: one segment
            l.stage_off = l.tables_off + round_up(2 * l.hops * (uint64_t)(d->n_channels + 1) * 8, kAlign256);
            l.relay_off = l.stage_off + (l.m ? 2 * (uint64_t)d->n_channels * l.cap : 0);
            s.total = l.relay_off + (l.m ? l.cap : 0);
        }
    }
    if (sum != d->n_elems) return R2_ERR_INVALID;
    if (s.total == 0) s.total = kAlign256;
    return R2_OK;
}

}  // namespace

extern "C" int r2_recursive_plan(uint32_t n_ranks, uint32_t gpus_per_rank, uint32_t n_channels,
                                 const uint32_t *weights, const uint64_t *fail_masks, uint32_t max_levels,
                                 r2_level *levels, uint32_t *n_levels)
{
    if (n_ranks < 2 || n_ranks > R2_MAX_RANKS || gpus_per_rank == 0) return R2_ERR_INVALID;
    if (n_channels == 0 || n_channels > R2_MAX_CHANNELS) return R2_ERR_INVALID;
    if (max_levels == 0 || max_levels > R2_MAX_LEVELS) return R2_ERR_INVALID;
    if (!weights || !fail_masks || !levels || !n_levels) return R2_ERR_INVALID;
    const uint32_t R = n_ranks, C = n_channels;
    const uint64_t full = C == 64 ? ~0ull : ((1ull << C) - 1);
    uint64_t own[R2_MAX_RANKS];
    for (uint32_t r = 0; r < R; ++r) own[r] = weight_of(weights, fail_masks[r] & full, C);

    uint64_t masks[R2_MAX_RANKS];
    for (uint32_t r = 0; r < R; ++r) masks[r] = fail_masks[r] & full;
    uint32_t order[R2_MAX_RANKS], p = 0;

    uint64_t members = R == 64 ? ~0ull : ((1ull << R) - 1);
    int rc = level_ring_order(R, C, masks, members, order, p);
    if (rc) return rc;
    uint64_t bw = ring_bandwidth(weights, masks, order, p, C, full);
    if (bw == 0) return R2_ERR_NO_HEALTHY_CHANNEL;  // a link of the global ring is left without a channel
    uint32_t L = 0;
    levels[L++] = r2_level{members, union_mask(masks, members, R, full), bw, bw, 0.0};
    while (L < max_levels) {
        uint64_t lo = ~0ull;
        for (uint32_t r = 0; r < R; ++r)
            if (((members >> r) & 1u) && own[r] < lo) lo = own[r];
        uint64_t rest = 0;
        for (uint32_t r = 0; r < R; ++r)
            if (((members >> r) & 1u) && own[r] > lo) rest |= 1ull << r;
        if (popcount64(rest) < 2) break;
        members = rest;
        if ((rc = level_ring_order(R, C, masks, members, order, p))) return rc;
        bw = ring_bandwidth(weights, masks, order, p, C, full);
        if (bw > levels[L - 1].bandwidth) {
            levels[L] = r2_level{members, union_mask(masks, members, R, full), bw, bw - levels[L - 1].bandwidth, 0.0};
            ++L;
        }
    }
    optimal_shares(levels, L, gpus_per_rank);
    *n_levels = L;
    return R2_OK;
}

extern "C" int r2_recursive_ring_order(uint32_t n_ranks, uint32_t n_channels, const uint64_t *fail_masks,
                                       uint64_t members, uint32_t *order)
{
    if (n_ranks < 2 || n_ranks > R2_MAX_RANKS || n_channels == 0 || n_channels > R2_MAX_CHANNELS) return R2_ERR_INVALID;
    if (!fail_masks || !order) return R2_ERR_INVALID;
    const uint64_t all = n_ranks == 64 ? ~0ull : ((1ull << n_ranks) - 1);
    if ((members & ~all) != 0 || popcount64(members) < 2) return R2_ERR_INVALID;
    uint32_t p = 0;
    return level_ring_order(n_ranks, n_channels, fail_masks, members, order, p);
}

extern "C" double r2_recursive_time(uint32_t n_ranks, uint32_t gpus_per_rank, const r2_level *levels,
                                    uint32_t n_levels, double bytes, double alpha, double beta)
{
    if (!levels || n_levels == 0 || n_levels > R2_MAX_LEVELS || gpus_per_rank == 0 || n_ranks < 2) return -1.0;
    if (!(beta > 0.0) || !(bytes >= 0.0) || !(alpha >= 0.0)) return -1.0;
    double red = 0.0, bc = 0.0;
    for (uint32_t k = 0; k < n_levels; ++k) {
        const unsigned mem = popcount64(levels[k].members);
        if (mem < 2 || mem > n_ranks || levels[k].increment == 0) return -1.0;
        const double p = (double)mem * gpus_per_rank;
        const double t = levels[k].share * bytes / ((double)levels[k].increment * beta);
        const double tr = 2.0 * (p - 1.0) * alpha + ring_factor(p) * t;
        if (tr > red) red = tr;
        if (k) {
            const double hops = (double)mem + 2.0 * (double)(n_ranks - mem) - 1.0;
            const double tb = hops * alpha + t;
            if (tb > bc) bc = tb;
        }
    }
    return red + bc;
}

extern "C" int r2_select_strategy(uint32_t n_ranks, uint32_t gpus_per_rank, uint32_t n_channels,
                                  const uint32_t *weights, const uint64_t *fail_masks, double bytes,
                                  double alpha, double beta, uint32_t *depth, double *times, uint32_t *n_depths)
{
    if (!depth || !(beta > 0.0) || !(bytes >= 0.0) || !(alpha >= 0.0)) return R2_ERR_INVALID;
    r2_level lv[R2_MAX_LEVELS];
    uint32_t full = 0;
    int rc = r2_recursive_plan(n_ranks, gpus_per_rank, n_channels, weights, fail_masks, R2_MAX_LEVELS, lv, &full);
    if (rc) return rc;
    uint32_t best = 0;
    double best_t = 0.0;
    for (uint32_t d = 0; d < full; ++d) {
        uint32_t L = 0;
        rc = r2_recursive_plan(n_ranks, gpus_per_rank, n_channels, weights, fail_masks, d + 1, lv, &L);
        if (rc) return rc;
        const double t = r2_recursive_time(n_ranks, gpus_per_rank, lv, L, bytes, alpha, beta);
        if (t < 0.0) return R2_ERR_INVALID;
        if (times) times[d] = t;
        if (d == 0 || t < best_t) {
            best = d;
            best_t = t;
        }
    }
    *depth = best;
    if (n_depths) *n_depths = full;
    return R2_OK;
}

extern "C" int r2_recursive_segments(const r2_recursive_desc *d, const r2_level *levels, uint64_t *level_elems)
{
    if (!d || !levels || !level_elems) return R2_ERR_INVALID;
    if (d->n_ranks < 2 || d->n_ranks > R2_MAX_RANKS || d->n_slabs == 0) return R2_ERR_INVALID;
    if (d->n_levels == 0 || d->n_levels > R2_MAX_LEVELS) return R2_ERR_INVALID;
    if (d->dtype != R2_F32 && d->dtype != R2_BF16) return R2_ERR_INVALID;
    const uint64_t per16 = d->dtype == R2_F32 ? 4 : 8;  // elements in a 16-byte vector
    const uint64_t g0 = (uint64_t)d->n_slabs * d->n_ranks * per16;
    if (d->n_elems % g0 != 0) return R2_ERR_INVALID;
    uint64_t used = 0;
    for (uint32_t k = d->n_levels; k-- > 1;) {
        const uint64_t p = popcount64(levels[k].members);
        if (p < 2 || p > d->n_ranks || !(levels[k].share >= 0.0) || !(levels[k].share <= 1.0)) return R2_ERR_INVALID;
        uint64_t a = p, b = d->n_ranks;  // lcm(p, R) through gcd
        while (b) {
            const uint64_t t = a % b;
            a = b;
            b = t;
        }
        const uint64_t g = (uint64_t)d->n_slabs * (p / a * d->n_ranks) * per16;
        uint64_t n = (uint64_t)(levels[k].share * (double)d->n_elems) / g * g;
        if (n > d->n_elems - used) n = (d->n_elems - used) / g * g;  // shares that sum to more than one
        level_elems[k] = n;
        used += n;
    }
    level_elems[0] = d->n_elems - used;
    return R2_OK;
}

extern "C" uint64_t r2_recursive_workspace_bytes(const r2_recursive_desc *desc, const r2_level *levels,
                                                 const uint64_t *level_elems)
{
    RecShape s;
    return rec_shape(desc, levels, level_elems, s) == R2_OK ? s.total : 0;
}

extern "C" int r2_recursive_allreduce_sim(const r2_recursive_desc *desc, void *const *rank_bufs,
                                          const uint32_t *weights, const uint64_t *fail_masks,
                                          const r2_level *levels, const uint64_t *level_elems, void *workspace,
                                          uint64_t workspace_bytes, void *stream)
{
    RecShape s;
    int rc = rec_shape(desc, levels, level_elems, s);
    if (rc) return rc;
    if (!rank_bufs || !weights || !fail_masks) return R2_ERR_INVALID;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return R2_ERR_INVALID;
    if (workspace_bytes < s.total) return R2_ERR_CAPACITY;
    const uint32_t R = desc->n_ranks, C = desc->n_channels;
    const uint64_t full = C == 64 ? ~0ull : ((1ull << C) - 1);
    for (uint32_t r = 0; r < R; ++r) {
        const uint64_t p = reinterpret_cast<uint64_t>(rank_bufs[r]);
        if (desc->n_elems && (!p || (p & 15u))) return R2_ERR_INVALID;
    }

    uint64_t masks[R2_MAX_RANKS];
    for (uint32_t r = 0; r < R; ++r) masks[r] = fail_masks[r] & full;

    // Everything is laid out and checked before the first launch: every level's ring order, that each of
    // its links has a channel, and the walk of its broadcast with the relays it needs.
    struct LevelWalk {
        uint32_t order[R2_MAX_RANKS], p, n;
        Visit visits[kMaxVisits];
    };
    std::vector<LevelWalk> walks;
    try {
        walks.resize(desc->n_levels);
    } catch (const std::bad_alloc &) {
        return R2_ERR_CAPACITY;
    }
    for (uint32_t k = 0; k < desc->n_levels; ++k) {
        LevelWalk &w = walks[k];
        w.p = w.n = 0;
        if (level_elems[k] == 0) continue;
        if ((rc = level_ring_order(R, C, masks, levels[k].members, w.order, w.p))) return rc;
        if (ring_bandwidth(weights, masks, w.order, w.p, C, full) == 0) return R2_ERR_NO_HEALTHY_CHANNEL;
        if ((rc = chain_visits(R, C, masks, levels[k].members, w.order, w.p, w.visits, w.n))) return rc;
    }

    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const r2_dtype dt = (r2_dtype)desc->dtype;
    uint64_t lo = 0;  // first element of the level's segment
    r2_epoch links[kMaxVisits], member_state[R2_MAX_RANKS];
    const r2_epoch *member_list[R2_MAX_RANKS];
    uint32_t ones[R2_MAX_RANKS];
    // The levels work on disjoint segments with workspaces of their own: each runs, ring and
    // broadcast chain, on a lane of its own, side by side with the others.
    r2::ForkJoin lanes((hipStream_t)stream);
    if (lanes.rc()) return lanes.rc();
    uint32_t n_busy = 0;
    for (uint32_t k = 0; k < desc->n_levels; ++k) {
        const LevelShape &l = s.lv[k];
        const LevelWalk &w = walks[k];
        const uint64_t seg_off = lo * s.elem;
        lo += level_elems[k];
        if (level_elems[k] == 0) continue;
        void *const lane = lanes.lane(n_busy++ % (r2::kSideStreams + 1));
        uint64_t *tables = reinterpret_cast<uint64_t *>(ws + l.tables_off);

        // 1. the level's ring over its members in the level's order, link by link: a link carries what
        //    both its ends still have
        void *seg[R2_MAX_RANKS];
        for (uint32_t i = 0; i < w.p; ++i) {
            seg[i] = static_cast<uint8_t *>(rank_bufs[w.order[i]]) + seg_off;
            member_state[i] = r2_epoch{0, masks[w.order[i]], weights};
            member_list[i] = &member_state[i];
            ones[i] = 1;
        }
        rc = r2_ring_rails_sim(&l.ring, seg, member_list, ones, ws + l.ring_off, l.ws_ring, nullptr, lane);
        if (rc) return rc;
        if (!w.n) continue;

        // 2. the broadcast chain; hop i joins visits[i] and visits[i+1] and has table i
        for (uint32_t i = 0; i + 1 < w.n; ++i)
            links[i] = r2_epoch{i, masks[w.visits[i].rank] | masks[w.visits[i + 1].rank], weights};
        rc = r2::launch_partition_epochs(links, w.n - 1, C, desc->align, l.bytes, w.n - 1, tables, nullptr,
                                         (hipStream_t)lane);
        if (rc) return rc;
        void *stage[2][R2_MAX_CHANNELS];
        for (uint32_t par = 0; par < 2; ++par)
            for (uint32_t c = 0; c < C; ++c) stage[par][c] = ws + l.stage_off + ((uint64_t)par * C + c) * l.cap;
        uint32_t last_member = 0;
        for (uint32_t i = 0; i < w.n; ++i)
            if (w.visits[i].role == kMember) last_member = i;
        for (uint32_t i = 0; i < w.n; ++i) {
            const bool first = i == 0, last = i + 1 == w.n;
            void *local = static_cast<uint8_t *>(rank_bufs[w.visits[i].rank]) + seg_off;
            int op;
            switch (w.visits[i].role) {
            case kGather: op = R2_OP_SUM; break;  // the ranks left out add themselves up
            case kMember: op = i == last_member ? R2_OP_SUM : R2_OP_SUM_FORWARD; break;
            case kTake: op = R2_OP_COPY; break;   // the ranks left out take the result, pass it on
            default:                              // a relay forwards what it gets; its own data is not involved
                op = R2_OP_COPY;
                local = ws + l.relay_off;
            }
            rc = r2_reduce_copy(local, l.bytes, dt, op, first ? nullptr : stage[(i + 1) & 1],
                                first ? nullptr : tables + (uint64_t)(i - 1) * (C + 1), last ? nullptr : stage[i & 1],
                                last ? nullptr : tables + (uint64_t)i * (C + 1), C, l.cap, nullptr, lane);
            if (rc) return rc;
        }
    }
    return lanes.join();
}

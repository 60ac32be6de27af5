// Host-side description of a simulated run, shared by ring.hip and rails.hip (not part of the ABI):
// the descriptor's validation, the sizes derived from it, the passes, and what the fused-column
// schedule needs.  R2CCL paper: Sec. 5.2 (ring steps and transmissions), Sec. 4.3 Technique II (a
// staging buffer per NIC channel), Sec. 5 (the other collectives' schedules).
#pragma once

#include "reduce_copy_device.h"
#include "ring_fused_device.h"

namespace r2 {
namespace {

bool valid_dtype(int d) { return d == R2_F32 || d == R2_BF16; }
uint64_t elem_bytes(int d) { return d == R2_F32 ? 4 : 2; }

// The stage bytes one launch writes are read back by the next launch.  Keeping that window well
// inside the 256 MiB Infinity Cache lets the read be served from it.
constexpr uint64_t kDefaultStageWindow = 128ull << 20;

// Channel buffers of ring chunks of 1 MiB and more are this much longer than the chunk.  Without it the
// buffers of all ranks and channels sit at power-of-two distances from each other and from the rank
// buffers, and with equal channels so do the slices inside them: every stream of a workgroup then maps
// to the same places in the caches and the memory channels.  Measured (128 KiB + 256 B against none):
// the all-reduce with no channel down 1010 -> 992 us at 128 MiB per rank, 4 ranks x 4 MiB fused
// 12.2 -> 10.7 us, 8 ranks x 8 MiB fused with three channels down 54 -> 45 us; pads of 1.25 KiB to 1 MiB
// were tried, several of which help one channel state and cost another a per cent.
constexpr uint64_t kStagePadBytes = (128ull << 10) + 256;
constexpr uint64_t kStagePadFromChunkBytes = 1ull << 20;

// R2_SCHED_AUTO picks the fused-column schedule when one ring step moves at most this many bytes
// per stream (summed over ranks and slabs): below it a launch per step is launch-bound.
constexpr uint64_t kFusedAutoBytes = 8ull << 20;

struct SimShape {
    uint32_t R, S, C, J, T_slab;
    uint64_t chunk_bytes, cap, n_tx;
    uint64_t tables_bytes, stage_off, total_bytes;
    // passes: the run is cut into groups of slabs, or one slab's chunks into byte ranges
    uint32_t slabs_per_pass, n_sub;
    uint64_t sub_bytes, n_passes;
    // What the run is.  Everything but the ring moves one message chunk per slab; the chains have one
    // rank active per step, the point-to-point kinds two steps and separate receive buffers.
    enum Kind { kRing, kSendRecv, kBroadcast, kReduce, kAllToAll } kind;
    uint32_t root;        // chains
    bool links;           // ring whose links have tables of their own (block r: r -> r+1), one row per transmission
    uint64_t tx_per_link; // transmissions of one rank: S * T_slab
    uint32_t a2a_chunks;  // all-to-all: the caller's chunks per block (S = (R-1) * a2a_chunks)
    bool two_lists() const { return kind == kSendRecv || kind == kAllToAll; }
    bool chain() const { return kind == kBroadcast || kind == kReduce; }
    uint32_t active() const { return chain() ? 1 : R; }  // ranks at work in one step
};

uint64_t round_up(uint64_t x, uint64_t m) { return (x + m - 1) / m * m; }

// Validates a descriptor and derives the sizes; returns an R2 code.
int shape_of(const r2_sim_desc *d, SimShape &s)
{
    if (!d) return R2_ERR_INVALID;
    if (d->n_ranks < 2 || d->n_ranks > R2_MAX_RANKS) return R2_ERR_INVALID;
    if (d->n_channels == 0 || d->n_channels > R2_MAX_CHANNELS) return R2_ERR_INVALID;
    if (d->n_slabs == 0) return R2_ERR_INVALID;
    if (d->align == 0 || d->align % 16 != 0) return R2_ERR_INVALID;
    if (!valid_dtype(d->dtype)) return R2_ERR_INVALID;
    s.links = (d->phases & R2_PHASE_LINKS) != 0;
    switch (d->phases & ~R2_PHASE_LINKS) {
    case R2_PHASE_RS:
    case R2_PHASE_AG:
    case R2_PHASE_RS | R2_PHASE_AG: s.kind = SimShape::kRing; break;
    case R2_PHASE_SENDRECV: s.kind = SimShape::kSendRecv; break;
    case R2_PHASE_BROADCAST: s.kind = SimShape::kBroadcast; break;
    case R2_PHASE_REDUCE: s.kind = SimShape::kReduce; break;
    case R2_PHASE_ALLTOALL: s.kind = SimShape::kAllToAll; break;
    default: return R2_ERR_INVALID;
    }
    if (d->schedule != R2_SCHED_AUTO && d->schedule != R2_SCHED_STEPS && d->schedule != R2_SCHED_FUSED &&
        d->schedule != R2_SCHED_STEPS_OVERLAP)
        return R2_ERR_INVALID;
    if (s.links && d->schedule == R2_SCHED_STEPS_OVERLAP) return R2_ERR_INVALID;
    if (s.links && s.kind != SimShape::kRing) return R2_ERR_INVALID;
    if (s.kind != SimShape::kRing && d->schedule == R2_SCHED_FUSED) return R2_ERR_INVALID;
    const int ring_phases = d->phases & ~R2_PHASE_LINKS;
    if (s.chain() ? (d->root < 0 || (uint32_t)d->root >= d->n_ranks) : d->root != 0) return R2_ERR_INVALID;
    s.R = d->n_ranks;
    s.root = (uint32_t)d->root;
    s.a2a_chunks = s.kind == SimShape::kAllToAll ? d->n_slabs : 0;
    // slabs as the schedule sees them: all-to-all has one per round and message chunk
    const uint64_t slabs = s.a2a_chunks ? (uint64_t)(s.R - 1) * d->n_slabs : d->n_slabs;
    if (slabs * s.R > 65535) return R2_ERR_INVALID;
    const bool blocks = s.kind == SimShape::kRing || s.kind == SimShape::kAllToAll;  // R pieces per slab
    const uint64_t per = blocks ? (uint64_t)d->n_slabs * s.R : d->n_slabs;
    if (d->n_elems % per != 0) return R2_ERR_INVALID;
    if (d->n_elems > (1ull << 60)) return R2_ERR_OVERFLOW;
    s.S = (uint32_t)slabs;
    s.C = d->n_channels;
    s.J = s.two_lists() ? 2 : ring_phases == (R2_PHASE_RS | R2_PHASE_AG) ? 2 * s.R - 1 : s.R;
    s.T_slab = s.J - 1;
    s.chunk_bytes = d->n_elems / per * elem_bytes(d->dtype);
    s.cap = round_up(s.chunk_bytes ? s.chunk_bytes : 1, 256) + (s.chunk_bytes >= kStagePadFromChunkBytes ? kStagePadBytes : 0);
    s.tx_per_link = (uint64_t)s.S * s.T_slab;
    s.n_tx = s.links ? s.R * s.tx_per_link : s.tx_per_link;  // rows of the tables
    s.tables_bytes = round_up(s.n_tx * (s.C + 1) * 8, 256);
    s.stage_off = s.tables_bytes;
    const unsigned __int128 stage = (unsigned __int128)2 * s.R * s.S * s.C * s.cap;
    if (stage > ((unsigned __int128)1 << 62)) return R2_ERR_OVERFLOW;
    s.total_bytes = s.stage_off + (uint64_t)stage;

    // The two-step exchanges use one stage parity only, so twice as much fits the same cache footprint.
    uint64_t window = d->stage_window_bytes ? d->stage_window_bytes
                      : s.two_lists()       ? 2 * kDefaultStageWindow
                                            : kDefaultStageWindow;
    const uint64_t per_slab = (uint64_t)s.active() * s.chunk_bytes;  // stage bytes a step writes per slab
    if (d->schedule == R2_SCHED_STEPS_OVERLAP) {
        // Two passes are in flight side by side: each gets half the window, and the run is cut into
        // at least two passes so that there is a pair to overlap.
        const uint64_t half_run = (per_slab * s.S + 1) / 2;
        window = window / 2 < half_run ? window / 2 : half_run;
        if (window == 0) window = 1;
    }
    if (per_slab > window) {
        const uint64_t tile_bytes = (uint64_t)kThreads * kUnroll * 16;
        const uint64_t parts = (per_slab + window - 1) / window;
        s.slabs_per_pass = 1;
        s.sub_bytes = round_up((s.chunk_bytes + parts - 1) / parts, tile_bytes);
        s.n_sub = (uint32_t)((s.chunk_bytes + s.sub_bytes - 1) / s.sub_bytes);
        s.n_passes = (uint64_t)s.S * s.n_sub;
    } else {
        const uint64_t fit = per_slab ? window / per_slab : s.S;
        s.slabs_per_pass = (uint32_t)(fit < 1 ? 1 : (fit > s.S ? s.S : fit));
        s.sub_bytes = s.chunk_bytes;
        s.n_sub = 1;
        s.n_passes = (s.S + s.slabs_per_pass - 1) / s.slabs_per_pass;
    }
    return R2_OK;
}

int check_workspace(const void *ws, uint64_t ws_bytes, const SimShape &s)
{
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return R2_ERR_INVALID;
    if (ws_bytes < s.total_bytes) return R2_ERR_CAPACITY;
    return R2_OK;
}

// The fused-column schedule needs whole 16-byte vectors everywhere and a grid that fits.
bool columns_fit(const SimShape &s)
{
    if (s.kind != SimShape::kRing) return false;
    if (s.chunk_bytes == 0 || s.chunk_bytes % 16 != 0) return false;
    const uint64_t cols = (s.chunk_bytes + kNarrowColBytes - 1) / kNarrowColBytes;
    return cols * s.S <= 0x7fffffffull;
}

// Vectors per lane of a run's columns (see kWideColumnsFrom).
unsigned fused_col_unroll(const SimShape &s)
{
    const uint64_t wide = (s.chunk_bytes + 2 * kNarrowColBytes - 1) / (2 * kNarrowColBytes);
    return wide * s.S >= kWideColumnsFrom ? 2 : 1;
}

}  // namespace
}  // namespace r2

// The kernels for one chunk and for one ring step of all ranks (the chunk worker they share is in
// reduce_copy_device.h, the fused-column kernels in ring_fused_device.h) and the host side of the ring
// schedule: descriptors, passes, launches and the C entry points.
//
// R2CCL paper: Sec. 2.1 (GPU kernels execute the collective over channels), Sec. 4.3 Technique II
// (per-NIC send staging buffers, chunk-granular progress), Sec. 5.2 (ring all-reduce = reduce-scatter,
// then all-gather), Sec. 5 and 5.1 (the other collectives keep their schedule under R2CCL-Balance),
// Sec. 6 (servers that lost different rails: the step kernel picks its tables per link; the host side
// of that ring is in rails.hip).
#include <mutex>
#include <new>
#include <vector>

#include "sim_shape.h"

namespace r2 {
namespace {

// ---------------------------------------------------------------- front end 1: one chunk

struct PtrList {
    uint64_t p[R2_MAX_CHANNELS];
};

template <Mode M, bool HAS_OUT, bool FWD = false, bool NT_OUT = false, bool KEEP = false>
__global__ __launch_bounds__(kThreads) void reduce_copy_kernel(ChunkJob job, const PtrList in_stage,
                                                               const PtrList out_stage, int32_t *status)
{
    __shared__ ChannelTable tin, tout;
    run_chunk<M, HAS_OUT, FWD, NT_OUT, KEEP>(
        job, [&](unsigned c) { return in_stage.p[c]; }, [&](unsigned c) { return out_stage.p[c]; },
        status, tin, tout);
}

// ---------------------------------------------------------------- front end 2: a ring step

struct StepArgs {
    uint64_t rank_buf[R2_MAX_RANKS];  // point-to-point: the send buffers at step 0, the receive buffers at step 1
    const uint64_t *tables;  // [S*T_slab][C+1]
    uint64_t stage;          // [2][R][S][C][cap]
    uint64_t chunk_bytes, cap;
    uint32_t R, S, C;
    uint32_t step;         // fused step j
    uint32_t T_slab;       // transmissions per slab
    uint32_t chunk_start;  // 1 when the run is an all-gather alone, else 0
    uint32_t per_slab;     // ring chunks per slab: R, or 1 where a slab is one message chunk
    uint32_t rank_base;    // the first rank this launch covers (chains: the one rank active at this step)
    uint32_t a2a_chunks;   // all-to-all: message chunks per block (a slab is chunk l % this of round l / this + 1), else 0
    uint64_t link_rows;    // > 0: `tables` holds a block of this many rows per ring link; rank r writes with block r
    uint32_t slab_begin, slab_count;  // the slabs this launch covers
    uint64_t lo, hi;                  // and the byte range of every ring chunk it moves
};

// blockIdx.y = (rank - rank_base) * slab_count + (slab - slab_begin), blockIdx.x = workgroup within
// the range.
template <Mode M, bool HAS_OUT, bool KEEP = false, bool NT_OUT = kNtStageStore>
__global__ __launch_bounds__(kThreads) void ring_step_kernel(const StepArgs a)
{
    __shared__ ChannelTable tin, tout;
    const uint32_t ri = blockIdx.y / a.slab_count, l = a.slab_begin + (blockIdx.y - ri * a.slab_count);
    const uint32_t r = (a.rank_base + ri) % a.R;
    const uint32_t j = a.step;
    const uint64_t row = (uint64_t)a.C + 1;
    const uint64_t t_out = (uint64_t)l * a.T_slab + j;
    uint32_t peer = (r + a.R - 1) % a.R;  // whose stage is read
    uint64_t piece;                       // which chunk-sized piece of the rank buffer is worked on
    if (a.a2a_chunks) {
        // round k: send the block for rank r+k (step 0), receive the block of rank r-k (step 1)
        const uint32_t k = l / a.a2a_chunks + 1, part = l - (k - 1) * a.a2a_chunks;
        peer = (r + a.R - k) % a.R;
        piece = (uint64_t)(j == 0 ? (r + k) % a.R : peer) * a.a2a_chunks + part;
    } else if (a.per_slab == 1) {
        piece = l;
    } else {
        piece = (uint64_t)l * a.per_slab + (r + a.chunk_start + 2 * a.R - j) % a.R;  // j <= 2R-2
    }

    ChunkJob job;
    job.local = reinterpret_cast<uint8_t *>(a.rank_buf[r]) + piece * a.chunk_bytes;
    job.bytes = a.chunk_bytes;
    job.lo = a.lo;
    job.hi = a.hi;
    job.in_off = M != kSend ? a.tables + (peer * a.link_rows + t_out - 1) * row : nullptr;
    job.out_off = HAS_OUT ? a.tables + (r * a.link_rows + t_out) * row : nullptr;
    job.cap = a.cap;
    job.C = a.C;
    // stage buffer of (parity, rank, slab, channel)
    const uint64_t in_base = a.stage + ((((uint64_t)((j + 1) & 1) * a.R + peer) * a.S + l) * a.C) * a.cap;
    const uint64_t out_base = a.stage + ((((uint64_t)(j & 1) * a.R + r) * a.S + l) * a.C) * a.cap;
    run_chunk<M, HAS_OUT, false, NT_OUT, KEEP>(
        job, [&](unsigned c) { return in_base + c * a.cap; },
        [&](unsigned c) { return out_base + c * a.cap; }, nullptr, tin, tout);
}

// All-to-all: a rank's own block goes from its send buffer to its receive buffer without touching a
// channel.  blockIdx.y = rank; 16-byte vectors where both addresses allow it, 2-byte units otherwise.
struct OwnBlockArgs {
    uint64_t src[R2_MAX_RANKS], dst[R2_MAX_RANKS];
    uint64_t bytes;  // per block; even
};

__global__ __launch_bounds__(kThreads) void own_block_copy_kernel(const OwnBlockArgs a)
{
    const uint64_t src = a.src[blockIdx.y], dst = a.dst[blockIdx.y];
    const uint64_t tid = (uint64_t)blockIdx.x * kThreads + threadIdx.x, n_threads = (uint64_t)gridDim.x * kThreads;
    const uint64_t n_vec = ((src | dst) & 15u) ? 0 : a.bytes / 16;
    for (uint64_t v = tid; v < n_vec; v += n_threads) store16<true>(dst + v * 16, load16<true>(src + v * 16));
    for (uint64_t i = n_vec * 8 + tid; i < a.bytes / 2; i += n_threads)
        *gptr<uint16_t>(dst + i * 2) = *gptr<const uint16_t>(src + i * 2);
}

// ---------------------------------------------------------------- host side

// One workgroup per tile of kThreads*kUnroll vectors: consecutive workgroups stream consecutive
// memory, which measured faster than fewer workgroups striding through the range.  (The kernels
// loop, so the cap only matters for ranges beyond 8 GiB.)
unsigned blocks_for(uint64_t range_bytes)
{
    const uint64_t tile_bytes = (uint64_t)kThreads * kUnroll * 16;
    uint64_t want = (range_bytes + tile_bytes - 1) / tile_bytes;
    if (want == 0) want = 1;
    const uint64_t limit = 1u << 20;
    return (unsigned)(want < limit ? want : limit);
}

Mode mode_of(bool has_in, int op, int dtype)
{
    if (!has_in) return kSend;
    if (op == R2_OP_COPY) return kCopy;
    return dtype == R2_F32 ? kSumF32 : kSumBF16;
}

int check_epochs(const r2_epoch *epochs, uint32_t n, const SimShape &s)
{
    if (!epochs || n == 0 || epochs[0].t_start != 0) return R2_ERR_INVALID;
    for (uint32_t i = 0; i < n; ++i) {
        if (!epochs[i].weights) return R2_ERR_INVALID;
        if (i && epochs[i].t_start <= epochs[i - 1].t_start) return R2_ERR_INVALID;
    }
    for (uint32_t i = 0; i < n; ++i) {
        if (epochs[i].t_start >= s.n_tx) break;  // never in force
        if (!any_healthy(epochs[i].weights, epochs[i].fail_mask, s.C)) return R2_ERR_NO_HEALTHY_CHANNEL;
    }
    return R2_OK;
}

// One channel state for every transmission of the run?
bool single_state(const r2_epoch *epochs, uint32_t n, const SimShape &s)
{
    return n < 2 || epochs[1].t_start >= s.n_tx;
}

// The plain ring's fused columns: not for per-link tables (rails.hip has those).
bool fused_eligible(const SimShape &s) { return !s.links && columns_fit(s); }

// A stage this large is gone from the caches before anybody reads it: written around them.
constexpr uint64_t kNtStageBytes = 128ull << 20;

// One fused step: `rows` (rank, slab) pairs, each moving bytes [lo, hi) of its ring chunk.  A stage of
// more than `cached_up_to` bytes per launch is written around the caches.
template <Mode M, bool HAS_OUT, bool KEEP = false>
void launch_step(const StepArgs &a, unsigned rows, uint64_t cached_up_to, hipStream_t st)
{
    const dim3 grid(blocks_for(a.hi - a.lo), rows);
    if (HAS_OUT && (uint64_t)rows * (a.hi - a.lo) > cached_up_to)
        hipLaunchKernelGGL((ring_step_kernel<M, HAS_OUT, KEEP, HAS_OUT>), grid, dim3(kThreads), 0, st, a);
    else
        hipLaunchKernelGGL((ring_step_kernel<M, HAS_OUT, KEEP, false>), grid, dim3(kThreads), 0, st, a);
}

// Decides between one launch per step and fused columns, and marks the steps before which a fused
// launch must end.  Inside a fused launch columns drift apart in time, so the data of transmission
// t (consumed at step t+1) and of transmission t+2 (same stage parity, written at step t+2) may
// only share a launch if both use the same table.  An epoch that starts at step c of some slab
// therefore forces a launch boundary before step c and another before step c+1.
int plan_schedule(const r2_sim_desc *desc, const SimShape &s, const r2_epoch *epochs, uint32_t n_epochs,
                  bool *cut /* [2*R2_MAX_RANKS] */)
{
    uint32_t n_cuts = 0;
    for (uint32_t j = 0; j < 2 * R2_MAX_RANKS; ++j) cut[j] = false;
    for (uint32_t i = 1; i < n_epochs && epochs[i].t_start < s.n_tx; ++i) {
        const uint32_t c = (uint32_t)(epochs[i].t_start % s.T_slab);
        if (c == 0) continue;  // a slab starts here: its stage buffers are its own
        for (uint32_t j = c; j <= c + 1 && j < s.T_slab; ++j) {
            if (!cut[j]) {
                cut[j] = true;
                ++n_cuts;
            }
        }
    }
    if (desc->schedule != R2_SCHED_AUTO) return desc->schedule;
    if (!fused_eligible(s)) return R2_SCHED_STEPS;
    // Launch-bound sizes gain from fewer launches; large ones keep one launch per ring step, the
    // schedule whose stage traffic really goes through memory.
    const uint64_t step_bytes = (uint64_t)s.R * s.S * s.chunk_bytes;
    const bool fewer = (uint64_t)(n_cuts + 1) * 2 <= s.n_passes * s.J;
    return step_bytes <= kFusedAutoBytes && fewer ? R2_SCHED_FUSED : R2_SCHED_STEPS;
}

template <Mode M, bool HAS_OUT, bool FWD = false, bool KEEP = false>
void launch_single(const ChunkJob &job, const PtrList &in, const PtrList &out, int32_t *status,
                   unsigned blocks, hipStream_t st)
{
    if (HAS_OUT && job.bytes > kNtStageBytes)
        hipLaunchKernelGGL((reduce_copy_kernel<M, HAS_OUT, FWD, HAS_OUT, KEEP>), dim3(blocks), dim3(kThreads), 0, st,
                           job, in, out, status);
    else
        hipLaunchKernelGGL((reduce_copy_kernel<M, HAS_OUT, FWD, false, KEEP>), dim3(blocks), dim3(kThreads), 0, st, job,
                           in, out, status);
}

}  // namespace
}  // namespace r2

using namespace r2;

extern "C" int r2_reduce_copy(void *local, uint64_t bytes, r2_dtype dtype, int op,
                              const void *const *in_stage, const uint64_t *in_offsets,
                              void *const *out_stage, const uint64_t *out_offsets,
                              uint32_t n_channels, uint64_t stage_capacity, int32_t *status,
                              void *stream)
{
    if (!valid_dtype(dtype) || (op != R2_OP_SUM && op != R2_OP_COPY && op != R2_OP_SUM_FORWARD && op != R2_OP_SUM_SEND))
        return R2_ERR_INVALID;
    if (n_channels == 0 || n_channels > R2_MAX_CHANNELS) return R2_ERR_INVALID;
    if (!in_stage && !out_stage) return R2_ERR_INVALID;
    if ((op == R2_OP_SUM_FORWARD || op == R2_OP_SUM_SEND) && (!in_stage || !out_stage)) return R2_ERR_INVALID;
    if ((in_stage && !in_offsets) || (out_stage && !out_offsets)) return R2_ERR_INVALID;
    if (bytes % elem_bytes(dtype) != 0) return R2_ERR_INVALID;
    if (bytes == 0) return R2_OK;
    if (!local || (reinterpret_cast<uintptr_t>(local) % elem_bytes(dtype)) != 0) return R2_ERR_INVALID;

    PtrList in{}, out{};
    for (uint32_t c = 0; c < n_channels; ++c) {
        if (in_stage) {
            in.p[c] = reinterpret_cast<uint64_t>(in_stage[c]);
            if (!in.p[c] || (in.p[c] & 15u)) return R2_ERR_INVALID;
        }
        if (out_stage) {
            out.p[c] = reinterpret_cast<uint64_t>(out_stage[c]);
            if (!out.p[c] || (out.p[c] & 15u)) return R2_ERR_INVALID;
        }
    }
    ChunkJob job{static_cast<uint8_t *>(local), bytes, 0, bytes, in_offsets, out_offsets, stage_capacity, n_channels};
    const unsigned blocks = blocks_for(bytes);
    hipStream_t st = (hipStream_t)stream;
    const Mode m = mode_of(in_stage != nullptr, op, dtype);
    const bool has_out = out_stage != nullptr;
    switch (m) {
    case kSend: launch_single<kSend, true>(job, in, out, status, blocks, st); break;
    case kSumF32:
        if (op == R2_OP_SUM_FORWARD) launch_single<kSumF32, true, true>(job, in, out, status, blocks, st);
        else if (op == R2_OP_SUM_SEND) launch_single<kSumF32, true, false, true>(job, in, out, status, blocks, st);
        else if (has_out) launch_single<kSumF32, true>(job, in, out, status, blocks, st);
        else launch_single<kSumF32, false>(job, in, out, status, blocks, st);
        break;
    case kSumBF16:
        if (op == R2_OP_SUM_FORWARD) launch_single<kSumBF16, true, true>(job, in, out, status, blocks, st);
        else if (op == R2_OP_SUM_SEND) launch_single<kSumBF16, true, false, true>(job, in, out, status, blocks, st);
        else if (has_out) launch_single<kSumBF16, true>(job, in, out, status, blocks, st);
        else launch_single<kSumBF16, false>(job, in, out, status, blocks, st);
        break;
    case kCopy:
        if (has_out) launch_single<kCopy, true>(job, in, out, status, blocks, st);
        else launch_single<kCopy, false>(job, in, out, status, blocks, st);
        break;
    }
    return hip_rc(hipGetLastError());
}

extern "C" uint32_t r2_sim_num_steps(const r2_sim_desc *desc)
{
    SimShape s;
    return shape_of(desc, s) == R2_OK ? s.J : 0;
}

extern "C" uint64_t r2_sim_num_transmissions(const r2_sim_desc *desc)
{
    SimShape s;
    return shape_of(desc, s) == R2_OK ? s.n_tx : 0;
}

extern "C" uint64_t r2_sim_workspace_bytes(const r2_sim_desc *desc)
{
    SimShape s;
    return shape_of(desc, s) == R2_OK ? s.total_bytes : 0;
}

extern "C" uint64_t r2_sim_stage_offset(const r2_sim_desc *desc)
{
    SimShape s;
    return shape_of(desc, s) == R2_OK ? s.stage_off : 0;
}

extern "C" uint64_t r2_sim_stage_capacity(const r2_sim_desc *desc)
{
    SimShape s;
    return shape_of(desc, s) == R2_OK ? s.cap : 0;
}

extern "C" int r2_sim_prepare(const r2_sim_desc *desc, const r2_epoch *epochs, uint32_t n_epochs,
                              void *workspace, uint64_t workspace_bytes, uint64_t *offsets_log,
                              void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (s.links) return R2_ERR_INVALID;  // per-link tables are made by r2_ring_rails_sim
    if ((rc = check_epochs(epochs, n_epochs, s))) return rc;
    if ((rc = check_workspace(workspace, workspace_bytes, s))) return rc;
    if (s.n_tx == 0) return R2_OK;
    return launch_partition_epochs(epochs, n_epochs, s.C, desc->align, s.chunk_bytes, s.n_tx,
                                   static_cast<uint64_t *>(workspace), offsets_log, (hipStream_t)stream);
}

extern "C" uint64_t r2_sim_num_passes(const r2_sim_desc *desc)
{
    SimShape s;
    return shape_of(desc, s) == R2_OK ? s.n_passes : 0;
}

extern "C" int r2_sim_step(const r2_sim_desc *desc, void *const *rank_bufs, uint64_t pass,
                           uint32_t step, void *workspace, uint64_t workspace_bytes, void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (!rank_bufs || step >= s.J || pass >= s.n_passes) return R2_ERR_INVALID;
    if ((rc = check_workspace(workspace, workspace_bytes, s))) return rc;
    StepArgs a{};
    const uint32_t first_buf = s.two_lists() && step == 1 ? s.R : 0;  // receives go into the second list
    for (uint32_t r = 0; r < s.R; ++r) {
        a.rank_buf[r] = reinterpret_cast<uint64_t>(rank_bufs[first_buf + r]);
        if (s.chunk_bytes && (!a.rank_buf[r] || (a.rank_buf[r] & 15u))) return R2_ERR_INVALID;
    }
    if (s.chunk_bytes == 0) return R2_OK;
    a.tables = static_cast<const uint64_t *>(workspace);
    a.stage = reinterpret_cast<uint64_t>(workspace) + s.stage_off;
    a.chunk_bytes = s.chunk_bytes;
    a.cap = s.cap;
    a.R = s.R;
    a.S = s.S;
    a.C = s.C;
    a.step = step;
    a.T_slab = s.T_slab;
    const int ring_phases = desc->phases & ~R2_PHASE_LINKS;
    a.chunk_start = ring_phases == R2_PHASE_AG ? 1 : 0;
    a.per_slab = s.kind == SimShape::kRing ? s.R : 1;
    a.a2a_chunks = s.a2a_chunks;
    a.link_rows = s.links ? s.tx_per_link : 0;
    // a chain has one rank at work per step: the step-th after the root, or after the root's successor
    a.rank_base = s.kind == SimShape::kBroadcast ? (s.root + step) % s.R
                  : s.kind == SimShape::kReduce  ? (s.root + 1 + step) % s.R
                                                 : 0;
    if (s.n_sub > 1) {  // one slab, one byte range of its chunks
        a.slab_begin = (uint32_t)(pass / s.n_sub);
        a.slab_count = 1;
        a.lo = (pass % s.n_sub) * s.sub_bytes;
        a.hi = a.lo + s.sub_bytes < s.chunk_bytes ? a.lo + s.sub_bytes : s.chunk_bytes;
    } else {  // a group of whole slabs
        a.slab_begin = (uint32_t)(pass * s.slabs_per_pass);
        a.slab_count = s.S - a.slab_begin < s.slabs_per_pass ? s.S - a.slab_begin : s.slabs_per_pass;
        a.lo = 0;
        a.hi = s.chunk_bytes;
    }

    const bool has_in = step > 0, has_out = step < s.J - 1;
    int op;
    if (ring_phases == R2_PHASE_AG || s.two_lists() || s.kind == SimShape::kBroadcast) op = R2_OP_COPY;
    else if (ring_phases == R2_PHASE_RS || s.kind == SimShape::kReduce) op = R2_OP_SUM;
    else op = step <= s.R - 1 ? R2_OP_SUM : R2_OP_COPY;
    const Mode m = mode_of(has_in, op, desc->dtype);
    const bool keep = s.kind == SimShape::kReduce && has_in && has_out;  // the sum is passed on, not kept

    const unsigned grid = s.active() * a.slab_count;  // rows of workgroups: one per (rank, slab)
    // the two-step exchanges use one stage parity only: twice as much stays within reach of the next step
    const uint64_t keep_cached = s.two_lists() ? 2 * kNtStageBytes : kNtStageBytes;
    hipStream_t st = (hipStream_t)stream;
    switch (m) {
    case kSend: launch_step<kSend, true>(a, grid, keep_cached, st); break;
    case kSumF32:
        if (keep) launch_step<kSumF32, true, true>(a, grid, keep_cached, st);
        else if (has_out) launch_step<kSumF32, true>(a, grid, keep_cached, st);
        else launch_step<kSumF32, false>(a, grid, keep_cached, st);
        break;
    case kSumBF16:
        if (keep) launch_step<kSumBF16, true, true>(a, grid, keep_cached, st);
        else if (has_out) launch_step<kSumBF16, true>(a, grid, keep_cached, st);
        else launch_step<kSumBF16, false>(a, grid, keep_cached, st);
        break;
    case kCopy:
        if (has_out) launch_step<kCopy, true>(a, grid, keep_cached, st); else launch_step<kCopy, false>(a, grid, keep_cached, st);
        break;
    }
    return hip_rc(hipGetLastError());
}

extern "C" int r2_sim_resolve_schedule(const r2_sim_desc *desc, const r2_epoch *epochs, uint32_t n_epochs)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (s.links) return R2_ERR_INVALID;  // one epoch list cannot say what a ring with per-link tables will do
    if ((rc = check_epochs(epochs, n_epochs, s))) return rc;
    if (desc->schedule == R2_SCHED_FUSED && s.chunk_bytes && !fused_eligible(s)) return R2_ERR_INVALID;
    // one slab whose state changes on the way has no two passes that may run side by side
    if (desc->schedule == R2_SCHED_STEPS_OVERLAP && s.S == 1 && !single_state(epochs, n_epochs, s)) return R2_SCHED_STEPS;
    bool cut[2 * R2_MAX_RANKS];
    return plan_schedule(desc, s, epochs, n_epochs, cut);
}

namespace r2 {
namespace {

// LDS bytes for the table rows of the steps [step_begin, step_end), or 0 if they do not fit.
uint32_t fused_row_bytes(const SimShape &s, uint32_t step_begin, uint32_t step_end)
{
    const uint32_t t_first = step_begin ? step_begin - 1 : 0;
    const uint32_t t_end = step_end < s.T_slab ? step_end : s.T_slab;
    const uint64_t row_bytes = t_end > t_first ? (uint64_t)(t_end - t_first) * (s.C + 1) * 8 : 8;
    return row_bytes <= kFusedLdsRowBytes ? (uint32_t)row_bytes : 0;
}

// One fused launch.  With `eb` the kernel partitions on its own (needs the rows to fit LDS).
int launch_fused(const r2_sim_desc *desc, const SimShape &s, void *const *rank_bufs, uint32_t step_begin,
                 uint32_t step_end, void *workspace, const EpochBatch *eb, uint64_t *log, hipStream_t stream)
{
    FusedArgs a{};
    for (uint32_t r = 0; r < s.R; ++r) {
        a.rank_buf[r] = reinterpret_cast<uint64_t>(rank_bufs[r]);
        if (!a.rank_buf[r] || (a.rank_buf[r] & 15u)) return R2_ERR_INVALID;
    }
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
    a.chunk_start = desc->phases == R2_PHASE_AG ? 1 : 0;
    a.sum_last = desc->phases == R2_PHASE_AG ? 0 : s.R - 1;
    a.j0 = step_begin;
    a.j1 = step_end;
    const uint32_t lds = fused_row_bytes(s, step_begin, step_end);
    a.rows_in_lds = lds != 0;
    if (eb && !lds) return R2_ERR_INVALID;
    const unsigned waves = s.R < kMaxFusedWaves ? s.R : kMaxFusedWaves;
    const dim3 grid((unsigned)(a.cols_per_chunk * s.S)), block(waves * kWave);
    const bool bf16 = desc->dtype == R2_BF16;
    if (eb) {
        if (unroll == 2) {
            if (bf16) hipLaunchKernelGGL((ring_fused_partition_kernel<true, 2>), grid, block, lds, stream, a, *eb);
            else hipLaunchKernelGGL((ring_fused_partition_kernel<false, 2>), grid, block, lds, stream, a, *eb);
        } else {
            if (bf16) hipLaunchKernelGGL((ring_fused_partition_kernel<true, 1>), grid, block, lds, stream, a, *eb);
            else hipLaunchKernelGGL((ring_fused_partition_kernel<false, 1>), grid, block, lds, stream, a, *eb);
        }
    } else {
        if (unroll == 2) {
            if (bf16) hipLaunchKernelGGL((ring_fused_kernel<true, 2>), grid, block, lds, stream, a);
            else hipLaunchKernelGGL((ring_fused_kernel<false, 2>), grid, block, lds, stream, a);
        } else {
            if (bf16) hipLaunchKernelGGL((ring_fused_kernel<true, 1>), grid, block, lds, stream, a);
            else hipLaunchKernelGGL((ring_fused_kernel<false, 1>), grid, block, lds, stream, a);
        }
    }
    return hip_rc(hipGetLastError());
}

}  // namespace
}  // namespace r2

extern "C" int r2_sim_fused_steps(const r2_sim_desc *desc, void *const *rank_bufs, uint32_t step_begin,
                                  uint32_t step_end, void *workspace, uint64_t workspace_bytes,
                                  void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (!rank_bufs || step_begin >= step_end || step_end > s.J) return R2_ERR_INVALID;
    if ((rc = check_workspace(workspace, workspace_bytes, s))) return rc;
    if (s.chunk_bytes == 0) {
        for (uint32_t r = 0; r < s.R; ++r)
            if (reinterpret_cast<uint64_t>(rank_bufs[r]) & 15u) return R2_ERR_INVALID;
        return R2_OK;
    }
    if (!fused_eligible(s)) return R2_ERR_INVALID;
    return launch_fused(desc, s, rank_bufs, step_begin, step_end, workspace, nullptr, nullptr, (hipStream_t)stream);
}

extern "C" int r2_ring_allreduce_sim(const r2_sim_desc *desc, void *const *rank_bufs,
                                     const r2_epoch *epochs, uint32_t n_epochs, void *workspace,
                                     uint64_t workspace_bytes, uint64_t *offsets_log, void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (!rank_bufs) return R2_ERR_INVALID;
    for (uint32_t r = 0; r < (s.two_lists() ? 2 * s.R : s.R); ++r) {
        const uint64_t p = reinterpret_cast<uint64_t>(rank_bufs[r]);
        if (s.chunk_bytes && (!p || (p & 15u))) return R2_ERR_INVALID;
    }
    if (s.links) return R2_ERR_INVALID;  // per-link tables come from r2_ring_rails_sim, not from epochs
    if (desc->schedule == R2_SCHED_FUSED && s.chunk_bytes && !fused_eligible(s)) return R2_ERR_INVALID;
    if ((rc = check_epochs(epochs, n_epochs, s))) return rc;
    if ((rc = check_workspace(workspace, workspace_bytes, s))) return rc;

    if (desc->schedule == R2_SCHED_STEPS_OVERLAP && s.S == 1 && !single_state(epochs, n_epochs, s)) {
        // One slab whose channel state changes on the way: its byte ranges cannot run side by side
        // (see below), so the run takes the plain step schedule, with that schedule's window.
        r2_sim_desc plain = *desc;
        plain.schedule = R2_SCHED_STEPS;
        return r2_ring_allreduce_sim(&plain, rank_bufs, epochs, n_epochs, workspace, workspace_bytes, offsets_log, stream);
    }

    bool cut[2 * R2_MAX_RANKS];
    const bool fused = s.chunk_bytes && plan_schedule(desc, s, epochs, n_epochs, cut) == R2_SCHED_FUSED;
    if (fused) {
        // The fused kernels partition for themselves if the whole epoch list fits one argument
        // block and every launch's rows fit LDS; otherwise the tables are prepared up front.
        bool self = n_epochs <= epochs_per_batch(s.C);
        uint32_t j0 = 0;
        for (uint32_t j = 1; j <= s.J && self; ++j)
            if (j == s.J || cut[j]) {
                self = fused_row_bytes(s, j0, j) != 0;
                j0 = j;
            }
        EpochBatch eb;
        if (self) fill_batch(eb, epochs, 0, n_epochs, s.C);
        else if ((rc = r2_sim_prepare(desc, epochs, n_epochs, workspace, workspace_bytes, offsets_log, stream)))
            return rc;
        j0 = 0;
        for (uint32_t j = 1; j <= s.J; ++j) {
            if (j == s.J || cut[j]) {
                if ((rc = launch_fused(desc, s, rank_bufs, j0, j, workspace, self ? &eb : nullptr,
                                       self ? offsets_log : nullptr, (hipStream_t)stream)))
                    return rc;
                j0 = j;
            }
        }
        return R2_OK;
    }
    if ((rc = r2_sim_prepare(desc, epochs, n_epochs, workspace, workspace_bytes, offsets_log, stream)))
        return rc;
    if (s.chunk_bytes == 0) return R2_OK;
    if (s.kind == SimShape::kAllToAll) {  // every rank keeps its own block: no channel involved
        OwnBlockArgs own{};
        own.bytes = s.chunk_bytes * s.a2a_chunks;
        for (uint32_t r = 0; r < s.R; ++r) {
            own.src[r] = reinterpret_cast<uint64_t>(rank_bufs[r]) + r * own.bytes;
            own.dst[r] = reinterpret_cast<uint64_t>(rank_bufs[s.R + r]) + r * own.bytes;
        }
        const uint64_t want = (own.bytes + kThreads * 16 - 1) / (kThreads * 16);
        const dim3 grid((unsigned)(want < 4096 ? want : 4096), s.R);
        hipLaunchKernelGGL(own_block_copy_kernel, grid, dim3(kThreads), 0, (hipStream_t)stream, own);
        if ((rc = hip_rc(hipGetLastError()))) return rc;
    }
    if (desc->schedule == R2_SCHED_STEPS_OVERLAP && s.n_passes >= 2) {
        // Two passes side by side, issued step by step alternately so that their launches interleave in
        // time.  Passes that cover different slabs share nothing.  Byte ranges of ONE slab share its
        // stage buffers: under one table their slices are disjoint, but a pass that is a step ahead and
        // already writes with a newer table would overwrite stage bytes the other has not read yet (the
        // hazard of the fused columns).  So such passes only run side by side while one channel state
        // holds for the whole run; otherwise the lanes are split by slab (even / odd), and a run of a
        // single slab was sent to the plain schedule above.  The fork point lies behind the partition
        // launch, which both lanes need.
        const bool by_slab = s.n_sub > 1 && !single_state(epochs, n_epochs, s);
        ForkJoin lanes((hipStream_t)stream);
        if (lanes.rc()) return lanes.rc();
        void *const lane[2] = {stream, lanes.lane(1)};
        uint64_t next[2] = {0, 0};  // per lane: the pass it takes next
        auto mine = [&](uint64_t p, unsigned l) { return ((by_slab ? p / s.n_sub : p) & 1u) == l; };
        for (;;) {
            for (unsigned l = 0; l < 2; ++l)
                while (next[l] < s.n_passes && !mine(next[l], l)) ++next[l];
            if (next[0] >= s.n_passes && next[1] >= s.n_passes) break;
            for (uint32_t j = 0; j < s.J; ++j)
                for (unsigned l = 0; l < 2; ++l)
                    if (next[l] < s.n_passes &&
                        (rc = r2_sim_step(desc, rank_bufs, next[l], j, workspace, workspace_bytes, lane[l])))
                        return rc;
            ++next[0];
            ++next[1];
        }
        return lanes.join();
    }
    for (uint64_t p = 0; p < s.n_passes; ++p)
        for (uint32_t j = 0; j < s.J; ++j)
            if ((rc = r2_sim_step(desc, rank_bufs, p, j, workspace, workspace_bytes, stream))) return rc;
    return R2_OK;
}

// ---------------------------------------------------------------- failures that strike in flight
//
// Sec. 4.3 Technique II.  An epoch marked in flight leaves the transmission it strikes in with the
// table of the state before it; the tables therefore see that epoch one transmission later, and an
// epoch that a later one overtakes that way never cuts a table.  Its failover plan is made by a
// launch of its own in front of the run.
extern "C" int r2_ring_allreduce_sim_inflight(const r2_sim_desc *desc, void *const *rank_bufs,
                                              const r2_epoch *epochs, const uint8_t *in_flight, uint32_t n_epochs,
                                              void *workspace, uint64_t workspace_bytes, uint64_t *offsets_log,
                                              uint64_t *plans, void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (s.links) return R2_ERR_INVALID;
    if ((rc = check_epochs(epochs, n_epochs, s))) return rc;
    bool any = false;
    for (uint32_t i = 0; in_flight && i < n_epochs; ++i) {
        if (!in_flight[i]) continue;
        if (i == 0) return R2_ERR_INVALID;  // no table before the first state
        if (epochs[i - 1].fail_mask & ~epochs[i].fail_mask) return R2_ERR_INVALID;  // failures only: recoveries
                                                                                    // come between transmissions
        any = true;
    }
    if (any && !plans) return R2_ERR_INVALID;
    if (!any) {
        if (plans) {  // every row is written: zero
            rc = launch_inflight_plans(epochs, nullptr, n_epochs, s.C, desc->align, s.chunk_bytes, s.n_tx, plans,
                                       (hipStream_t)stream);
            if (rc) return rc;
        }
        return r2_ring_allreduce_sim(desc, rank_bufs, epochs, n_epochs, workspace, workspace_bytes, offsets_log, stream);
    }
    try {
        std::vector<r2_epoch> seen;  // the list as the tables see it
        seen.reserve(n_epochs);
        for (uint32_t i = 0; i < n_epochs; ++i) {
            r2_epoch e = epochs[i];
            if (in_flight[i]) ++e.t_start;
            while (!seen.empty() && seen.back().t_start >= e.t_start) seen.pop_back();
            seen.push_back(e);
        }
        if (!rank_bufs) return R2_ERR_INVALID;
        if ((rc = check_workspace(workspace, workspace_bytes, s))) return rc;
        rc = launch_inflight_plans(epochs, in_flight, n_epochs, s.C, desc->align, s.chunk_bytes, s.n_tx, plans,
                                   (hipStream_t)stream);
        if (rc) return rc;
        return r2_ring_allreduce_sim(desc, rank_bufs, seen.data(), (uint32_t)seen.size(), workspace, workspace_bytes,
                                     offsets_log, stream);
    } catch (const std::bad_alloc &) {
        return R2_ERR_CAPACITY;
    }
}

// ---------------------------------------------------------------- the run whose workspace is a static array
//
// For callers that cannot allocate.  The tables and the stage area of the run live in a file-scope
// device array; each GPU the library's code object is loaded on holds its own copy at its own
// address, which is asked for once per device and kept.  In host code the array's name is only a
// handle for that query: every use of the memory goes through the address it returned.
namespace r2 {
namespace {

static __device__ __align__(256) unsigned char scratch[R2_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices];  // per device: where `scratch` lives there, or null while unknown

// The current device's copy of `scratch`.  The first call on a device looks the address up; nothing
// is allocated then or later.
int scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return R2_ERR_DEVICE;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return R2_ERR_DEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return R2_OK;
}

}  // namespace
}  // namespace r2

extern "C" int r2_ring_allreduce_sim_static(const r2_sim_desc *desc, void *const *rank_bufs,
                                            const r2_epoch *epochs, uint32_t n_epochs,
                                            uint64_t *offsets_log, void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    // the overlapped schedule creates its side stream and events at first use: not for a caller that may not allocate
    if (desc->schedule == R2_SCHED_STEPS_OVERLAP) return R2_ERR_INVALID;
    if (s.total_bytes > R2_STATIC_WORKSPACE_BYTES) return R2_ERR_CAPACITY;
    void *ws = nullptr;
    if ((rc = scratch_of_current_device(&ws))) return rc;
    // Nothing in the workspace has to start at zero: every table row is written (by the partition
    // launch, or by the fused kernels themselves) before a step reads it, and a step only reads the
    // stage bytes the step before it wrote.  What an earlier call left there is never looked at.
    return r2_ring_allreduce_sim(desc, rank_bufs, epochs, n_epochs, ws, R2_STATIC_WORKSPACE_BYTES, offsets_log, stream);
}

extern "C" int r2_collective_sim(const r2_sim_desc *desc, void *const *rank_bufs, const r2_epoch *epochs,
                                 uint32_t n_epochs, void *workspace, uint64_t workspace_bytes,
                                 uint64_t *offsets_log, void *stream)
{
    return r2_ring_allreduce_sim(desc, rank_bufs, epochs, n_epochs, workspace, workspace_bytes, offsets_log, stream);
}

extern "C" int r2_sendrecv_sim(const r2_sim_desc *desc, const void *const *send_bufs, void *const *recv_bufs,
                               const r2_epoch *epochs, uint32_t n_epochs, void *workspace,
                               uint64_t workspace_bytes, uint64_t *offsets_log, void *stream)
{
    if (!desc || desc->phases != R2_PHASE_SENDRECV || !send_bufs || !recv_bufs) return R2_ERR_INVALID;
    if (desc->n_ranks < 2 || desc->n_ranks > R2_MAX_RANKS) return R2_ERR_INVALID;
    void *both[2 * R2_MAX_RANKS];
    for (uint32_t r = 0; r < desc->n_ranks; ++r) {
        both[r] = const_cast<void *>(send_bufs[r]);  // step 0 only reads them
        both[desc->n_ranks + r] = recv_bufs[r];
        for (uint32_t q = 0; q < desc->n_ranks; ++q)
            if (send_bufs[q] == recv_bufs[r] && desc->n_elems) return R2_ERR_INVALID;  // no in-place exchange
    }
    return r2_ring_allreduce_sim(desc, both, epochs, n_epochs, workspace, workspace_bytes, offsets_log, stream);
}

extern "C" int r2_alltoall_sim(const r2_sim_desc *desc, const void *const *send_bufs, void *const *recv_bufs,
                               const r2_epoch *epochs, uint32_t n_epochs, void *workspace,
                               uint64_t workspace_bytes, uint64_t *offsets_log, void *stream)
{
    if (!desc || desc->phases != R2_PHASE_ALLTOALL || !send_bufs || !recv_bufs) return R2_ERR_INVALID;
    if (desc->n_ranks < 2 || desc->n_ranks > R2_MAX_RANKS) return R2_ERR_INVALID;
    void *both[2 * R2_MAX_RANKS];
    for (uint32_t r = 0; r < desc->n_ranks; ++r) {
        both[r] = const_cast<void *>(send_bufs[r]);  // only read
        both[desc->n_ranks + r] = recv_bufs[r];
        for (uint32_t q = 0; q < desc->n_ranks; ++q)
            if (send_bufs[q] == recv_bufs[r] && desc->n_elems) return R2_ERR_INVALID;  // no in-place exchange
    }
    return r2_ring_allreduce_sim(desc, both, epochs, n_epochs, workspace, workspace_bytes, offsets_log, stream);
}

extern "C" const char *r2_strerror(int code)
{
    switch (code) {
    case R2_OK: return "success";
    case R2_ERR_INVALID: return "invalid argument";
    case R2_ERR_NO_HEALTHY_CHANNEL: return "no healthy channel left";
    case R2_ERR_OVERFLOW: return "size does not fit 64 bits";
    case R2_ERR_CAPACITY: return "stage buffer or workspace too small";
    case R2_ERR_DEVICE: return "HIP runtime error";
    default: return "unknown r2ccl error code";
    }
}

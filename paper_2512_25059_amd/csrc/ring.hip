// Fused reduce-copy and the ring schedule built from it.
//
// R2CCL paper: Sec. 2.1 (a collective's data is cut over channels, each bound to a NIC, and GPU
// kernels execute the collective over them), Sec. 4.3 Technique II (per-NIC send staging buffers,
// chunk-granular progress), Sec. 5.2 (ring all-reduce = reduce-scatter, then all-gather).
//
// The data path is bandwidth-bound: per 16-byte vector two loads, one add, two stores.  Every lane
// moves whole 16-byte vectors; a wavefront touches 1 KiB of consecutive addresses per access.  The
// channel of a vector is found by a short binary search in an LDS copy of the offsets table.
#include <type_traits>

#include "r2_internal.h"

namespace r2 {
namespace {

constexpr unsigned kThreads = 256;
constexpr unsigned kUnroll = 4;        // 16-byte vectors in flight per lane and stream
constexpr unsigned kBlocksPerCU = 8;   // grid target: this many workgroups per compute unit
constexpr unsigned kComputeUnits = 256;

enum Mode : int { kSend = 0, kSumF32 = 1, kSumBF16 = 2, kCopy = 3 };

// ---------------------------------------------------------------- arithmetic on 16-byte vectors

__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }

// fp32 -> bf16, round to nearest even; NaN stays NaN (quiet).
__device__ inline uint32_t to_bf16(float f)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ inline uint32_t add_bf16x2(uint32_t a, uint32_t b)
{
    const uint32_t lo = to_bf16(bf16_lo(a) + bf16_lo(b));
    const uint32_t hi = to_bf16(bf16_hi(a) + bf16_hi(b));
    return lo | (hi << 16);
}

template <Mode M>
__device__ inline uint4 combine(const uint4 &incoming, const uint4 &local)
{
    if constexpr (M == kSumF32) {
        uint4 v;
        v.x = __float_as_uint(__uint_as_float(incoming.x) + __uint_as_float(local.x));
        v.y = __float_as_uint(__uint_as_float(incoming.y) + __uint_as_float(local.y));
        v.z = __float_as_uint(__uint_as_float(incoming.z) + __uint_as_float(local.z));
        v.w = __float_as_uint(__uint_as_float(incoming.w) + __uint_as_float(local.w));
        return v;
    } else if constexpr (M == kSumBF16) {
        uint4 v;
        v.x = add_bf16x2(incoming.x, local.x);
        v.y = add_bf16x2(incoming.y, local.y);
        v.z = add_bf16x2(incoming.z, local.z);
        v.w = add_bf16x2(incoming.w, local.w);
        return v;
    } else if constexpr (M == kCopy) {
        return incoming;
    } else {
        return local;
    }
}

// ---------------------------------------------------------------- channel tables in LDS

struct ChannelTable {
    uint64_t off[R2_MAX_CHANNELS + 1];
    uint64_t delta[R2_MAX_CHANNELS];  // stage address of chunk byte b in channel c is delta[c] + b
};

// Channel that owns chunk byte b: the first c with off[c+1] > b (zero-length slices are skipped).
__device__ inline uint32_t find_channel(const uint64_t *off, uint32_t C, uint64_t b)
{
    uint32_t lo = 0, hi = C - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (off[mid + 1] > b) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// Lanes 0..C of the workgroup copy one table to LDS and check it.  Returns 0 or an R2_ERR code
// (per lane; the caller combines them).
__device__ inline int load_table(ChannelTable &t, const uint64_t *__restrict__ g_off,
                                 uint64_t base_c, uint32_t C, uint64_t bytes, uint64_t cap)
{
    const unsigned c = threadIdx.x;
    int bad = 0;
    if (c <= C) {
        const uint64_t o = g_off[c];
        t.off[c] = o;
        if (c == 0 && o != 0) bad = R2_ERR_INVALID;
        if (c == C && o != bytes) bad = R2_ERR_INVALID;
        if (c < C) {
            const uint64_t next = g_off[c + 1];
            if (next < o) bad = R2_ERR_INVALID;
            else if (next - o > cap) bad = R2_ERR_CAPACITY;
            if (next != o && (o & 15u)) bad = R2_ERR_INVALID;  // a non-empty slice starts on 16 B
            t.delta[c] = base_c - o;
        }
    }
    return bad;
}

// ---------------------------------------------------------------- the chunk worker

struct ChunkJob {
    uint8_t *local;
    uint64_t bytes;
    const uint64_t *in_off;   // device table or null
    const uint64_t *out_off;  // device table or null
    uint64_t cap;
    uint32_t C;
};

template <Mode M, bool HAS_OUT, typename InPtr, typename OutPtr>
__device__ inline void run_chunk(const ChunkJob &job, InPtr in_ptr, OutPtr out_ptr, int32_t *status,
                                 ChannelTable &tin, ChannelTable &tout)
{
    constexpr bool HAS_IN = M != kSend;
    constexpr bool NEED_LOCAL = M != kCopy;
    const uint32_t C = job.C;

    // Tables to LDS, with a sanity check whose verdict is the same in every workgroup.
    int bad = 0;
    if constexpr (HAS_IN) {
        const unsigned c = threadIdx.x;
        bad = load_table(tin, job.in_off, c < C ? in_ptr(c) : 0, C, job.bytes, job.cap);
    }
    if constexpr (HAS_OUT) {
        const unsigned c = threadIdx.x;
        const int b2 = load_table(tout, job.out_off, c < C ? out_ptr(c) : 0, C, job.bytes, job.cap);
        if (!bad) bad = b2;
    }
    if (__syncthreads_or(bad)) {
        if (bad && status) atomicMin(status, bad);
        return;
    }

    uint8_t *const local = job.local;
    const bool aligned = (reinterpret_cast<uintptr_t>(local) & 15u) == 0;
    const uint64_t nvec = aligned ? job.bytes / 16 : 0;

    const uint64_t tile = (uint64_t)kThreads * kUnroll;
    for (uint64_t v0 = (uint64_t)blockIdx.x * tile; v0 < nvec; v0 += (uint64_t)gridDim.x * tile) {
        uint4 inc[kUnroll], loc[kUnroll];
#pragma unroll
        for (unsigned u = 0; u < kUnroll; ++u) {
            const uint64_t v = v0 + u * kThreads + threadIdx.x;
            if (v < nvec) {
                const uint64_t b = v * 16;
                if constexpr (HAS_IN) {
                    const uint32_t c = find_channel(tin.off, C, b);
                    inc[u] = *reinterpret_cast<const uint4 *>(tin.delta[c] + b);
                }
                if constexpr (NEED_LOCAL) loc[u] = *reinterpret_cast<const uint4 *>(local + b);
            }
        }
#pragma unroll
        for (unsigned u = 0; u < kUnroll; ++u) {
            const uint64_t v = v0 + u * kThreads + threadIdx.x;
            if (v < nvec) {
                const uint64_t b = v * 16;
                const uint4 r = combine<M>(inc[u], loc[u]);
                if constexpr (HAS_IN) *reinterpret_cast<uint4 *>(local + b) = r;
                if constexpr (HAS_OUT) {
                    const uint32_t c = find_channel(tout.off, C, b);
                    *reinterpret_cast<uint4 *>(tout.delta[c] + b) = r;
                }
            }
        }
    }

    // What the vectors did not cover, one element at a time: the last bytes % 16 of an aligned
    // chunk, or all of a chunk whose address is only element-aligned.
    using Elem = typename std::conditional<M == kSumF32, uint32_t, uint16_t>::type;
    const uint64_t first = nvec * 16;
    const uint64_t n_el = (job.bytes - first) / sizeof(Elem);
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < n_el;
         i += (uint64_t)gridDim.x * kThreads) {
        const uint64_t b = first + i * sizeof(Elem);
        Elem x_in = 0, x_loc = 0;
        if constexpr (HAS_IN) {
            const uint32_t c = find_channel(tin.off, C, b);
            x_in = *reinterpret_cast<const Elem *>(tin.delta[c] + b);
        }
        if constexpr (NEED_LOCAL) x_loc = *reinterpret_cast<const Elem *>(local + b);
        Elem r;
        if constexpr (M == kSumF32) r = __float_as_uint(__uint_as_float(x_in) + __uint_as_float(x_loc));
        else if constexpr (M == kSumBF16) r = (Elem)to_bf16(bf16_lo(x_in) + bf16_lo(x_loc));
        else if constexpr (M == kCopy) r = x_in;
        else r = x_loc;
        if constexpr (HAS_IN) *reinterpret_cast<Elem *>(local + b) = r;
        if constexpr (HAS_OUT) {
            const uint32_t c = find_channel(tout.off, C, b);
            *reinterpret_cast<Elem *>(tout.delta[c] + b) = r;
        }
    }
}

// ---------------------------------------------------------------- front end 1: one chunk

struct PtrList {
    uint64_t p[R2_MAX_CHANNELS];
};

template <Mode M, bool HAS_OUT>
__global__ __launch_bounds__(kThreads) void reduce_copy_kernel(ChunkJob job, const PtrList in_stage,
                                                               const PtrList out_stage, int32_t *status)
{
    __shared__ ChannelTable tin, tout;
    run_chunk<M, HAS_OUT>(
        job, [&](unsigned c) { return in_stage.p[c]; }, [&](unsigned c) { return out_stage.p[c]; },
        status, tin, tout);
}

// ---------------------------------------------------------------- front end 2: a ring step

struct StepArgs {
    uint64_t rank_buf[R2_MAX_RANKS];
    const uint64_t *tables;  // [S*T_slab][C+1]
    uint64_t stage;          // [2][R][S][C][cap]
    uint64_t chunk_bytes, cap;
    uint32_t R, S, C;
    uint32_t step;         // fused step j
    uint32_t T_slab;       // transmissions per slab
    uint32_t chunk_start;  // 1 when the run is an all-gather alone, else 0
};

// blockIdx.y = rank * S + slab, blockIdx.x = workgroup within that chunk.
template <Mode M, bool HAS_OUT>
__global__ __launch_bounds__(kThreads) void ring_step_kernel(const StepArgs a)
{
    __shared__ ChannelTable tin, tout;
    const uint32_t r = blockIdx.y / a.S, l = blockIdx.y - r * a.S;
    const uint32_t j = a.step;
    const uint32_t chunk = (r + a.chunk_start + 2 * a.R - j) % a.R;  // j <= 2R-2
    const uint32_t peer = (r + a.R - 1) % a.R;
    const uint64_t row = (uint64_t)a.C + 1;
    const uint64_t t_out = (uint64_t)l * a.T_slab + j;

    ChunkJob job;
    job.local = reinterpret_cast<uint8_t *>(a.rank_buf[r]) + ((uint64_t)l * a.R + chunk) * a.chunk_bytes;
    job.bytes = a.chunk_bytes;
    job.in_off = M != kSend ? a.tables + (t_out - 1) * row : nullptr;
    job.out_off = HAS_OUT ? a.tables + t_out * row : nullptr;
    job.cap = a.cap;
    job.C = a.C;
    // stage buffer of (parity, rank, slab, channel)
    const uint64_t in_base = a.stage + ((((uint64_t)((j + 1) & 1) * a.R + peer) * a.S + l) * a.C) * a.cap;
    const uint64_t out_base = a.stage + ((((uint64_t)(j & 1) * a.R + r) * a.S + l) * a.C) * a.cap;
    run_chunk<M, HAS_OUT>(
        job, [&](unsigned c) { return in_base + c * a.cap; },
        [&](unsigned c) { return out_base + c * a.cap; }, nullptr, tin, tout);
}

// ---------------------------------------------------------------- host side

unsigned blocks_for(uint64_t bytes, uint64_t n_chunks)
{
    const uint64_t tile_bytes = (uint64_t)kThreads * kUnroll * 16;
    uint64_t want = (bytes + tile_bytes - 1) / tile_bytes;
    if (want == 0) want = 1;
    uint64_t limit = ((uint64_t)kComputeUnits * kBlocksPerCU + n_chunks - 1) / n_chunks;
    if (limit == 0) limit = 1;
    return (unsigned)(want < limit ? want : limit);
}

bool valid_dtype(int d) { return d == R2_F32 || d == R2_BF16; }
uint64_t elem_bytes(int d) { return d == R2_F32 ? 4 : 2; }

Mode mode_of(bool has_in, int op, int dtype)
{
    if (!has_in) return kSend;
    if (op == R2_OP_COPY) return kCopy;
    return dtype == R2_F32 ? kSumF32 : kSumBF16;
}

struct SimShape {
    uint32_t R, S, C, J, T_slab;
    uint64_t chunk_bytes, cap, n_tx;
    uint64_t tables_bytes, stage_off, total_bytes;
};

uint64_t round_up(uint64_t x, uint64_t m) { return (x + m - 1) / m * m; }

// Validates a descriptor and derives the sizes; returns an R2 code.
int shape_of(const r2_sim_desc *d, SimShape &s)
{
    if (!d) return R2_ERR_INVALID;
    if (d->n_ranks < 2 || d->n_ranks > R2_MAX_RANKS) return R2_ERR_INVALID;
    if (d->n_channels == 0 || d->n_channels > R2_MAX_CHANNELS) return R2_ERR_INVALID;
    if (d->n_slabs == 0 || (uint64_t)d->n_slabs * d->n_ranks > 65535) return R2_ERR_INVALID;
    if (d->align == 0 || d->align % 16 != 0) return R2_ERR_INVALID;
    if (!valid_dtype(d->dtype)) return R2_ERR_INVALID;
    if (d->phases != R2_PHASE_RS && d->phases != R2_PHASE_AG && d->phases != (R2_PHASE_RS | R2_PHASE_AG))
        return R2_ERR_INVALID;
    const uint64_t per = (uint64_t)d->n_slabs * d->n_ranks;
    if (d->n_elems % per != 0) return R2_ERR_INVALID;
    if (d->n_elems > (1ull << 60)) return R2_ERR_OVERFLOW;
    s.R = d->n_ranks;
    s.S = d->n_slabs;
    s.C = d->n_channels;
    s.J = d->phases == (R2_PHASE_RS | R2_PHASE_AG) ? 2 * s.R - 1 : s.R;
    s.T_slab = s.J - 1;
    s.chunk_bytes = d->n_elems / per * elem_bytes(d->dtype);
    s.cap = round_up(s.chunk_bytes ? s.chunk_bytes : 1, 256);
    s.n_tx = (uint64_t)s.S * s.T_slab;
    s.tables_bytes = round_up(s.n_tx * (s.C + 1) * 8, 256);
    s.stage_off = s.tables_bytes;
    const unsigned __int128 stage = (unsigned __int128)2 * s.R * s.S * s.C * s.cap;
    if (stage > ((unsigned __int128)1 << 62)) return R2_ERR_OVERFLOW;
    s.total_bytes = s.stage_off + (uint64_t)stage;
    return R2_OK;
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

int check_workspace(const void *ws, uint64_t ws_bytes, const SimShape &s)
{
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return R2_ERR_INVALID;
    if (ws_bytes < s.total_bytes) return R2_ERR_CAPACITY;
    return R2_OK;
}

template <Mode M, bool HAS_OUT>
void launch_step(const StepArgs &a, dim3 grid, hipStream_t st)
{
    hipLaunchKernelGGL((ring_step_kernel<M, HAS_OUT>), grid, dim3(kThreads), 0, st, a);
}

template <Mode M, bool HAS_OUT>
void launch_single(const ChunkJob &job, const PtrList &in, const PtrList &out, int32_t *status,
                   unsigned blocks, hipStream_t st)
{
    hipLaunchKernelGGL((reduce_copy_kernel<M, HAS_OUT>), dim3(blocks), dim3(kThreads), 0, st, job, in,
                       out, status);
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
    if (!valid_dtype(dtype) || (op != R2_OP_SUM && op != R2_OP_COPY)) return R2_ERR_INVALID;
    if (n_channels == 0 || n_channels > R2_MAX_CHANNELS) return R2_ERR_INVALID;
    if (!in_stage && !out_stage) return R2_ERR_INVALID;
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
    ChunkJob job{static_cast<uint8_t *>(local), bytes, in_offsets, out_offsets, stage_capacity, n_channels};
    const unsigned blocks = blocks_for(bytes, 1);
    hipStream_t st = (hipStream_t)stream;
    const Mode m = mode_of(in_stage != nullptr, op, dtype);
    const bool has_out = out_stage != nullptr;
    switch (m) {
    case kSend: launch_single<kSend, true>(job, in, out, status, blocks, st); break;
    case kSumF32:
        if (has_out) launch_single<kSumF32, true>(job, in, out, status, blocks, st);
        else launch_single<kSumF32, false>(job, in, out, status, blocks, st);
        break;
    case kSumBF16:
        if (has_out) launch_single<kSumBF16, true>(job, in, out, status, blocks, st);
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
    if ((rc = check_epochs(epochs, n_epochs, s))) return rc;
    if ((rc = check_workspace(workspace, workspace_bytes, s))) return rc;
    if (s.n_tx == 0) return R2_OK;
    return launch_partition_epochs(epochs, n_epochs, s.C, desc->align, s.chunk_bytes, s.n_tx,
                                   static_cast<uint64_t *>(workspace), offsets_log, (hipStream_t)stream);
}

extern "C" int r2_sim_step(const r2_sim_desc *desc, void *const *rank_bufs, uint32_t step,
                           void *workspace, uint64_t workspace_bytes, void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (!rank_bufs || step >= s.J) return R2_ERR_INVALID;
    if ((rc = check_workspace(workspace, workspace_bytes, s))) return rc;
    StepArgs a{};
    for (uint32_t r = 0; r < s.R; ++r) {
        a.rank_buf[r] = reinterpret_cast<uint64_t>(rank_bufs[r]);
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
    a.chunk_start = desc->phases == R2_PHASE_AG ? 1 : 0;

    const bool has_in = step > 0, has_out = step < s.J - 1;
    int op;
    if (desc->phases == R2_PHASE_AG) op = R2_OP_COPY;
    else if (desc->phases == R2_PHASE_RS) op = R2_OP_SUM;
    else op = step <= s.R - 1 ? R2_OP_SUM : R2_OP_COPY;
    const Mode m = mode_of(has_in, op, desc->dtype);

    const uint64_t n_chunks = (uint64_t)s.R * s.S;
    const dim3 grid(blocks_for(s.chunk_bytes, n_chunks), (unsigned)n_chunks);
    hipStream_t st = (hipStream_t)stream;
    switch (m) {
    case kSend: launch_step<kSend, true>(a, grid, st); break;
    case kSumF32:
        if (has_out) launch_step<kSumF32, true>(a, grid, st); else launch_step<kSumF32, false>(a, grid, st);
        break;
    case kSumBF16:
        if (has_out) launch_step<kSumBF16, true>(a, grid, st); else launch_step<kSumBF16, false>(a, grid, st);
        break;
    case kCopy:
        if (has_out) launch_step<kCopy, true>(a, grid, st); else launch_step<kCopy, false>(a, grid, st);
        break;
    }
    return hip_rc(hipGetLastError());
}

extern "C" int r2_ring_allreduce_sim(const r2_sim_desc *desc, void *const *rank_bufs,
                                     const r2_epoch *epochs, uint32_t n_epochs, void *workspace,
                                     uint64_t workspace_bytes, uint64_t *offsets_log, void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (!rank_bufs) return R2_ERR_INVALID;
    for (uint32_t r = 0; r < s.R; ++r) {
        const uint64_t p = reinterpret_cast<uint64_t>(rank_bufs[r]);
        if (s.chunk_bytes && (!p || (p & 15u))) return R2_ERR_INVALID;
    }
    if ((rc = r2_sim_prepare(desc, epochs, n_epochs, workspace, workspace_bytes, offsets_log, stream)))
        return rc;
    for (uint32_t j = 0; j < s.J; ++j)
        if ((rc = r2_sim_step(desc, rank_bufs, j, workspace, workspace_bytes, stream))) return rc;
    return R2_OK;
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

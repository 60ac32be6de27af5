// Fused reduce-copy and the ring schedule built from it.
//
// R2CCL paper: Sec. 2.1 (a collective's data is cut over channels, each bound to a NIC, and GPU
// kernels execute the collective over them), Sec. 4.3 Technique II (per-NIC send staging buffers,
// chunk-granular progress), Sec. 5.2 (ring all-reduce = reduce-scatter, then all-gather).
//
// The data path is bandwidth-bound: per 16-byte vector two loads, one add, two stores.  Every lane
// moves whole 16-byte vectors; a wavefront touches 1 KiB of consecutive addresses per access.  The
// slice that holds a tile is found by a wavefront-wide comparison against the offsets table, which
// every wavefront holds in its lanes; only tiles that straddle a cut search an LDS copy per lane.
#include <type_traits>

#include "partition_device.h"

namespace r2 {
namespace {

// Launch shape and cache policy; the defaults are the measured best on MI355X.
#ifndef R2_THREADS
#define R2_THREADS 256
#endif
#ifndef R2_UNROLL
#define R2_UNROLL 2
#endif
#ifndef R2_NT_LOCAL_LOAD
#define R2_NT_LOCAL_LOAD 1
#endif
#ifndef R2_NT_LOCAL_STORE
#define R2_NT_LOCAL_STORE 1
#endif
#ifndef R2_NT_STAGE_LOAD
#define R2_NT_STAGE_LOAD 1
#endif
#ifndef R2_NT_STAGE_STORE
#define R2_NT_STAGE_STORE 0
#endif
constexpr unsigned kThreads = R2_THREADS;
constexpr unsigned kUnroll = R2_UNROLL;             // 16-byte vectors in flight per lane and stream

// A 16-byte vector as the compiler's native type, so that one access is one dwordx4 instruction.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Addresses are kept as integers; they all point into device (global) memory, and saying so gives
// global_load/global_store instead of the slower flat (generic address) instructions.
#define R2_GLOBAL __attribute__((address_space(1)))
#define R2_LDS __attribute__((address_space(3)))
template <typename T>
__device__ inline R2_GLOBAL T *gptr(uint64_t addr)
{
    return (R2_GLOBAL T *)addr;
}

// Every byte is touched once per launch: stream past the caches (non-temporal hint).
template <bool NT>
__device__ inline u32x4 load16(uint64_t addr)
{
    if constexpr (NT) return __builtin_nontemporal_load(gptr<const u32x4>(addr));
    else return *gptr<const u32x4>(addr);
}
template <bool NT>
__device__ inline void store16(uint64_t addr, u32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, gptr<u32x4>(addr));
    else *gptr<u32x4>(addr) = v;
}
constexpr bool kNtLocalLoad = R2_NT_LOCAL_LOAD, kNtLocalStore = R2_NT_LOCAL_STORE;
constexpr bool kNtStageLoad = R2_NT_STAGE_LOAD, kNtStageStore = R2_NT_STAGE_STORE;

enum Mode : int { kSend = 0, kSumF32 = 1, kSumBF16 = 2, kCopy = 3 };

// ---------------------------------------------------------------- arithmetic on 16-byte vectors

__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Two bf16 sums at once: widen (exact), add in fp32, narrow with round-to-nearest-even.  The
// narrowing is the hardware's packed convert (v_cvt_pk_bf16_f32 on gfx950).
__device__ inline uint32_t add_bf16x2(uint32_t a, uint32_t b)
{
    f32x2 s;
    s.x = bf16_lo(a) + bf16_lo(b);
    s.y = bf16_hi(a) + bf16_hi(b);
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(s, bf16x2));
}

__device__ inline uint16_t add_bf16(uint16_t a, uint16_t b)
{
    const float s = bf16_lo(a) + bf16_lo(b);
    return __builtin_bit_cast(uint16_t, (__bf16)s);
}

template <Mode M>
__device__ inline u32x4 combine(const u32x4 &incoming, const u32x4 &local)
{
    if constexpr (M == kSumF32) {
        u32x4 v;
        v.x = __float_as_uint(__uint_as_float(incoming.x) + __uint_as_float(local.x));
        v.y = __float_as_uint(__uint_as_float(incoming.y) + __uint_as_float(local.y));
        v.z = __float_as_uint(__uint_as_float(incoming.z) + __uint_as_float(local.z));
        v.w = __float_as_uint(__uint_as_float(incoming.w) + __uint_as_float(local.w));
        return v;
    } else if constexpr (M == kSumBF16) {
        u32x4 v;
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

// The slice that holds chunk byte b0, remembered from tile to tile: a workgroup walks the chunk
// front to back and slices are long, so the table is searched only when a cut is crossed.
struct Span {
    uint64_t lo = 0, hi = 0, delta = 0;
};

// One table as every wavefront holds it: lane c has slice c's bounds (lanes from C on hold nothing),
// and whether the table is acceptable.  Read straight from memory by each wavefront for itself -- a
// few cached loads -- so that the common path needs neither LDS nor a workgroup barrier.
struct LaneRow {
    uint64_t off = 0, next = 0;
    int bad = 0;  // 0 or an R2_ERR code
};
__device__ inline LaneRow load_row(const uint64_t *__restrict__ g_off, uint32_t C, uint64_t bytes, uint64_t cap)
{
    const unsigned c = threadIdx.x % kWave;
    LaneRow r;
    if (c < C) {
        r.off = g_off[c];
        r.next = g_off[c + 1];
        if (c == 0 && r.off != 0) r.bad = R2_ERR_INVALID;
        if (c == C - 1 && r.next != bytes) r.bad = R2_ERR_INVALID;
        if (r.next < r.off) r.bad = R2_ERR_INVALID;
        else if (r.next - r.off > cap) r.bad = R2_ERR_CAPACITY;
        if (r.next != r.off && (r.off & 15u)) r.bad = R2_ERR_INVALID;  // a non-empty slice starts on 16 B
    }
    return r;
}
__device__ inline uint64_t lane_value(uint64_t x, uint32_t lane)  // x of a wave-uniform lane
{
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)x, lane);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(x >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}
// The slice that holds byte b0 (wave-uniform, below the chunk's size): one lane's bounds contain it.
template <typename Ptr>
__device__ inline void locate(const LaneRow &r, uint32_t C, uint64_t b0, Span &s, Ptr base_of)
{
    if (b0 < s.lo || b0 >= s.hi) {
        const unsigned lane = threadIdx.x % kWave;
        const uint64_t holds = __ballot(lane < C && r.off <= b0 && b0 < r.next);
        const uint32_t c = __builtin_amdgcn_readfirstlane((uint32_t)__builtin_ctzll(holds));
        s.lo = lane_value(r.off, c);
        s.hi = lane_value(r.next, c);
        s.delta = base_of(c) - s.lo;
    }
}

// ---------------------------------------------------------------- the chunk worker

struct ChunkJob {
    uint8_t *local;
    uint64_t bytes;           // the whole chunk: what the tables partition
    uint64_t lo, hi;          // the part of it this launch moves; lo is a multiple of 16, and so
                              // is hi unless hi == bytes
    const uint64_t *in_off;   // device table or null
    const uint64_t *out_off;  // device table or null
    uint64_t cap;
    uint32_t C;
};

// FWD (sums only): the outgoing stage gets the incoming data unchanged instead of the sum.
// NT_OUT: the outgoing stage is written with non-temporal stores (a chunk too large for the next
// reader to find it in cache).
// KEEP (sums only): the result goes to the outgoing stage only, the local chunk stays as it was.
template <Mode M, bool HAS_OUT, bool FWD = false, bool NT_OUT = kNtStageStore, bool KEEP = false, typename InPtr,
          typename OutPtr>
__device__ inline void run_chunk(const ChunkJob &job, InPtr in_ptr, OutPtr out_ptr, int32_t *status,
                                 ChannelTable &tin, ChannelTable &tout)
{
    constexpr bool HAS_IN = M != kSend;
    constexpr bool NEED_LOCAL = M != kCopy;
    constexpr bool PUT_LOCAL = HAS_IN && !KEEP;
    static_assert(!KEEP || ((M == kSumF32 || M == kSumBF16) && HAS_OUT && !FWD), "KEEP is a sum that is only sent on");
    const uint32_t C = job.C;

    // Every wavefront reads the tables for itself and checks them; the verdict is the same in every
    // wavefront of every workgroup, so a bad table moves nothing anywhere.
    LaneRow rin, rout;
    int bad = 0;
    if constexpr (HAS_IN) {
        rin = load_row(job.in_off, C, job.bytes, job.cap);
        bad = rin.bad;
    }
    if constexpr (HAS_OUT) {
        rout = load_row(job.out_off, C, job.bytes, job.cap);
        if (!bad) bad = rout.bad;
    }
    if (__any(bad)) {
        if (bad && status) atomicMin(status, bad);
        return;
    }
    // The rare paths (a tile that straddles a cut, a ragged tail, an unaligned chunk) look channels up
    // per lane in an LDS copy of the tables, made when first needed; whether it is needed is the same
    // for all threads of the workgroup, so the barrier inside is reached by all or none.
    bool tables_in_lds = false;
    auto tables_to_lds = [&]() {
        if (tables_in_lds) return;
        const unsigned c = threadIdx.x;
        if (c < C) {
            if constexpr (HAS_IN) {
                tin.off[c] = rin.off;
                tin.delta[c] = in_ptr(c) - rin.off;
                if (c == C - 1) tin.off[C] = rin.next;
            }
            if constexpr (HAS_OUT) {
                tout.off[c] = rout.off;
                tout.delta[c] = out_ptr(c) - rout.off;
                if (c == C - 1) tout.off[C] = rout.next;
            }
        }
        __syncthreads();
        tables_in_lds = true;
    };

    uint8_t *const local = job.local;
    const bool aligned = (reinterpret_cast<uintptr_t>(local) & 15u) == 0;
    const uint64_t vbegin = job.lo / 16;
    const uint64_t nvec = aligned ? job.hi / 16 : vbegin;  // vectors [vbegin, nvec)

    // Whole 16-byte vectors, a tile of kThreads*kUnroll consecutive vectors per iteration.  If one
    // slice holds the whole tile (nearly always) its address delta is wave-uniform; a tile that
    // straddles a cut lets every lane look its own vector up.
    const uint64_t local_addr = reinterpret_cast<uint64_t>(local);
    const uint64_t tile = (uint64_t)kThreads * kUnroll;
    Span sin, sout;
    for (uint64_t v0 = vbegin + (uint64_t)blockIdx.x * tile; v0 < nvec; v0 += (uint64_t)gridDim.x * tile) {
        const uint64_t b0 = v0 * 16;
        const uint64_t b1 = (v0 + tile < nvec ? v0 + tile : nvec) * 16;
        bool in_one = true, out_one = true;
        if constexpr (HAS_IN) {
            locate(rin, C, b0, sin, in_ptr);
            in_one = b1 <= sin.hi;
        }
        if constexpr (HAS_OUT) {
            locate(rout, C, b0, sout, out_ptr);
            out_one = b1 <= sout.hi;
        }
        u32x4 inc[kUnroll], loc[kUnroll];
        if (v0 + tile <= nvec && in_one && out_one) {
            // Full tile inside one slice of either table: straight-line code, all loads of the
            // tile in flight together.
            const uint64_t b = (v0 + threadIdx.x) * 16;
#pragma unroll
            for (unsigned u = 0; u < kUnroll; ++u) {
                if constexpr (HAS_IN) inc[u] = load16<kNtStageLoad>(sin.delta + b + u * (kThreads * 16));
                if constexpr (NEED_LOCAL) loc[u] = load16<kNtLocalLoad>(local_addr + b + u * (kThreads * 16));
            }
#pragma unroll
            for (unsigned u = 0; u < kUnroll; ++u) {
                const u32x4 r = combine<M>(inc[u], loc[u]);
                if constexpr (PUT_LOCAL) store16<kNtLocalStore>(local_addr + b + u * (kThreads * 16), r);
                if constexpr (HAS_OUT) store16<NT_OUT>(sout.delta + b + u * (kThreads * 16), FWD ? inc[u] : r);
            }
            continue;
        }
        // The chunk's last, partial tile, or a tile that straddles a cut: every lane checks its
        // bounds and, where needed, looks its channel up.
        if (!in_one || !out_one) tables_to_lds();
#pragma unroll
        for (unsigned u = 0; u < kUnroll; ++u) {
            const uint64_t v = v0 + u * kThreads + threadIdx.x;
            if (v < nvec) {
                const uint64_t b = v * 16;
                if constexpr (HAS_IN) {
                    const uint64_t d = in_one ? sin.delta : tin.delta[find_channel(tin.off, C, b)];
                    inc[u] = load16<kNtStageLoad>(d + b);
                }
                if constexpr (NEED_LOCAL) loc[u] = load16<kNtLocalLoad>(local_addr + b);
            }
        }
#pragma unroll
        for (unsigned u = 0; u < kUnroll; ++u) {
            const uint64_t v = v0 + u * kThreads + threadIdx.x;
            if (v < nvec) {
                const uint64_t b = v * 16;
                const u32x4 r = combine<M>(inc[u], loc[u]);
                if constexpr (PUT_LOCAL) store16<kNtLocalStore>(local_addr + b, r);
                if constexpr (HAS_OUT) {
                    const uint64_t d = out_one ? sout.delta : tout.delta[find_channel(tout.off, C, b)];
                    store16<NT_OUT>(d + b, FWD ? inc[u] : r);
                }
            }
        }
    }

    // What the vectors did not cover, one element at a time: the last bytes % 16 of an aligned
    // chunk, or everything if the chunk's address is only element-aligned.
    using Elem = typename std::conditional<M == kSumF32, uint32_t, uint16_t>::type;
    const uint64_t first = nvec * 16;
    const uint64_t n_el = (job.hi - first) / sizeof(Elem);
    if (n_el) tables_to_lds();
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < n_el;
         i += (uint64_t)gridDim.x * kThreads) {
        const uint64_t b = first + i * sizeof(Elem);
        Elem x_in = 0, x_loc = 0;
        if constexpr (HAS_IN) {
            const uint32_t c = find_channel(tin.off, C, b);
            x_in = *gptr<const Elem>(tin.delta[c] + b);
        }
        if constexpr (NEED_LOCAL) x_loc = *gptr<const Elem>(local_addr + b);
        Elem r;
        if constexpr (M == kSumF32) r = __float_as_uint(__uint_as_float(x_in) + __uint_as_float(x_loc));
        else if constexpr (M == kSumBF16) r = add_bf16(x_in, x_loc);
        else if constexpr (M == kCopy) r = x_in;
        else r = x_loc;
        if constexpr (PUT_LOCAL) *gptr<Elem>(local_addr + b) = r;
        if constexpr (HAS_OUT) {
            const uint32_t c = find_channel(tout.off, C, b);
            *gptr<Elem>(tout.delta[c] + b) = FWD ? x_in : r;
        }
    }
}

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
    uint32_t link_tables;  // 1: row r of `tables` is the link r -> r+1, for every transmission of rank r
    uint32_t slab_begin, slab_count;  // the slabs this launch covers
    uint64_t lo, hi;                  // and the byte range of every ring chunk it moves
};

// blockIdx.y = (rank - rank_base) * slab_count + (slab - slab_begin), blockIdx.x = workgroup within
// the range.
template <Mode M, bool HAS_OUT, bool KEEP = false>
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
    job.in_off = M != kSend ? a.tables + (a.link_tables ? peer : t_out - 1) * row : nullptr;
    job.out_off = HAS_OUT ? a.tables + (a.link_tables ? r : t_out) * row : nullptr;
    job.cap = a.cap;
    job.C = a.C;
    // stage buffer of (parity, rank, slab, channel)
    const uint64_t in_base = a.stage + ((((uint64_t)((j + 1) & 1) * a.R + peer) * a.S + l) * a.C) * a.cap;
    const uint64_t out_base = a.stage + ((((uint64_t)(j & 1) * a.R + r) * a.S + l) * a.C) * a.cap;
    run_chunk<M, HAS_OUT, false, kNtStageStore, KEEP>(
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

// ---------------------------------------------------------------- front end 3: fused columns
//
// Element position b of a ring chunk travels round the ring on its own: what step j of rank r does
// at b depends only on what step j-1 of rank r-1 did at b.  A "column" is a byte range of the ring
// chunks of one slab, taken through several consecutive steps of ALL ranks by one workgroup: wave w
// plays rank w (w + 16, ... if there are more ranks than waves), a workgroup barrier separates the
// steps, and the stage round trip between two steps stays in that compute unit's L2.  One launch
// then replaces one launch per step.  It is only valid while the channel state of every slab stays
// the same over the steps of the launch: then a stage location belongs to one column, and columns
// may drift apart in time without overwriting each other's unread data (see plan_schedule).

// A column is 1 or 2 vectors per lane wide (1 or 2 KiB; template parameter U).  All ranks of a column
// share one compute unit, so its steps are bound by that unit's instruction issue as much as by the
// hand-off: while the narrow columns of a run do not fill the GPU they are the faster ones (half the
// work per step and unit, twice the units busy); wide columns halve the per-column overhead once they do.
constexpr unsigned kNarrowColBytes = kWave * 16;
#ifndef R2_WIDE_FROM
#define R2_WIDE_FROM 256
#endif
constexpr uint64_t kWideColumnsFrom = R2_WIDE_FROM;  // wide columns from this many of them on (one per compute unit)
constexpr unsigned kMaxFusedWaves = 16;

struct ColInfo {  // the slice of one transmission's table that holds the column's first byte
    uint64_t lo, hi;
    uint32_t c, pad;
};

struct FusedArgs {
    uint64_t rank_buf[R2_MAX_RANKS];
    const uint64_t *tables;  // [S*T_slab][C+1]
    uint64_t stage;          // [2][R][S][C][cap]
    uint64_t chunk_bytes, cap;
    uint64_t cols_per_chunk;
    uint32_t R, S, C, J, T_slab;
    uint32_t chunk_start;  // 1 when the run is an all-gather alone, else 0
    uint32_t sum_last;     // last fused step that adds (R-1 in an all-reduce); 0 = none
    uint32_t j0, j1;       // the steps of this launch: [j0, j1)
    uint32_t rows_in_lds;  // the table rows of the launch fit the dynamic LDS block
    uint32_t align;        // partition alignment (only used when the kernel partitions itself)
    uint64_t *tables_out;  // where the first column of each slab records the rows it computed
    uint64_t *log_out;     // ... and the caller's log, or null
};

constexpr uint32_t kFusedLdsRowBytes = 48 * 1024;  // at most this much LDS for table rows

// One wave's share of one step on a full-width column, with every choice fixed at compile time so
// that the code is straight-line: all loads of the step are issued before the first use, and
// nothing waits for the stores.  KIND: 0 copy-send, 1 sum, 2 copy.  The caller supplies, per vector
// of the lane, the addresses in the incoming stage, the outgoing stage and the local buffer.
template <unsigned U, int KIND, bool HAS_OUT, bool BF16>
__device__ inline void column_step(const uint64_t (&ain)[U], const uint64_t (&aout)[U],
                                   const uint64_t (&aloc)[U])
{
    constexpr bool HAS_IN = KIND != 0, READS_LOCAL = KIND != 2;
    u32x4 inc[U], loc[U];
#pragma unroll
    for (unsigned u = 0; u < U; ++u) {
        if constexpr (HAS_IN) inc[u] = load16<false>(ain[u]);
        if constexpr (READS_LOCAL) loc[u] = load16<kNtLocalLoad>(aloc[u]);
    }
#pragma unroll
    for (unsigned u = 0; u < U; ++u) {
        u32x4 v;
        if constexpr (KIND == 0) v = loc[u];
        else if constexpr (KIND == 2) v = inc[u];
        else v = combine<BF16 ? kSumBF16 : kSumF32>(inc[u], loc[u]);
        if constexpr (HAS_IN) store16<kNtLocalStore>(aloc[u], v);
        if constexpr (HAS_OUT) store16<false>(aout[u], v);
    }
}

// find_channel without a data-dependent branch (every lane runs the same number of rounds, and the
// lookups of independent vectors interleave): the last c < C with off[c] <= b.  Since off never
// decreases, that is the slice with off[c+1] > b.  top = the largest power of two below C (0 if C=1).
template <typename RowPtr>
__device__ inline uint32_t find_channel_flat(RowPtr off, uint32_t C, uint32_t top, uint64_t b)
{
    uint32_t c = 0;
    for (uint32_t s = top; s; s >>= 1) {
        const uint32_t m = c + s;
        const uint32_t mm = m < C ? m : C - 1;
        c = (m < C && off[mm] <= b) ? m : c;
    }
    return c;
}

#ifdef R2_FUSED_TIMING
__device__ uint64_t g_dbg[256];
#define R2_STAMP(i) do { if (blockIdx.x == 0 && threadIdx.x == 0) g_dbg[i] = wall_clock64(); } while (0)
#else
#define R2_STAMP(i) do {} while (0)
#endif

// PARTITION: the kernel computes the table rows it needs itself, from the channel states in `eb`
// (every workgroup for its own use, in LDS; the first column of each slab also records them in
// the workspace and the log), so that no partition launch has to run in front of it.
template <bool BF16, bool PARTITION, unsigned U>
__device__ inline void fused_body(const FusedArgs &a, const EpochBatch *eb)
{
    R2_STAMP(0);
    __shared__ ColInfo info[2 * R2_MAX_RANKS];  // by transmission within the slab
    const uint32_t l = (uint32_t)(blockIdx.x / a.cols_per_chunk);
    const uint64_t k = blockIdx.x - (uint64_t)l * a.cols_per_chunk;
    const uint64_t b0 = k * (kWave * 16 * U);
    const uint64_t b1 = b0 + (kWave * 16 * U) < a.chunk_bytes ? b0 + (kWave * 16 * U) : a.chunk_bytes;
    const uint32_t C = a.C;
    const uint64_t row = (uint64_t)C + 1;
    const uint64_t *slab_tables = a.tables + (uint64_t)l * a.T_slab * row;

    // The table rows of the transmissions this launch reads or writes, [t_first, t_end), are copied
    // to LDS when they fit: a column that straddles a cut looks its vectors up there every step.
    extern __shared__ uint64_t s_rows[];
    const uint32_t t_first = a.j0 ? a.j0 - 1 : 0;
    const uint32_t t_end = a.j1 < a.T_slab ? a.j1 : a.T_slab;
    const uint64_t *rows = slab_tables;  // rows + t * row = table of transmission t
    // The wave index is made visibly wave-uniform: everything indexed by rank (the kernel-argument
    // array of rank buffers above all) then goes through scalar loads and the scalar cache instead
    // of a vector load from the argument block, which measured about 2 us per step.
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t lane = threadIdx.x % kWave, n_waves = blockDim.x / kWave;
    const bool one_rank = a.R <= n_waves;                       // a wave plays one rank
    const bool ragged_width = b0 + (kWave * 16 * U) > a.chunk_bytes;  // the chunk's last, narrower column

    // What a wave that plays one rank needs per step depends on the launch arguments only, so it is
    // worked out here, ahead of the prologue's barriers: the slab of its buffer, its own stage and its
    // predecessor's (parity 0; parity 1 is R ranks further), and the ring chunk it starts at, which
    // goes one down per step.  (With more ranks than waves these describe the wave's first rank and
    // are not used.)
    const uint64_t per_rank = (uint64_t)a.S * C * a.cap;  // stage bytes of one (parity, rank)
    const uint64_t slab_stage = a.stage + (uint64_t)l * C * a.cap;
    const uint32_t my_rank = wave < a.R ? wave : 0;
    const uint32_t my_peer = (my_rank + a.R - 1) % a.R;
    const uint64_t my_slab = a.rank_buf[my_rank] + (uint64_t)l * a.R * a.chunk_bytes;
    const uint64_t my_in0 = slab_stage + (uint64_t)my_peer * per_rank;
    const uint64_t my_out0 = slab_stage + (uint64_t)my_rank * per_rank;
    const uint64_t parity_stride = (uint64_t)a.R * per_rank;
    const uint32_t my_chunk = (my_rank + a.chunk_start + 2 * a.R - a.j0) % a.R;

    // A launch that starts at step 0 begins with every rank staging a chunk of its own buffer.
    // Where that chunk lies depends on nothing computed below, so its loads are issued first and
    // their latency passes while the tables are made.
    const bool preload = a.j0 == 0 && one_rank && !ragged_width;
    u32x4 pre[U] = {};
    if (preload) {
        const uint64_t src = my_slab + (uint64_t)my_chunk * a.chunk_bytes + b0;  // j0 = 0: my_chunk is step 0's
#pragma unroll
        for (unsigned u = 0; u < U; ++u) pre[u] = load16<kNtLocalLoad>(src + (uint64_t)(u * kWave + lane) * 16);
    }

    // changed[t]: the table of transmission t may differ from that of t-1.  Tables mostly repeat,
    // and then the stage offsets of a step can be carried over.
    __shared__ uint32_t changed[2 * R2_MAX_RANKS];
    const R2_LDS uint64_t *lds_rows = (const R2_LDS uint64_t *)s_rows;
    bool slow;
    if constexpr (PARTITION) {  // always with the rows in LDS
        // One wave per channel state in force within [t_first, t_end): it cuts the chunk once, into
        // the row of the first transmission the state governs here.  Then one thread per
        // transmission copies its state's row and notes the slice that holds the column.
        const uint64_t tg0 = (uint64_t)l * a.T_slab;  // transmission index (of the whole run) of the slab's first
        const uint32_t e_lo = epoch_at(*eb, tg0 + t_first), e_hi = epoch_at(*eb, tg0 + t_end - 1);
        auto first_tx = [&](uint32_t e) { return e == e_lo ? t_first : (uint32_t)(eb->t_start[e] - tg0); };
        for (uint32_t ev = e_lo + wave; ev <= e_hi; ev += n_waves) {
            const uint32_t e = __builtin_amdgcn_readfirstlane(ev);
            const uint32_t weight = lane < C ? eb->weights[e * C + lane] : 0;
            uint64_t W;
            const uint64_t o = partition_lane(weight, (eb->fail_mask[e] >> lane) & 1u, C, a.chunk_bytes, a.align, &W);
            uint64_t *lds_row = s_rows + (uint64_t)(first_tx(e) - t_first) * row;
            if (lane < C) lds_row[lane] = o;
            if (lane == 0) lds_row[C] = a.chunk_bytes;
        }
        __syncthreads();
        // A group of 16, 32 or 64 lanes (enough for a row) per transmission, lane c of the group for
        // entry c of the row: with few channels one round serves every transmission of the launch.
        const uint32_t width = row <= 16 ? 16 : row <= 32 ? 32 : kWave;
        const uint32_t per = kWave / width, c = lane % width;
        for (uint32_t t = t_first + wave * per + lane / width; t < t_end; t += n_waves * per) {
            uint32_t ts = t_first;  // the first transmission (here) of the state in force at t
            for (uint32_t k = e_lo + 1; k <= e_hi; ++k) {
                const uint64_t begins = eb->t_start[k];
                if (begins <= tg0 + t) ts = (uint32_t)(begins - tg0);
            }
            const R2_LDS uint64_t *src = lds_rows + (uint64_t)(ts - t_first) * row;
            const uint64_t lo = c < C ? src[c] : 0, hi = c < C ? src[c + 1] : 0;
            if (t != ts) {  // C may be the whole wavefront: lane 0 also writes the row's last entry
                if (c < C) s_rows[(uint64_t)(t - t_first) * row + c] = lo;
                if (c == 0) s_rows[(uint64_t)(t - t_first) * row + C] = a.chunk_bytes;
            }
            if (c < C && lo <= b0 && b0 < hi) {  // the one slice that holds the column's first byte
                info[t].lo = lo;
                info[t].hi = hi;
                info[t].c = c;
            }
            if (c == 0) changed[t] = t == ts;  // the first transmission of a state, or of this launch
        }
        __syncthreads();
        R2_STAMP(1);
        rows = s_rows - (uint64_t)t_first * row;
        slow = ragged_width;
    } else {
        if (a.rows_in_lds) {
            const uint32_t n = (t_end - t_first) * (uint32_t)row;
            for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) s_rows[i] = slab_tables[(uint64_t)t_first * row + i];
            __syncthreads();
            rows = s_rows - (uint64_t)t_first * row;
        }
        // Which slice holds the column's first byte, for every such transmission.
        for (uint32_t t = t_first + threadIdx.x; t < t_end; t += blockDim.x) {
            const uint64_t *off = rows + t * row;
            const uint32_t c = find_channel(off, C, b0);
            info[t].lo = off[c];
            info[t].hi = off[c + 1];
            info[t].c = c;
        }
        __syncthreads();
        R2_STAMP(1);
        // (lane c compares entry c of the two rows)
        for (uint32_t t = t_first + wave; t < t_end; t += n_waves) {
            bool eq = false;
            if (a.rows_in_lds && t > t_first) {
                eq = true;
                if (lane < C)
                    eq = lds_rows[(uint64_t)(t - t_first) * row + lane] == lds_rows[(uint64_t)(t - 1 - t_first) * row + lane];
                eq = __all(eq);
            }
            if (lane == 0) changed[t] = !eq;
        }
        // Straddling columns need the rows in LDS for the fast loop; otherwise they take the slow one.
        int straddles = 0;
        if (!a.rows_in_lds)
            for (uint32_t t = t_first + threadIdx.x; t < t_end; t += blockDim.x)
                if (b1 > info[t].hi) straddles = 1;
        slow = ragged_width || __syncthreads_or(straddles);
    }
    // The first column of a slab records the rows it computed for the caller: last of all, so that
    // no step waits for these stores.
    auto record_rows = [&]() {
        if (!PARTITION || k != 0) return;
        const uint32_t n = (t_end - t_first) * (uint32_t)row;
        const uint64_t at = ((uint64_t)l * a.T_slab + t_first) * row;
        for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) {
            const uint64_t v = lds_rows[i];
            a.tables_out[at + i] = v;
            if (a.log_out) a.log_out[at + i] = v;
        }
    };
    auto local_of = [&](uint32_t r, uint32_t j) {
        const uint32_t chunk = (r + a.chunk_start + 2 * a.R - j) % a.R;
        return a.rank_buf[r] + ((uint64_t)l * a.R + chunk) * a.chunk_bytes;
    };

    if (!slow) {
        // Full-width column: straight-line steps and barriers only.  Where the column lies inside
        // one slice of a table its stage delta is uniform; where it straddles a cut every lane
        // looks its vectors up in the (LDS) row, without branching.
        uint32_t top = 0;
        while ((top ? top * 2 : 1) < C) top = top ? top * 2 : 1;
        uint64_t bu[U];
#pragma unroll
        for (unsigned u = 0; u < U; ++u) bu[u] = b0 + (uint64_t)(u * kWave + lane) * 16;

        // Stage offset (within one rank's stage of one parity) of each of the lane's vectors under
        // the table of transmission t.
        auto deltas_for = [&](uint32_t t, uint64_t(&d)[U]) {
            if (b1 <= info[t].hi) {
                const uint64_t base = (uint64_t)info[t].c * a.cap - info[t].lo;
#pragma unroll
                for (unsigned u = 0; u < U; ++u) d[u] = base + bu[u];
            } else {  // only reached with the rows in LDS
                const R2_LDS uint64_t *off = lds_rows + (uint64_t)(t - t_first) * row;
#pragma unroll
                for (unsigned u = 0; u < U; ++u) {
                    const uint32_t c = find_channel_flat(off, C, top, bu[u]);
                    d[u] = (uint64_t)c * a.cap - off[c] + bu[u];
                }
            }
        };
        // One rank's share of step j, given where its chunk and its stages are.
        auto rank_step = [&](bool has_in, bool has_out, bool summing, uint64_t local_addr,
                             uint64_t in_base, uint64_t out_base, const uint64_t(&din)[U],
                             const uint64_t(&dout)[U]) {
            uint64_t ain[U], aout[U], aloc[U];
#pragma unroll
            for (unsigned u = 0; u < U; ++u) {
                ain[u] = in_base + din[u];
                aout[u] = out_base + dout[u];
                aloc[u] = local_addr + bu[u];
            }
            if (!has_in) {
                column_step<U, 0, true, BF16>(ain, aout, aloc);
            } else if (summing) {
                if (has_out) column_step<U, 1, true, BF16>(ain, aout, aloc);
                else column_step<U, 1, false, BF16>(ain, aout, aloc);
            } else {
                if (has_out) column_step<U, 2, true, BF16>(ain, aout, aloc);
                else column_step<U, 2, false, BF16>(ain, aout, aloc);
            }
        };


        // The table a step reads with is the one the step before wrote with, and tables mostly
        // repeat from step to step, so the offsets are carried along and looked up only on change.
        uint64_t dcur[U];
        if (one_rank) {
            // A wave that plays one rank runs the steps as up to five stretches of one kind each --
            // copy-send, sums that stage onward, a last sum, copies that stage onward, a last copy --
            // so that the body of each stretch is a handful of loads and stores between two
            // barriers, with wave-uniform address updates and no per-step decisions beyond "did the
            // table change", which is one bit of a mask held in scalar registers.
            const uint32_t ti = t_first + lane;
            const uint64_t chg_lo = __ballot(ti < t_end && changed[ti] != 0);
            const uint64_t chg_hi = __ballot(ti + kWave < t_end && changed[ti + kWave] != 0);
            auto table_changes_at = [&](uint32_t j) {  // j within [t_first, t_end)
                const uint32_t i = j - t_first;
                return ((i < kWave ? chg_lo >> i : chg_hi >> (i - kWave)) & 1u) != 0;
            };
            uint32_t chunk = my_chunk;
            uint64_t loc = my_slab + (uint64_t)chunk * a.chunk_bytes;  // the ring chunk of the step
            auto next_chunk = [&]() {
                if (chunk) {
                    --chunk;
                    loc -= a.chunk_bytes;
                } else {
                    chunk = a.R - 1;
                    loc += (uint64_t)(a.R - 1) * a.chunk_bytes;
                }
            };
            // Steps [j, j_end) of one KIND (1 sum, 2 copy), all of them staging onward or none.
            auto stretch = [&](auto kind_tag, auto out_tag, uint32_t &j, uint32_t j_end) {
                constexpr int KIND = decltype(kind_tag)::value;
                constexpr bool HAS_OUT = decltype(out_tag)::value;
                if constexpr (KIND == 1 && HAS_OUT) {
                    // Sums: the local chunk of step j+1 is untouched until then, so it is loaded
                    // during step j, behind step j's own loads, and is in registers when its turn
                    // comes.  Two register sets alternate; the barrier does not wait for loads.
                    u32x4 set_a[U], set_b[U];
                    // AHEAD is a compile-time choice so that each variant is straight-line code and
                    // the waits the compiler places count exactly the loads that variant issued.
                    auto sum_step = [&](auto ahead_tag, u32x4(&cur)[U], u32x4(&nxt)[U]) {
                        constexpr bool AHEAD = decltype(ahead_tag)::value;
                        const uint64_t in_base = my_in0 + ((j + 1) & 1 ? parity_stride : 0);
                        const uint64_t out_base = my_out0 + (j & 1 ? parity_stride : 0);
                        u32x4 inc[U];
                        uint64_t aloc[U];
#pragma unroll
                        for (unsigned u = 0; u < U; ++u) {
                            inc[u] = load16<false>(in_base + dcur[u]);
                            aloc[u] = loc + bu[u];
                        }
                        next_chunk();
                        if constexpr (AHEAD) {
#pragma unroll
                            for (unsigned u = 0; u < U; ++u) nxt[u] = load16<kNtLocalLoad>(loc + bu[u]);
                        }
                        if (table_changes_at(j)) deltas_for(j, dcur);
#pragma unroll
                        for (unsigned u = 0; u < U; ++u) {
                            const u32x4 v = combine<BF16 ? kSumBF16 : kSumF32>(inc[u], cur[u]);
                            store16<kNtLocalStore>(aloc[u], v);
                            store16<false>(out_base + dcur[u], v);
                        }
                        __syncthreads();  // the next step reads what other waves of this workgroup just staged
                        R2_STAMP(2 + j);
                        ++j;
                    };
                    using Yes = std::integral_constant<bool, true>;
                    using No = std::integral_constant<bool, false>;
                    if (j < j_end) {
#pragma unroll
                        for (unsigned u = 0; u < U; ++u) set_a[u] = load16<kNtLocalLoad>(loc + bu[u]);
                        for (;;) {
                            if (j + 1 >= j_end) {
                                sum_step(No{}, set_a, set_b);
                                break;
                            }
                            sum_step(Yes{}, set_a, set_b);
                            if (j + 1 >= j_end) {
                                sum_step(No{}, set_b, set_a);
                                break;
                            }
                            sum_step(Yes{}, set_b, set_a);
                        }
                    }
                    return;
                }
                if constexpr (KIND == 2) {
                    // Copies: two register sets alternate here too, so that a step's loads never
                    // have to wait until the previous step's stores have read their data.
                    u32x4 set_a[U], set_b[U];
                    auto copy_step = [&](u32x4(&buf)[U]) {
                        const uint64_t in_base = my_in0 + ((j + 1) & 1 ? parity_stride : 0);
                        const uint64_t out_base = my_out0 + (j & 1 ? parity_stride : 0);
                        uint64_t aloc[U];
#pragma unroll
                        for (unsigned u = 0; u < U; ++u) {
                            buf[u] = load16<false>(in_base + dcur[u]);
                            aloc[u] = loc + bu[u];
                        }
                        if (HAS_OUT && table_changes_at(j)) deltas_for(j, dcur);
#pragma unroll
                        for (unsigned u = 0; u < U; ++u) {
                            store16<kNtLocalStore>(aloc[u], buf[u]);
                            if constexpr (HAS_OUT) store16<false>(out_base + dcur[u], buf[u]);
                        }
                        next_chunk();
                        __syncthreads();  // the next step reads what other waves of this workgroup just staged
                        R2_STAMP(2 + j);
                        ++j;
                    };
                    while (j < j_end) {
                        copy_step(set_a);
                        if (j >= j_end) break;
                        copy_step(set_b);
                    }
                    return;
                }
                for (; j < j_end; ++j) {
                    const uint64_t in_base = my_in0 + ((j + 1) & 1 ? parity_stride : 0);
                    const uint64_t out_base = my_out0 + (j & 1 ? parity_stride : 0);
                    uint64_t ain[U], aout[U], aloc[U];
#pragma unroll
                    for (unsigned u = 0; u < U; ++u) {
                        ain[u] = in_base + dcur[u];
                        aloc[u] = loc + bu[u];
                    }
                    if (HAS_OUT && table_changes_at(j)) deltas_for(j, dcur);
#pragma unroll
                    for (unsigned u = 0; u < U; ++u) aout[u] = out_base + dcur[u];
                    column_step<U, KIND, HAS_OUT, BF16>(ain, aout, aloc);
                    next_chunk();
                    __syncthreads();  // the next step reads what other waves of this workgroup just staged
                    R2_STAMP(2 + j);
                }
            };
            using std::integral_constant;
            uint32_t j = a.j0;
            const uint32_t last = a.J - 1;  // the one step that stages nothing
            if (j == 0) {  // copy-send: nothing comes in, the chunk goes out under table 0
                deltas_for(0, dcur);
                uint64_t aout[U], aloc[U];
#pragma unroll
                for (unsigned u = 0; u < U; ++u) {
                    aout[u] = my_out0 + dcur[u];
                    aloc[u] = loc + bu[u];
                }
                if (preload) {  // the chunk is already in registers
#pragma unroll
                    for (unsigned u = 0; u < U; ++u) store16<false>(aout[u], pre[u]);
                } else {
                    column_step<U, 0, true, BF16>(aout, aout, aloc);
                }
                next_chunk();
                __syncthreads();
                R2_STAMP(2);
                j = 1;
            } else {
                deltas_for(j - 1, dcur);  // the table the launch's first step reads with
            }
            const uint32_t sum_end = a.sum_last + 1 < a.j1 ? a.sum_last + 1 : a.j1;  // sums are steps 1..sum_last
            stretch(integral_constant<int, 1>{}, integral_constant<bool, true>{}, j, sum_end < last ? sum_end : last);
            if (j < sum_end) stretch(integral_constant<int, 1>{}, integral_constant<bool, false>{}, j, sum_end);
            stretch(integral_constant<int, 2>{}, integral_constant<bool, true>{}, j, a.j1 < last ? a.j1 : last);
            if (j < a.j1) stretch(integral_constant<int, 2>{}, integral_constant<bool, false>{}, j, a.j1);
        } else {
            bool have = false;  // dcur holds the offsets of the previous transmission
            for (uint32_t j = a.j0; j < a.j1; ++j) {
                const bool has_in = j > 0, has_out = j + 1 < a.J;
                const bool summing = has_in && j <= a.sum_last;
                uint64_t din[U], dout[U];
                if (has_in && !have) deltas_for(j - 1, dcur);  // first step of the launch
#pragma unroll
                for (unsigned u = 0; u < U; ++u) din[u] = dcur[u];
                if (has_out && (!(has_in || have) || changed[j])) deltas_for(j, dcur);
                have = true;
#pragma unroll
                for (unsigned u = 0; u < U; ++u) dout[u] = dcur[u];
                for (uint32_t rv = wave; rv < a.R; rv += n_waves) {
                    const uint32_t r = __builtin_amdgcn_readfirstlane(rv);
                    const uint32_t peer = (r + a.R - 1) % a.R;
                    rank_step(has_in, has_out, summing, local_of(r, j),
                              slab_stage + ((uint64_t)((j + 1) & 1) * a.R + peer) * per_rank,
                              slab_stage + ((uint64_t)(j & 1) * a.R + r) * per_rank, din, dout);
                }
                __syncthreads();  // the next step reads what other waves of this workgroup just staged
                R2_STAMP(2 + j);
            }
        }
        record_rows();
        return;
    }

    // The chunk's last column when the chunk is not a whole number of columns (or, if the rows did
    // not fit LDS, a column that straddles a cut): per-lane bounds and lookups.
    for (uint32_t j = a.j0; j < a.j1; ++j) {
        const bool has_in = j > 0, has_out = j + 1 < a.J;
        const bool summing = has_in && j <= a.sum_last;
        uint64_t in_lo = 0, out_lo = 0;
        uint32_t in_c = 0, out_c = 0;
        bool in_one = true, out_one = true;
        if (has_in) {
            in_lo = info[j - 1].lo;
            in_c = info[j - 1].c;
            in_one = b1 <= info[j - 1].hi;
        }
        if (has_out) {
            out_lo = info[j].lo;
            out_c = info[j].c;
            out_one = b1 <= info[j].hi;
        }
        const uint64_t *in_row = rows + (uint64_t)(has_in ? j - 1 : t_first) * row;
        const uint64_t *out_row = rows + (uint64_t)(has_out ? j : t_first) * row;

        for (uint32_t rv = wave; rv < a.R; rv += n_waves) {
            const uint32_t r = __builtin_amdgcn_readfirstlane(rv);
            const uint32_t peer = (r + a.R - 1) % a.R;
            const uint64_t local_addr = local_of(r, j);
            const uint64_t in_base = slab_stage + ((uint64_t)((j + 1) & 1) * a.R + peer) * per_rank;
            const uint64_t out_base = slab_stage + ((uint64_t)(j & 1) * a.R + r) * per_rank;

            u32x4 inc[U], loc[U];
#pragma unroll
            for (unsigned u = 0; u < U; ++u) {
                const uint64_t b = b0 + (uint64_t)(u * kWave + lane) * 16;
                if (b < b1) {
                    if (has_in) {
                        uint64_t d;
                        if (in_one) {
                            d = in_base + (uint64_t)in_c * a.cap - in_lo;
                        } else {
                            const uint32_t c = find_channel(in_row, C, b);
                            d = in_base + (uint64_t)c * a.cap - in_row[c];
                        }
                        inc[u] = load16<false>(d + b);
                    }
                    if (!has_in || summing) loc[u] = load16<kNtLocalLoad>(local_addr + b);
                }
            }
#pragma unroll
            for (unsigned u = 0; u < U; ++u) {
                const uint64_t b = b0 + (uint64_t)(u * kWave + lane) * 16;
                if (b < b1) {
                    u32x4 v;
                    if (!has_in) v = loc[u];
                    else if (!summing) v = inc[u];
                    else v = BF16 ? combine<kSumBF16>(inc[u], loc[u]) : combine<kSumF32>(inc[u], loc[u]);
                    if (has_in) store16<kNtLocalStore>(local_addr + b, v);
                    if (has_out) {
                        uint64_t d;
                        if (out_one) {
                            d = out_base + (uint64_t)out_c * a.cap - out_lo;
                        } else {
                            const uint32_t c = find_channel(out_row, C, b);
                            d = out_base + (uint64_t)c * a.cap - out_row[c];
                        }
                        store16<false>(d + b, v);
                    }
                }
            }
        }
        __syncthreads();
    }
    record_rows();
}
template <bool BF16, unsigned U>
__global__ __launch_bounds__(kMaxFusedWaves *kWave) void ring_fused_kernel(const FusedArgs a)
{
    fused_body<BF16, false, U>(a, nullptr);
}

static_assert(sizeof(FusedArgs) + sizeof(EpochBatch) <= 4000, "kernel arguments must fit 4 KiB");

template <bool BF16, unsigned U>
__global__ __launch_bounds__(kMaxFusedWaves *kWave) void ring_fused_partition_kernel(const FusedArgs a, const EpochBatch eb)
{
    fused_body<BF16, true, U>(a, &eb);
}

#ifdef R2_FUSED_TIMING
}  // namespace
}  // namespace r2
extern "C" int r2_debug_read(uint64_t *out, int n)
{
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(r2::g_dbg), n * 8) == hipSuccess ? 0 : -5;
}
namespace r2 {
namespace {
#endif

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

bool valid_dtype(int d) { return d == R2_F32 || d == R2_BF16; }
uint64_t elem_bytes(int d) { return d == R2_F32 ? 4 : 2; }

Mode mode_of(bool has_in, int op, int dtype)
{
    if (!has_in) return kSend;
    if (op == R2_OP_COPY) return kCopy;
    return dtype == R2_F32 ? kSumF32 : kSumBF16;
}

// The stage bytes one launch writes are read back by the next launch.  Keeping that window well
// inside the 256 MiB Infinity Cache lets the read be served from it.
constexpr uint64_t kDefaultStageWindow = 128ull << 20;

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
    bool links;           // ring with one table per link (row r: r -> r+1) instead of one per transmission
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
    if (d->schedule != R2_SCHED_AUTO && d->schedule != R2_SCHED_STEPS && d->schedule != R2_SCHED_FUSED)
        return R2_ERR_INVALID;
    if (s.links && s.kind != SimShape::kRing) return R2_ERR_INVALID;
    if ((s.kind != SimShape::kRing || s.links) && d->schedule == R2_SCHED_FUSED) return R2_ERR_INVALID;
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
    s.cap = round_up(s.chunk_bytes ? s.chunk_bytes : 1, 256);
    s.n_tx = s.links ? s.R : (uint64_t)s.S * s.T_slab;  // rows of the tables
    s.tables_bytes = round_up(s.n_tx * (s.C + 1) * 8, 256);
    s.stage_off = s.tables_bytes;
    const unsigned __int128 stage = (unsigned __int128)2 * s.R * s.S * s.C * s.cap;
    if (stage > ((unsigned __int128)1 << 62)) return R2_ERR_OVERFLOW;
    s.total_bytes = s.stage_off + (uint64_t)stage;

    const uint64_t window = d->stage_window_bytes ? d->stage_window_bytes : kDefaultStageWindow;
    const uint64_t per_slab = (uint64_t)s.active() * s.chunk_bytes;  // stage bytes a step writes per slab
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

template <Mode M, bool HAS_OUT, bool KEEP = false>
void launch_step(const StepArgs &a, dim3 grid, hipStream_t st)
{
    hipLaunchKernelGGL((ring_step_kernel<M, HAS_OUT, KEEP>), grid, dim3(kThreads), 0, st, a);
}

// The fused-column schedule needs whole 16-byte vectors everywhere and a grid that fits.
bool fused_eligible(const SimShape &s)
{
    if (s.kind != SimShape::kRing || s.links) return false;
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

// A stage this large is gone from the caches before anybody reads it back: written around them.
constexpr uint64_t kNtStageBytes = 128ull << 20;

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
    a.link_tables = s.links;
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

    const dim3 grid(blocks_for(a.hi - a.lo), s.active() * a.slab_count);
    hipStream_t st = (hipStream_t)stream;
    switch (m) {
    case kSend: launch_step<kSend, true>(a, grid, st); break;
    case kSumF32:
        if (keep) launch_step<kSumF32, true, true>(a, grid, st);
        else if (has_out) launch_step<kSumF32, true>(a, grid, st);
        else launch_step<kSumF32, false>(a, grid, st);
        break;
    case kSumBF16:
        if (keep) launch_step<kSumBF16, true, true>(a, grid, st);
        else if (has_out) launch_step<kSumBF16, true>(a, grid, st);
        else launch_step<kSumBF16, false>(a, grid, st);
        break;
    case kCopy:
        if (has_out) launch_step<kCopy, true>(a, grid, st); else launch_step<kCopy, false>(a, grid, st);
        break;
    }
    return hip_rc(hipGetLastError());
}

extern "C" int r2_sim_resolve_schedule(const r2_sim_desc *desc, const r2_epoch *epochs, uint32_t n_epochs)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if ((rc = check_epochs(epochs, n_epochs, s))) return rc;
    if (desc->schedule == R2_SCHED_FUSED && s.chunk_bytes && !fused_eligible(s)) return R2_ERR_INVALID;
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
    for (uint64_t p = 0; p < s.n_passes; ++p)
        for (uint32_t j = 0; j < s.J; ++j)
            if ((rc = r2_sim_step(desc, rank_bufs, p, j, workspace, workspace_bytes, stream))) return rc;
    return R2_OK;
}

extern "C" int r2_ring_rails_sim(const r2_sim_desc *desc, void *const *rank_bufs, const uint32_t *weights,
                                 const uint64_t *fail_masks, void *workspace, uint64_t workspace_bytes,
                                 uint64_t *offsets_log, void *stream)
{
    SimShape s;
    int rc = shape_of(desc, s);
    if (rc) return rc;
    if (!s.links || !rank_bufs || !weights || !fail_masks) return R2_ERR_INVALID;
    for (uint32_t r = 0; r < s.R; ++r) {
        const uint64_t p = reinterpret_cast<uint64_t>(rank_bufs[r]);
        if (s.chunk_bytes && (!p || (p & 15u))) return R2_ERR_INVALID;
    }
    if ((rc = check_workspace(workspace, workspace_bytes, s))) return rc;
    // One table per link, cut by the channels that are up at both of its ends.
    const uint64_t full = s.C == 64 ? ~0ull : ((1ull << s.C) - 1);
    r2_epoch links[R2_MAX_RANKS];
    for (uint32_t r = 0; r < s.R; ++r) {
        links[r] = r2_epoch{r, (fail_masks[r] | fail_masks[(r + 1) % s.R]) & full, weights};
        if (!any_healthy(weights, links[r].fail_mask, s.C)) return R2_ERR_NO_HEALTHY_CHANNEL;
    }
    if ((rc = launch_partition_epochs(links, s.R, s.C, desc->align, s.chunk_bytes, s.R,
                                      static_cast<uint64_t *>(workspace), offsets_log, (hipStream_t)stream)))
        return rc;
    if (s.chunk_bytes == 0) return R2_OK;
    for (uint64_t p = 0; p < s.n_passes; ++p)
        for (uint32_t j = 0; j < s.J; ++j)
            if ((rc = r2_sim_step(desc, rank_bufs, p, j, workspace, workspace_bytes, stream))) return rc;
    return R2_OK;
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

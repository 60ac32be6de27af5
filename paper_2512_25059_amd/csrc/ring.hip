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

__device__ inline uint64_t uniform64(uint64_t x)  // tell the compiler the value is wave-uniform
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// The slice that holds chunk byte b0, remembered from tile to tile: a workgroup walks the chunk
// front to back and slices are long, so the table is searched only when a cut is crossed.
struct Span {
    uint64_t lo = 0, hi = 0, delta = 0;
};
__device__ inline void locate(const ChannelTable &t, uint32_t C, uint64_t b0, Span &s)
{
    if (b0 < s.lo || b0 >= s.hi) {
        const uint32_t c = find_channel(t.off, C, b0);
        s.lo = uniform64(t.off[c]);
        s.hi = uniform64(t.off[c + 1]);
        s.delta = uniform64(t.delta[c]);
    }
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
    uint64_t bytes;           // the whole chunk: what the tables partition
    uint64_t lo, hi;          // the part of it this launch moves; lo is a multiple of 16, and so
                              // is hi unless hi == bytes
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
            locate(tin, C, b0, sin);
            in_one = b1 <= sin.hi;
        }
        if constexpr (HAS_OUT) {
            locate(tout, C, b0, sout);
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
                if constexpr (HAS_IN) store16<kNtLocalStore>(local_addr + b + u * (kThreads * 16), r);
                if constexpr (HAS_OUT) store16<kNtStageStore>(sout.delta + b + u * (kThreads * 16), r);
            }
            continue;
        }
        // The chunk's last, partial tile, or a tile that straddles a cut: every lane checks its
        // bounds and, where needed, looks its channel up.
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
                if constexpr (HAS_IN) store16<kNtLocalStore>(local_addr + b, r);
                if constexpr (HAS_OUT) {
                    const uint64_t d = out_one ? sout.delta : tout.delta[find_channel(tout.off, C, b)];
                    store16<kNtStageStore>(d + b, r);
                }
            }
        }
    }

    // What the vectors did not cover, one element at a time: the last bytes % 16 of an aligned
    // chunk, or everything if the chunk's address is only element-aligned.
    using Elem = typename std::conditional<M == kSumF32, uint32_t, uint16_t>::type;
    const uint64_t first = nvec * 16;
    const uint64_t n_el = (job.hi - first) / sizeof(Elem);
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
        if constexpr (HAS_IN) *gptr<Elem>(local_addr + b) = r;
        if constexpr (HAS_OUT) {
            const uint32_t c = find_channel(tout.off, C, b);
            *gptr<Elem>(tout.delta[c] + b) = r;
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
    uint32_t slab_begin, slab_count;  // the slabs this launch covers
    uint64_t lo, hi;                  // and the byte range of every ring chunk it moves
};

// blockIdx.y = rank * slab_count + (slab - slab_begin), blockIdx.x = workgroup within the range.
template <Mode M, bool HAS_OUT>
__global__ __launch_bounds__(kThreads) void ring_step_kernel(const StepArgs a)
{
    __shared__ ChannelTable tin, tout;
    const uint32_t r = blockIdx.y / a.slab_count, l = a.slab_begin + (blockIdx.y - r * a.slab_count);
    const uint32_t j = a.step;
    const uint32_t chunk = (r + a.chunk_start + 2 * a.R - j) % a.R;  // j <= 2R-2
    const uint32_t peer = (r + a.R - 1) % a.R;
    const uint64_t row = (uint64_t)a.C + 1;
    const uint64_t t_out = (uint64_t)l * a.T_slab + j;

    ChunkJob job;
    job.local = reinterpret_cast<uint8_t *>(a.rank_buf[r]) + ((uint64_t)l * a.R + chunk) * a.chunk_bytes;
    job.bytes = a.chunk_bytes;
    job.lo = a.lo;
    job.hi = a.hi;
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

struct SimShape {
    uint32_t R, S, C, J, T_slab;
    uint64_t chunk_bytes, cap, n_tx;
    uint64_t tables_bytes, stage_off, total_bytes;
    // passes: the run is cut into groups of slabs, or one slab's chunks into byte ranges
    uint32_t slabs_per_pass, n_sub;
    uint64_t sub_bytes, n_passes;
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

    const uint64_t window = d->stage_window_bytes ? d->stage_window_bytes : kDefaultStageWindow;
    const uint64_t per_slab = (uint64_t)s.R * s.chunk_bytes;  // stage bytes a step writes per slab
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
    ChunkJob job{static_cast<uint8_t *>(local), bytes, 0, bytes, in_offsets, out_offsets, stage_capacity, n_channels};
    const unsigned blocks = blocks_for(bytes);
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
    if (desc->phases == R2_PHASE_AG) op = R2_OP_COPY;
    else if (desc->phases == R2_PHASE_RS) op = R2_OP_SUM;
    else op = step <= s.R - 1 ? R2_OP_SUM : R2_OP_COPY;
    const Mode m = mode_of(has_in, op, desc->dtype);

    const dim3 grid(blocks_for(a.hi - a.lo), s.R * a.slab_count);
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
    for (uint64_t p = 0; p < s.n_passes; ++p)
        for (uint32_t j = 0; j < s.J; ++j)
            if ((rc = r2_sim_step(desc, rank_bufs, p, j, workspace, workspace_bytes, stream))) return rc;
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

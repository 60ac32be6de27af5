// The chunk worker of libr2ccl: one fused reduce-copy over a byte range of a chunk, as device code
// shared by the kernels of ring.hip (included there only; not part of the ABI).
//
// R2CCL paper: Sec. 2.1 (a collective's data is cut over channels, each bound to a NIC), Sec. 4.3
// Technique II (per-NIC send staging buffers), Sec. 5.2 (a ring step adds the incoming chunk into the
// local buffer and passes it on).
//
// The data path is bandwidth-bound: per 16-byte vector two loads, one add, two stores.  Every lane
// moves whole 16-byte vectors; a wavefront touches 1 KiB of consecutive addresses per access.  The
// slice that holds a tile is found by a wavefront-wide comparison against the offsets table, which
// every wavefront holds in its lanes; only tiles that straddle a cut search an LDS copy per lane.
#pragma once

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

}  // namespace
}  // namespace r2

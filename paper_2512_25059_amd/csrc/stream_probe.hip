// Measurement aid, not part of libr2ccl.so: what this GPU's memory system gives a bare kernel with the
// step kernel's access shape (256 threads, two 16-byte vectors per lane and stream, one 8 KiB tile per
// workgroup) and none of its tables, slices or argument block.  bench.py --stream-mix times these
// launches beside the product's, so that the step kernel's distance from "what a plain stream mix gets"
// can be re-measured by anyone.  Two patterns:
//
//   cold mix      n_read + n_write streams of `bytes` each, all non-temporal, over buffers the caller
//                 rotates so that nothing is found in any cache;
//   ring pattern  the streams of one ring step when the stage written by one launch is read by the next
//                 (Sec. 5 of the paper: local chunk in, incoming stage in, local chunk out, outgoing stage
//                 out): local streams and the stage read non-temporal, the stage write cacheable (the step
//                 kernel's policy), locals rotated, two stage buffers alternating.
//
// Both entry points launch on the caller's stream and return; timing is the caller's (events on that
// stream).  Buffers are the caller's device memory, at least `bytes` long each, 16-byte aligned; `bytes`
// must be a multiple of 8 KiB.  Return value: 0, or -1 for arguments that do not fit the above.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define R2P_GLOBAL __attribute__((address_space(1)))

constexpr uint32_t kThreads = 256;
constexpr uint32_t kVectorsPerLane = 2;
constexpr uint64_t kTileBytes = (uint64_t)kThreads * kVectorsPerLane * 16;

__device__ inline u32x4 load_nt(uint64_t a) { return __builtin_nontemporal_load((R2P_GLOBAL const u32x4 *)a); }
__device__ inline void store_nt(uint64_t a, u32x4 v) { __builtin_nontemporal_store(v, (R2P_GLOBAL u32x4 *)a); }
__device__ inline void store_cached(uint64_t a, u32x4 v) { *(R2P_GLOBAL u32x4 *)a = v; }

// something that depends on both operands, so that neither load can be dropped
__device__ inline u32x4 mix(u32x4 a, u32x4 b)
{
    a.x = __float_as_uint(__uint_as_float(a.x) + __uint_as_float(b.x));
    a.y += b.y;
    a.z ^= b.z;
    a.w += b.w;
    return a;
}

template <int READS, int WRITES>
__global__ __launch_bounds__(kThreads) void cold_mix_kernel(uint64_t r0, uint64_t r1, uint64_t w0, uint64_t w1,
                                                             uint64_t n_vectors)
{
    const uint64_t first = (uint64_t)blockIdx.x * (kThreads * kVectorsPerLane) + threadIdx.x;
    u32x4 x[kVectorsPerLane];
#pragma unroll
    for (uint32_t u = 0; u < kVectorsPerLane; ++u) {
        const uint64_t v = first + u * kThreads;
        x[u] = u32x4{1, 2, 3, 4};
        if (v >= n_vectors) continue;
        if (READS >= 1) x[u] = load_nt(r0 + v * 16);
        if (READS >= 2) x[u] = mix(x[u], load_nt(r1 + v * 16));
    }
#pragma unroll
    for (uint32_t u = 0; u < kVectorsPerLane; ++u) {
        const uint64_t v = first + u * kThreads;
        if (v >= n_vectors) continue;
        if (WRITES >= 1) store_nt(w0 + v * 16, x[u]);
        if (WRITES >= 2) store_nt(w1 + v * 16, x[u]);
        // a read-only launch keeps its loads alive through a store that never happens on real data
        if (WRITES == 0 && x[u].x == 0x12345678u && x[u].y == 0x9abcdef0u && x[u].z == 0x0fedcba9u) store_nt(w0 + v * 16, x[u]);
    }
}

enum Kind { kSum = 0, kCopy = 1, kLastCopy = 2, kSend = 3 };

template <int KIND>
__global__ __launch_bounds__(kThreads) void ring_pattern_kernel(uint64_t local, uint64_t stage_in, uint64_t stage_out,
                                                                 uint64_t n_vectors)
{
    const uint64_t first = (uint64_t)blockIdx.x * (kThreads * kVectorsPerLane) + threadIdx.x;
    u32x4 x[kVectorsPerLane];
#pragma unroll
    for (uint32_t u = 0; u < kVectorsPerLane; ++u) {
        const uint64_t v = first + u * kThreads;
        x[u] = u32x4{1, 2, 3, 4};
        if (v >= n_vectors) continue;
        if (KIND != kSend) x[u] = load_nt(stage_in + v * 16);
        if (KIND == kSum) x[u] = mix(x[u], load_nt(local + v * 16));
        if (KIND == kSend) x[u] = load_nt(local + v * 16);
    }
#pragma unroll
    for (uint32_t u = 0; u < kVectorsPerLane; ++u) {
        const uint64_t v = first + u * kThreads;
        if (v >= n_vectors) continue;
        if (KIND != kSend) store_nt(local + v * 16, x[u]);
        if (KIND != kLastCopy) store_cached(stage_out + v * 16, x[u]);
    }
}

bool fits(uint64_t bytes, int launches)
{
    return bytes != 0 && bytes % kTileBytes == 0 && bytes / kTileBytes <= 0x7fffffffull && launches >= 0;
}

}  // namespace

// Launch i of `launches` reads buffers[(4i) % n], buffers[(4i+1) % n] and writes buffers[(4i+2) % n],
// buffers[(4i+3) % n] (as many of them as it has streams).  `buffers`: host array of n >= 4 device addresses.
extern "C" int r2probe_cold_mix(int n_read, int n_write, const uint64_t *buffers, int n_buffers, uint64_t bytes,
                                int launches, hipStream_t stream)
{
    if (!buffers || n_buffers < 4 || n_read < 0 || n_read > 2 || n_write < 0 || n_write > 2 || n_read + n_write == 0 ||
        !fits(bytes, launches))
        return -1;
    for (int b = 0; b < n_buffers; ++b)
        if (!buffers[b] || buffers[b] % 16) return -1;
    const dim3 grid((unsigned)(bytes / kTileBytes)), block(kThreads);
    const uint64_t nv = bytes / 16;
    for (int i = 0; i < launches; ++i) {
        const uint64_t r0 = buffers[(4 * i) % n_buffers], r1 = buffers[(4 * i + 1) % n_buffers];
        const uint64_t w0 = buffers[(4 * i + 2) % n_buffers], w1 = buffers[(4 * i + 3) % n_buffers];
#define R2P_MIX(R, W) \
    if (n_read == R && n_write == W) hipLaunchKernelGGL((cold_mix_kernel<R, W>), grid, block, 0, stream, r0, r1, w0, w1, nv)
        R2P_MIX(1, 0); R2P_MIX(2, 0); R2P_MIX(0, 1); R2P_MIX(0, 2);
        R2P_MIX(1, 1); R2P_MIX(2, 1); R2P_MIX(1, 2); R2P_MIX(2, 2);
#undef R2P_MIX
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// kind: 0 sum (local in, stage in, local out, stage out), 1 copy with stage (stage in, local out, stage out),
// 2 last copy (stage in, local out), 3 send (local in, stage out).  Launch i works on locals[i % n] and reads
// the stage buffer launch i-1 wrote (the two stage buffers alternate).
extern "C" int r2probe_ring_pattern(int kind, const uint64_t *locals, int n_locals, uint64_t stage_a, uint64_t stage_b,
                                    uint64_t bytes, int launches, hipStream_t stream)
{
    if (!locals || n_locals < 1 || kind < 0 || kind > 3 || !stage_a || !stage_b || stage_a % 16 || stage_b % 16 ||
        !fits(bytes, launches))
        return -1;
    for (int b = 0; b < n_locals; ++b)
        if (!locals[b] || locals[b] % 16) return -1;
    const dim3 grid((unsigned)(bytes / kTileBytes)), block(kThreads);
    const uint64_t nv = bytes / 16;
    for (int i = 0; i < launches; ++i) {
        const uint64_t local = locals[i % n_locals];
        const uint64_t in = (i & 1) ? stage_a : stage_b, out = (i & 1) ? stage_b : stage_a;
        switch (kind) {
        case kSum: hipLaunchKernelGGL((ring_pattern_kernel<kSum>), grid, block, 0, stream, local, in, out, nv); break;
        case kCopy: hipLaunchKernelGGL((ring_pattern_kernel<kCopy>), grid, block, 0, stream, local, in, out, nv); break;
        case kLastCopy: hipLaunchKernelGGL((ring_pattern_kernel<kLastCopy>), grid, block, 0, stream, local, in, out, nv); break;
        default: hipLaunchKernelGGL((ring_pattern_kernel<kSend>), grid, block, 0, stream, local, in, out, nv); break;
        }
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

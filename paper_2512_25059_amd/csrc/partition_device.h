// Device-side partition arithmetic shared by the kernels of libr2ccl (not part of the ABI).
//
// R2CCL paper, Sec. 5.1 (R2CCL-Balance): healthy NICs share the data in proportion to their
// bandwidth, a failed NIC carries nothing.  The rounding rule is stated in r2ccl.h.
#pragma once

#include "r2_internal.h"

namespace r2 {

// floor(r * p / w) for a 128-bit product, by restoring division; needs r*p < w * 2^64.
__device__ inline uint64_t div128(uint64_t hi, uint64_t lo, uint64_t w)
{
    uint64_t rem = hi, quo = 0;
    for (int i = 63; i >= 0; --i) {
        const uint64_t carry = rem >> 63;
        rem = (rem << 1) | ((lo >> i) & 1u);
        if (carry || rem >= w) {
            rem -= w;
            quo |= 1ull << i;
        }
    }
    return quo;
}

// floor(U * P / W) without overflow, for P <= W, W > 0.  U = q*W + r gives q*P + floor(r*P/W);
// q*P <= U fits, and r*P < W^2 is divided in 128 bits when it does not fit 64.
__device__ inline uint64_t mul_div_floor(uint64_t U, uint64_t P, uint64_t W)
{
    if (((U | W) >> 32) == 0) return U * P / W;  // the usual sizes: the product fits 64 bits
    const uint64_t q = U / W, r = U - q * W;
    const uint64_t lo = r * P, hi = __umul64hi(r, P);
    const uint64_t frac = hi == 0 ? lo / W : div128(hi, lo, W);
    return q * P + frac;
}

// The whole wavefront partitions one chunk.  Lane c carries channel c's weight (lanes >= C carry
// nothing).  The cumulative bandwidth in front of each channel is a wavefront-wide inclusive scan.
// Returns the lane's cut point offsets[lane] (meaningful for lane < C); *total_weight receives W.
__device__ inline uint64_t partition_lane(uint32_t weight, bool failed, uint32_t C, uint64_t bytes,
                                          uint32_t align, uint64_t *total_weight)
{
    const unsigned lane = threadIdx.x & (kWave - 1);
    const uint32_t e = (lane < C && !failed) ? weight : 0;
    uint64_t P = 0, W = 0;  // bandwidth of the channels before this one; total
    if (C <= 16) {
        // Few channels: a walk over them with the running sum in scalar registers beats the
        // log-step scan, whose every round is a round trip through the cross-lane network.
        for (uint32_t c = 0; c < C; ++c) {
            const uint32_t wc = __builtin_amdgcn_readlane(e, c);
            if (lane == c) P = W;
            W += wc;
        }
    } else {
        uint64_t incl = e;
#pragma unroll
        for (unsigned d = 1; d < kWave; d <<= 1) {
            if (d < C) {  // lanes from C on carry nothing: log2(C) rounds reach every channel
                const uint64_t up = __shfl_up(incl, d, kWave);
                if (lane >= d) incl += up;
            }
        }
        W = __shfl(incl, C - 1, kWave);
        P = incl - e;
    }

    *total_weight = W;
    if (W == 0) return 0;
    if (P == W) return bytes;
    return (uint64_t)align * mul_div_floor(bytes / align, P, W);
}

// As partition_lane, storing the row (C+1 entries) to `row` and, if not null, to `row2`.
__device__ inline void partition_wave(uint32_t weight, bool failed, uint32_t C, uint64_t bytes,
                                      uint32_t align, uint64_t *row, uint64_t *row2, int32_t *status)
{
    const unsigned lane = threadIdx.x & (kWave - 1);
    uint64_t W;
    const uint64_t o = partition_lane(weight, failed, C, bytes, align, &W);
    if (lane < C) {
        row[lane] = o;
        if (row2) row2[lane] = o;
    }
    if (lane == 0) {
        const uint64_t end = W == 0 ? 0 : bytes;
        row[C] = end;
        if (row2) row2[C] = end;
        if (status) *status = W == 0 ? R2_ERR_NO_HEALTHY_CHANNEL : R2_OK;
    }
}

// Channel states travel by value in the kernel argument block: no host-to-device copy, no
// allocation.  A batch holds as many epochs as fit.
constexpr uint32_t kBatchEpochs = 32;
constexpr uint32_t kBatchWeights = 640;

struct EpochBatch {
    uint64_t t_start[kBatchEpochs];
    uint64_t fail_mask[kBatchEpochs];
    uint32_t weights[kBatchWeights];  // [n][C]
    uint32_t n;
};

// Epochs that fit one batch, for n_channels channels.
inline uint32_t epochs_per_batch(uint32_t C) { return kBatchWeights / C < kBatchEpochs ? kBatchWeights / C : kBatchEpochs; }

// Copies epochs [i0, i1) into a batch (host side).
inline void fill_batch(EpochBatch &b, const r2_epoch *epochs, uint32_t i0, uint32_t i1, uint32_t C)
{
    b.n = i1 - i0;
    for (uint32_t k = 0; k < b.n; ++k) {
        b.t_start[k] = epochs[i0 + k].t_start;
        b.fail_mask[k] = epochs[i0 + k].fail_mask;
        for (uint32_t c = 0; c < C; ++c) b.weights[k * C + c] = epochs[i0 + k].weights[c];
    }
}

// The state in force at transmission t: the last epoch of the batch that started at or before t.
__device__ inline uint32_t epoch_at(const EpochBatch &b, uint64_t t)
{
    uint32_t i = 0;
    for (uint32_t k = 1; k < b.n; ++k)
        if (b.t_start[k] <= t) i = k;
    return i;
}

}  // namespace r2

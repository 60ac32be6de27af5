// Channel partition on the device: one wavefront per chunk to partition, one lane per channel.
//
// Follows the R2CCL paper, Sec. 5.1 (R2CCL-Balance): the data a server must move is spread over
// its healthy NICs in proportion to their bandwidth, a failed NIC carries nothing, and the volume
// itself is unchanged ("Overhead Analysis").  The rounding rule is stated in r2ccl.h.
#include <mutex>

#include "partition_device.h"

namespace r2 {
namespace {

constexpr unsigned kBlock = 256;  // four problems per workgroup
constexpr unsigned kWavesPerBlock = kBlock / kWave;

__global__ __launch_bounds__(kBlock) void partition_arrays_kernel(
    const uint32_t *__restrict__ weights, const uint64_t *__restrict__ fail_mask,
    const uint64_t *__restrict__ bytes, uint32_t C, uint32_t align, uint32_t n_problems,
    uint64_t *__restrict__ offsets, int32_t *__restrict__ status)
{
    const uint64_t p = (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (p >= n_problems) return;  // whole wavefront leaves together
    const unsigned lane = threadIdx.x & (kWave - 1);
    const uint32_t w = lane < C ? weights[p * C + lane] : 0;
    const bool failed = (fail_mask[p] >> lane) & 1u;
    partition_wave(w, failed, C, bytes[p], align, offsets + p * (C + 1), nullptr,
                   status ? status + p : nullptr);
}

__global__ __launch_bounds__(kBlock) void partition_epochs_kernel(
    const EpochBatch batch, uint32_t C, uint32_t align, uint64_t bytes, uint64_t t_begin,
    uint64_t t_end, uint64_t *__restrict__ tables, uint64_t *__restrict__ log)
{
    const uint64_t t = t_begin + (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (t >= t_end) return;  // whole wavefront leaves together
    const uint32_t i = epoch_at(batch, t);
    const unsigned lane = threadIdx.x & (kWave - 1);
    const uint32_t w = lane < C ? batch.weights[i * C + lane] : 0;
    const bool failed = (batch.fail_mask[i] >> lane) & 1u;
    partition_wave(w, failed, C, bytes, align, tables + t * (C + 1),
                   log ? log + t * (C + 1) : nullptr, nullptr);
}

// In-flight failover plan: wave (p, f) shares the slice of channel f of problem p out over the
// channels that are still healthy, if f is among the channels that have just failed.
__global__ __launch_bounds__(kBlock) void rollback_plan_kernel(
    const uint64_t *__restrict__ offsets, const uint32_t *__restrict__ weights,
    const uint64_t *__restrict__ mask_before, const uint64_t *__restrict__ mask_after, uint32_t C,
    uint32_t align, uint32_t n_problems, uint64_t *__restrict__ plan, int32_t *__restrict__ status)
{
    const uint64_t w_id = (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (w_id >= (uint64_t)n_problems * C) return;  // whole wavefront leaves together
    const uint32_t p = (uint32_t)(w_id / C), f = (uint32_t)(w_id - (uint64_t)p * C);
    const unsigned lane = threadIdx.x & (kWave - 1);
    const uint64_t before = mask_before[p], after = mask_after[p];
    const uint64_t *off = offsets + (uint64_t)p * (C + 1);
    uint64_t *row = plan + ((uint64_t)p * C + f) * (C + 1);
    const uint64_t len = off[f + 1] - off[f];
    const bool newly = ((after >> f) & 1u) && !((before >> f) & 1u);
    if (!newly || len == 0) {
        if (lane <= C) row[lane] = 0;
        if (C == kWave && lane == 0) row[C] = 0;
        return;
    }
    const uint32_t w = lane < C ? weights[(uint64_t)p * C + lane] : 0;
    int32_t st = R2_OK;
    partition_wave(w, (after >> lane) & 1u, C, len, align, row, nullptr, &st);
    // a problem's status only ever goes from R2_OK to an error (the caller clears it beforehand)
    if (lane == 0 && status && st != R2_OK) atomicMin(status + p, st);
}

// Failover plans of a run's in-flight epochs (Sec. 4.3 Technique II): wave (k, f) looks at epoch k of
// the batch.  If that epoch strikes in flight within the run and channel f newly fails in it, the wave
// cuts the chunk by the state before (epoch k-1) to find slice f, and shares that slice's bytes out
// over the channels the epoch leaves up; otherwise row f of the epoch's plan is zero.  Epoch 0 of a
// batch only serves as the state before epoch 1, unless `first_is_real` (then it is the run's first
// epoch, which has no plan: zero rows).
__global__ __launch_bounds__(kBlock) void inflight_plan_kernel(const EpochBatch batch, uint32_t in_flight_bits,
                                                               uint32_t first_epoch, bool first_is_real, uint32_t C,
                                                               uint32_t align, uint64_t bytes, uint64_t n_tx,
                                                               uint64_t *__restrict__ plans)
{
    const uint64_t w_id = (uint64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
    if (w_id >= (uint64_t)batch.n * C) return;  // whole wavefront leaves together
    const uint32_t k = (uint32_t)(w_id / C), f = (uint32_t)(w_id - (uint64_t)k * C);
    if (k == 0 && !first_is_real) return;
    const unsigned lane = threadIdx.x & (kWave - 1);
    uint64_t *row = plans + (((uint64_t)first_epoch + k) * C + f) * (C + 1);
    const bool struck = k > 0 && ((in_flight_bits >> k) & 1u) && batch.t_start[k] < n_tx;
    const uint64_t before = k > 0 ? batch.fail_mask[k - 1] : 0, after = batch.fail_mask[k];
    uint64_t len = 0;
    if (struck && ((after >> f) & 1u) && !((before >> f) & 1u)) {
        uint64_t W;
        const uint32_t w_old = lane < C ? batch.weights[(k - 1) * C + lane] : 0;
        const uint64_t cut = partition_lane(w_old, (before >> lane) & 1u, C, bytes, align, &W);
        const uint64_t lo = __shfl(cut, f, kWave);
        const uint64_t hi = f + 1 < C ? __shfl(cut, f + 1, kWave) : bytes;
        len = W ? hi - lo : 0;
    }
    if (len == 0) {
        if (lane <= C) row[lane] = 0;
        if (C == kWave && lane == 0) row[C] = 0;
        return;
    }
    const uint32_t w_new = lane < C ? batch.weights[k * C + lane] : 0;
    partition_wave(w_new, (after >> lane) & 1u, C, len, align, row, nullptr, nullptr);
}

// The row r2_partition (host pointers in, host pointers out) has the device write.
static __device__ __align__(256) uint64_t host_call_row[R2_MAX_CHANNELS + 1];

}  // namespace

int launch_partition_epochs(const r2_epoch *epochs, uint32_t n_epochs, uint32_t C, uint32_t align,
                            uint64_t chunk_bytes, uint64_t n_tx, uint64_t *tables, uint64_t *log,
                            hipStream_t stream)
{
    const uint32_t per_batch = epochs_per_batch(C);
    for (uint32_t i0 = 0; i0 < n_epochs; i0 += per_batch) {
        const uint32_t i1 = i0 + per_batch < n_epochs ? i0 + per_batch : n_epochs;
        const uint64_t t_begin = epochs[i0].t_start;
        if (t_begin >= n_tx) break;
        uint64_t t_end = i1 < n_epochs ? epochs[i1].t_start : n_tx;
        if (t_end > n_tx) t_end = n_tx;
        EpochBatch b;
        fill_batch(b, epochs, i0, i1, C);
        const uint64_t n = t_end - t_begin;
        const uint64_t blocks = (n + kWavesPerBlock - 1) / kWavesPerBlock;
        if (blocks > 0x7fffffffull) return R2_ERR_OVERFLOW;
        hipLaunchKernelGGL(partition_epochs_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, stream,
                           b, C, align, chunk_bytes, t_begin, t_end, tables, log);
        const int rc = hip_rc(hipGetLastError());
        if (rc) return rc;
    }
    return R2_OK;
}

int launch_inflight_plans(const r2_epoch *epochs, const uint8_t *in_flight, uint32_t n_epochs, uint32_t C,
                          uint32_t align, uint64_t chunk_bytes, uint64_t n_tx, uint64_t *plans, hipStream_t stream)
{
    const uint32_t per_batch = epochs_per_batch(C);  // >= 10: a batch holds the state before and its successors
    for (uint32_t i0 = 0; i0 < n_epochs;) {
        const uint32_t i1 = i0 + per_batch < n_epochs ? i0 + per_batch : n_epochs;
        EpochBatch b;
        fill_batch(b, epochs, i0, i1, C);
        uint32_t bits = 0;
        for (uint32_t k = 1; k < b.n; ++k)
            if (in_flight && in_flight[i0 + k]) bits |= 1u << k;
        const uint64_t waves = (uint64_t)b.n * C;
        const unsigned blocks = (unsigned)((waves + kWavesPerBlock - 1) / kWavesPerBlock);
        hipLaunchKernelGGL(inflight_plan_kernel, dim3(blocks), dim3(kBlock), 0, stream, b, bits, i0, i0 == 0, C,
                           align, chunk_bytes, n_tx, plans);
        const int rc = hip_rc(hipGetLastError());
        if (rc) return rc;
        if (i1 == n_epochs) break;
        i0 = i1 - 1;  // the last epoch of this batch is the state before the next batch's first
    }
    return R2_OK;
}

}  // namespace r2

extern "C" int r2_partition_device(const uint32_t *weights, const uint64_t *fail_mask,
                                   const uint64_t *bytes, uint32_t n_channels, uint32_t align,
                                   uint32_t n_problems, uint64_t *offsets, int32_t *status,
                                   void *stream)
{
    if (n_channels == 0 || n_channels > R2_MAX_CHANNELS || align == 0) return R2_ERR_INVALID;
    if (n_problems == 0) return R2_OK;
    if (!weights || !fail_mask || !bytes || !offsets) return R2_ERR_INVALID;
    const unsigned blocks = (n_problems + r2::kWavesPerBlock - 1) / r2::kWavesPerBlock;
    hipLaunchKernelGGL(r2::partition_arrays_kernel, dim3(blocks), dim3(r2::kBlock), 0,
                       (hipStream_t)stream, weights, fail_mask, bytes, n_channels, align, n_problems,
                       offsets, status);
    return r2::hip_rc(hipGetLastError());
}

extern "C" int r2_rollback_plan_device(const uint64_t *offsets, const uint32_t *weights,
                                       const uint64_t *mask_before, const uint64_t *mask_after,
                                       uint32_t n_channels, uint32_t align, uint32_t n_problems,
                                       uint64_t *plan, int32_t *status, void *stream)
{
    if (n_channels == 0 || n_channels > R2_MAX_CHANNELS || align == 0) return R2_ERR_INVALID;
    if (n_problems == 0) return R2_OK;
    if (!offsets || !weights || !mask_before || !mask_after || !plan) return R2_ERR_INVALID;
    const uint64_t waves = (uint64_t)n_problems * n_channels;
    const uint64_t blocks = (waves + r2::kWavesPerBlock - 1) / r2::kWavesPerBlock;
    if (blocks > 0x7fffffffull) return R2_ERR_OVERFLOW;
    hipLaunchKernelGGL(r2::rollback_plan_kernel, dim3((unsigned)blocks), dim3(r2::kBlock), 0,
                       (hipStream_t)stream, offsets, weights, mask_before, mask_after, n_channels, align,
                       n_problems, plan, status);
    return r2::hip_rc(hipGetLastError());
}

extern "C" int r2_partition(const uint32_t *weights, uint64_t fail_mask, uint32_t n_channels,
                            uint64_t bytes, uint32_t align, uint64_t *offsets)
{
    if (!weights || !offsets || n_channels == 0 || n_channels > R2_MAX_CHANNELS || align == 0)
        return R2_ERR_INVALID;
    if (!r2::any_healthy(weights, fail_mask, n_channels)) {
        for (uint32_t c = 0; c <= n_channels; ++c) offsets[c] = 0;
        return R2_ERR_NO_HEALTHY_CHANNEL;
    }
    // The one row this call needs lives in a small static device array (each GPU has its own copy,
    // whose address is asked for once per device): nothing is allocated.  Calls are serialised, since
    // they share the row.
    static std::mutex lock;
    static uint64_t *rows[64];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return R2_ERR_DEVICE;
    std::lock_guard<std::mutex> hold(lock);
    if (!rows[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(r2::host_call_row)) != hipSuccess || !p) return R2_ERR_DEVICE;
        rows[dev] = static_cast<uint64_t *>(p);
    }
    uint64_t *d_row = rows[dev];
    const r2_epoch ep = {0, fail_mask, weights};
    int rc = r2::launch_partition_epochs(&ep, 1, n_channels, align, bytes, 1, d_row, nullptr, nullptr);
    if (rc == R2_OK)
        rc = r2::hip_rc(hipMemcpy(offsets, d_row, (size_t)(n_channels + 1) * sizeof(uint64_t), hipMemcpyDeviceToHost));
    return rc;
}

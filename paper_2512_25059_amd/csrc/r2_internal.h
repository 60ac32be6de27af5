// Internal declarations shared by the translation units of libr2ccl (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "r2ccl_ext.h"

namespace r2 {

constexpr unsigned kWave = 64;  // CDNA wavefront width; one lane per channel in the partition

inline int hip_rc(hipError_t e) { return e == hipSuccess ? R2_OK : R2_ERR_DEVICE; }

// True if at least one channel of this state can carry data.
inline bool any_healthy(const uint32_t *weights, uint64_t fail_mask, uint32_t C)
{
    for (uint32_t c = 0; c < C; ++c)
        if (!((fail_mask >> c) & 1u) && weights[c] != 0) return true;
    return false;
}

// Enqueue the partition of transmissions [0, n_tx) of a run whose channel state is given by the
// epoch list; every transmission partitions `chunk_bytes`.  tables / log: device [n_tx][C+1]
// (log may be null).  Epochs must already be validated.
int launch_partition_epochs(const r2_epoch *epochs, uint32_t n_epochs, uint32_t C, uint32_t align,
                            uint64_t chunk_bytes, uint64_t n_tx, uint64_t *tables, uint64_t *log,
                            hipStream_t stream);

// Enqueue the failover plans of the epochs marked in flight (in_flight[i] != 0; may be null): plans is
// device [n_epochs][C][C+1], every row of which is written (zero where there is nothing to re-carry).
// Epochs and flags must already be validated.
int launch_inflight_plans(const r2_epoch *epochs, const uint8_t *in_flight, uint32_t n_epochs, uint32_t C,
                          uint32_t align, uint64_t chunk_bytes, uint64_t n_tx, uint64_t *plans, hipStream_t stream);

// Independent pieces of one call (the rings of a split or recursive all-reduce) run side by side:
// the caller's stream forks into a few library-owned streams of default priority and joins them
// again before the call's dependent work, all with events, so the call stays asynchronous and in
// order on the caller's stream (and can be captured into a graph).  The streams are created once
// per device and live until the process ends.
constexpr unsigned kSideStreams = 3;

class ForkJoin {
public:
    // Lane 0 is the caller's stream, lanes 1..kSideStreams the library's.  rc() is R2_OK unless a
    // runtime call failed; after a failure the remaining calls do nothing.
    explicit ForkJoin(hipStream_t user);
    ~ForkJoin();
    ForkJoin(const ForkJoin &) = delete;
    ForkJoin &operator=(const ForkJoin &) = delete;
    hipStream_t lane(unsigned i);  // lane i, forked off the caller's stream where this object was made
    int join();                    // the caller's stream waits for every lane that was used
    int rc() const { return rc_; }

private:
    hipStream_t user_;
    struct Pool *pool_;
    bool used_[kSideStreams] = {};
    int rc_ = R2_OK;
};

}  // namespace r2

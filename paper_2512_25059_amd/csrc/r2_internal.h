// Internal declarations shared by the translation units of libr2ccl (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "r2ccl.h"

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

}  // namespace r2

// The fused-column schedule of the ring as device code (included by ring.hip only; not part of the
// ABI): one workgroup takes a column of the ring chunks of one slab through all steps of all ranks.
// R2CCL paper: Sec. 5.2 (the ring's steps), Sec. 5.1 (the partition the kernel can compute itself).
#pragma once

#include "reduce_copy_device.h"

namespace r2 {
namespace {

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

// PARTITION: the kernel computes the table rows it needs itself, from the channel states in `eb`
// (every workgroup for its own use, in LDS; the first column of each slab also records them in
// the workspace and the log), so that no partition launch has to run in front of it.
// The kernel-argument block (rank buffers, sizes, channel states: up to 4 KiB) is read in several
// dependent rounds -- sizes, then the wave's rank buffer, then the state in force, then its weights
// -- and in a launch whose arguments were just written every first touch of one of its 64-byte lines
// is a trip to memory.  One vector load, a lane per line, asks for all of them at once when the
// kernel starts; the rounds then meet L2.  The value is handed to keep_touched() once the prologue
// is over, which only keeps the load from being dropped.
__device__ inline uint32_t touch_kernel_arguments(uint32_t bytes)
{
    const uint32_t at = (threadIdx.x % kWave) * 64;
    uint32_t v = 0;
    if (threadIdx.x < kWave && at < bytes) {
        const char __attribute__((address_space(4))) *args =
            (const char __attribute__((address_space(4))) *)__builtin_amdgcn_kernarg_segment_ptr();
        v = *(const uint32_t __attribute__((address_space(4))) *)(args + at);
    }
    return v;
}
__device__ inline void keep_touched(uint32_t v) { asm volatile("" ::"v"(v)); }

template <bool BF16, bool PARTITION, unsigned U>
__device__ inline void fused_body(const FusedArgs &a, const EpochBatch *eb)
{
    const uint32_t touched = touch_kernel_arguments(sizeof(FusedArgs) + (PARTITION ? sizeof(EpochBatch) : 0));
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
    keep_touched(touched);

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

}  // namespace
}  // namespace r2

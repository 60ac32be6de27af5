// Fused columns for a ring whose links have tables of their own (included by ring.hip only; not
// part of the ABI).  R2CCL paper: Sec. 5.1 (every server spreads what it sends over its own healthy
// NICs), Sec. 6 "Topology-Aware Logical Re-ranking" (a link carries data on the rails both ends still
// have), Sec. 5.2 (the ring's steps).
#pragma once

#include "ring_fused_device.h"

namespace r2 {
namespace {

// The column idea is that of ring_fused_device.h: one workgroup takes a byte range of the ring
// chunks of one slab through the steps [j0, j1) of ALL ranks, a wave per rank, a barrier per step.
// What differs is the table: rank r reads with the table of the link (r-1) -> r for transmission
// j-1 and stages onward with the table of its own link r -> r+1 for transmission j, so no table is
// shared between ranks.  Every table row the launch can touch, [R links][t_first, t_end)[C+1], is
// put into LDS once, followed by the slice of each row that holds the column's first byte and a
// flag that says whether the row differs from the link's row before; a wave then carries its two
// sets of stage offsets (own link, predecessor's link) from step to step and looks them up again
// only where a flag is set.
//
// Dynamic LDS: rows (8 bytes each entry), then one ColInfo per (link, transmission).
constexpr uint32_t kLinksLdsBytes = 56 * 1024;

// PARTITION: the kernel cuts the chunk itself, from the links' channel states in `eb` (strung on one
// axis: link r's transmission t is r * link_rows + t), every workgroup for its own use; the first
// column of each slab also records the rows in the workspace and the log.  No partition launch has
// to run in front then.
template <bool BF16, unsigned U, bool PARTITION>
__device__ inline void fused_links_body(const FusedArgs &a, const uint64_t link_rows, const EpochBatch *eb)
{
    const uint32_t touched =
        touch_kernel_arguments(sizeof(FusedArgs) + 8 + (PARTITION ? sizeof(EpochBatch) : 0));
    extern __shared__ uint64_t s_link[];
    constexpr uint64_t kWidth = (uint64_t)kWave * 16 * U;
    const uint32_t l = (uint32_t)(blockIdx.x / a.cols_per_chunk);
    const uint64_t k = blockIdx.x - (uint64_t)l * a.cols_per_chunk;
    const uint64_t b0 = k * kWidth;
    const uint64_t b1 = b0 + kWidth < a.chunk_bytes ? b0 + kWidth : a.chunk_bytes;
    const uint32_t C = a.C, R = a.R;
    const uint32_t row = C + 1;
    const uint32_t t_first = a.j0 ? a.j0 - 1 : 0;
    const uint32_t t_end = a.j1 < a.T_slab ? a.j1 : a.T_slab;
    const uint32_t n_t = t_end - t_first;        // transmissions of a link this launch reads or writes
    const uint32_t link_entries = n_t * row;     // ... and their table entries
    const R2_LDS uint64_t *rows = (const R2_LDS uint64_t *)s_link;
    R2_LDS ColInfo *info = (R2_LDS ColInfo *)(s_link + (uint64_t)R * link_entries);

    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t lane = threadIdx.x % kWave, n_waves = blockDim.x / kWave;
    // A wave that plays one rank on a full-width column takes the fast path below.  If the launch
    // starts at step 0 it begins by staging a chunk of its own buffer, whose address depends on
    // nothing the prologue computes: loaded here, its latency passes while the tables are made.
    const bool fast = R <= n_waves && b0 + kWidth <= a.chunk_bytes;
    u32x4 pre[U] = {};
    if (fast && a.j0 == 0) {
        const uint64_t src = a.rank_buf[wave] + ((uint64_t)l * R + (wave + a.chunk_start) % R) * a.chunk_bytes + b0;
#pragma unroll
        for (unsigned u = 0; u < U; ++u) pre[u] = load16<kNtLocalLoad>(src + (uint64_t)(u * kWave + lane) * 16);
    }
    uint32_t top = 0;  // the largest power of two below C (0 if C = 1)
    while ((top ? top * 2 : 1) < C) top = top ? top * 2 : 1;
    // ColInfo::pad of a row: it may differ from the row of the link's transmission before (always
    // set for the first of the launch).  Tables mostly repeat, and then stage offsets are carried over.
    if constexpr (PARTITION) {
        // A wave per link walks the states in force over its transmissions here (mostly one): it cuts
        // the chunk once per state, finds the slice that holds the column's first byte in registers,
        // and then fills every row the state governs with all lanes at once -- a wave is slow at
        // anything it does row by row.
        for (uint32_t lv = wave; lv < R; lv += n_waves) {
            const uint32_t link = __builtin_amdgcn_readfirstlane(lv);
            const uint64_t tg0 = (uint64_t)link * link_rows + (uint64_t)l * a.T_slab + t_first;
            uint32_t e = epoch_at(*eb, tg0);  // the last state that started at or before the first row
            for (uint32_t ti0 = 0; ti0 < n_t; ++e) {
                // rows [ti0, ti1): up to where the next state begins (a later link's lie beyond n_t)
                const uint64_t next_begins = e + 1 < eb->n ? eb->t_start[e + 1] : ~0ull;
                const uint32_t ti1 = next_begins - tg0 < n_t ? (uint32_t)(next_begins - tg0) : n_t;
                const uint32_t weight = lane < C ? eb->weights[e * C + lane] : 0;
                uint64_t W;
                const bool failed = (eb->fail_mask[e] >> lane) & 1u;
                const uint64_t cut = partition_lane(weight, failed, C, a.chunk_bytes, a.align, &W);
                // the last channel whose cut point is at or before b0 (channel 0's is 0)
                const uint32_t c0 = 63 - (uint32_t)__builtin_clzll(__ballot(lane < C && cut <= b0));
                const uint64_t lo = __shfl(cut, c0, kWave);
                const uint64_t hi = c0 + 1 < C ? __shfl(cut, (c0 + 1) % kWave, kWave) : a.chunk_bytes;
                const uint32_t n_entries = (ti1 - ti0) * row;
                uint64_t *dst = s_link + (uint64_t)(link * n_t + ti0) * row;
                for (uint32_t i0 = 0; i0 < n_entries; i0 += kWave) {  // every lane takes part in the shuffle
                    const uint32_t c = (i0 + lane) % row;
                    const uint64_t v = __shfl(cut, c % kWave, kWave);
                    if (i0 + lane < n_entries) dst[i0 + lane] = c == C ? a.chunk_bytes : v;
                }
                for (uint32_t ti = ti0 + lane; ti < ti1; ti += kWave) {
                    R2_LDS ColInfo *ci = info + (link * n_t + ti);
                    ci->lo = lo;
                    ci->hi = hi;
                    ci->c = c0;
                    ci->pad = ti == ti0;
                }
                ti0 = ti1;
            }
        }
        __syncthreads();
    } else {
        for (uint32_t i = threadIdx.x; i < R * link_entries; i += blockDim.x) {
            const uint32_t link = i / link_entries, e = i - link * link_entries;
            s_link[i] = a.tables[((uint64_t)link * link_rows + (uint64_t)l * a.T_slab + t_first) * row + e];
        }
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < R * n_t; i += blockDim.x) {
            const R2_LDS uint64_t *off = rows + (uint64_t)i * row;
            const uint32_t c = find_channel_flat(off, C, top, b0);
            info[i].lo = off[c];
            info[i].hi = off[c + 1];
            info[i].c = c;
            uint32_t differs = i % n_t == 0;
            const R2_LDS uint64_t *before = differs ? off : off - row;  // the same link's row before
            for (uint32_t e = 0; e < row; ++e) differs |= off[e] != before[e];
            info[i].pad = differs;
        }
        __syncthreads();
    }
    // The first column of a slab records the rows for the caller: last of all, so that no step waits
    // for these stores.
    auto record_rows = [&]() {
        if (!PARTITION || k != 0) return;
        for (uint32_t i = threadIdx.x; i < R * link_entries; i += blockDim.x) {
            const uint32_t link = i / link_entries, e = i - link * link_entries;
            const uint64_t at = ((uint64_t)link * link_rows + (uint64_t)l * a.T_slab + t_first) * row + e;
            const uint64_t v = rows[i];
            a.tables_out[at] = v;
            if (a.log_out) a.log_out[at] = v;
        }
    };

    keep_touched(touched);
    const uint64_t per_rank = (uint64_t)a.S * C * a.cap;  // stage bytes of one (parity, rank)
    const uint64_t slab_stage = a.stage + (uint64_t)l * C * a.cap;

    // Stage offset (within one rank's stage of one parity) of chunk byte b under the table of
    // transmission t of `link`: uniform where the column lies inside one slice, looked up per lane
    // where it straddles a cut.
    auto stage_offset = [&](uint32_t link, uint32_t t, uint64_t b) {
        const uint32_t i = link * n_t + (t - t_first);
        if (b1 <= info[i].hi) return (uint64_t)info[i].c * a.cap - info[i].lo + b;
        const R2_LDS uint64_t *off = rows + (uint64_t)i * row;
        const uint32_t c = find_channel_flat(off, C, top, b);
        return (uint64_t)c * a.cap - off[c] + b;
    };

    if (fast) {
        // Everything a step needs besides the incoming data is fetched off its critical path: the
        // stage offsets it reads with were looked up during the step before (behind that step's
        // stores), those it writes with are looked up while its loads are in flight, and the local
        // chunk -- untouched until its step as long as the ring still sums -- was loaded a step
        // ahead.  Two register sets alternate, so nothing is moved between steps; the barrier does
        // not wait for loads.
        const uint32_t r = wave, peer = (r + R - 1) % R;
        const uint64_t my_slab = a.rank_buf[r] + (uint64_t)l * R * a.chunk_bytes;
        const uint64_t in0 = slab_stage + (uint64_t)peer * per_rank, out0 = slab_stage + (uint64_t)r * per_rank;
        const uint64_t parity_stride = (uint64_t)R * per_rank;
        uint64_t bu[U], din[U];
#pragma unroll
        for (unsigned u = 0; u < U; ++u) bu[u] = b0 + (uint64_t)(u * kWave + lane) * 16;
        auto local_of = [&](uint32_t j) {  // the ring chunk of step j
            return my_slab + (uint64_t)((r + a.chunk_start + 2 * R - j) % R) * a.chunk_bytes;
        };
        // bit i: the table of transmission t_first + i of the own link (the predecessor's) is not the
        // one before it.  With a wave per rank a launch has at most 2 * 16 - 2 transmissions.
        static_assert(2 * kMaxFusedWaves - 2 < kWave, "one ballot must cover a launch's transmissions");
        const uint64_t out_changes = __ballot(lane < n_t && info[r * n_t + (lane < n_t ? lane : 0)].pad != 0);
        const uint64_t in_changes = __ballot(lane < n_t && info[peer * n_t + (lane < n_t ? lane : 0)].pad != 0);
        uint64_t dout[U];
#pragma unroll
        for (unsigned u = 0; u < U; ++u) {  // the offsets under the launch's first tables; carried from there
            din[u] = stage_offset(peer, t_first, bu[u]);
            dout[u] = stage_offset(r, t_first, bu[u]);
        }
        uint32_t j = a.j0;
        // One step, its kind fixed at compile time so that the code is straight-line and the waits
        // the compiler places count exactly the loads that variant issued (with a run-time "is the
        // next local chunk loaded ahead" they would cover the worst case, and the load ahead would
        // be waited for in the same step).  KIND: 0 copy-send (cur = the chunk, already loaded),
        // 1 sum (cur = the local chunk, loaded a step ahead; AHEAD: load the next one into nxt),
        // 2 copy (cur = where the incoming data goes: two sets alternate, so that a step's loads
        // never wait until the previous step's stores have read their registers).
        auto step = [&](auto kind_tag, auto out_tag, auto ahead_tag, u32x4(&cur)[U], u32x4(&nxt)[U]) {
            constexpr int KIND = decltype(kind_tag)::value;
            constexpr bool HAS_OUT = decltype(out_tag)::value, AHEAD = decltype(ahead_tag)::value;
            const uint64_t local_addr = local_of(j);
            u32x4 inc[U] = {};
            if constexpr (KIND != 0) {
                const uint64_t in_base = in0 + ((j + 1) & 1 ? parity_stride : 0);
#pragma unroll
                for (unsigned u = 0; u < U; ++u) {
                    if constexpr (KIND == 2) cur[u] = load16<false>(in_base + din[u]);
                    else inc[u] = load16<false>(in_base + din[u]);
                }
            }
            if constexpr (AHEAD) {
                const uint64_t next_addr = local_of(j + 1);
#pragma unroll
                for (unsigned u = 0; u < U; ++u) nxt[u] = load16<kNtLocalLoad>(next_addr + bu[u]);
            }
            if (HAS_OUT && j > t_first && ((out_changes >> (j - t_first)) & 1)) {
#pragma unroll
                for (unsigned u = 0; u < U; ++u) dout[u] = stage_offset(r, j, bu[u]);
            }
            const uint64_t out_base = out0 + (j & 1 ? parity_stride : 0);
#pragma unroll
            for (unsigned u = 0; u < U; ++u) {
                u32x4 v;
                if constexpr (KIND == 1) v = combine<BF16 ? kSumBF16 : kSumF32>(inc[u], cur[u]);
                else v = cur[u];
                if constexpr (KIND != 0) store16<kNtLocalStore>(local_addr + bu[u], v);
                if constexpr (HAS_OUT) store16<false>(out_base + dout[u], v);
            }
            // step j+1 reads what the predecessor stages at this step
            if (j + 1 < a.j1 && j > t_first && ((in_changes >> (j - t_first)) & 1)) {
#pragma unroll
                for (unsigned u = 0; u < U; ++u) din[u] = stage_offset(peer, j, bu[u]);
            }
            __syncthreads();  // the next step reads what other waves of this workgroup just staged
            ++j;
        };
        using Send = std::integral_constant<int, 0>;
        using Sum = std::integral_constant<int, 1>;
        using Copy = std::integral_constant<int, 2>;
        using Yes = std::integral_constant<bool, true>;
        using No = std::integral_constant<bool, false>;
        u32x4 set_a[U] = {}, set_b[U] = {};
        // The steps [j, j_end), all sums that stage onward or all sums that do not: the first loads
        // its local chunk itself, every other finds it loaded by the step before.
        auto sums = [&](auto out_tag, uint32_t j_end) {
            if (j >= j_end) return;
            const uint64_t first_addr = local_of(j);
#pragma unroll
            for (unsigned u = 0; u < U; ++u) set_a[u] = load16<kNtLocalLoad>(first_addr + bu[u]);
            for (;;) {
                if (j + 1 >= j_end) {
                    step(Sum{}, out_tag, No{}, set_a, set_b);
                    break;
                }
                step(Sum{}, out_tag, Yes{}, set_a, set_b);
                if (j + 1 >= j_end) {
                    step(Sum{}, out_tag, No{}, set_b, set_a);
                    break;
                }
                step(Sum{}, out_tag, Yes{}, set_b, set_a);
            }
        };
        auto copies = [&](auto out_tag, uint32_t j_end) {
            while (j < j_end) {
                step(Copy{}, out_tag, No{}, set_a, set_b);
                if (j >= j_end) break;
                step(Copy{}, out_tag, No{}, set_b, set_a);
            }
        };
        const uint32_t last = a.J - 1;  // the one step that stages nothing
        const uint32_t sum_end = a.sum_last + 1 < a.j1 ? a.sum_last + 1 : a.j1;  // sums are steps 1..sum_last
        if (j == 0) step(Send{}, Yes{}, No{}, pre, set_b);  // the chunk was loaded before the tables were made
        sums(Yes{}, sum_end < last ? sum_end : last);
        sums(No{}, sum_end);
        copies(Yes{}, a.j1 < last ? a.j1 : last);
        copies(No{}, a.j1);
        record_rows();
        return;
    }

    // More ranks than waves, or the chunk's last, narrower column: per-lane bounds, lookups in place.
    for (uint32_t j = a.j0; j < a.j1; ++j) {
        const bool has_in = j > 0, has_out = j + 1 < a.J;
        const bool summing = has_in && j <= a.sum_last;
        for (uint32_t rv = wave; rv < R; rv += n_waves) {
            const uint32_t r = __builtin_amdgcn_readfirstlane(rv);
            const uint32_t peer = (r + R - 1) % R;
            const uint32_t chunk = (r + a.chunk_start + 2 * R - j) % R;
            const uint64_t local_addr = a.rank_buf[r] + ((uint64_t)l * R + chunk) * a.chunk_bytes;
            const uint64_t in_base = slab_stage + ((uint64_t)((j + 1) & 1) * R + peer) * per_rank;
            const uint64_t out_base = slab_stage + ((uint64_t)(j & 1) * R + r) * per_rank;

            u32x4 inc[U] = {}, loc[U] = {};
#pragma unroll
            for (unsigned u = 0; u < U; ++u) {
                const uint64_t b = b0 + (uint64_t)(u * kWave + lane) * 16;
                if (b < b1) {
                    if (has_in) inc[u] = load16<false>(in_base + stage_offset(peer, j - 1, b));
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
                    else v = combine<BF16 ? kSumBF16 : kSumF32>(inc[u], loc[u]);
                    if (has_in) store16<kNtLocalStore>(local_addr + b, v);
                    if (has_out) store16<false>(out_base + stage_offset(r, j, b), v);
                }
            }
        }
        __syncthreads();  // the next step reads what other waves of this workgroup just staged
    }
    record_rows();
}

template <bool BF16, unsigned U>
__global__ __launch_bounds__(kMaxFusedWaves *kWave) void ring_fused_links_kernel(const FusedArgs a,
                                                                                const uint64_t link_rows)
{
    fused_links_body<BF16, U, false>(a, link_rows, nullptr);
}

static_assert(sizeof(FusedArgs) + 8 + sizeof(EpochBatch) <= 4000, "kernel arguments must fit 4 KiB");

template <bool BF16, unsigned U>
__global__ __launch_bounds__(kMaxFusedWaves *kWave) void ring_fused_links_partition_kernel(const FusedArgs a,
                                                                                          const uint64_t link_rows,
                                                                                          const EpochBatch eb)
{
    fused_links_body<BF16, U, true>(a, link_rows, &eb);
}

}  // namespace
}  // namespace r2

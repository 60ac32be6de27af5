// Bridge-based logical re-ranking of a ring (R2CCL paper, Sec. 6 "Topology-Aware Logical Re-ranking",
// Appendix D Algorithm 1).  Host-side integer work on a handful of nodes; no device code.
//
// A node's rail set is a 64-bit mask; the capacity of a ring edge is the number of rails its two
// ends share.  Edges narrower than the narrowest node (B_global) are repaired, worst first, by
// moving a "bridge" node with wide enough connectivity in between, provided that closing the gap it
// leaves behind does not create a narrow edge.
#include <algorithm>
#include <cstdint>
#include <new>
#include <vector>

#include "r2ccl.h"

namespace {

inline uint32_t shared_rails(uint64_t a, uint64_t b) { return (uint32_t)__builtin_popcountll(a & b); }

int rerank(const uint32_t *ring, const uint64_t *rails, uint32_t n, uint32_t *out_ring, uint32_t *n_relocated)
{
    std::vector<char> seen(n, 0);
    for (uint32_t i = 0; i < n; ++i) {
        if (ring[i] >= n || seen[ring[i]]) return R2_ERR_INVALID;  // must be a permutation of 0..n-1
        seen[ring[i]] = 1;
    }
    std::vector<uint32_t> cur(ring, ring + n);
    uint32_t moved = 0;

    uint32_t b_global = 65;
    for (uint32_t i = 0; i < n; ++i) b_global = std::min(b_global, (uint32_t)__builtin_popcountll(rails[i]));

    struct Cand {
        uint32_t u, v, gap;
    };
    std::vector<Cand> cands;
    for (uint32_t i = 0; i < n; ++i) {
        const uint32_t u = ring[i], v = ring[(i + 1) % n];
        const uint32_t cap = shared_rails(rails[u], rails[v]);
        if (cap < b_global) cands.push_back({u, v, b_global - cap});
    }
    // worst gap first; equal gaps keep their order round the ring
    std::stable_sort(cands.begin(), cands.end(), [](const Cand &a, const Cand &b) { return a.gap > b.gap; });

    for (const Cand &c : cands) {
        // position of u; the pair is only repaired while v still follows u
        uint32_t pu = 0;
        while (cur[pu] != c.u) ++pu;
        if (n < 3 || cur[(pu + 1) % n] != c.v) continue;
        for (uint32_t pw = 0; pw < n; ++pw) {
            const uint32_t w = cur[pw];
            if (w == c.u || w == c.v) continue;
            const uint32_t x = cur[(pw + n - 1) % n], y = cur[(pw + 1) % n];
            const uint32_t new_cap = std::min(shared_rails(rails[c.u], rails[w]), shared_rails(rails[w], rails[c.v]));
            const uint32_t removal_cap = shared_rails(rails[x], rails[y]);
            if (new_cap >= b_global && removal_cap >= b_global) {
                cur.erase(cur.begin() + pw);
                uint32_t qu = 0;
                while (cur[qu] != c.u) ++qu;
                cur.insert(cur.begin() + qu + 1, w);
                ++moved;
                break;
            }
        }
    }
    std::copy(cur.begin(), cur.end(), out_ring);
    if (n_relocated) *n_relocated = moved;
    return R2_OK;
}

}  // namespace

extern "C" int r2_bridge_rerank(const uint32_t *ring, const uint64_t *rails, uint32_t n,
                                uint32_t *out_ring, uint32_t *n_relocated)
{
    if (!ring || !rails || !out_ring || n == 0) return R2_ERR_INVALID;
    try {
        return rerank(ring, rails, n, out_ring, n_relocated);
    } catch (const std::bad_alloc &) {  // the working copies are host allocations; nothing may unwind into C
        return R2_ERR_CAPACITY;
    }
}

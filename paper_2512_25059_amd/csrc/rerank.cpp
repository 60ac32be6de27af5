// Bridge-based logical re-ranking of a ring (R2CCL paper, Sec. 6 "Topology-Aware Logical Re-ranking",
// Appendix D Algorithm 1).  Host-side integer work on a handful of nodes; no device code.
//
// A node's rail set is a 64-bit mask; the width of a ring edge is the number of rails its two ends
// share.  Edges narrower than the narrowest node are repaired, worst first, by moving a "bridge" node
// with wide enough connectivity in between, provided that closing the gap it leaves behind does not
// create a narrow edge.
//
// Layout: the ring is a doubly linked list over node ids (succ/pred arrays), so taking a bridge out
// and putting it between two neighbours is a constant number of pointer updates; the pairwise rail
// overlaps are counted once into an n x n byte matrix; the broken edges wait in one bucket per gap
// size (a gap is at most 64 rails), which gives "worst first, ties in ring order" without a sort.
#include <cstdint>
#include <new>
#include <vector>

#include "r2ccl_ext.h"

namespace {

class LinkedRing {
public:
    LinkedRing(const uint32_t *order, uint32_t n) : succ_(n), pred_(n), first_(order[0]), n_(n)
    {
        for (uint32_t i = 0; i < n; ++i) {
            const uint32_t a = order[i], b = order[(i + 1) % n];
            succ_[a] = b;
            pred_[b] = a;
        }
    }
    uint32_t first() const { return first_; }
    uint32_t after(uint32_t node) const { return succ_[node]; }
    uint32_t before(uint32_t node) const { return pred_[node]; }
    // Takes `node` out of the ring and puts it right behind `anchor`.  The walk's starting point stays
    // where it was, unless the node that moves was that point: then its successor takes over.
    void move_behind(uint32_t node, uint32_t anchor)
    {
        const uint32_t left = pred_[node], right = succ_[node];
        succ_[left] = right;
        pred_[right] = left;
        if (first_ == node) first_ = right;
        const uint32_t follower = succ_[anchor];
        succ_[anchor] = node;
        pred_[node] = anchor;
        succ_[node] = follower;
        pred_[follower] = node;
    }
    void write(uint32_t *out) const
    {
        uint32_t node = first_;
        for (uint32_t i = 0; i < n_; ++i, node = succ_[node]) out[i] = node;
    }

private:
    std::vector<uint32_t> succ_, pred_;
    uint32_t first_, n_;
};

int rerank(const uint32_t *ring, const uint64_t *rails, uint32_t n, uint32_t *out_ring, uint32_t *n_relocated)
{
    std::vector<char> seen(n, 0);
    for (uint32_t i = 0; i < n; ++i) {
        if (ring[i] >= n || seen[ring[i]]) return R2_ERR_INVALID;  // must be a permutation of 0..n-1
        seen[ring[i]] = 1;
    }

    // rails two nodes have in common, and the fewest rails any node has left
    std::vector<uint8_t> common((size_t)n * n);
    uint32_t floor_width = 64;
    for (uint32_t a = 0; a < n; ++a) {
        const uint32_t own = (uint32_t)__builtin_popcountll(rails[a]);
        if (own < floor_width) floor_width = own;
        for (uint32_t b = 0; b < n; ++b) common[(size_t)a * n + b] = (uint8_t)__builtin_popcountll(rails[a] & rails[b]);
    }
    auto wide = [&](uint32_t a, uint32_t b) { return common[(size_t)a * n + b] >= floor_width; };

    // the edges of the ring as given that are too narrow, bucketed by how many rails they lack
    struct Edge {
        uint32_t tail, head;
    };
    std::vector<std::vector<Edge>> by_gap(65);
    for (uint32_t i = 0; i < n; ++i) {
        const uint32_t a = ring[i], b = ring[(i + 1) % n];
        const uint32_t have = common[(size_t)a * n + b];
        if (have < floor_width) by_gap[floor_width - have].push_back({a, b});
    }

    LinkedRing lr(ring, n);
    uint32_t moved = 0;
    for (uint32_t gap = 64; gap >= 1 && n >= 3; --gap) {
        for (const Edge &e : by_gap[gap]) {
            if (lr.after(e.tail) != e.head) continue;  // an earlier move already separated the pair
            uint32_t w = lr.first();
            for (uint32_t seen_nodes = 0; seen_nodes < n; ++seen_nodes, w = lr.after(w)) {
                if (w == e.tail || w == e.head) continue;
                // w bridges the pair if it is wide towards both, and its own neighbours are wide
                // towards each other once it has left
                if (wide(e.tail, w) && wide(w, e.head) && wide(lr.before(w), lr.after(w))) {
                    lr.move_behind(w, e.tail);
                    ++moved;
                    break;
                }
            }
        }
    }
    lr.write(out_ring);
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

"""Oracle for the bridge-based logical re-ranking of a ring.

TEST INFRASTRUCTURE ONLY.  Written from the description in the R2CCL paper (Sec. 6,
"Topology-Aware Logical Re-ranking", and Appendix D, Algorithm 1) with plain Python sets and
lists; it shares nothing with the product's implementation.

Readings where the algorithm is silent: candidates of equal severity keep their order round the
ring; bridge nodes are tried in the ring's current order; a candidate pair whose two nodes are no
longer neighbours (an earlier relocation took one of them away) is skipped; "relocate between u
and v" puts the bridge right after u.
"""
from typing import Dict, List, Sequence, Set, Tuple


def bridge_rerank(ring: Sequence[int], rails: Dict[int, Set[int]]) -> Tuple[List[int], int]:
    """Returns (re-ranked ring, number of relocations)."""
    order = list(ring)
    n = len(order)
    narrowest = min(len(rails[node]) for node in order)

    def width(a: int, b: int) -> int:
        return len(rails[a] & rails[b])

    # neighbours whose common rails are fewer than what the narrowest node could sustain
    broken = []
    for i in range(n):
        u, v = order[i], order[(i + 1) % n]
        if width(u, v) < narrowest:
            broken.append((narrowest - width(u, v), i, u, v))
    broken.sort(key=lambda item: (-item[0], item[1]))

    relocations = 0
    for _, _, u, v in broken:
        at = order.index(u)
        if n < 3 or order[(at + 1) % n] != v:
            continue
        for w in list(order):
            if w in (u, v):
                continue
            k = order.index(w)
            before, after = order[k - 1], order[(k + 1) % n]
            fits = min(width(u, w), width(w, v)) >= narrowest
            gap_closes = width(before, after) >= narrowest
            if fits and gap_closes:
                order.remove(w)
                order.insert(order.index(u) + 1, w)
                relocations += 1
                break
    return order, relocations

"""A ring whose servers lost different rails (Sec. 6, "Topology-Aware Logical Re-ranking"): pins for
the oracle.  What the ring computes is fixed by its definition whatever the rails; with the same
rails everywhere it must be the plain ring of the C oracle byte for byte; a link carries data only
on rails both ends still have; re-ranking with a bridge node widens the narrowest link."""
import numpy as np
import pytest
import torch

import oracle as o
from oracle import rails, rerank


def _bufs(rng, R, N, dtype):
    vals = [rng.standard_normal(N).astype(np.float32) for _ in range(R)]
    if dtype == o.F32:
        return vals
    return [torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy() for v in vals]


@pytest.mark.parametrize("phases", [o.PHASE_RS, o.PHASE_AG, o.PHASE_AR])
@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_same_rails_everywhere_is_the_plain_ring(dtype, phases):
    rng = np.random.default_rng(31)
    for R, S, C, E in ((2, 1, 2, 24), (3, 2, 4, 40), (5, 1, 3, 7), (4, 3, 8, 64)):
        n_tx = S * o.num_transmissions(R, phases)
        epochs = [(0, int(rng.integers(0, (1 << C) - 1)), [int(x) for x in rng.integers(1, 100, C)])]
        for t in sorted(set(int(x) for x in rng.integers(1, n_tx + 1, 2))):  # a schedule that changes on the way
            epochs.append((t, int(rng.integers(0, (1 << C) - 1)), [int(x) for x in rng.integers(1, 100, C)]))
        a = _bufs(rng, R, S * R * E, dtype)
        b = [x.copy() for x in a]
        cap = (E * a[0].itemsize + 255) // 256 * 256
        log, stage_c = o.ring_sim(a, dtype, S, C, 16, epochs, phases, cap)
        tables, stage_p = rails.ring_rails_sim(b, dtype, S, C, 16, [epochs] * R, phases)
        for r in range(R):
            assert a[r].tobytes() == b[r].tobytes()
            assert tables[r].tolist() == log.tolist()
        assert stage_c.tobytes() == stage_p.tobytes()


@pytest.mark.parametrize("phases", [o.PHASE_RS, o.PHASE_AG, o.PHASE_AR])
@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_result_does_not_depend_on_the_rails(dtype, phases):
    rng = np.random.default_rng(32)
    for _ in range(12):
        R, S, C = int(rng.integers(2, 7)), int(rng.integers(1, 4)), int(rng.integers(2, 8))
        E = int(rng.integers(1, 80))
        w = [int(x) for x in rng.integers(1, 100, C)]
        keep_up = int(rng.integers(0, C))  # one rail survives everywhere, so every link has a channel
        masks = [int(rng.integers(0, 1 << C)) & ~(1 << keep_up) for _ in range(R)]
        bufs = _bufs(rng, R, S * R * E, dtype)
        keep = [x.copy() for x in bufs]
        tables, stage = rails.ring_rails_sim(bufs, dtype, S, C, 16, rails.static_epochs(w, masks), phases)
        want = o.expected(keep, dtype, S, phases)
        for r in range(R):
            assert bufs[r].tobytes() == want[r].tobytes()
        nbytes = E * bufs[0].itemsize
        for r in range(R):
            m = masks[r] | masks[(r + 1) % R]
            for row in tables[r]:
                assert row.tolist() == o.partition(w, m, nbytes, 16).tolist()
            for c in range(C):
                if (m >> c) & 1:  # down at either end: the link puts nothing on it, in any step or slab
                    assert np.all(tables[r][:, c + 1] == tables[r][:, c])
                    assert np.all(stage[:, r, :, c] == 0xA5)


def test_last_transmission_of_every_rank_reassembles_to_what_it_holds():
    """After an all-reduce the last chunk a rank staged (step 2R-3) is the finished chunk it also keeps;
    its slices, cut by its own link's table, put back in channel order, are that chunk."""
    rng = np.random.default_rng(33)
    R, S, C, E = 4, 2, 4, 24
    w, masks = [3, 1, 4, 1], [0b0001, 0b0010, 0, 0b1000]
    bufs = _bufs(rng, R, S * R * E, o.F32)
    tables, stage = rails.ring_rails_sim(bufs, o.F32, S, C, 16, rails.static_epochs(w, masks), o.PHASE_AR)
    j = 2 * R - 3
    for l in range(S):
        for r in range(R):
            c = (r - j) % R
            raw = bufs[r][(l * R + c) * E:(l * R + c + 1) * E].tobytes()
            row = tables[r][l * (2 * R - 2) + j]
            got = b"".join(stage[j & 1, r, l, k, : int(row[k + 1] - row[k])].tobytes() for k in range(C))
            assert got == raw


def test_a_failure_at_one_server_changes_its_two_links_from_then_on():
    """Sec. 5.1 is per server: server 2 loses NIC 1 at transmission 3 and gets it back, slower, at 6.
    Only the links 1 -> 2 and 2 -> 3 change, only from transmission 3 on, and a channel is as fast as
    the slower of its two ends.  By hand for 64-byte chunks, 4 channels, alignment 16."""
    R, S, C, E = 4, 2, 4, 16
    w = [1, 1, 1, 1]
    sched = [[(0, 0, w)] for _ in range(R)]
    sched[2] = [(0, 0, w), (3, 0b0010, w), (6, 0, [1, 3, 1, 1])]
    rng = np.random.default_rng(36)
    bufs = _bufs(rng, R, S * R * E, o.F32)
    keep = [b.copy() for b in bufs]
    tables, _ = rails.ring_rails_sim(bufs, o.F32, S, C, 16, sched, o.PHASE_AR)
    assert [b.tobytes() for b in bufs] == [x.tobytes() for x in o.expected(keep, o.F32, S, o.PHASE_AR)]
    quarters, thirds = [0, 16, 32, 48, 64], [0, 16, 16, 32, 64]  # 4 units over 4 channels / over 3: 1, 1, 2
    for r in range(R):
        for t in range(S * 6):
            touches = r in (1, 2)
            want = thirds if touches and 3 <= t < 6 else quarters  # min(1, 3) = 1: back to quarters at 6
            assert tables[r, t].tolist() == want, (r, t)
    # the other way round: a faster NIC at one end only does not speed the link up; at both ends it does
    sched[3] = [(0, 0, w), (6, 0, [1, 3, 1, 1])]
    assert rails.link_state(sched, 2, 7) == (0, [1, 3, 1, 1])
    assert rails.link_state(sched, 1, 7) == (0, [1, 1, 1, 1])
    assert rails.link_tables(sched, 12, 96, 16)[2, 7].tolist() == [0, 16, 64, 80, 96]  # 6 units: 1, 3, 1, 1


def test_link_bandwidth_by_hand():
    w = [10, 20, 30, 40]
    masks = [0b0001, 0b0010, 0, 0b1100]
    assert rails.link_masks(masks) == [0b0011, 0b0010, 0b1100, 0b1101]
    assert rails.link_bandwidth(w, masks) == [70, 80, 30, 20]
    assert rails.ring_bandwidth(w, masks) == 20


def test_bridge_reranking_widens_the_narrowest_link():
    """The paper's scenario: neighbours A and B lose different rails, C and D are healthy.  In the order
    A B C D the link A-B is left with the rails both still have; with a healthy node moved between
    them every link has as many rails as the narrowest node."""
    w = [1, 1]
    masks = {0: 0b01, 1: 0b10, 2: 0, 3: 0}  # A lost rail 0, B lost rail 1
    ring = [0, 1, 2, 3]
    with pytest.raises(o.NoHealthyChannel):
        rails.link_tables(rails.static_epochs(w, [masks[n] for n in ring]), 1, 64, 16)
    assert rails.ring_bandwidth(w, [masks[n] for n in ring]) == 0
    alive = {n: {c for c in range(2) if not (m >> c) & 1} for n, m in masks.items()}
    order, moved = rerank.bridge_rerank(ring, alive)
    assert moved == 1 and sorted(order) == ring
    assert rails.ring_bandwidth(w, [masks[n] for n in order]) == 1  # = what A or B alone could sustain
    # and the re-ranked ring still computes the all-reduce, rank for rank
    rng = np.random.default_rng(34)
    xs = _bufs(rng, 4, 4 * 16, o.BF16)
    by_node = {n: xs[n] for n in ring}
    bufs = [by_node[n].copy() for n in order]
    rails.ring_rails_sim(bufs, o.BF16, 1, 2, 16, rails.static_epochs(w, [masks[n] for n in order]), o.PHASE_AR)
    want = o.expected([by_node[n] for n in order], o.BF16, 1, o.PHASE_AR)
    for i in range(4):
        assert bufs[i].tobytes() == want[i].tobytes()


def test_reranking_never_narrows_the_ring_on_random_failures():
    rng = np.random.default_rng(35)
    improved = 0
    for _ in range(300):
        n, C = int(rng.integers(3, 9)), int(rng.integers(2, 6))
        masks = [int(rng.integers(0, 1 << C)) if rng.random() < 0.5 else 0 for _ in range(n)]
        masks = [m if m != (1 << C) - 1 else 0 for m in masks]  # every node keeps a rail
        alive = {i: {c for c in range(C) if not (masks[i] >> c) & 1} for i in range(n)}
        order, _ = rerank.bridge_rerank(list(range(n)), alive)
        before = rails.ring_bandwidth([1] * C, masks)
        after = rails.ring_bandwidth([1] * C, [masks[i] for i in order])
        assert after >= before
        improved += after > before
    assert improved > 10

"""Point-to-point under R2CCL-Balance (Sec. 5.1; Sec. 8 / Appendix E): pins for the oracle.
The definition is fixed by what a send/receive is: the receiver ends with the sender's bytes,
whatever the channel schedule; the stage slices hold exactly the sender's bytes, cut at the table."""
import numpy as np
import pytest

import oracle as o
from oracle import sendrecv as sr


def _bufs(rng, R, N, dtype):
    if dtype == o.F32:
        return [rng.standard_normal(N).astype(np.float32) for _ in range(R)]
    return [rng.integers(0, 1 << 16, N).astype(np.uint16) for _ in range(R)]


@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_receiver_gets_the_senders_bytes_under_any_schedule(dtype):
    rng = np.random.default_rng(11)
    for _ in range(30):
        R, S, C = int(rng.integers(2, 6)), int(rng.integers(1, 7)), int(rng.integers(1, 7))
        E = int(rng.integers(1, 200))
        w = [int(x) for x in rng.integers(1, 100, C)]
        epochs = [(0, 0, w)]
        for t in sorted(set(int(x) for x in rng.integers(1, S + 1, 3))):
            mask = int(rng.integers(0, (1 << C) - 1))  # never all failed
            epochs.append((t, mask, [int(x) for x in rng.integers(1, 100, C)]))
        send = _bufs(rng, R, S * E, dtype)
        recv = [np.zeros_like(x) for x in send]
        keep = [x.copy() for x in send]
        log, stage = sr.sendrecv_sim(send, recv, dtype, S, C, 16, epochs)
        want = sr.sendrecv_expected(keep)
        for r in range(R):
            assert recv[r].tobytes() == want[r].tobytes()
            assert send[r].tobytes() == keep[r].tobytes()  # the send buffers are only read
        # each chunk's table is the partition under the state in force at its transmission
        nbytes = E * send[0].itemsize
        for l in range(S):
            _, mask, ws = sr.state_at(epochs, l)
            assert log[l].tolist() == o.partition(ws, mask, nbytes, 16).tolist()
            # the slices, put back in channel order, are the chunk; bytes beyond a slice are untouched
            for r in range(R):
                raw = keep[r][l * E:(l + 1) * E].tobytes()
                got = b"".join(stage[r, l, c, : int(log[l][c + 1] - log[l][c])].tobytes() for c in range(C))
                assert got == raw
                for c in range(C):
                    assert np.all(stage[r, l, c, int(log[l][c + 1] - log[l][c]):] == 0xA5)
                    if (mask >> c) & 1:
                        assert log[l][c + 1] == log[l][c]  # a failed channel carries nothing


def test_state_at():
    ep = [(0, 0, [1]), (3, 1, [1]), (7, 0, [1])]
    assert [sr.state_at(ep, t)[1] for t in (0, 2, 3, 6, 7, 100)] == [0, 0, 1, 1, 0, 0]

"""GPU parity: point-to-point through the partitioned stage buffers (R2_PHASE_SENDRECV) vs the oracle,
byte for byte: receive buffers, offsets log, stage area."""
import numpy as np
import pytest
import torch

from gpu_util import FILL, assert_same_stage, say
from oracle import sendrecv as sr

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _dev(a):
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


def _run(r2, oracle, send, dtype, S, C, align, epochs, window=0, check_stage=True):
    R, N = len(send), send[0].size
    gdt = r2.F32 if dtype == "f32" else r2.BF16
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    desc = r2.SimDesc(R, S, C, align, N, gdt, r2.PHASE_SENDRECV, window, 0)
    assert r2.r2_sim_num_steps(desc) == 2 and r2.r2_sim_num_transmissions(desc) == S
    need = r2.r2_sim_workspace_bytes(desc)
    ws = torch.full((need,), FILL, dtype=torch.uint8, device="cuda")
    log = torch.full((S, C + 1), -1, dtype=torch.int64, device="cuda")
    sb = [_dev(x) for x in send]
    rb = [torch.zeros_like(t) for t in sb]
    r2.r2_sendrecv_sim(desc, sb, rb, epochs, ws, log)
    torch.cuda.synchronize()
    o_recv = [np.zeros_like(x) for x in send]
    o_log, o_stage = sr.sendrecv_sim(send, o_recv, odt, S, C, align, epochs)
    want = sr.sendrecv_expected(send)
    for r in range(R):
        got = rb[r].cpu().numpy().view(send[r].dtype)
        assert got.tobytes() == want[r].tobytes(), f"rank {r} vs definition"
        assert got.tobytes() == o_recv[r].tobytes(), f"rank {r} vs step-by-step oracle"
        assert sb[r].cpu().numpy().view(send[r].dtype).tobytes() == send[r].tobytes(), "send buffer changed"
    assert log.cpu().numpy().view(np.uint64).tolist() == o_log.tolist()
    if check_stage:
        cap = r2.r2_sim_stage_capacity(desc)
        off = r2.r2_sim_stage_offset(desc)
        st = ws[off:off + 2 * R * S * C * cap].cpu().numpy().reshape(2, R, S, C, cap)
        assert_same_stage(st[0], o_stage, "stage area (parity 0)")
        assert np.all(st[1] == FILL), "parity 1 is never used by a two-step exchange"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sendrecv_small(r2, oracle, dtype):
    rng = np.random.default_rng(700)
    per16 = 4 if dtype == "f32" else 8
    w = [50000] * 8
    for R, S, E in ((2, 1, per16 * 100), (4, 5, per16 * 1031), (8, 3, 7), (3, 2, per16 * 512 * 9 + 3)):
        N = S * E
        say(f"sendrecv {dtype} R={R} S={S} N={N}")
        send = [rng.integers(0, 1 << 16, N).astype(np.uint16) if dtype == "bf16"
                else rng.standard_normal(N).astype(np.float32) for _ in range(R)]
        epochs = [(0, 0, w), (1, 0b00100100, w), (3, 0b1, [1, 2, 3, 4, 5, 6, 7, 8])]
        _run(r2, oracle, send, dtype, S, 8, 256, epochs)


def test_sendrecv_large_with_passes(r2, oracle):
    """Chunks of 8 MiB per rank, a stage window that forces byte-range passes, a channel that fails
    after the second chunk."""
    rng = np.random.default_rng(701)
    R, S, C = 4, 4, 8
    N = S * (2 << 20)  # fp32: 8 MiB per chunk
    send = [rng.standard_normal(N).astype(np.float32) for _ in range(R)]
    w = [50000] * C
    epochs = [(0, 0, w), (2, 0b00001000, w)]
    say(f"sendrecv large R={R} S={S} N={N} window=16MiB")
    _run(r2, oracle, send, "f32", S, C, 256, epochs, window=16 << 20, check_stage=False)
    say("sendrecv large, default window")
    _run(r2, oracle, send, "f32", S, C, 256, epochs)


def test_sendrecv_argument_errors(r2):
    desc = r2.SimDesc(4, 2, 8, 256, 2 * 64, r2.F32, r2.PHASE_SENDRECV, 0, 0)
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    sb = [torch.ones(128, dtype=torch.float32, device="cuda") for _ in range(4)]
    rb = [torch.zeros(128, dtype=torch.float32, device="cuda") for _ in range(4)]
    w = [1] * 8
    with pytest.raises(r2.R2Error):  # wrong phase
        r2.r2_sendrecv_sim(r2.SimDesc(4, 2, 8, 256, 128, r2.F32, r2.PHASE_AR, 0, 0), sb, rb, [(0, 0, w)], ws)
    with pytest.raises(r2.R2Error):  # in place
        r2.r2_sendrecv_sim(desc, sb, [sb[1], rb[1], rb[2], rb[3]], [(0, 0, w)], ws)
    with pytest.raises(r2.R2Error) as e:  # every channel down for chunk 1
        r2.r2_sendrecv_sim(desc, sb, rb, [(0, 0, w), (1, 0xFF, w)], ws)
    assert e.value.code == -2
    assert r2.r2_sim_num_steps(r2.SimDesc(4, 2, 8, 256, 128, r2.F32, r2.PHASE_SENDRECV, 0, r2.SCHED_FUSED)) == 0
    assert r2.r2_sim_num_steps(r2.SimDesc(4, 3, 8, 256, 128, r2.F32, r2.PHASE_SENDRECV, 0, 0)) == 0  # 128 % 3
    with pytest.raises(r2.R2Error):  # the fused entry point does not run it
        r2.r2_sim_fused_steps(desc, sb + rb, 0, 2, ws)
    torch.cuda.synchronize()
    assert all(float(t.sum()) == 0.0 for t in rb)  # nothing ran


@pytest.mark.parametrize("seed", [1, 2])
def test_sendrecv_random_configurations(r2, oracle, seed):
    """Random ring sizes, chunk counts and sizes (ragged included), channel counts, alignments, pass windows
    and channel states that change between chunks."""
    rng = np.random.default_rng(800 + seed)
    for case in range(20):
        R, S, C = int(rng.integers(2, 17)), int(rng.integers(1, 9)), int(rng.integers(1, 13))
        dtype = "f32" if rng.random() < 0.5 else "bf16"
        es = 4 if dtype == "f32" else 2
        E = int(rng.integers(1, 5000))
        align = (16, 64, 256)[int(rng.integers(0, 3))]
        eps, t0 = [], 0
        while t0 < S:
            mask = int(rng.integers(0, (1 << C) - 1)) if C > 1 else 0
            eps.append((t0, mask, [int(x) for x in rng.integers(1, 60000, C)]))
            t0 += int(rng.integers(1, S + 1))
        window = 0 if rng.random() < 0.5 else int(rng.integers(1, 6)) * R * E * es // 2 + 256
        send = [rng.integers(0, 1 << 16, S * E).astype(np.uint16) if dtype == "bf16"
                else rng.standard_normal(S * E).astype(np.float32) for _ in range(R)]
        say(f"sendrecv random {seed}.{case} {dtype} R={R} S={S} C={C} E={E} align={align} window={window} epochs={len(eps)}")
        _run(r2, oracle, send, dtype, S, C, align, eps, window=window, check_stage=window == 0 or len(eps) == 1)

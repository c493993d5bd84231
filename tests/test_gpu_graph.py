"""The decode call (split + merge launches) recorded into a HIP graph and replayed: the library
enqueues kernels only (no allocation, no synchronisation, no memset), so for a fixed cache state a
serving loop can replay the call with new queries.  Every replay is checked against the eager call
and the oracle, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2506_04642_amd import synth
from parity_util import ATTN_TOL, append_both, make_pair, to_dev

pytestmark = pytest.mark.gpu

BF16 = 1
CHAN, CROSS = 0, 1


@pytest.fixture(scope="module")
def kv():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_04642_amd import binding

    return binding


@pytest.mark.parametrize("mode,bits", [(CHAN, 4), (CHAN, 2), (CROSS, 8)])
def test_decode_call_replayed_from_a_graph(kv, oracle, mode, bits):
    import torch

    print("case graph mode=%d bits=%d" % (mode, bits), flush=True)
    B, Hq, Hkv, T = 2, 8, 2, 2048 + 11
    gpu, orc = make_pair(kv, oracle, B=B, Hq=Hq, Hkv=Hkv, T_max=2048 + 64, dtype=BF16, mode=mode, k_bits=(bits,))
    k, v = synth.make_kv(1500 + bits, B, T, Hkv, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16)
    q_static = to_dev(synth.make_q(1, B, Hq, 128, BF16), BF16)
    out_static = torch.zeros((B, Hq, 128), dtype=torch.float32, device="cuda:0")
    gpu.attend(0, q_static, out=out_static)  # warm-up: one-time occupancy queries happen outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        gpu.attend(0, q_static, out=out_static)
    torch.cuda.synchronize()
    for rep in range(4):
        q = synth.make_q(10 + rep, B, Hq, 128, BF16)
        qd = to_dev(q, BF16)
        eager = gpu.attend(0, qd).clone()  # eager work between the replays
        torch.cuda.synchronize()
        q_static.copy_(qd)
        out_static.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_static, eager), "replay %d differs from the eager call" % rep
        err = float(np.max(np.abs(out_static.cpu().numpy().astype(np.float64) - orc.attend(0, q))))
        assert err <= ATTN_TOL, (rep, err)


def test_calls_on_a_stream_of_their_own(kv, oracle):
    """The library enqueues on the stream it is given: the same calls on a side stream give the
    same cache bytes and outputs as on the default stream."""
    import torch

    from parity_util import check_bytes

    print("case side stream", flush=True)
    B, Hq, Hkv, T = 2, 8, 2, 700
    gpu, orc = make_pair(kv, oracle, B=B, Hq=Hq, Hkv=Hkv, T_max=1024, dtype=BF16, mode=CHAN, k_bits=(4,))
    k, v = synth.make_kv(1700, B, T, Hkv, 128, BF16)
    kd, vd = to_dev(k, BF16), to_dev(v, BF16)
    q = synth.make_q(1701, B, Hq, 128, BF16)
    qd = to_dev(q, BF16)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        gpu.append(0, kd[:, :T - 1], vd[:, :T - 1])
        out = gpu.append_attend(0, kd[:, T - 1:], vd[:, T - 1:], qd)
    side.synchronize()
    orc.append(0, k, v)
    check_bytes(gpu, orc, 0)
    err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - orc.attend(0, q))))
    assert err <= ATTN_TOL

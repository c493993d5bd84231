"""The decode call (split + merge launches) recorded into a HIP graph and replayed: the library
enqueues kernels only (no allocation, no synchronisation, no memset), so for a fixed cache state a
serving loop can replay the call with new queries.  Every replay is checked against the eager call
and the oracle, with eager work and synchronisations between the replays.  With the lengths on the
device (kv_decode_step_dev) one recording replays whole decode steps while the cache grows."""
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


@pytest.mark.parametrize("mode,Hkv,G", [(CHAN, 2, 32), (2, 2, 32), (CROSS, 4, 32), (CROSS, 8, 32), (CHAN, 2, 64), (CROSS, 8, 128),
                                        (2, 2, 128)],
                         ids=["channel_mean", "no_mean", "cross_head_4", "cross_head_8", "channel_mean_g64", "cross_head_8_g128",
                              "no_mean_g128"])
def test_growing_decode_loop_replayed_from_one_graph(kv, oracle, mode, Hkv, G):
    """Two layers (4- and 2-bit), three sequences of different lengths: one recording of
    kv_decode_step_dev per layer is replayed for 40 steps or more, across at least one block flush of
    every sequence; every step's output equals that of the eager one-call step on a twin cache, bit for
    bit, and the oracle's within the tolerance; at the end the descriptor catches up and the cache's
    bytes are the oracle's."""
    import torch

    print("case graph_steps mode=%d Hkv=%d G=%d" % (mode, Hkv, G), flush=True)
    B, Hq, steps = 3, 8, max(40, G + 12)
    bits = (4, 2)
    # sequence 0 fills its raw buffer on the second step (and once more G steps later), sequence 1 on step 14
    prompts = [5 * G + G - 2, G - 15, 2 * G + 3]
    mk = lambda: make_pair(kv, oracle, L=2, B=B, Hq=Hq, Hkv=Hkv, T_max=12 * G, G=G, Gc=G, dtype=BF16, mode=mode, k_bits=bits)
    gpu, orc = mk()
    twin, _ = mk()
    warm, _ = mk()
    for c in (gpu, twin, warm):
        kv.kv_set_decode_path(c.handle, 2)
        # a recorded step keeps the split count it was planned with while the eager call plans anew as
        # the cache grows: pinned, so that the two sum in the same order
        kv.kv_set_decode_splits(c.handle, 2)
    for l in range(2):
        for b, n in enumerate(prompts):
            k, v = synth.make_kv(2000 + 10 * l + b, 1, n, Hkv, 128, BF16)
            for c in (gpu, twin, warm):
                c.append_seq(l, b, to_dev(k[0], BF16), to_dev(v[0], BF16))
            orc.append_seq(l, b, k[0], v[0])
    ks, vs = synth.make_kv(2100, B, steps, Hkv, 128, BF16)
    kd, vd = to_dev(ks, BF16), to_dev(vs, BF16)
    k_st = [torch.zeros((B, Hkv, 128), dtype=torch.bfloat16, device="cuda:0") for _ in range(2)]
    v_st = [torch.zeros_like(k_st[0]) for _ in range(2)]
    q_st = [torch.zeros((B, Hq, 128), dtype=torch.bfloat16, device="cuda:0") for _ in range(2)]
    o_st = [torch.zeros((B, Hq, 128), dtype=torch.float32, device="cuda:0") for _ in range(2)]
    # one-time queries (occupancy, attributes) happen outside the capture: a step on a throwaway cache
    warm.lengths_to_device()
    for l in range(2):
        warm.step_dev(l, k_st[l], v_st[l], q_st[l], o_st[l])
    torch.cuda.synchronize()
    gpu.lengths_to_device()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        for l in range(2):
            gpu.step_dev(l, k_st[l], v_st[l], q_st[l], o_st[l])
    torch.cuda.synchronize()
    assert gpu.lengths(0, 0) == (5 * G, G - 2)  # the recording enqueued nothing yet and the descriptor stays behind
    for s in range(steps):
        qs = [synth.make_q(2200 + 2 * s + l, B, Hq, 128, BF16) for l in range(2)]
        for l in range(2):
            k_st[l].copy_(kd[:, s])
            v_st[l].copy_(vd[:, s])
            q_st[l].copy_(to_dev(qs[l], BF16))
            o_st[l].zero_()
        graph.replay()
        eager = [twin.append_attend(l, kd[:, s:s + 1], vd[:, s:s + 1], to_dev(qs[l], BF16)) for l in range(2)]  # eager work between the replays
        torch.cuda.synchronize()
        for l in range(2):
            assert torch.equal(o_st[l], eager[l]), "step %d layer %d differs from the eager step" % (s, l)
            orc.append(l, ks[:, s:s + 1], vs[:, s:s + 1])
            if s % 7 == 0 or s == steps - 1:
                err = float(np.max(np.abs(o_st[l].cpu().numpy().astype(np.float64) - orc.attend(l, qs[l]))))
                assert err <= ATTN_TOL, (s, l, err)
    gpu.advance(steps)
    for l in range(2):
        for b in range(B):
            assert gpu.lengths(l, b) == twin.lengths(l, b) == (orc.packed_len(l, b), orc.resid_len(l, b))
    # the cache holds the oracle's bytes, and the descriptor is good for the ordinary calls again
    for l in range(2):
        img = orc.layer_image(l)
        m = img["valid"]
        for c in (gpu, twin):
            got = c.layers[l].cpu().numpy()
            bad = np.flatnonzero(got[m] != img["bytes"][m])
            assert bad.size == 0, "layer %d: first differing valid byte at offset %d (%d differ)" % (l, np.flatnonzero(m)[bad[0]], bad.size)
        q = to_dev(synth.make_q(2300 + l, B, Hq, 128, BF16), BF16)
        assert torch.equal(gpu.attend(l, q), twin.attend(l, q))


def test_device_length_steps_stop_at_capacity(kv, oracle):
    """A sequence that has no room for another token keeps its state: the step attends over what is
    cached (the eager call would refuse the whole step with KV_E_CAPACITY), and kv_cache_advance
    follows the same rule."""
    import torch

    print("case graph_steps_capacity", flush=True)
    B, Hq, Hkv, G = 2, 8, 2, 32
    gpu, orc = make_pair(kv, oracle, B=B, Hq=Hq, Hkv=Hkv, T_max=2 * G, dtype=BF16, mode=CHAN, k_bits=(4,))
    kv.kv_set_decode_path(gpu.handle, 2)
    k, v = synth.make_kv(2500, B, 2 * G + 4, Hkv, 128, BF16)
    kd, vd = to_dev(k, BF16), to_dev(v, BF16)
    for b, n in enumerate((G + 28, 9)):  # sequence 0 is four tokens short of its capacity
        gpu.append_seq(0, b, kd[b, :n], vd[b, :n])
        orc.append_seq(0, b, k[b, :n], v[b, :n])
    gpu.lengths_to_device()
    out = torch.zeros((B, Hq, 128), dtype=torch.float32, device="cuda:0")
    for s in range(7):
        q = synth.make_q(2600 + s, B, Hq, 128, BF16)
        gpu.step_dev(0, kd[:, G + 28 + s], vd[:, G + 28 + s], to_dev(q, BF16), out)
        torch.cuda.synchronize()
        for b, n0 in enumerate((G + 28, 9)):
            if n0 + s + 1 <= 2 * G:
                t = G + 28 + s
                orc.append_seq(0, b, k[b, t:t + 1], v[b, t:t + 1])
        err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - orc.attend(0, q))))
        assert err <= ATTN_TOL, (s, err)
    gpu.advance(7)
    assert gpu.lengths(0, 0) == (2 * G, 0) == (orc.packed_len(0, 0), orc.resid_len(0, 0))
    assert gpu.lengths(0, 1) == (0, 16) == (orc.packed_len(0, 1), orc.resid_len(0, 1))
    with pytest.raises(kv.KVError) as e:
        gpu.append(0, kd[:, :1], vd[:, :1])
    assert e.value.status == kv.KV_E_CAPACITY

"""GPU parity with sequences of different lengths (requests joining and leaving slots of the
batch): cache bytes bit for bit, attention within 2e-3, against the CPU oracle."""
import numpy as np
import pytest

from paper_2506_04642_amd import synth
import parity_util
from parity_util import ATTN_TOL, check_bytes, make_pair, to_dev

pytestmark = pytest.mark.gpu

F16, BF16 = 0, 1
CHAN, CROSS, NONE = 0, 1, 2


@pytest.fixture(scope="module")
def kv():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_04642_amd import binding

    return binding


def check_lengths(gpu, orc, layer, B):
    for b in range(B):
        assert gpu.lengths(layer, b) == (orc.packed_len(layer, b), orc.resid_len(layer, b)), b


def check_attend(gpu, orc, layer, q, dtype):
    import torch

    out = gpu.attend(layer, to_dev(q, dtype))
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    want = orc.attend(layer, q)
    assert np.all(np.isfinite(got))
    err = float(np.max(np.abs(got - want)))
    assert err <= ATTN_TOL, "attention max-abs error %.3e" % err


@pytest.mark.parametrize("path", [0, 1, 2], ids=["auto", "valu", "mfma"])
@pytest.mark.parametrize("bits,G,mode,Hkv", [(4, 32, CHAN, 2), (2, 64, CHAN, 2), (8, 32, NONE, 2), (4, 32, CROSS, 2),
                                              (4, 128, CHAN, 2), (2, 128, NONE, 2), (8, 128, CROSS, 2),
                                              # a multiple of 4 kv heads: the cross-head mean's terms inside the matrix-core kernel
                                              (2, 32, CROSS, 8), (4, 64, CROSS, 8), (8, 64, CROSS, 4), (4, 128, CROSS, 8),
                                              (2, 128, CROSS, 4)])
def test_requests_join_step_and_leave(kv, oracle, path, bits, G, mode, Hkv):
    """Four slots: prompts of different lengths enter one by one (one slot stays empty at first),
    everybody decodes for a while through the one-call step, one request leaves and a new one
    takes its slot, decoding goes on."""
    import torch

    print("case ragged path=%d bits=%d G=%d mode=%d Hkv=%d" % (path, bits, G, mode, Hkv), flush=True)
    parity_util.DECODE_PATH = path
    try:
        B, g, R = 4, 4, G
        T_max = 12 * G
        gpu, orc = make_pair(kv, oracle, B=B, Hq=Hkv * g, Hkv=Hkv, T_max=T_max, G=G, Gc=G, R=R, dtype=BF16, mode=mode,
                             k_bits=(bits,))
        prompts = {0: 5 * G + 3, 1: 17, 3: 2 * G + G - 2}
        seed = 600 + bits + G
        for b, n in prompts.items():
            k, v = synth.make_kv(seed + b, 1, n, Hkv, 128, BF16)
            gpu.append_seq(0, b, to_dev(k[0], BF16), to_dev(v[0], BF16))
            orc.append_seq(0, b, k[0], v[0])
        check_lengths(gpu, orc, 0, B)
        with pytest.raises(kv.KVError) as e:
            gpu.lengths(0)
        assert e.value.status == kv.KV_E_UNSUPPORTED
        check_bytes_ragged(gpu, orc, 0)
        check_attend(gpu, orc, 0, synth.make_q(seed, B, Hkv * g, 128, BF16), BF16)  # slot 2 is empty: zeros

        steps = G + 5
        ks, vs = synth.make_kv(seed + 50, B, 2 * steps, Hkv, 128, BF16)
        kd, vd = to_dev(ks, BF16), to_dev(vs, BF16)
        for s in range(steps):
            q = synth.make_q(seed * 7 + s, B, Hkv * g, 128, BF16)
            out = gpu.append_attend(0, kd[:, s:s + 1], vd[:, s:s + 1], to_dev(q, BF16))
            orc.append(0, ks[:, s:s + 1], vs[:, s:s + 1])
            torch.cuda.synchronize()
            check_lengths(gpu, orc, 0, B)
            err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - orc.attend(0, q))))
            assert err <= ATTN_TOL, "step %d: %.3e" % (s, err)
        check_bytes_ragged(gpu, orc, 0)

        # request 0 leaves, a new prompt takes its slot; two-call steps from here on
        kv.kv_cache_reset_seq(gpu.handle, 0, 0)
        orc.reset_seq(0, 0)
        k, v = synth.make_kv(seed + 90, 1, G + 9, Hkv, 128, BF16)
        gpu.append_seq(0, 0, to_dev(k[0], BF16), to_dev(v[0], BF16))
        orc.append_seq(0, 0, k[0], v[0])
        for s in range(steps, steps + 4):
            gpu.append(0, kd[:, s:s + 1], vd[:, s:s + 1])
            orc.append(0, ks[:, s:s + 1], vs[:, s:s + 1])
            check_attend(gpu, orc, 0, synth.make_q(seed * 11 + s, B, Hkv * g, 128, BF16), BF16)
        check_lengths(gpu, orc, 0, B)
        check_bytes_ragged(gpu, orc, 0)
    finally:
        parity_util.DECODE_PATH = 0


def check_bytes_ragged(gpu, orc, layer):
    import torch

    torch.cuda.synchronize()
    img = orc.layer_image(layer)
    got = gpu.layers[layer].cpu().numpy()
    m = img["valid"]
    bad = np.flatnonzero(got[m] != img["bytes"][m])
    assert bad.size == 0, "first differing valid byte at offset %d (%d differ)" % (np.flatnonzero(m)[bad[0]], bad.size)


def test_bulk_append_with_unequal_lengths_and_errors(kv, oracle):
    """A batch-wide bulk append on sequences that already differ (runs of equal state share a
    launch), capacity checked for every sequence before anything is enqueued."""
    import torch

    print("case ragged bulk", flush=True)
    B, Hkv, G = 5, 2, 32
    gpu, orc = make_pair(kv, oracle, B=B, Hq=4, Hkv=Hkv, T_max=8 * G, G=G, Gc=G, dtype=F16, k_bits=(4,), v_bits=(2,))
    for b, n in ((1, 40), (2, 40), (4, 7)):
        k, v = synth.make_kv(700 + b, 1, n, Hkv, 128, F16)
        gpu.append_seq(0, b, to_dev(k[0], F16), to_dev(v[0], F16))
        orc.append_seq(0, b, k[0], v[0])
    k, v = synth.make_kv(710, B, 3 * G + 11, Hkv, 128, F16)
    gpu.append(0, to_dev(k, F16), to_dev(v, F16))
    orc.append(0, k, v)
    check_lengths(gpu, orc, 0, B)
    check_bytes_ragged(gpu, orc, 0)
    check_attend(gpu, orc, 0, synth.make_q(7, B, 4, 128, F16), F16)
    # the longest sequence has 40 + 107 = 147 tokens; 110 more would overflow 256 for it only
    big = torch.zeros((B, 110, Hkv, 128), dtype=torch.float16, device="cuda:0")
    with pytest.raises(kv.KVError) as e:
        gpu.append(0, big, big)
    assert e.value.status == kv.KV_E_CAPACITY
    check_lengths(gpu, orc, 0, B)
    for bad_seq in (-1, B):
        with pytest.raises(kv.KVError) as e:
            kv.kv_cache_reset_seq(gpu.handle, 0, bad_seq)
        assert e.value.status == kv.KV_E_BAD_CONFIG
        with pytest.raises(kv.KVError) as e:
            gpu.lengths(0, bad_seq)
        assert e.value.status == kv.KV_E_BAD_CONFIG


def test_many_sequences_of_different_lengths(kv, oracle):
    """200 slots with prompts of 0 .. 3 blocks plus a tail: more sequences than the first version of
    the length table held (64); batch-wide decode steps afterwards."""
    import torch

    print("case ragged 200 sequences", flush=True)
    B, Hkv, g, G = 200, 1, 4, 32
    gpu, orc = make_pair(kv, oracle, B=B, Hq=Hkv * g, Hkv=Hkv, T_max=6 * G, G=G, Gc=G, R=G, dtype=BF16, mode=CHAN,
                         k_bits=(4,))
    rng = np.random.default_rng(99)
    for b in range(B):
        n = int(rng.integers(0, 3 * G + 20))
        if b % 17 == 5 or n == 0:
            continue  # empty slots among the others
        k, v = synth.make_kv(9000 + b, 1, n, Hkv, 128, BF16)
        gpu.append_seq(0, b, to_dev(k[0], BF16), to_dev(v[0], BF16))
        orc.append_seq(0, b, k[0], v[0])
    check_lengths(gpu, orc, 0, B)
    check_attend(gpu, orc, 0, synth.make_q(31, B, Hkv * g, 128, BF16), BF16)
    ks, vs = synth.make_kv(9500, B, 3, Hkv, 128, BF16)
    kd, vd = to_dev(ks, BF16), to_dev(vs, BF16)
    for s in range(3):
        q = synth.make_q(40 + s, B, Hkv * g, 128, BF16)
        out = gpu.append_attend(0, kd[:, s:s + 1], vd[:, s:s + 1], to_dev(q, BF16))
        orc.append(0, ks[:, s:s + 1], vs[:, s:s + 1])
        torch.cuda.synchronize()
        err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - orc.attend(0, q))))
        assert err <= ATTN_TOL, "step %d: %.3e" % (s, err)
    check_lengths(gpu, orc, 0, B)
    check_bytes_ragged(gpu, orc, 0)


@pytest.mark.parametrize("path", [0, 1], ids=["auto", "valu"])
@pytest.mark.parametrize("mode", [CHAN, CROSS])
def test_active_set(kv, oracle, mode, path):
    """Batch-wide calls with some slots switched off: only the active sequences take tokens, the
    others keep their contents and get zeros from the decode calls while they are off."""
    import torch

    print("case active set mode=%d path=%d" % (mode, path), flush=True)
    parity_util.DECODE_PATH = path
    try:
        B, Hkv, g, G = 6, 2, 4, 32
        gpu, orc = make_pair(kv, oracle, B=B, Hq=Hkv * g, Hkv=Hkv, T_max=8 * G, G=G, Gc=G, R=G, dtype=BF16, mode=mode,
                             k_bits=(4,))
        k, v = synth.make_kv(1200, B, 2 * G + 20, Hkv, 128, BF16)
        gpu.append(0, to_dev(k, BF16), to_dev(v, BF16))  # everyone active at first
        orc.append(0, k, v)
        active = [1, 0, 1, 1, 0, 1]
        kv.kv_cache_set_active(gpu.handle, active)
        steps = G  # crosses a block boundary of the active sequences
        ks, vs = synth.make_kv(1201, B, steps + 3, Hkv, 128, BF16)
        kd, vd = to_dev(ks, BF16), to_dev(vs, BF16)
        on = [b for b in range(B) if active[b]]
        off = [b for b in range(B) if not active[b]]
        for s in range(steps):
            q = synth.make_q(1300 + s, B, Hkv * g, 128, BF16)
            out = gpu.append_attend(0, kd[:, s:s + 1], vd[:, s:s + 1], to_dev(q, BF16))
            for b in on:
                orc.append_seq(0, b, ks[b, s:s + 1], vs[b, s:s + 1])
            torch.cuda.synchronize()
            got = out.cpu().numpy().astype(np.float64)
            want = orc.attend(0, q)
            assert float(np.max(np.abs(got[on] - want[on]))) <= ATTN_TOL, s
            assert not got[off].any(), "a sequence that is off must get zeros"
        check_lengths(gpu, orc, 0, B)
        # a bulk append under the mask, then everyone on again: the sequences that were off are intact
        gpu.append(0, kd[:, steps:steps + 3], vd[:, steps:steps + 3])
        for b in on:
            orc.append_seq(0, b, ks[b, steps:steps + 3], vs[b, steps:steps + 3])
        kv.kv_cache_set_active(gpu.handle, None)
        check_lengths(gpu, orc, 0, B)
        check_bytes_ragged(gpu, orc, 0)
        check_attend(gpu, orc, 0, synth.make_q(1400, B, Hkv * g, 128, BF16), BF16)
        with pytest.raises(kv.KVError) as e:
            kv.kv_cache_set_active(gpu.handle, [1, 0])
        assert e.value.status == kv.KV_E_BAD_CONFIG
    finally:
        parity_util.DECODE_PATH = 0

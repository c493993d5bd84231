"""GPU parity of the one-call decode step (append one token, then attend; Alg. 1 steps 8-9)
against the CPU oracle and against the two separate calls."""
import numpy as np
import pytest

from paper_2506_04642_amd import synth
import parity_util
from parity_util import ATTN_TOL, append_both, check_bytes, make_pair, to_dev

pytestmark = pytest.mark.gpu

F16, BF16 = 0, 1
CHAN, CROSS, NONE = 0, 1, 2


@pytest.fixture(scope="module")
def kv():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_04642_amd import binding

    return binding


def run_steps(kv, oracle, *, bits, G, R, mode, g, Hkv, B, T0, steps, dtype, path, seed):
    """Prefill T0 tokens, then `steps` decode steps through the one-call entry; every step's output
    is checked against the oracle and against a second cache driven by append + attend."""
    import torch

    parity_util.DECODE_PATH = path
    try:
        Hq = Hkv * g
        kw = dict(B=B, Hq=Hq, Hkv=Hkv, T_max=(T0 + steps + G + R) // G * G + R, G=G, Gc=G if G <= 64 else 32, R=R,
                  dtype=dtype, mode=mode, k_bits=(bits,))
        fused, orc = make_pair(kv, oracle, **kw)
        plain, _ = make_pair(kv, oracle, **kw)
        k, v = synth.make_kv(seed, B, T0 + steps, Hkv, 128, dtype)
        if T0:
            append_both(fused, orc, 0, k[:, :T0], v[:, :T0], dtype)
            plain.append(0, to_dev(k[:, :T0], dtype), to_dev(v[:, :T0], dtype))
        kd, vd = to_dev(k, dtype), to_dev(v, dtype)
        worst = 0.0
        for s in range(steps):
            q = synth.make_q(seed * 131 + s, B, Hq, 128, dtype)
            qd = to_dev(q, dtype)
            t = T0 + s
            out_f = fused.append_attend(0, kd[:, t:t + 1], vd[:, t:t + 1], qd)
            plain.append(0, kd[:, t:t + 1], vd[:, t:t + 1])
            out_p = plain.attend(0, qd)
            orc.append(0, k[:, t:t + 1], v[:, t:t + 1])
            torch.cuda.synchronize()
            assert fused.lengths(0) == plain.lengths(0) == (orc.packed_len(0), orc.resid_len(0))
            assert torch.equal(out_f, out_p), "step %d: one-call result differs from append + attend" % s
            want = orc.attend(0, q)
            err = float(np.max(np.abs(out_f.cpu().numpy().astype(np.float64) - want)))
            assert err <= ATTN_TOL, "step %d: attention max-abs error %.3e" % (s, err)
            worst = max(worst, err)
        check_bytes(fused, orc, 0)
        return worst
    finally:
        parity_util.DECODE_PATH = 0


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("G,R", [(32, 32), (64, 64), (32, 64), (32, 128)])
def test_decode_steps_across_block_boundaries(kv, oracle, bits, G, R):
    """Starts a few tokens before a block completes, so the steps cover: token kept raw (fused
    kernel), token that completes a block (separate launches), first token after a flush."""
    print("case append_attend bits=%d G=%d R=%d" % (bits, G, R), flush=True)
    T0 = 5 * R + R - 3
    run_steps(kv, oracle, bits=bits, G=G, R=R, mode=CHAN, g=4, Hkv=2, B=2, T0=T0, steps=R + 6, dtype=BF16,
              path=0, seed=400 + bits)


@pytest.mark.parametrize("path,mode,g", [(1, CHAN, 4), (0, CROSS, 2), (0, NONE, 8), (2, CHAN, 3)])
def test_decode_steps_other_paths(kv, oracle, path, mode, g):
    print("case append_attend path=%d mode=%d g=%d" % (path, mode, g), flush=True)
    run_steps(kv, oracle, bits=4, G=32, R=32, mode=mode, g=g, Hkv=2, B=2, T0=150, steps=40, dtype=F16, path=path,
              seed=410 + path + mode)


def test_decode_steps_from_an_empty_cache(kv, oracle):
    print("case append_attend empty start", flush=True)
    run_steps(kv, oracle, bits=4, G=32, R=32, mode=CHAN, g=4, Hkv=1, B=1, T0=0, steps=70, dtype=BF16, path=0, seed=420)


def test_append_attend_errors_leave_the_cache_unchanged(kv, oracle):
    import torch

    print("case append_attend errors", flush=True)
    gpu, _ = make_pair(kv, oracle, B=1, Hq=4, Hkv=1, T_max=64, dtype=F16, k_bits=(4,))
    k = torch.zeros((1, 1, 128), dtype=torch.float16, device="cuda:0")
    q = torch.zeros((1, 4, 128), dtype=torch.float16, device="cuda:0")
    out = torch.zeros((1, 4, 128), dtype=torch.float32, device="cuda:0")
    ws, wsb = gpu.workspace.data_ptr(), gpu.ws_bytes
    ok = (gpu.handle, 0, k.data_ptr(), k.data_ptr(), k.stride(0), k.stride(1), q.data_ptr(), out.data_ptr(), ws, wsb, 0)

    def expect(args, code):
        with pytest.raises(kv.KVError) as e:
            kv.kv_append_decode_attn(*args)
        assert e.value.status == code
        assert gpu.lengths(0) == (0, 0)

    expect(ok[:2] + (0,) + ok[3:], kv.KV_E_NULL)
    expect(ok[:6] + (0,) + ok[7:], kv.KV_E_NULL)
    expect(ok[:7] + (0,) + ok[8:], kv.KV_E_NULL)
    expect(ok[:9] + (16,) + ok[10:], kv.KV_E_WORKSPACE)
    expect(ok[:2] + (k.data_ptr() + 2,) + ok[3:], kv.KV_E_ALIGN)
    expect((gpu.handle, 3) + ok[2:], kv.KV_E_BAD_LAYER)
    kv.kv_append_decode_attn(*ok)
    assert gpu.lengths(0) == (0, 1)
    full = torch.zeros((1, 63, 1, 128), dtype=torch.float16, device="cuda:0")
    gpu.append(0, full, full)
    with pytest.raises(kv.KVError) as e:
        kv.kv_append_decode_attn(*ok)
    assert e.value.status == kv.KV_E_CAPACITY

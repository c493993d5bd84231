"""GPU parity of kv_compressv_append (Alg. 1 step 3: the value projection fused with the values'
compression) against the CPU oracle, in two stages.
  (i)  the projected values as the kernels rounded them (the optional v_proj output) against the
       oracle's projection (binary64 dot products rounded once): every element within one unit in
       the last place of the 16-bit type, nearly all equal;
  (ii) the cache bytes against the oracle's encoder applied to the kernels' own projected values:
       bit for bit.
The matrix cores accumulate in binary32, so (i) cannot be bit-exact; everything after the rounding
of the projection is."""
import numpy as np
import pytest

from paper_2506_04642_amd import synth
from parity_util import check_attention, check_bytes, make_pair, to_dev

pytestmark = pytest.mark.gpu

F16, BF16 = 0, 1
CHAN, CROSS, NONE = 0, 1, 2


@pytest.fixture(scope="module")
def kv():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_04642_amd import binding

    return binding


def _ordered(bits16):
    """16-bit float patterns as integers that are monotone in the value (for distances in ulps)."""
    b = bits16.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def _from_dev16(t):
    import torch

    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _check_projection(oracle, got, x, w, dtype):
    """Stage (i).  got, x: uint16 [..., n_out], [..., kdim].  The kernels accumulate in binary32, one
    rounding per matrix instruction (32 k-values) plus what happens inside it: against the exact sum E,
    |V - E| <= half a 16-bit ulp of V + (kdim / 32 + 8) * 2^-24 * sum|x w|; where the sum does not
    cancel (|E| >= sum|x w| / 64) that is within one ulp of the oracle's once-rounded value; and nearly
    all values are equal to it."""
    want = oracle.project(x, w, dtype)
    acc, mag = oracle.project_f64(x, w, dtype)
    gv = synth.bits16_to_f32(got, dtype).astype(np.float64)
    sig = 8 if dtype == BF16 else 11
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(gv), 2.0 ** -14))) - (sig - 1))
    slack = (x.shape[-1] / 32 + 8) * 2.0 ** -24 * mag
    assert np.all(np.abs(gv - acc) <= 0.5 * ulp + slack), "projection error beyond the binary32 accumulation bound"
    dist = np.abs(_ordered(got) - _ordered(want))
    big = np.abs(acc) >= mag / 64
    assert big.mean() > 0.5 and dist[big].max() <= 1, "projected value %d ulps from the exactly rounded one" % dist[big].max()
    assert np.mean(dist == 0) > 0.97, "only %.3f of the projected values equal the exactly rounded ones" % np.mean(dist == 0)


def _append_both(kv, gpu, orc, oracle, layer, k, x, w, dtype, chunks, rope=None, check_proj=True):
    """Feeds the chunks to kv_compressv_append and, with the kernels' projected values, to the oracle's
    plain append; returns the projected values of the GPU, uint16 [B, T, H, d]."""
    import torch

    B, T, H, d = k.shape
    kd, xd, wd = to_dev(k, dtype), to_dev(x, dtype), to_dev(w, dtype)
    got_all = np.zeros((B, T, H, d), dtype=np.uint16)
    pos = 0
    for n in chunks:
        if n == 0:
            continue
        vp = torch.zeros((B, n, H, d), dtype=kd.dtype, device="cuda:0")
        cos = sin = None
        tabs = None
        if rope is not None:
            cos_h, sin_h, pairing = rope
            cos, sin = torch.from_numpy(cos_h[pos:pos + n].copy()).to("cuda:0"), torch.from_numpy(sin_h[pos:pos + n].copy()).to("cuda:0")
            tabs = (cos_h[pos:pos + n], sin_h[pos:pos + n], pairing)
        gpu.append_compressv(layer, kd[:, pos:pos + n], xd[:, pos:pos + n], wd, cos, sin,
                             rope[2] if rope is not None else 0, v_proj=vp)
        torch.cuda.synchronize()
        got = _from_dev16(vp)
        got_all[:, pos:pos + n] = got
        orc.append(layer, k[:, pos:pos + n], got, rope_tables=tabs)
        pos += n
    assert pos == T
    if check_proj:
        _check_projection(oracle, got_all.reshape(B, T, H * d), x, w, dtype)
    return got_all


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("Gc", [32, 64, 128])
@pytest.mark.parametrize("dtype,mode", [(BF16, CHAN), (F16, CHAN), (BF16, NONE)])
def test_bulk_prefill_formats(kv, oracle, bits, Gc, dtype, mode):
    """One bulk call: 9 whole blocks per sequence (18 groups: three workgroup tiles, the last one partly
    empty) and a raw tail of 13 tokens."""
    print("case compressv bulk bits=%d Gc=%d dtype=%d mode=%d" % (bits, Gc, dtype, mode), flush=True)
    B, H, T, kdim = 2, 2, 9 * 32 + 13, 256
    gpu, orc = make_pair(kv, oracle, B=B, Hq=2 * H, Hkv=H, T_max=10 * 32, Gc=Gc, dtype=dtype, mode=mode, k_bits=(bits,))
    k, _ = synth.make_kv(700 + bits, B, T, H, 128, dtype)
    x, w = synth.make_xw(700 + Gc, B, T, kdim, H * 128, dtype)
    _append_both(kv, gpu, orc, oracle, 0, k, x, w, dtype, [T])
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(700, B, 2 * H, 128, dtype), dtype)


@pytest.mark.parametrize("H", [1, 3, 8])
def test_head_counts(kv, oracle, H):
    """Odd head counts run one head per workgroup, even ones two."""
    print("case compressv heads H=%d" % H, flush=True)
    B, T, kdim = 3, 4 * 32 + 7, 192
    gpu, orc = make_pair(kv, oracle, B=B, Hq=H, Hkv=H, T_max=5 * 32, dtype=BF16, k_bits=(4,))
    k, _ = synth.make_kv(710 + H, B, T, H, 128, BF16)
    x, w = synth.make_xw(710 + H, B, T, kdim, H * 128, BF16)
    _append_both(kv, gpu, orc, oracle, 0, k, x, w, BF16, [T])
    check_bytes(gpu, orc, 0)


@pytest.mark.parametrize("R", [32, 64])
@pytest.mark.parametrize("bits", [2, 8])
def test_chunked_calls_equal_the_bulk_call(kv, oracle, R, bits):
    """Calls of uneven sizes: tokens that complete a block begun by an earlier call, blocks that wait in
    the residual buffer whole (R = 64), single tokens (the decode step's kernel), tails.  Every token's
    projected value is the same whichever kernel produced it, so the cache bytes equal the bulk call's."""
    print("case compressv chunks R=%d bits=%d" % (R, bits), flush=True)
    B, H, kdim = 2, 2, 320
    chunks = [5, 40, 1, 1, 1, 100, 27, 32, 64, 3, 70, 1]
    T = sum(chunks)
    k, _ = synth.make_kv(720 + R, B, T, H, 128, BF16)
    x, w = synth.make_xw(720 + bits, B, T, kdim, H * 128, BF16)
    T_max = (T // R + 1) * R
    gpu, orc = make_pair(kv, oracle, B=B, Hq=4 * H, Hkv=H, T_max=T_max, R=R, dtype=BF16, k_bits=(bits,))
    v_chunked = _append_both(kv, gpu, orc, oracle, 0, k, x, w, BF16, chunks)
    check_bytes(gpu, orc, 0)
    gpu2, orc2 = make_pair(kv, oracle, B=B, Hq=4 * H, Hkv=H, T_max=T_max, R=R, dtype=BF16, k_bits=(bits,))
    v_bulk = _append_both(kv, gpu2, orc2, oracle, 0, k, x, w, BF16, [T], check_proj=False)
    check_bytes(gpu2, orc2, 0)
    assert np.array_equal(v_chunked, v_bulk)
    assert np.array_equal(gpu.layers[0].cpu().numpy()[orc.layer_image(0)["valid"]],
                          gpu2.layers[0].cpu().numpy()[orc2.layer_image(0)["valid"]])
    check_attention(gpu, orc, 0, synth.make_q(720, B, 4 * H, 128, BF16), BF16)


@pytest.mark.parametrize("B", [1, 20, 70, 300])
def test_decode_steps(kv, oracle, B):
    """One token per sequence and call across two block boundaries: up to 64 rows go through the
    streaming kernel (one wave per 16 rows and 16 channels), more than 256 through the tiled one."""
    print("case compressv decode B=%d" % B, flush=True)
    H, kdim, T = 2, 256, 70
    gpu, orc = make_pair(kv, oracle, B=B, Hq=H, Hkv=H, T_max=96, dtype=BF16, k_bits=(4,))
    k, _ = synth.make_kv(730 + B, B, T, H, 128, BF16)
    x, w = synth.make_xw(730 + B, B, T, kdim, H * 128, BF16)
    _append_both(kv, gpu, orc, oracle, 0, k, x, w, BF16, [1] * T)
    check_bytes(gpu, orc, 0)


@pytest.mark.parametrize("pairing", [0, 1])
def test_rotary_keys_and_projected_values_in_one_call(kv, oracle, pairing):
    """Alg. 1 steps 3, 5 and 8 together: pre-rotation keys with tables, values from the projection."""
    print("case compressv rope pairing=%d" % pairing, flush=True)
    B, H, kdim = 2, 4, 256
    chunks = [45, 1, 90, 20]
    T = sum(chunks)
    gpu, orc = make_pair(kv, oracle, B=B, Hq=H, Hkv=H, T_max=160, dtype=BF16, k_bits=(4,))
    k, _ = synth.make_kv(740, B, T, H, 128, BF16)
    x, w = synth.make_xw(740, B, T, kdim, H * 128, BF16)
    cos, sin = synth.rope_tables(np.arange(T), 128)
    _append_both(kv, gpu, orc, oracle, 0, k, x, w, BF16, chunks, rope=(cos, sin, pairing))
    check_bytes(gpu, orc, 0)


def test_mixed_layers_strided_inputs_and_no_debug_output(kv, oracle):
    """A three-layer 2/4/8-bit cache; inputs that are views into larger tensors; and the production form of
    the call (no v_proj tensor) must write the same cache bytes as the inspected form."""
    import torch

    print("case compressv mixed layers", flush=True)
    B, H, kdim, T = 2, 2, 256, 100
    bits = (2, 4, 8)
    gpu, orc = make_pair(kv, oracle, L=3, B=B, Hq=H, Hkv=H, T_max=128, dtype=BF16, k_bits=bits)
    plain, _ = make_pair(kv, oracle, L=3, B=B, Hq=H, Hkv=H, T_max=128, dtype=BF16, k_bits=bits)
    for l in range(3):
        k, _ = synth.make_kv(750 + l, B, T, H, 128, BF16)
        x, w = synth.make_xw(750 + l, B, T, kdim, H * 128, BF16)
        _append_both(kv, gpu, orc, oracle, l, k, x, w, BF16, [T])
        check_bytes(gpu, orc, l)
        big_k = torch.zeros((B, T + 9, H + 1, 128), dtype=torch.bfloat16, device="cuda:0")
        big_x = torch.zeros((B, T + 4, kdim + 64), dtype=torch.bfloat16, device="cuda:0")
        big_k[:, 3:3 + T, 1:] = to_dev(k, BF16)
        big_x[:, 2:2 + T, :kdim] = to_dev(x, BF16)
        plain.append_compressv(l, big_k[:, 3:3 + T, 1:], big_x[:, 2:2 + T, :kdim], to_dev(w, BF16))
        torch.cuda.synchronize()
        m = orc.layer_image(l)["valid"]
        assert np.array_equal(plain.layers[l].cpu().numpy()[m], gpu.layers[l].cpu().numpy()[m])


def test_formats_without_a_fused_kernel_are_refused(kv, oracle):
    import torch

    print("case compressv unsupported", flush=True)
    x16, w16 = synth.make_xw(760, 1, 8, 128, 128, BF16)
    k16, _ = synth.make_kv(760, 1, 8, 1, 128, BF16)
    kd, xd, wd = to_dev(k16, BF16), to_dev(x16, BF16), to_dev(w16, BF16)
    for kw in (dict(G=64, Gc=64), dict(mode=CROSS), dict(k_bits=(4,), v_bits=(2,)), dict(k_bits=(16,))):
        args = dict(B=1, Hq=1, Hkv=1, T_max=128, dtype=BF16, k_bits=(4,))
        args.update(kw)
        gpu, _ = make_pair(kv, oracle, **args)
        with pytest.raises(kv.KVError) as e:
            gpu.append_compressv(0, kd, xd, wd)
        assert e.value.status == kv.KV_E_UNSUPPORTED
        assert gpu.lengths(0) == (0, 0)
    gpu, _ = make_pair(kv, oracle, B=1, Hq=1, Hkv=1, T_max=32, dtype=BF16, k_bits=(4,))
    with pytest.raises(kv.KVError) as e:  # model_dim must be a multiple of 64
        kv.kv_compressv_append(gpu.handle, 0, kd.data_ptr(), 8 * 128, 128, 128, xd.data_ptr(), 8 * 128, 128, wd.data_ptr(), 96, 8)
    assert e.value.status == kv.KV_E_BAD_CONFIG
    k40, _ = synth.make_kv(761, 1, 40, 1, 128, BF16)
    x40, _ = synth.make_xw(761, 1, 40, 128, 128, BF16)
    with pytest.raises(kv.KVError) as e:
        gpu.append_compressv(0, to_dev(k40, BF16), to_dev(x40, BF16), wd)
    assert e.value.status == kv.KV_E_CAPACITY
    torch.cuda.synchronize()


def test_llama_shape_sampled(kv, oracle):
    """The full-cache workload's layer shape (8 kv heads, model_dim 4096, batch 16) on a 2048-token prefill
    call: sampled rows of the projection against the oracle, sampled units of the cache against the
    oracle's encoder on the kernels' projected values."""
    import torch

    print("case compressv llama shape", flush=True)
    B, H, kdim, T, bits = 16, 8, 4096, 2048, 4
    cfg = kv.make_config(1, B, 4 * H, H, 128, T + 32, 32, 32, 32, kv.KV_BF16, kv.KV_MEAN_CHANNEL_BLOCK, [bits], [bits])
    gpu = kv.KVCache(cfg, zero=False)
    dev = torch.device("cuda:0")
    kd, _ = synth.make_kv_torch(770, B, T, H, 128, BF16, dev)
    xd, wd = synth.make_xw_torch(770, B, T, kdim, H * 128, BF16, dev)
    vp = torch.zeros((B, T, H, 128), dtype=torch.bfloat16, device=dev)
    gpu.append_compressv(0, kd, xd, wd, v_proj=vp)
    torch.cuda.synchronize()
    assert gpu.lengths(0) == (T, 0)
    rng = np.random.default_rng(770)
    w16 = _from_dev16(wd)
    rows = [(int(b), int(t)) for b, t in zip(rng.integers(0, B, 24), rng.integers(0, T, 24))] + [(0, 0), (B - 1, T - 1)]
    xs = np.stack([_from_dev16(xd[b, t]) for b, t in rows])
    got = np.stack([_from_dev16(vp[b, t]).reshape(-1) for b, t in rows])
    _check_projection(oracle, got, xs, w16, BF16)
    # sampled sequences: the oracle encodes the kernels' values; compare those units' records
    lay = kv.kv_cache_describe(gpu.handle, 0)
    raw = gpu.layers[0].cpu().numpy()
    NB = (T + 32) // 32
    for b in (0, 7, 15):
        ocfg = oracle.OracleConfig(1, 1, 4 * H, H, 128, T + 32, 32, 32, 32, BF16, CHAN, [bits], [bits])
        orc = oracle.OracleCache(ocfg)
        orc.append(0, _from_dev16(kd[b:b + 1]), _from_dev16(vp[b:b + 1]))
        img = orc.layer_image(0)
        n_rec = H * NB * lay.rec_bytes
        mine = raw[b * n_rec:(b + 1) * n_rec]
        m = img["valid"][:n_rec]
        assert m.sum() == H * (T // 32) * (2 * 32 * 128 * bits // 8 + 512 + 256 + 32 * 4 * 4 + 256)
        assert np.array_equal(mine[m], img["bytes"][:n_rec][m])

"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.
Packed codes and metadata must match bit for bit; attention within 2e-3 max-abs."""
import numpy as np
import pytest

from paper_2506_04642_amd import synth
import parity_util
from parity_util import ATTN_TOL, append_both, check_attention, check_bytes, make_pair, to_dev

pytestmark = pytest.mark.gpu

F16, BF16 = 0, 1
CHAN, CROSS, NONE = 0, 1, 2


@pytest.fixture(scope="module")
def kv():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_04642_amd import binding

    return binding


@pytest.fixture(autouse=True, params=[1, 0], ids=["valu", "auto"])
def decode_path(request):
    """Every case runs on the vector-ALU kernels and on the automatic choice (matrix-core kernels
    wherever they support the configuration)."""
    parity_util.DECODE_PATH = request.param
    yield request.param
    parity_util.DECODE_PATH = 0


# ------------------------------------------------------------------ config 0: one head, fp16


@pytest.mark.parametrize("T", [1, 31, 32, 33, 1024, 1037])
def test_single_head_fp16_4bit(kv, oracle, T):
    print("case single_head T=%d" % T, flush=True)
    gpu, orc = make_pair(kv, oracle, T_max=2048, dtype=F16, k_bits=(4,))
    k, v = synth.make_kv(100 + T, 1, T, 1, 128, F16)
    append_both(gpu, orc, 0, k, v, F16)
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(100 + T, 1, 1, 128, F16), F16)


# ------------------------------------------------------------------ config 1: Llama-3-8B layer


@pytest.mark.parametrize("T", [8192, 8193, 8205])
def test_llama8b_layer_bf16_4bit(kv, oracle, T):
    print("case llama8b_layer T=%d" % T, flush=True)
    gpu, orc = make_pair(kv, oracle, B=1, Hq=32, Hkv=8, T_max=8192 + 32, dtype=BF16, k_bits=(4,))
    k, v = synth.make_kv(1000, 1, T, 8, 128, BF16)
    # bulk prefill of T-1 tokens, then one decode step: append 1, attend
    append_both(gpu, orc, 0, k, v, BF16, chunks=[T - 1, 1])
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(1000, 1, 32, 128, BF16), BF16)


# ------------------------------------------------------------------ sweep of formats


@pytest.mark.parametrize("bits", [2, 4, 8, 16])
@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("G,Gc", [(32, 32), (64, 64), (128, 32), (32, 128), (128, 128)])
def test_bit_widths_and_groups(kv, oracle, bits, dtype, G, Gc):
    print("case widths bits=%d dtype=%d G=%d Gc=%d" % (bits, dtype, G, Gc), flush=True)
    T = 3 * G + 5
    gpu, orc = make_pair(kv, oracle, B=2, Hq=8, Hkv=2, T_max=4 * G, G=G, Gc=Gc, dtype=dtype, k_bits=(bits,))
    k, v = synth.make_kv(7 * bits + G, 2, T, 2, 128, dtype)
    append_both(gpu, orc, 0, k, v, dtype)
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(bits + G, 2, 8, 128, dtype), dtype)


@pytest.mark.parametrize("mode", [CHAN, CROSS, NONE])
@pytest.mark.parametrize("G,Gc,bits", [(64, 32, 4), (64, 64, 2), (64, 128, 8), (128, 128, 4), (128, 128, 2), (128, 32, 8), (128, 64, 2)])
def test_bulk_append_of_long_blocks_in_uneven_calls(kv, oracle, G, Gc, bits, mode):
    """Blocks of 64 / 128 tokens through the bulk append (a workgroup per item, a wave per 32-token
    part): calls that leave raw tokens behind, calls whose first block takes rows from the raw buffer
    and rows from the call, a call of many blocks, and more items than one launch holds workgroups."""
    print("case long blocks G=%d Gc=%d bits=%d mode=%d" % (G, Gc, bits, mode), flush=True)
    B, H = 4, 8
    chunks = [G - 7, 2 * G + 3, 5, 27 * G + 1, G - 2]  # 30 blocks in all: 1920 items for 32 units
    T = sum(chunks)
    gpu, orc = make_pair(kv, oracle, B=B, Hq=H, Hkv=H, T_max=31 * G, G=G, Gc=Gc, dtype=BF16, mode=mode, k_bits=(bits,))
    k, v = synth.make_kv(4100 + G + bits, B, T, H, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16, chunks=chunks)
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(4100 + G, B, H, 128, BF16), BF16)


@pytest.mark.parametrize("mode", [CHAN, NONE])
@pytest.mark.parametrize("g", [4, 8])
@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("G,Gc", [(32, 64), (32, 128), (64, 32), (64, 128), (128, 32), (128, 64)])
def test_mixed_group_sizes(kv, oracle, decode_path, G, Gc, bits, g, mode):
    """Key groups (tokens) and value groups (channels) of different sizes: served by the matrix-core
    kernels under the automatic choice (several chunks per wave, a ragged tail of raw tokens, one and
    two head groups)."""
    print("case mixed groups G=%d Gc=%d bits=%d g=%d mode=%d" % (G, Gc, bits, g, mode), flush=True)
    B, H = 2, 2
    T = 9 * 128 + 77
    gpu, orc = make_pair(kv, oracle, B=B, Hq=H * g, Hkv=H, T_max=10 * 128, G=G, Gc=Gc, dtype=BF16, mode=mode, k_bits=(bits,))
    k, v = synth.make_kv(6100 + G + bits + g, B, T, H, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16, chunks=[T - 1, 1])
    assert kv.kv_decode_path_used(gpu.handle, 0) == (1 if decode_path == 1 else 2)
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(6100 + G + g, B, H * g, 128, BF16), BF16)


@pytest.mark.parametrize("G,R", [(64, 128), (64, 192), (128, 256)])
def test_long_blocks_with_a_longer_raw_buffer(kv, oracle, G, R):
    """Blocks of 64 / 128 tokens with a raw buffer of several blocks (R > G): a flush compresses R / G
    blocks at once, most of whose rows come from the raw buffer and the rest from the call."""
    print("case long blocks G=%d R=%d" % (G, R), flush=True)
    B, H = 2, 4
    chunks = [R - 3, 5, 2 * R + G + 1, 1, R - 1]
    T = sum(chunks)
    gpu, orc = make_pair(kv, oracle, B=B, Hq=2 * H, Hkv=H, T_max=8 * R, G=G, Gc=G, R=R, dtype=F16, k_bits=(4,))
    k, v = synth.make_kv(5200 + G + R, B, T, H, 128, F16)
    append_both(gpu, orc, 0, k, v, F16, chunks=chunks)
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(5200 + G, B, 2 * H, 128, F16), F16)


@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("bits", [2, 4, 8])
def test_exact_ties_round_to_the_even_code(kv, oracle, bits, G):
    """Groups built so that zero = 0 and scale = 1 exactly (minimum 0, maximum 2^bits - 1) and the
    other members sit at k + 1/2: every one of them is a tie, which must go to the even code
    (binary16 inputs, no centring, so that nothing else rounds on the way)."""
    print("case ties bits=%d G=%d" % (bits, G), flush=True)
    qmax = (1 << bits) - 1
    B, H, T = 2, 2, 2 * G
    halves = np.array([(k % qmax) + 0.5 for k in range(128)], dtype=np.float32)
    k = np.zeros((B, T, H, 128), dtype=np.float32)
    v = np.zeros((B, T, H, 128), dtype=np.float32)
    # keys: a group is one channel over the G tokens of a block
    for t in range(T):
        tin = t % G
        k[:, t] = 0.0 if tin == 0 else (qmax if tin == 1 else halves[(tin + np.arange(128)) % 128])
    # values: a group is G (= Gc) channels of one token
    for c in range(128):
        cin = c % G
        v[:, :, :, c] = 0.0 if cin == 0 else (qmax if cin == 1 else halves[(cin + np.arange(T)) % 128][None, :, None])
    kb = k.astype(np.float16).view(np.uint16)
    vb = v.astype(np.float16).view(np.uint16)
    assert np.array_equal(kb.view(np.float16).astype(np.float32), k)  # all values are exact in binary16
    gpu, orc = make_pair(kv, oracle, B=B, Hq=H, Hkv=H, T_max=T, G=G, Gc=G, dtype=F16, mode=NONE, k_bits=(bits,))
    append_both(gpu, orc, 0, kb, vb, F16)
    check_bytes(gpu, orc, 0)
    # the oracle's own codes: ties went to even (pins the expectation, not only the agreement)
    kr = orc.reconstruct(0, 0, 0)  # keys of sequence 0, [H, T, d]; zero = 0 and scale = 1: the codes themselves
    for blk in range(T // G):
        assert np.all(kr[:, blk * G + 2:(blk + 1) * G] % 2 == 0)


@pytest.mark.parametrize("kb,vb", [(2, 4), (4, 2), (8, 2), (4, 8)])
def test_different_widths_for_keys_and_values(kv, oracle, kb, vb):
    print("case kv_widths kb=%d vb=%d" % (kb, vb), flush=True)
    gpu, orc = make_pair(kv, oracle, B=1, Hq=4, Hkv=1, T_max=256, dtype=BF16, k_bits=(kb,), v_bits=(vb,))
    k, v = synth.make_kv(kb * 10 + vb, 1, 200, 1, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16)
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(3, 1, 4, 128, BF16), BF16)


@pytest.mark.parametrize("mode", [CHAN, NONE])
@pytest.mark.parametrize("g", [4, 8])
@pytest.mark.parametrize("kb,vb", [(2, 4), (2, 8), (4, 2), (4, 8), (8, 2), (8, 4)])
def test_different_widths_on_both_kernel_families(kv, oracle, decode_path, kb, vb, g, mode):
    """Keys and values of different widths (groups of 32): the matrix-core kernels serve them under the
    automatic choice; several chunks per wave, a ragged tail of raw tokens, one and two head groups, a
    one-call decode step at the end."""
    print("case kv_widths both kb=%d vb=%d g=%d mode=%d" % (kb, vb, g, mode), flush=True)
    B, H = 2, 2
    T = 40 * 32 + 19
    gpu, orc = make_pair(kv, oracle, B=B, Hq=H * g, Hkv=H, T_max=42 * 32, dtype=BF16, mode=mode, k_bits=(kb,), v_bits=(vb,))
    k, v = synth.make_kv(7100 + 10 * kb + vb + g, B, T, H, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16, chunks=[T - 1, 1])
    assert kv.kv_decode_path_used(gpu.handle, 0) == (1 if decode_path == 1 else 2)
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(7100 + kb + g, B, H * g, 128, BF16), BF16)


@pytest.mark.parametrize("mode", [CHAN, NONE, CROSS])
@pytest.mark.parametrize("g", [1, 2, 4, 8])
def test_mean_modes_and_query_groups(kv, oracle, mode, g):
    print("case modes mode=%d g=%d" % (mode, g), flush=True)
    Hkv = 2
    gpu, orc = make_pair(kv, oracle, B=2, Hq=Hkv * g, Hkv=Hkv, T_max=512, dtype=BF16, mode=mode, k_bits=(4,))
    k, v = synth.make_kv(50 + g, 2, 300, Hkv, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16)
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(g, 2, Hkv * g, 128, BF16), BF16)


def test_decode_path_used_reports_the_kernel_family(kv, oracle):
    """Under the automatic choice a layer whose format the matrix-core kernels do not take runs on the
    vector-ALU kernels; kv_decode_path_used says so, and forcing the matrix cores refuses such a layer."""
    print("case path_used", flush=True)
    gpu, orc = make_pair(kv, oracle, L=3, B=1, Hq=4, Hkv=1, T_max=128, dtype=BF16, k_bits=(4, 4, 16), v_bits=(4, 2, 16))
    k, v = synth.make_kv(91, 1, 40, 1, 128, BF16)
    for l in range(3):
        append_both(gpu, orc, l, k, v, BF16)
    # (layer 1: keys and values of different widths, which the matrix-core kernels take with groups of 32;
    # layer 2: a 16-bit layer, which they do not)
    want = (1, 1, 1) if parity_util.DECODE_PATH == 1 else (2, 2, 1)
    assert tuple(kv.kv_decode_path_used(gpu.handle, l) for l in range(3)) == want
    kv.kv_set_decode_path(gpu.handle, 2)
    assert kv.kv_decode_path_used(gpu.handle, 0) == 2 and kv.kv_decode_path_used(gpu.handle, 1) == 2
    with pytest.raises(kv.KVError) as e:
        kv.kv_decode_path_used(gpu.handle, 2)
    assert e.value.status == kv.KV_E_UNSUPPORTED


def test_mixed_layer_map(kv, oracle):
    print("case mixed_layer_map", flush=True)
    bits = (8, 4, 2, 16, 2, 4)
    gpu, orc = make_pair(kv, oracle, L=6, B=2, Hq=8, Hkv=2, T_max=256, dtype=BF16, k_bits=bits)
    for l in range(6):
        k, v = synth.make_kv(200 + l, 2, 150, 2, 128, BF16)
        append_both(gpu, orc, l, k, v, BF16)
    for l in range(6):
        check_bytes(gpu, orc, l)
        check_attention(gpu, orc, l, synth.make_q(l, 2, 8, 128, BF16), BF16)


# ------------------------------------------------------------------ append semantics


@pytest.mark.parametrize("R", [32, 64])
def test_single_token_appends_equal_bulk(kv, oracle, R):
    print("case single_appends R=%d" % R, flush=True)
    T = 77
    gpu, orc = make_pair(kv, oracle, B=2, Hq=4, Hkv=2, T_max=128, R=R, dtype=F16, k_bits=(4,), v_bits=(2,))
    k, v = synth.make_kv(9, 2, T, 2, 128, F16)
    append_both(gpu, orc, 0, k, v, F16, chunks=[1] * T)
    check_bytes(gpu, orc, 0)
    q = synth.make_q(9, 2, 4, 128, F16)
    check_attention(gpu, orc, 0, q, F16)
    # uneven chunks through a second pair must give the same bytes
    gpu2, orc2 = make_pair(kv, oracle, B=2, Hq=4, Hkv=2, T_max=128, R=R, dtype=F16, k_bits=(4,), v_bits=(2,))
    append_both(gpu2, orc2, 0, k, v, F16, chunks=[5, 40, 0, 31, 1])
    check_bytes(gpu2, orc2, 0)


def test_strided_input_views(kv, oracle):
    """k_new / v_new given as strided views (a slice of a larger [B, T, 3H, d] projection)."""
    import torch

    print("case strided_views", flush=True)
    gpu, orc = make_pair(kv, oracle, B=2, Hq=4, Hkv=2, T_max=128, dtype=BF16, k_bits=(4,))
    k, v = synth.make_kv(12, 2, 70, 2, 128, BF16)
    big_k = torch.zeros((2, 70, 6, 128), dtype=torch.bfloat16, device="cuda:0")
    big_v = torch.zeros_like(big_k)
    big_k[:, :, 2:4] = to_dev(k, BF16)
    big_v[:, :, 2:4] = to_dev(v, BF16)
    gpu.append(0, big_k[:, :, 2:4], big_v[:, :, 2:4])
    orc.append(0, k, v)
    check_bytes(gpu, orc, 0)


def test_capacity_and_empty_errors(kv, oracle):
    print("case capacity_errors", flush=True)
    gpu, orc = make_pair(kv, oracle, T_max=64, dtype=F16, k_bits=(4,))
    q = to_dev(synth.make_q(1, 1, 1, 128, F16), F16)
    with pytest.raises(kv.KVError) as e:
        gpu.attend(0, q)
    assert e.value.status == kv.KV_E_EMPTY
    k, v = synth.make_kv(1, 1, 65, 1, 128, F16)
    with pytest.raises(kv.KVError) as e:
        gpu.append(0, to_dev(k, F16), to_dev(v, F16))
    assert e.value.status == kv.KV_E_CAPACITY
    assert gpu.lengths(0) == (0, 0)
    gpu.append(0, to_dev(k[:, :64], F16), to_dev(v[:, :64], F16))
    assert gpu.lengths(0) == (64, 0)


# ------------------------------------------------------------------ split-K merge


def test_result_does_not_depend_on_the_split_count(kv, oracle):
    """The log-sum-exp merge is an identity: 1, 2, 7 or 64 splits give the same attention."""
    import torch

    print("case split_independence", flush=True)
    gpu, orc = make_pair(kv, oracle, B=1, Hq=4, Hkv=1, T_max=4096, dtype=BF16, k_bits=(4,))
    k, v = synth.make_kv(33, 1, 2048 + 9, 1, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16)
    q = synth.make_q(33, 1, 4, 128, BF16)
    gpu.workspace = torch.empty(4 * 64 * 132 * 4 * 2, dtype=torch.uint8, device="cuda:0")
    gpu.ws_bytes = gpu.workspace.numel()
    outs = []
    for ns in (1, 2, 7, 64):
        kv.kv_set_decode_splits(gpu.handle, ns)
        assert kv.kv_decode_splits(gpu.handle, 0) <= ns
        check_attention(gpu, orc, 0, q, BF16)
        outs.append(gpu.attend(0, to_dev(q, BF16)).cpu().numpy())
    for o in outs[1:]:
        assert np.max(np.abs(o - outs[0])) < 1e-5


@pytest.mark.parametrize("g", [4, 8])
def test_split_count_with_blocks_of_128(kv, oracle, g):
    """Blocks of 128 tokens are dealt to the splits whole (their two halves stay in one wave): any
    split count, also more splits than blocks and counts that do not divide them, gives the same
    attention."""
    import torch

    print("case split_independence_g128 g=%d" % g, flush=True)
    gpu, orc = make_pair(kv, oracle, B=2, Hq=2 * g, Hkv=2, T_max=24 * 128, G=128, Gc=128, dtype=BF16, k_bits=(4,))
    k, v = synth.make_kv(35, 2, 21 * 128 + 77, 2, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16)
    q = synth.make_q(35, 2, 2 * g, 128, BF16)
    gpu.workspace = torch.empty(2 * 2 * g * 64 * 132 * 4 * 2, dtype=torch.uint8, device="cuda:0")
    gpu.ws_bytes = gpu.workspace.numel()
    outs = []
    for ns in (1, 2, 5, 7, 21, 64):
        kv.kv_set_decode_splits(gpu.handle, ns)
        assert kv.kv_decode_splits(gpu.handle, 0) <= ns
        check_attention(gpu, orc, 0, q, BF16)
        outs.append(gpu.attend(0, to_dev(q, BF16)).cpu().numpy())
    for o in outs[1:]:
        assert np.max(np.abs(o - outs[0])) < 1e-5


def test_repeat_calls_are_bitwise_reproducible(kv, oracle):
    print("case reproducible", flush=True)
    gpu, orc = make_pair(kv, oracle, B=2, Hq=8, Hkv=2, T_max=1024, dtype=BF16, k_bits=(2,))
    k, v = synth.make_kv(44, 2, 1000, 2, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16)
    q = to_dev(synth.make_q(44, 2, 8, 128, BF16), BF16)
    a = gpu.attend(0, q).cpu().numpy()
    b = gpu.attend(0, q).cpu().numpy()
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_drifting_channel_means(kv, oracle):
    """Keys whose channel means drift along the sequence (the reasoning-style workload)."""
    print("case drift", flush=True)
    gpu, orc = make_pair(kv, oracle, B=1, Hq=8, Hkv=2, T_max=2048, dtype=BF16, k_bits=(2,))
    k, v = synth.make_kv(55, 1, 2000, 2, 128, BF16, n_drift=8, slope=0.01)
    append_both(gpu, orc, 0, k, v, BF16)
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(55, 1, 8, 128, BF16), BF16)


# ------------------------------------------------------------------ full size, sampled units


@pytest.mark.parametrize("decode_path", [0], indirect=True, ids=["auto"])
def test_full_cache_shape_sampled_units(kv, oracle, decode_path):
    """The benchmark's launch configuration (batch 16, 8 kv / 32 query heads, context 32768 plus a
    13-token raw tail, one layer per bit width): cache bytes and attention of sampled sequences
    against the oracle, which computes those sequences one by one."""
    import torch

    print("case full_cache_shape", flush=True)
    B, Hq, Hkv, d, G, T = 16, 32, 8, 128, 32, 32768 + 13
    bits = (2, 4, 8)
    cfg = kv.make_config(3, B, Hq, Hkv, d, 32768 + 64, G, G, G, kv.KV_BF16, kv.KV_MEAN_CHANNEL_BLOCK,
                         list(bits), list(bits))
    gpu = kv.KVCache(cfg, zero=False)
    sample = (0, 11)
    ocfg = oracle.OracleConfig(3, len(sample), Hq, Hkv, d, 32768 + 64, G, G, G, BF16, CHAN, list(bits), list(bits))
    orc = oracle.OracleCache(ocfg)
    for l in range(3):
        host_k, host_v = [], []
        for t0 in range(0, T, 8192):
            n = min(8192, T - t0)
            k, v = synth.make_kv_torch(900 + 10 * l + t0 // 8192, B, n, Hkv, d, BF16, "cuda:0")
            gpu.append(l, k, v)
            host_k.append(k[list(sample)].cpu())
            host_v.append(v[list(sample)].cpu())
        k16 = torch.cat(host_k, 1).view(torch.int16).numpy().view(np.uint16)
        v16 = torch.cat(host_v, 1).view(torch.int16).numpy().view(np.uint16)
        orc.append(l, k16, v16)
    torch.cuda.synchronize()
    for l in range(3):
        print("  layer %d (%d-bit) splits=%d" % (l, bits[l], kv.kv_decode_splits(gpu.handle, l)), flush=True)
        assert gpu.lengths(l) == (orc.packed_len(l), orc.resid_len(l)) == (32768, 13)
        lay = kv.kv_cache_describe(gpu.handle, l)
        img = orc.layer_image(l)  # image of a cache that holds only the sampled sequences
        NB = (32768 + 64) // G
        dev = gpu.layers[l]
        for si, b in enumerate(sample):
            # records of the 8 units of sequence b, and their raw residual rows
            n_rec = 32768 // G
            for h in range(Hkv):
                g0 = ((b * Hkv + h) * NB) * lay.rec_bytes
                o0 = ((si * Hkv + h) * NB) * lay.rec_bytes
                got = dev[g0:g0 + n_rec * lay.rec_bytes].cpu().numpy()
                want = img["bytes"][o0:o0 + n_rec * lay.rec_bytes]
                m = img["valid"][o0:o0 + n_rec * lay.rec_bytes]
                assert np.array_equal(got[m], want[m]), (l, b, h)
        q = synth.make_q_torch(77 + l, B, Hq, d, BF16, "cuda:0")
        out = gpu.attend(l, q)
        torch.cuda.synchronize()
        q16 = q[list(sample)].cpu().view(torch.int16).numpy().view(np.uint16)
        want = orc.attend(l, q16)
        got = out[list(sample)].cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(got - want)))
        print("  attention max-abs error %.3e" % err, flush=True)
        assert err <= 2e-3


def _full_size_sampled(kv, oracle, *, B, Hq, Hkv, G, T, bits, sample, seed, n_drift=0, decode_steps=0):
    """Fills one layer per bit width at a workload's full size on the GPU, re-does the sampled
    sequences with the oracle and compares their cache bytes and attention outputs; then
    `decode_steps` one-call decode steps (append + attend) checked the same way at the end."""
    import torch

    d, L = 128, len(bits)
    T_max = (T + decode_steps + G) // G * G + G
    cfg = kv.make_config(L, B, Hq, Hkv, d, T_max, G, G, G, kv.KV_BF16, kv.KV_MEAN_CHANNEL_BLOCK, list(bits), list(bits))
    gpu = kv.KVCache(cfg, zero=False)
    ocfg = oracle.OracleConfig(L, len(sample), Hq, Hkv, d, T_max, G, G, G, BF16, CHAN, list(bits), list(bits))
    orc = oracle.OracleCache(ocfg)
    as_u16 = lambda t: t.contiguous().view(torch.int16).numpy().view(np.uint16)
    for l in range(L):
        host_k, host_v = [], []
        for t0 in range(0, T, 8192):
            n = min(8192, T - t0)
            k, v = synth.make_kv_torch(seed + 10 * l + t0 // 8192, B, n, Hkv, d, BF16, "cuda:0", n_drift=n_drift, t0=t0)
            gpu.append(l, k, v)
            host_k.append(k[list(sample)].cpu())
            host_v.append(v[list(sample)].cpu())
        orc.append(l, as_u16(torch.cat(host_k, 1)), as_u16(torch.cat(host_v, 1)))
    for s in range(decode_steps):
        for l in range(L):
            k, v = synth.make_kv_torch(seed + 5000 + 10 * l + s, B, 1, Hkv, d, BF16, "cuda:0", n_drift=n_drift, t0=T + s)
            q = synth.make_q_torch(seed + 7000 + 10 * l + s, B, Hq, d, BF16, "cuda:0")
            out = gpu.append_attend(l, k, v, q)
            orc.append(l, as_u16(k[list(sample)].cpu()), as_u16(v[list(sample)].cpu()))
            if s == decode_steps - 1:
                torch.cuda.synchronize()
                want = orc.attend(l, as_u16(q[list(sample)].cpu()))
                err = float(np.max(np.abs(out[list(sample)].cpu().numpy().astype(np.float64) - want)))
                print("  layer %d after %d steps: attention max-abs error %.3e" % (l, decode_steps, err), flush=True)
                assert err <= 2e-3
    torch.cuda.synchronize()
    NB = T_max // G
    for l in range(L):
        print("  layer %d (%d-bit) splits=%d" % (l, bits[l], kv.kv_decode_splits(gpu.handle, l)), flush=True)
        assert gpu.lengths(l) == (orc.packed_len(l), orc.resid_len(l))
        lay = kv.kv_cache_describe(gpu.handle, l)
        img = orc.layer_image(l)  # image of a cache that holds only the sampled sequences
        dev = gpu.layers[l]
        n_rec = orc.packed_len(l) // G
        for si, b in enumerate(sample):
            for h in range(Hkv):
                g0 = ((b * Hkv + h) * NB) * lay.rec_bytes
                o0 = ((si * Hkv + h) * NB) * lay.rec_bytes
                got = dev[g0:g0 + n_rec * lay.rec_bytes].cpu().numpy()
                want = img["bytes"][o0:o0 + n_rec * lay.rec_bytes]
                m = img["valid"][o0:o0 + n_rec * lay.rec_bytes]
                assert np.array_equal(got[m], want[m]), (l, b, h)
        q = synth.make_q_torch(seed + 77 + l, B, Hq, d, BF16, "cuda:0")
        out = gpu.attend(l, q)
        torch.cuda.synchronize()
        want = orc.attend(l, as_u16(q[list(sample)].cpu()))
        err = float(np.max(np.abs(out[list(sample)].cpu().numpy().astype(np.float64) - want)))
        print("  attention max-abs error %.3e" % err, flush=True)
        assert err <= 2e-3
    gpu.close()


@pytest.mark.parametrize("decode_path", [0], indirect=True, ids=["auto"])
def test_long_context_full_size(kv, oracle, decode_path):
    """The 70B-shaped long-context workload at its full size (batch 1, 64 query / 8 kv heads, 131072
    tokens plus a raw tail, groups of 64, one layer per bit width) in the launch configuration
    the library picks for it."""
    print("case long_context_full", flush=True)
    _full_size_sampled(kv, oracle, B=1, Hq=64, Hkv=8, G=64, T=131072 + 29, bits=(2, 4, 8), sample=(0,), seed=1300)


@pytest.mark.parametrize("decode_path", [0], indirect=True, ids=["auto"])
def test_long_context_blocks_of_128(kv, oracle, decode_path):
    """Blocks and value groups of 128 (the group size of the paper's storage example, Sec. 3): a long
    sequence with 64 query / 8 kv heads and one with 32 / 8, one layer per bit width, a raw tail."""
    print("case long_context_g128", flush=True)
    _full_size_sampled(kv, oracle, B=1, Hq=64, Hkv=8, G=128, T=32768 + 128 + 77, bits=(2, 4, 8), sample=(0,), seed=1500)
    _full_size_sampled(kv, oracle, B=4, Hq=32, Hkv=8, G=128, T=8192 + 5, bits=(2, 4, 8), sample=(1, 3), seed=1510,
                       decode_steps=8)


@pytest.mark.parametrize("decode_path", [0], indirect=True, ids=["auto"])
def test_prefill_then_decode_full_size(kv, oracle, decode_path):
    """The prefill-then-decode workload at its full batch (64 sequences, 16384-token bulk prefill,
    drifting key channels, one layer per bit width), two sampled sequences, then 40 one-call decode
    steps that cross a block boundary."""
    print("case prefill_decode_full", flush=True)
    _full_size_sampled(kv, oracle, B=64, Hq=32, Hkv=8, G=32, T=16384, bits=(2, 4, 8), sample=(3, 60), seed=1400,
                       n_drift=8, decode_steps=40)


@pytest.mark.parametrize("decode_path", [0], indirect=True, ids=["auto"])
@pytest.mark.parametrize("bits,G,Hq,Hkv", [(4, 32, 32, 8), (2, 32, 32, 8), (8, 32, 32, 8), (4, 128, 32, 8), (2, 128, 32, 8),
                                            (8, 128, 32, 8),
                                            # eight query heads per kv head (two head groups per wave), four kv heads
                                            (8, 32, 32, 4), (8, 32, 64, 8), (4, 32, 64, 8), (2, 32, 16, 4)])
def test_full_cache_shape_cross_head_sampled_units(kv, oracle, decode_path, bits, G, Hq, Hkv):
    """The same launch configuration with the mean over the kv heads (Eq. 1-2), with groups of 32 and of
    128 (the format of the paper's Sec. 3 storage example): one layer of each width (4 bits: a workgroup
    of eight waves per sequence and split; 2 and 8 bits: two workgroups of four that share the split's
    mean rows), records, mean plane and attention of sampled sequences against the oracle."""
    import torch

    print("case full_cache_shape_cross_head bits=%d G=%d Hq=%d Hkv=%d" % (bits, G, Hq, Hkv), flush=True)
    B, d, T = 16, 128, 32768 + 13
    cap = 32768 + 2 * G
    cfg = kv.make_config(1, B, Hq, Hkv, d, cap, G, G, G, kv.KV_BF16, kv.KV_MEAN_CROSS_HEAD, [bits], [bits])
    gpu = kv.KVCache(cfg, zero=False)
    sample = (3, 15)
    ocfg = oracle.OracleConfig(1, len(sample), Hq, Hkv, d, cap, G, G, G, BF16, CROSS, [bits], [bits])
    orc = oracle.OracleCache(ocfg)
    host_k, host_v = [], []
    for t0 in range(0, T, 8192):
        n = min(8192, T - t0)
        k, v = synth.make_kv_torch(950 + t0 // 8192, B, n, Hkv, d, BF16, "cuda:0")
        gpu.append(0, k, v)
        host_k.append(k[list(sample)].cpu())
        host_v.append(v[list(sample)].cpu())
    k16 = torch.cat(host_k, 1).view(torch.int16).numpy().view(np.uint16)
    v16 = torch.cat(host_v, 1).view(torch.int16).numpy().view(np.uint16)
    orc.append(0, k16, v16)
    torch.cuda.synchronize()
    assert gpu.lengths(0) == (orc.packed_len(0), orc.resid_len(0)) == (32768, 13)
    lay = kv.kv_cache_describe(gpu.handle, 0)
    img = orc.layer_image(0)
    NB, n_rec = cap // G, 32768 // G
    dev = gpu.layers[0]
    olay = oracle.tada.record_layout(ocfg, 0)
    plane = 2 * G * d * 2  # bytes of one block's K and V mean rows
    for si, b in enumerate(sample):
        for h in range(Hkv):
            g0 = ((b * Hkv + h) * NB) * lay.rec_bytes
            o0 = ((si * Hkv + h) * NB) * lay.rec_bytes
            got = dev[g0:g0 + n_rec * lay.rec_bytes].cpu().numpy()
            m = img["valid"][o0:o0 + n_rec * lay.rec_bytes]
            assert np.array_equal(got[m], img["bytes"][o0:o0 + n_rec * lay.rec_bytes][m]), (b, h)
        g0, o0 = lay.xmean_off + b * NB * plane, olay["xmean_off"] + si * NB * plane
        got = dev[g0:g0 + n_rec * plane].cpu().numpy()
        assert img["valid"][o0:o0 + n_rec * plane].all()
        assert np.array_equal(got, img["bytes"][o0:o0 + n_rec * plane]), ("mean plane", b)
    q = synth.make_q_torch(79, B, Hq, d, BF16, "cuda:0")
    out = gpu.attend(0, q)
    torch.cuda.synchronize()
    q16 = q[list(sample)].cpu().view(torch.int16).numpy().view(np.uint16)
    want = orc.attend(0, q16)
    err = float(np.max(np.abs(out[list(sample)].cpu().numpy().astype(np.float64) - want)))
    print("  splits=%d attention max-abs error %.3e" % (kv.kv_decode_splits(gpu.handle, 0), err), flush=True)
    assert err <= 2e-3


# ------------------------------------------------------------------ cross-head mean (Eq. 1-2 as printed)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("Hkv,g", [(1, 1), (8, 4), (2, 8)])
@pytest.mark.parametrize("G", [32, 64, 128])
def test_cross_head_mean(kv, oracle, bits, Hkv, g, G):
    """The paper's own centring: the mean over the kv heads, one binary16 row per token shared by
    all heads.  With a single kv head the deviation is zero and the cache recovers fp16 inputs."""
    print("case cross_head bits=%d Hkv=%d g=%d G=%d" % (bits, Hkv, g, G), flush=True)
    T = 3 * G + 7
    gpu, orc = make_pair(kv, oracle, B=2, Hq=Hkv * g, Hkv=Hkv, T_max=4 * G, G=G, Gc=G, dtype=F16, mode=CROSS,
                         k_bits=(bits,))
    k, v = synth.make_kv(300 + bits + Hkv, 2, T, Hkv, 128, F16)
    append_both(gpu, orc, 0, k, v, F16, chunks=[2 * G + 3, 1, 1, G - 5 + 7])
    check_bytes(gpu, orc, 0)
    check_attention(gpu, orc, 0, synth.make_q(bits, 2, Hkv * g, 128, F16), F16)


def test_cross_head_mean_mixed_layers_bf16(kv, oracle):
    print("case cross_head_mixed", flush=True)
    bits = (4, 16, 2)
    gpu, orc = make_pair(kv, oracle, L=3, B=1, Hq=32, Hkv=8, T_max=512, dtype=BF16, mode=CROSS, k_bits=bits)
    for l in range(3):
        k, v = synth.make_kv(400 + l, 1, 300, 8, 128, BF16)
        append_both(gpu, orc, l, k, v, BF16)
        check_bytes(gpu, orc, l)
        check_attention(gpu, orc, l, synth.make_q(l, 1, 32, 128, BF16), BF16)


@pytest.mark.parametrize("decode_path", [2], indirect=True, ids=["mfma"])
@pytest.mark.parametrize("bits,G,g,T,Hkv", [(4, 32, 3, 2000 + 13, 4), (2, 32, 5, 1056, 4), (8, 64, 4, 1600 + 40, 4),
                                            (4, 64, 8, 704, 4), (4, 128, 4, 2048 + 128 + 50, 4), (2, 128, 8, 1280, 4),
                                            (8, 128, 3, 1664 + 7, 4), (4, 128, 6, 1536 + 128 + 9, 8), (2, 128, 2, 2304 + 1, 8), (8, 32, 4, 1500 + 9, 8), (2, 32, 8, 1056 + 32, 8),
                                            (4, 64, 5, 1344 + 3, 8), (8, 64, 8, 960, 8), (2, 64, 2, 2048 + 70, 8),
                                            (4, 32, 4, 1120 + 31, 8), (4, 32, 2, 700, 2),
                                            # the remaining instances of the form with both mean terms inside the kernel
                                            (4, 32, 6, 900 + 7, 8), (8, 32, 8, 1200 + 5, 4), (2, 32, 3, 1300, 4),
                                            (4, 64, 4, 1100 + 64, 8), (4, 64, 2, 1000, 4), (2, 64, 7, 900 + 1, 4),
                                            (8, 128, 6, 1536 + 20, 8), (4, 128, 3, 1400, 8), (8, 32, 7, 2100 + 3, 8),
                                            # more kv heads: three, four or eight workgroups share a sequence's split
                                            (4, 32, 1, 1100 + 7, 32), (2, 64, 2, 900, 16), (8, 32, 1, 1300, 32),
                                            (4, 128, 3, 1500, 12), (4, 32, 2, 1000 + 5, 24), (8, 64, 5, 800, 12)])
def test_cross_head_mean_on_the_matrix_cores(kv, oracle, decode_path, bits, G, g, T, Hkv):
    """Cross-head mean with the deviations on the matrix-core kernel; the two dense mean terms inside
    that kernel (a multiple of 4 kv heads: a workgroup of 4 or 8 waves, or several that share a sequence's
    split, with one or two groups of four query heads per kv head; blocks of 128 tokens as two halves) or
    in kernels of their own (other head counts);
    several splits, an odd block count, a raw tail."""
    print("case cross_head_mfma bits=%d G=%d g=%d T=%d Hkv=%d" % (bits, G, g, T, Hkv), flush=True)
    gpu, orc = make_pair(kv, oracle, B=2, Hq=Hkv * g, Hkv=Hkv, T_max=(T // G + 2) * G, G=G, Gc=G, dtype=BF16, mode=CROSS,
                         k_bits=(bits,))
    k, v = synth.make_kv(500 + bits + g, 2, T, Hkv, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16, chunks=[T - 1, 1])
    check_bytes(gpu, orc, 0)
    q = synth.make_q(500 + bits, 2, Hkv * g, 128, BF16)
    check_attention(gpu, orc, 0, q, BF16)
    import torch
    a = gpu.attend(0, to_dev(q, BF16))
    b = gpu.attend(0, to_dev(q, BF16))
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("decode_path", [2], indirect=True, ids=["mfma"])
def test_cross_head_mean_with_a_forced_split_count(kv, oracle, decode_path):
    """A forced split count above the automatic one moves the dense mean arrays further back in the
    workspace: the stock workspace is refused, one of kv_decode_workspace_need's size gives the
    oracle's attention (the partials of 64 splits would otherwise run into those arrays)."""
    import torch

    print("case cross_head_forced_splits", flush=True)
    B, Hkv, g, T = 16, 6, 4, 128 * 32 + 5
    # (6 kv heads: a format whose dense mean terms run as kernels of their own and pass through the workspace)
    gpu, orc = make_pair(kv, oracle, B=B, Hq=Hkv * g, Hkv=Hkv, T_max=33 * 128, G=128, Gc=128, dtype=BF16, mode=CROSS,
                         k_bits=(4,))
    k, v = synth.make_kv(611, B, T, Hkv, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16)
    q = synth.make_q(611, B, Hkv * g, 128, BF16)
    auto = kv.kv_decode_splits(gpu.handle, 0)
    stock = gpu.ws_bytes
    assert kv.kv_decode_workspace_need(gpu.handle, 0) <= stock
    kv.kv_set_decode_splits(gpu.handle, 64)
    assert auto < kv.kv_decode_splits(gpu.handle, 0) <= 64
    need = kv.kv_decode_workspace_need(gpu.handle, 0)
    assert need > stock
    with pytest.raises(kv.KVError) as e:
        gpu.attend(0, to_dev(q, BF16))
    assert e.value.status == kv.KV_E_WORKSPACE
    gpu.workspace = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    gpu.ws_bytes = need
    check_attention(gpu, orc, 0, q, BF16, units=[(0, 0), (7, 3), (15, 5)])


# ------------------------------------------------------------------ matrix-core kernels, forced


@pytest.mark.parametrize("decode_path", [2], indirect=True, ids=["mfma"])
@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("g", [1, 3, 4, 5, 8])
@pytest.mark.parametrize("G,mode", [(32, CHAN), (64, CHAN), (64, NONE), (128, CHAN), (128, NONE)])
def test_matrix_core_kernels(kv, oracle, decode_path, bits, g, G, mode):
    """Path 2 refuses to fall back, so these cases prove the int8 matrix-core kernels themselves:
    one and two head groups per wave, both block sizes, with and without block means, a partial
    last chunk and a raw tail."""
    print("case mfma bits=%d g=%d G=%d mode=%d" % (bits, g, G, mode), flush=True)
    Hkv = 2
    T = 21 * G + 9  # odd block count: the last 64-token chunk of a G=32 cache is half empty
    gpu, orc = make_pair(kv, oracle, B=2, Hq=Hkv * g, Hkv=Hkv, T_max=24 * G, G=G, Gc=G, dtype=BF16, mode=mode,
                         k_bits=(bits,))
    k, v = synth.make_kv(500 + bits + g, 2, T, Hkv, 128, BF16)
    append_both(gpu, orc, 0, k, v, BF16)
    check_bytes(gpu, orc, 0)
    q = synth.make_q(g, 2, Hkv * g, 128, BF16)
    check_attention(gpu, orc, 0, q, BF16)
    for ns in (1, 3):
        kv.kv_set_decode_splits(gpu.handle, ns)
        check_attention(gpu, orc, 0, q, BF16)


@pytest.mark.parametrize("decode_path", [2], indirect=True, ids=["mfma"])
def test_long_context_70b_shape(kv, oracle, decode_path):
    """64 query / 8 kv heads (two head groups per wave), batch 1, group size 64, a mixed layer map
    with 8-bit ends, outlier channels: the long-context workload at a reduced context."""
    print("case 70b_shape", flush=True)
    bits = (8, 2, 4, 8)
    gpu, orc = make_pair(kv, oracle, L=4, B=1, Hq=64, Hkv=8, T_max=8192 + 64, G=64, Gc=64, dtype=BF16, k_bits=bits)
    for l in range(4):
        k, v = synth.make_kv(600 + l, 1, 8192 + 17, 8, 128, BF16)
        append_both(gpu, orc, l, k, v, BF16, chunks=[8192, 17])
        check_bytes(gpu, orc, l)
        check_attention(gpu, orc, l, synth.make_q(l, 1, 64, 128, BF16), BF16)


@pytest.mark.parametrize("decode_path", [2, 1], indirect=True, ids=["mfma", "valu"])
def test_prefill_then_decode_steps_with_drift(kv, oracle, decode_path):
    """Bulk prefill, then decode steps that append one token and attend, on keys whose channel
    means drift along the sequence; checked after every few steps and across a block flush."""
    print("case prefill_decode", flush=True)
    bits = (2, 8, 4)
    gpu, orc = make_pair(kv, oracle, L=3, B=3, Hq=8, Hkv=2, T_max=1024 + 64, dtype=BF16, k_bits=bits)
    steps = 40
    for l in range(3):
        k, v = synth.make_kv(700 + l, 3, 1024 + steps, 2, 128, BF16, n_drift=8, slope=0.01)
        append_both(gpu, orc, l, k[:, :1024], v[:, :1024], BF16)
        for s in range(steps):
            append_both(gpu, orc, l, k[:, 1024 + s:1025 + s], v[:, 1024 + s:1025 + s], BF16)
            if s % 13 == 0 or s in (31, 32, steps - 1):
                check_attention(gpu, orc, l, synth.make_q(l * 100 + s, 3, 8, 128, BF16), BF16)
        check_bytes(gpu, orc, l)


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("mode", [CHAN, CROSS])
def test_output_in_the_16_bit_type(kv, oracle, dtype, mode):
    """The narrowing merge: the 32-bit result rounded to nearest even in the cache's 16-bit type.
    Bitwise against the 32-bit output of the same cache; against the oracle within 2e-3 plus half a
    unit in the last place of the 16-bit type."""
    import torch

    print("case out16 dtype=%d mode=%d" % (dtype, mode), flush=True)
    gpu, orc = make_pair(kv, oracle, B=2, Hq=8, Hkv=2, T_max=1024 + 64, dtype=dtype, mode=mode, k_bits=(4,))
    k, v = synth.make_kv(810 + dtype, 2, 1024 + 9, 2, 128, dtype)
    append_both(gpu, orc, 0, k, v, dtype)
    q = synth.make_q(811, 2, 8, 128, dtype)
    qd = to_dev(q, dtype)
    out32 = gpu.attend(0, qd)
    out16 = gpu.attend16(0, qd)
    torch.cuda.synchronize()
    assert out16.dtype == qd.dtype
    assert torch.equal(out16, out32.to(out16.dtype)), "narrowing differs from round-to-nearest-even of the 32-bit output"
    want = orc.attend(0, q)
    half_ulp = 2.0 ** (-9 if dtype == BF16 else -12)
    err = np.abs(out16.float().cpu().numpy().astype(np.float64) - want)
    assert np.all(err <= ATTN_TOL + half_ulp * np.abs(want) + 1e-7)


# ------------------------------------------------------------------ degenerate inputs


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("mode", [CHAN, CROSS, NONE])
def test_degenerate_values(kv, oracle, bits, mode):
    """Groups with zero range (scale 0), all-zero tokens, zeros of both signs, binary16-subnormal
    magnitudes and a few large values: same bytes as the oracle, finite attention."""
    print("case degenerate bits=%d mode=%d" % (bits, mode), flush=True)
    B, Hkv, g, G, T = 2, 2, 4, 32, 4 * 32 + 5
    rng = np.random.default_rng(800 + bits)
    x = np.zeros((2, B, T, Hkv, 128), dtype=np.float32)
    x[:, :, 0:32] = 0.0                                  # an all-zero block
    x[:, :, 32:64] = 1.5                                 # a constant block: every group has zero range
    x[:, :, 64:96] = rng.standard_normal((2, B, 32, Hkv, 128)) * 1e-6   # below binary16 normal range
    x[:, :, 96:] = rng.standard_normal((2, B, T - 96, Hkv, 128))
    x[:, :, 96:128, :, 5] = 0.0                          # a constant channel inside a varying block
    x[:, :, 100, :, :] = 0.0                             # a constant token (value groups of zero range)
    x[:, :, 110, :, 7] = 300.0                           # outliers
    x[:, :, 111, :, 9] = -250.0
    kb = synth.f32_to_bits16(x[0], F16)
    vb = synth.f32_to_bits16(x[1], F16)
    kb[:, 1:32:2] |= 0x8000                              # negative zeros among the zeros
    vb[:, 100, :, ::3] |= 0x8000
    gpu, orc = make_pair(kv, oracle, B=B, Hq=Hkv * g, Hkv=Hkv, T_max=6 * G, G=G, Gc=G, dtype=F16, mode=mode, k_bits=(bits,))
    append_both(gpu, orc, 0, kb, vb, F16, chunks=[40, T - 40])
    check_bytes(gpu, orc, 0)
    # Two bounds, one per kernel family (the error model of include/tadakv.h).  The vector-ALU kernels
    # accumulate in binary32 throughout and stay within the stated 2e-3 on these inputs too (outputs reach
    # +-300: that is 7e-6 relative).  The matrix-core kernels carry q*scale and p*scale as 23-bit fixed
    # point relative to the largest such weight of a block / 64-token chunk, which costs up to
    # 1.6e-5 x the largest range of a quantisation group: 2e-3 holds up to ranges of 128 (the workloads'
    # are below 30), and the planted values of 300 make the bound 4.9e-3 here.
    q = synth.make_q(800 + bits, B, Hkv * g, 128, F16)
    assert kv.kv_decode_path_used(gpu.handle, 0) == (1 if parity_util.DECODE_PATH == 1 else 2)
    group_range = 300.0 + 2 * 4.5  # the outlier against a group of N(0,1) values
    bound = 2e-3 if parity_util.DECODE_PATH == 1 else max(2e-3, 1.6e-5 * group_range)
    err = check_attention(gpu, orc, 0, q, F16, tol=bound)
    print("  attention max-abs error %.3e (bound %.1e)" % (err, bound), flush=True)

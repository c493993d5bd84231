"""GPU parity of paged placement (block slots shared through a block table): the same contents as
dense placement, found where the table says.  The oracle keeps its dense image; the test gathers the
GPU's records through the table before comparing bytes."""
import numpy as np
import pytest

from paper_2506_04642_amd import synth
import parity_util
from parity_util import ATTN_TOL, to_dev

pytestmark = pytest.mark.gpu

BF16 = 1
CHAN, CROSS, NONE = 0, 1, 2


@pytest.fixture(scope="module")
def kv():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_04642_amd import binding

    return binding


def make_paged(kv, oracle, *, B, Hkv, g, T_max, G, R, mode, bits, pool, seed, path):
    import torch

    cfg = kv.make_config(1, B, Hkv * g, Hkv, 128, T_max, G, G, R, BF16, mode, [bits], [bits], pool_blocks=pool)
    ocfg = oracle.OracleConfig(1, B, Hkv * g, Hkv, 128, T_max, G, G, R, BF16, mode, [bits], [bits])
    gpu = kv.KVCache(cfg, zero=True)
    kv.kv_set_decode_path(gpu.handle, path)
    NB = T_max // G
    # every slot is handed out once, in a seeded order; the rest of the table holds out-of-range
    # entries, which no kernel may follow (and which are clamped if one did)
    rng = np.random.default_rng(seed)
    table = np.full((B, NB + 3), 10 ** 6, dtype=np.int32)
    table[:, NB:] = -7
    slots = rng.permutation(pool)
    return gpu, oracle.OracleCache(ocfg), table, list(slots)


def give_blocks(table, slots, b, upto_blocks):
    """Sequence b gets slots for its logical blocks below upto_blocks."""
    for j in range(upto_blocks):
        if table[b, j] >= 10 ** 6:
            table[b, j] = slots.pop()


def push_table(gpu, table):
    import torch

    if not hasattr(gpu, "_table"):
        gpu.set_block_table(torch.from_numpy(table.copy()).to("cuda:0"))
    else:
        gpu._table.copy_(torch.from_numpy(table))


def check_bytes_paged(kv, oracle, gpu, orc, table):
    import torch

    torch.cuda.synchronize()
    cfg = orc.cfg
    H, G, d, B = cfg.n_kv_heads, cfg.group_tokens, cfg.head_dim, cfg.batch
    NB = cfg.max_tokens // G
    img = orc.layer_image(0)
    lo = oracle.record_layout(cfg, 0)
    lg = kv.kv_cache_describe(gpu.handle, 0)
    got = gpu.layers[0].cpu().numpy()
    REC = lg.rec_bytes
    assert REC == lo["rec_bytes"]
    for b in range(B):
        assert gpu.lengths(0, b) == (orc.packed_len(0, b), orc.resid_len(0, b))
        for j in range(orc.packed_len(0, b) // G):
            p = int(table[b, j])
            for h in range(H):
                go, oo = (p * H + h) * REC, ((b * H + h) * NB + j) * REC
                m = img["valid"][oo:oo + REC]
                assert m.any()
                assert np.array_equal(got[go:go + REC][m], img["bytes"][oo:oo + REC][m]), (b, j, h)
            if cfg.mean_mode == CROSS:
                sz = 2 * G * d * 2
                go, oo = lg.xmean_off + p * sz, lo["xmean_off"] + (b * NB + j) * sz
                m = img["valid"][oo:oo + sz]
                assert np.array_equal(got[go:go + sz][m], img["bytes"][oo:oo + sz][m]), (b, j)
    sz = B * H * cfg.resid_cap * d * 2
    for name in ("k_resid_off", "v_resid_off"):
        go, oo = getattr(lg, name), lo[name]
        m = img["valid"][oo:oo + sz]
        assert np.array_equal(got[go:go + sz][m], img["bytes"][oo:oo + sz][m]), name


@pytest.mark.parametrize("path", [0, 1], ids=["auto", "valu"])
@pytest.mark.parametrize("bits,G,R,mode,g,Hkv", [(4, 32, 32, CHAN, 4, 2), (2, 64, 64, CHAN, 8, 2), (8, 32, 64, NONE, 2, 2),
                                                 (4, 32, 32, CROSS, 4, 2), (2, 64, 64, CROSS, 2, 2), (8, 128, 128, CHAN, 8, 2),
                                                 (2, 128, 128, NONE, 3, 2), (4, 128, 128, CROSS, 4, 2),
                                                 # a multiple of 4 kv heads: the cross-head mean's terms inside the matrix-core kernel
                                                 (4, 32, 32, CROSS, 4, 8), (2, 64, 64, CROSS, 2, 4), (8, 128, 128, CROSS, 3, 4),
                                                 (8, 32, 64, CROSS, 8, 8), (4, 128, 128, CROSS, 4, 8), (2, 32, 32, CROSS, 6, 4)])
def test_paged_prompts_then_decode_steps(kv, oracle, bits, G, R, mode, g, Hkv, path):
    """Prompts of different lengths enter their slots one by one (slots handed out as needed, in a
    shuffled order, from a pool smaller than batch x capacity), then batch-wide one-call decode steps
    run across block boundaries while new slots are handed out."""
    import torch

    print("case paged bits=%d G=%d R=%d mode=%d g=%d Hkv=%d path=%d" % (bits, G, R, mode, g, Hkv, path), flush=True)
    B = 4
    NB = 12
    gpu, orc, table, slots = make_paged(kv, oracle, B=B, Hkv=Hkv, g=g, T_max=NB * G, G=G, R=R, mode=mode, bits=bits,
                                        pool=26, seed=50 + bits + G, path=path)
    prompts = {0: 5 * G + 3, 1: 17, 3: 7 * G + G - 2}  # slot 2 stays empty for now
    steps = R + 5
    for b, n in prompts.items():
        give_blocks(table, slots, b, (n + steps) // G + 1)
    give_blocks(table, slots, 2, steps // G + 1)
    push_table(gpu, table)
    seed = 700 + bits + G
    for b, n in prompts.items():
        k, v = synth.make_kv(seed + b, 1, n, Hkv, 128, BF16)
        gpu.append_seq(0, b, to_dev(k[0], BF16), to_dev(v[0], BF16))
        orc.append_seq(0, b, k[0], v[0])
    check_bytes_paged(kv, oracle, gpu, orc, table)
    q = synth.make_q(seed, B, Hkv * g, 128, BF16)
    out = gpu.attend(0, to_dev(q, BF16))
    torch.cuda.synchronize()
    assert float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - orc.attend(0, q)))) <= ATTN_TOL
    ks, vs = synth.make_kv(seed + 50, B, steps, Hkv, 128, BF16)
    kd, vd = to_dev(ks, BF16), to_dev(vs, BF16)
    for s in range(steps):
        q = synth.make_q(seed * 7 + s, B, Hkv * g, 128, BF16)
        out = gpu.append_attend(0, kd[:, s:s + 1], vd[:, s:s + 1], to_dev(q, BF16))
        orc.append(0, ks[:, s:s + 1], vs[:, s:s + 1])
        torch.cuda.synchronize()
        err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - orc.attend(0, q))))
        assert err <= ATTN_TOL, "step %d: %.3e" % (s, err)
    check_bytes_paged(kv, oracle, gpu, orc, table)

    # sequence 3 leaves; its slots go back to the pool and a new prompt takes them, in another order
    kv.kv_cache_reset_seq(gpu.handle, 0, 3)
    orc.reset_seq(0, 3)
    freed = [int(x) for x in table[3, :NB] if x < 10 ** 6]
    table[3, :NB] = 10 ** 6
    slots.extend(freed[::-1])
    n = 3 * G + 11
    give_blocks(table, slots, 3, n // G + 1)
    push_table(gpu, table)
    k, v = synth.make_kv(seed + 99, 1, n, Hkv, 128, BF16)
    gpu.append_seq(0, 3, to_dev(k[0], BF16), to_dev(v[0], BF16))
    orc.append_seq(0, 3, k[0], v[0])
    q = synth.make_q(seed + 5, B, Hkv * g, 128, BF16)
    out = gpu.attend(0, to_dev(q, BF16))
    torch.cuda.synchronize()
    assert float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - orc.attend(0, q)))) <= ATTN_TOL
    check_bytes_paged(kv, oracle, gpu, orc, table)


def test_paged_bulk_append_with_rotation(kv, oracle):
    """Bulk rotate-and-append of a uniform batch into shuffled slots."""
    import torch

    print("case paged rope", flush=True)
    B, Hkv, g, G = 2, 2, 4, 32
    NB = 8
    gpu, orc, table, slots = make_paged(kv, oracle, B=B, Hkv=Hkv, g=g, T_max=NB * G, G=G, R=G, mode=CHAN, bits=4, pool=12,
                                        seed=3, path=0)
    T = 5 * G + 9
    for b in range(B):
        give_blocks(table, slots, b, T // G + 1)
    push_table(gpu, table)
    k, v = synth.make_kv(880, B, T, Hkv, 128, BF16)
    cos, sin = synth.rope_tables(np.arange(100, 100 + T), 128, 500000.0)
    gpu.append_rope(0, to_dev(k, BF16), to_dev(v, BF16), torch.from_numpy(cos).to("cuda:0"),
                    torch.from_numpy(sin).to("cuda:0"), 0)
    orc.append(0, k, v, rope_tables=(cos, sin, 0))
    check_bytes_paged(kv, oracle, gpu, orc, table)
    q = synth.make_q(881, B, Hkv * g, 128, BF16)
    out = gpu.attend(0, to_dev(q, BF16))
    torch.cuda.synchronize()
    assert float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - orc.attend(0, q)))) <= ATTN_TOL


@pytest.mark.parametrize("bits,G,Hkv,g", [(4, 32, 8, 4), (2, 64, 4, 2), (8, 128, 4, 5)])
def test_paged_cross_head_long_sequence_single_split(kv, oracle, bits, G, Hkv, g):
    """Mean over the heads under paged placement, one split: a wave takes 80 chunks and more of its head,
    so the window of block slots that it keeps (64 chunks) moves while the mean rows of the chunk after
    the next are looked up through it."""
    import torch

    print("case paged cross long bits=%d G=%d Hkv=%d g=%d" % (bits, G, Hkv, g), flush=True)
    B = 2
    T = 64 * 83 + G // 2 + 3
    NB = T // G + 2
    gpu, orc, table, slots = make_paged(kv, oracle, B=B, Hkv=Hkv, g=g, T_max=NB * G, G=G, R=G, mode=CROSS, bits=bits,
                                        pool=2 * NB - 1, seed=700 + bits, path=2)
    for b, n in enumerate((T, T - 64 * 9 - 5)):
        give_blocks(table, slots, b, n // G + 1)
    push_table(gpu, table)
    for b, n in enumerate((T, T - 64 * 9 - 5)):
        k, v = synth.make_kv(710 + b, 1, n, Hkv, 128, BF16)
        gpu.append_seq(0, b, to_dev(k[0], BF16), to_dev(v[0], BF16))
        orc.append_seq(0, b, k[0], v[0])
    check_bytes_paged(kv, oracle, gpu, orc, table)
    kv.kv_set_decode_splits(gpu.handle, 1)
    assert kv.kv_decode_splits(gpu.handle, 0) == 1
    q = synth.make_q(720, B, Hkv * g, 128, BF16)
    out = gpu.attend(0, to_dev(q, BF16))
    torch.cuda.synchronize()
    assert float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - orc.attend(0, q)))) <= ATTN_TOL


@pytest.mark.parametrize("mode,Hkv,G", [(CHAN, 2, 32), (CROSS, 4, 32), (CROSS, 8, 64)])
def test_paged_decode_steps_replayed_from_one_graph(kv, oracle, mode, Hkv, G):
    """Decode steps on device-resident lengths over a paged cache: the blocks that the replayed steps will
    fill have their slots beforehand; every replay equals the eager one-call step on a twin cache with
    the same table bit for bit (same split count), the oracle within the tolerance, and at the end the
    records gathered through the table are the oracle's."""
    import torch

    print("case paged graph steps mode=%d Hkv=%d G=%d" % (mode, Hkv, G), flush=True)
    B, g, steps = 3, 2, G + 12
    NB = 12
    prompts = [5 * G + G - 2, G - 15, 2 * G + 3]
    caches = []
    for _ in range(3):  # the replayed cache, its eager twin, one for the one-time queries outside the capture
        gpu, orc, table, slots = make_paged(kv, oracle, B=B, Hkv=Hkv, g=g, T_max=NB * G, G=G, R=G, mode=mode, bits=4,
                                            pool=3 * NB - 4, seed=900 + G, path=2)
        for b, n in enumerate(prompts):
            give_blocks(table, slots, b, (n + steps) // G + 1)
        push_table(gpu, table)
        kv.kv_set_decode_splits(gpu.handle, 2)
        caches.append((gpu, orc, table))
    (gpu, orc, table), (twin, _, _), (warm, _, _) = caches
    for b, n in enumerate(prompts):
        k, v = synth.make_kv(910 + b, 1, n, Hkv, 128, BF16)
        for c in (gpu, twin, warm):
            c.append_seq(0, b, to_dev(k[0], BF16), to_dev(v[0], BF16))
        orc.append_seq(0, b, k[0], v[0])
    ks, vs = synth.make_kv(920, B, steps, Hkv, 128, BF16)
    kd, vd = to_dev(ks, BF16), to_dev(vs, BF16)
    k_st = torch.zeros((B, Hkv, 128), dtype=torch.bfloat16, device="cuda:0")
    v_st = torch.zeros_like(k_st)
    q_st = torch.zeros((B, Hkv * g, 128), dtype=torch.bfloat16, device="cuda:0")
    o_st = torch.zeros((B, Hkv * g, 128), dtype=torch.float32, device="cuda:0")
    warm.lengths_to_device()
    warm.step_dev(0, k_st, v_st, q_st, o_st)
    torch.cuda.synchronize()
    gpu.lengths_to_device()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        gpu.step_dev(0, k_st, v_st, q_st, o_st)
    torch.cuda.synchronize()
    for s_ in range(steps):
        q = synth.make_q(930 + s_, B, Hkv * g, 128, BF16)
        k_st.copy_(kd[:, s_])
        v_st.copy_(vd[:, s_])
        q_st.copy_(to_dev(q, BF16))
        o_st.zero_()
        graph.replay()
        eager = twin.append_attend(0, kd[:, s_:s_ + 1], vd[:, s_:s_ + 1], to_dev(q, BF16))
        torch.cuda.synchronize()
        assert torch.equal(o_st, eager), "step %d differs from the eager step" % s_
        orc.append(0, ks[:, s_:s_ + 1], vs[:, s_:s_ + 1])
        if s_ % 9 == 0 or s_ == steps - 1:
            assert float(np.max(np.abs(o_st.cpu().numpy().astype(np.float64) - orc.attend(0, q)))) <= ATTN_TOL, s_
    gpu.advance(steps)
    for b in range(B):
        assert gpu.lengths(0, b) == twin.lengths(0, b) == (orc.packed_len(0, b), orc.resid_len(0, b))
    check_bytes_paged(kv, oracle, gpu, orc, table)


def test_paged_cache_needs_a_table(kv, oracle):
    import torch

    print("case paged errors", flush=True)
    cfg = kv.make_config(1, 1, 4, 1, 128, 128, 32, 32, 32, BF16, CHAN, [4], [4], pool_blocks=3)
    gpu = kv.KVCache(cfg)
    k = torch.zeros((1, 1, 1, 128), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(kv.KVError) as e:
        gpu.append(0, k, k)
    assert e.value.status == kv.KV_E_BAD_CONFIG
    with pytest.raises(kv.KVError) as e:
        kv.kv_cache_set_block_table(gpu.handle, 0, 4)
    assert e.value.status == kv.KV_E_NULL
    t = torch.zeros((1, 3), dtype=torch.int32, device="cuda:0")
    with pytest.raises(kv.KVError) as e:
        gpu.set_block_table(t)  # stride below max_tokens / G
    assert e.value.status == kv.KV_E_BAD_CONFIG
    dense = kv.KVCache(kv.make_config(1, 1, 4, 1, 128, 128, 32, 32, 32, BF16, CHAN, [4], [4]))
    with pytest.raises(kv.KVError) as e:
        dense.set_block_table(torch.zeros((1, 4), dtype=torch.int32, device="cuda:0"))
    assert e.value.status == kv.KV_E_BAD_CONFIG

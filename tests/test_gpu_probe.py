"""The streaming-read probe that the benchmark uses as its measured bandwidth ceiling: it must run
over any size (whole 16-byte pieces), leave the buffer alone and refuse bad arguments."""
import pytest

pytestmark = pytest.mark.gpu


def test_stream_read_probe_runs_and_writes_nothing():
    import torch

    from paper_2506_04642_amd import binding as kv

    print("case stream_read_probe", flush=True)
    buf = torch.arange(0, (3 << 20) + 5, dtype=torch.int64, device="cuda:0")
    ref = buf.clone()
    sink = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    for nbytes in (16, 4096, 65536 + 48, buf.numel() * 8):
        kv.kv_stream_read_probe(buf.data_ptr(), nbytes, sink.data_ptr(), st)
        kv.kv_stream_read_probe(buf.data_ptr() + 16, nbytes - 16 if nbytes > 16 else 16, 0, st)
    torch.cuda.synchronize()
    assert torch.equal(buf, ref) and int(sink.item()) == 0
    for args, status in (((0, 64, 0, 0), kv.KV_E_NULL), ((buf.data_ptr() + 8, 64, 0, 0), kv.KV_E_ALIGN),
                         ((buf.data_ptr(), 8, 0, 0), kv.KV_E_BAD_CONFIG)):
        with pytest.raises(kv.KVError) as e:
            kv.kv_stream_read_probe(*args)
        assert e.value.status == status


def test_split_kernel_stamps_its_own_events():
    """kv_time_next_split: the next matrix-core split launch records its begin and end into the two
    events; the time between them is positive, no longer than what events recorded around the call
    measure, the request is one-shot, and the attention result is what it is without it."""
    import numpy as np
    import torch

    from paper_2506_04642_amd import binding as kv, synth

    print("case kv_time_next_split", flush=True)
    B, Hq, Hkv, T = 2, 8, 2, 4096 + 7
    cfg = kv.make_config(1, B, Hq, Hkv, 128, 8192, 32, 32, 32, kv.KV_BF16, kv.KV_MEAN_CHANNEL_BLOCK, [4], [4])
    cache = kv.KVCache(cfg)
    k, v = synth.make_kv_torch(11, B, T, Hkv, 128, synth.BF16, "cuda:0")
    q = synth.make_q_torch(12, B, Hq, 128, synth.BF16, "cuda:0")
    cache.append(0, k, v)
    assert kv.kv_decode_path_used(cache.handle, 0) == 2
    want = cache.attend(0, q).clone()
    stream = torch.cuda.current_stream()
    ws, wsb, sp = cache.workspace.data_ptr(), cache.ws_bytes, stream.cuda_stream
    out = torch.empty_like(want)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for e in ev:
        e.record(stream)  # (the handles exist from here on)
    torch.cuda.synchronize()
    inner, outer = [], []
    for rep in range(5):
        ev[2].record(stream)
        kv.kv_time_next_split(ev[0].cuda_event, ev[1].cuda_event)
        kv.kv_decode_attn_split(cache.handle, 0, q.data_ptr(), ws, wsb, sp)
        ev[3].record(stream)
        kv.kv_decode_attn_merge(cache.handle, 0, out.data_ptr(), ws, wsb, sp)
        torch.cuda.synchronize()
        inner.append(ev[0].elapsed_time(ev[1]))
        outer.append(ev[2].elapsed_time(ev[3]))
        assert torch.equal(out, want)
    assert min(inner) > 0.0
    assert np.median(inner) <= np.median(outer) * 1.02
    # one-shot: a launch without a new request leaves the events as they are
    before = ev[0].elapsed_time(ev[1])
    kv.kv_decode_attn_split(cache.handle, 0, q.data_ptr(), ws, wsb, sp)
    torch.cuda.synchronize()
    assert ev[0].elapsed_time(ev[1]) == before
    # one of the two missing
    with pytest.raises(kv.KVError) as e:
        kv.kv_time_next_split(ev[0].cuda_event, 0)
    assert e.value.status == kv.KV_E_NULL
    kv.kv_time_next_split(0, 0)
    cache.close()

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

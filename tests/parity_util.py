"""Shared driver for the GPU parity tests: feeds the same seeded 16-bit inputs to the HIP path
(through the C ABI) and to the CPU oracle, and compares cache bytes and attention outputs."""
import numpy as np

from paper_2506_04642_amd import synth

ATTN_TOL = 2e-3  # max-abs error of the attention output against the binary64 oracle
DECODE_PATH = 0  # 0 automatic, 1 vector-ALU kernels, 2 matrix-core kernels (set by the tests)


def to_dev(bits16: np.ndarray, dtype: int, device="cuda:0"):
    import torch

    t = torch.from_numpy(np.ascontiguousarray(bits16).view(np.int16))
    return t.view(torch.float16 if dtype == synth.F16 else torch.bfloat16).to(device)


def make_pair(kv, oracle, *, L=1, B=1, Hq=1, Hkv=1, T_max=1024, G=32, Gc=32, R=None, dtype=0, mode=0,
              k_bits=(4,), v_bits=None, zero=True):
    v_bits = k_bits if v_bits is None else v_bits
    R = G if R is None else R
    cfg = kv.make_config(L, B, Hq, Hkv, 128, T_max, G, Gc, R, dtype, mode, list(k_bits), list(v_bits))
    ocfg = oracle.OracleConfig(L, B, Hq, Hkv, 128, T_max, G, Gc, R, dtype, mode, list(k_bits), list(v_bits))
    gpu = kv.KVCache(cfg, zero=zero)
    kv.kv_set_decode_path(gpu.handle, DECODE_PATH)
    return gpu, oracle.OracleCache(ocfg)


def append_both(gpu, orc, layer, k_bits16, v_bits16, dtype, chunks=None):
    """k/v uint16 [B, T, H, d]; appended in the given chunk sizes (default: one bulk call)."""
    T = k_bits16.shape[1]
    chunks = [T] if chunks is None else chunks
    assert sum(chunks) == T
    kd, vd = to_dev(k_bits16, dtype), to_dev(v_bits16, dtype)
    pos = 0
    for n in chunks:
        if n:
            gpu.append(layer, kd[:, pos:pos + n], vd[:, pos:pos + n])
            orc.append(layer, k_bits16[:, pos:pos + n], v_bits16[:, pos:pos + n])
        pos += n


def check_bytes(gpu, orc, layer):
    import torch

    torch.cuda.synchronize()
    img = orc.layer_image(layer)
    got = gpu.layers[layer].cpu().numpy()
    assert got.size == img["bytes"].size
    assert gpu.lengths(layer) == (orc.packed_len(layer), orc.resid_len(layer))
    m = img["valid"]
    bad = np.flatnonzero(got[m] != img["bytes"][m])
    assert bad.size == 0, "first differing valid byte at offset %d of %d (%d differ)" % (
        np.flatnonzero(m)[bad[0]], m.size, bad.size)


def check_attention(gpu, orc, layer, q_bits16, dtype, units=None, tol=ATTN_TOL):
    import torch

    out = gpu.attend(layer, to_dev(q_bits16, dtype))
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    want = orc.attend(layer, q_bits16, units=units)
    mask = ~np.isnan(want)
    assert mask.any()
    assert np.all(np.isfinite(got[mask]))
    err = np.max(np.abs(got[mask] - want[mask]))
    assert err <= tol, "attention max-abs error %.3e > %.1e" % (err, tol)
    return err

"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the method: it only draws Llama-shaped key / value / query
tensors with the outlier structure the workloads call for and narrows them to 16 bits.  The
16-bit tensor *is* the input; both the HIP path and the CPU oracle receive the same bytes.

Recipe (stands in for the paper's LongBench / GSM8k activations, Sec. 4.1, which need model
weights and datasets that are not available here):
  keys   ~ N(0,1); per (layer, kv head) ``n_outlier`` of the d channels get a constant offset
           drawn from N(20, sigma=2); optionally ``n_drift`` further channels get +slope*t;
  values ~ N(0,1);   queries ~ N(0,1).
"""
from __future__ import annotations

import numpy as np

F16, BF16 = 0, 1


def f32_to_bits16(x: np.ndarray, dtype: int) -> np.ndarray:
    """Narrow float32 to 16-bit patterns (round to nearest even), as uint16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    u = x.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bits16_to_f32(b: np.ndarray, dtype: int) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    if dtype == F16:
        return b.view(np.float16).astype(np.float32)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def rope_tables(positions, d: int, base: float = 500000.0):
    """cos / sin tables [len(positions), d/2] (float32) of the usual rotary schedule: pair i of
    the token at position p turns by p * base^(-2i/d).  Input data for the fused rotate-and-append
    call; the caller of the library owns the schedule."""
    pos = np.asarray(positions, dtype=np.float64)[:, None]
    inv = np.asarray(base, dtype=np.float64) ** (-np.arange(0, d, 2, dtype=np.float64) / d)
    ang = pos * inv[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def channel_structure(seed: int, H: int, d: int, n_outlier: int = 4, n_drift: int = 0):
    """Per kv head: outlier channel ids + offsets, and drift channel ids (disjoint)."""
    rng = np.random.default_rng(seed)
    off = np.zeros((H, d), dtype=np.float32)
    drift = np.zeros((H, d), dtype=np.float32)
    for h in range(H):
        perm = rng.permutation(d)
        oc = perm[:n_outlier]
        off[h, oc] = rng.normal(20.0, 2.0, size=n_outlier).astype(np.float32)
        if n_drift:
            drift[h, perm[n_outlier:n_outlier + n_drift]] = 1.0
    return off, drift


def make_kv(seed: int, B: int, T: int, H: int, d: int, dtype: int, n_outlier: int = 4,
            n_drift: int = 0, slope: float = 0.01, t0: int = 0):
    """K, V as uint16 [B, T, H, d] (token-major, the layout an append call takes)."""
    rng = np.random.default_rng(seed)
    off, drift = channel_structure(seed + 7919, H, d, n_outlier, n_drift)
    k = rng.standard_normal((B, T, H, d), dtype=np.float32)
    v = rng.standard_normal((B, T, H, d), dtype=np.float32)
    k += off[None, None]
    if n_drift:
        t = (np.arange(T, dtype=np.float32) + np.float32(t0))[None, :, None, None]
        k += np.float32(slope) * t * drift[None, None]
    return f32_to_bits16(k, dtype), f32_to_bits16(v, dtype)


def make_q(seed: int, B: int, Hq: int, d: int, dtype: int) -> np.ndarray:
    rng = np.random.default_rng(seed + 104729)
    return f32_to_bits16(rng.standard_normal((B, Hq, d), dtype=np.float32), dtype)


def make_xw(seed: int, B: int, T: int, model_dim: int, n_out: int, dtype: int):
    """Inputs of the value projection (Alg. 1 step 3): the layer input X ~ N(0,1) as uint16
    [B, T, model_dim] and the weights W_V ~ N(0, 1/model_dim) as uint16 [n_out, model_dim] (one row
    per output channel, the layout of a linear layer's weight), so that the projected values are
    about N(0,1) like the values of make_kv."""
    rng = np.random.default_rng(seed + 611953)
    x = rng.standard_normal((B, T, model_dim), dtype=np.float32)
    w = rng.standard_normal((n_out, model_dim), dtype=np.float32) * np.float32(model_dim ** -0.5)
    return f32_to_bits16(x, dtype), f32_to_bits16(w, dtype)


def layer_bits(seed: int, n_layers: int, scheme: str = "mixed248"):
    """Per-layer bit map.  'mixed248': u<0.25 -> 8, u<0.625 -> 4, else 2 (about a quarter of
    the layers at 8 bits).  'mixed24_8ends': 8-bit on the first and last two layers, the rest
    50/50 from {2,4}."""
    rng = np.random.default_rng(seed)
    u = rng.random(n_layers)
    if scheme == "mixed248":
        bits = np.where(u < 0.25, 8, np.where(u < 0.625, 4, 2))
    elif scheme == "mixed24_8ends":
        bits = np.where(u < 0.5, 4, 2)
        bits[:2] = 8
        bits[-2:] = 8
    else:
        raise ValueError(scheme)
    return [int(b) for b in bits]


# ---------------------------------------------------------------------------- device-side draws


def make_kv_torch(seed: int, B: int, T: int, H: int, d: int, dtype: int, device, n_outlier: int = 4,
                  n_drift: int = 0, slope: float = 0.01, t0: int = 0, shared_sigma: float = 0.0):
    """Same recipe drawn on the device for shapes too large to ship from the host.
    Returns torch tensors [B, T, H, d] of the 16-bit dtype.  shared_sigma > 0 adds to keys and to
    values a component N(0, shared_sigma^2) per (sequence, token, channel) that all kv heads have in
    common (the structure the mean over heads, Eq. 1-2, is meant to remove); 0 leaves the streams
    of the other parameters untouched."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    tdt = torch.float16 if dtype == F16 else torch.bfloat16
    off, drift = channel_structure(seed + 7919, H, d, n_outlier, n_drift)
    off_t = torch.from_numpy(off).to(device)
    k = torch.randn((B, T, H, d), generator=gen, device=device, dtype=torch.float32)
    k += off_t[None, None]
    if n_drift:
        t = (torch.arange(T, device=device, dtype=torch.float32) + float(t0))[None, :, None, None]
        k += float(slope) * t * torch.from_numpy(drift).to(device)[None, None]
    shared = None
    if shared_sigma > 0.0:
        gen2 = torch.Generator(device=device)
        gen2.manual_seed(seed + 15485863)
        shared = float(shared_sigma) * torch.randn((2, B, T, 1, d), generator=gen2, device=device, dtype=torch.float32)
        k += shared[0]
    k16 = k.to(tdt)
    del k
    v = torch.randn((B, T, H, d), generator=gen, device=device, dtype=torch.float32)
    if shared is not None:
        v += shared[1]
    v16 = v.to(tdt)
    return k16, v16


def make_xw_torch(seed: int, B: int, T: int, model_dim: int, n_out: int, dtype: int, device):
    """make_xw's recipe drawn on the device: X [B, T, model_dim], W_V [n_out, model_dim], 16-bit."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed + 611953)
    tdt = torch.float16 if dtype == F16 else torch.bfloat16
    x = torch.randn((B, T, model_dim), generator=gen, device=device, dtype=torch.float32).to(tdt)
    w = (torch.randn((n_out, model_dim), generator=gen, device=device, dtype=torch.float32) * float(model_dim ** -0.5)).to(tdt)
    return x, w


def make_q_torch(seed: int, B: int, Hq: int, d: int, dtype: int, device):
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed + 104729)
    tdt = torch.float16 if dtype == F16 else torch.bfloat16
    return torch.randn((B, Hq, d), generator=gen, device=device, dtype=torch.float32).to(tdt)

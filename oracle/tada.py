"""Python face of the CPU oracle -- TEST INFRASTRUCTURE, not the product.

The arithmetic lives in ``tada_oracle.c`` (plain C, binary32 for the encoder, binary64 for
attention).  This module adds what is bookkeeping rather than arithmetic: the residual-token
policy of Sec. 3.3 ("Residual tokens", Eq. 9-10), the per-layer bit map (Sec. 3.3 "Searching
for quantization precision", App. B) and the byte image of a layer's cache as the storage
format documents it, so that a device buffer can be compared with it byte for byte.

Nothing here is imported by, or imports, the HIP path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tada_oracle.c")
_LIB = os.path.join(_HERE, "libtada_oracle.so")

F16, BF16 = 0, 1
ROPE_HALF, ROPE_INTERLEAVED = 0, 1
MEAN_CHANNEL_BLOCK, MEAN_CROSS_HEAD, MEAN_NONE = 0, 1, 2
K, V = 0, 1


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _c():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        i = ctypes.c_int
        lib.orc_f16_to_f32.restype = ctypes.c_float
        lib.orc_f16_to_f32.argtypes = [ctypes.c_uint16]
        lib.orc_bf16_to_f32.restype = ctypes.c_float
        lib.orc_bf16_to_f32.argtypes = [ctypes.c_uint16]
        for name in ("orc_f32_to_f16_rne", "orc_f32_to_f16_down", "orc_f32_to_f16_up"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_uint16
            fn.argtypes = [ctypes.c_float]
        lib.orc_encode_block.restype = i
        lib.orc_encode_block.argtypes = [u16p, i, i, i, i, i, i, i, i, u8p, u16p, u16p, u16p]
        lib.orc_decode_block.restype = i
        lib.orc_decode_block.argtypes = [u8p, u16p, u16p, u16p, i, i, i, i, i, i, f32p]
        lib.orc_pack_codes.restype = i
        lib.orc_pack_codes.argtypes = [u8p, i, i, i, i, u8p]
        lib.orc_unpack_codes.restype = i
        lib.orc_unpack_codes.argtypes = [u8p, i, i, i, i, u8p]
        lib.orc_attention.restype = i
        lib.orc_attention.argtypes = [f64p, f32p, f32p, i, i, i, f64p]
        lib.orc_f32_to_bf16_rne.restype = ctypes.c_uint16
        lib.orc_f32_to_bf16_rne.argtypes = [ctypes.c_float]
        lib.orc_rope.restype = i
        lib.orc_rope.argtypes = [u16p, i, i, i, i, f32p, f32p, i, u16p]
        lib.orc_project.restype = i
        lib.orc_project.argtypes = [u16p, u16p, i, i, i, i, u16p]
        lib.orc_project_f64.restype = i
        lib.orc_project_f64.argtypes = [u16p, u16p, i, i, i, i, f64p, f64p]
        lib.orc_f64_to_16_rne.restype = ctypes.c_uint16
        lib.orc_f64_to_16_rne.argtypes = [ctypes.c_double, i]
        lib.orc_widen.restype = None
        lib.orc_widen.argtypes = [u16p, i, ctypes.c_size_t, f32p]
        _lib = lib
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


# ----------------------------------------------------------------------------- scalar helpers


def f16_to_f32(h: int) -> float:
    return float(_c().orc_f16_to_f32(int(h) & 0xFFFF))


def f32_to_f16(f: float, mode: str = "rne") -> int:
    fn = {"rne": _c().orc_f32_to_f16_rne, "down": _c().orc_f32_to_f16_down, "up": _c().orc_f32_to_f16_up}[mode]
    return int(fn(ctypes.c_float(f)))


def widen(x: np.ndarray, dtype: int) -> np.ndarray:
    """16-bit patterns (uint16) -> binary32, exact."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    out = np.empty(x.shape, dtype=np.float32)
    _c().orc_widen(_p(x, ctypes.c_uint16), dtype, x.size, _p(out, ctypes.c_float))
    return out


def f32_to_bf16(f: float) -> int:
    return int(_c().orc_f32_to_bf16_rne(ctypes.c_float(f)))


def rope(x: np.ndarray, dtype: int, cos: np.ndarray, sin: np.ndarray, pairing: int) -> np.ndarray:
    """Rotary embedding of key rows (Alg. 1 step 5): x uint16 [T, H, d], cos/sin float32 [T, d/2]
    -> rotated rows, uint16 [T, H, d] (binary32 arithmetic, rounded to the 16-bit type)."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    T, H, d = x.shape
    cos = np.ascontiguousarray(cos, dtype=np.float32)
    sin = np.ascontiguousarray(sin, dtype=np.float32)
    assert cos.shape == (T, d // 2) and sin.shape == (T, d // 2)
    out = np.empty_like(x)
    rc = _c().orc_rope(_p(x, ctypes.c_uint16), dtype, T, H, d, _p(cos, ctypes.c_float), _p(sin, ctypes.c_float),
                       pairing, _p(out, ctypes.c_uint16))
    if rc != 0:
        raise ValueError("orc_rope: bad argument")
    return out


def f64_to_16(v: float, dtype: int) -> int:
    """binary64 -> the 16-bit type's pattern, one rounding (nearest even)."""
    return int(_c().orc_f64_to_16_rne(ctypes.c_double(v), dtype))


def project(x: np.ndarray, w: np.ndarray, dtype: int) -> np.ndarray:
    """The value projection of Alg. 1 step 3: x uint16 [..., kdim], w uint16 [n_out, kdim] (one row of
    weights per output channel) -> uint16 [..., n_out]; binary64 dot products rounded once to the
    16-bit type."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    w = np.ascontiguousarray(w, dtype=np.uint16)
    kdim = x.shape[-1]
    n_out = w.shape[0]
    assert w.shape == (n_out, kdim)
    rows = x.size // kdim
    out = np.empty(x.shape[:-1] + (n_out,), dtype=np.uint16)
    if _c().orc_project(_p(x, ctypes.c_uint16), _p(w, ctypes.c_uint16), dtype, rows, kdim, n_out,
                        _p(out, ctypes.c_uint16)) != 0:
        raise ValueError("orc_project rejected its arguments")
    return out


def project_f64(x: np.ndarray, w: np.ndarray, dtype: int):
    """The dot products of ``project`` before their rounding, and the sums of the products' magnitudes:
    two float64 arrays [..., n_out]."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    w = np.ascontiguousarray(w, dtype=np.uint16)
    kdim, n_out = x.shape[-1], w.shape[0]
    assert w.shape == (n_out, kdim)
    rows = x.size // kdim
    acc = np.empty(x.shape[:-1] + (n_out,), dtype=np.float64)
    mag = np.empty_like(acc)
    if _c().orc_project_f64(_p(x, ctypes.c_uint16), _p(w, ctypes.c_uint16), dtype, rows, kdim, n_out,
                            _p(acc, ctypes.c_double), _p(mag, ctypes.c_double)) != 0:
        raise ValueError("orc_project_f64 rejected its arguments")
    return acc, mag


# ----------------------------------------------------------------------------- block functions


def encode_block(x: np.ndarray, dtype: int, Gc: int, bits: int, mean_mode: int, which: int) -> dict:
    """Encode one block.  x: uint16 [G, H, d].  Returns logical codes and 16-bit metadata."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    G, H, d = x.shape
    codes = np.zeros((H, G, d), dtype=np.uint8)
    if which == K:
        scale = np.zeros((H, d), dtype=np.uint16)
    else:
        scale = np.zeros((H, G, d // Gc), dtype=np.uint16)
    zero = np.zeros_like(scale)
    if mean_mode == MEAN_CHANNEL_BLOCK:
        mean = np.zeros((H, d), dtype=np.uint16)
    elif mean_mode == MEAN_CROSS_HEAD:
        mean = np.zeros((G, d), dtype=np.uint16)
    else:
        mean = np.zeros((0,), dtype=np.uint16)
    rc = _c().orc_encode_block(_p(x, ctypes.c_uint16), dtype, G, H, d, Gc, bits, mean_mode, which,
                               _p(codes, ctypes.c_uint8), _p(scale, ctypes.c_uint16),
                               _p(zero, ctypes.c_uint16),
                               _p(mean, ctypes.c_uint16) if mean.size else None)
    if rc != 0:
        raise ValueError("orc_encode_block rejected its arguments")
    return {"codes": codes, "scale": scale, "zero": zero, "mean": mean}


def decode_block(enc: dict, Gc: int, mean_mode: int, which: int) -> np.ndarray:
    """Reconstruct x^ [H, G, d] float32 from a block's logical codes and metadata."""
    codes = enc["codes"]
    H, G, d = codes.shape
    out = np.empty((H, G, d), dtype=np.float32)
    mean = enc["mean"]
    rc = _c().orc_decode_block(_p(codes, ctypes.c_uint8), _p(enc["scale"], ctypes.c_uint16),
                               _p(enc["zero"], ctypes.c_uint16),
                               _p(mean, ctypes.c_uint16) if mean.size else None,
                               G, H, d, Gc, mean_mode, which, _p(out, ctypes.c_float))
    if rc != 0:
        raise ValueError("orc_decode_block rejected its arguments")
    return out


def pack_codes(codes: np.ndarray, which: int, bits: int) -> np.ndarray:
    """codes uint8 [G, d] of one head -> packed bytes."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    G, d = codes.shape
    out = np.empty(G * d * bits // 8, dtype=np.uint8)
    if _c().orc_pack_codes(_p(codes, ctypes.c_uint8), which, bits, G, d, _p(out, ctypes.c_uint8)) != 0:
        raise ValueError("orc_pack_codes rejected its arguments")
    return out


def unpack_codes(packed: np.ndarray, which: int, bits: int, G: int, d: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    out = np.empty((G, d), dtype=np.uint8)
    if _c().orc_unpack_codes(_p(packed, ctypes.c_uint8), which, bits, G, d, _p(out, ctypes.c_uint8)) != 0:
        raise ValueError("orc_unpack_codes rejected its arguments")
    return out


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Eq. 5-6 in binary64.  q [g, d] float64, k/v [T, d] float32 -> [g, d] float64."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    g, d = q.shape
    T = k.shape[0]
    out = np.empty((g, d), dtype=np.float64)
    if _c().orc_attention(_p(q, ctypes.c_double), _p(k, ctypes.c_float), _p(v, ctypes.c_float),
                          T, d, g, _p(out, ctypes.c_double)) != 0:
        raise ValueError("orc_attention rejected its arguments")
    return out


# ----------------------------------------------------------------------------- cache


def _align(n: int, a: int) -> int:
    return (n + a - 1) // a * a


@dataclass
class OracleConfig:
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    max_tokens: int
    group_tokens: int
    group_channels: int
    resid_cap: int
    dtype: int
    mean_mode: int
    k_bits: Sequence[int]
    v_bits: Sequence[int]


@dataclass
class _Layer:
    # per batch element: list of encoded blocks (dicts for K and V) and the raw residual
    k_blocks: List[List[dict]] = field(default_factory=list)
    v_blocks: List[List[dict]] = field(default_factory=list)
    k_resid: List[np.ndarray] = field(default_factory=list)  # each [r, H, d] uint16
    v_resid: List[np.ndarray] = field(default_factory=list)


class OracleCache:
    """The KV cache of Algorithm 1 (KVCache.update) with the residual buffer of Sec. 3.3.

    Tokens enter the raw residual buffer one at a time; when it holds ``resid_cap`` tokens all
    of them are compressed as ``resid_cap / group_tokens`` blocks and the buffer restarts empty.
    """

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        H, d = cfg.n_kv_heads, cfg.head_dim
        self.layers = []
        for _ in range(cfg.n_layers):
            L = _Layer()
            for _b in range(cfg.batch):
                L.k_blocks.append([])
                L.v_blocks.append([])
                L.k_resid.append(np.zeros((0, H, d), dtype=np.uint16))
                L.v_resid.append(np.zeros((0, H, d), dtype=np.uint16))
            self.layers.append(L)

    # -- lengths
    def packed_len(self, layer: int, b: int = 0) -> int:
        return len(self.layers[layer].k_blocks[b]) * self.cfg.group_tokens

    def resid_len(self, layer: int, b: int = 0) -> int:
        return self.layers[layer].k_resid[b].shape[0]

    def reset_seq(self, layer: int, b: int) -> None:
        """Sequence b leaves: its blocks and residual buffer (Sec. 3.3: both are per sequence) are dropped."""
        cfg, L = self.cfg, self.layers[layer]
        L.k_blocks[b], L.v_blocks[b] = [], []
        L.k_resid[b] = np.zeros((0, cfg.n_kv_heads, cfg.head_dim), dtype=np.uint16)
        L.v_resid[b] = np.zeros((0, cfg.n_kv_heads, cfg.head_dim), dtype=np.uint16)

    # -- append
    def _flush(self, layer: int, b: int) -> None:
        cfg, L = self.cfg, self.layers[layer]
        G = cfg.group_tokens
        kb, vb = cfg.k_bits[layer], cfg.v_bits[layer]
        kr, vr = L.k_resid[b], L.v_resid[b]
        for j in range(kr.shape[0] // G):
            xk, xv = kr[j * G:(j + 1) * G], vr[j * G:(j + 1) * G]
            if kb == 16:
                L.k_blocks[b].append({"raw": xk.copy()})
            else:
                L.k_blocks[b].append(encode_block(xk, cfg.dtype, cfg.group_channels, kb, cfg.mean_mode, K))
            if vb == 16:
                L.v_blocks[b].append({"raw": xv.copy()})
            else:
                L.v_blocks[b].append(encode_block(xv, cfg.dtype, cfg.group_channels, vb, cfg.mean_mode, V))
        H, d = cfg.n_kv_heads, cfg.head_dim
        L.k_resid[b] = np.zeros((0, H, d), dtype=np.uint16)
        L.v_resid[b] = np.zeros((0, H, d), dtype=np.uint16)

    def append(self, layer: int, k_new: np.ndarray, v_new: np.ndarray, rope_tables=None) -> None:
        """k_new, v_new: uint16 [B, n_new, H, d] (post-RoPE keys, values).  With
        rope_tables = (cos [n_new, d/2], sin, pairing) the keys are pre-RoPE and are rotated first
        (Alg. 1 step 5); the result equals rotating them as a step of its own and appending."""
        cfg, L = self.cfg, self.layers[layer]
        n = k_new.shape[1]
        if rope_tables is not None:
            cos, sin, pairing = rope_tables
            k_new = np.stack([rope(k_new[b], cfg.dtype, cos, sin, pairing) for b in range(cfg.batch)])
        if any(self.packed_len(layer, b) + self.resid_len(layer, b) + n > cfg.max_tokens for b in range(cfg.batch)):
            raise OverflowError("append exceeds max_tokens")
        for b in range(cfg.batch):
            self._append_one(layer, b, k_new[b], v_new[b])

    def append_compressv(self, layer: int, k_new: np.ndarray, x: np.ndarray, w_v: np.ndarray) -> np.ndarray:
        """Alg. 1 steps 3 and 8: the values are the projection of the layer input, x uint16
        [B, n_new, model_dim] against w_v uint16 [Hkv * d, model_dim], a 16-bit tensor; keys as in
        append.  Returns the projected values, uint16 [B, n_new, Hkv, d]."""
        cfg = self.cfg
        v = project(x, w_v, cfg.dtype).reshape(x.shape[0], x.shape[1], cfg.n_kv_heads, cfg.head_dim)
        self.append(layer, k_new, v)
        return v

    def append_seq(self, layer: int, b: int, k_new: np.ndarray, v_new: np.ndarray) -> None:
        """Tokens of one sequence only: k_new, v_new uint16 [n_new, H, d]."""
        if self.packed_len(layer, b) + self.resid_len(layer, b) + k_new.shape[0] > self.cfg.max_tokens:
            raise OverflowError("append exceeds max_tokens")
        self._append_one(layer, b, k_new, v_new)

    def _append_one(self, layer: int, b: int, k_new: np.ndarray, v_new: np.ndarray) -> None:
        cfg, L = self.cfg, self.layers[layer]
        n = k_new.shape[0]
        done = 0
        while done < n:
            take = min(cfg.resid_cap - L.k_resid[b].shape[0], n - done)
            L.k_resid[b] = np.concatenate([L.k_resid[b], k_new[done:done + take]], axis=0)
            L.v_resid[b] = np.concatenate([L.v_resid[b], v_new[done:done + take]], axis=0)
            done += take
            if L.k_resid[b].shape[0] == cfg.resid_cap:
                self._flush(layer, b)

    # -- reconstruction and attention
    def reconstruct(self, layer: int, b: int, which: int) -> np.ndarray:
        """All tokens of batch element b as float32 [H, T, d]: decoded blocks, then the raw tail."""
        cfg, L = self.cfg, self.layers[layer]
        blocks = L.k_blocks[b] if which == K else L.v_blocks[b]
        resid = L.k_resid[b] if which == K else L.v_resid[b]
        parts = []
        for e in blocks:
            if "raw" in e:
                parts.append(np.transpose(widen(e["raw"], cfg.dtype), (1, 0, 2)))
            else:
                parts.append(decode_block(e, cfg.group_channels, cfg.mean_mode, which))
        if resid.shape[0]:
            parts.append(np.transpose(widen(resid, cfg.dtype), (1, 0, 2)))
        if not parts:
            return np.zeros((cfg.n_kv_heads, 0, cfg.head_dim), dtype=np.float32)
        return np.ascontiguousarray(np.concatenate(parts, axis=1))

    def attend(self, layer: int, q: np.ndarray, units=None) -> np.ndarray:
        """q uint16 [B, Hq, d] -> float64 [B, Hq, d]; query head i reads kv head i // (Hq/Hkv).

        ``units``: optional iterable of (b, h) pairs to restrict the work to (others stay NaN)."""
        cfg = self.cfg
        g = cfg.n_q_heads // cfg.n_kv_heads
        qf = widen(q, cfg.dtype).astype(np.float64)
        out = np.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), np.nan, dtype=np.float64)
        todo = {}
        for (b, h) in (units if units is not None else [(b, h) for b in range(cfg.batch) for h in range(cfg.n_kv_heads)]):
            todo.setdefault(b, []).append(h)
        for b, heads in todo.items():
            kh = self.reconstruct(layer, b, K)
            vh = self.reconstruct(layer, b, V)
            for h in heads:
                if kh.shape[1] == 0:  # a sequence that holds no token: nothing to attend to, zeros
                    out[b, h * g:(h + 1) * g] = 0.0
                else:
                    out[b, h * g:(h + 1) * g] = attention(qf[b, h * g:(h + 1) * g], kh[h], vh[h])
        return out

    # -- storage format
    def record_bytes(self, layer: int) -> int:
        return record_layout(self.cfg, layer)["rec_bytes"]

    def layer_image(self, layer: int) -> dict:
        """Byte image of the layer's cache buffer as the storage format states it.

        Returns {"bytes": uint8 array of the full layer buffer (unwritten parts zero),
                 "valid": boolean mask of the bytes the format defines for the current lengths}.
        """
        cfg, L = self.cfg, self.layers[layer]
        lay = record_layout(cfg, layer)
        buf = np.zeros(lay["layer_bytes"], dtype=np.uint8)
        valid = np.zeros(lay["layer_bytes"], dtype=bool)
        H, d, G, Gc = cfg.n_kv_heads, cfg.head_dim, cfg.group_tokens, cfg.group_channels
        NB = cfg.max_tokens // G
        kb, vb = cfg.k_bits[layer], cfg.v_bits[layer]

        def put(off, arr):
            raw = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
            buf[off:off + raw.size] = raw
            valid[off:off + raw.size] = True

        for b in range(cfg.batch):
            for j, (ek, ev) in enumerate(zip(L.k_blocks[b], L.v_blocks[b])):
                for h in range(H):
                    base = ((b * H + h) * NB + j) * lay["rec_bytes"]
                    if kb == 16:
                        put(base + lay["k_codes"], ek["raw"][:, h, :])
                    else:
                        put(base + lay["k_codes"], pack_codes(ek["codes"][h], K, kb))
                        put(base + lay["k_scale"], ek["scale"][h])
                        put(base + lay["k_zero"], ek["zero"][h])
                        if cfg.mean_mode == MEAN_CHANNEL_BLOCK:
                            put(base + lay["k_mean"], ek["mean"][h])
                    if vb == 16:
                        put(base + lay["v_codes"], ev["raw"][:, h, :])
                    else:
                        put(base + lay["v_codes"], pack_codes(ev["codes"][h], V, vb))
                        sz = np.stack([ev["scale"][h], ev["zero"][h]], axis=-1)  # [G, d/Gc, 2]
                        put(base + lay["v_meta"], sz)
                        if cfg.mean_mode == MEAN_CHANNEL_BLOCK:
                            put(base + lay["v_mean"], ev["mean"][h])
                if cfg.mean_mode == MEAN_CROSS_HEAD:
                    mo = lay["xmean_off"] + (b * NB + j) * 2 * G * d * 2
                    if kb != 16:
                        put(mo, ek["mean"])
                    if vb != 16:
                        put(mo + G * d * 2, ev["mean"])
            r = L.k_resid[b].shape[0]
            for h in range(H):
                u = b * H + h
                put(lay["k_resid_off"] + u * cfg.resid_cap * d * 2, L.k_resid[b][:, h, :])
                put(lay["v_resid_off"] + u * cfg.resid_cap * d * 2, L.v_resid[b][:, h, :])
            del r
        return {"bytes": buf, "valid": valid}


def record_layout(cfg: OracleConfig, layer: int) -> dict:
    """Offsets of the storage format for one layer.

    Layer buffer = records [U][NB] | cross-head mean plane [B][NB][2][G][d] f16 (CROSS_HEAD only)
                 | raw K residual [U][R][d] | raw V residual [U][R][d]; regions 256-byte aligned.
    Record (one unit, one block of G tokens) = K codes | K scale[d] | K zero[d] | K mean[d]
                 | V codes | V (scale,zero)[G][d/Gc] | V mean[d]; mean parts only in
                 CHANNEL_BLOCK mode; a 16-bit side holds the raw [G][d] rows and no metadata.
    """
    H, d, G, Gc = cfg.n_kv_heads, cfg.head_dim, cfg.group_tokens, cfg.group_channels
    kb, vb = cfg.k_bits[layer], cfg.v_bits[layer]
    chan_mean = cfg.mean_mode == MEAN_CHANNEL_BLOCK
    off = 0
    lay = {}
    lay["k_codes"] = off
    off += G * d * kb // 8
    if kb != 16:
        lay["k_scale"] = off
        off += d * 2
        lay["k_zero"] = off
        off += d * 2
        if chan_mean:
            lay["k_mean"] = off
            off += d * 2
    lay["v_codes"] = off
    off += G * d * vb // 8
    if vb != 16:
        lay["v_meta"] = off
        off += G * (d // Gc) * 4
        if chan_mean:
            lay["v_mean"] = off
            off += d * 2
    lay["rec_bytes"] = _align(off, 256)
    U = cfg.batch * H
    NB = cfg.max_tokens // G
    total = _align(U * NB * lay["rec_bytes"], 256)
    lay["xmean_off"] = total
    if cfg.mean_mode == MEAN_CROSS_HEAD:
        total = _align(total + cfg.batch * NB * 2 * G * d * 2, 256)
    lay["k_resid_off"] = total
    total = _align(total + U * cfg.resid_cap * d * 2, 256)
    lay["v_resid_off"] = total
    total = _align(total + U * cfg.resid_cap * d * 2, 256)
    lay["layer_bytes"] = total
    return lay


def kv_bytes_ratio(n_heads: int, head_dim: int, G: int, Gc: int, bits: Sequence[int], mean_mode: int) -> float:
    """Bytes the format stores per cached token (all heads, K and V, averaged over the layers in
    ``bits``) divided by the 16-bit cache's bytes, counted from the arrays ``encode_block``
    actually returns for a block -- the quantity of the paper's memory formula in Sec. 3."""
    rng = np.random.default_rng(0)
    x = rng.integers(0x3000, 0x3C00, size=(G, n_heads, head_dim), dtype=np.uint16)  # finite f16
    total = 0.0
    for b in bits:
        n = 0
        for which in (K, V):
            if b == 16:
                n += x.size * 2
                continue
            e = encode_block(x, F16, Gc, b, mean_mode, which)
            n += e["codes"].size * b // 8 + e["scale"].nbytes + e["zero"].nbytes + e["mean"].nbytes
        total += n / (2 * x.size * 2)
    return total / len(bits)

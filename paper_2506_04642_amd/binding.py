"""ctypes binding of libtadakv.so: the same names as include/tadakv.h, argument marshalling only.

Every step of the hot path runs in the library's HIP kernels.  There is no fallback: if the
library has not been built, importing this module raises.  PyTorch appears only in ``KVCache``,
a convenience holder that allocates the device buffers (torch tensors) and passes their pointers
and the current HIP stream to the C ABI.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtadakv.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libtadakv.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
        "(or paper_2506_04642_amd/build.py) first; there is no fallback path")

_lib = ctypes.CDLL(LIB_PATH)

KV_OK = 0
KV_E_NULL, KV_E_BAD_CONFIG, KV_E_BAD_BITS, KV_E_BAD_LAYER, KV_E_CAPACITY = -1, -2, -3, -4, -5
KV_E_WORKSPACE, KV_E_ALIGN, KV_E_HIP, KV_E_EMPTY, KV_E_UNSUPPORTED = -6, -7, -8, -9, -10
KV_F16, KV_BF16 = 0, 1
KV_MEAN_CHANNEL_BLOCK, KV_MEAN_CROSS_HEAD, KV_MEAN_NONE = 0, 1, 2

EXPORTS = [
    "kv_cache_bytes", "kv_workspace_bytes", "kv_cache_create", "kv_cache_destroy", "kv_cache_set_block_table", "kv_cache_set_active", "kv_cache_reset",
    "kv_cache_len", "kv_cache_len_seq", "kv_cache_reset_seq", "kv_cache_describe", "kv_quant_append", "kv_quant_append_seq", "kv_rope_quant_append", "kv_compressv_append", "kv_append_decode_attn", "kv_append_decode_attn_split", "kv_decode_attn", "kv_decode_attn_split",
    "kv_decode_attn_merge", "kv_decode_attn_merge16", "kv_dequant", "kv_decode_splits", "kv_decode_bytes", "kv_set_decode_path", "kv_decode_path_used", "kv_set_decode_splits", "kv_decode_workspace_need", "kv_decode_attn_static", "kv_dev_lengths_bytes", "kv_cache_lengths_to_device", "kv_decode_step_dev", "kv_cache_advance", "kv_stream_read_probe", "kv_time_next_split", "kv_strerror", "kv_last_hip_error",
]


class kv_config(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int32), ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("max_tokens", ctypes.c_int32),
        ("group_tokens", ctypes.c_int32), ("group_channels", ctypes.c_int32), ("resid_cap", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("mean_mode", ctypes.c_int32),
        ("k_bits", ctypes.POINTER(ctypes.c_uint8)), ("v_bits", ctypes.POINTER(ctypes.c_uint8)),
        ("pool_blocks", ctypes.c_int32),
    ]


class kv_layer_layout(ctypes.Structure):
    _fields_ = [("k_bits", ctypes.c_int32), ("v_bits", ctypes.c_int32)] + [
        (n, ctypes.c_int64) for n in (
            "rec_bytes", "k_codes", "k_scale", "k_zero", "k_mean", "v_codes", "v_meta", "v_mean",
            "xmean_off", "k_resid_off", "v_resid_off", "layer_bytes")]


_vp = ctypes.c_void_p
_i32 = ctypes.c_int32
_i64 = ctypes.c_int64
_szp = ctypes.POINTER(ctypes.c_size_t)
_cfgp = ctypes.POINTER(kv_config)

_lib.kv_cache_bytes.argtypes = [_cfgp, _i32, _szp]
_lib.kv_workspace_bytes.argtypes = [_cfgp, _szp]
_lib.kv_cache_create.argtypes = [_cfgp, ctypes.POINTER(_vp), ctypes.POINTER(_vp)]
_lib.kv_cache_destroy.argtypes = [_vp]
_lib.kv_cache_set_block_table.argtypes = [_vp, _vp, _i32]
_lib.kv_cache_set_active.argtypes = [_vp, ctypes.POINTER(ctypes.c_uint8), _i32]
_lib.kv_cache_reset.argtypes = [_vp, _i32]
_lib.kv_cache_len.argtypes = [_vp, _i32, ctypes.POINTER(_i32), ctypes.POINTER(_i32)]
_lib.kv_cache_len_seq.argtypes = [_vp, _i32, _i32, ctypes.POINTER(_i32), ctypes.POINTER(_i32)]
_lib.kv_cache_reset_seq.argtypes = [_vp, _i32, _i32]
_lib.kv_quant_append_seq.argtypes = [_vp, _i32, _i32, _vp, _vp, _i32, _i64, _i64, _vp]
_lib.kv_cache_describe.argtypes = [_vp, _i32, ctypes.POINTER(kv_layer_layout)]
_lib.kv_quant_append.argtypes = [_vp, _i32, _vp, _vp, _i32, _i64, _i64, _i64, _vp]
_lib.kv_rope_quant_append.argtypes = [_vp, _i32, _vp, _vp, _i32, _i64, _i64, _i64, _vp, _vp, _i32, _vp]
_lib.kv_compressv_append.argtypes = [_vp, _i32, _vp, _i64, _i64, _i64, _vp, _i64, _i64, _vp, _i32, _i32, _vp, _vp, _i32, _vp, _vp]
_lib.kv_decode_attn.argtypes = [_vp, _i32, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.kv_append_decode_attn.argtypes = [_vp, _i32, _vp, _vp, _i64, _i64, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.kv_append_decode_attn_split.argtypes = [_vp, _i32, _vp, _vp, _i64, _i64, _vp, _vp, ctypes.c_size_t, _vp]
_lib.kv_decode_attn_split.argtypes = [_vp, _i32, _vp, _vp, ctypes.c_size_t, _vp]
_lib.kv_decode_attn_merge.argtypes = [_vp, _i32, _vp, _vp, ctypes.c_size_t, _vp]
_lib.kv_decode_attn_merge16.argtypes = [_vp, _i32, _vp, _vp, ctypes.c_size_t, _vp]
_lib.kv_dequant.argtypes = [_vp, _i32, _vp, _vp, _i32, _vp]
_lib.kv_decode_splits.argtypes = [_vp, _i32, ctypes.POINTER(_i32)]
_lib.kv_decode_bytes.argtypes = [_vp, _i32, _szp]
_lib.kv_set_decode_path.argtypes = [_vp, _i32]
_lib.kv_set_decode_splits.argtypes = [_vp, _i32]
_lib.kv_decode_path_used.argtypes = [_vp, _i32, ctypes.POINTER(_i32)]
_lib.kv_decode_workspace_need.argtypes = [_vp, _i32, _szp]
_lib.kv_decode_attn_static.argtypes = [_vp, _i32, _vp, _vp, _vp]
_lib.kv_dev_lengths_bytes.argtypes = [_cfgp, _szp]
_lib.kv_cache_lengths_to_device.argtypes = [_vp, _vp, _vp]
_lib.kv_decode_step_dev.argtypes = [_vp, _i32, _vp, _vp, _i64, _i64, _vp, _vp, _vp, ctypes.c_size_t, _vp]
_lib.kv_cache_advance.argtypes = [_vp, _i32, _i32]
_lib.kv_stream_read_probe.argtypes = [_vp, ctypes.c_size_t, _vp, _vp]
_lib.kv_time_next_split.argtypes = [_vp, _vp]
_lib.kv_strerror.argtypes = [_i32]
_lib.kv_strerror.restype = ctypes.c_char_p
_lib.kv_last_hip_error.argtypes = []
_lib.kv_last_hip_error.restype = ctypes.c_char_p
for _n in EXPORTS:
    if _n not in ("kv_strerror", "kv_last_hip_error"):
        getattr(_lib, _n).restype = _i32


class KVError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = " [%s]" % kv_last_hip_error() if status == KV_E_HIP else ""
        super().__init__("%s: %s (%d)%s" % (where, kv_strerror(status), status, detail))


def kv_strerror(status: int) -> str:
    return _lib.kv_strerror(status).decode()


def kv_last_hip_error() -> str:
    return _lib.kv_last_hip_error().decode()


def _check(status: int, where: str) -> None:
    if status != KV_OK:
        raise KVError(status, where)


def make_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, max_tokens, group_tokens,
                group_channels, resid_cap, dtype, mean_mode, k_bits: Sequence[int],
                v_bits: Sequence[int], pool_blocks: int = 0) -> kv_config:
    """Fill a kv_config; the bit arrays are kept alive on the returned object.  pool_blocks > 0
    asks for paged placement (block slots shared through kv_cache_set_block_table)."""
    kb = (ctypes.c_uint8 * len(k_bits))(*k_bits)
    vb = (ctypes.c_uint8 * len(v_bits))(*v_bits)
    cfg = kv_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, max_tokens, group_tokens,
                    group_channels, resid_cap, dtype, mean_mode,
                    ctypes.cast(kb, ctypes.POINTER(ctypes.c_uint8)),
                    ctypes.cast(vb, ctypes.POINTER(ctypes.c_uint8)), pool_blocks)
    cfg._keep = (kb, vb)
    return cfg


# ---- thin wrappers, one per C entry point (raw status codes are turned into KVError)


def kv_cache_bytes(cfg: kv_config, layer: int) -> int:
    n = ctypes.c_size_t()
    _check(_lib.kv_cache_bytes(ctypes.byref(cfg), layer, ctypes.byref(n)), "kv_cache_bytes")
    return n.value


def kv_cache_set_active(cache: int, active: Optional[Sequence[int]]) -> None:
    """active: one flag per sequence, or None for all."""
    if active is None:
        _check(_lib.kv_cache_set_active(cache, None, 0), "kv_cache_set_active")
        return
    arr = (ctypes.c_uint8 * len(active))(*[1 if x else 0 for x in active])
    _check(_lib.kv_cache_set_active(cache, arr, len(active)), "kv_cache_set_active")


def kv_cache_set_block_table(cache: int, table_ptr: int, stride: int) -> None:
    _check(_lib.kv_cache_set_block_table(cache, table_ptr, stride), "kv_cache_set_block_table")


def kv_workspace_bytes(cfg: kv_config) -> int:
    n = ctypes.c_size_t()
    _check(_lib.kv_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)), "kv_workspace_bytes")
    return n.value


def kv_cache_create(cfg: kv_config, layer_ptrs: Sequence[int]) -> int:
    arr = (_vp * len(layer_ptrs))(*layer_ptrs)
    out = _vp()
    _check(_lib.kv_cache_create(ctypes.byref(cfg), arr, ctypes.byref(out)), "kv_cache_create")
    return out.value


def kv_cache_destroy(cache: int) -> None:
    _check(_lib.kv_cache_destroy(cache), "kv_cache_destroy")


def kv_cache_reset(cache: int, layer: int = -1) -> None:
    _check(_lib.kv_cache_reset(cache, layer), "kv_cache_reset")


def kv_cache_len(cache: int, layer: int):
    p, r = _i32(), _i32()
    _check(_lib.kv_cache_len(cache, layer, ctypes.byref(p), ctypes.byref(r)), "kv_cache_len")
    return p.value, r.value


def kv_cache_len_seq(cache: int, layer: int, seq: int):
    p, r = _i32(), _i32()
    _check(_lib.kv_cache_len_seq(cache, layer, seq, ctypes.byref(p), ctypes.byref(r)), "kv_cache_len_seq")
    return p.value, r.value


def kv_cache_reset_seq(cache: int, layer: int, seq: int) -> None:
    _check(_lib.kv_cache_reset_seq(cache, layer, seq), "kv_cache_reset_seq")


def kv_quant_append_seq(cache: int, layer: int, seq: int, k_ptr: int, v_ptr: int, n_new: int, stride_t: int,
                        stride_h: int, stream: int = 0) -> None:
    _check(_lib.kv_quant_append_seq(cache, layer, seq, k_ptr, v_ptr, n_new, stride_t, stride_h, stream),
           "kv_quant_append_seq")


def kv_cache_describe(cache: int, layer: int) -> kv_layer_layout:
    out = kv_layer_layout()
    _check(_lib.kv_cache_describe(cache, layer, ctypes.byref(out)), "kv_cache_describe")
    return out


def kv_quant_append(cache: int, layer: int, k_ptr: int, v_ptr: int, n_new: int, stride_b: int,
                    stride_t: int, stride_h: int, stream: int = 0) -> None:
    _check(_lib.kv_quant_append(cache, layer, k_ptr, v_ptr, n_new, stride_b, stride_t, stride_h, stream),
           "kv_quant_append")


KV_ROPE_HALF, KV_ROPE_INTERLEAVED = 0, 1


def kv_rope_quant_append(cache: int, layer: int, k_ptr: int, v_ptr: int, n_new: int, stride_b: int,
                         stride_t: int, stride_h: int, cos_ptr: int, sin_ptr: int, pairing: int,
                         stream: int = 0) -> None:
    _check(_lib.kv_rope_quant_append(cache, layer, k_ptr, v_ptr, n_new, stride_b, stride_t, stride_h,
                                     cos_ptr, sin_ptr, pairing, stream), "kv_rope_quant_append")


def kv_compressv_append(cache: int, layer: int, k_ptr: int, k_stride_b: int, k_stride_t: int, k_stride_h: int,
                        x_ptr: int, x_stride_b: int, x_stride_t: int, w_ptr: int, model_dim: int, n_new: int,
                        cos_ptr: int = 0, sin_ptr: int = 0, pairing: int = 0, v_proj_ptr: int = 0, stream: int = 0) -> None:
    _check(_lib.kv_compressv_append(cache, layer, k_ptr, k_stride_b, k_stride_t, k_stride_h, x_ptr, x_stride_b,
                                    x_stride_t, w_ptr, model_dim, n_new, cos_ptr or None, sin_ptr or None, pairing,
                                    v_proj_ptr or None, stream), "kv_compressv_append")


def kv_decode_attn(cache: int, layer: int, q_ptr: int, out_ptr: int, ws_ptr: int, ws_bytes: int,
                   stream: int = 0) -> None:
    _check(_lib.kv_decode_attn(cache, layer, q_ptr, out_ptr, ws_ptr, ws_bytes, stream), "kv_decode_attn")


def kv_append_decode_attn(cache: int, layer: int, k_ptr: int, v_ptr: int, stride_b: int, stride_h: int,
                          q_ptr: int, out_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(_lib.kv_append_decode_attn(cache, layer, k_ptr, v_ptr, stride_b, stride_h, q_ptr, out_ptr, ws_ptr,
                                      ws_bytes, stream), "kv_append_decode_attn")


def kv_append_decode_attn_split(cache: int, layer: int, k_ptr: int, v_ptr: int, stride_b: int, stride_h: int,
                                q_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(_lib.kv_append_decode_attn_split(cache, layer, k_ptr, v_ptr, stride_b, stride_h, q_ptr, ws_ptr,
                                            ws_bytes, stream), "kv_append_decode_attn_split")


def kv_decode_attn_split(cache: int, layer: int, q_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(_lib.kv_decode_attn_split(cache, layer, q_ptr, ws_ptr, ws_bytes, stream), "kv_decode_attn_split")


def kv_decode_attn_merge(cache: int, layer: int, out_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(_lib.kv_decode_attn_merge(cache, layer, out_ptr, ws_ptr, ws_bytes, stream), "kv_decode_attn_merge")


def kv_dequant(cache: int, layer: int, k_out_ptr: int, v_out_ptr: int, t_cap: int, stream: int = 0) -> None:
    _check(_lib.kv_dequant(cache, layer, k_out_ptr, v_out_ptr, t_cap, stream), "kv_dequant")


def kv_decode_attn_merge16(cache: int, layer: int, out16_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(_lib.kv_decode_attn_merge16(cache, layer, out16_ptr, ws_ptr, ws_bytes, stream), "kv_decode_attn_merge16")


def kv_decode_splits(cache: int, layer: int) -> int:
    n = _i32()
    _check(_lib.kv_decode_splits(cache, layer, ctypes.byref(n)), "kv_decode_splits")
    return n.value


def kv_decode_bytes(cache: int, layer: int) -> int:
    n = ctypes.c_size_t()
    _check(_lib.kv_decode_bytes(cache, layer, ctypes.byref(n)), "kv_decode_bytes")
    return n.value


def kv_set_decode_path(cache: int, path: int) -> None:
    _check(_lib.kv_set_decode_path(cache, path), "kv_set_decode_path")


def kv_decode_path_used(cache: int, layer: int) -> int:
    n = _i32()
    _check(_lib.kv_decode_path_used(cache, layer, ctypes.byref(n)), "kv_decode_path_used")
    return n.value


def kv_set_decode_splits(cache: int, n_splits: int) -> None:
    _check(_lib.kv_set_decode_splits(cache, n_splits), "kv_set_decode_splits")


KV_STATIC_WORKSPACE_BYTES = 8 << 20


def kv_decode_workspace_need(cache: int, layer: int) -> int:
    n = ctypes.c_size_t()
    _check(_lib.kv_decode_workspace_need(cache, layer, ctypes.byref(n)), "kv_decode_workspace_need")
    return n.value


def kv_decode_attn_static(cache: int, layer: int, q_ptr: int, out_ptr: int, stream: int = 0) -> None:
    _check(_lib.kv_decode_attn_static(cache, layer, q_ptr, out_ptr, stream), "kv_decode_attn_static")


def kv_dev_lengths_bytes(cfg: kv_config) -> int:
    n = ctypes.c_size_t()
    _check(_lib.kv_dev_lengths_bytes(ctypes.byref(cfg), ctypes.byref(n)), "kv_dev_lengths_bytes")
    return n.value


def kv_cache_lengths_to_device(cache: int, dev_ptr: int, stream: int = 0) -> None:
    _check(_lib.kv_cache_lengths_to_device(cache, dev_ptr, stream), "kv_cache_lengths_to_device")


def kv_decode_step_dev(cache: int, layer: int, k_ptr: int, v_ptr: int, stride_b: int, stride_h: int, q_ptr: int,
                       out_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(_lib.kv_decode_step_dev(cache, layer, k_ptr, v_ptr, stride_b, stride_h, q_ptr, out_ptr, ws_ptr, ws_bytes,
                                   stream), "kv_decode_step_dev")


def kv_cache_advance(cache: int, layer: int, n_steps: int) -> None:
    _check(_lib.kv_cache_advance(cache, layer, n_steps), "kv_cache_advance")


def kv_time_next_split(begin_event: int, end_event: int) -> None:
    """hipEvent_t handles (torch.cuda.Event(enable_timing=True).cuda_event of events recorded once before)."""
    _check(_lib.kv_time_next_split(begin_event or None, end_event or None), "kv_time_next_split")


def kv_stream_read_probe(buf_ptr: int, nbytes: int, sink_ptr: int = 0, stream: int = 0) -> None:
    _check(_lib.kv_stream_read_probe(buf_ptr, nbytes, sink_ptr or None, stream), "kv_stream_read_probe")


# ---- memory / stream plumbing


class KVCache:
    """Owns the device buffers (torch uint8 tensors) of a cache and forwards calls to the C ABI
    on torch's current HIP stream.  No arithmetic happens here."""

    def __init__(self, cfg: kv_config, device="cuda:0", zero: bool = True):
        import torch

        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        alloc = torch.zeros if zero else torch.empty
        self.layers = [alloc(kv_cache_bytes(cfg, l), dtype=torch.uint8, device=self.device)
                       for l in range(cfg.n_layers)]
        self.ws_bytes = kv_workspace_bytes(cfg)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)
        self.handle: Optional[int] = kv_cache_create(cfg, [t.data_ptr() for t in self.layers])

    def set_block_table(self, table) -> None:
        """Paged placement: table is a device int32 tensor [batch, stride] of block slots; it is kept
        alive here and read by the kernels when they run."""
        assert table.dtype == self.torch.int32 and table.is_contiguous() and table.dim() == 2
        self._table = table
        kv_cache_set_block_table(self.handle, table.data_ptr(), table.shape[1])

    def close(self):
        if self.handle:
            kv_cache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def append(self, layer: int, k_new, v_new) -> None:
        """k_new, v_new: device tensors [B, n_new, Hkv, d], 16-bit, last dim contiguous."""
        assert k_new.shape == v_new.shape and k_new.stride() == v_new.stride()
        assert k_new.stride(3) == 1 and k_new.element_size() == 2
        kv_quant_append(self.handle, layer, k_new.data_ptr(), v_new.data_ptr(), k_new.shape[1],
                        k_new.stride(0), k_new.stride(1), k_new.stride(2), self._stream())

    def append_seq(self, layer: int, seq: int, k_new, v_new) -> None:
        """k_new, v_new: device tensors [n_new, Hkv, d] of one sequence of the batch."""
        assert k_new.shape == v_new.shape and k_new.stride() == v_new.stride()
        assert k_new.stride(2) == 1 and k_new.element_size() == 2
        kv_quant_append_seq(self.handle, layer, seq, k_new.data_ptr(), v_new.data_ptr(), k_new.shape[0],
                            k_new.stride(0), k_new.stride(1), self._stream())

    def append_rope(self, layer: int, k_pre, v_new, cos, sin, pairing: int = KV_ROPE_HALF) -> None:
        """As append, with pre-rotation keys and float32 device tables cos, sin [n_new, d/2]."""
        torch = self.torch
        assert k_pre.shape == v_new.shape and k_pre.stride() == v_new.stride()
        assert k_pre.stride(3) == 1 and k_pre.element_size() == 2
        assert cos.dtype == torch.float32 and sin.dtype == torch.float32
        assert cos.is_contiguous() and sin.is_contiguous()
        assert tuple(cos.shape) == (k_pre.shape[1], k_pre.shape[3] // 2) and cos.shape == sin.shape
        kv_rope_quant_append(self.handle, layer, k_pre.data_ptr(), v_new.data_ptr(), k_pre.shape[1],
                             k_pre.stride(0), k_pre.stride(1), k_pre.stride(2), cos.data_ptr(),
                             sin.data_ptr(), pairing, self._stream())

    def append_compressv(self, layer: int, k_new, x, w_v, cos=None, sin=None, pairing: int = KV_ROPE_HALF, v_proj=None) -> None:
        """Alg. 1 steps 3 and 8: k_new [B, n_new, Hkv, d], x [B, n_new, model_dim], w_v [Hkv * d, model_dim]
        (all 16-bit device tensors); optional rotary tables for the keys; v_proj, if given, a contiguous
        [B, n_new, Hkv, d] tensor that receives the projected values."""
        assert k_new.stride(3) == 1 and x.stride(2) == 1 and w_v.is_contiguous()
        assert x.shape[0] == k_new.shape[0] and x.shape[1] == k_new.shape[1] and w_v.shape[1] == x.shape[2]
        assert v_proj is None or (v_proj.is_contiguous() and tuple(v_proj.shape) == tuple(k_new.shape))
        kv_compressv_append(self.handle, layer, k_new.data_ptr(), k_new.stride(0), k_new.stride(1), k_new.stride(2),
                            x.data_ptr(), x.stride(0), x.stride(1), w_v.data_ptr(), x.shape[2], k_new.shape[1],
                            cos.data_ptr() if cos is not None else 0, sin.data_ptr() if sin is not None else 0, pairing,
                            v_proj.data_ptr() if v_proj is not None else 0, self._stream())

    def attend(self, layer: int, q, out=None):
        """q: device [B, Hq, d] 16-bit contiguous -> float32 [B, Hq, d]."""
        torch = self.torch
        assert q.is_contiguous()
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=self.device)
        kv_decode_attn(self.handle, layer, q.data_ptr(), out.data_ptr(), self.workspace.data_ptr(),
                       self.ws_bytes, self._stream())
        return out

    def dequant(self, layer: int, t_cap: int):
        """The layer's reconstructed keys and values, float32 [B, t_cap, Hkv, d] each (zeros past a
        sequence's length)."""
        torch = self.torch
        shape = (self.cfg.batch, t_cap, self.cfg.n_kv_heads, self.cfg.head_dim)
        k = torch.zeros(shape, dtype=torch.float32, device=self.device)
        v = torch.zeros(shape, dtype=torch.float32, device=self.device)
        kv_dequant(self.handle, layer, k.data_ptr(), v.data_ptr(), t_cap, self._stream())
        return k, v

    def attend16(self, layer: int, q):
        """As attend, with the output in q's 16-bit type (split, then the narrowing merge)."""
        torch = self.torch
        assert q.is_contiguous()
        out = torch.empty(q.shape, dtype=q.dtype, device=self.device)
        kv_decode_attn_split(self.handle, layer, q.data_ptr(), self.workspace.data_ptr(), self.ws_bytes, self._stream())
        kv_decode_attn_merge16(self.handle, layer, out.data_ptr(), self.workspace.data_ptr(), self.ws_bytes, self._stream())
        return out

    def append_attend(self, layer: int, k_new, v_new, q, out=None):
        """One decode step: k_new, v_new [B, 1, Hkv, d] (or [B, Hkv, d]), q [B, Hq, d] -> float32 [B, Hq, d]."""
        torch = self.torch
        if k_new.dim() == 4:
            assert k_new.shape[1] == 1
            k_new, v_new = k_new[:, 0], v_new[:, 0]
        assert k_new.shape == v_new.shape and k_new.stride() == v_new.stride()
        assert k_new.stride(2) == 1 and k_new.element_size() == 2 and q.is_contiguous()
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=self.device)
        kv_append_decode_attn(self.handle, layer, k_new.data_ptr(), v_new.data_ptr(), k_new.stride(0),
                              k_new.stride(1), q.data_ptr(), out.data_ptr(), self.workspace.data_ptr(),
                              self.ws_bytes, self._stream())
        return out

    def lengths_to_device(self):
        """Device-resident lengths for decode steps that are replayed from a HIP graph: the lengths the
        cache holds now go to a device array (allocated here on first use)."""
        torch = self.torch
        if getattr(self, "dev_lengths", None) is None:
            self.dev_lengths = torch.zeros(kv_dev_lengths_bytes(self.cfg) // 4, dtype=torch.int32, device=self.device)
        kv_cache_lengths_to_device(self.handle, self.dev_lengths.data_ptr(), self._stream())

    def step_dev(self, layer: int, k_new, v_new, q, out) -> None:
        """One decode step on the device-resident lengths: k_new, v_new [B, Hkv, d], q [B, Hq, d] 16-bit,
        out [B, Hq, d] float32.  The cache's own lengths stay as they are (advance())."""
        assert k_new.shape == v_new.shape and k_new.stride() == v_new.stride()
        assert k_new.stride(2) == 1 and k_new.element_size() == 2 and q.is_contiguous() and out.is_contiguous()
        kv_decode_step_dev(self.handle, layer, k_new.data_ptr(), v_new.data_ptr(), k_new.stride(0), k_new.stride(1),
                           q.data_ptr(), out.data_ptr(), self.workspace.data_ptr(), self.ws_bytes, self._stream())

    def advance(self, n_steps: int, layer: int = -1) -> None:
        kv_cache_advance(self.handle, layer, n_steps)

    def lengths(self, layer: int, seq: Optional[int] = None):
        return kv_cache_len(self.handle, layer) if seq is None else kv_cache_len_seq(self.handle, layer, seq)

"""CPU oracle for the TaDA hot path -- TEST INFRASTRUCTURE, not the product.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It shares no code with the HIP path and never imports it.
"""
from .tada import (  # noqa: F401
    OracleConfig,
    OracleCache,
    attention,
    build_oracle,
    decode_block,
    encode_block,
    f16_to_f32,
    f64_to_16,
    f32_to_bf16,
    f32_to_f16,
    kv_bytes_ratio,
    pack_codes,
    project,
    project_f64,
    record_layout,
    rope,
    unpack_codes,
    widen,
)

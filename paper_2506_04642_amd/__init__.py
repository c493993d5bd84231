"""MI355X-native TaDA KV-cache hot path: mean-centred group quantisation with bit-packed append,
and decode attention that dequantises inside QK^T / softmax / PV (arxiv 2506.04642, Sec. 3 and
App. A).  The compute lives in ``csrc/`` (HIP for gfx950) behind the C ABI of
``include/tadakv.h``; ``binding`` marshals arguments to it and nothing else.
"""

__all__ = ["binding", "synth", "build"]

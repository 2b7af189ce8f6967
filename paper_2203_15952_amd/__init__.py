"""MI355X-native quantized dense layer for native quantization-aware training
(arxiv 2203.15952): abs-max quantizers, int4 weight packing, int8 MFMA
contraction with fused de-quantization, straight-through backward.

The compute lives in the HIP library under ``csrc/`` behind the C ABI declared
in ``include/aqt.h``; ``binding`` marshals arguments to it and nothing else.
"""
import importlib

__all__ = ["binding", "inputs"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)

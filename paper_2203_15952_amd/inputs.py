"""Seeded synthetic inputs shaped like the Conformer (L) dense layers.

This module holds no arithmetic of the quantization method: it only draws
tensors.  Tests, the smoke check and the benchmark feed the same host buffers
to the HIP library and to the CPU checker.

The shapes follow the Conformer (L) encoder of the paper's LibriSpeech setup
(Sec. 3.2: model width 512, 8 heads, depthwise kernel 32; feed-forward width
4x) at 32 utterances x 400 frames = 12800 tokens (65536 tokens for the training
step).  They stand in for LibriSpeech / Voice-Search features, which are not
available here.  "N(0, v)" is read as variance v.

Generator: numpy.random.default_rng(seed), float32 standard normals drawn in
the order activations, weights, bias, upstream gradient, then scaled in
float32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

EPI_NONE, EPI_SWISH, EPI_GLU = 0, 1, 2


@dataclass
class DenseCase:
    """One quantized dense layer call."""
    name: str
    M: int
    K: int
    N: int
    bits_x: int
    bits_w: int
    epilogue: int = EPI_NONE
    x: Optional[np.ndarray] = None      # [M, K] float32
    w: Optional[np.ndarray] = None      # [K, N] float32
    bias: Optional[np.ndarray] = None   # [N] float32
    dy: Optional[np.ndarray] = None     # [M, N] float32 (training step only)


def _normal(rng, shape, std):
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def _weights(rng, K, N):
    return _normal(rng, (K, N), 1.0 / np.sqrt(K))


def config1(seed: int = 0) -> List[DenseCase]:
    """Single layer, forward only: 256x256 -> 1024, int8 x int4."""
    rng = np.random.default_rng(seed)
    x = _normal(rng, (256, 256), 1.0)
    w = _weights(rng, 256, 1024)
    return [DenseCase("cfg1_dense", 256, 256, 1024, 8, 4, EPI_NONE, x, w)]


def config2(seed: int = 2, tokens: int = 12800) -> List[DenseCase]:
    """Feed-forward module: 512 -> 2048 (Swish) -> 512, int8 x int4.

    Each layer is drawn with its own activation tensor so that the two calls
    can be checked independently; the chained module feeds the second layer
    with the first one's output instead.
    """
    rng = np.random.default_rng(seed)
    x1 = _normal(rng, (tokens, 512), 1.0)
    w1 = _weights(rng, 512, 2048)
    w2 = _weights(rng, 2048, 512)
    x2 = _normal(rng, (tokens, 2048), 1.0)
    return [DenseCase("cfg2_ffn1_swish", tokens, 512, 2048, 8, 4, EPI_SWISH, x1, w1),
            DenseCase("cfg2_ffn2", tokens, 2048, 512, 8, 4, EPI_NONE, x2, w2)]


def config3(seed: int = 3, tokens: int = 12800) -> List[DenseCase]:
    """Self-attention projections, int8 x int8; 1% of activations are +-8 outliers."""
    rng = np.random.default_rng(seed)
    x = _normal(rng, (tokens, 512), 1.0)
    wqkv = _weights(rng, 512, 1536)
    wo = _weights(rng, 512, 512)
    hit = rng.random((tokens, 512)) < 0.01
    sign = np.where(rng.random((tokens, 512)) < 0.5, np.float32(-8.0), np.float32(8.0))
    x = np.where(hit, sign, x).astype(np.float32)
    return [DenseCase("cfg3_qkv", tokens, 512, 1536, 8, 8, EPI_NONE, x, wqkv),
            DenseCase("cfg3_out", tokens, 512, 512, 8, 8, EPI_NONE, x, wo)]


def config4(seed: int = 4, tokens: int = 12800) -> List[DenseCase]:
    """Convolution-module pointwise layers: 512 -> 1024 (int4, GLU -> 512), 512 -> 512 (int8)."""
    rng = np.random.default_rng(seed)
    x = _normal(rng, (tokens, 512), 1.0)
    w1 = _weights(rng, 512, 1024)
    w2 = _weights(rng, 512, 512)
    x2 = _normal(rng, (tokens, 512), 1.0)
    return [DenseCase("cfg4_pw1_glu", tokens, 512, 1024, 8, 4, EPI_GLU, x, w1),
            DenseCase("cfg4_pw2", tokens, 512, 512, 8, 8, EPI_NONE, x2, w2)]


def config5(seed: int = 1, tokens: int = 65536) -> List[DenseCase]:
    """Training step: two independent layers 512 -> 2048 and 2048 -> 512, int8 x int4,
    each with its own activations and upstream gradient (std 0.1)."""
    rng = np.random.default_rng(seed)
    x1 = _normal(rng, (tokens, 512), 1.0)
    x2 = _normal(rng, (tokens, 2048), 1.0)
    w1 = _weights(rng, 512, 2048)
    w2 = _weights(rng, 2048, 512)
    dy1 = _normal(rng, (tokens, 2048), 0.1)
    dy2 = _normal(rng, (tokens, 512), 0.1)
    return [DenseCase("cfg5_l1", tokens, 512, 2048, 8, 4, EPI_NONE, x1, w1, None, dy1),
            DenseCase("cfg5_l2", tokens, 2048, 512, 8, 4, EPI_NONE, x2, w2, None, dy2)]


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def small_case(seed: int, M: int, K: int, N: int, bits_x: int = 8, bits_w: int = 4,
               epilogue: int = EPI_NONE, with_bias: bool = False, with_dy: bool = True,
               outliers: bool = False) -> DenseCase:
    """A layer of arbitrary (ragged) shape with the same value recipe, for parity tests."""
    rng = np.random.default_rng(seed)
    x = _normal(rng, (M, K), 1.0)
    w = _weights(rng, K, N)
    bias = _normal(rng, (N,), 0.5) if with_bias else None
    dy = _normal(rng, (M, N), 0.1) if with_dy else None
    if outliers:
        hit = rng.random((M, K)) < 0.01
        x = np.where(hit, np.float32(8.0), x).astype(np.float32)
    return DenseCase(f"small_{M}x{K}x{N}_s{seed}", M, K, N, bits_x, bits_w, epilogue, x, w, bias, dy)

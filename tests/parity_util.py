"""Comparison rules between the HIP library and the CPU oracle.

Integer results (codes, packed bytes, masks, int32 accumulators) and scales
(each a single correctly rounded float32 operation) are compared for equality.

Float outputs: the de-quantized value v = float(acc) * (s_x * s_w) carries three
float32 roundings (~1.8e-7) and must sit within 1e-6 relative of the float64
oracle.  Where a bias is added the sum can cancel, so the yardstick is
|acc s_x s_w| + |bias|.  Activations propagate v's own tolerance through their
derivative (|swish'| <= 1.1, |sigmoid'| <= 1/4) on top of their own 1e-6.

Gradients: max-norm within 1e-4 of the oracle's max-norm, and every element
within 1e-4 of the sum of the magnitudes of its terms (a per-element relative
test is meaningless where a sum cancels).

Weight-only forward (a float contraction with no stated bar of its own): the
float operand is split into two bf16 terms, |a - hi - lo| <= 2^-18 |a|, every
product with an integer code is exact in float32, and the float32 accumulation
of K terms adds about sqrt(K) 2^-24 (typical) of the sum of magnitudes.  The
bound is 2^-15 of the sum of the magnitudes of the terms per element and 2^-15
of the largest reference value in max-norm: a factor 8 over the split error,
and small enough that a contraction which lost its low-order pass (errors of
2^-9 per term) fails it at every fan-in the layers here have.
"""
import numpy as np

REL_Y = 1e-6
REL_G = 1e-4
REL_F = 2.0 ** -15   # weight-only forward, see above
TINY = 1e-37   # below the float32 normal range relative error is not defined


def unpack_mask(words, n):
    """Bit i of the word array -> element i (uint8 0/1)."""
    w = np.ascontiguousarray(words).view(np.uint32)
    bits = ((w[:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1).astype(np.uint8)
    return bits.reshape(-1)[:n]


def sigmoid(v):
    return 1.0 / (1.0 + np.exp(-v))


def check_forward(y_gpu, ora, s_x, s_w, bias, epilogue):
    """ora: dict from the oracle with acc (int), pre (float64), y (float64)."""
    y = np.asarray(y_gpu, dtype=np.float64)
    pre = ora["pre"]
    mono = np.abs(ora["acc"].astype(np.float64) * float(s_x) * s_w.astype(np.float64)[None, :])
    tol_v = REL_Y * (mono + (0 if bias is None else np.abs(bias.astype(np.float64))[None, :])) + TINY
    if epilogue == 0:
        bad = np.abs(y - pre) > tol_v
    elif epilogue == 1:
        tol = REL_Y * np.abs(ora["y"]) + 1.1 * tol_v
        bad = np.abs(y - ora["y"]) > tol
    else:
        h = pre.shape[1] // 2
        a, g = pre[:, :h], pre[:, h:]
        tol = REL_Y * np.abs(ora["y"]) + sigmoid(g) * tol_v[:, :h] + 0.25 * np.abs(a) * tol_v[:, h:] + TINY
        bad = np.abs(y - ora["y"]) > tol
    assert not bad.any(), f"{bad.sum()} of {bad.size} outputs outside tolerance"


def check_grad(g_gpu, g_ref, g_abs, what):
    g = np.asarray(g_gpu, dtype=np.float64)
    err = np.abs(g - g_ref)
    assert err.max() <= REL_G * np.abs(g_ref).max() + TINY, f"{what}: max-norm error {err.max()}"
    bad = err > REL_G * g_abs + TINY
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} elements outside 1e-4 of sum|terms|"


def check_float_forward(y_gpu, ora, epilogue):
    """Weight-only forward: a float contraction, so the pre-activation value is held to
    REL_F of the sum of the magnitudes of its terms (and of the largest value, in max-norm)
    and activations propagate that tolerance through their derivatives.  ora: dict(pre, y, mag) from the oracle."""
    y = np.asarray(y_gpu, dtype=np.float64)
    pre, tol_v = ora["pre"], REL_F * ora["mag"] + TINY
    if epilogue == 0:
        bad = np.abs(y - pre) > tol_v
        assert np.abs(y - pre).max() <= REL_F * np.abs(pre).max() + TINY, "max-norm error"
    elif epilogue == 1:
        bad = np.abs(y - ora["y"]) > REL_Y * np.abs(ora["y"]) + 1.1 * tol_v
    else:
        h = pre.shape[1] // 2
        a, g = pre[:, :h], pre[:, h:]
        tol = REL_Y * np.abs(ora["y"]) + sigmoid(g) * tol_v[:, :h] + 0.25 * np.abs(a) * tol_v[:, h:] + TINY
        bad = np.abs(y - ora["y"]) > tol
    assert not bad.any(), f"{bad.sum()} of {bad.size} outputs outside tolerance"

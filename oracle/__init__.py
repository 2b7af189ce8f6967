"""CPU oracle for the quantized dense layer of native QAT (arxiv 2203.15952).

TEST INFRASTRUCTURE ONLY.  This package wraps ``aqt_oracle.c`` (plain C, built
with gcc) for the tests, the smoke check and the benchmark's CPU-baseline leg.
It shares nothing with the HIP library and must never be imported by it.

Every function returns numpy arrays; the arithmetic all lives in the C file,
whose header says which passage of the paper each routine follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aqt_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

AXIS_ALL = -1
EPI_NONE, EPI_SWISH, EPI_GLU = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _c():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i8(a):
    return np.ascontiguousarray(a, dtype=np.int8)


def num_threads() -> int:
    return int(_c().oracle_num_threads())


def _scale_len(rows, cols, axis):
    return 1 if axis == AXIS_ALL else (cols if axis == 0 else rows)


def quantize(x, bits: int, axis: int, want_mask: bool = False):
    """Fig. 2 + the 127/7 rule.  Returns (codes int8, scale f32[, mask u8])."""
    x = _f32(x)
    rows, cols = x.shape
    q = np.empty((rows, cols), np.int8)
    s = np.empty(_scale_len(rows, cols, axis), np.float32)
    mask = np.empty((rows, cols), np.uint8) if want_mask else None
    rc = _c().oracle_quantize(_p(x), ctypes.c_int64(rows), ctypes.c_int64(cols), bits, axis,
                              _p(q), _p(s), _p(mask))
    if rc == 1:
        raise FloatingPointError("non-finite input")
    if rc:
        raise ValueError(f"oracle_quantize rc={rc}")
    return (q, s, mask) if want_mask else (q, s)


def quantize_with_scale(x, bits: int, axis: int, scale):
    """Element-wise half of Fig. 2 with caller-supplied scales.  Returns (codes, mask)."""
    x = _f32(x)
    rows, cols = x.shape
    scale = _f32(np.atleast_1d(scale))
    assert scale.size == _scale_len(rows, cols, axis)
    q = np.empty((rows, cols), np.int8)
    mask = np.empty((rows, cols), np.uint8)
    rc = _c().oracle_quantize_with_scale(_p(x), ctypes.c_int64(rows), ctypes.c_int64(cols), bits,
                                         axis, _p(scale), _p(q), _p(mask))
    if rc:
        raise ValueError(f"oracle_quantize_with_scale rc={rc}")
    return q, mask


def pack_int4(codes_kn):
    """codes [K,N] -> bytes [N, ceil(K/2)], low nibble = even k."""
    codes_kn = _i8(codes_kn)
    K, N = codes_kn.shape
    out = np.empty((N, (K + 1) // 2), np.uint8)
    _c().oracle_pack_int4(_p(codes_kn), ctypes.c_int64(K), ctypes.c_int64(N), _p(out))
    return out


def _out_cols(N, epilogue):
    return N // 2 if epilogue == EPI_GLU else N


def dense_fwd_q(xq, s_x, wq_kn, s_w, bias=None, epilogue: int = EPI_NONE):
    """Integer contraction + de-quantization.  Returns dict(acc int32, y f64, pre f64)."""
    xq, wq_kn, s_w = _i8(xq), _i8(wq_kn), _f32(s_w)
    M, K = xq.shape
    K2, N = wq_kn.shape
    assert K == K2 and s_w.size == N
    bias = None if bias is None else _f32(bias)
    acc = np.empty((M, N), np.int32)
    y = np.empty((M, _out_cols(N, epilogue)), np.float64)
    pre = np.empty((M, N), np.float64)
    rc = _c().oracle_dense_fwd_q(_p(xq), ctypes.c_float(float(s_x)), _p(wq_kn), _p(s_w),
                                 ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(N),
                                 _p(bias), epilogue, _p(acc), _p(y), _p(pre))
    if rc == 3:
        raise OverflowError("integer sum does not fit int32")
    if rc:
        raise ValueError(f"oracle_dense_fwd_q rc={rc}")
    return dict(acc=acc, y=y, pre=pre)


def dense_fwd_wonly(x, wq_kn, s_w, bias=None, epilogue: int = EPI_NONE):
    """Weight-only forward (float32 activations x de-quantized integer weights).
    Returns dict(y f64, pre f64, mag f64)."""
    x, wq_kn, s_w = _f32(x), _i8(wq_kn), _f32(s_w)
    M, K = x.shape
    K2, N = wq_kn.shape
    assert K == K2 and s_w.size == N
    bias = None if bias is None else _f32(bias)
    y = np.empty((M, _out_cols(N, epilogue)), np.float64)
    pre = np.empty((M, N), np.float64)
    mag = np.empty((M, N), np.float64)
    rc = _c().oracle_dense_fwd_wonly(_p(x), _p(wq_kn), _p(s_w), ctypes.c_int64(M), ctypes.c_int64(K),
                                     ctypes.c_int64(N), _p(bias), epilogue, _p(y), _p(pre), _p(mag))
    if rc:
        raise ValueError(f"oracle_dense_fwd_wonly rc={rc}")
    return dict(y=y, pre=pre, mag=mag)


def dense_fwd_wonly_sampled(x, wq_kn, s_w, idx_m, idx_n, bias=None):
    """Weight-only pre-activation values and term magnitudes at sampled positions."""
    x, wq_kn, s_w = _f32(x), _i8(wq_kn), _f32(s_w)
    K, N = wq_kn.shape
    bias = None if bias is None else _f32(bias)
    im = np.ascontiguousarray(idx_m, np.int64)
    inn = np.ascontiguousarray(idx_n, np.int64)
    pre = np.empty(im.size, np.float64)
    mag = np.empty(im.size, np.float64)
    _c().oracle_dense_fwd_wonly_sampled(_p(x), _p(wq_kn), _p(s_w), ctypes.c_int64(K), ctypes.c_int64(N),
                                        _p(bias), _p(im), _p(inn), ctypes.c_int64(im.size), _p(pre), _p(mag))
    return pre, mag


def dense_fwd(x, w, bits_x: int, bits_w: int, bias=None, epilogue: int = EPI_NONE):
    """Whole forward layer.  Returns dict(xq, s_x, wq, s_w, acc, y, pre)."""
    x, w = _f32(x), _f32(w)
    M, K = x.shape
    K2, N = w.shape
    assert K == K2
    bias = None if bias is None else _f32(bias)
    xq = np.empty((M, K), np.int8)
    s_x = np.empty(1, np.float32)
    wq = np.empty((K, N), np.int8)
    s_w = np.empty(N, np.float32)
    acc = np.empty((M, N), np.int32)
    y = np.empty((M, _out_cols(N, epilogue)), np.float64)
    pre = np.empty((M, N), np.float64)
    rc = _c().oracle_dense_fwd(_p(x), _p(w), ctypes.c_int64(M), ctypes.c_int64(K),
                               ctypes.c_int64(N), bits_x, bits_w, _p(bias), epilogue,
                               _p(xq), _p(s_x), _p(wq), _p(s_w), _p(acc), _p(y), _p(pre))
    if rc == 1:
        raise FloatingPointError("non-finite input")
    if rc == 3:
        raise OverflowError("integer sum does not fit int32")
    if rc:
        raise ValueError(f"oracle_dense_fwd rc={rc}")
    return dict(xq=xq, s_x=s_x, wq=wq, s_w=s_w, acc=acc, y=y, pre=pre)


def dense_bwd(dy, xq, s_x, wq_kn, s_w, mask_x=None, mask_w=None,
              want_dx=True, want_dw=True, want_dbias=True):
    """Straight-through backward in float64.  Returns dict(dx, dw, dbias, dx_abs, dw_abs)."""
    dy, xq, wq_kn, s_w = _f32(dy), _i8(xq), _i8(wq_kn), _f32(s_w)
    M, N = dy.shape
    K = xq.shape[1]
    assert xq.shape == (M, K) and wq_kn.shape == (K, N) and s_w.size == N
    mx = None if mask_x is None else np.ascontiguousarray(mask_x, np.uint8)
    mw = None if mask_w is None else np.ascontiguousarray(mask_w, np.uint8)
    dx = np.empty((M, K), np.float64) if want_dx else None
    dxa = np.empty((M, K), np.float64) if want_dx else None
    dw = np.empty((K, N), np.float64) if want_dw else None
    dwa = np.empty((K, N), np.float64) if want_dw else None
    db = np.empty(N, np.float64) if want_dbias else None
    _c().oracle_dense_bwd(_p(dy), _p(xq), ctypes.c_float(float(s_x)), _p(mx), _p(wq_kn), _p(s_w),
                          _p(mw), ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(N),
                          _p(dx), _p(dw), _p(db), _p(dxa), _p(dwa))
    return dict(dx=dx, dw=dw, dbias=db, dx_abs=dxa, dw_abs=dwa)


def _idx(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def dense_fwd_q_sampled(xq, s_x, wq_kn, s_w, idx_m, idx_n, bias=None):
    """The forward definition at listed (m, n) only.  Returns (acc int64, pre f64)."""
    xq, wq_kn, s_w = _i8(xq), _i8(wq_kn), _f32(s_w)
    K, N = wq_kn.shape
    idx_m, idx_n = _idx(idx_m), _idx(idx_n)
    cnt = idx_m.size
    bias = None if bias is None else _f32(bias)
    acc = np.empty(cnt, np.int64)
    pre = np.empty(cnt, np.float64)
    _c().oracle_dense_fwd_q_sampled(_p(xq), ctypes.c_float(float(s_x)), _p(wq_kn), _p(s_w),
                                    ctypes.c_int64(K), ctypes.c_int64(N), _p(bias),
                                    _p(idx_m), _p(idx_n), ctypes.c_int64(cnt), _p(acc), _p(pre))
    return acc, pre


def dense_bwd_dx_sampled(dy, wq_kn, s_w, idx_m, idx_k):
    dy, wq_kn, s_w = _f32(dy), _i8(wq_kn), _f32(s_w)
    K, N = wq_kn.shape
    idx_m, idx_k = _idx(idx_m), _idx(idx_k)
    cnt = idx_m.size
    dx = np.empty(cnt, np.float64)
    dxa = np.empty(cnt, np.float64)
    _c().oracle_dense_bwd_dx_sampled(_p(dy), _p(wq_kn), _p(s_w), ctypes.c_int64(K),
                                     ctypes.c_int64(N), _p(idx_m), _p(idx_k),
                                     ctypes.c_int64(cnt), _p(dx), _p(dxa))
    return dx, dxa


def dense_bwd_dw_sampled(dy, xq, s_x, idx_k, idx_n):
    dy, xq = _f32(dy), _i8(xq)
    M, N = dy.shape
    K = xq.shape[1]
    idx_k, idx_n = _idx(idx_k), _idx(idx_n)
    cnt = idx_k.size
    dw = np.empty(cnt, np.float64)
    dwa = np.empty(cnt, np.float64)
    _c().oracle_dense_bwd_dw_sampled(_p(dy), _p(xq), ctypes.c_float(float(s_x)),
                                     ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(N),
                                     _p(idx_k), _p(idx_n), ctypes.c_int64(cnt), _p(dw), _p(dwa))
    return dw, dwa


def epilogue_dact(pre, epilogue: int):
    """Derivative factors of the activation: dv[m,n] = dout[m, n mod out_cols] * dact[m,n]."""
    pre = np.ascontiguousarray(pre, np.float64)
    M, N = pre.shape
    dact = np.empty((M, N), np.float64)
    rc = _c().oracle_epilogue_dact(_p(pre), ctypes.c_int64(M), ctypes.c_int64(N), epilogue, _p(dact))
    if rc:
        raise ValueError(f"oracle_epilogue_dact rc={rc}")
    return dact


def dense_bwd_epi(dout, pre, epilogue: int, xq, s_x, wq_kn, s_w, mask_x=None, mask_w=None,
                  want_dx=True, want_dw=True, want_dbias=True):
    """Straight-through backward through the activation, float64.
    Returns dict(dx, dw, dbias, dx_abs, dw_abs, dv)."""
    dout, xq, wq_kn, s_w = _f32(dout), _i8(xq), _i8(wq_kn), _f32(s_w)
    pre = np.ascontiguousarray(pre, np.float64)
    M, N = pre.shape
    K = xq.shape[1]
    assert dout.shape == (M, _out_cols(N, epilogue)) and wq_kn.shape == (K, N)
    mx = None if mask_x is None else np.ascontiguousarray(mask_x, np.uint8)
    mw = None if mask_w is None else np.ascontiguousarray(mask_w, np.uint8)
    dx = np.empty((M, K), np.float64) if want_dx else None
    dxa = np.empty((M, K), np.float64) if want_dx else None
    dw = np.empty((K, N), np.float64) if want_dw else None
    dwa = np.empty((K, N), np.float64) if want_dw else None
    db = np.empty(N, np.float64) if want_dbias else None
    dv = np.empty((M, N), np.float64)
    rc = _c().oracle_dense_bwd_epi(_p(dout), _p(pre), epilogue, _p(xq), ctypes.c_float(float(s_x)), _p(mx),
                                   _p(wq_kn), _p(s_w), _p(mw), ctypes.c_int64(M), ctypes.c_int64(K),
                                   ctypes.c_int64(N), _p(dx), _p(dw), _p(db), _p(dxa), _p(dwa), _p(dv))
    if rc:
        raise ValueError(f"oracle_dense_bwd_epi rc={rc}")
    return dict(dx=dx, dw=dw, dbias=db, dx_abs=dxa, dw_abs=dwa, dv=dv)


def layernorm(x, gamma=None, beta=None, eps: float = 1e-6):
    """Per-row layer normalisation in float64 (biased variance)."""
    x = _f32(x)
    M, D = x.shape
    g = None if gamma is None else _f32(gamma)
    b = None if beta is None else _f32(beta)
    y = np.empty((M, D), np.float64)
    _c().oracle_layernorm(_p(x), ctypes.c_int64(M), ctypes.c_int64(D), _p(g), _p(b), ctypes.c_double(eps), _p(y))
    return y


def fake_matmul_f32(xq, wq_kn):
    """Product of the codes carried and accumulated in float32 (the "fake quantization" arithmetic)."""
    xq, wq_kn = _i8(xq), _i8(wq_kn)
    M, K = xq.shape
    N = wq_kn.shape[1]
    out = np.empty((M, N), np.float32)
    _c().oracle_fake_matmul_f32(_p(xq), _p(wq_kn), ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(N), _p(out))
    return out


def depthwise_conv(x, w, bias=None, pad_left: int = 0, want_abs: bool = False):
    """Depthwise convolution along time, float64.  x [B,T,C], w [kw,C], zero frames outside an utterance."""
    x, w = _f32(x), _f32(w)
    B, T, C = x.shape
    kw = w.shape[0]
    b = None if bias is None else _f32(bias)
    out = np.empty((B, T, C), np.float64)
    ab = np.empty((B, T, C), np.float64) if want_abs else None
    _c().oracle_depthwise_conv(_p(x), _p(w), _p(b), ctypes.c_int64(B), ctypes.c_int64(T), ctypes.c_int64(C),
                               ctypes.c_int64(kw), ctypes.c_int64(pad_left), _p(out), _p(ab))
    return (out, ab) if want_abs else out


def depthwise_conv_bwd(dout, x, w, pad_left: int = 0):
    """Gradients of depthwise_conv with respect to x, w and bias (float64) and the absolute-term sums."""
    x, w = _f32(x), _f32(w)
    dout = np.ascontiguousarray(dout, np.float64)
    B, T, C = x.shape
    kw = w.shape[0]
    dx, dxa = np.empty((B, T, C), np.float64), np.empty((B, T, C), np.float64)
    dw, dwa = np.empty((kw, C), np.float64), np.empty((kw, C), np.float64)
    db = np.empty(C, np.float64)
    _c().oracle_depthwise_conv_bwd(_p(dout), _p(x), _p(w), ctypes.c_int64(B), ctypes.c_int64(T), ctypes.c_int64(C),
                                   ctypes.c_int64(kw), ctypes.c_int64(pad_left), _p(dx), _p(dw), _p(db), _p(dxa),
                                   _p(dwa))
    return dict(dx=dx, dw=dw, dbias=db, dx_abs=dxa, dw_abs=dwa)


def affine_swish(v, a=None, b=None):
    """Per-channel scale and shift, then Swish; returns (out, d out / d v), float64.  v [M,C]."""
    v = np.ascontiguousarray(v, np.float64)
    M, C = v.shape
    aa = None if a is None else _f32(a)
    bb = None if b is None else _f32(b)
    out, df = np.empty((M, C), np.float64), np.empty((M, C), np.float64)
    _c().oracle_affine_swish(_p(v), ctypes.c_int64(M), ctypes.c_int64(C), _p(aa), _p(bb), _p(out), _p(df))
    return out, df


def attention(qkv, heads: int, left: int = -1, right: int = -1, want_mags: bool = False):
    """Scaled dot-product self-attention per utterance and head over the frames t - left .. t + right
    (negative: unlimited), float64.  qkv [B,T,3D] -> ctx [B,T,D] (and the magnitudes the error bounds use)."""
    qkv = _f32(qkv)
    B, T, D3 = qkv.shape
    D = D3 // 3
    ctx = np.empty((B, T, D), np.float64)
    smag = np.empty((B, T, heads), np.float64) if want_mags else None
    vmag = np.empty((B, T, D), np.float64) if want_mags else None
    rc = _c().oracle_attention(_p(qkv), ctypes.c_int64(B), ctypes.c_int64(T), ctypes.c_int64(D), ctypes.c_int64(heads),
                               ctypes.c_int64(left), ctypes.c_int64(right), _p(ctx), _p(smag), _p(vmag))
    if rc:
        raise ValueError(f"oracle_attention rc={rc}")
    return (ctx, smag, vmag) if want_mags else ctx


def attention_bwd(qkv, dctx, heads: int, left: int = -1, right: int = -1):
    """Gradient of attention() with respect to qkv for the upstream gradient dctx [B,T,D]; returns
    (dqkv [B,T,3D] float64, the sums of the magnitudes of the terms)."""
    qkv = _f32(qkv)
    B, T, D3 = qkv.shape
    D = D3 // 3
    dctx = np.ascontiguousarray(dctx, np.float64).reshape(B, T, D)
    dqkv, mag = np.empty((B, T, D3), np.float64), np.empty((B, T, D3), np.float64)
    rc = _c().oracle_attention_bwd(_p(qkv), _p(dctx), ctypes.c_int64(B), ctypes.c_int64(T), ctypes.c_int64(D),
                                   ctypes.c_int64(heads), ctypes.c_int64(left), ctypes.c_int64(right), _p(dqkv), _p(mag))
    if rc:
        raise ValueError(f"oracle_attention_bwd rc={rc}")
    return dqkv, mag


def layernorm_bwd(x, dy, gamma=None, eps: float = 1e-6):
    """Gradient of layernorm(): returns (dx [M,D], dgamma [D], dbeta [D]), float64."""
    x = _f32(x)
    M, D = x.shape
    dy = np.ascontiguousarray(dy, np.float64)
    g = None if gamma is None else _f32(gamma)
    dx, dg, db = np.empty((M, D), np.float64), np.empty(D, np.float64), np.empty(D, np.float64)
    _c().oracle_layernorm_bwd(_p(x), ctypes.c_int64(M), ctypes.c_int64(D), _p(g), ctypes.c_double(eps), _p(dy), _p(dx),
                              _p(dg), _p(db))
    return dx, dg, db

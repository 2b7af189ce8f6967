"""Thin ctypes binding over libaqt.so (the C ABI in include/aqt.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream, every step of the computation runs in the library's kernels.  There is
no CPU or PyTorch fallback: if the library is missing, importing a function here
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("AQT_LIB", os.path.join(_PKG, "libaqt.so"))   # AQT_LIB: e.g. the tracing build

AQT_OK, AQT_ERR_INVALID_ARG, AQT_ERR_UNSUPPORTED, AQT_ERR_WORKSPACE, AQT_ERR_HIP, AQT_ERR_NONFINITE, AQT_ERR_SCRATCH = range(7)
AQT_AXIS_ALL, AQT_AXIS_ROWS, AQT_AXIS_COLS = -1, 0, 1
AQT_EPI_NONE, AQT_EPI_SWISH, AQT_EPI_GLU = 0, 1, 2
(AQT_OP_QUANTIZE, AQT_OP_QUANTIZE_WEIGHTS, AQT_OP_DENSE_FWD, AQT_OP_DENSE_FWD_Q, AQT_OP_DENSE_BWD,
 AQT_OP_DENSE_FWD_WONLY, AQT_OP_DENSE_BWD_EPI, AQT_OP_LAYERNORM_QUANTIZE, AQT_OP_FFN_FWD, AQT_OP_FFN_BWD,
 AQT_OP_DEPTHWISE_CONV_BWD, AQT_OP_CONV_MODULE_FWD, AQT_OP_CONV_MODULE_BWD, AQT_OP_MHSA_FWD,
 AQT_OP_CONFORMER_LAYER_FWD, AQT_OP_ATTENTION_BWD, AQT_OP_LAYERNORM_BWD, AQT_OP_MHSA_BWD,
 AQT_OP_CONFORMER_LAYER_BWD) = range(19)
AQT_POLICY_ALL, AQT_POLICY_EXCEPT_FIRST_LAST, AQT_POLICY_EXCEPT_ATTENTION, AQT_POLICY_FIRST_K = range(4)

# every symbol include/aqt.h declares
SYMBOLS = ["aqt_status_string", "aqt_last_hip_error", "aqt_version", "aqt_workspace_bytes",
           "aqt_packed_weight_bytes", "aqt_quantize", "aqt_quantize_with_scale", "aqt_quantize_weights",
           "aqt_unpack_weights", "aqt_dense_fwd_q", "aqt_dense_fwd_q_absmax", "aqt_quantize_with_absmax",
           "aqt_dense_fwd_wonly", "aqt_dense_fwd", "aqt_dense_bwd", "aqt_dense_fwd_q_static",
           "aqt_static_scratch_bytes", "aqt_layernorm_quantize", "aqt_fake_matmul_f32", "aqt_policy_preset",
           "aqt_policy_weight_bytes", "aqt_ffn_fwd", "aqt_ffn_bwd", "aqt_prepared_weight_bytes",
           "aqt_prepare_weights", "aqt_dense_fwd_q_prepared", "aqt_depthwise_conv_fwd", "aqt_depthwise_conv_bwd",
           "aqt_conv_module_fwd", "aqt_conv_module_bwd", "aqt_attention_fwd", "aqt_mhsa_fwd",
           "aqt_residual_add", "aqt_conformer_layer_fwd", "aqt_attention_bwd",
           "aqt_layernorm_bwd", "aqt_mhsa_bwd", "aqt_conformer_layer_bwd"]


class AqtError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().aqt_status_string(status).decode()
        if status == AQT_ERR_HIP:
            msg += f" (hipError {lib().aqt_last_hip_error()})"
        super().__init__(f"{where}: {msg}")


class aqt_saved(ctypes.Structure):
    _fields_ = [("xq", ctypes.c_void_p), ("s_x", ctypes.c_void_p), ("mask_x", ctypes.c_void_p),
                ("wq_packed", ctypes.c_void_p), ("wq_kn", ctypes.c_void_p), ("s_w", ctypes.c_void_p),
                ("mask_w", ctypes.c_void_p), ("dact", ctypes.c_void_p), ("wprep", ctypes.c_void_p)]


class aqt_dense_policy(ctypes.Structure):
    _fields_ = [("bits_w", ctypes.c_int), ("bits_x", ctypes.c_int), ("weights_ready", ctypes.c_int)]


class aqt_layer_policy(ctypes.Structure):
    _fields_ = [(n, aqt_dense_policy) for n in ("ffn1_in", "ffn1_out", "attn_qkv", "attn_out", "conv_pw1",
                                                "conv_pw2", "ffn2_in", "ffn2_out")]


class aqt_ffn_saved(ctypes.Structure):
    _fields_ = [("l1", aqt_saved), ("l2", aqt_saved), ("h", ctypes.c_void_p), ("xn", ctypes.c_void_p),
                ("row_stats", ctypes.c_void_p)]


class aqt_conv_saved(ctypes.Structure):
    _fields_ = [("pw1", aqt_saved), ("pw2", aqt_saved), ("g", ctypes.c_void_p), ("s", ctypes.c_void_p),
                ("dfac", ctypes.c_void_p), ("row_stats", ctypes.c_void_p)]


class aqt_mhsa_saved(ctypes.Structure):
    _fields_ = [("qkv", aqt_saved), ("out", aqt_saved), ("qkv_f", ctypes.c_void_p), ("ctx", ctypes.c_void_p),
                ("row_stats", ctypes.c_void_p), ("lse", ctypes.c_void_p)]


LAYER_WEIGHT_NAMES = ("ffn1_ln_g", "ffn1_ln_b", "ffn1_w1", "ffn1_b1", "ffn1_w2", "ffn1_b2",
                      "att_ln_g", "att_ln_b", "att_wqkv", "att_bqkv", "att_wo", "att_bo",
                      "conv_ln_g", "conv_ln_b", "conv_w1", "conv_b1", "conv_wdw", "conv_bdw", "conv_norm_scale",
                      "conv_norm_shift", "conv_w2", "conv_b2",
                      "ffn2_ln_g", "ffn2_ln_b", "ffn2_w1", "ffn2_b1", "ffn2_w2", "ffn2_b2", "out_ln_g", "out_ln_b")


class aqt_conformer_layer_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in LAYER_WEIGHT_NAMES]


class aqt_conformer_layer_shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int64), ("T", ctypes.c_int64), ("D", ctypes.c_int64), ("H", ctypes.c_int64),
                ("heads", ctypes.c_int), ("kw", ctypes.c_int), ("pad_left", ctypes.c_int),
                ("left_context", ctypes.c_int), ("right_context", ctypes.c_int), ("ln_eps", ctypes.c_float)]


class aqt_conformer_layer_saved(ctypes.Structure):
    _fields_ = [("ffn1", aqt_ffn_saved), ("ffn2", aqt_ffn_saved), ("att", aqt_mhsa_saved), ("conv", aqt_conv_saved),
                ("r1", ctypes.c_void_p), ("r2", ctypes.c_void_p), ("r3", ctypes.c_void_p), ("r4", ctypes.c_void_p),
                ("m", ctypes.c_void_p), ("out_row_stats", ctypes.c_void_p)]


class aqt_conformer_layer_grads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in LAYER_WEIGHT_NAMES]


_lib = None
_i64, _int, _vp, _sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t


def lib() -> ctypes.CDLL:
    """Load libaqt.so; fail loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2203_15952_amd.build` (there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        L.aqt_status_string.restype = ctypes.c_char_p
        L.aqt_status_string.argtypes = [_int]
        L.aqt_last_hip_error.restype = _int
        L.aqt_version.restype = _int
        L.aqt_workspace_bytes.restype = _sz
        L.aqt_workspace_bytes.argtypes = [_int, _i64, _i64, _i64, _int, _int]
        L.aqt_packed_weight_bytes.restype = _sz
        L.aqt_packed_weight_bytes.argtypes = [_i64, _i64, _int]
        L.aqt_quantize.argtypes = [_vp, _i64, _i64, _i64, _int, _int, _vp, _vp, _vp, _vp, _sz, _vp, _vp]
        L.aqt_quantize_with_scale.argtypes = [_vp, _i64, _i64, _i64, _int, _int, _vp, _vp, _vp, _vp]
        L.aqt_quantize_weights.argtypes = [_vp, _i64, _i64, _int, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _vp]
        L.aqt_unpack_weights.argtypes = [_vp, _i64, _i64, _int, _vp, _vp]
        L.aqt_dense_fwd_q.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp, _int, _vp, _vp,
                                      _vp, _sz, _vp]
        L.aqt_dense_fwd_q_absmax.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp, _int, _vp,
                                             _vp, _vp, _sz, _vp]
        L.aqt_dense_fwd_q_static.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp, _int, _vp, _vp]
        L.aqt_static_scratch_bytes.restype = _sz
        L.aqt_prepared_weight_bytes.restype = _sz
        L.aqt_prepared_weight_bytes.argtypes = [_i64, _i64, _int]
        L.aqt_prepare_weights.argtypes = [_vp, _i64, _i64, _int, _vp, _vp]
        L.aqt_dense_fwd_q_prepared.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp, _int, _vp, _vp]
        L.aqt_quantize_with_absmax.argtypes = [_vp, _i64, _i64, _i64, _int, _vp, _vp, _vp, _vp, _vp, _vp]
        L.aqt_dense_fwd_wonly.argtypes = [_vp, _vp, _vp, _i64, _i64, _i64, _int, _vp, _int, _vp, _vp, _sz, _vp]
        L.aqt_dense_fwd.argtypes = [_vp, _vp, _i64, _i64, _i64, _int, _int, _vp, _int, _vp,
                                    ctypes.POINTER(aqt_saved), _vp, _sz, _vp, _vp]
        L.aqt_dense_bwd.argtypes = [_vp, ctypes.POINTER(aqt_saved), _i64, _i64, _i64, _int, _int, _int, _vp, _vp,
                                    _vp, _vp, _sz, _vp]
        L.aqt_layernorm_quantize.argtypes = [_vp, _i64, _i64, _vp, _vp, ctypes.c_float, _int, _vp, _vp, _vp, _vp,
                                             _vp, _sz, _vp, _vp]
        L.aqt_fake_matmul_f32.argtypes = [_vp, _vp, _i64, _i64, _i64, _vp, _vp]
        L.aqt_policy_preset.argtypes = [_int, _int, _int, _int, _int, ctypes.POINTER(aqt_layer_policy)]
        L.aqt_policy_weight_bytes.restype = _sz
        L.aqt_policy_weight_bytes.argtypes = [ctypes.POINTER(aqt_layer_policy), _int, _i64, _i64]
        L.aqt_ffn_fwd.argtypes = [_vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _vp, _i64, _i64, _i64,
                                  ctypes.POINTER(aqt_dense_policy), _vp, ctypes.POINTER(aqt_ffn_saved), _vp, _sz,
                                  _vp, _vp]
        L.aqt_ffn_bwd.argtypes = [_vp, ctypes.POINTER(aqt_ffn_saved), _i64, _i64, _i64,
                                  ctypes.POINTER(aqt_dense_policy), _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.aqt_depthwise_conv_fwd.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _int, _int, _vp, _vp, _int, _vp, _vp,
                                             _vp, _vp]
        L.aqt_depthwise_conv_bwd.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _vp, _vp, _vp, _vp,
                                             _sz, _vp]
        L.aqt_conv_module_fwd.argtypes = [_vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                          _i64, _i64, _i64, _int, _int, ctypes.POINTER(aqt_dense_policy), _vp,
                                          ctypes.POINTER(aqt_conv_saved), _vp, _sz, _vp, _vp]
        L.aqt_conv_module_bwd.argtypes = [_vp, ctypes.POINTER(aqt_conv_saved), _vp, _i64, _i64, _i64, _int, _int,
                                          ctypes.POINTER(aqt_dense_policy), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                          _sz, _vp]
        L.aqt_attention_fwd.argtypes = [_vp, _i64, _i64, _i64, _int, _int, _int, _vp, _vp, _vp, _vp]
        L.aqt_attention_bwd.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _int, _vp, _vp, _sz, _vp]
        L.aqt_mhsa_fwd.argtypes = [_vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int,
                                   _int, ctypes.POINTER(aqt_dense_policy), _vp, ctypes.POINTER(aqt_mhsa_saved), _vp,
                                   _sz, _vp, _vp]
        L.aqt_residual_add.argtypes = [_vp, _vp, ctypes.c_float, _vp, _i64, _vp]
        L.aqt_conformer_layer_fwd.argtypes = [_vp, ctypes.POINTER(aqt_conformer_layer_weights),
                                              ctypes.POINTER(aqt_conformer_layer_shape),
                                              ctypes.POINTER(aqt_layer_policy), _vp,
                                              ctypes.POINTER(aqt_conformer_layer_saved), _vp, _sz, _vp, _vp]
        L.aqt_layernorm_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
        L.aqt_mhsa_bwd.argtypes = [_vp, ctypes.POINTER(aqt_mhsa_saved), _i64, _i64, _i64, _int, _int, _int,
                                   ctypes.POINTER(aqt_dense_policy), _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.aqt_conformer_layer_bwd.argtypes = [_vp, _vp, ctypes.POINTER(aqt_conformer_layer_weights),
                                              ctypes.POINTER(aqt_conformer_layer_shape),
                                              ctypes.POINTER(aqt_layer_policy),
                                              ctypes.POINTER(aqt_conformer_layer_saved), _vp,
                                              ctypes.POINTER(aqt_conformer_layer_grads), _vp, _sz, _vp]
        for name in SYMBOLS:
            getattr(L, name)  # AttributeError if the library lacks a declared entry point
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != AQT_OK:
        raise AqtError(status, where)


def _dev(t: torch.Tensor, dtype, name: str):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous {dtype} device tensor")
    return t


def _words(n: int) -> int:
    return (n + 31) // 32


def aqt_workspace_bytes(op: int, M: int, K: int, N: int, bits_x: int = 8, bits_w: int = 4) -> int:
    return int(lib().aqt_workspace_bytes(op, M, K, N, bits_x, bits_w))


def aqt_packed_weight_bytes(K: int, N: int, bits_w: int) -> int:
    return int(lib().aqt_packed_weight_bytes(K, N, bits_w))


def workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def new_status(device="cuda") -> torch.Tensor:
    return torch.zeros(1, dtype=torch.int32, device=device)


def aqt_quantize(x, bits: int, axis: int, *, q=None, scale=None, clip_mask=None, want_mask=False,
                 ws=None, dev_status=None, ldx: Optional[int] = None, cols: Optional[int] = None):
    """aqt_quantize: returns (q int8 [rows, cols], scale float32, clip_mask or None)."""
    _dev(x, torch.float32, "x")
    rows = x.shape[0]
    cols = x.shape[1] if cols is None else cols
    ldx = x.shape[1] if ldx is None else ldx
    n_scale = 1 if axis == AQT_AXIS_ALL else (cols if axis == AQT_AXIS_ROWS else rows)
    q = torch.empty((rows, cols), dtype=torch.int8, device=x.device) if q is None else q
    scale = torch.empty(n_scale, dtype=torch.float32, device=x.device) if scale is None else scale
    if want_mask and clip_mask is None:
        clip_mask = torch.empty(_words(rows * cols), dtype=torch.int32, device=x.device)
    ws = workspace(aqt_workspace_bytes(AQT_OP_QUANTIZE, rows, cols, 1), x.device) if ws is None else ws
    st = lib().aqt_quantize(_ptr(x), rows, cols, ldx, bits, axis, _ptr(q), _ptr(scale), _ptr(clip_mask),
                            _ptr(ws), ws.numel(), _stream(), _ptr(dev_status))
    _check(st, "aqt_quantize")
    return q, scale, clip_mask


def aqt_quantize_with_scale(x, bits: int, axis: int, scale, *, q=None, clip_mask=None, want_mask=True):
    """aqt_quantize_with_scale: returns (q, clip_mask or None)."""
    _dev(x, torch.float32, "x")
    _dev(scale, torch.float32, "scale")
    rows, cols = x.shape
    q = torch.empty((rows, cols), dtype=torch.int8, device=x.device) if q is None else q
    if want_mask and clip_mask is None:
        clip_mask = torch.empty(_words(rows * cols), dtype=torch.int32, device=x.device)
    st = lib().aqt_quantize_with_scale(_ptr(x), rows, cols, cols, bits, axis, _ptr(scale), _ptr(q),
                                       _ptr(clip_mask), _stream())
    _check(st, "aqt_quantize_with_scale")
    return q, clip_mask


def aqt_quantize_weights(w, bits_w: int, *, wq_packed=None, s_w=None, wq_kn=None, clip_mask_w=None,
                         want_kn=True, want_mask=False, ws=None, dev_status=None):
    """aqt_quantize_weights: returns (wq_packed uint8, s_w float32 [N], wq_kn int8 [K,N] or None, mask or None)."""
    _dev(w, torch.float32, "w")
    K, N = w.shape
    if wq_packed is None:
        wq_packed = torch.empty(aqt_packed_weight_bytes(K, N, bits_w), dtype=torch.uint8, device=w.device)
    s_w = torch.empty(N, dtype=torch.float32, device=w.device) if s_w is None else s_w
    if want_kn and wq_kn is None:
        wq_kn = torch.empty((K, N), dtype=torch.int8, device=w.device)
    if want_mask and clip_mask_w is None:
        clip_mask_w = torch.empty(_words(K * N), dtype=torch.int32, device=w.device)
    ws = workspace(aqt_workspace_bytes(AQT_OP_QUANTIZE_WEIGHTS, 1, K, N), w.device) if ws is None else ws
    st = lib().aqt_quantize_weights(_ptr(w), K, N, bits_w, _ptr(wq_packed), _ptr(s_w), _ptr(wq_kn),
                                    _ptr(clip_mask_w), _ptr(ws), ws.numel(), _stream(), _ptr(dev_status))
    _check(st, "aqt_quantize_weights")
    return wq_packed, s_w, wq_kn, clip_mask_w


def aqt_unpack_weights(wq_packed, K: int, N: int, bits_w: int):
    codes = torch.empty((K, N), dtype=torch.int8, device=wq_packed.device)
    st = lib().aqt_unpack_weights(_ptr(wq_packed), K, N, bits_w, _ptr(codes), _stream())
    _check(st, "aqt_unpack_weights")
    return codes


def _out_cols(N: int, epilogue: int) -> int:
    return N // 2 if epilogue == AQT_EPI_GLU else N


def aqt_dense_fwd_q(xq, s_x, wq_packed, s_w, N: int, bits_x: int, bits_w: int, *, bias=None,
                    epilogue: int = AQT_EPI_NONE, y=None, acc_out=None, want_acc=False, ws=None):
    """aqt_dense_fwd_q: returns (y float32, acc int32 or None)."""
    _dev(xq, torch.int8, "xq")
    M, K = xq.shape
    if ws is None:
        ws = workspace(aqt_workspace_bytes(AQT_OP_DENSE_FWD_Q, M, K, N, bits_x, bits_w))
    y = torch.empty((M, _out_cols(N, epilogue)), dtype=torch.float32, device=xq.device) if y is None else y
    if want_acc and acc_out is None:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    st = lib().aqt_dense_fwd_q(_ptr(xq), _ptr(s_x), _ptr(wq_packed), _ptr(s_w), M, K, N, bits_x, bits_w,
                               _ptr(bias), epilogue, _ptr(y), _ptr(acc_out), _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_dense_fwd_q")
    return y, acc_out


def aqt_static_scratch_bytes() -> int:
    return int(lib().aqt_static_scratch_bytes())


def aqt_dense_fwd_q_static(xq, s_x, wq_packed, s_w, N: int, bits_x: int, bits_w: int, *, bias=None,
                           epilogue: int = AQT_EPI_NONE, y):
    """aqt_dense_fwd_q_static: the caller passes every buffer, the call allocates nothing."""
    _dev(xq, torch.int8, "xq")
    _dev(y, torch.float32, "y")
    M, K = xq.shape
    st = lib().aqt_dense_fwd_q_static(_ptr(xq), _ptr(s_x), _ptr(wq_packed), _ptr(s_w), M, K, N, bits_x, bits_w,
                                      _ptr(bias), epilogue, _ptr(y), _stream())
    _check(st, "aqt_dense_fwd_q_static")
    return y


def aqt_prepare_weights(wq_packed, K: int, N: int, bits_w: int):
    """aqt_prepare_weights: the forward operand re-ordered once for the matrix cores."""
    nbytes = int(lib().aqt_prepared_weight_bytes(K, N, bits_w))
    if nbytes == 0:
        raise AqtError(AQT_ERR_UNSUPPORTED, "aqt_prepared_weight_bytes")
    wprep = torch.empty(nbytes, dtype=torch.uint8, device=wq_packed.device)
    st = lib().aqt_prepare_weights(_ptr(wq_packed), K, N, bits_w, _ptr(wprep), _stream())
    _check(st, "aqt_prepare_weights")
    return wprep


def aqt_dense_fwd_q_prepared(xq, s_x, wprep, s_w, N: int, bits_x: int, bits_w: int, *, bias=None,
                             epilogue: int = AQT_EPI_NONE, y=None):
    """aqt_dense_fwd_q_prepared: the serving forward on a prepared weight operand, no workspace."""
    _dev(xq, torch.int8, "xq")
    M, K = xq.shape
    y = torch.empty((M, _out_cols(N, epilogue)), dtype=torch.float32, device=xq.device) if y is None else y
    st = lib().aqt_dense_fwd_q_prepared(_ptr(xq), _ptr(s_x), _ptr(wprep), _ptr(s_w), M, K, N, bits_x, bits_w,
                                        _ptr(bias), epilogue, _ptr(y), _stream())
    _check(st, "aqt_dense_fwd_q_prepared")
    return y


def aqt_dense_fwd_q_absmax(xq, s_x, wq_packed, s_w, N: int, bits_x: int, bits_w: int, *, bias=None,
                           epilogue: int = AQT_EPI_NONE, y=None, y_absmax=None, ws=None):
    """aqt_dense_fwd_q_absmax: returns (y float32, y_absmax float32 [1])."""
    _dev(xq, torch.int8, "xq")
    M, K = xq.shape
    if ws is None:
        ws = workspace(aqt_workspace_bytes(AQT_OP_DENSE_FWD_Q, M, K, N, bits_x, bits_w))
    y = torch.empty((M, _out_cols(N, epilogue)), dtype=torch.float32, device=xq.device) if y is None else y
    y_absmax = torch.empty(1, dtype=torch.float32, device=xq.device) if y_absmax is None else y_absmax
    st = lib().aqt_dense_fwd_q_absmax(_ptr(xq), _ptr(s_x), _ptr(wq_packed), _ptr(s_w), M, K, N, bits_x, bits_w,
                                      _ptr(bias), epilogue, _ptr(y), _ptr(y_absmax), _ptr(ws), ws.numel(),
                                      _stream())
    _check(st, "aqt_dense_fwd_q_absmax")
    return y, y_absmax


def aqt_quantize_with_absmax(x, bits: int, absmax, *, q=None, scale=None, clip_mask=None, want_mask=False,
                             dev_status=None):
    """aqt_quantize_with_absmax: returns (q int8, scale float32 [1], clip_mask or None)."""
    _dev(x, torch.float32, "x")
    _dev(absmax, torch.float32, "absmax")
    rows, cols = x.shape
    q = torch.empty((rows, cols), dtype=torch.int8, device=x.device) if q is None else q
    scale = torch.empty(1, dtype=torch.float32, device=x.device) if scale is None else scale
    if want_mask and clip_mask is None:
        clip_mask = torch.empty(_words(rows * cols), dtype=torch.int32, device=x.device)
    st = lib().aqt_quantize_with_absmax(_ptr(x), rows, cols, cols, bits, _ptr(absmax), _ptr(q), _ptr(scale),
                                        _ptr(clip_mask), _stream(), _ptr(dev_status))
    _check(st, "aqt_quantize_with_absmax")
    return q, scale, clip_mask


def aqt_dense_fwd_wonly(x, wq_packed, s_w, N: int, bits_w: int, *, bias=None, epilogue: int = AQT_EPI_NONE,
                        y=None, ws=None):
    """aqt_dense_fwd_wonly: float32 activations x integer weights; returns y float32."""
    _dev(x, torch.float32, "x")
    M, K = x.shape
    if ws is None:
        ws = workspace(aqt_workspace_bytes(AQT_OP_DENSE_FWD_WONLY, M, K, N, 8, bits_w))
    y = torch.empty((M, _out_cols(N, epilogue)), dtype=torch.float32, device=x.device) if y is None else y
    st = lib().aqt_dense_fwd_wonly(_ptr(x), _ptr(wq_packed), _ptr(s_w), M, K, N, bits_w, _ptr(bias), epilogue,
                                   _ptr(y), _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_dense_fwd_wonly")
    return y


class Saved:
    """Device buffers the forward keeps for the backward, plus their aqt_saved view."""

    def __init__(self, M: int, K: int, N: int, bits_w: int, device="cuda", masks: bool = False,
                 dact: bool = False):
        self.M, self.K, self.N, self.bits_w = M, K, N, bits_w
        self.wprep = None
        self.dact = torch.empty((M, N), dtype=torch.float32, device=device) if dact else None
        self.xq = torch.empty((M, K), dtype=torch.int8, device=device)
        self.s_x = torch.empty(1, dtype=torch.float32, device=device)
        self.wq_packed = torch.empty(aqt_packed_weight_bytes(K, N, bits_w), dtype=torch.uint8, device=device)
        self.wq_kn = torch.empty((K, N), dtype=torch.int8, device=device)
        self.s_w = torch.empty(N, dtype=torch.float32, device=device)
        self.mask_x = torch.empty(_words(M * K), dtype=torch.int32, device=device) if masks else None
        self.mask_w = torch.empty(_words(K * N), dtype=torch.int32, device=device) if masks else None
        self.refresh()

    def refresh(self):
        def a(t):
            return None if t is None else t.data_ptr()
        self.c = aqt_saved(a(self.xq), a(self.s_x), a(self.mask_x), a(self.wq_packed), a(self.wq_kn),
                           a(self.s_w), a(self.mask_w), a(self.dact), a(self.wprep))
        return self

    def prepare(self, w):
        """Serving: quantize the float32 weights w [K,N] into this layer's buffers once and, where the shape
        has one, keep the operand in matrix-core order; module calls with weights_ready = 1 then skip both."""
        aqt_quantize_weights(w, self.bits_w, wq_packed=self.wq_packed, s_w=self.s_w, wq_kn=self.wq_kn)
        if int(lib().aqt_prepared_weight_bytes(self.K, self.N, self.bits_w)):
            self.wprep = aqt_prepare_weights(self.wq_packed, self.K, self.N, self.bits_w)
        return self.refresh()


def aqt_dense_fwd(x, w, bits_x: int, bits_w: int, *, bias=None, epilogue: int = AQT_EPI_NONE, y=None,
                  saved: Optional[Saved] = None, ws=None, dev_status=None):
    """aqt_dense_fwd: returns y float32 [M,N] ([M,N/2] for GLU)."""
    _dev(x, torch.float32, "x")
    _dev(w, torch.float32, "w")
    M, K = x.shape
    N = w.shape[1]
    y = torch.empty((M, _out_cols(N, epilogue)), dtype=torch.float32, device=x.device) if y is None else y
    if ws is None:
        ws = workspace(aqt_workspace_bytes(AQT_OP_DENSE_FWD, M, K, N, bits_x, bits_w), x.device)
    sp = ctypes.byref(saved.c) if saved is not None else None
    st = lib().aqt_dense_fwd(_ptr(x), _ptr(w), M, K, N, bits_x, bits_w, _ptr(bias), epilogue, _ptr(y), sp,
                             _ptr(ws), ws.numel(), _stream(), _ptr(dev_status))
    _check(st, "aqt_dense_fwd")
    return y


def aqt_dense_bwd(dy, saved: Saved, bits_x: int, bits_w: int, *, epilogue: int = AQT_EPI_NONE, dx=None, dw=None,
                  dbias=None, want_dx=True, want_dw=True, want_dbias=False, ws=None):
    """aqt_dense_bwd: returns (dx [M,K], dw [K,N], dbias [N]); skipped outputs are None.
    dy is the gradient with respect to the layer's output ([M,N/2] for GLU)."""
    _dev(dy, torch.float32, "dy")
    M = dy.shape[0]
    N = saved.N
    K = saved.K
    if want_dx and dx is None:
        dx = torch.empty((M, K), dtype=torch.float32, device=dy.device)
    if want_dw and dw is None:
        dw = torch.empty((K, N), dtype=torch.float32, device=dy.device)
    if want_dbias and dbias is None:
        dbias = torch.empty(N, dtype=torch.float32, device=dy.device)
    if ws is None:
        op = AQT_OP_DENSE_BWD if epilogue == AQT_EPI_NONE else AQT_OP_DENSE_BWD_EPI
        ws = workspace(aqt_workspace_bytes(op, M, K, N, bits_x, bits_w), dy.device)
    st = lib().aqt_dense_bwd(_ptr(dy), ctypes.byref(saved.c), M, K, N, bits_x, bits_w, epilogue, _ptr(dx), _ptr(dw),
                             _ptr(dbias), _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_dense_bwd")
    return dx, dw, dbias


def aqt_layernorm_quantize(x, bits: int = 8, *, gamma=None, beta=None, eps: float = 1e-6, quantize=True,
                           want_y=False, want_stats=False, ws=None, dev_status=None):
    """aqt_layernorm_quantize: returns (q int8 or None, scale or None, y float32 or None, row_stats or None)."""
    _dev(x, torch.float32, "x")
    M, D = x.shape
    q = torch.empty((M, D), dtype=torch.int8, device=x.device) if quantize else None
    scale = torch.empty(1, dtype=torch.float32, device=x.device) if quantize else None
    y = torch.empty((M, D), dtype=torch.float32, device=x.device) if want_y else None
    stats = torch.empty((M, 2), dtype=torch.float32, device=x.device) if want_stats else None
    ws = workspace(aqt_workspace_bytes(AQT_OP_LAYERNORM_QUANTIZE, M, D, 1), x.device) if ws is None else ws
    st = lib().aqt_layernorm_quantize(_ptr(x), M, D, _ptr(gamma), _ptr(beta), eps, bits, _ptr(q), _ptr(scale),
                                      _ptr(y), _ptr(stats), _ptr(ws), ws.numel(), _stream(), _ptr(dev_status))
    _check(st, "aqt_layernorm_quantize")
    return q, scale, y, stats


def aqt_fake_matmul_f32(xq, wq_kn, *, out=None):
    """aqt_fake_matmul_f32: product of the codes carried and accumulated in float32."""
    _dev(xq, torch.int8, "xq")
    _dev(wq_kn, torch.int8, "wq_kn")
    M, K = xq.shape
    N = wq_kn.shape[1]
    out = torch.empty((M, N), dtype=torch.float32, device=xq.device) if out is None else out
    st = lib().aqt_fake_matmul_f32(_ptr(xq), _ptr(wq_kn), M, K, N, _ptr(out), _stream())
    _check(st, "aqt_fake_matmul_f32")
    return out


def aqt_policy_preset(pattern: int, n_layers: int, k: int, bits_w: int, bits_x: int):
    """aqt_policy_preset: returns a ctypes array of n_layers aqt_layer_policy (host memory, no GPU)."""
    arr = (aqt_layer_policy * n_layers)()
    st = lib().aqt_policy_preset(pattern, n_layers, k, bits_w, bits_x, arr)
    _check(st, "aqt_policy_preset")
    return arr


def aqt_policy_weight_bytes(policy, n_layers: int, d_model: int, d_ff: int) -> int:
    return int(lib().aqt_policy_weight_bytes(policy, n_layers, d_model, d_ff))


class FfnSaved:
    """Device buffers of the feed-forward module (aqt_ffn_fwd / aqt_ffn_bwd) and their aqt_ffn_saved view."""

    def __init__(self, M: int, D: int, H: int, policy, device="cuda"):
        (bw1, bx1), (bw2, bx2) = policy
        self.M, self.D, self.H = M, D, H
        self.l1 = Saved(M, D, H, bw1, device, dact=True)
        self.l2 = Saved(M, H, D, bw2, device)
        self.h = torch.empty((M, H), dtype=torch.float32, device=device)
        self.xn = torch.empty((M, D), dtype=torch.float32, device=device)
        self.row_stats = torch.empty((M, 2), dtype=torch.float32, device=device)
        self.policy = (aqt_dense_policy * 2)(aqt_dense_policy(bw1, bx1), aqt_dense_policy(bw2, bx2))
        self.refresh()

    def refresh(self):
        self.c = aqt_ffn_saved(self.l1.c, self.l2.c, self.h.data_ptr(), self.xn.data_ptr(), self.row_stats.data_ptr())
        return self

    def prepare(self, w1, w2):
        """Serving: quantize both weight matrices once; later calls skip the weight quantizers."""
        self.l1.prepare(w1)
        self.l2.prepare(w2)
        self.policy[0].weights_ready = self.policy[1].weights_ready = 1
        return self.refresh()


def aqt_ffn_fwd(x, w1, b1, w2, b2, saved: FfnSaved, *, gamma=None, beta=None, eps: float = 1e-6, y=None, ws=None,
                dev_status=None):
    """aqt_ffn_fwd: y = dense(swish(dense(layernorm(x), w1) + b1), w2) + b2 at the saved policy's precisions."""
    _dev(x, torch.float32, "x")
    M, D = x.shape
    H = saved.H
    y = torch.empty((M, D), dtype=torch.float32, device=x.device) if y is None else y
    ws = workspace(aqt_workspace_bytes(AQT_OP_FFN_FWD, M, D, H), x.device) if ws is None else ws
    st = lib().aqt_ffn_fwd(_ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(w1), _ptr(b1), _ptr(w2), _ptr(b2), M, D, H,
                           saved.policy, _ptr(y), ctypes.byref(saved.c), _ptr(ws), ws.numel(), _stream(),
                           _ptr(dev_status))
    _check(st, "aqt_ffn_fwd")
    return y


def aqt_ffn_bwd(dy, saved: FfnSaved, *, want_db=True, ws=None):
    """aqt_ffn_bwd: returns (dxn [M,D], dw1 [D,H], db1 [H] or None, dw2 [H,D], db2 [D] or None)."""
    _dev(dy, torch.float32, "dy")
    M, D, H = saved.M, saved.D, saved.H
    dev = dy.device
    dxn = torch.empty((M, D), dtype=torch.float32, device=dev)
    dw1 = torch.empty((D, H), dtype=torch.float32, device=dev)
    dw2 = torch.empty((H, D), dtype=torch.float32, device=dev)
    db1 = torch.empty(H, dtype=torch.float32, device=dev) if want_db else None
    db2 = torch.empty(D, dtype=torch.float32, device=dev) if want_db else None
    ws = workspace(aqt_workspace_bytes(AQT_OP_FFN_BWD, M, D, H), dev) if ws is None else ws
    st = lib().aqt_ffn_bwd(_ptr(dy), ctypes.byref(saved.c), M, D, H, saved.policy, _ptr(dxn), _ptr(dw1), _ptr(db1),
                           _ptr(dw2), _ptr(db2), _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_ffn_bwd")
    return dxn, dw1, db1, dw2, db2


def aqt_depthwise_conv_fwd(x, w, *, bias=None, pad_left: int = 0, norm_scale=None, norm_shift=None, swish=False,
                           want_dfac=False, want_absmax=False):
    """aqt_depthwise_conv_fwd: x [B,T,C], w [kw,C]; returns (out, dfac or None, absmax word or None)."""
    _dev(x, torch.float32, "x")
    _dev(w, torch.float32, "w")
    B, T, C = x.shape
    kw = w.shape[0]
    out = torch.empty_like(x)
    dfac = torch.empty_like(x) if want_dfac else None
    m = torch.empty(1, dtype=torch.float32, device=x.device) if want_absmax else None
    st = lib().aqt_depthwise_conv_fwd(_ptr(x), B, T, C, _ptr(w), _ptr(bias), kw, pad_left, _ptr(norm_scale),
                                      _ptr(norm_shift), int(bool(swish)), _ptr(out), _ptr(dfac), _ptr(m), _stream())
    _check(st, "aqt_depthwise_conv_fwd")
    return out, dfac, m


def aqt_depthwise_conv_bwd(dout, x, w, *, dfac=None, pad_left: int = 0, want_dx=True, want_dw=True,
                           want_dbias=True, ws=None):
    """aqt_depthwise_conv_bwd: returns (dx [B,T,C], dw [kw,C], dbias [C]); skipped outputs are None."""
    _dev(dout, torch.float32, "dout")
    B, T, C = dout.shape
    kw = w.shape[0]
    dev = dout.device
    dx = torch.empty_like(dout) if want_dx else None
    dw = torch.empty((kw, C), dtype=torch.float32, device=dev) if want_dw else None
    db = torch.empty(C, dtype=torch.float32, device=dev) if want_dbias else None
    ws = workspace(aqt_workspace_bytes(AQT_OP_DEPTHWISE_CONV_BWD, B * T, C, kw), dev) if ws is None else ws
    st = lib().aqt_depthwise_conv_bwd(_ptr(dout), _ptr(dfac), _ptr(x), _ptr(w), B, T, C, kw, pad_left, _ptr(dx),
                                      _ptr(dw), _ptr(db), _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_depthwise_conv_bwd")
    return dx, dw, db


class ConvSaved:
    """Device buffers of the convolution module (aqt_conv_module_fwd / _bwd) and their aqt_conv_saved view."""

    def __init__(self, B: int, T: int, D: int, policy, device="cuda"):
        (bw1, bx1), (bw2, bx2) = policy
        M = B * T
        self.B, self.T, self.D, self.M = B, T, D, M
        self.pw1 = Saved(M, D, 2 * D, bw1, device, dact=True)
        self.pw2 = Saved(M, D, D, bw2, device)
        self.g = torch.empty((M, D), dtype=torch.float32, device=device)
        self.s = torch.empty((M, D), dtype=torch.float32, device=device)
        self.dfac = torch.empty((M, D), dtype=torch.float32, device=device)
        self.row_stats = torch.empty((M, 2), dtype=torch.float32, device=device)
        self.policy = (aqt_dense_policy * 2)(aqt_dense_policy(bw1, bx1), aqt_dense_policy(bw2, bx2))
        self.refresh()

    def refresh(self):
        self.c = aqt_conv_saved(self.pw1.c, self.pw2.c, self.g.data_ptr(), self.s.data_ptr(), self.dfac.data_ptr(),
                                self.row_stats.data_ptr())
        return self

    def prepare(self, w1, w2):
        """Serving: quantize both pointwise weight matrices once; later calls skip the weight quantizers."""
        self.pw1.prepare(w1)
        self.pw2.prepare(w2)
        self.policy[0].weights_ready = self.policy[1].weights_ready = 1
        return self.refresh()


def aqt_conv_module_fwd(x, w1, b1, w_dw, b_dw, w2, b2, saved: ConvSaved, *, pad_left: int, gamma=None, beta=None,
                        eps: float = 1e-6, norm_scale=None, norm_shift=None, y=None, ws=None, dev_status=None):
    """aqt_conv_module_fwd: layernorm, pointwise + GLU, depthwise + normalisation + Swish, pointwise.  x [B*T,D]."""
    _dev(x, torch.float32, "x")
    M, D = x.shape
    kw = w_dw.shape[0]
    y = torch.empty((M, D), dtype=torch.float32, device=x.device) if y is None else y
    ws = workspace(aqt_workspace_bytes(AQT_OP_CONV_MODULE_FWD, M, D, kw), x.device) if ws is None else ws
    st = lib().aqt_conv_module_fwd(_ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(w1), _ptr(b1), _ptr(w_dw), _ptr(b_dw),
                                   _ptr(norm_scale), _ptr(norm_shift), _ptr(w2), _ptr(b2), saved.B, saved.T, D, kw,
                                   pad_left, saved.policy, _ptr(y), ctypes.byref(saved.c), _ptr(ws), ws.numel(),
                                   _stream(), _ptr(dev_status))
    _check(st, "aqt_conv_module_fwd")
    return y


def aqt_conv_module_bwd(dy, saved: ConvSaved, w_dw, *, pad_left: int, ws=None):
    """aqt_conv_module_bwd: returns dict(dxn, dw1, db1, dw_dw, db_dw, dw2, db2)."""
    _dev(dy, torch.float32, "dy")
    M, D = saved.M, saved.D
    kw = w_dw.shape[0]
    dev = dy.device
    f32 = dict(dtype=torch.float32, device=dev)
    o = dict(dxn=torch.empty((M, D), **f32), dw1=torch.empty((D, 2 * D), **f32), db1=torch.empty(2 * D, **f32),
             dw_dw=torch.empty((kw, D), **f32), db_dw=torch.empty(D, **f32), dw2=torch.empty((D, D), **f32),
             db2=torch.empty(D, **f32))
    ws = workspace(aqt_workspace_bytes(AQT_OP_CONV_MODULE_BWD, M, D, kw), dev) if ws is None else ws
    st = lib().aqt_conv_module_bwd(_ptr(dy), ctypes.byref(saved.c), _ptr(w_dw), saved.B, saved.T, D, kw, pad_left,
                                   saved.policy, _ptr(o["dxn"]), _ptr(o["dw1"]), _ptr(o["db1"]), _ptr(o["dw_dw"]),
                                   _ptr(o["db_dw"]), _ptr(o["dw2"]), _ptr(o["db2"]), _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_conv_module_bwd")
    return o


def aqt_attention_fwd(qkv, B: int, T: int, heads: int, *, left: int = -1, right: int = -1, want_absmax=False,
                      lse=None):
    """aqt_attention_fwd: qkv [B*T, 3D] -> (ctx [B*T, D], absmax word or None); lse [B*T, heads] is filled if given."""
    _dev(qkv, torch.float32, "qkv")
    M, D3 = qkv.shape
    D = D3 // 3
    ctx = torch.empty((M, D), dtype=torch.float32, device=qkv.device)
    m = torch.empty(1, dtype=torch.float32, device=qkv.device) if want_absmax else None
    st = lib().aqt_attention_fwd(_ptr(qkv), B, T, D, heads, left, right, _ptr(ctx), _ptr(m), _ptr(lse), _stream())
    _check(st, "aqt_attention_fwd")
    return ctx, m


def aqt_attention_bwd(qkv, ctx, dctx, lse, B: int, T: int, heads: int, *, left: int = -1, right: int = -1, ws=None):
    """aqt_attention_bwd: returns dqkv [B*T, 3D]."""
    _dev(qkv, torch.float32, "qkv")
    _dev(dctx, torch.float32, "dctx")
    M, D3 = qkv.shape
    D = D3 // 3
    dqkv = torch.empty_like(qkv)
    ws = workspace(aqt_workspace_bytes(AQT_OP_ATTENTION_BWD, M, 1, heads), qkv.device) if ws is None else ws
    st = lib().aqt_attention_bwd(_ptr(qkv), _ptr(ctx), _ptr(dctx), _ptr(lse), B, T, D, heads, left, right, _ptr(dqkv),
                                 _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_attention_bwd")
    return dqkv


class MhsaSaved:
    """Device buffers of the self-attention module (aqt_mhsa_fwd) and their aqt_mhsa_saved view."""

    def __init__(self, B: int, T: int, D: int, policy, device="cuda", heads: int = 0):
        (bw1, bx1), (bw2, bx2) = policy
        M = B * T
        self.B, self.T, self.D, self.M = B, T, D, M
        self.qkv = Saved(M, D, 3 * D, bw1, device)
        self.out = Saved(M, D, D, bw2, device)
        self.qkv_f = torch.empty((M, 3 * D), dtype=torch.float32, device=device)
        self.ctx = torch.empty((M, D), dtype=torch.float32, device=device)
        self.row_stats = torch.empty((M, 2), dtype=torch.float32, device=device)
        # the softmax normalisers, kept for the backward when the head count is given
        self.lse = torch.empty((M, heads), dtype=torch.float32, device=device) if heads else None
        self.policy = (aqt_dense_policy * 2)(aqt_dense_policy(bw1, bx1), aqt_dense_policy(bw2, bx2))
        self.refresh()

    def refresh(self):
        self.c = aqt_mhsa_saved(self.qkv.c, self.out.c, self.qkv_f.data_ptr(), self.ctx.data_ptr(),
                                self.row_stats.data_ptr(), None if self.lse is None else self.lse.data_ptr())
        return self

    def prepare(self, wqkv, wo):
        """Serving: quantize both projection matrices once; later calls skip the weight quantizers."""
        self.qkv.prepare(wqkv)
        self.out.prepare(wo)
        self.policy[0].weights_ready = self.policy[1].weights_ready = 1
        return self.refresh()


def aqt_mhsa_fwd(x, wqkv, bqkv, wo, bo, saved: MhsaSaved, heads: int, *, left: int = -1, right: int = -1, gamma=None,
                 beta=None, eps: float = 1e-6, y=None, ws=None, dev_status=None):
    """aqt_mhsa_fwd: layernorm, fused QKV projection, float attention, output projection.  x [B*T, D]."""
    _dev(x, torch.float32, "x")
    M, D = x.shape
    y = torch.empty((M, D), dtype=torch.float32, device=x.device) if y is None else y
    ws = workspace(aqt_workspace_bytes(AQT_OP_MHSA_FWD, M, D, 1), x.device) if ws is None else ws
    st = lib().aqt_mhsa_fwd(_ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(wqkv), _ptr(bqkv), _ptr(wo), _ptr(bo),
                            saved.B, saved.T, D, heads, left, right, saved.policy, _ptr(y), ctypes.byref(saved.c),
                            _ptr(ws), ws.numel(), _stream(), _ptr(dev_status))
    _check(st, "aqt_mhsa_fwd")
    return y


def aqt_residual_add(x, m, alpha: float, out=None):
    """aqt_residual_add: out = x + alpha * m."""
    _dev(x, torch.float32, "x")
    _dev(m, torch.float32, "m")
    out = torch.empty_like(x) if out is None else out
    _check(lib().aqt_residual_add(_ptr(x), _ptr(m), alpha, _ptr(out), x.numel(), _stream()), "aqt_residual_add")
    return out


class LayerSaved:
    """Device buffers of one encoder layer (aqt_conformer_layer_fwd) and their aqt_conformer_layer_saved view.
    policy: an aqt_layer_policy."""

    def __init__(self, B: int, T: int, D: int, H: int, policy, device="cuda", heads: int = 0):
        def pair(a, b):
            return ((a.bits_w, a.bits_x), (b.bits_w, b.bits_x))
        M = B * T
        self.policy = policy
        self.ffn1 = FfnSaved(M, D, H, pair(policy.ffn1_in, policy.ffn1_out), device)
        self.ffn2 = FfnSaved(M, D, H, pair(policy.ffn2_in, policy.ffn2_out), device)
        self.att = MhsaSaved(B, T, D, pair(policy.attn_qkv, policy.attn_out), device, heads=heads)
        self.out_row_stats = torch.empty((M, 2), dtype=torch.float32, device=device)
        self.conv = ConvSaved(B, T, D, pair(policy.conv_pw1, policy.conv_pw2), device)
        self.r = [torch.empty((M, D), dtype=torch.float32, device=device) for _ in range(4)]
        self.m = torch.empty((M, D), dtype=torch.float32, device=device)
        self.refresh()

    def refresh(self):
        self.c = aqt_conformer_layer_saved(self.ffn1.c, self.ffn2.c, self.att.c, self.conv.c,
                                           *[t.data_ptr() for t in self.r], self.m.data_ptr(),
                                           self.out_row_stats.data_ptr())
        return self

    def prepare(self, weights: dict):
        """Serving: quantize the eight weight matrices of the layer once (names as in LAYER_WEIGHT_NAMES) and
        mark every dense layer of the policy weights_ready; later layer calls skip the weight quantizers."""
        self.ffn1.prepare(weights["ffn1_w1"], weights["ffn1_w2"])
        self.ffn2.prepare(weights["ffn2_w1"], weights["ffn2_w2"])
        self.att.prepare(weights["att_wqkv"], weights["att_wo"])
        self.conv.prepare(weights["conv_w1"], weights["conv_w2"])
        pol = aqt_layer_policy.from_buffer_copy(self.policy)
        for name, _ in aqt_layer_policy._fields_:
            getattr(pol, name).weights_ready = 1
        self.policy = pol
        return self.refresh()


def aqt_conformer_layer_fwd(x, weights: dict, saved: LayerSaved, *, B: int, T: int, H: int, heads: int, kw: int,
                            pad_left: int, left: int = -1, right: int = -1, eps: float = 1e-6, y=None, ws=None,
                            dev_status=None):
    """aqt_conformer_layer_fwd: weights maps the field names of aqt_conformer_layer_weights to device tensors
    (missing or None: NULL).  x [B*T, D] -> y [B*T, D]."""
    _dev(x, torch.float32, "x")
    M, D = x.shape
    unknown = set(weights) - set(LAYER_WEIGHT_NAMES)
    if unknown:
        raise ValueError(f"unknown weight names {sorted(unknown)}")
    wc = aqt_conformer_layer_weights(*[None if weights.get(n) is None else weights[n].data_ptr()
                                       for n in LAYER_WEIGHT_NAMES])
    sh = aqt_conformer_layer_shape(B, T, D, H, heads, kw, pad_left, left, right, eps)
    y = torch.empty((M, D), dtype=torch.float32, device=x.device) if y is None else y
    ws = workspace(aqt_workspace_bytes(AQT_OP_CONFORMER_LAYER_FWD, M, D, H), x.device) if ws is None else ws
    st = lib().aqt_conformer_layer_fwd(_ptr(x), ctypes.byref(wc), ctypes.byref(sh), ctypes.byref(saved.policy),
                                       _ptr(y), ctypes.byref(saved.c), _ptr(ws), ws.numel(), _stream(),
                                       _ptr(dev_status))
    _check(st, "aqt_conformer_layer_fwd")
    return y


def aqt_layernorm_bwd(x, row_stats, dy, *, gamma=None, add=None, want_affine=True, ws=None):
    """aqt_layernorm_bwd: returns (dx [M,D], dgamma [D] or None, dbeta [D] or None)."""
    _dev(x, torch.float32, "x")
    _dev(dy, torch.float32, "dy")
    M, D = x.shape
    dx = torch.empty_like(x)
    dg = torch.empty(D, dtype=torch.float32, device=x.device) if want_affine else None
    db = torch.empty(D, dtype=torch.float32, device=x.device) if want_affine else None
    ws = workspace(aqt_workspace_bytes(AQT_OP_LAYERNORM_BWD, M, D, 1), x.device) if ws is None else ws
    st = lib().aqt_layernorm_bwd(_ptr(x), _ptr(row_stats), _ptr(gamma), _ptr(dy), _ptr(add), M, D, _ptr(dx), _ptr(dg),
                                 _ptr(db), _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_layernorm_bwd")
    return dx, dg, db


def aqt_mhsa_bwd(dy, saved: MhsaSaved, heads: int, *, left: int = -1, right: int = -1, ws=None):
    """aqt_mhsa_bwd: returns dict(dxn, dwqkv, dbqkv, dwo, dbo)."""
    _dev(dy, torch.float32, "dy")
    M, D = saved.M, saved.D
    f32 = dict(dtype=torch.float32, device=dy.device)
    o = dict(dxn=torch.empty((M, D), **f32), dwqkv=torch.empty((D, 3 * D), **f32), dbqkv=torch.empty(3 * D, **f32),
             dwo=torch.empty((D, D), **f32), dbo=torch.empty(D, **f32))
    ws = workspace(aqt_workspace_bytes(AQT_OP_MHSA_BWD, M, D, heads), dy.device) if ws is None else ws
    st = lib().aqt_mhsa_bwd(_ptr(dy), ctypes.byref(saved.c), saved.B, saved.T, D, heads, left, right, saved.policy,
                            _ptr(o["dxn"]), _ptr(o["dwqkv"]), _ptr(o["dbqkv"]), _ptr(o["dwo"]), _ptr(o["dbo"]),
                            _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_mhsa_bwd")
    return o


def aqt_conformer_layer_bwd(dy, x, weights: dict, saved: LayerSaved, *, B: int, T: int, H: int, heads: int, kw: int,
                            pad_left: int, left: int = -1, right: int = -1, eps: float = 1e-6, want=None, ws=None):
    """aqt_conformer_layer_bwd: returns (dx [B*T, D], dict of weight gradients).  `want`: names of the weights whose
    gradients are wanted (default: every weight present in `weights` except the fixed normalisation of the
    convolution module)."""
    _dev(dy, torch.float32, "dy")
    M, D = x.shape
    fixed = ("conv_norm_scale", "conv_norm_shift")
    want = [n for n in LAYER_WEIGHT_NAMES if weights.get(n) is not None and n not in fixed] if want is None else want
    grads = {n: torch.empty_like(weights[n]) for n in want}
    wc = aqt_conformer_layer_weights(*[None if weights.get(n) is None else weights[n].data_ptr()
                                       for n in LAYER_WEIGHT_NAMES])
    gc = aqt_conformer_layer_grads(*[grads[n].data_ptr() if n in grads else None for n in LAYER_WEIGHT_NAMES])
    sh = aqt_conformer_layer_shape(B, T, D, H, heads, kw, pad_left, left, right, eps)
    dx = torch.empty_like(x)
    ws = workspace(aqt_workspace_bytes(AQT_OP_CONFORMER_LAYER_BWD, M, D, H), x.device) if ws is None else ws
    st = lib().aqt_conformer_layer_bwd(_ptr(dy), _ptr(x), ctypes.byref(wc), ctypes.byref(sh),
                                       ctypes.byref(saved.policy), ctypes.byref(saved.c), _ptr(dx), ctypes.byref(gc),
                                       _ptr(ws), ws.numel(), _stream())
    _check(st, "aqt_conformer_layer_bwd")
    return dx, grads

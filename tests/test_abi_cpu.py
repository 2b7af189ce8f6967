"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import pytest

from paper_2203_15952_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2203_15952_amd import build
        build.build()
    return B.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "aqt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aqt_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert set(names) == set(B.SYMBOLS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings_and_version(L):
    seen = {L.aqt_status_string(i).decode() for i in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert L.aqt_status_string(99).decode() == "unknown status"
    assert L.aqt_version() >= 100


def test_packed_weight_bytes_formula(L):
    # half a byte per int4 parameter, fan-in padded to a whole byte; one byte for int8
    assert B.aqt_packed_weight_bytes(512, 2048, 4) == 2048 * 256
    assert B.aqt_packed_weight_bytes(5, 3, 4) == 3 * 3
    assert B.aqt_packed_weight_bytes(5, 3, 8) == 15
    assert B.aqt_packed_weight_bytes(5, 3, 2) == 9
    assert B.aqt_packed_weight_bytes(0, 3, 4) == 0 and B.aqt_packed_weight_bytes(5, 3, 9) == 0


def test_workspace_sizes_are_shape_functions(L):
    q = B.aqt_workspace_bytes(B.AQT_OP_QUANTIZE, 10, 10, 1)
    assert q >= 4096 * 4
    f = B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD, 12800, 512, 2048, 8, 4)
    assert f >= 12800 * 512 + 2048 * 256 + 2048 * 4 + q
    assert B.aqt_workspace_bytes(B.AQT_OP_DENSE_BWD, 65536, 512, 2048) > 0
    assert B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD_Q, 1, 512, 2048) >= 512 * 2048          # int8 fragments
    assert B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD_WONLY, 1, 512, 2048) >= 2 * 512 * 2048  # bf16 fragments
    assert B.aqt_workspace_bytes(B.AQT_OP_QUANTIZE_WEIGHTS, 1, 512, 2048) >= 16 * 2048 * 4   # slab maxima
    assert B.aqt_workspace_bytes(99, 1, 1, 1) == 0
    assert B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD, 0, 512, 2048, 8, 4) == 0


def test_argument_errors_are_synchronous_and_touch_no_gpu(L):
    one = ctypes.c_void_p(256)   # never dereferenced: every call below must fail its checks first
    none = None
    assert L.aqt_quantize(none, 4, 4, 4, 8, -1, one, one, none, one, 1 << 20, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_quantize(one, 0, 4, 4, 8, -1, one, one, none, one, 1 << 20, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_quantize(one, 4, 4, 3, 8, -1, one, one, none, one, 1 << 20, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_quantize(one, 4, 4, 4, 8, 7, one, one, none, one, 1 << 20, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_quantize(one, 4, 4, 4, 9, -1, one, one, none, one, 1 << 20, none, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_quantize(one, 4, 4, 4, 1, -1, one, one, none, one, 1 << 20, none, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_quantize(one, 4, 4, 4, 8, -1, one, one, none, none, 0, none, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_quantize(one, 4, 4, 4, 8, -1, one, one, none, one, 16, none, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_quantize_with_scale(one, 4, 4, 4, 8, -1, none, one, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_quantize_weights(one, 4, 4, 12, one, one, none, none, none, 0, none, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_quantize_weights(one, 4, 4, 4, one, one, none, none, none, 0, none, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_quantize_weights(one, 4, 4, 4, none, one, none, none, none, 0, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_unpack_weights(none, 4, 4, 4, one, none) == B.AQT_ERR_INVALID_ARG
    # GLU needs an even N; epilogue must be known; K must keep 16*K*qmax_x*qmax_w inside int32
    assert L.aqt_dense_fwd_q(one, one, one, one, 4, 4, 5, 8, 4, none, B.AQT_EPI_GLU, one, none, none, 0, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_dense_fwd_q(one, one, one, one, 4, 4, 4, 8, 4, none, 3, one, none, none, 0, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_dense_fwd_q(one, one, one, one, 4, 200000, 4, 8, 4, none, 0, one, none, none, 0, none) == B.AQT_ERR_UNSUPPORTED
    # int8 weights are not expanded, so the factor 16 does not apply to them: K = 9000 fits (the call
    # then fails on its missing workspace), K = 140000 does not
    assert L.aqt_dense_fwd_q(one, one, one, one, 4, 9000, 4, 8, 8, none, 0, one, none, none, 0, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_dense_fwd_q(one, one, one, one, 4, 140000, 4, 8, 8, none, 0, one, none, none, 0, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_dense_fwd_q(one, one, one, one, 4, 9000, 4, 8, 4, none, 0, one, none, none, 0, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_dense_fwd_q(one, one, one, one, 4, 160000, 4, 8, 4, none, 0, one, none, none, 0, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_dense_fwd_q(one, one, one, one, 4, 4, 4, 8, 4, none, 0, one, none, none, 0, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_dense_fwd_q(one, one, one, one, 4, 4, 4, 8, 4, none, 0, one, none, one, 8, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_dense_fwd_q_absmax(one, one, one, one, 4, 4, 4, 8, 4, none, 0, one, none, one, 1 << 20, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_dense_fwd_q_absmax(one, one, one, one, 4, 4, 5, 8, 4, none, B.AQT_EPI_GLU, one, one, one, 1 << 20, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_dense_fwd_q_absmax(one, one, one, one, 4, 4, 4, 8, 4, none, 0, one, one, none, 0, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_quantize_with_absmax(one, 4, 4, 4, 8, none, one, one, none, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_quantize_with_absmax(one, 4, 4, 3, 8, one, one, one, none, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_quantize_with_absmax(one, 4, 4, 4, 9, one, one, one, none, none, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_dense_fwd_wonly(one, one, none, 4, 4, 4, 4, none, 0, one, one, 1 << 20, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_dense_fwd_wonly(one, one, one, 4, 4, 5, 4, none, B.AQT_EPI_GLU, one, one, 1 << 20, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_dense_fwd_wonly(one, one, one, 4, 4, 4, 4, none, 0, one, none, 0, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_dense_fwd(one, one, 4, 4, 4, 8, 4, none, 0, one, None, none, 0, none, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_dense_fwd(one, none, 4, 4, 4, 8, 4, none, 0, one, None, one, 1 << 30, none, none) == B.AQT_ERR_INVALID_ARG
    sv = B.aqt_saved(None, None, None, None, None, None, None, None)
    assert L.aqt_dense_bwd(one, ctypes.byref(sv), 4, 4, 4, 8, 4, 0, one, one, none, one, 1 << 30, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_dense_bwd(one, None, 4, 4, 4, 8, 4, 0, one, one, none, one, 1 << 30, none) == B.AQT_ERR_INVALID_ARG
    sv = B.aqt_saved(256, 256, None, 256, 256, 256, None, None)
    assert L.aqt_dense_bwd(one, ctypes.byref(sv), 4, 4, 4, 8, 4, 0, one, one, none, none, 0, none) == B.AQT_ERR_WORKSPACE
    # an activation needs the saved derivative factors, and a workspace that also holds dv
    assert L.aqt_dense_bwd(one, ctypes.byref(sv), 4, 4, 4, 8, 4, B.AQT_EPI_SWISH, one, one, none, one, 1 << 30, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_dense_bwd(one, ctypes.byref(sv), 4, 4, 5, 8, 4, B.AQT_EPI_GLU, one, one, none, one, 1 << 30, none) == B.AQT_ERR_UNSUPPORTED
    assert B.aqt_workspace_bytes(B.AQT_OP_DENSE_BWD_EPI, 100, 64, 32) >= B.aqt_workspace_bytes(B.AQT_OP_DENSE_BWD, 100, 64, 32) + 100 * 32 * 4
    # layer normalisation, float32-emulated product, feed-forward module: argument checks
    assert L.aqt_layernorm_quantize(none, 4, 4, none, none, 1e-6, 8, one, one, none, none, one, 1 << 20, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_layernorm_quantize(one, 4, 4, none, none, 1e-6, 8, one, none, none, none, one, 1 << 20, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_layernorm_quantize(one, 4, 4, none, none, 1e-6, 9, one, one, none, none, one, 1 << 20, none, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_layernorm_quantize(one, 4, 4, none, none, 1e-6, 8, one, one, none, none, none, 0, none, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_fake_matmul_f32(one, none, 4, 4, 4, one, none) == B.AQT_ERR_INVALID_ARG
    fs = B.aqt_ffn_saved()
    pol = (B.aqt_dense_policy * 2)(B.aqt_dense_policy(4, 8), B.aqt_dense_policy(4, 8))
    assert L.aqt_ffn_fwd(one, none, none, 1e-6, one, none, one, none, 4, 4, 4, pol, one, ctypes.byref(fs), one, 1 << 30, none, none) == B.AQT_ERR_INVALID_ARG
    bad = (B.aqt_dense_policy * 2)(B.aqt_dense_policy(9, 8), B.aqt_dense_policy(4, 8))
    assert L.aqt_ffn_fwd(one, none, none, 1e-6, one, none, one, none, 4, 4, 4, bad, one, ctypes.byref(fs), one, 1 << 30, none, none) == B.AQT_ERR_UNSUPPORTED
    wo = (B.aqt_dense_policy * 2)(B.aqt_dense_policy(4, 0), B.aqt_dense_policy(4, 8))
    assert L.aqt_ffn_bwd(one, ctypes.byref(fs), 4, 4, 4, wo, one, one, none, one, none, one, 1 << 30, none) == B.AQT_ERR_UNSUPPORTED
    assert B.aqt_workspace_bytes(B.AQT_OP_FFN_FWD, 128, 512, 2048) > 0 and B.aqt_workspace_bytes(B.AQT_OP_FFN_BWD, 128, 512, 2048) > 128 * 2048 * 4


def _filled(struct_type, skip=()):
    """A struct whose pointer fields all hold the same never-dereferenced address (nested structs too)."""
    st = struct_type()
    for name, typ in struct_type._fields_:
        if name in skip:
            continue
        if typ is ctypes.c_void_p:
            setattr(st, name, 256)
        elif issubclass(typ, ctypes.Structure):
            setattr(st, name, _filled(typ, skip))
    return st


def test_module_and_layer_argument_errors_are_synchronous(L):
    one, none, big = ctypes.c_void_p(256), None, 1 << 40
    i8 = (B.aqt_dense_policy * 2)(B.aqt_dense_policy(8, 8, 0), B.aqt_dense_policy(8, 8, 0))
    # depthwise convolution: pad_left must lie inside the kernel, the tap gradient needs a workspace
    assert L.aqt_depthwise_conv_fwd(one, 2, 8, 4, one, none, 3, 3, none, none, 0, one, none, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_depthwise_conv_fwd(one, 2, 8, 4, one, none, 0, 0, none, none, 0, one, none, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_depthwise_conv_fwd(one, 2, 8, 4, none, none, 3, 1, none, none, 0, one, none, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_depthwise_conv_bwd(one, none, none, one, 2, 8, 4, 3, 1, one, one, none, one, big, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_depthwise_conv_bwd(one, none, one, none, 2, 8, 4, 3, 1, one, one, none, one, big, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_depthwise_conv_bwd(one, none, one, one, 2, 8, 4, 3, 1, one, one, none, none, 0, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_depthwise_conv_bwd(one, none, one, one, 2, 8, 4, 3, 1, one, one, none, one, 16, none) == B.AQT_ERR_WORKSPACE
    assert B.aqt_workspace_bytes(B.AQT_OP_DEPTHWISE_CONV_BWD, 16, 4, 3) > 0
    # attention: the model width must split into heads of at most 64 columns
    assert L.aqt_attention_fwd(one, 2, 8, 30, 4, -1, -1, one, none, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_attention_fwd(one, 2, 8, 32, 0, -1, -1, one, none, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_attention_fwd(one, 2, 8, 256, 2, -1, -1, one, none, none, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_attention_bwd(one, one, one, none, 2, 8, 32, 4, -1, -1, one, one, big, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_attention_bwd(one, one, one, one, 2, 8, 256, 2, -1, -1, one, one, big, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_attention_bwd(one, one, one, one, 2, 8, 32, 4, -1, -1, one, none, 0, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_attention_bwd(one, one, one, one, 2, 8, 32, 4, -1, -1, one, one, 8, none) == B.AQT_ERR_WORKSPACE
    # residual sum, layer normalisation backward
    assert L.aqt_residual_add(one, none, 0.5, one, 4, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_residual_add(one, one, 0.5, one, 0, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_layernorm_bwd(one, none, none, one, none, 4, 4, one, none, none, none, 0, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_layernorm_bwd(one, one, none, one, none, 4, 4, one, one, none, none, 0, none) == B.AQT_ERR_WORKSPACE
    assert L.aqt_layernorm_bwd(one, one, none, one, none, 4, 4, one, none, one, one, 8, none) == B.AQT_ERR_WORKSPACE
    # convolution module
    cs = _filled(B.aqt_conv_saved)
    assert L.aqt_conv_module_fwd(one, none, none, 1e-6, one, none, one, none, none, none, one, none, 2, 8, 4, 3, 3, i8,
                                 one, ctypes.byref(cs), one, big, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_conv_module_fwd(one, none, none, 1e-6, one, none, one, none, none, none, none, none, 2, 8, 4, 3, 1, i8,
                                 one, ctypes.byref(cs), one, big, none, none) == B.AQT_ERR_INVALID_ARG   # no w2
    wo = (B.aqt_dense_policy * 2)(B.aqt_dense_policy(8, 0, 0), B.aqt_dense_policy(8, 8, 0))
    assert L.aqt_conv_module_fwd(one, none, none, 1e-6, one, none, one, none, none, none, one, none, 2, 8, 4, 3, 1, wo,
                                 one, ctypes.byref(cs), one, big, none, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_conv_module_fwd(one, none, none, 1e-6, one, none, one, none, none, none, one, none, 2, 8, 4, 3, 1, i8,
                                 one, ctypes.byref(cs), one, 64, none, none) == B.AQT_ERR_WORKSPACE
    no_g = _filled(B.aqt_conv_saved, skip=("g",))
    assert L.aqt_conv_module_fwd(one, none, none, 1e-6, one, none, one, none, none, none, one, none, 2, 8, 4, 3, 1, i8,
                                 one, ctypes.byref(no_g), one, big, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_conv_module_bwd(one, ctypes.byref(no_g), one, 2, 8, 4, 3, 1, i8, one, one, none, one, none, one, none,
                                 one, big, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_conv_module_bwd(one, ctypes.byref(cs), one, 2, 8, 4, 3, 1, i8, one, one, none, one, none, one, none,
                                 one, 64, none) == B.AQT_ERR_WORKSPACE
    # self-attention module
    ms = _filled(B.aqt_mhsa_saved)
    assert L.aqt_mhsa_fwd(one, none, none, 1e-6, one, none, one, none, 2, 8, 30, 4, -1, -1, i8, one, ctypes.byref(ms),
                          one, big, none, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_mhsa_fwd(one, none, none, 1e-6, one, none, one, none, 2, 8, 256, 2, -1, -1, i8, one, ctypes.byref(ms),
                          one, big, none, none) == B.AQT_ERR_UNSUPPORTED
    assert L.aqt_mhsa_fwd(one, none, none, 1e-6, none, none, one, none, 2, 8, 32, 4, -1, -1, i8, one, ctypes.byref(ms),
                          one, big, none, none) == B.AQT_ERR_INVALID_ARG   # training form without the float weights
    assert L.aqt_mhsa_fwd(one, none, none, 1e-6, one, none, one, none, 2, 8, 32, 4, -1, -1, i8, one, ctypes.byref(ms),
                          one, 64, none, none) == B.AQT_ERR_WORKSPACE
    no_lse = _filled(B.aqt_mhsa_saved, skip=("lse",))
    assert L.aqt_mhsa_bwd(one, ctypes.byref(no_lse), 2, 8, 32, 4, -1, -1, i8, one, one, none, one, none, one, big,
                          none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_mhsa_bwd(one, ctypes.byref(ms), 2, 8, 32, 4, -1, -1, i8, one, one, none, one, none, one, 64,
                          none) == B.AQT_ERR_WORKSPACE
    # encoder layer: everything is checked before the first launch, whichever module the mistake sits in
    w = _filled(B.aqt_conformer_layer_weights)
    sv = _filled(B.aqt_conformer_layer_saved)
    gr = B.aqt_conformer_layer_grads()
    pol = B.aqt_layer_policy()
    assert L.aqt_policy_preset(B.AQT_POLICY_ALL, 1, 0, 8, 8, ctypes.byref(pol)) == B.AQT_OK

    def shape(**kw):
        d = dict(B=2, T=8, D=32, H=64, heads=4, kw=3, pad_left=1, left_context=-1, right_context=-1, ln_eps=1e-6)
        d.update(kw)
        return B.aqt_conformer_layer_shape(**d)

    def fwd(shp, weights=w, policy=pol, saved=sv, ws_bytes=big):
        return L.aqt_conformer_layer_fwd(one, ctypes.byref(weights), ctypes.byref(shp), ctypes.byref(policy), one,
                                         ctypes.byref(saved), one, ws_bytes, none, none)

    def bwd(shp, weights=w, policy=pol, saved=sv, grads=gr, ws_bytes=big):
        return L.aqt_conformer_layer_bwd(one, one, ctypes.byref(weights), ctypes.byref(shp), ctypes.byref(policy),
                                         ctypes.byref(saved), one, ctypes.byref(grads), one, ws_bytes, none)

    assert fwd(shape(T=0)) == B.AQT_ERR_INVALID_ARG
    assert fwd(shape(heads=5)) == B.AQT_ERR_INVALID_ARG            # the attention module's check
    assert fwd(shape(D=256, heads=2)) == B.AQT_ERR_UNSUPPORTED
    assert fwd(shape(pad_left=3)) == B.AQT_ERR_INVALID_ARG         # the convolution module's check
    assert fwd(shape(), ws_bytes=64) == B.AQT_ERR_WORKSPACE
    no_w = _filled(B.aqt_conformer_layer_weights, skip=("ffn2_w2",))
    assert fwd(shape(), weights=no_w) == B.AQT_ERR_INVALID_ARG     # the last module's weights, in training form
    no_r = _filled(B.aqt_conformer_layer_saved, skip=("r3",))
    assert fwd(shape(), saved=no_r) == B.AQT_ERR_INVALID_ARG
    bad = B.aqt_layer_policy()
    L.aqt_policy_preset(B.AQT_POLICY_ALL, 1, 0, 8, 8, ctypes.byref(bad))
    bad.conv_pw2 = B.aqt_dense_policy(8, 0, 0)                     # weight-only is a feed-forward-module form
    assert fwd(shape(), policy=bad) == B.AQT_ERR_UNSUPPORTED
    assert bwd(shape(T=0)) == B.AQT_ERR_INVALID_ARG
    assert bwd(shape(D=256, heads=2)) == B.AQT_ERR_UNSUPPORTED
    assert bwd(shape(), ws_bytes=64) == B.AQT_ERR_WORKSPACE
    frozen = B.aqt_conformer_layer_grads()
    frozen.conv_norm_scale = 256                                    # the fixed statistics take no gradient
    assert bwd(shape(), grads=frozen) == B.AQT_ERR_UNSUPPORTED
    assert bwd(shape(), saved=no_r) == B.AQT_ERR_INVALID_ARG
    no_lse = _filled(B.aqt_conformer_layer_saved, skip=("lse",))     # found by the attention module's check ...
    assert bwd(shape(), saved=no_lse) == B.AQT_ERR_INVALID_ARG
    no_dact = _filled(B.aqt_conformer_layer_saved, skip=("dact",))   # ... and the feed-forward module's, up front
    assert bwd(shape(), saved=no_dact) == B.AQT_ERR_INVALID_ARG
    need = B.aqt_workspace_bytes(B.AQT_OP_CONFORMER_LAYER_FWD, 16, 32, 64)
    assert need > 0 and fwd(shape(), ws_bytes=need - 1) == B.AQT_ERR_WORKSPACE


def test_precision_policies_follow_table_2_patterns(L):
    # Table 2: int4 on the selected layers, int8 on the rest; E6 spares the first and last layer, E7 the
    # self-attention projections, E8 - E13 take the first k layers
    n = 6
    names = ("ffn1_in", "ffn1_out", "attn_qkv", "attn_out", "conv_pw1", "conv_pw2", "ffn2_in", "ffn2_out")

    def bits_w(p):
        return [[getattr(l, nm).bits_w for nm in names] for l in p]
    allp = B.aqt_policy_preset(B.AQT_POLICY_ALL, n, 0, 4, 8)
    assert bits_w(allp) == [[4] * 8] * n and all(getattr(l, nm).bits_x == 8 for l in allp for nm in names)
    e6 = B.aqt_policy_preset(B.AQT_POLICY_EXCEPT_FIRST_LAST, n, 0, 4, 8)
    assert bits_w(e6) == [[8] * 8] + [[4] * 8] * (n - 2) + [[8] * 8]
    e7 = B.aqt_policy_preset(B.AQT_POLICY_EXCEPT_ATTENTION, n, 0, 4, 8)
    assert bits_w(e7) == [[4, 4, 8, 8, 4, 4, 4, 4]] * n
    e10 = B.aqt_policy_preset(B.AQT_POLICY_FIRST_K, n, 3, 4, 0)
    assert bits_w(e10) == [[4] * 8] * 3 + [[8] * 8] * 3 and e10[0].ffn1_in.bits_x == 0
    with pytest.raises(B.AqtError):
        B.aqt_policy_preset(B.AQT_POLICY_FIRST_K, n, n + 1, 4, 8)
    with pytest.raises(B.AqtError):
        B.aqt_policy_preset(7, n, 0, 4, 8)
    # model-size side of the trade-off: half a byte per int4 weight, one byte per int8 weight, 4 bytes per scale
    d, ff = 512, 2048
    per_layer_weights = 4 * d * ff + 3 * d * d + d * d + 2 * d * d + d * d
    per_layer_scales = 4 * (2 * ff + 2 * d + 3 * d + d + 2 * d + d)
    i8 = B.aqt_policy_weight_bytes(B.aqt_policy_preset(B.AQT_POLICY_ALL, n, 0, 8, 8), n, d, ff)
    i4 = B.aqt_policy_weight_bytes(allp, n, d, ff)
    assert i8 == n * (per_layer_weights + per_layer_scales) and i4 == n * (per_layer_weights // 2 + per_layer_scales)
    sizes = [B.aqt_policy_weight_bytes(B.aqt_policy_preset(B.AQT_POLICY_FIRST_K, n, k, 4, 8), n, d, ff) for k in range(n + 1)]
    assert sizes[0] == i8 and sizes[-1] == i4 and all(a > b for a, b in zip(sizes, sizes[1:]))   # E8 .. E13 shrink monotonically
    assert i4 < B.aqt_policy_weight_bytes(e7, n, d, ff) < i8

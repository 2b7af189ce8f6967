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
    sv = B.aqt_saved(None, None, None, None, None, None, None)
    assert L.aqt_dense_bwd(one, ctypes.byref(sv), 4, 4, 4, 8, 4, one, one, none, one, 1 << 30, none) == B.AQT_ERR_INVALID_ARG
    assert L.aqt_dense_bwd(one, None, 4, 4, 4, 8, 4, one, one, none, one, 1 << 30, none) == B.AQT_ERR_INVALID_ARG
    sv = B.aqt_saved(256, 256, None, 256, 256, 256, None)
    assert L.aqt_dense_bwd(one, ctypes.byref(sv), 4, 4, 4, 8, 4, one, one, none, none, 0, none) == B.AQT_ERR_WORKSPACE

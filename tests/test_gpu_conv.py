"""Parity of the convolution module's pieces (depthwise convolution along time with the
normalisation, Swish and abs-max fused behind it, its gradients, and the module as one call)
against the CPU oracle.  The chain is checked stage by stage, each quantized stage with the
oracle fed the very float32 buffer the GPU stage consumed."""
import numpy as np
import pytest
import torch

import oracle
from paper_2203_15952_amd import binding as B
from parity_util import REL_Y, TINY, check_forward, check_grad

pytestmark = pytest.mark.gpu
F = np.float32
U = 2.0 ** -24   # float32 unit round-off


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def say(*a):
    print(*a, flush=True)


def conv_inputs(seed, B_, T, C, kw):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B_, T, C)).astype(F)
    w = (rng.standard_normal((kw, C)) / np.sqrt(kw)).astype(F)
    bias = (0.1 * rng.standard_normal(C)).astype(F)
    a = (1 + 0.1 * rng.standard_normal(C)).astype(F)
    b = (0.1 * rng.standard_normal(C)).astype(F)
    dout = (0.1 * rng.standard_normal((B_, T, C))).astype(F)
    return x, w, bias, a, b, dout


def check_depthwise_forward(out, dfac, x, w, bias, a, b, pl, swish):
    """The convolution is a float32 multiply-add chain of kw (+1) terms: within (kw + 1) u of the sum of
    the magnitudes of its terms; scale and shift add one rounding each; Swish and its slope carry that
    tolerance through their derivatives (|swish'| <= 1.1, |swish''| <= 1/2) on top of their own 1e-6."""
    kw = w.shape[0]
    v, v_abs = oracle.depthwise_conv(x, w, bias, pad_left=pl, want_abs=True)
    C = x.shape[-1]
    a64 = np.ones(C) if a is None else a.astype(np.float64)
    b64 = np.zeros(C) if b is None else b.astype(np.float64)
    tol_n = np.abs(a64) * (kw + 1) * U * v_abs + 2 * U * (np.abs(v * a64) + np.abs(b64)) + TINY
    n = v * a64 + b64
    if swish:
        ref, dref = oracle.affine_swish(v.reshape(-1, C), a, b)
        ref, dref = ref.reshape(v.shape), dref.reshape(v.shape)
        tol_o = REL_Y * np.abs(ref) + 1.1 * tol_n
        tol_d = np.abs(a64) * (4e-6 + 0.5 * tol_n)
    else:
        ref, dref = n, np.broadcast_to(a64, v.shape)
        tol_o, tol_d = tol_n, 0.0
    bad = np.abs(out.astype(np.float64) - ref) > tol_o
    assert not bad.any(), f"{bad.sum()} of {bad.size} outputs outside tolerance"
    if dfac is not None:
        bad = np.abs(dfac.astype(np.float64) - dref) > tol_d
        assert not bad.any(), f"{bad.sum()} of {bad.size} slopes outside tolerance"


DW_CASES = [
    # B, T, C, kw, pad_left, affine, swish       (which kernel)
    (32, 400, 512, 32, 15, True, True),          # the convolution module's shape (Sec. 3.2: kernel 32)
    (2, 37, 70, 15, 14, True, True),             # causal, kernel 15 (Sec. 3.3); ragged channels and frames
    (1, 5, 3, 32, 15, False, False),             # utterance shorter than the kernel
    (3, 50, 64, 40, 20, True, True),             # kernel beyond 32: the general kernel
    (2, 100, 130, 1, 0, True, False),            # a single tap
    (1, 1, 1, 1, 0, False, True),
    (4, 129, 96, 16, 8, False, True),            # exactly 16 taps; one frame beyond four runs
    (5, 128, 64, 17, 0, True, True),             # anti-causal: looks only ahead
]


@pytest.mark.parametrize("B_,T,C,kw,pl,affine,swish", DW_CASES)
def test_depthwise_conv_forward(B_, T, C, kw, pl, affine, swish):
    say("depthwise fwd", B_, T, C, kw, pl, affine, swish)
    x, w, bias, a, b, _ = conv_inputs(300 + T + kw, B_, T, C, kw)
    if not affine:
        a = b = None
    out, dfac, m = B.aqt_depthwise_conv_fwd(dev(x), dev(w), bias=dev(bias), pad_left=pl, norm_scale=dev(a),
                                            norm_shift=dev(b), swish=swish, want_dfac=True, want_absmax=True)
    out_h, dfac_h = host(out), host(dfac)
    check_depthwise_forward(out_h, dfac_h, x, w, bias, a, b, pl, swish)
    # the word is the maximum of the very values written, and the one-pass quantizer on it gives the
    # oracle's codes of that buffer
    assert host(m)[0] == np.abs(out_h).max()
    q, s, _ = B.aqt_quantize_with_absmax(out.view(B_ * T, C), 8, m)
    q_ref, s_ref = oracle.quantize(out_h.reshape(B_ * T, C), 8, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(s), s_ref)
    np.testing.assert_array_equal(host(q), q_ref)
    # without the optional outputs and the bias
    out2, _, _ = B.aqt_depthwise_conv_fwd(dev(x), dev(w), pad_left=pl)
    check_depthwise_forward(host(out2), None, x, w, None, None, None, pl, False)


@pytest.mark.parametrize("B_,T,C,kw,pl,affine,swish", DW_CASES)
def test_depthwise_conv_backward(B_, T, C, kw, pl, affine, swish):
    say("depthwise bwd", B_, T, C, kw, pl)
    x, w, _, _, _, dout = conv_inputs(400 + T + kw, B_, T, C, kw)
    rng = np.random.default_rng(1)
    dfac = (0.5 + rng.random((B_, T, C))).astype(F) if affine else None
    dx, dw, db = B.aqt_depthwise_conv_bwd(dev(dout), dev(x), dev(w), dfac=dev(dfac), pad_left=pl)
    dv = dout.astype(np.float64) * (1.0 if dfac is None else dfac.astype(np.float64))
    g = oracle.depthwise_conv_bwd(dv, x, w, pad_left=pl)
    check_grad(host(dx), g["dx"], g["dx_abs"], "dx")
    check_grad(host(dw), g["dw"], g["dw_abs"], "dw")
    check_grad(host(db), g["dbias"], np.abs(dv).sum((0, 1)), "dbias")
    # fixed summation order: the same bits on a second run; each output alone gives the same values
    dx2, dw2, db2 = B.aqt_depthwise_conv_bwd(dev(dout), dev(x), dev(w), dfac=dev(dfac), pad_left=pl)
    for p, q in ((dx, dx2), (dw, dw2), (db, db2)):
        np.testing.assert_array_equal(host(p), host(q))
    dx3, _, _ = B.aqt_depthwise_conv_bwd(dev(dout), None, dev(w), dfac=dev(dfac), pad_left=pl, want_dw=False,
                                         want_dbias=False)
    np.testing.assert_array_equal(host(dx3), host(dx))
    _, _, db3 = B.aqt_depthwise_conv_bwd(dev(dout), None, dev(w), dfac=dev(dfac), pad_left=pl, want_dx=False,
                                         want_dw=False)
    np.testing.assert_array_equal(host(db3), host(db))


def test_depthwise_conv_argument_errors():
    x = torch.zeros((2, 8, 4), device="cuda")
    w = torch.zeros((3, 4), device="cuda")
    for pl in (-1, 3):
        with pytest.raises(B.AqtError) as e:
            B.aqt_depthwise_conv_fwd(x, w, pad_left=pl)
        assert e.value.status == B.AQT_ERR_INVALID_ARG
    with pytest.raises(B.AqtError) as e:
        B.aqt_depthwise_conv_bwd(x, x, w, pad_left=1, ws=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == B.AQT_ERR_WORKSPACE


# ----------------------------------------------------------------------------
# the convolution module as one call
# ----------------------------------------------------------------------------
def module_inputs(seed, B_, T, D, kw):
    rng = np.random.default_rng(seed)
    M = B_ * T
    d = dict(
        x=(rng.standard_normal((M, D)) * 2 + 0.5).astype(F),
        gamma=(1 + 0.1 * rng.standard_normal(D)).astype(F), beta=(0.1 * rng.standard_normal(D)).astype(F),
        w1=(rng.standard_normal((D, 2 * D)) / np.sqrt(D)).astype(F), b1=(0.1 * rng.standard_normal(2 * D)).astype(F),
        w_dw=(rng.standard_normal((kw, D)) / np.sqrt(kw)).astype(F), b_dw=(0.1 * rng.standard_normal(D)).astype(F),
        na=(1 + 0.1 * rng.standard_normal(D)).astype(F), nb=(0.1 * rng.standard_normal(D)).astype(F),
        w2=(rng.standard_normal((D, D)) / np.sqrt(D)).astype(F), b2=(0.1 * rng.standard_normal(D)).astype(F),
        dy=(0.1 * rng.standard_normal((M, D))).astype(F))
    return d


def rows_of(M):
    mid = (M // 256) * 128
    return np.unique(np.r_[0:min(128, M), mid:min(mid + 128, M), max(0, M - 256):M])


@pytest.mark.parametrize("B_,T,D,kw,pl,policy", [
    (32, 400, 512, 32, 15, ((4, 8), (8, 8))),   # the convolution-module configuration: int4 then int8 weights
    (3, 300, 256, 15, 14, ((8, 8), (4, 8))),    # causal kernel 15; tuned kernels, ragged M
    (2, 19, 24, 32, 15, ((4, 8), (8, 4))),      # shapes the general kernels take
])
def test_conv_module_chain_stage_by_stage(B_, T, D, kw, pl, policy):
    say("conv module", B_, T, D, kw, pl, policy)
    M = B_ * T
    i = module_inputs(500 + M, B_, T, D, kw)
    (bw1, bx1), (bw2, bx2) = policy
    sv = B.ConvSaved(B_, T, D, policy)
    status = B.new_status()
    d = {k: dev(v) for k, v in i.items()}
    y = B.aqt_conv_module_fwd(d["x"], d["w1"], d["b1"], d["w_dw"], d["b_dw"], d["w2"], d["b2"], sv, pad_left=pl,
                              gamma=d["gamma"], beta=d["beta"], eps=1e-6, norm_scale=d["na"], norm_shift=d["nb"],
                              dev_status=status)
    assert host(status)[0] == 0
    rows = rows_of(M)
    # stage 1: normalisation + quantizer; the normalised values themselves from the same kernel asked to write them
    q_a, s_a, xn_t, _ = B.aqt_layernorm_quantize(d["x"], bx1, gamma=d["gamma"], beta=d["beta"], eps=1e-6, want_y=True)
    xn = host(xn_t)
    ref = oracle.layernorm(i["x"], i["gamma"], i["beta"], 1e-6)
    assert (np.abs(xn - ref) <= 1e-5 * (1 + np.abs(ref))).all()
    xq1, sx1 = oracle.quantize(xn, bx1, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(sv.pw1.s_x), sx1)
    np.testing.assert_array_equal(host(sv.pw1.xq), xq1)
    # stage 2: first pointwise convolution with the GLU
    wq1, sw1 = oracle.quantize(i["w1"], bw1, 0)
    np.testing.assert_array_equal(host(sv.pw1.wq_kn), wq1)
    g = host(sv.g)
    o1 = oracle.dense_fwd_q(xq1[rows], sx1[0], wq1, sw1, i["b1"], oracle.EPI_GLU)
    check_forward(g[rows], o1, sx1[0], sw1, i["b1"], 2)
    # stage 3: depthwise convolution, normalisation, Swish on the GPU's own g
    s = host(sv.s)
    check_depthwise_forward(s.reshape(B_, T, D), host(sv.dfac).reshape(B_, T, D), g.reshape(B_, T, D), i["w_dw"],
                            i["b_dw"], i["na"], i["nb"], pl, True)
    # stage 4: second quantizer on the GPU's own s (one pass, the maximum came from the depthwise kernel)
    xq2, sx2 = oracle.quantize(s, bx2, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(sv.pw2.s_x), sx2)
    np.testing.assert_array_equal(host(sv.pw2.xq), xq2)
    # stage 5: second pointwise convolution
    wq2, sw2 = oracle.quantize(i["w2"], bw2, 0)
    np.testing.assert_array_equal(host(sv.pw2.wq_kn), wq2)
    y_h = host(y)
    o2 = oracle.dense_fwd_q(xq2[rows], sx2[0], wq2, sw2, i["b2"], 0)
    check_forward(y_h[rows], o2, sx2[0], sw2, i["b2"], 0)
    # the one call equals the same entry points called one by one, bit for bit
    wp1, s_w1, _, _ = B.aqt_quantize_weights(d["w1"], bw1)
    g_b, _ = B.aqt_dense_fwd_q(q_a, s_a, wp1, s_w1, 2 * D, bx1, bw1, bias=d["b1"], epilogue=B.AQT_EPI_GLU)
    s_b, _, m_b = B.aqt_depthwise_conv_fwd(g_b.view(B_, T, D), d["w_dw"], bias=d["b_dw"], pad_left=pl,
                                           norm_scale=d["na"], norm_shift=d["nb"], swish=True, want_absmax=True)
    q_b, sx_b, _ = B.aqt_quantize_with_absmax(s_b.view(M, D), bx2, m_b)
    wp2, s_w2, _, _ = B.aqt_quantize_weights(d["w2"], bw2)
    y_b, _ = B.aqt_dense_fwd_q(q_b, sx_b, wp2, s_w2, D, bx2, bw2, bias=d["b2"])
    np.testing.assert_array_equal(host(y_b), y_h)
    if M > 2000:
        return
    # backward, stage by stage, the oracle fed the float32 gradient the GPU passed down at each stage
    o = B.aqt_conv_module_bwd(d["dy"], sv, d["w_dw"], pad_left=pl)
    g2 = oracle.dense_bwd(i["dy"], xq2, sx2[0], wq2, sw2)
    check_grad(host(o["dw2"]), g2["dw"], g2["dw_abs"], "dw2")
    check_grad(host(o["db2"]), g2["dbias"], np.abs(i["dy"].astype(np.float64)).sum(0), "db2")
    sv2 = B.Saved(M, D, D, bw2)           # the second layer alone, to look at the gradient handed down
    sv2.xq.copy_(sv.pw2.xq); sv2.s_x.copy_(sv.pw2.s_x); sv2.wq_kn.copy_(sv.pw2.wq_kn); sv2.s_w.copy_(sv.pw2.s_w)
    ds, _, _ = B.aqt_dense_bwd(d["dy"], sv2, bx2, bw2, want_dw=False)
    ds_h = host(ds)
    check_grad(ds_h, g2["dx"], g2["dx_abs"], "ds")
    dfac_h = host(sv.dfac)
    dv = (ds_h.astype(np.float64) * dfac_h.astype(np.float64)).reshape(B_, T, D)
    gd = oracle.depthwise_conv_bwd(dv, g.reshape(B_, T, D), i["w_dw"], pad_left=pl)
    check_grad(host(o["dw_dw"]), gd["dw"], gd["dw_abs"], "dw_dw")
    check_grad(host(o["db_dw"]), gd["dbias"], np.abs(dv).sum((0, 1)), "db_dw")
    dg, _, _ = B.aqt_depthwise_conv_bwd(ds.view(B_, T, D), None, d["w_dw"], dfac=sv.dfac.view(B_, T, D), pad_left=pl,
                                        want_dw=False, want_dbias=False)
    dg_h = host(dg).reshape(M, D)
    check_grad(dg_h, gd["dx"].reshape(M, D), gd["dx_abs"].reshape(M, D), "dg")
    pre1 = oracle.dense_fwd_q(xq1, sx1[0], wq1, sw1, i["b1"], oracle.EPI_GLU)["pre"]
    g1 = oracle.dense_bwd_epi(dg_h, pre1, oracle.EPI_GLU, xq1, sx1[0], wq1, sw1)
    check_grad(host(o["dxn"]), g1["dx"], g1["dx_abs"], "dxn")
    check_grad(host(o["dw1"]), g1["dw"], g1["dw_abs"], "dw1")
    check_grad(host(o["db1"]), g1["dbias"], np.abs(g1["dv"]).sum(0), "db1")


def test_conv_module_rejects_float_activations():
    sv = B.ConvSaved(1, 64, 128, ((4, 0), (8, 8)))
    z = torch.zeros((64, 128), device="cuda")
    w1, wd, w2 = torch.zeros((128, 256), device="cuda"), torch.zeros((15, 128), device="cuda"), torch.zeros((128, 128), device="cuda")
    with pytest.raises(B.AqtError) as e:
        B.aqt_conv_module_fwd(z, w1, None, wd, None, w2, None, sv, pad_left=14)
    assert e.value.status == B.AQT_ERR_UNSUPPORTED

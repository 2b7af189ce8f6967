"""Parity of the self-attention module's pieces (the float attention core and the module as one
call) against the CPU oracle; the chain is checked stage by stage, each quantized stage with the
oracle fed the very float32 buffer the GPU stage consumed."""
import numpy as np
import pytest
import torch

import oracle
from paper_2203_15952_amd import binding as B
from parity_util import TINY, check_forward

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


def check_attention(ctx, qkv, B_, T, D, heads, left, right):
    """A scaled score is a float32 chain of dh multiply-adds and one more product: within
    e_s = (dh + 2) u of the sum of the magnitudes of its terms (smag).  exp turns that absolute error
    into a relative error of each weight (plus the exponential's own few u), numerator and normaliser
    are sums of at most T such weights, so their ratio is within 2 (2 e_s smag + (T + 16) u) of the
    float64 result, relative to sum_j p_j |v_j| (vmag)."""
    dh = D // heads
    ref, smag, vmag = oracle.attention(qkv.reshape(B_, T, 3 * D), heads, left, right, want_mags=True)
    rel = 2.0 * (2.0 * (dh + 2) * U * np.repeat(smag, dh, axis=2) + (T + 16) * U)
    bad = np.abs(ctx.reshape(B_, T, D).astype(np.float64) - ref) > rel * vmag + TINY
    assert not bad.any(), f"{bad.sum()} of {bad.size} attention outputs outside tolerance"


ATT_CASES = [
    # B, T, D, heads, left, right
    (32, 400, 512, 8, -1, -1),      # the self-attention configuration: 8 heads of 64, whole utterance
    (2, 70, 128, 2, 23, 0),         # causal with 23 frames of left context (Sec. 3.3); ragged tile
    (1, 130, 72, 2, -1, 3),         # heads of 36 (Conformer S), a little right context
    (3, 65, 12, 3, 5, 7),
    (1, 1, 1, 1, -1, -1),
    (2, 200, 256, 4, 30, 30),       # windows that skip whole key tiles
]


@pytest.mark.parametrize("B_,T,D,heads,left,right", ATT_CASES)
def test_attention_forward(B_, T, D, heads, left, right):
    say("attention", B_, T, D, heads, left, right)
    rng = np.random.default_rng(600 + T + D)
    qkv = rng.standard_normal((B_ * T, 3 * D)).astype(F)
    ctx, m = B.aqt_attention_fwd(dev(qkv), B_, T, heads, left=left, right=right, want_absmax=True)
    ctx_h = host(ctx)
    check_attention(ctx_h, qkv, B_, T, D, heads, left, right)
    assert host(m)[0] == np.abs(ctx_h).max()
    q, s, _ = B.aqt_quantize_with_absmax(ctx, 8, m)
    q_ref, s_ref = oracle.quantize(ctx_h, 8, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(s), s_ref)
    np.testing.assert_array_equal(host(q), q_ref)
    # same bits on a second run (the only atomic is a maximum)
    ctx2, _ = B.aqt_attention_fwd(dev(qkv), B_, T, heads, left=left, right=right)
    np.testing.assert_array_equal(host(ctx2), ctx_h)


def test_attention_window_of_the_frame_itself_returns_the_values():
    rng = np.random.default_rng(610)
    B_, T, D = 2, 100, 128
    qkv = rng.standard_normal((B_ * T, 3 * D)).astype(F)
    ctx, _ = B.aqt_attention_fwd(dev(qkv), B_, T, 2, left=0, right=0)
    np.testing.assert_array_equal(host(ctx), qkv[:, 2 * D:])


def test_attention_argument_errors():
    z = torch.zeros((8, 3 * 130), device="cuda")
    with pytest.raises(B.AqtError) as e:
        B.aqt_attention_fwd(z, 1, 8, 1)          # a head of 130 columns
    assert e.value.status == B.AQT_ERR_UNSUPPORTED
    with pytest.raises(B.AqtError) as e:
        B.aqt_attention_fwd(z, 1, 8, 4)          # 130 is not a multiple of 4 heads
    assert e.value.status == B.AQT_ERR_INVALID_ARG


def rows_of(M):
    mid = (M // 256) * 128
    return np.unique(np.r_[0:min(128, M), mid:min(mid + 128, M), max(0, M - 256):M])


@pytest.mark.parametrize("B_,T,D,heads,left,right,policy,outliers", [
    (32, 400, 512, 8, -1, -1, ((8, 8), (8, 8)), True),    # the self-attention configuration, int8 x int8
    (3, 70, 128, 4, 23, 0, ((4, 8), (8, 8)), False),      # causal, ragged, int4 projection weights
    (2, 19, 24, 2, -1, 2, ((8, 4), (4, 8)), False),       # shapes the general kernels take
])
def test_mhsa_chain_stage_by_stage(B_, T, D, heads, left, right, policy, outliers):
    say("mhsa", B_, T, D, heads, left, right, policy)
    M = B_ * T
    rng = np.random.default_rng(700 + M)
    x = rng.standard_normal((M, D)).astype(F)
    if outliers:   # 1 % of the entries at +-8 standard deviations
        hit = rng.random((M, D)) < 0.01
        x[hit] = np.where(rng.random(int(hit.sum())) < 0.5, F(-8.0), F(8.0))
    gamma, beta = (1 + 0.1 * rng.standard_normal(D)).astype(F), (0.1 * rng.standard_normal(D)).astype(F)
    wqkv, bqkv = (rng.standard_normal((D, 3 * D)) / np.sqrt(D)).astype(F), (0.1 * rng.standard_normal(3 * D)).astype(F)
    wo, bo = (rng.standard_normal((D, D)) / np.sqrt(D)).astype(F), (0.1 * rng.standard_normal(D)).astype(F)
    (bw1, bx1), (bw2, bx2) = policy
    sv = B.MhsaSaved(B_, T, D, policy)
    status = B.new_status()
    x_d, g_d, b_d, wqkv_d, bqkv_d, wo_d, bo_d = (dev(a) for a in (x, gamma, beta, wqkv, bqkv, wo, bo))
    y = B.aqt_mhsa_fwd(x_d, wqkv_d, bqkv_d, wo_d, bo_d, sv, heads, left=left, right=right, gamma=g_d, beta=b_d,
                       dev_status=status)
    assert host(status)[0] == 0
    rows = rows_of(M)
    # stage 1: normalisation + quantizer
    q_a, s_a, xn_t, _ = B.aqt_layernorm_quantize(x_d, bx1, gamma=g_d, beta=b_d, eps=1e-6, want_y=True)
    xn = host(xn_t)
    ref = oracle.layernorm(x, gamma, beta, 1e-6)
    assert (np.abs(xn - ref) <= 1e-5 * (1 + np.abs(ref))).all()
    xq1, sx1 = oracle.quantize(xn, bx1, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(sv.qkv.s_x), sx1)
    np.testing.assert_array_equal(host(sv.qkv.xq), xq1)
    # stage 2: fused projection
    wq1, sw1 = oracle.quantize(wqkv, bw1, 0)
    np.testing.assert_array_equal(host(sv.qkv.wq_kn), wq1)
    qkv_h = host(sv.qkv_f)
    check_forward(qkv_h[rows], oracle.dense_fwd_q(xq1[rows], sx1[0], wq1, sw1, bqkv, 0), sx1[0], sw1, bqkv, 0)
    # stage 3: attention on the GPU's own projections
    ctx_h = host(sv.ctx)
    check_attention(ctx_h, qkv_h, B_, T, D, heads, left, right)
    # stage 4: quantizer on the GPU's own attention result; stage 5: output projection
    xq2, sx2 = oracle.quantize(ctx_h, bx2, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(sv.out.s_x), sx2)
    np.testing.assert_array_equal(host(sv.out.xq), xq2)
    wq2, sw2 = oracle.quantize(wo, bw2, 0)
    np.testing.assert_array_equal(host(sv.out.wq_kn), wq2)
    y_h = host(y)
    check_forward(y_h[rows], oracle.dense_fwd_q(xq2[rows], sx2[0], wq2, sw2, bo, 0), sx2[0], sw2, bo, 0)
    # the one call equals the same entry points called one by one, bit for bit
    wp1, s_w1, _, _ = B.aqt_quantize_weights(wqkv_d, bw1)
    qkv_b, _ = B.aqt_dense_fwd_q(q_a, s_a, wp1, s_w1, 3 * D, bx1, bw1, bias=bqkv_d)
    ctx_b, m_b = B.aqt_attention_fwd(qkv_b, B_, T, heads, left=left, right=right, want_absmax=True)
    q_b, sx_b, _ = B.aqt_quantize_with_absmax(ctx_b, bx2, m_b)
    wp2, s_w2, _, _ = B.aqt_quantize_weights(wo_d, bw2)
    y_b, _ = B.aqt_dense_fwd_q(q_b, sx_b, wp2, s_w2, D, bx2, bw2, bias=bo_d)
    np.testing.assert_array_equal(host(y_b), y_h)


@pytest.mark.parametrize("B_,T,D,heads,left,right", ATT_CASES)
def test_attention_backward(B_, T, D, heads, left, right):
    from parity_util import check_grad
    say("attention bwd", B_, T, D, heads, left, right)
    rng = np.random.default_rng(650 + T + D)
    M = B_ * T
    qkv = rng.standard_normal((M, 3 * D)).astype(F)
    dctx = (0.1 * rng.standard_normal((M, D))).astype(F)
    qkv_d, dctx_d = dev(qkv), dev(dctx)
    lse = torch.empty((M, heads), dtype=torch.float32, device="cuda")
    ctx, _ = B.aqt_attention_fwd(qkv_d, B_, T, heads, left=left, right=right, lse=lse)
    dqkv = B.aqt_attention_bwd(qkv_d, ctx, dctx_d, lse, B_, T, heads, left=left, right=right)
    ref, mag = oracle.attention_bwd(qkv.reshape(B_, T, 3 * D), dctx.reshape(B_, T, D), heads, left, right)
    got = host(dqkv).reshape(B_, T, 3 * D)
    for name, sl in (("dq", slice(0, D)), ("dk", slice(D, 2 * D)), ("dv", slice(2 * D, 3 * D))):
        check_grad(got[:, :, sl], ref[:, :, sl], mag[:, :, sl], name)
    # the forward with lse gives the same ctx as without; the backward has one summation order
    ctx0, _ = B.aqt_attention_fwd(qkv_d, B_, T, heads, left=left, right=right)
    np.testing.assert_array_equal(host(ctx0), host(ctx))
    dqkv2 = B.aqt_attention_bwd(qkv_d, ctx, dctx_d, lse, B_, T, heads, left=left, right=right)
    np.testing.assert_array_equal(host(dqkv2), host(dqkv))
    if M <= 400:   # lse is log2 of the sum of exponentials of the scaled scores
        dh = D // heads
        q, k = (qkv[:, i * D:(i + 1) * D].astype(np.float64).reshape(B_, T, heads, dh) for i in range(2))
        sc = np.einsum("bthd,bjhd->bthj", q, k) / np.sqrt(dh)
        t_i, j_i = np.arange(T)[:, None], np.arange(T)[None, :]
        ok = np.ones((T, T), bool)
        if left >= 0:
            ok &= j_i >= t_i - left
        if right >= 0:
            ok &= j_i <= t_i + right
        sc = np.where(ok[None, :, None, :], sc, -np.inf)
        want = np.log2(np.exp(sc - sc.max(-1, keepdims=True)).sum(-1)) + sc.max(-1) * np.log2(np.e)
        np.testing.assert_allclose(host(lse).reshape(B_, T, heads), want, rtol=0, atol=2e-5 * (1 + np.abs(want).max()))


@pytest.mark.parametrize("B_,T,D,heads,left,right,policy", [
    (8, 200, 512, 8, -1, -1, ((8, 8), (8, 8))),
    (3, 70, 128, 4, 23, 0, ((4, 8), (8, 8))),
    (2, 19, 24, 2, -1, 2, ((8, 4), (4, 8))),
])
def test_mhsa_backward_stage_by_stage(B_, T, D, heads, left, right, policy):
    from parity_util import check_grad
    say("mhsa bwd", B_, T, D, heads, left, right, policy)
    M = B_ * T
    rng = np.random.default_rng(750 + M)
    x = rng.standard_normal((M, D)).astype(F)
    wqkv, bqkv = (rng.standard_normal((D, 3 * D)) / np.sqrt(D)).astype(F), (0.1 * rng.standard_normal(3 * D)).astype(F)
    wo, bo = (rng.standard_normal((D, D)) / np.sqrt(D)).astype(F), (0.1 * rng.standard_normal(D)).astype(F)
    dy = (0.1 * rng.standard_normal((M, D))).astype(F)
    (bw1, bx1), (bw2, bx2) = policy
    sv = B.MhsaSaved(B_, T, D, policy, heads=heads)
    B.aqt_mhsa_fwd(dev(x), dev(wqkv), dev(bqkv), dev(wo), dev(bo), sv, heads, left=left, right=right)
    o = B.aqt_mhsa_bwd(dev(dy), sv, heads, left=left, right=right)
    # output projection against the oracle on the GPU's own codes
    xq2, sx2, wq2, sw2 = host(sv.out.xq), host(sv.out.s_x), host(sv.out.wq_kn), host(sv.out.s_w)
    g2 = oracle.dense_bwd(dy, xq2, sx2[0], wq2, sw2)
    check_grad(host(o["dwo"]), g2["dw"], g2["dw_abs"], "dwo")
    check_grad(host(o["dbo"]), g2["dbias"], np.abs(dy.astype(np.float64)).sum(0), "dbo")
    sv2 = B.Saved(M, D, D, bw2)
    sv2.xq.copy_(sv.out.xq); sv2.s_x.copy_(sv.out.s_x); sv2.wq_kn.copy_(sv.out.wq_kn); sv2.s_w.copy_(sv.out.s_w)
    dctx, _, _ = B.aqt_dense_bwd(dev(dy), sv2, bx2, bw2, want_dw=False)
    dctx_h = host(dctx)
    check_grad(dctx_h, g2["dx"], g2["dx_abs"], "dctx")
    # attention: the oracle fed the float32 gradient and projections the GPU used
    qkv_h = host(sv.qkv_f)
    dqkv = B.aqt_attention_bwd(sv.qkv_f, sv.ctx, dctx, sv.lse, B_, T, heads, left=left, right=right)
    ref, mag = oracle.attention_bwd(qkv_h.reshape(B_, T, 3 * D), dctx_h.reshape(B_, T, D), heads, left, right)
    dqkv_h = host(dqkv)
    check_grad(dqkv_h, ref.reshape(M, 3 * D), mag.reshape(M, 3 * D), "dqkv")
    # fused projection
    xq1, sx1, wq1, sw1 = host(sv.qkv.xq), host(sv.qkv.s_x), host(sv.qkv.wq_kn), host(sv.qkv.s_w)
    g1 = oracle.dense_bwd(dqkv_h, xq1, sx1[0], wq1, sw1)
    check_grad(host(o["dxn"]), g1["dx"], g1["dx_abs"], "dxn")
    check_grad(host(o["dwqkv"]), g1["dw"], g1["dw_abs"], "dwqkv")
    check_grad(host(o["dbqkv"]), g1["dbias"], np.abs(dqkv_h.astype(np.float64)).sum(0), "dbqkv")

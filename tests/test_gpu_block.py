"""Parity of the block-level pieces (backward through Swish / GLU, layer normalisation fused
with the quantizer, the feed-forward module as one call, the float32-emulated product)
against the CPU oracle.  Chains are checked stage by stage: every quantized stage is
compared with the oracle fed the very float32 buffer the GPU stage consumed, because a
float32 value that differs in its last bit from a float64 evaluation can flip a code."""
import numpy as np
import pytest
import torch

import oracle
from paper_2203_15952_amd import binding as B
from paper_2203_15952_amd import inputs
from parity_util import REL_F, check_float_forward, check_forward, check_grad

pytestmark = pytest.mark.gpu
F = np.float32


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def say(*a):
    print(*a, flush=True)


# ----------------------------------------------------------------------------
# backward through the activation
# ----------------------------------------------------------------------------
ACT_BWD_CASES = [
    # M, K, N, bits_w, epilogue          (which kernels)
    (300, 128, 256, 4, 1),               # tuned forward / dX, general dW; ragged M
    (512, 256, 512, 8, 2),               # tuned everywhere, GLU: dy is [M, N/2]
    (37, 50, 24, 4, 2),                  # general kernels, GLU
    (5, 7, 3, 8, 1),
    (1000, 512, 2048, 4, 1),             # the feed-forward shape, Swish
]


@pytest.mark.parametrize("M,K,N,bw,epi", ACT_BWD_CASES)
def test_dense_bwd_through_activation(M, K, N, bw, epi):
    say("bwd through activation", M, K, N, bw, epi)
    c = inputs.small_case(500 + M + N, M, K, N, 8, bw, epi, with_bias=True, with_dy=False)
    oc = N // 2 if epi == 2 else N
    rng = np.random.default_rng(M + epi)
    dout = (rng.standard_normal((M, oc)) * 0.1).astype(F)
    ora = oracle.dense_fwd(c.x, c.w, 8, bw, c.bias, epi)
    sv = B.Saved(M, K, N, bw, dact=True)
    y = B.aqt_dense_fwd(dev(c.x), dev(c.w), 8, bw, bias=dev(c.bias), epilogue=epi, saved=sv)
    np.testing.assert_array_equal(host(sv.xq), ora["xq"])
    np.testing.assert_array_equal(host(sv.wq_kn), ora["wq"])
    check_forward(host(y), ora, ora["s_x"][0], ora["s_w"], c.bias, epi)
    # the saved derivative factors against the textbook derivatives of the float64 value
    dact_ref = oracle.epilogue_dact(ora["pre"], epi)
    err = np.abs(host(sv.dact) - dact_ref)
    assert (err <= 2e-6 + 1e-5 * np.abs(dact_ref)).all(), err.max()
    g = oracle.dense_bwd_epi(dout, ora["pre"], epi, ora["xq"], ora["s_x"][0], ora["wq"], ora["s_w"])
    dx, dw, db = B.aqt_dense_bwd(dev(dout), sv, 8, bw, epilogue=epi, want_dbias=True)
    check_grad(host(dx), g["dx"], g["dx_abs"], "dx")
    check_grad(host(dw), g["dw"], g["dw_abs"], "dw")
    check_grad(host(db), g["dbias"], np.abs(g["dv"]).sum(0), "dbias")
    # without saved factors the call is refused
    sv0 = B.Saved(M, K, N, bw)
    B.aqt_dense_fwd(dev(c.x), dev(c.w), 8, bw, bias=dev(c.bias), epilogue=epi, saved=sv0)
    with pytest.raises(B.AqtError) as e:
        B.aqt_dense_bwd(dev(dout), sv0, 8, bw, epilogue=epi)
    assert e.value.status == B.AQT_ERR_INVALID_ARG


# ----------------------------------------------------------------------------
# layer normalisation fused with the per-tensor quantizer
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("M,D,affine", [(12800, 512, True), (12800, 512, False), (100, 77, True), (3, 1, False),
                                        (4099, 144, True)])
@pytest.mark.parametrize("bits", [8, 4])
def test_layernorm_quantize(M, D, affine, bits):
    say("layernorm + quantize", M, D, affine, bits)
    rng = np.random.default_rng(M + D + bits)
    x = (rng.standard_normal((M, D)) * 3 + 1).astype(F)
    if M > 2:
        x[2] = 5.0                                    # a constant row: zero variance
    gamma = (1 + 0.1 * rng.standard_normal(D)).astype(F) if affine else None
    beta = (0.1 * rng.standard_normal(D)).astype(F) if affine else None
    status = B.new_status()
    q, s, y, stats = B.aqt_layernorm_quantize(dev(x), bits, gamma=None if gamma is None else dev(gamma),
                                              beta=None if beta is None else dev(beta), eps=1e-6, want_y=True,
                                              want_stats=True, dev_status=status)
    y_h = host(y)
    ref = oracle.layernorm(x, gamma, beta, 1e-6)
    assert (np.abs(y_h - ref) <= 1e-5 * (1 + np.abs(ref))).all()
    xd = x.astype(np.float64)
    st = host(stats)
    np.testing.assert_allclose(st[:, 0], xd.mean(1), rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose(st[:, 1], 1 / np.sqrt(xd.var(1) + 1e-6), rtol=1e-4)
    # the codes are Fig. 2 applied to exactly the float32 values the kernel formed
    q_ref, s_ref = oracle.quantize(y_h, bits, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(s), s_ref)
    np.testing.assert_array_equal(host(q), q_ref)
    assert host(status)[0] == 0
    # and identical to the stand-alone quantizer run on the written values
    q2, s2, _ = B.aqt_quantize(y, bits, B.AQT_AXIS_ALL)
    np.testing.assert_array_equal(host(q2), host(q))
    np.testing.assert_array_equal(host(s2), host(s))
    # values only
    _, _, y3, _ = B.aqt_layernorm_quantize(dev(x), bits, gamma=None if gamma is None else dev(gamma),
                                           beta=None if beta is None else dev(beta), quantize=False, want_y=True)
    np.testing.assert_array_equal(host(y3), y_h)


# ----------------------------------------------------------------------------
# the float32-emulated product against the native integer product (Sec. 1)
# ----------------------------------------------------------------------------
def test_fake_float32_product_equals_int32_accumulators_until_24_bits():
    say("fake float32 product")
    rng = np.random.default_rng(60)
    for (M, K, N) in [(256, 1024, 256), (130, 1040, 70), (5, 33, 3)]:
        # int8 x int8: K * 127 * 127 < 2^24 for K <= 1040, so float32 carries every sum exactly
        xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
        wq = rng.integers(-127, 128, (K, N)).astype(np.int8)
        xq[0, :], wq[:, 0] = 127, 127
        exact = xq.astype(np.int64) @ wq.astype(np.int64)
        assert np.abs(exact).max() < 2 ** 24
        fake = host(B.aqt_fake_matmul_f32(dev(xq), dev(wq)))
        np.testing.assert_array_equal(fake.astype(np.int64), exact)
        if K % 128 == 0 and N % 128 == 0:
            # the native integer path on the same codes (int8 weights, fan-in contiguous per channel)
            s_x = dev(np.ones(1, F))
            s_w = dev(np.ones(N, F))
            wq_nk = dev(np.ascontiguousarray(wq.T)).view(torch.uint8).reshape(-1)
            _, acc = B.aqt_dense_fwd_q(dev(xq), s_x, wq_nk, s_w, N, 8, 8, want_acc=True)
            np.testing.assert_array_equal(host(acc), exact)
            np.testing.assert_array_equal(host(acc), fake.astype(np.int64))


def test_fake_float32_product_departs_from_integers_beyond_24_bits():
    # 1041 products of 127 * 127 sum to 16790289 > 2^24: float32 cannot hold the odd sum, the int32
    # accumulator can (Sec. 1: float emulation differs once sums do not fit the 23-bit mantissa)
    xq = np.full((128, 1152), 0, np.int8)
    wq = np.full((1152, 128), 0, np.int8)
    xq[:, :1041], wq[:1041, :] = 127, 127
    fake = host(B.aqt_fake_matmul_f32(dev(xq), dev(wq))).astype(np.float64)
    assert (fake != 16790289.0).all() and (np.abs(fake - 16790289.0) <= 2.0).all()
    s_x, s_w = dev(np.ones(1, F)), dev(np.ones(128, F))
    wq_nk = dev(np.ascontiguousarray(wq.T)).view(torch.uint8).reshape(-1)
    _, acc = B.aqt_dense_fwd_q(dev(xq), s_x, wq_nk, s_w, 128, 8, 8, want_acc=True)
    assert (host(acc) == 16790289).all()
    # generic same-sign data: sums of about 2^25, rounded at many partial sums
    rng = np.random.default_rng(61)
    K = 4096
    xq = rng.integers(1, 128, (256, K)).astype(np.int8)
    wq = rng.integers(100, 128, (K, 128)).astype(np.int8)
    exact = xq.astype(np.int64) @ wq.astype(np.int64)
    fake = host(B.aqt_fake_matmul_f32(dev(xq), dev(wq))).astype(np.float64)
    assert (fake != exact).mean() > 0.2
    assert np.abs(fake - exact).max() <= K * 2.0 ** -24 * exact.max()
    wq_nk = dev(np.ascontiguousarray(wq.T)).view(torch.uint8).reshape(-1)
    _, acc = B.aqt_dense_fwd_q(dev(xq), dev(np.ones(1, F)), wq_nk, dev(np.ones(128, F)), 128, 8, 8, want_acc=True)
    np.testing.assert_array_equal(host(acc), exact)


# ----------------------------------------------------------------------------
# the feed-forward module as one call
# ----------------------------------------------------------------------------
def ffn_inputs(seed, M, D, H):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((M, D)) * 2 + 0.5).astype(F)
    gamma = (1 + 0.1 * rng.standard_normal(D)).astype(F)
    beta = (0.1 * rng.standard_normal(D)).astype(F)
    w1 = (rng.standard_normal((D, H)) / np.sqrt(D)).astype(F)
    b1 = (0.1 * rng.standard_normal(H)).astype(F)
    w2 = (rng.standard_normal((H, D)) / np.sqrt(H)).astype(F)
    b2 = (0.1 * rng.standard_normal(D)).astype(F)
    dy = (rng.standard_normal((M, D)) * 0.1).astype(F)
    return x, gamma, beta, w1, b1, w2, b2, dy


def rows_of(M):
    mid = (M // 256) * 128
    return np.unique(np.r_[0:min(128, M), mid:min(mid + 128, M), max(0, M - 256):M])


@pytest.mark.parametrize("M,D,H,policy", [
    (12800, 512, 2048, ((4, 8), (4, 8))),      # the feed-forward configuration: int4 weights, int8 activations
    (1000, 256, 512, ((8, 8), (4, 4))),        # int8 x int8 first, int4 x int4 second; ragged M
    (70, 40, 24, ((4, 8), (8, 8))),            # shapes the general kernels take
    (33, 27, 22, ((4, 8), (4, 8))),            # odd fan-in under packed codes, widths that are no multiple of 4
])
def test_ffn_chain_stage_by_stage(M, D, H, policy):
    say("ffn chain", M, D, H, policy)
    x, gamma, beta, w1, b1, w2, b2, dy = ffn_inputs(70 + M, M, D, H)
    (bw1, bx1), (bw2, bx2) = policy
    sv = B.FfnSaved(M, D, H, policy)
    status = B.new_status()
    y = B.aqt_ffn_fwd(dev(x), dev(w1), dev(b1), dev(w2), dev(b2), sv, gamma=dev(gamma), beta=dev(beta), eps=1e-6,
                      dev_status=status)
    assert host(status)[0] == 0
    rows = rows_of(M)
    # stage 1: normalisation (float32 against float64), then the quantizer on the GPU's own values
    xn = host(sv.xn)
    ref = oracle.layernorm(x, gamma, beta, 1e-6)
    assert (np.abs(xn - ref) <= 1e-5 * (1 + np.abs(ref))).all()
    xq1, sx1 = oracle.quantize(xn, bx1, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(sv.l1.s_x), sx1)
    np.testing.assert_array_equal(host(sv.l1.xq), xq1)
    # stage 2: first layer with Swish, on those codes
    wq1, sw1 = oracle.quantize(w1, bw1, 0)
    np.testing.assert_array_equal(host(sv.l1.wq_kn), wq1)
    np.testing.assert_array_equal(host(sv.l1.s_w), sw1)
    h = host(sv.h)
    o1 = oracle.dense_fwd_q(xq1[rows], sx1[0], wq1, sw1, b1, oracle.EPI_SWISH)
    check_forward(h[rows], o1, sx1[0], sw1, b1, 1)
    # stage 3: second quantizer on the GPU's own h (one pass, the maximum came from the first contraction)
    xq2, sx2 = oracle.quantize(h, bx2, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(sv.l2.s_x), sx2)
    np.testing.assert_array_equal(host(sv.l2.xq), xq2)
    # stage 4: second layer
    wq2, sw2 = oracle.quantize(w2, bw2, 0)
    np.testing.assert_array_equal(host(sv.l2.wq_kn), wq2)
    o2 = oracle.dense_fwd_q(xq2[rows], sx2[0], wq2, sw2, b2, 0)
    y_h = host(y)
    check_forward(y_h[rows], o2, sx2[0], sw2, b2, 0)
    # the one call equals the same entry points called one by one, bit for bit
    q_a, s_a, _, _ = B.aqt_layernorm_quantize(dev(x), bx1, gamma=dev(gamma), beta=dev(beta), eps=1e-6)
    wp1, s_w1, _, _ = B.aqt_quantize_weights(dev(w1), bw1)
    h_b, m_b = B.aqt_dense_fwd_q_absmax(q_a, s_a, wp1, s_w1, H, bx1, bw1, bias=dev(b1), epilogue=B.AQT_EPI_SWISH)
    q_b, s_b, _ = B.aqt_quantize_with_absmax(h_b, bx2, m_b)
    wp2, s_w2, _, _ = B.aqt_quantize_weights(dev(w2), bw2)
    y_b, _ = B.aqt_dense_fwd_q(q_b, s_b, wp2, s_w2, D, bx2, bw2, bias=dev(b2))
    np.testing.assert_array_equal(host(y_b), y_h)
    if M > 2000:
        return
    # backward, stage by stage: the second layer against the oracle, then the first layer through the
    # Swish with the oracle fed the float32 gradient the GPU passed down
    dxn, dw1, db1, dw2, db2 = B.aqt_ffn_bwd(dev(dy), sv)
    g2 = oracle.dense_bwd(dy, xq2, sx2[0], wq2, sw2)
    check_grad(host(dw2), g2["dw"], g2["dw_abs"], "dw2")
    check_grad(host(db2), g2["dbias"], np.abs(dy.astype(np.float64)).sum(0), "db2")
    sv2 = B.Saved(M, H, D, bw2)          # the same second layer alone, to look at the gradient handed down
    sv2.xq.copy_(sv.l2.xq); sv2.s_x.copy_(sv.l2.s_x); sv2.wq_kn.copy_(sv.l2.wq_kn); sv2.s_w.copy_(sv.l2.s_w)
    dh, _, _ = B.aqt_dense_bwd(dev(dy), sv2, bx2, bw2, want_dw=False)
    dh_h = host(dh)
    check_grad(dh_h, g2["dx"], g2["dx_abs"], "dh")
    pre1 = oracle.dense_fwd_q(xq1, sx1[0], wq1, sw1, b1, oracle.EPI_SWISH)["pre"]
    g1 = oracle.dense_bwd_epi(dh_h, pre1, oracle.EPI_SWISH, xq1, sx1[0], wq1, sw1)
    check_grad(host(dxn), g1["dx"], g1["dx_abs"], "dxn")
    check_grad(host(dw1), g1["dw"], g1["dw_abs"], "dw1")
    check_grad(host(db1), g1["dbias"], np.abs(g1["dv"]).sum(0), "db1")


def test_ffn_chain_weight_only_policy():
    # I4W / I8W (Sec. 4.1): float32 activations, integer weights; forward only
    M, D, H = 600, 256, 512
    say("ffn chain weight-only", M, D, H)
    x, gamma, beta, w1, b1, w2, b2, dy = ffn_inputs(90, M, D, H)
    policy = ((4, 0), (8, 0))
    sv = B.FfnSaved(M, D, H, policy)
    y = B.aqt_ffn_fwd(dev(x), dev(w1), dev(b1), dev(w2), dev(b2), sv, gamma=dev(gamma), beta=dev(beta))
    xn, h = host(sv.xn), host(sv.h)
    ref = oracle.layernorm(x, gamma, beta, 1e-6)
    assert (np.abs(xn - ref) <= 1e-5 * (1 + np.abs(ref))).all()
    wq1, sw1 = oracle.quantize(w1, 4, 0)
    wq2, sw2 = oracle.quantize(w2, 8, 0)
    check_float_forward(h, oracle.dense_fwd_wonly(xn, wq1, sw1, b1, oracle.EPI_SWISH), 1)
    check_float_forward(host(y), oracle.dense_fwd_wonly(h, wq2, sw2, b2, 0), 0)
    with pytest.raises(B.AqtError) as e:
        B.aqt_ffn_bwd(dev(dy), sv)
    assert e.value.status == B.AQT_ERR_UNSUPPORTED
    # mixed: float32 activations into the first layer, int8 activations into the second
    sv2 = B.FfnSaved(M, D, H, ((4, 0), (4, 8)))
    y2 = B.aqt_ffn_fwd(dev(x), dev(w1), dev(b1), dev(w2), dev(b2), sv2, gamma=dev(gamma), beta=dev(beta))
    h2 = host(sv2.h)
    np.testing.assert_array_equal(h2, h)
    xq2, sx2 = oracle.quantize(h2, 8, oracle.AXIS_ALL)
    np.testing.assert_array_equal(host(sv2.l2.xq), xq2)
    wq2b, sw2b = oracle.quantize(w2, 4, 0)
    check_forward(host(y2), oracle.dense_fwd_q(xq2, sx2[0], wq2b, sw2b, b2, 0), sx2[0], sw2b, b2, 0)


# ----------------------------------------------------------------------------
# backward of the normalisation
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("M,D,affine,with_add", [(12800, 512, True, True), (100, 77, True, False), (3, 1, False, True),
                                                 (257, 1024, True, True), (64, 2048, True, True), (1, 512, False, False),
                                                 (1000, 144, True, True)])
def test_layernorm_backward(M, D, affine, with_add):
    say("layernorm bwd", M, D, affine, with_add)
    rng = np.random.default_rng(900 + M + D)
    x = (rng.standard_normal((M, D)) * 2 + 0.5).astype(F)
    gamma = (1 + 0.2 * rng.standard_normal(D)).astype(F) if affine else None
    beta = (0.1 * rng.standard_normal(D)).astype(F) if affine else None
    dy = rng.standard_normal((M, D)).astype(F)
    add = rng.standard_normal((M, D)).astype(F) if with_add else None
    _, _, _, stats = B.aqt_layernorm_quantize(dev(x), 8, gamma=None if gamma is None else dev(gamma),
                                              beta=None if beta is None else dev(beta), want_stats=True)
    dx, dg, db = B.aqt_layernorm_bwd(dev(x), stats, dev(dy), gamma=None if gamma is None else dev(gamma),
                                     add=None if add is None else dev(add))
    rdx, rdg, rdb = oracle.layernorm_bwd(x, dy, gamma, 1e-6)
    # dx is a difference of three terms: hold it to 1e-5 of the sum of their magnitudes (float32 row sums over D
    # terms and the forward's own float32 statistics); the column sums to the gradient bar
    xd = x.astype(np.float64)
    r = 1.0 / np.sqrt(xd.var(1, keepdims=True) + 1e-6)
    xh = (xd - xd.mean(1, keepdims=True)) * r
    g = dy.astype(np.float64) * (1.0 if gamma is None else gamma.astype(np.float64))
    mag = (np.abs(g) + np.abs(g).mean(1, keepdims=True) + np.abs(xh) * np.abs(g * xh).mean(1, keepdims=True)) * r
    want = rdx + (0.0 if add is None else add.astype(np.float64))
    bad = np.abs(host(dx) - want) > 1e-5 * (mag + (0.0 if add is None else np.abs(add))) + 1e-30
    assert not bad.any(), f"{bad.sum()} of {bad.size} dx outside tolerance"
    check_grad(host(dg), rdg, (np.abs(dy.astype(np.float64)) * np.abs(xh)).sum(0), "dgamma")
    check_grad(host(db), rdb, np.abs(dy.astype(np.float64)).sum(0), "dbeta")
    dx2, dg2, db2 = B.aqt_layernorm_bwd(dev(x), stats, dev(dy), gamma=None if gamma is None else dev(gamma),
                                        add=None if add is None else dev(add))
    for p, q in ((dx, dx2), (dg, dg2), (db, db2)):
        np.testing.assert_array_equal(host(p), host(q))
    dx3, _, _ = B.aqt_layernorm_bwd(dev(x), stats, dev(dy), gamma=None if gamma is None else dev(gamma),
                                    add=None if add is None else dev(add), want_affine=False)
    np.testing.assert_array_equal(host(dx3), host(dx))

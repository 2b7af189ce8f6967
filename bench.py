#!/usr/bin/env python3
"""Benchmark of the quantized dense training step on one MI355X.

A step is one pass of the whole hot path over one batch: for each of the two
feed-forward layers of the training-step configuration (65536 tokens, 512->2048
and 2048->512, int8 activations x int4 weights), quantize the activations per
tensor, quantize and pack the weights per output channel, run the int8 MFMA
contraction with fused de-quantization, then the straight-through backward
(dX and dW).  Inputs are seeded synthetic tensors already resident in HBM.

Prints ONE JSON line.  `value` is 6 GEMMs x 2MNK integer/float operations per
step over the step time.  `roofline` describes the kernel that takes the most
time in the step, timed live with HIP events on the launch stream over the timed
steps; the per-kernel table under `kernels` comes from an untimed probe pass that
brackets every segment with events.
`cpu_baseline` is the CPU oracle timed on a bounded row sample of the same
workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
PEAK_INT8_TOPS = 5000.0      # dense int8 MFMA
PEAK_BF16_TFLOPS = 2500.0    # dense bf16 MFMA

# HBM traffic per launch in MiB (read, written) of each segment's kernels at the default
# workload (65536 tokens), from rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by a 1 GiB copy;
# source: profiles/training_step_cfg5_hbm_traffic.txt.  Keys: (layer index, segment).
# The figures belong to the kernels of library version PROFILED_VERSION; any other build
# (a tile variant changed, a kernel rewritten) reports traffic as null instead of stale numbers.
PROFILED_VERSION = 201
MEASURED_TRAFFIC_MIB = {
    (0, "quantize_x"): (128.0 + 128.1, 0.1 + 32.0),      # abs-max pass + code pass
    (1, "quantize_x"): (512.0 + 512.1, 0.1 + 128.0),
    (0, "quantize_w"): (4.1 + 4.2, 2.1 + 1.5),           # slab maxima + quantize / pack
    (1, "quantize_w"): (4.0 + 4.1, 0.5 + 1.5),
    (0, "fwd_gemm"): (0.5 + 40.3, 0.5 + 523.3),          # fragment re-order + contraction
    (1, "fwd_gemm"): (0.5 + 145.4, 0.5 + 136.0),
    (0, "bwd_dx"): (2.0 + 544.2, 2.0 + 128.2),
    (1, "bwd_dx"): (2.0 + 202.0, 2.0 + 512.8),
    (0, "bwd_dw"): (544.1 + 64.1, 64.0 + 4.0),           # slab partials + fold
    (1, "bwd_dw"): (256.1 + 64.1, 64.0 + 4.0),
}


class _NoEvents:
    def record_at(self, i):
        pass


_NO_EVENTS = _NoEvents()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps; the card needs a few tens of milliseconds of load to reach its steady clocks")
    ap.add_argument("--tokens", type=int, default=65536, help="rows of the activation tensors")
    ap.add_argument("--cpu-rows", type=int, default=24576, help="row sample the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the extra figures of the fused abs-max path (keeps a profile to the timed steps)")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the per-layer figures of the forward-only configurations (12800-token shapes)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain elementwise copy of 1 GiB (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2203_15952_amd import binding as B
    from paper_2203_15952_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()

    cases = inputs.config5(seed=1, tokens=args.tokens)
    layers = []
    for c in cases:
        L = dict(c=c, x=torch.from_numpy(c.x).cuda(), w=torch.from_numpy(c.w).cuda(),
                 dy=torch.from_numpy(c.dy).cuda())
        L["sv"] = B.Saved(c.M, c.K, c.N, c.bits_w)
        L["y"] = torch.empty((c.M, c.N), dtype=torch.float32, device="cuda")
        L["dx"] = torch.empty((c.M, c.K), dtype=torch.float32, device="cuda")
        L["dw"] = torch.empty((c.K, c.N), dtype=torch.float32, device="cuda")
        L["ws_q"] = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_QUANTIZE, c.M, c.K, 1))
        L["ws_b"] = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_DENSE_BWD, c.M, c.K, c.N))
        L["ws_w"] = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_QUANTIZE_WEIGHTS, 1, c.K, c.N))
        L["ws_f"] = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD_Q, c.M, c.K, c.N))
        layers.append(L)
    status = B.new_status()

    # One step = these segments, each a C-ABI call that launches one kernel family.
    seg_names = ["quantize_x", "quantize_w", "fwd_gemm", "bwd_dx", "bwd_dw"]

    def run_step(events=None):
        for li, L in enumerate(layers):
            c, sv = L["c"], L["sv"]
            def mark(i):
                if events is not None:
                    h = events[li]
                    if isinstance(h, list):
                        h[i].record()
                    else:
                        h.record_at(i)
            mark(0)
            B.aqt_quantize(L["x"], c.bits_x, B.AQT_AXIS_ALL, q=sv.xq, scale=sv.s_x, ws=L["ws_q"], dev_status=status)
            mark(1)
            B.aqt_quantize_weights(L["w"], c.bits_w, wq_packed=sv.wq_packed, s_w=sv.s_w, wq_kn=sv.wq_kn,
                                   ws=L["ws_w"], dev_status=status)
            mark(2)
            B.aqt_dense_fwd_q(sv.xq, sv.s_x, sv.wq_packed, sv.s_w, c.N, c.bits_x, c.bits_w, y=L["y"], ws=L["ws_f"])
            mark(3)
            B.aqt_dense_bwd(L["dy"], sv, c.bits_x, c.bits_w, dx=L["dx"], want_dw=False, ws=L["ws_b"])
            mark(4)
            B.aqt_dense_bwd(L["dy"], sv, c.bits_x, c.bits_w, dw=L["dw"], want_dx=False, ws=L["ws_b"])
            mark(5)

    t_w = time.perf_counter()
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    # The card needs on the order of 100 ms of load to settle at its steady clocks; when the
    # requested warm-up is shorter than that, keep stepping (untimed) until it has had them.
    while time.perf_counter() - t_w < 0.15:
        for _ in range(10):
            run_step()
        torch.cuda.synchronize()

    # Untimed probe pass with an event around every segment: the per-kernel table, and which
    # segment dominates.  (Twelve event records per step cost about 3 % of a step, so the timed
    # steps below carry events around the dominant segment only.)
    probe_steps = max(1, min(20, args.steps))
    ev = [[[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in layers] for _ in range(probe_steps)]
    for s in range(probe_steps):
        run_step(ev[s])
    torch.cuda.synchronize()
    seg_ms = {}
    for li, L in enumerate(layers):
        for i, name in enumerate(seg_names):
            tot = sum(ev[s][li][i].elapsed_time(ev[s][li][i + 1]) for s in range(probe_steps))
            seg_ms[(li, name)] = tot / probe_steps
    dom_key = max(seg_ms, key=lambda k: seg_ms[k])
    dom_li, dom_i = dom_key[0], seg_names.index(dom_key[1])

    class OnlyDominant:
        """Event holder for the timed steps: records the two events bracketing the dominant segment."""
        def __init__(self):
            self.e = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))

        def __getitem__(self, li):
            return self if li == dom_li else _NO_EVENTS

        def record_at(self, i):
            if i == dom_i:
                self.e[0].record()
            elif i == dom_i + 1:
                self.e[1].record()

    dom_ev = [OnlyDominant() for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        run_step(dom_ev[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms_timed = sum(d.e[0].elapsed_time(d.e[1]) for d in dom_ev) / args.steps
    assert int(status.item()) == 0, "non-finite input reported by the library"

    # Extra figures, outside `value`: layer 1 with a Swish epilogue that also emits max|y|, and the
    # one-pass quantizer of layer 2's input that consumes it, beside their plain counterparts.
    fused = None
    if not args.no_extras:
        L1 = layers[0]
        c1, sv1 = L1["c"], L1["sv"]
        y1 = layers[1]["x"]                       # same shape as layer 2's input: reuse the buffer
        m1 = torch.empty(1, dtype=torch.float32, device="cuda")
        xq2, s2 = layers[1]["sv"].xq, layers[1]["sv"].s_x

        def timed(fn, n=30):
            for _ in range(5):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n
        fused = {
            "fwd_swish_ms": timed(lambda: B.aqt_dense_fwd_q(sv1.xq, sv1.s_x, sv1.wq_packed, sv1.s_w, c1.N, c1.bits_x,
                                                             c1.bits_w, epilogue=B.AQT_EPI_SWISH, y=y1, ws=L1["ws_f"])),
            "fwd_swish_absmax_ms": timed(lambda: B.aqt_dense_fwd_q_absmax(sv1.xq, sv1.s_x, sv1.wq_packed, sv1.s_w, c1.N,
                                                                           c1.bits_x, c1.bits_w, epilogue=B.AQT_EPI_SWISH,
                                                                           y=y1, y_absmax=m1, ws=L1["ws_f"])),
            "quantize_two_pass_ms": timed(lambda: B.aqt_quantize(y1, 8, B.AQT_AXIS_ALL, q=xq2, scale=s2,
                                                                 ws=layers[1]["ws_q"], dev_status=status)),
            "quantize_one_pass_known_absmax_ms": timed(lambda: B.aqt_quantize_with_absmax(y1, 8, m1, q=xq2, scale=s2,
                                                                                         dev_status=status)),
            "tensor": [c1.M, c1.N],
        }
        # the training forward as ONE call (quantize x, quantize + pack w, contraction), per layer;
        # layer 2 runs on the Swish output written above, which is what a chained block feeds it
        ws_fused = [B.workspace(B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD, L["c"].M, L["c"].K, L["c"].N)) for L in layers]
        fused["dense_fwd_one_call_ms"] = [
            timed(lambda L=L, w=w: B.aqt_dense_fwd(L["x"], L["w"], L["c"].bits_x, L["c"].bits_w, y=L["y"], saved=L["sv"],
                                                   ws=w, dev_status=status))
            for L, w in zip(layers, ws_fused)]
        # weight-only modes (float32 activations x int4 weights) on both layer shapes; the
        # contraction is two bf16 MFMA passes over a hi/lo split of x
        ws_wo = [B.workspace(B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD_WONLY, L["c"].M, L["c"].K, L["c"].N)) for L in layers]
        wo_ms = [timed(lambda L=L, w=w: B.aqt_dense_fwd_wonly(L["x"], L["sv"].wq_packed, L["sv"].s_w, L["c"].N,
                                                              L["c"].bits_w, y=L["y"], ws=w))
                 for L, w in zip(layers, ws_wo)]
        fused["weight_only_fwd_ms"] = wo_ms
        fused["weight_only_fwd_tflops"] = [2.0 * L["c"].M * L["c"].K * L["c"].N / ms / 1e9 for L, ms in zip(layers, wo_ms)]
        by = 5.0 * c1.M * c1.N
        fused["quantize_one_pass_gbs"] = by / fused["quantize_one_pass_known_absmax_ms"] / 1e6
        fused["quantize_one_pass_hbm_frac"] = fused["quantize_one_pass_gbs"] / PEAK_HBM_GBS

    def timed_loop(fn, n=30, warm=5):
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    # The forward-only configurations (single layer; feed-forward, self-attention and convolution
    # module layers at 12800 tokens): per quantized layer the contraction alone, the activation
    # quantizer alone and the training forward as one call.  Not part of `value`.
    per_config = None
    if not args.no_configs:
        per_config = {}
        for cfg in (1, 2, 3, 4):
            for c in inputs.CONFIGS[cfg]():
                x_d, w_d = torch.from_numpy(c.x).cuda(), torch.from_numpy(c.w).cuda()
                sv = B.Saved(c.M, c.K, c.N, c.bits_w)
                oc = c.N // 2 if c.epilogue == B.AQT_EPI_GLU else c.N
                y_d = torch.empty((c.M, oc), dtype=torch.float32, device="cuda")
                ws_q = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_QUANTIZE, c.M, c.K, 1))
                ws_f = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD_Q, c.M, c.K, c.N))
                ws_d = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD, c.M, c.K, c.N, c.bits_x, c.bits_w))
                B.aqt_dense_fwd(x_d, w_d, c.bits_x, c.bits_w, epilogue=c.epilogue, y=y_d, saved=sv, ws=ws_d,
                                dev_status=status)
                q_ms = timed_loop(lambda: B.aqt_quantize(x_d, c.bits_x, B.AQT_AXIS_ALL, q=sv.xq, scale=sv.s_x, ws=ws_q,
                                                         dev_status=status))
                g_ms = timed_loop(lambda: B.aqt_dense_fwd_q(sv.xq, sv.s_x, sv.wq_packed, sv.s_w, c.N, c.bits_x, c.bits_w,
                                                            epilogue=c.epilogue, y=y_d, ws=ws_f))
                f_ms = timed_loop(lambda: B.aqt_dense_fwd(x_d, w_d, c.bits_x, c.bits_w, epilogue=c.epilogue, y=y_d,
                                                          saved=sv, ws=ws_d, dev_status=status))
                # serving form: weights re-ordered for the matrix cores once, no per-call pass, no workspace
                wprep = B.aqt_prepare_weights(sv.wq_packed, c.K, c.N, c.bits_w)
                p_ms = timed_loop(lambda: B.aqt_dense_fwd_q_prepared(sv.xq, sv.s_x, wprep, sv.s_w, c.N, c.bits_x,
                                                                     c.bits_w, epilogue=c.epilogue, y=y_d))
                mnk2 = 2.0 * c.M * c.K * c.N
                pk = 0.5 if c.bits_w <= 4 else 1.0
                by = c.M * c.K + c.K * c.N * pk + 4.0 * c.M * oc
                cap = min(PEAK_INT8_TOPS, mnk2 / by * PEAK_HBM_GBS / 1e3)
                tops = mnk2 / g_ms / 1e9
                qby = 5.0 * c.M * c.K
                per_config[c.name] = {
                    "shape_MKN": [c.M, c.K, c.N], "bits_x_w": [c.bits_x, c.bits_w], "epilogue": c.epilogue,
                    "gemm_ms": g_ms, "tops": tops, "pct_int8_peak": 100.0 * tops / PEAK_INT8_TOPS,
                    "roofline_cap_tops": cap, "pct_roofline_cap": 100.0 * tops / cap,
                    "gemm_prepared_weights_ms": p_ms, "pct_roofline_cap_prepared_weights": 100.0 * (mnk2 / p_ms / 1e9) / cap,
                    "quantize_x_ms": q_ms, "quantize_x_gbs_5B_per_elem": qby / q_ms / 1e6,
                    "quantize_x_hbm_frac_5B_per_elem": qby / q_ms / 1e6 / PEAK_HBM_GBS,
                    "dense_fwd_one_call_ms": f_ms}
                del x_d, w_d, sv, y_d, ws_q, ws_f, ws_d, wprep
        torch.cuda.empty_cache()

    if fused is not None:
        # the feed-forward module of the 12800-token configuration as one call (normalisation fused with
        # the first quantizer, max|h| from the first contraction, one-pass second quantizer), forward and
        # straight-through backward down to the normalised input
        Mf, Df, Hf = 12800, 512, 2048
        gen = torch.Generator(device="cuda").manual_seed(2)
        xf = torch.randn((Mf, Df), device="cuda", generator=gen)
        w1f = torch.randn((Df, Hf), device="cuda", generator=gen) / Df ** 0.5
        w2f = torch.randn((Hf, Df), device="cuda", generator=gen) / Hf ** 0.5
        dyf = torch.randn((Mf, Df), device="cuda", generator=gen) * 0.1
        fsv = B.FfnSaved(Mf, Df, Hf, ((4, 8), (4, 8)))
        yf = torch.empty((Mf, Df), dtype=torch.float32, device="cuda")
        ws_ff = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_FFN_FWD, Mf, Df, Hf))
        ws_fb = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_FFN_BWD, Mf, Df, Hf))
        fused["ffn_module_fwd_ms"] = timed_loop(lambda: B.aqt_ffn_fwd(xf, w1f, None, w2f, None, fsv, y=yf, ws=ws_ff,
                                                                      dev_status=status))
        fused["ffn_module_bwd_ms"] = timed_loop(lambda: B.aqt_ffn_bwd(dyf, fsv, want_db=False, ws=ws_fb))
        fused["ffn_module_shape_MDH"] = [Mf, Df, Hf]
        # the convolution module of the 12800-token configuration (32 utterances x 400 frames, width 512,
        # depthwise kernel 32; int4 then int8 pointwise weights) as one call, and its float middle alone:
        # depthwise convolution + normalisation + Swish + abs-max in one pass, 8 B/element of HBM traffic
        Bc, Tc, kwc = 32, 400, 32
        wdw = torch.randn((kwc, Df), device="cuda", generator=gen) / kwc ** 0.5
        wp1 = torch.randn((Df, 2 * Df), device="cuda", generator=gen) / Df ** 0.5
        wp2 = torch.randn((Df, Df), device="cuda", generator=gen) / Df ** 0.5
        csv = B.ConvSaved(Bc, Tc, Df, ((4, 8), (8, 8)))
        ws_cf = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_CONV_MODULE_FWD, Mf, Df, kwc))
        ws_cb = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_CONV_MODULE_BWD, Mf, Df, kwc))
        fused["conv_module_fwd_ms"] = timed_loop(lambda: B.aqt_conv_module_fwd(
            xf, wp1, None, wdw, None, wp2, None, csv, pad_left=15, y=yf, ws=ws_cf, dev_status=status))
        fused["conv_module_bwd_ms"] = timed_loop(lambda: B.aqt_conv_module_bwd(dyf, csv, wdw, pad_left=15, ws=ws_cb))
        g3 = csv.g.view(Bc, Tc, Df)
        dw_ms = timed_loop(lambda: B.aqt_depthwise_conv_fwd(g3, wdw, pad_left=15, swish=True, want_absmax=True))
        fused["depthwise_swish_absmax_fwd_ms"] = dw_ms
        fused["depthwise_fwd_hbm_frac_8B_per_elem"] = 8.0 * Mf * Df / dw_ms / 1e6 / PEAK_HBM_GBS
        fused["conv_module_shape_BTDk"] = [Bc, Tc, Df, kwc]
        # the self-attention module (fused projection, float attention over whole utterances, output projection,
        # int8 x int8) and its float core alone; one whole encoder layer under two of Table 2's policies
        Hh = 8
        wqkv = torch.randn((Df, 3 * Df), device="cuda", generator=gen) / Df ** 0.5
        wo = torch.randn((Df, Df), device="cuda", generator=gen) / Df ** 0.5
        msv = B.MhsaSaved(Bc, Tc, Df, ((8, 8), (8, 8)))
        ws_m = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_MHSA_FWD, Mf, Df, 1))
        fused["mhsa_module_fwd_ms"] = timed_loop(lambda: B.aqt_mhsa_fwd(xf, wqkv, None, wo, None, msv, Hh, y=yf, ws=ws_m,
                                                                        dev_status=status), n=20)
        att_ms = timed_loop(lambda: B.aqt_attention_fwd(msv.qkv_f, Bc, Tc, Hh, want_absmax=True), n=20)
        fused["attention_core_fwd_ms"] = att_ms
        fused["attention_core_tflops_f32"] = 4.0 * Bc * Hh * Tc * Tc * (Df // Hh) / att_ms / 1e9
        lw = {"ffn1_w1": w1f, "ffn1_w2": w2f, "ffn2_w1": w1f, "ffn2_w2": w2f, "att_wqkv": wqkv, "att_wo": wo,
              "conv_w1": wp1, "conv_wdw": wdw, "conv_w2": wp2}
        ws_l = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_CONFORMER_LAYER_FWD, Mf, Df, Hf))
        layer_ms = {}
        for name, pattern, bw in (("int8", B.AQT_POLICY_ALL, 8), ("int4_except_attention", B.AQT_POLICY_EXCEPT_ATTENTION, 4)):
            pol = B.aqt_policy_preset(pattern, 1, 0, bw, 8)[0]
            lsv = B.LayerSaved(Bc, Tc, Df, Hf, pol, heads=Hh)
            layer_ms[name] = timed_loop(lambda: B.aqt_conformer_layer_fwd(
                xf, lw, lsv, B=Bc, T=Tc, H=Hf, heads=Hh, kw=kwc, pad_left=15, y=yf, ws=ws_l, dev_status=status), n=10, warm=3)
            if name == "int8":     # training: straight-through backward of the whole layer, and the serving form
                ws_lb = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_CONFORMER_LAYER_BWD, Mf, Df, Hf))
                fused["encoder_layer_bwd_ms"] = timed_loop(lambda: B.aqt_conformer_layer_bwd(
                    dyf, xf, lw, lsv, B=Bc, T=Tc, H=Hf, heads=Hh, kw=kwc, pad_left=15, ws=ws_lb), n=10, warm=3)
                lsv.prepare(lw)
                fused["encoder_layer_fwd_serving_ms"] = timed_loop(lambda: B.aqt_conformer_layer_fwd(
                    xf, lw, lsv, B=Bc, T=Tc, H=Hf, heads=Hh, kw=kwc, pad_left=15, y=yf, ws=ws_l, dev_status=status), n=10, warm=3)
                del ws_lb
            del lsv
        fused["encoder_layer_fwd_ms"] = layer_ms
        fused["encoder_layer_shape"] = {"utterances": Bc, "frames": Tc, "d_model": Df, "d_ff": Hf, "heads": Hh, "kernel": kwc}
        del wdw, wp1, wp2, csv, ws_cf, ws_cb, g3, wqkv, wo, msv, ws_m, ws_l
        # native integer product against its float32 emulation ("fake" quantization's arithmetic, Sec. 1) on
        # the 2048 -> 512 layer of the training step: same codes, int8 matrix cores vs float32 matrix cores
        L2 = layers[1]
        c2, sv2 = L2["c"], L2["sv"]
        wq8 = sv2.wq_kn.t().contiguous().view(torch.uint8).reshape(-1)      # int8 codes, fan-in contiguous
        s1 = torch.ones(c2.N, dtype=torch.float32, device="cuda")
        fo = torch.empty((c2.M, c2.N), dtype=torch.float32, device="cuda")
        native_ms = timed_loop(lambda: B.aqt_dense_fwd_q(sv2.xq, sv2.s_x, wq8, s1, c2.N, 8, 8, y=L2["y"], ws=L2["ws_f"]),
                               n=20)
        fake_ms = timed_loop(lambda: B.aqt_fake_matmul_f32(sv2.xq, sv2.wq_kn, out=fo), n=5, warm=2)
        fused["native_int8_vs_fake_f32"] = {"shape_MKN": [c2.M, c2.K, c2.N], "native_int8_ms": native_ms,
                                            "fake_f32_ms": fake_ms, "fake_over_native": fake_ms / native_ms}
        del xf, w1f, w2f, dyf, fsv, yf, ws_ff, ws_fb, fo

    if args.calibrate_copy:
        # known traffic: 2^28 floats read (1 GiB) and written (1 GiB) by one elementwise kernel
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(2):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gemm_ops = sum(2.0 * L["c"].M * L["c"].K * L["c"].N for L in layers)      # one GEMM per layer
    total_ops = 3.0 * gemm_ops                                                  # fwd + dX + dW
    value = total_ops / (ms_per_step * 1e-3) / 1e12

    def seg_roofline(li, name):
        c = layers[li]["c"]
        ms = seg_ms[(li, name)]
        mnk2 = 2.0 * c.M * c.K * c.N
        pk = 0.5 if c.bits_w <= 4 else 1.0
        if name == "quantize_x":
            by = c.M * c.K * 5.0                      # 4 B read + 1 B code written per element
            return dict(bound="hbm", achieved=by / ms / 1e6, peak=PEAK_HBM_GBS, unit="GB/s")
        if name == "quantize_w":
            by = c.K * c.N * (4.0 + 1.0 + pk) + 4.0 * c.N
            return dict(bound="hbm", achieved=by / ms / 1e6, peak=PEAK_HBM_GBS, unit="GB/s")
        if name == "fwd_gemm":
            # int8 MFMA work; whether HBM or MFMA bounds it depends on K (fp32 output)
            by = c.M * c.K + c.K * c.N * pk + 4.0 * c.M * c.N
            t_hbm, t_mfma = by / (PEAK_HBM_GBS * 1e9), mnk2 / (PEAK_INT8_TOPS * 1e12)
            if t_hbm >= t_mfma:
                return dict(bound="hbm", achieved=by / ms / 1e6, peak=PEAK_HBM_GBS, unit="GB/s")
            return dict(bound="mfma", achieved=mnk2 / ms / 1e9, peak=PEAK_INT8_TOPS, unit="TOP/s")
        # backward contractions run on bf16 MFMA (codes exact in bf16, float operand split hi/lo)
        return dict(bound="mfma", achieved=mnk2 / ms / 1e9, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s")

    def seg_traffic(li, name):
        """Measured HBM bytes per launch (profiles/), or None away from the profiled workload."""
        if args.tokens != 65536 or B.lib().aqt_version() != PROFILED_VERSION:
            return None
        rd, wr = MEASURED_TRAFFIC_MIB[(li, name)]
        return (rd + wr) * 1048576.0

    kernels = {}
    for (li, name), ms in seg_ms.items():
        c = layers[li]["c"]
        r = seg_roofline(li, name)
        r["frac"] = r["achieved"] / r["peak"]
        r["ms"] = ms
        tr = seg_traffic(li, name)
        r["traffic"] = tr
        if tr is not None:      # measured HBM bytes over measured time, against the 8 TB/s peak
            r["hbm_gbs_measured_bytes"] = tr / ms / 1e6
            r["hbm_frac_measured_bytes"] = tr / ms / 1e6 / PEAK_HBM_GBS
        if name in ("fwd_gemm", "bwd_dx", "bwd_dw"):
            mnk2 = 2.0 * c.M * c.K * c.N
            pk = 0.5 if c.bits_w <= 4 else 1.0
            if name == "fwd_gemm":
                by, peak = c.M * c.K + c.K * c.N * pk + 4.0 * c.M * c.N, PEAK_INT8_TOPS
            elif name == "bwd_dx":
                by, peak = 4.0 * c.M * c.N + c.K * c.N + 4.0 * c.M * c.K, PEAK_BF16_TFLOPS / 2   # two bf16 passes
            else:
                by, peak = c.M * c.K + 4.0 * c.M * c.N + 4.0 * c.K * c.N, PEAK_BF16_TFLOPS / 2
            cap = min(peak, mnk2 / by * PEAK_HBM_GBS / 1e3)      # T(FL)OP/s the roofline allows
            r["tops"] = mnk2 / ms / 1e9
            r["pct_of_mfma_peak_for_dtype"] = 100.0 * r["tops"] / (PEAK_INT8_TOPS if name == "fwd_gemm" else PEAK_BF16_TFLOPS)
            r["pct_of_roofline_cap"] = 100.0 * r["tops"] / cap
        kernels[f"{c.name}.{name}"] = r
    seg_ms[dom_key] = dom_ms_timed            # the dominant kernel's roofline comes from the timed steps
    roof = dict(seg_roofline(*dom_key))
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = seg_traffic(*dom_key)
    roof["kernel"] = f"{layers[dom_key[0]]['c'].name}.{dom_key[1]}"
    roof["launches"] = {"quantize_x": "abs-max pass + code pass", "quantize_w": "slab maxima + quantize/pack",
                        "fwd_gemm": "fragment re-order (about 5 us) + contraction",
                        "bwd_dx": "fragment re-order (about 4 us) + contraction",
                        "bwd_dw": "contraction + slab fold (about 12 us)"}[dom_key[1]]
    if dom_key[1] in ("bwd_dx", "bwd_dw"):
        roof["note"] = ("achieved counts the algorithmic 2MNK; the kernel issues 4MNK MFMA flops (bf16 hi/lo split of the "
                        "float32 operand), so frac = 0.5 would be every matrix-core cycle busy at the peak's clock")
    roof["avg_ms"] = seg_ms[dom_key]

    cpu = None
    if args.cpu_rows > 0:
        import oracle
        rows = min(args.cpu_rows, args.tokens)
        t_cpu, ops_cpu = 0.0, 0.0
        for L in layers:
            c = L["c"]
            xs, dys = c.x[:rows], c.dy[:rows]
            t = time.perf_counter()
            f = oracle.dense_fwd(xs, c.w, c.bits_x, c.bits_w)
            oracle.dense_bwd(dys, f["xq"], f["s_x"][0], f["wq"], f["s_w"], want_dbias=False)
            t_cpu += time.perf_counter() - t
            ops_cpu += 3 * 2.0 * rows * c.K * c.N
        cpu = dict(value=ops_cpu / t_cpu / 1e12, unit="TOPS", cores=oracle.num_threads(), kind="oracle",
                   sample=f"first {rows} of {args.tokens} rows of both layers: quantize + int64 forward + "
                          f"float64 dX and dW, {t_cpu:.1f} s", seconds=t_cpu)

    out = {
        "metric": "quantized dense fwd+bwd TOPS (int8 x int4, int32 acc)",
        "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 x int4 -> int32 (forward), bf16x2 -> f32 (backward)", "data": "synthetic",
        "config": {"workload": "training step, forward + straight-through backward, "
                               f"{args.tokens} tokens, Linear 512->2048 and 2048->512, int4 weights per channel, "
                               "int8 activations per tensor, seed 1 (the fwd+bwd configuration of the metric)",
                   "tokens": args.tokens, "layers": [[c.K, c.N] for c in cases]},
        "pct_of_int8_mfma_peak": 100.0 * value / PEAK_INT8_TOPS,
        "roofline": roof,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "configs": per_config,
        "extras": fused,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()

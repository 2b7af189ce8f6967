"""Time one Conformer encoder layer (Sec. 3.2) and its modules on the GPU at a given shape and precision
policy (Sec. 4.2 / Table 2) and print one JSON line.  Synthetic weights and inputs, seeded.

    python -m paper_2203_15952_amd.layer_bench --pattern except_attention --bits-w 4
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding as B

PATTERNS = {"all": B.AQT_POLICY_ALL, "except_first_last": B.AQT_POLICY_EXCEPT_FIRST_LAST,
            "except_attention": B.AQT_POLICY_EXCEPT_ATTENTION, "first_k": B.AQT_POLICY_FIRST_K}


def timed(fn, n, warm):
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--utterances", type=int, default=32)
    ap.add_argument("--frames", type=int, default=400)
    ap.add_argument("--d-model", type=int, default=512)
    ap.add_argument("--d-ff", type=int, default=2048)
    ap.add_argument("--heads", type=int, default=8)
    ap.add_argument("--kernel", type=int, default=32)
    ap.add_argument("--pad-left", type=int, default=15)
    ap.add_argument("--left-context", type=int, default=-1)
    ap.add_argument("--right-context", type=int, default=-1)
    ap.add_argument("--pattern", choices=sorted(PATTERNS), default="all")
    ap.add_argument("--bits-w", type=int, default=8)
    ap.add_argument("--bits-x", type=int, default=8)
    ap.add_argument("--serving", action="store_true",
                    help="quantize the weights once (prepared operands) instead of in every call")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    a = ap.parse_args()
    Bc, T, D, H, kw = a.utterances, a.frames, a.d_model, a.d_ff, a.kernel
    M = Bc * T
    gen = torch.Generator(device="cuda").manual_seed(0)

    def mat(k, n):
        return torch.randn((k, n), device="cuda", generator=gen) / k ** 0.5

    x = torch.randn((M, D), device="cuda", generator=gen)
    w = {"ffn1_w1": mat(D, H), "ffn1_w2": mat(H, D), "ffn2_w1": mat(D, H), "ffn2_w2": mat(H, D),
         "att_wqkv": mat(D, 3 * D), "att_wo": mat(D, D), "conv_w1": mat(D, 2 * D), "conv_wdw": mat(kw, D),
         "conv_w2": mat(D, D)}
    pol = B.aqt_policy_preset(PATTERNS[a.pattern], 1, 1, a.bits_w, a.bits_x)[0]

    def pair(p, q):
        return ((p.bits_w, p.bits_x), (q.bits_w, q.bits_x))

    y = torch.empty((M, D), dtype=torch.float32, device="cuda")
    ws = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_CONFORMER_LAYER_FWD, M, D, H))
    status = B.new_status()
    sv = B.LayerSaved(Bc, T, D, H, pol, heads=a.heads)
    if a.serving:
        sv.prepare(w)
    out = {"shape": {"utterances": Bc, "frames": T, "d_model": D, "d_ff": H, "heads": a.heads, "kernel": kw},
           "policy": {"pattern": a.pattern, "bits_w": a.bits_w, "bits_x": a.bits_x},
           "weights": "quantized once (serving)" if a.serving else "quantized in every call (training)", "unit": "ms"}

    def layer():
        return B.aqt_conformer_layer_fwd(x, w, sv, B=Bc, T=T, H=H, heads=a.heads, kw=kw, pad_left=a.pad_left,
                                         left=a.left_context, right=a.right_context, y=y, ws=ws, dev_status=status)

    out["encoder_layer_fwd"] = timed(layer, a.steps, a.warmup)
    # the same call recorded once into a HIP graph and replayed: the library allocates nothing and launches
    # only kernels on the caller's stream, so the whole layer is capturable
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):
            layer()
    torch.cuda.current_stream().wait_stream(side)
    with torch.cuda.graph(graph):
        layer()
    eager = y.clone()
    graph.replay()
    torch.cuda.synchronize()
    out["graph_replay_equals_eager"] = bool(torch.equal(y, eager))
    out["encoder_layer_fwd_graph_replay"] = timed(graph.replay, a.steps, a.warmup)
    if not a.serving:
        # training: straight-through backward of the whole layer (input gradient and all weight gradients)
        dy = torch.randn((M, D), device="cuda", generator=gen) * 0.1
        wsb = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_CONFORMER_LAYER_BWD, M, D, H))
        layer()
        out["encoder_layer_bwd"] = timed(lambda: B.aqt_conformer_layer_bwd(
            dy, x, w, sv, B=Bc, T=T, H=H, heads=a.heads, kw=kw, pad_left=a.pad_left, left=a.left_context,
            right=a.right_context, ws=wsb), a.steps, a.warmup)
        dctx = torch.randn((M, D), device="cuda", generator=gen) * 0.1
        wsa = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_ATTENTION_BWD, M, 1, a.heads))
        out["attention_core_bwd"] = timed(lambda: B.aqt_attention_bwd(
            sv.att.qkv_f, sv.att.ctx, dctx, sv.att.lse, Bc, T, a.heads, left=a.left_context, right=a.right_context,
            ws=wsa), a.steps, a.warmup)
    out["ffn_module_fwd"] = timed(lambda: B.aqt_ffn_fwd(x, w["ffn1_w1"], None, w["ffn1_w2"], None, sv.ffn1, y=y, ws=ws,
                                                        dev_status=status), a.steps, a.warmup)
    out["mhsa_module_fwd"] = timed(lambda: B.aqt_mhsa_fwd(x, w["att_wqkv"], None, w["att_wo"], None, sv.att, a.heads,
                                                          left=a.left_context, right=a.right_context, y=y, ws=ws,
                                                          dev_status=status), a.steps, a.warmup)
    out["attention_core_fwd"] = timed(lambda: B.aqt_attention_fwd(sv.att.qkv_f, Bc, T, a.heads, left=a.left_context,
                                                                  right=a.right_context, want_absmax=True),
                                      a.steps, a.warmup)
    out["conv_module_fwd"] = timed(lambda: B.aqt_conv_module_fwd(x, w["conv_w1"], None, w["conv_wdw"], None,
                                                                 w["conv_w2"], None, sv.conv, pad_left=a.pad_left, y=y,
                                                                 ws=ws, dev_status=status), a.steps, a.warmup)
    out["depthwise_fwd"] = timed(lambda: B.aqt_depthwise_conv_fwd(sv.conv.g.view(Bc, T, D), w["conv_wdw"],
                                                                  pad_left=a.pad_left, swish=True, want_dfac=True,
                                                                  want_absmax=True), a.steps, a.warmup)
    out["status"] = int(status.item())
    print(json.dumps(out))


if __name__ == "__main__":
    main()

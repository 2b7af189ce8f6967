"""Native quantization-aware training end to end on synthetic data: a small stack of Conformer encoder
layers (Sec. 3.2) is trained from scratch with every dense layer quantized in the forward pass and
straight-through gradients in the backward pass (Sec. 2.2), under a per-layer precision policy (Sec. 4.2:
here int4 weights in the first k layers, int8 in the rest), and then served from weights quantized once:
what is trained is what is served, bit for bit.

All layer arithmetic runs in libaqt (aqt_conformer_layer_fwd / _bwd); PyTorch holds the float32 master
weights and applies the optimizer step.  The task is synthetic (fit a fixed random smooth map of the input
frames); it shows that the gradients train the quantized network, nothing about speech.

    python -m paper_2203_15952_amd.train_demo --steps 200
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding as B


def init_layer(gen, D, H, kw):
    def mat(k, n):
        return torch.randn((k, n), device="cuda", generator=gen) / k ** 0.5

    w = {}
    for p in ("ffn1", "ffn2"):
        w.update({f"{p}_ln_g": torch.ones(D, device="cuda"), f"{p}_ln_b": torch.zeros(D, device="cuda"),
                  f"{p}_w1": mat(D, H), f"{p}_b1": torch.zeros(H, device="cuda"),
                  f"{p}_w2": mat(H, D), f"{p}_b2": torch.zeros(D, device="cuda")})
    w.update(att_ln_g=torch.ones(D, device="cuda"), att_ln_b=torch.zeros(D, device="cuda"), att_wqkv=mat(D, 3 * D),
             att_bqkv=torch.zeros(3 * D, device="cuda"), att_wo=mat(D, D), att_bo=torch.zeros(D, device="cuda"))
    w.update(conv_ln_g=torch.ones(D, device="cuda"), conv_ln_b=torch.zeros(D, device="cuda"), conv_w1=mat(D, 2 * D),
             conv_b1=torch.zeros(2 * D, device="cuda"), conv_wdw=mat(kw, D), conv_bdw=torch.zeros(D, device="cuda"),
             conv_w2=mat(D, D), conv_b2=torch.zeros(D, device="cuda"))
    w.update(out_ln_g=torch.ones(D, device="cuda"), out_ln_b=torch.zeros(D, device="cuda"))
    return w


class Stack:
    """n_layers encoder layers and a float32 linear read-out; forward and backward through libaqt."""

    def __init__(self, n_layers, Bc, T, D, H, heads, kw, pad_left, left, right, policy, seed=0):
        gen = torch.Generator(device="cuda").manual_seed(seed)
        self.geo = dict(B=Bc, T=T, H=H, heads=heads, kw=kw, pad_left=pad_left, left=left, right=right)
        self.w = [init_layer(gen, D, H, kw) for _ in range(n_layers)]
        self.saved = [B.LayerSaved(Bc, T, D, H, policy[i], heads=heads) for i in range(n_layers)]
        self.policy = policy
        M = Bc * T
        self.acts = [torch.empty((M, D), device="cuda") for _ in range(n_layers + 1)]
        self.ws_f = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_CONFORMER_LAYER_FWD, M, D, H))
        self.ws_b = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_CONFORMER_LAYER_BWD, M, D, H))
        self.status = B.new_status()

    def forward(self, x):
        self.acts[0].copy_(x)
        for i, (w, sv) in enumerate(zip(self.w, self.saved)):
            B.aqt_conformer_layer_fwd(self.acts[i], w, sv, y=self.acts[i + 1], ws=self.ws_f, dev_status=self.status,
                                      **self.geo)
        return self.acts[-1]

    def backward(self, dy):
        grads = [None] * len(self.w)
        for i in reversed(range(len(self.w))):
            dy, grads[i] = B.aqt_conformer_layer_bwd(dy, self.acts[i], self.w[i], self.saved[i], ws=self.ws_b, **self.geo)
        return grads

    def parameters(self):
        return [(i, k, v) for i, w in enumerate(self.w) for k, v in w.items()]


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=2)
    ap.add_argument("--int4-layers", type=int, default=1, help="the first k layers get int4 weights (Table 2, E8-E13)")
    ap.add_argument("--utterances", type=int, default=8)
    ap.add_argument("--frames", type=int, default=128)
    ap.add_argument("--d-model", type=int, default=256)
    ap.add_argument("--d-ff", type=int, default=1024)
    ap.add_argument("--heads", type=int, default=4)
    ap.add_argument("--kernel", type=int, default=15)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--lr", type=float, default=2e-3)
    a = ap.parse_args(argv)
    Bc, T, D, H = a.utterances, a.frames, a.d_model, a.d_ff
    M = Bc * T
    policy = B.aqt_policy_preset(B.AQT_POLICY_FIRST_K, a.layers, a.int4_layers, 4, 8)
    net = Stack(a.layers, Bc, T, D, H, a.heads, a.kernel, a.kernel - 1, 23, 0, policy)     # causal, 23 frames of history
    gen = torch.Generator(device="cuda").manual_seed(1)
    x = torch.randn((M, D), device="cuda", generator=gen)
    # target: a fixed smooth map of the current and the previous frame
    R1, R2 = (torch.randn((D, D), device="cuda", generator=gen) / D ** 0.5 for _ in range(2))
    prev = torch.roll(x.view(Bc, T, D), 1, dims=1).reshape(M, D)
    target = torch.tanh(x @ R1) + 0.5 * torch.tanh(prev @ R2)
    # Adam on the float32 master weights
    m = {(i, k): torch.zeros_like(v) for i, k, v in net.parameters()}
    v2 = {(i, k): torch.zeros_like(v) for i, k, v in net.parameters()}
    losses = []
    for step in range(1, a.steps + 1):
        y = net.forward(x)
        diff = y - target
        losses.append(float((diff * diff).mean()))
        grads = net.backward(diff * (2.0 / diff.numel()))
        for i, k, p in net.parameters():
            g = grads[i].get(k)
            if g is None:
                continue
            m[(i, k)].mul_(0.9).add_(g, alpha=0.1)
            v2[(i, k)].mul_(0.999).addcmul_(g, g, value=0.001)
            mh, vh = m[(i, k)] / (1 - 0.9 ** step), v2[(i, k)] / (1 - 0.999 ** step)
            p.sub_(a.lr * mh / (vh.sqrt() + 1e-8))
    y_train = net.forward(x).clone()
    final = float(((y_train - target) ** 2).mean())
    # serving: quantize every weight matrix once, keep the matrix-core operands, forward again
    for w, sv in zip(net.w, net.saved):
        sv.prepare(w)
    y_serve = net.forward(x)
    out = {"layers": a.layers, "int4_layers": a.int4_layers, "tokens": M, "d_model": D, "steps": a.steps,
           "loss_first": losses[0], "loss_last": final, "loss_every_10th": [round(l, 5) for l in losses[::10]],
           "served_equals_trained_bit_for_bit": bool(torch.equal(y_serve, y_train)),
           "weight_bytes_quantized": B.aqt_policy_weight_bytes(policy, a.layers, D, H),
           "weight_bytes_float32": a.layers * 4 * (4 * D * H + 3 * D * D + D * D + 2 * D * D + D * D),
           "device_status": int(net.status.item())}
    print(json.dumps(out))
    return out


if __name__ == "__main__":
    main()

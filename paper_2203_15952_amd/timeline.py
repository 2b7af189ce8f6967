"""Per-tile timelines of the three GEMM kernels at the training-step shapes.

Builds the library once more with -DAQT_TIMELINE (into libaqt_timeline.so; the product
library is untouched), runs the forward, dX and dW of both training-step layers on seeded
synthetic inputs, and prints, per kernel and layer, what wavefront 0 of every workgroup
stamped: shader-clock cycles spent before the main loop (first loads), in it, issuing the
stores, waiting for them, and the idle time of a compute unit's workgroup slot between the
end of one workgroup and the start of the next one in it.  From the MFMA count of the main loop it
derives how busy the matrix pipes were while the main loops ran.

    python -m paper_2203_15952_amd.timeline            # on an MI355X

A tracing aid: nothing in the product path or the tests depends on it.
"""
from __future__ import annotations

import collections
import ctypes
import os
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
TRACE_LIB = os.path.join(PKG, "libaqt_timeline.so")


def main():
    from paper_2203_15952_amd import build
    if "--no-build" not in sys.argv:
        build.build(defines=["AQT_TIMELINE"], out=TRACE_LIB)
    os.environ["AQT_LIB"] = TRACE_LIB
    import numpy as np
    import torch
    from paper_2203_15952_amd import binding as B
    from paper_2203_15952_amd import inputs

    L = B.lib()

    def pull(which, nblocks):
        buf = np.zeros(nblocks * 8, np.int64)
        fn = L.aqt_timeline_fwd if which == "fwd" else L.aqt_timeline_bwd
        rc = fn(buf.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(buf.nbytes))
        assert rc == 0, rc
        return buf.reshape(nblocks, 8)

    def report(name, a, mfma_per_wave, cycles_per_mfma, waves_per_simd):
        # clocks of different XCDs have different origins: all differences are taken within one workgroup,
        # or between workgroups of one compute unit
        st, pro, loop, epi, done = (a[:, i] for i in range(5))
        hw, xcc = a[:, 5], a[:, 6]
        cu = xcc * 4096 + ((hw >> 13) & 7) * 512 + ((hw >> 12) & 1) * 256 + ((hw >> 8) & 15)
        per_cu = collections.defaultdict(list)
        for i in range(a.shape[0]):
            per_cu[int(cu[i])].append(i)
        gaps, spans = [], []
        for idx in per_cu.values():
            idx.sort(key=lambda i: st[i])
            # workgroup slots of the compute unit: greedily chain each workgroup to the earliest finished one
            ends = []
            for i in idx:
                free = [e for e in ends if e <= st[i]]
                if free:
                    e = max(free)
                    gaps.append(st[i] - e)
                    ends.remove(e)
                ends.append(done[i])
            spans.append(max(done[i] for i in idx) - min(st[i] for i in idx))
        main = (loop - pro).mean()
        busy = mfma_per_wave * cycles_per_mfma * waves_per_simd / main
        print(f"{name}: {a.shape[0]} workgroups on {len(per_cu)} compute units, "
              f"{a.shape[0] / len(per_cu):.1f} per compute unit")
        print(f"   cycles per workgroup: first loads {(pro - st).mean():8.0f} | main loop {main:8.0f} | "
              f"issuing stores {(epi - loop).mean():8.0f} | waiting for stores {(done - epi).mean():6.0f} | "
              f"whole {(done - st).mean():8.0f} (min {(done - st).min()}, max {(done - st).max()})")
        print(f"   matrix pipes busy inside the main loops: {100 * busy:.0f} %   "
              f"(all {waves_per_simd} wavefronts of a SIMD inside, {mfma_per_wave} MFMAs of {cycles_per_mfma} cycles each)")
        if gaps:
            print(f"   idle cycles of a workgroup slot between two workgroups: mean {np.mean(gaps):.0f}, median {np.median(gaps):.0f}")
        print(f"   compute unit busy from first start to last end: mean {np.mean(spans):.0f} cycles, max {np.max(spans)}")

    torch.cuda.set_device(0)
    for c in inputs.config5():
        M, K, N = c.M, c.K, c.N
        print(f"--- layer {K} -> {N}, {M} tokens, int8 x int4")
        sv = B.Saved(M, K, N, c.bits_w)
        x, w, dy = (torch.from_numpy(t).cuda() for t in (c.x, c.w, c.dy))
        y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        dx = torch.empty((M, K), dtype=torch.float32, device="cuda")
        dw = torch.empty((K, N), dtype=torch.float32, device="cuda")
        B.aqt_dense_fwd(x, w, 8, 4, y=y, saved=sv)
        ws_f = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_DENSE_FWD_Q, M, K, N))
        ws_b = B.workspace(B.aqt_workspace_bytes(B.AQT_OP_DENSE_BWD, M, K, N))
        for _ in range(4):
            B.aqt_dense_fwd_q(sv.xq, sv.s_x, sv.wq_packed, sv.s_w, N, 8, 4, y=y, ws=ws_f)
        torch.cuda.synchronize()
        wide = (M // 128) * (N // 256) >= (384 if K >= 1024 else 2048)
        tiles = (M // 128) * (N // (256 if wide else 128))
        stages = K // 128
        report("forward (two workgroups of 4 wavefronts per compute unit)", pull("fwd", tiles),
               stages * 4 * (8 if wide else 4), 32, 2)
        for _ in range(4):
            B.aqt_dense_bwd(dy, sv, 8, 4, dx=dx, want_dw=False, ws=ws_b)
        torch.cuda.synchronize()
        report("dX (one workgroup of 8 wavefronts per compute unit)", pull("bwd", (M // 128) * (K // 512)),
               (N // 32) * 32, 32, 2)
        for _ in range(4):
            B.aqt_dense_bwd(dy, sv, 8, 4, dw=dw, want_dx=False, ws=ws_b)
        torch.cuda.synchronize()
        report("dW (one workgroup of 8 wavefronts per compute unit)", pull("bwd", 256),
               (M // 16 // 32) * 32, 32, 2)
        del sv, x, w, dy, y, dx, dw
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()

"""GPTQ vs GPTAQ latency of the per-layer loop on n x n layers (the shape of the paper's Fig. 4b,
Section 5.6), on synthetic inputs:  python -m paper_2504_02692_amd.latency_sweep [n ...]

For each n: H, dXXT from 4n synthetic tokens, one gptaq_prepare (timed), then the column loop with
only the first update term (GPTQ) and with both terms (GPTAQ), W4 g128, B = 128.
"""
from __future__ import annotations

import sys

import torch

from . import binding as B
from . import synth


def time_ms(fn, reps=3):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def main(sizes):
    print(f"{'n':>6s} {'prepare ms':>11s} {'GPTQ ms':>9s} {'GPTAQ ms':>9s} {'extra':>7s}")
    for n in sizes:
        tokens = 4 * n
        X, Xt = synth.make_activations_device(tokens, n, 0, f"sweep{n}", "cuda")
        H = torch.zeros((n, n), device="cuda"); A = torch.zeros_like(H)
        B.gptaq_accumulate(X, Xt, H, A, B.workspace(B.gptaq_accumulate_workspace_bytes(tokens, n)))
        H0, A0 = H.clone(), A.clone()
        wsp = B.workspace(B.gptaq_prepare_workspace_bytes(n))

        def prep():
            H.copy_(H0); A.copy_(A0)
            B.gptaq_prepare(H, A, 0.01, wsp)
        t_prep = time_ms(prep) - time_ms(lambda: (H.copy_(H0), A.copy_(A0)))
        prep()
        W0 = synth.make_weights_device(n, n, 0, f"sweep{n}", "cuda")
        W = W0.clone()
        wsq = B.workspace(B.gptaq_quantize_workspace_bytes(n, n))

        def run(terms):
            W.copy_(W0)
            B.gptaq_quantize_layer(W, H, A if terms & 2 else None, 4, 128, False, 128, wsq, terms=terms)
        t_copy = time_ms(lambda: W.copy_(W0))
        t_gptq = time_ms(lambda: run(1)) - t_copy
        t_gptaq = time_ms(lambda: run(3)) - t_copy
        print(f"{n:6d} {t_prep:11.3f} {t_gptq:9.3f} {t_gptaq:9.3f} {100 * (t_gptaq / t_gptq - 1):6.1f}%")


if __name__ == "__main__":
    main([int(a) for a in sys.argv[1:]] or [1024, 2048, 4096, 8192])

"""Timings of the entry points beside the main path (act_order, clip-range search, activation fake-quantiser,
code packing) on Llama-2-7B-shaped inputs:  python -m paper_2504_02692_amd.extras_bench

Each figure is the mean of 5 repetitions after one warm-up, from HIP events; the bandwidth figures use the bytes the
operation has to move (inputs read once, outputs written once).
"""
from __future__ import annotations

import torch

from . import binding as B
from . import synth


def time_ms(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def main():
    dev = "cuda"
    print(f"{'operation':58s} {'size':>22s} {'ms':>9s} {'GB/s':>8s}")
    for n in (4096, 11008):
        tokens = 8192
        X, Xt = synth.make_activations_device(tokens, n, 0, f"extras{n}", dev)
        H = torch.zeros((n, n), device=dev); A = torch.zeros_like(H)
        B.gptaq_accumulate(X, Xt, H, A, B.workspace(B.gptaq_accumulate_workspace_bytes(tokens, n)))
        B.gptaq_symmetrize(H)
        t = time_ms(lambda: B.gptaq_act_order(H))
        print(f"{'act_order: rank the diagonal of H':58s} {f'n = {n}':>22s} {t:9.3f} {'':>8s}")
        perm = B.gptaq_act_order(H)
        ws = B.workspace(B.gptaq_permute_hessian_workspace_bytes(n))
        t = time_ms(lambda: B.gptaq_permute_hessian(H, A, perm, ws))
        print(f"{'act_order: permute H and dXXT (rows and columns)':58s} {f'n = {n}':>22s} {t:9.3f} {4 * n * n * 4 / t / 1e6:8.0f}")
        m = 4096
        W = synth.make_weights_device(m, n, 0, f"w{n}", dev)
        t = time_ms(lambda: B.gptaq_permute_columns_f32(W, perm))
        print(f"{'act_order: permute the columns of W (fp32)':58s} {f'{m} x {n}':>22s} {t:9.3f} {2 * m * n * 4 / t / 1e6:8.0f}")
        codes = torch.randint(0, 16, (m, n), dtype=torch.uint8, device=dev)
        t = time_ms(lambda: B.gptaq_permute_columns_u8(codes, perm, inverse=True))
        print(f"{'act_order: un-permute the codes (uint8)':58s} {f'{m} x {n}':>22s} {t:9.3f} {2 * m * n / t / 1e6:8.0f}")
        for bits in (4, 3):
            t = time_ms(lambda: B.gptaq_pack_codes(codes % (1 << bits), bits))
            out_bytes = m * B.gptaq_packed_words_per_row(n, bits) * 4
            print(f"{f'pack {bits}-bit codes into 32-bit words':58s} {f'{m} x {n}':>22s} {t:9.3f} {(m * n + out_bytes) / t / 1e6:8.0f}")
        Xa = X[:8192]
        t = time_ms(lambda: B.gptaq_fake_quant_activations(Xa, 4, 0.9))
        print(f"{'activation fake-quantiser (per token, asym, clip 0.9, A4)':58s} {f'{Xa.shape[0]} x {n}':>22s} {t:9.3f} {2 * Xa.numel() * 2 / t / 1e6:8.0f}")
        # clip-range search: the column loop with and without the search (prepare once, quantise a fresh copy each time)
        Hc, Ac = H.clone(), A.clone()
        B.gptaq_prepare(Hc, Ac, 0.01, B.workspace(B.gptaq_prepare_workspace_bytes(n)))
        wsq = B.workspace(B.gptaq_quantize_workspace_bytes(m, n))
        Wc = W.clone()

        def quant(grid, steps):
            Wc.copy_(W)
            B.gptaq_quantize_layer(Wc, Hc, Ac, 4, 128, False, 128, wsq, mse_grid=grid, mse_steps=steps)
        t0 = time_ms(lambda: quant(0, 0))
        t1 = time_ms(lambda: quant(100, 20))
        print(f"{'quantize W4 g128, min-max ranges':58s} {f'{m} x {n}':>22s} {t0:9.3f} {'':>8s}")
        print(f"{'quantize W4 g128, clip-range search (grid 100, 20 steps)':58s} {f'{m} x {n}':>22s} {t1:9.3f} {'':>8s}")
        del X, Xt, H, A, W, codes, Hc, Ac, Wc


if __name__ == "__main__":
    main()

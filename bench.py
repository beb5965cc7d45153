#!/usr/bin/env python3
"""Benchmark of the GPTAQ per-layer solve on one MI355X.

A "step" is one pass of the whole hot path over one transformer block's layer set:
for every distinct layer input  H, dXXT <- accumulate over all calibration tokens,
U, P <- prepare; then for every layer that reads that input  quantize_layer.
Inputs are synthetic (paper_2504_02692_amd/synth.py) and resident in HBM before the timed
region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama7b] [--chunk 32768] [--staged] [--full-dxxt]
    python bench.py --extras      (timing table of act_order, packing, activation quantiser, clip-range search)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA


def cpu_baseline(wl, budget_s: float = 20.0):
    """Times the fp64 oracle (as it stands) on a bounded sample of the first layer's problem and
    extrapolates each stage by its exact operation count to one average layer of the workload."""
    import threadpoolctl  # noqa: F401  (only to report the BLAS thread count)
    from oracle import gptaq_oracle as O
    from paper_2504_02692_amd import synth
    cores = os.cpu_count() or 1
    try:
        cores = max(i["num_threads"] for i in threadpoolctl.threadpool_info()) if threadpoolctl.threadpool_info() else cores
    except Exception:
        pass
    n_s, tok_s, m_s = 4096, 32768, 512
    Xb, Xtb = synth.make_activations(tok_s, n_s, wl.seed, "cpu", wl.n_outliers, wl.outlier_scale, wl.noise,
                                     empirical_sigma=False)
    W = synth.make_weights(m_s, n_s, wl.seed, "cpu")
    t0 = time.perf_counter(); H, A = O.accumulate(Xb, Xtb); t_acc = time.perf_counter() - t0
    t0 = time.perf_counter(); U, P, dead = O.prepare(H, A, wl.damp); t_prep = time.perf_counter() - t0
    t0 = time.perf_counter(); ref = O.quantize_layer(W, U, P, wl.bits, wl.group, wl.sym); t_q = time.perf_counter() - t0
    # the same loop with the oracle's lazy-batched (BLAS-3) variant: the fairer CPU figure, reported beside it
    t0 = time.perf_counter(); blk = O.quantize_layer_blocked(W, U, P, wl.bits, wl.group, wl.sym, wl.blocksize)
    t_qb = time.perf_counter() - t0
    same = bool((ref["codes"] == blk["codes"]).all())
    # operation counts: accumulate ~ n^2 k, prepare ~ n^3, quantize ~ m n^2
    acc = sum(n * n * wl.tokens for n in wl.inputs().values()) / (n_s * n_s * tok_s) * t_acc
    prep = sum(n ** 3 for n in wl.inputs().values()) / n_s ** 3 * t_prep
    quant = sum(l.m * l.n * l.n for l in wl.layers) / (m_s * n_s * n_s) * t_q
    ms_per_layer = (acc + prep + quant) * 1e3 / len(wl.layers)
    ms_blocked = (acc + prep + quant * t_qb / t_q) * 1e3 / len(wl.layers)
    return {"value": ms_per_layer, "unit": "ms/layer", "cores": int(cores), "kind": "oracle",
            "value_with_blocked_loop": ms_blocked, "blocked_loop_s": t_qb, "blocked_equals_unblocked": same,
            "sample": f"fp64 numpy oracle timed on n={n_s}, {tok_s} tokens, {m_s} rows "
                      f"(accumulate {t_acc:.2f}s, prepare {t_prep:.2f}s, quantize {t_q:.2f}s), each stage scaled by "
                      f"its operation count (n^2 k, n^3, m n^2) to the workload's layer set: extrapolated"}


def time_ms(fn, reps=5):
    import torch
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def extras():
    """Timings of the entry points beside the main path (act_order, clip-range search, activation fake-quantiser,
    code packing) on Llama-2-7B-shaped inputs: mean of 5 repetitions after one warm-up, HIP events; GB/s = bytes the
    operation has to move (inputs read once, outputs written once) / time."""
    import torch
    from paper_2504_02692_amd import binding as B
    from paper_2504_02692_amd import synth
    dev = "cuda"
    print(f"{'operation':58s} {'size':>22s} {'ms':>9s} {'GB/s':>8s}")
    for n in (4096, 11008):
        tokens = 32768
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
        # the two-pass route (order first, then the sums of the reordered inputs, upper triangle of dXXT only)
        diag = torch.zeros(n, device=dev)
        t = time_ms(lambda: B.gptaq_accumulate_diag(X, diag))
        print(f"{'act_order, two passes: diagonal of H from X':58s} {f'{tokens} x {n}':>22s} {t:9.3f} {tokens * n * 2 / t / 1e6:8.0f}")
        inv = B.gptaq_invert_permutation(perm)
        wsa = B.workspace(B.gptaq_accumulate_workspace_bytes(tokens, n))
        H2 = torch.zeros((n, n), device=dev); A2 = torch.zeros_like(H2)
        for name, fn in (("accumulate, every entry of dXXT", lambda: B.gptaq_accumulate(X, Xt, H2, A2, wsa)),
                         ("accumulate, upper triangle of dXXT", lambda: B.gptaq_accumulate_upper(X, Xt, H2, A2, wsa)),
                         ("accumulate, upper triangle, reordered inputs", lambda: B.gptaq_accumulate_upper_permuted(X, Xt, inv, H2, A2, wsa))):
            t = time_ms(fn)
            print(f"{name:58s} {f'{tokens} x {n}':>22s} {t:9.3f} {'':>8s}")
        del H2, A2, wsa
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



def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llama7b")
    ap.add_argument("--chunk", type=int, default=32768, help="tokens per gptaq_accumulate call")
    ap.add_argument("--staged", action="store_true",
                    help="hand the chunks to gptaq_accumulate_staged (products per 32768 pending tokens)")
    ap.add_argument("--full-dxxt", action="store_true",
                    help="accumulate every entry of dXXT (what act_order needs) instead of the entries with col >= row, "
                         "which are all that Eq. 17 reads when the columns are taken in their natural order")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", action="store_true",
                    help="print the timing table of the entry points beside the main path and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the solve has no collective step); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2504_02692_amd import binding as B
    from paper_2504_02692_amd import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        return 2
    B.load()
    if args.extras:
        extras()
        return 0
    dev = torch.device("cuda:0")
    wl = synth.workload(args.workload)
    inputs = wl.inputs()

    # ---- resident inputs
    acts = {iid: synth.make_activations_device(wl.tokens, n, wl.seed, iid, dev, wl.n_outliers, wl.outlier_scale,
                                               wl.noise) for iid, n in inputs.items()}
    # Layers that share an input share U and P and their rows are independent (Step 1 of the paper), so they
    # are solved as one stacked matrix: q/k/v as 12288 x 4096, gate/up as 22016 x 4096.
    groups = {iid: [l for l in wl.layers if l.input_id == iid] for iid in inputs}
    W0 = {iid: torch.cat([synth.make_weights_device(l.m, l.n, wl.seed, l.name, dev) for l in ls], dim=0)
          for iid, ls in groups.items()}
    rounds = args.steps + args.warmup
    Wwork = {iid: [W0[iid].clone() for _ in range(rounds)] for iid in inputs}
    HA = {iid: (torch.empty((n, n), device=dev), torch.empty((n, n), device=dev)) for iid, n in inputs.items()}
    nmax, mmax = max(inputs.values()), max(w.shape[0] for w in W0.values())
    ws_acc = B.workspace(B.gptaq_accumulate_workspace_bytes(32768 if args.staged else args.chunk, nmax))
    ws_prep = B.workspace(B.gptaq_prepare_workspace_bytes(nmax))
    ws_q = B.workspace(B.gptaq_quantize_workspace_bytes(mmax, nmax))
    outs = {iid: (torch.empty(tuple(w.shape), dtype=torch.uint8, device=dev),
                  torch.empty((w.shape[0], max(1, w.shape[1] // wl.group) if wl.group > 0 else 1), device=dev),
                  torch.empty((w.shape[0], max(1, w.shape[1] // wl.group) if wl.group > 0 else 1), device=dev))
            for iid, w in W0.items()}
    info = {iid: torch.zeros(2, dtype=torch.int32, device=dev) for iid in inputs}
    dead = {iid: torch.zeros(n, dtype=torch.uint8, device=dev) for iid, n in inputs.items()}
    stage_ms = {"accumulate": 0.0, "prepare": 0.0, "quantize": 0.0}

    def accumulate(iid, upper):
        X, Xt = acts[iid]
        H, A = HA[iid]
        H.zero_(); A.zero_()
        pending = 0
        for t0 in range(0, wl.tokens, args.chunk):
            t1 = min(wl.tokens, t0 + args.chunk)
            if args.staged:
                pending = B.gptaq_accumulate_staged(X[t0:t1], Xt[t0:t1], H, A, ws_acc, pending, flush=t1 == wl.tokens,
                                                    upper=upper)
            else:
                (B.gptaq_accumulate_upper if upper else B.gptaq_accumulate)(X[t0:t1], Xt[t0:t1], H, A, ws_acc)

    upper = not args.full_dxxt

    def step(r: int, ev=None):
        for iid, n in inputs.items():
            H, A = HA[iid]
            if ev: ev[0].record()
            accumulate(iid, upper)
            if ev: ev[1].record()
            B.gptaq_prepare(H, A, wl.damp, ws_prep, dead=dead[iid], info=info[iid])
            if ev: ev[2].record()
            c, s, z = outs[iid]
            B.gptaq_quantize_layer(Wwork[iid][r], H, A, wl.bits, wl.group, wl.sym, wl.blocksize, ws_q,
                                   dead=dead[iid], codes=c, scales=s, zeros=z)
            if ev:
                ev[3].record(); ev[3].synchronize()
                stage_ms["accumulate"] += ev[0].elapsed_time(ev[1])
                stage_ms["prepare"] += ev[1].elapsed_time(ev[2])
                stage_ms["quantize"] += ev[2].elapsed_time(ev[3])

    for r in range(args.warmup):
        step(r)
    torch.cuda.synchronize()
    B.gptaq_profile_enable(1 << 0)            # only the dominant kernel is bracketed in the timed region
    t_start = time.perf_counter()
    for r in range(args.warmup, rounds):
        step(r)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    launches, gemm_ms = B.gptaq_profile_read(0)
    B.gptaq_profile_enable(0)
    for iid in inputs:
        assert info[iid].cpu().tolist()[0] == 0, "factorisation reported a non-positive pivot"

    # stage and kernel split: one extra, untimed pass with every kernel bracketed
    Wwork = {iid: [W0[iid].clone()] for iid in inputs}
    B.gptaq_profile_enable((1 << len(B.PROFILE_TAGS)) - 1)
    step(0, ev=[torch.cuda.Event(enable_timing=True) for _ in range(4)])
    torch.cuda.synchronize()
    prof = {name: B.gptaq_profile_read(i) for i, name in enumerate(B.PROFILE_TAGS)}
    B.gptaq_profile_enable(0)

    # the accumulation alone in both forms, untimed extra passes (the other form's number is context for the headline)
    acc_ms = {}
    for form in ("upper", "full"):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for iid in inputs:
            accumulate(iid, form == "upper")
        e1.record(); e1.synchronize()
        acc_ms[form] = e0.elapsed_time(e1)

    # what the matrix cores of this machine sustain on nothing but MFMAs (all-ones and random operands), measured here
    peak_ones, clk_ones = B.gptaq_measure_mfma_peak(False, 50)
    peak_rand, clk_rand = B.gptaq_measure_mfma_peak(True, 50)
    hbm_copy = B.gptaq_measure_hbm_copy(1 << 30, 10)          # GB/s of a plain 1 GiB streaming copy (read + written)

    ms_per_step = elapsed * 1e3 / args.steps
    n_layers = len(wl.layers)
    # dominant kernel: the accumulate MFMA GEMM.  Algorithmic flop per launch over c tokens of an n-wide input =
    # n(n+1)c [H, upper half] + 2 n^2 c [all of dXXT], or + n(n+1)c when only the entries of dXXT with col >= row are
    # accumulated.  Executed: every dXXT product twice (exact hi/lo split of dX).
    flops = 0.0
    for iid, n in inputs.items():
        flops += (n * (n + 1) + (n * (n + 1) if upper else 2 * n * n)) * float(wl.tokens)
    flops *= args.steps
    executed_ratio = 1.5 if upper else 5.0 / 3.0
    achieved = flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    # secondary kernels (from the untimed, fully bracketed pass).  The super-block kernel does the column steps and every
    # update inside a 1024-column super-block: against HBM with 17 algorithmic bytes per weight (read W 4, write W^ 4,
    # code 1, -E and V 8).  The trailing update has 2 m n^2 algorithmic flop per layer; the part inside the super-blocks
    # runs in that kernel, the rest in the far-update GEMM.
    wbytes = 17.0 * sum(l.m * l.n for l in wl.layers)
    tflop = 2.0 * sum(l.m * l.n * l.n for l in wl.layers)
    far_flop = 0.0
    for l in wl.layers:
        for sb_end in range(1024, l.n, 1024):
            far_flop += 2.0 * l.m * 1024 * (l.n - sb_end) * 2
    t_sb, t_far = prof["column_loop"][1] * 1e-3, prof["trailing_gemm"][1] * 1e-3
    t_q = stage_ms["quantize"] * 1e-3
    overlap = ("; bracketed on the stream it runs on: the kernels of a tall matrix's two row halves and of a short "
               "matrix's two far chains run beside each other, so these times overlap and sum to more than the stage")
    other = {
        "quantize_stage": {"bound": "hbm", "achieved": wbytes / t_q / 1e9, "peak": 8000.0, "unit": "GB/s",
                           "frac": wbytes / t_q / 1e9 / 8000.0, "frac_of_measured_copy": wbytes / t_q / 1e9 / hbm_copy,
                           "trailing_update_tflops": tflop / t_q / 1e12,
                           "note": "the whole quantize stage (events around it in the stage-split pass): 17 algorithmic bytes per weight, "
                                   "and the 2 m n^2 algorithmic flop of the trailing update over the same time"},
        "superblock_kernel": {"bound": "hbm", "achieved": wbytes / t_sb / 1e9, "peak": 8000.0, "unit": "GB/s",
                              "frac": wbytes / t_sb / 1e9 / 8000.0, "frac_of_measured_copy": wbytes / t_sb / 1e9 / hbm_copy,
                              "mfma_tflops_inside": (tflop - far_flop) / t_sb / 1e12,
                              "note": "column steps + updates inside 1024-column super-blocks; bound by the chain of "
                                      "sequential column steps (n per layer), not by bandwidth" + overlap},
        "far_update_gemm": {"bound": "mfma", "achieved": far_flop / t_far / 1e12 if t_far > 0 else 0.0,
                            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                            "frac": far_flop / t_far / 1e12 / PEAK_BF16_TFLOPS if t_far > 0 else 0.0,
                            "note": "algorithmic flop of the updates that leave a super-block; executed x3 (bf16 hi/lo "
                                    "split of both operands)" + overlap},
        "trailing_update_total": {"bound": "mfma", "achieved": tflop / (t_sb + t_far) / 1e12, "peak": PEAK_BF16_TFLOPS,
                                  "unit": "TFLOP/s", "frac": tflop / (t_sb + t_far) / 1e12 / PEAK_BF16_TFLOPS,
                                  "note": "2 m n^2 algorithmic flop over super-block kernel + far GEMM time"},
    }
    # HBM-side bytes per launch of the dominant kernel come from two separate rocprofv3 --pmc runs of this same command
    # (FETCH_SIZE, WRITE_SIZE); they are quoted only when the committed summary is for this workload and chunk size
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", f"{wl.name}_block_hbm_traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        if tj.get("workload") == wl.name and tj.get("chunk", 32768) == args.chunk and not args.staged \
                and tj.get("dxxt", "full") == ("upper" if upper else "full"):
            traffic, traffic_src = tj.get("bytes_per_launch_avg"), "profiles/" + os.path.basename(tpath)
    out = {
        "metric": "ms_per_layer_solve", "value": ms_per_step / n_layers, "unit": "ms/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16 MFMA -> fp32 (factor: fp64 data, int8-sliced block products)",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: " + ", ".join(f"{l.name} {l.m}x{l.n}" for l in wl.layers) +
                               f"; {wl.tokens} tokens; W{wl.bits} g{wl.group} {'sym' if wl.sym else 'asym'} "
                               f"B{wl.blocksize}; accumulate chunk {args.chunk}{' (staged)' if args.staged else ''}; "
                               f"dXXT: {'entries with col >= row (all that Eq. 17 reads in natural column order)' if upper else 'all entries'}; "
                               f"layers with a common input (q/k/v, gate/up) quantised as one stacked matrix",
                   "layers_per_step": n_layers},
        "roofline": {"bound": "mfma", "kernel": "gemm_nt_kernel<256> (accumulate: H and dXXT)",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_src,
                     "launches": launches, "avg_launch_ms": gemm_ms / max(1, launches),
                     "executed": achieved * executed_ratio,
                     "algorithmic_flop_note": ("n(n+1)c for H plus n(n+1)c for the entries of dXXT with col >= row; the same "
                                               "launches priced at the 3 n^2 c of a full dXXT would read "
                                               f"{achieved * 1.5:.0f} TFLOP/s") if upper else "n(n+1)c for H plus 2 n^2 c for dXXT",
                     "measured_mfma_loop": {"ones_tflops": peak_ones, "ones_clock_ghz": clk_ones,
                                            "random_tflops": peak_rand, "random_clock_ghz": clk_rand,
                                            "executed_frac_of_random": achieved * executed_ratio / peak_rand,
                                            "note": "pure bf16 MFMA loop on all CUs for 50 ms (power-limited clock); "
                                                    "executed = every dXXT product twice (exact hi/lo split of dX): "
                                                    + ("3 n^2 c against 2 n^2 c algorithmic" if upper else
                                                       "5 n^2 c against 3 n^2 c algorithmic")},
                     "measured_hbm_copy_gbps": hbm_copy},
        "other_kernels": other,
        "stages_ms_per_step": stage_ms,
        "accumulate_ms_per_step_by_form": {"dxxt_upper": acc_ms["upper"], "dxxt_full": acc_ms["full"],
                                           "timed_path_uses": "dxxt_upper" if upper else "dxxt_full",
                                           "ms_per_step_with_the_other_form": ms_per_step + (acc_ms["full"] - acc_ms["upper"]) * (1 if upper else -1),
                                           "note": "the step is timed with one form; the accumulation alone is then timed in both, and the "
                                                   "difference gives what the step would take with the other (every entry of dXXT is "
                                                   "what act_order in one pass needs)"},
        "kernels_ms_per_step": {k: v[1] for k, v in prof.items()},
        "kernel_launches_per_step": {k: v[0] for k, v in prof.items()},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

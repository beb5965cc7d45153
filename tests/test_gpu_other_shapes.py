"""Parity on the other layer sets the paper calibrates (synthetic stand-ins, see synth.workload):
EVA-02-Large shapes (W4 per-channel and W3 g128, symmetric), Llama-3-70B shapes (W3 g128 and W2 g64,
8192- and 28672-wide Hessians) and Llama-3-405B shapes (65536 tokens, the 53248-wide Hessian of
down_proj: the largest size the paper reports, Table 9).

Small sizes go against the whole fp64 oracle.  Where the fp64 oracle (or one host factorisation) does not
fit the time budget, each stage is checked on what can be computed exactly:
  accumulate : fp64 sums over ALL tokens for sampled sets of neurons;
  prepare    : (a) the trailing s x s corner of U against the oracle's prepare of the trailing corner of
               H + lam I (for H + lam I = V V^T with V upper, the corner of V only depends on the corner of
               H + lam I); (b) sampled columns of U^T U against columns of (H + lam I)^-1 obtained by fp64
               iterative refinement (residuals with the untouched H in fp64; the refinement contracts only
               if U^T U is a good approximate inverse, and its limit does not depend on U); (c) sampled rows
               of P against Eq. 17 evaluated in fp64 from the same U, and late rows against Eq. 16 by a
               direct fp64 solve;
  quantize   : the oracle's column loop on sampled rows (rows are independent, Step 1) with the near-tie
               protocol, plus whole-matrix properties.
torch fp64 matrix-vector products on the GPU serve as the library primitive of these reference steps.
"""
import numpy as np
import pytest
import torch

from oracle import gptaq_oracle as O
from paper_2504_02692_amd import binding as B
from paper_2504_02692_amd import synth
from tests import parity_util as PU
from tests.test_gpu_fullsize import accumulate_full, bits_of, check_sampled_blocks

pytestmark = pytest.mark.gpu


def layer_of(wl, name):
    return [l for l in wl.layers if l.name == name][0]


def quantize_rows(wl, layer, U_d, P_d, U64, P64, bits, group, sym, label, nrows=32, Xs=None, Xts=None):
    """GPU quantize of the whole layer, oracle on sampled rows.  `layer` may be a list of layers that share the
    input: they are quantised as one stacked matrix, the way bench.py runs q/k/v and gate/up."""
    layers = layer if isinstance(layer, (list, tuple)) else [layer]
    n = layers[0].n
    W0 = torch.cat([synth.make_weights_device(l.m, n, wl.seed, l.name, "cuda") for l in layers], dim=0)
    m = W0.shape[0]
    Wd = W0.clone()
    ws = B.workspace(B.gptaq_quantize_workspace_bytes(m, n))
    codes, scales, zeros = B.gptaq_quantize_layer(Wd, U_d, P_d, bits, group, sym, wl.blocksize, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, m - 1], rng.choice(m, nrows, replace=False)]))
    ridx = torch.as_tensor(rows, device="cuda")
    got = dict(What=Wd[ridx].cpu().numpy(), codes=codes[ridx].cpu().numpy(), scales=scales[ridx].cpu().numpy(),
               zeros=zeros[ridx].cpu().numpy())
    PU.check_against_oracle(W0[ridx].cpu().numpy(), U64, P64, got, bits, group, sym, Xb=Xs, Xtb=Xts, label=label)
    assert int(codes.max().item()) <= 2 ** bits - 1
    assert bool((scales > 0).all()) and bool((zeros == torch.round(zeros)).all())
    if group > 0:                       # the returned grid reproduces the returned weights, whole matrix
        G = n // group
        for r0 in range(0, m, 16384):   # (in slabs of rows: the stacked matrices are several GB)
            r1 = min(m, r0 + 16384)
            rec = (scales[r0:r1, :, None] * (codes[r0:r1].view(r1 - r0, G, group).float() - zeros[r0:r1, :, None]))
            assert torch.allclose(rec.view(r1 - r0, n), Wd[r0:r1], rtol=1e-6, atol=1e-9)
            del rec


# ------------------------------------------------------------------------------------- EVA-02 shapes
@pytest.mark.parametrize("bits,group", [(4, 0), (3, 128)])
def test_eva02_attention_input_whole_oracle(bits, group):
    wl = synth.workload("eva02")
    n = 1024
    Xb, Xtb = synth.make_activations(wl.tokens, n, wl.seed, "attn_in", wl.n_outliers, wl.outlier_scale, wl.noise)
    H, A = PU.gpu_accumulate(Xb, Xtb, chunks=[0, 8192, 16384, 24576, wl.tokens])
    Hg = H.cpu().numpy().astype(np.float64)
    Hg = np.triu(Hg) + np.triu(Hg, 1).T
    Ho, Ao = O.accumulate(Xb, Xtb)
    eh, ea = PU.rel_fro(Hg, Ho), PU.rel_fro(A.cpu().numpy(), Ao)
    print(f"[eva02 n={n}] H {eh:.3e} dXXT {ea:.3e}")
    assert eh <= 1e-5 and ea <= 1e-5
    U64, P64, _ = O.prepare(Ho, Ao, wl.damp)
    dead, info = PU.gpu_prepare(H, A, wl.damp)
    assert info.cpu().tolist() == [0, 0]
    eu, ep = PU.rel_fro(H.cpu().numpy(), U64), PU.rel_fro(A.cpu().numpy(), P64)
    print(f"[eva02 n={n}] U {eu:.3e} P {ep:.3e}")
    assert eu <= 1e-6 and ep <= 5e-5
    layer = layer_of(wl, "qkv")
    W = synth.make_weights(layer.m, n, wl.seed, layer.name)
    got = PU.gpu_quantize(W, H, A, bits, group, True, wl.blocksize)
    # the whole chain (accumulate -> prepare -> quantize on the GPU) against the all-fp64 oracle chain ...
    PU.check_against_oracle(W, U64, P64, got, bits, group, True, Xb=Xb[::8], Xtb=Xtb[::8],
                            label=f"eva02 qkv 3072x1024 W{bits} g{group} sym, all-fp64 oracle")
    # ... and the column loop alone: the oracle's loop fed with the library's own factors
    PU.check_against_oracle(W, H.cpu().numpy().astype(np.float64), A.cpu().numpy().astype(np.float64), got, bits, group,
                            True, label=f"eva02 qkv 3072x1024 W{bits} g{group} sym, library factors")


def test_eva02_mlp_input_4096():
    wl = synth.workload("eva02")
    n, iid = 4096, "mlp_mid"
    X, Xt, H, A = accumulate_full(wl, iid, n)
    Hg, Ag = check_sampled_blocks(wl, iid, n, X, Xt, H, A)
    U64, P64, _ = O.prepare(Hg, Ag, wl.damp)
    dd, info = B.gptaq_prepare(H, A, wl.damp, B.workspace(B.gptaq_prepare_workspace_bytes(n)))
    torch.cuda.synchronize()
    assert info.cpu().tolist() == [0, 0]
    eu, ep = PU.rel_fro(H.cpu().numpy(), U64), PU.rel_fro(A.cpu().numpy(), P64)
    print(f"[eva02 n={n}] U {eu:.3e} P {ep:.3e}")
    assert eu <= 1e-6 and ep <= 5e-5
    tok = torch.arange(0, wl.tokens, 8, device="cuda")
    for bits, group in ((4, 0), (3, 128)):
        # the oracle's loop runs on the fp64 factors (fp64 prepare of the sums checked above), not on the library's
        quantize_rows(wl, layer_of(wl, "fc2"), H, A, U64, P64, bits, group, True,
                      f"eva02 fc2 W{bits} g{group} sym, fp64 factors", Xs=bits_of(X[tok]), Xts=bits_of(Xt[tok]))


# ----------------------------------------------------------------- large Hessians: reference pieces
def prepare_and_check_large(wl, iid, n, H, A, Ag_rows, corner=1536, ncols=6):
    """Runs gptaq_prepare on (H, A) in place and checks U and P as the module docstring says.
    Ag_rows: {row index: fp64 row of dXXT} for the rows of P to be checked.  Returns fp64 device U."""
    Hup = H.clone()                                             # upper triangle of H, untouched
    lam = float(wl.damp * torch.diagonal(Hup).double().mean().item())
    dd, info = B.gptaq_prepare(H, A, wl.damp, B.workspace(B.gptaq_prepare_workspace_bytes(n)))
    torch.cuda.synchronize()
    assert info.cpu().tolist() == [0, 0]
    torch.cuda.empty_cache()
    U = H.double()
    assert bool((torch.diagonal(U) > 0).all())
    assert float(torch.tril(H[-2048:, -2048:], -1).abs().max()) == 0.0 and float(H[n // 2, 0]) == 0.0
    # (a) trailing corner against the oracle
    s = corner
    Hc = Hup[n - s:, n - s:].double().cpu().numpy()
    Hc = np.triu(Hc) + np.triu(Hc, 1).T
    Uc = O.inverse_cholesky(Hc + lam * np.eye(s)).T            # upper U with (.)^-1 = U^T U
    ec = PU.rel_fro(U[n - s:, n - s:].cpu().numpy(), Uc)
    print(f"[{iid} n={n}] trailing {s}x{s} corner of U vs oracle: {ec:.3e}")
    assert ec <= 1e-6
    # (b) sampled columns of U^T U by iterative refinement with the untouched H in fp64
    H64 = torch.triu(Hup.double())                              # diagonal tiles also hold their lower halves
    del Hup

    def apply_H(x):                                             # (H + lam I) x from the stored upper triangle
        d = torch.diagonal(H64)
        return torch.mv(H64, x) + torch.mv(H64.t(), x) - d * x + lam * x

    def apply_inv(x):                                           # U^T U x
        return torch.mv(U.t(), torch.mv(U, x))

    rng = np.random.default_rng(3)
    cols = np.unique(np.concatenate([[0, n - 1], synth.outlier_channels(n, wl.n_outliers, wl.seed, iid)[:2],
                                     rng.choice(n, ncols, replace=False)]))
    worst = 0.0
    for j in cols:
        e = torch.zeros(n, dtype=torch.float64, device="cuda"); e[j] = 1.0
        x0 = apply_inv(e)
        x = x0.clone()
        for _ in range(4):
            r = e - apply_H(x)
            x = x + apply_inv(r)
        res = float(torch.linalg.norm(e - apply_H(x)))
        assert res <= 1e-9, (j, res)                            # the refinement converged: x is the fp64 column
        err = float(torch.linalg.norm(x0 - x) / torch.linalg.norm(x))
        worst = max(worst, err)
        assert err <= 1e-5, (j, err)
    print(f"[{iid} n={n}] columns of U^T U vs refined columns of (H + lam I)^-1: worst {worst:.3e}")
    # (c) rows of P: Eq. 17 in fp64 from the same U; late rows: Eq. 16 by a direct solve
    Pd = A.double()
    for q, a in Ag_rows.items():
        a64 = torch.as_tensor(a, dtype=torch.float64, device="cuda")
        o = torch.mv(U, a64)                                    # (dXXT[q, :] U^T)
        o[: q + 1] = 0.0                                        # (.) M_U: strictly upper
        ref = torch.mv(U.t(), o)
        err = float(torch.linalg.norm(Pd[q] - ref) / torch.linalg.norm(ref))
        print(f"[{iid} n={n}] P row {q} vs Eq. 17 in fp64: {err:.3e}")
        assert err <= 5e-5 and float(Pd[q, : q + 1].abs().max()) == 0.0
        if n - q <= 2048:
            Hq = H64[q + 1:, q + 1:].cpu().numpy()
            Hq = np.triu(Hq) + np.triu(Hq, 1).T + lam * np.eye(n - q - 1)
            ref16 = np.linalg.solve(Hq, a[q + 1:])
            e16 = np.linalg.norm(Pd[q, q + 1:].cpu().numpy() - ref16) / np.linalg.norm(ref16)
            print(f"[{iid} n={n}] P row {q} vs Eq. 16 (direct solve): {e16:.3e}")
            assert e16 <= 1e-4
    del H64
    return U, Pd


def rows_of_dxxt(A, rows):
    return {int(q): A[int(q)].double().cpu().numpy() for q in rows}


# ------------------------------------------------------------------------------- Llama-3-70B shapes
def test_llama70b_attention_input_8192():
    wl = synth.workload("llama70b")
    n, iid = 8192, "attn_in"
    X, Xt, H, A = accumulate_full(wl, iid, n)
    check_sampled_blocks(wl, iid, n, X, Xt, H, A)
    rows = rows_of_dxxt(A, [0, n // 3, n - 700, n - 2])
    U, Pd = prepare_and_check_large(wl, iid, n, H, A, rows)
    tok = torch.arange(0, wl.tokens, wl.tokens // 2048, device="cuda")[:2048]
    Xs, Xts = bits_of(X[tok]), bits_of(Xt[tok])
    del X, Xt
    U64, P64 = U.cpu().numpy(), Pd.cpu().numpy()
    del U, Pd
    quantize_rows(wl, layer_of(wl, "q_proj"), H, A, U64, P64, 3, 128, False, "70b q_proj 8192x8192 W3 g128", Xs=Xs, Xts=Xts)
    quantize_rows(wl, layer_of(wl, "k_proj"), H, A, U64, P64, 2, 64, False, "70b k_proj 1024x8192 W2 g64", Xs=Xs, Xts=Xts)
    # gate and up (28672 x 8192 each) at full width, stacked to 57344 rows.  Their own input has the same width as this
    # one and differs from it only in its random draws, so the factors prepared above serve as its U and P here.
    quantize_rows(wl, [layer_of(wl, "gate_proj"), layer_of(wl, "up_proj")], H, A, U64, P64, 3, 128, False,
                  "70b gate+up 57344x8192 W3 g128", nrows=20)


def test_llama70b_mlp_down_input_28672():
    wl = synth.workload("llama70b")
    n, iid = 28672, "mlp_mid"
    X, Xt, H, A = accumulate_full(wl, iid, n)
    check_sampled_blocks(wl, iid, n, X, Xt, H, A)
    del X, Xt
    torch.cuda.empty_cache()
    rows = rows_of_dxxt(A, [0, n // 2, n - 900, n - 2])
    U, Pd = prepare_and_check_large(wl, iid, n, H, A, rows)
    U64, P64 = U.cpu().numpy(), Pd.cpu().numpy()
    del U, Pd
    torch.cuda.empty_cache()
    quantize_rows(wl, layer_of(wl, "down_proj"), H, A, U64, P64, 3, 128, False, "70b down_proj 8192x28672 W3 g128", nrows=14)


# ------------------------------------------------------------------------------ Llama-3-405B shapes
def test_llama405b_attention_and_mlp_inputs_16384():
    """The 16384-wide inputs of the Llama-3-405B-shaped set (65536 tokens): accumulate and prepare on the attention
    input, then q_proj (16384 x 16384), k and v stacked (2048 x 16384) and gate and up stacked (106496 x 16384).
    The MLP input has the same width and differs only in its random draws, so gate/up are quantised with the same
    factors (accumulate and prepare at this width are covered by the attention input)."""
    wl = synth.workload("llama405b")
    n, iid = 16384, "attn_in"
    X, Xt, H, A = accumulate_full(wl, iid, n)
    check_sampled_blocks(wl, iid, n, X, Xt, H, A)
    rows = rows_of_dxxt(A, [0, n // 3, n - 1100, n - 2])
    U, Pd = prepare_and_check_large(wl, iid, n, H, A, rows, ncols=4)
    tok = torch.arange(0, wl.tokens, wl.tokens // 1024, device="cuda")[:1024]
    Xs, Xts = bits_of(X[tok]), bits_of(Xt[tok])
    del X, Xt
    U64, P64 = U.cpu().numpy(), Pd.cpu().numpy()
    del U, Pd
    torch.cuda.empty_cache()
    quantize_rows(wl, layer_of(wl, "q_proj"), H, A, U64, P64, 4, 128, False, "405b q_proj 16384x16384 W4 g128", nrows=14,
                  Xs=Xs, Xts=Xts)
    quantize_rows(wl, [layer_of(wl, "k_proj"), layer_of(wl, "v_proj")], H, A, U64, P64, 4, 128, False,
                  "405b k+v 2048x16384 W4 g128", nrows=14, Xs=Xs, Xts=Xts)
    quantize_rows(wl, [layer_of(wl, "gate_proj"), layer_of(wl, "up_proj")], H, A, U64, P64, 4, 128, False,
                  "405b gate+up 106496x16384 W4 g128", nrows=14)


def test_llama405b_mlp_down_input_53248():
    wl = synth.workload("llama405b")
    n, iid = 53248, "mlp_mid"
    X, Xt, H, A = accumulate_full(wl, iid, n)
    check_sampled_blocks(wl, iid, n, X, Xt, H, A)
    del X, Xt
    torch.cuda.empty_cache()
    rows = rows_of_dxxt(A, [0, n - 1200, n - 2])
    U, Pd = prepare_and_check_large(wl, iid, n, H, A, rows, ncols=3)
    U64, P64 = U.cpu().numpy(), Pd.cpu().numpy()
    del U, Pd
    torch.cuda.empty_cache()
    quantize_rows(wl, layer_of(wl, "down_proj"), H, A, U64, P64, 4, 128, False, "405b down_proj 16384x53248 W4 g128", nrows=6)

"""Parity of the HIP path (through the C ABI) with the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import gptaq_oracle as O
from paper_2504_02692_amd import synth
from tests import parity_util as PU

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c1():
    wl = synth.workload("c1")
    Xb, Xtb = synth.make_activations(wl.tokens, 512, wl.seed, "x", wl.n_outliers, wl.outlier_scale, wl.noise)
    W = synth.make_weights(512, 512, wl.seed, "fc")
    H, A = O.accumulate(Xb, Xtb)
    U, P, dead = O.prepare(H, A, wl.damp)
    return dict(wl=wl, Xb=Xb, Xtb=Xtb, W=W, H=H, A=A, U=U, P=P)


def upper_to_full(Hd):
    h = Hd.cpu().numpy().astype(np.float64)
    return np.triu(h) + np.triu(h, 1).T


# ------------------------------------------------------------------ accumulate
def test_accumulate_c1(c1):
    Hd, Ad = PU.gpu_accumulate(c1["Xb"], c1["Xtb"])
    eh, ea = PU.rel_fro(upper_to_full(Hd), c1["H"]), PU.rel_fro(Ad.cpu().numpy(), c1["A"])
    print(f"H rel. Frobenius {eh:.3e}  dXXT rel. Frobenius {ea:.3e}")
    assert eh <= 1e-5 and ea <= 1e-5


def test_accumulate_streamed_chunks_and_small_workspace(c1):
    # three unequal chunks, the last one through a workspace that only holds 128 tokens
    Hd, Ad = PU.gpu_accumulate(c1["Xb"], c1["Xtb"], chunks=[0, 1000, 3000, 4096],
                               ws_bytes=3 * 512 * 128 * 2)
    assert PU.rel_fro(upper_to_full(Hd), c1["H"]) <= 1e-5
    assert PU.rel_fro(Ad.cpu().numpy(), c1["A"]) <= 1e-5


@pytest.mark.parametrize("tokens,n", [(1, 8), (77, 200), (333, 1096), (640, 2304)])
def test_accumulate_ragged_shapes(tokens, n):
    Xb, Xtb = synth.make_activations(tokens, n, 4, "rag", 3, 20.0)
    H, A = O.accumulate(Xb, Xtb)
    Hd, Ad = PU.gpu_accumulate(Xb, Xtb)
    assert PU.rel_fro(upper_to_full(Hd), H) <= 1e-5
    assert PU.rel_fro(Ad.cpu().numpy(), A) <= 1e-5


def test_accumulate_staged_small_chunks():
    # 2048-token samples (Section 5.1) staged into 32768-token product launches: 34 samples + a ragged
    # tail cross one launch boundary and leave a partial launch for the flush
    from paper_2504_02692_amd import binding as B
    n, chunk, tokens = 200, 2048, 34 * 2048 + 77
    Xb, Xtb = synth.make_activations(tokens, n, 6, "staged", 3, 20.0)
    H, A = O.accumulate(Xb, Xtb)
    X, Xt = PU.to_dev_bf16(Xb), PU.to_dev_bf16(Xtb)
    Hd = torch.zeros((n, n), device="cuda"); Ad = torch.zeros_like(Hd)
    ws = B.workspace(B.gptaq_accumulate_workspace_bytes(32768, n))
    pending, seen = 0, []
    for t0 in range(0, tokens, chunk):
        last = t0 + chunk >= tokens
        pending = B.gptaq_accumulate_staged(X[t0:t0 + chunk], Xt[t0:t0 + chunk], Hd, Ad, ws, pending, flush=last)
        seen.append(pending)
    assert seen[:16] == [2048 * (i + 1) % 32768 for i in range(16)] and seen[-1] == 0
    assert PU.rel_fro(upper_to_full(Hd), H) <= 1e-5
    assert PU.rel_fro(Ad.cpu().numpy(), A) <= 1e-5
    # the same launches as direct calls on 32768-token chunks: bit-identical sums
    H2, A2 = PU.gpu_accumulate(Xb, Xtb, chunks=[0, 32768, 65536, tokens])
    assert torch.equal(Hd, H2) and torch.equal(Ad, A2)
    # one call with everything (it crosses two launch boundaries inside the call)
    H3 = torch.zeros_like(Hd); A3 = torch.zeros_like(Hd)
    assert B.gptaq_accumulate_staged(X, Xt, H3, A3, ws, 0, flush=True) == 0
    assert torch.equal(H3, H2) and torch.equal(A3, A2)
    # a flush with nothing to add changes nothing
    assert B.gptaq_accumulate_staged(None, None, Hd, Ad, ws, 0, flush=True) == 0
    assert torch.equal(Hd, H2)


@pytest.mark.parametrize("tokens,n,chunks", [(4096, 512, None), (333, 1096, None), (640, 2304, [0, 200, 640]),
                                             (1500, 520, [0, 64, 1500])])
def test_accumulate_upper_is_the_full_sum_on_and_above_the_diagonal(tokens, n, chunks):
    """gptaq_accumulate_upper: H and the entries of dXXT with col >= row equal the full call's bit for bit (and so
    meet the oracle to the same bar); every entry below the diagonal is either untouched (zero) or the full call's
    value; and the factors prepared from it are the full ones, bit for bit (Eq. 17 reads nothing below the diagonal)."""
    Xb, Xtb = synth.make_activations(tokens, n, 9, "upper", 3, 20.0)
    H, A = O.accumulate(Xb, Xtb)
    Hf, Af = PU.gpu_accumulate(Xb, Xtb, chunks=chunks)
    Hu, Au = PU.gpu_accumulate(Xb, Xtb, chunks=chunks, upper=True)
    assert torch.equal(Hu, Hf)
    af, au = Af.cpu().numpy(), Au.cpu().numpy()
    assert np.array_equal(np.triu(au), np.triu(af))
    assert PU.rel_fro(np.triu(au), np.triu(A)) <= 1e-5
    low = np.tril(np.ones((n, n), bool), -1)
    assert np.all((au[low] == 0) | (au[low] == af[low]))
    assert np.count_nonzero(au[low]) < np.count_nonzero(af[low]) or n <= 128        # and it did leave work out
    damp = 0.01
    Hg, Ag = Hu.clone(), Au.clone()
    Ag[torch.tril(torch.ones((n, n), dtype=torch.bool, device="cuda"))] = float("nan")   # prepare must not even look there
    df, inf_f = PU.gpu_prepare(Hf, Af, damp)
    du, inf_u = PU.gpu_prepare(Hu, Au, damp)
    dg, inf_g = PU.gpu_prepare(Hg, Ag, damp)
    assert inf_f.cpu().tolist() == [0, 0] and inf_u.cpu().tolist() == [0, 0] and inf_g.cpu().tolist() == [0, 0]
    assert torch.equal(Hu, Hf) and torch.equal(Au, Af) and torch.equal(du, df)      # U, P, dead flags
    assert torch.equal(Hg, Hf) and torch.equal(Ag, Af)


def test_accumulate_staged_upper_equals_direct_upper_calls():
    from paper_2504_02692_amd import binding as B
    n, chunk, tokens = 392, 2048, 17 * 2048 + 77
    Xb, Xtb = synth.make_activations(tokens, n, 6, "staged-upper", 3, 20.0)
    X, Xt = PU.to_dev_bf16(Xb), PU.to_dev_bf16(Xtb)
    Hd = torch.zeros((n, n), device="cuda"); Ad = torch.zeros_like(Hd)
    ws = B.workspace(B.gptaq_accumulate_workspace_bytes(32768, n))
    pending = 0
    for t0 in range(0, tokens, chunk):
        pending = B.gptaq_accumulate_staged(X[t0:t0 + chunk], Xt[t0:t0 + chunk], Hd, Ad, ws, pending,
                                            flush=t0 + chunk >= tokens, upper=True)
    assert pending == 0
    H2, A2 = PU.gpu_accumulate(Xb, Xtb, chunks=[0, 32768, tokens], upper=True)
    assert torch.equal(Hd, H2) and torch.equal(Ad, A2)
    _, A = O.accumulate(Xb, Xtb)
    assert PU.rel_fro(np.triu(Ad.cpu().numpy()), np.triu(A)) <= 1e-5


def test_symmetrize(c1):
    from paper_2504_02692_amd import binding as B
    Hd, _ = PU.gpu_accumulate(c1["Xb"], c1["Xtb"])
    B.gptaq_symmetrize(Hd)
    h = Hd.cpu().numpy()
    assert np.array_equal(h, h.T)
    assert PU.rel_fro(h, c1["H"]) <= 1e-5


# --------------------------------------------------------------------- prepare
def run_prepare(H64, A64, damp):
    n = H64.shape[0]
    Hd = torch.from_numpy(np.triu(H64).astype(np.float32)).cuda()      # lower triangle deliberately absent
    Ad = torch.from_numpy(A64.astype(np.float32)).cuda()
    dead, info = PU.gpu_prepare(Hd, Ad, damp)
    return Hd, Ad, dead, info


def test_prepare_c1(c1):
    Ud, Pd, dead, info = run_prepare(c1["H"], c1["A"], c1["wl"].damp)
    assert info.cpu().tolist() == [0, 0]
    U, P = Ud.cpu().numpy(), Pd.cpu().numpy()
    assert np.all(np.tril(U, -1) == 0) and np.all(np.tril(P) == 0)
    eu, ep = PU.rel_fro(U, c1["U"]), PU.rel_fro(P, c1["P"])
    print(f"U rel. Frobenius {eu:.3e}  P rel. Frobenius {ep:.3e}")
    assert eu <= 1e-6 and ep <= 5e-5


# (sizes around the 64-column inner and 256-column outer blocks of the sweep: one partial tile, exactly one outer block,
#  an outer block of one / three inner blocks, several outer blocks with a ragged last one)
@pytest.mark.parametrize("n,k", [(8, 64), (100, 400), (200, 1000), (256, 1000), (320, 1300), (704, 2900), (1160, 2400)])
def test_prepare_ragged_sizes(n, k):
    Xb, Xtb = synth.make_activations(k, n, 5, "prep", 2, 20.0)
    H, A = O.accumulate(Xb, Xtb)
    U, P, _ = O.prepare(H, A, 0.01)
    Ud, Pd, dead, info = run_prepare(H, A, 0.01)
    assert info.cpu().tolist() == [0, 0]
    assert PU.rel_fro(Ud.cpu().numpy(), U) <= 1e-6
    assert PU.rel_fro(Pd.cpu().numpy(), P) <= 5e-5


def test_prepare_ill_conditioned_hessian():
    # The rank-256 products of the factor sweep run in 46-bit row-scaled fixed point.  A Hessian whose damped
    # condition number is ~1e7-1e8 (strongly correlated inputs, a few outlier channels with 1e4 times the energy,
    # damping 1e-6 of the mean diagonal instead of 1e-2) amplifies any error of the factorisation by that factor:
    # U must still reach the oracle to a few fp32 roundings.  n = 900 spans four outer blocks, the first one
    # partial.  (P is a product of fp32-grade GEMMs whose terms cancel at this conditioning; it is only held to
    # 1e-2 here, its bar on the paper's 1 % damping is in the tests above.)
    rng = np.random.default_rng(77)
    n, k = 900, 2400
    Z = rng.standard_normal((k, 60)) @ rng.standard_normal((60, n)) + 0.02 * rng.standard_normal((k, n))
    Z[:, rng.choice(n, 5, replace=False)] *= 100.0
    # both sides start from the same fp32 values (at this condition number the rounding of H to fp32 alone
    # moves U by 1e-3)
    H = (Z.T @ Z).astype(np.float32).astype(np.float64)
    H = np.triu(H) + np.triu(H, 1).T
    A = (0.05 * rng.standard_normal((k, n)).T @ Z).astype(np.float32).astype(np.float64)
    damp = 1e-6
    lam = damp * np.mean(np.diag(H))
    ev = np.linalg.eigvalsh(H + lam * np.eye(n))
    cond = ev[-1] / ev[0]
    U, P, _ = O.prepare(H, A, damp)
    Ud, Pd, dead, info = run_prepare(H, A, damp)
    assert info.cpu().tolist() == [0, 0]
    eu, ep = PU.rel_fro(Ud.cpu().numpy(), U), PU.rel_fro(Pd.cpu().numpy(), P)
    print(f"cond(H + lam I) = {cond:.2e}: U rel. Frobenius {eu:.3e}  P rel. Frobenius {ep:.3e}")
    assert cond > 1e6
    assert eu <= 1e-6 and ep <= 1e-2


def test_prepare_reports_dead_inputs_and_bad_pivots():
    Xb, Xtb = synth.make_activations(300, 96, 6, "dead", 2, 20.0)
    Xb = Xb.copy(); Xb[:, 17] = 0
    H, A = O.accumulate(Xb, Xtb)
    U, P, dead = O.prepare(H, A, 0.01)
    Ud, Pd, dd, info = run_prepare(H, A, 0.01)
    assert info.cpu().tolist() == [0, 1]
    assert dd.cpu().numpy().astype(bool).tolist() == dead.tolist()
    assert PU.rel_fro(Ud.cpu().numpy(), U) <= 1e-6 and PU.rel_fro(Pd.cpu().numpy(), P) <= 5e-5
    # an indefinite "Hessian" with no damping: the factorisation must flag a pivot, not hang or fault
    Hbad = np.eye(70); Hbad[40, 40] = -1.0
    _, _, _, info = run_prepare(Hbad, np.zeros((70, 70)), 0.0)
    assert info.cpu().tolist()[0] == 41
    # a NaN or an Inf that has crept into the sums is reported by the row it sits in (negative), not as a pivot
    Hn = H.copy(); Hn[5, 60] = np.nan
    _, _, _, info = run_prepare(Hn, A, 0.01)
    assert info.cpu().tolist()[0] == -(1 + 5)
    An = A.copy(); An[33, 60] = np.inf
    _, _, _, info = run_prepare(H, An, 0.01)
    assert info.cpu().tolist()[0] == -(1 + 33)
    # entries of dXXT on or below the diagonal are not read at all (Eq. 17 has no use for them)
    An = A.copy(); An[33, 2] = np.inf; An[7, 7] = np.nan
    U2, P2, _, info = run_prepare(H, An, 0.01)
    assert info.cpu().tolist() == [0, 1]
    assert torch.equal(U2, Ud) and torch.equal(P2, Pd)


# -------------------------------------------------------------------- quantize
def dev(a):
    return torch.from_numpy(np.asarray(a, np.float32).copy()).cuda()


def test_quantize_c1_from_oracle_factors(c1):
    """Column loop + trailing update in isolation: U, P come from the oracle (rounded to fp32)."""
    wl = c1["wl"]
    U32, P32 = c1["U"].astype(np.float32), c1["P"].astype(np.float32)
    got = PU.gpu_quantize(c1["W"], dev(U32), dev(P32), wl.bits, wl.group, wl.sym, wl.blocksize)
    PU.check_against_oracle(c1["W"], U32.astype(np.float64), P32.astype(np.float64), got, wl.bits, wl.group,
                            wl.sym, Xb=c1["Xb"], Xtb=c1["Xtb"], label="c1 loop only")


def test_whole_path_c1(c1):
    """accumulate -> prepare -> quantize, all on the GPU, against the all-fp64 oracle."""
    wl = c1["wl"]
    Hd, Ad = PU.gpu_accumulate(c1["Xb"], c1["Xtb"])
    dead, info = PU.gpu_prepare(Hd, Ad, wl.damp)
    assert info.cpu().tolist() == [0, 0]
    got = PU.gpu_quantize(c1["W"], Hd, Ad, wl.bits, wl.group, wl.sym, wl.blocksize)
    PU.check_against_oracle(c1["W"], c1["U"], c1["P"], got, wl.bits, wl.group, wl.sym,
                            Xb=c1["Xb"], Xtb=c1["Xtb"], label="c1 whole path")


@pytest.mark.parametrize("bits,group,sym,blocksize,m,n", [
    (4, 128, False, 128, 512, 512),      # W4 g128 (Llama-7B setting)
    (3, 128, False, 128, 300, 512),      # W3 g128, ragged rows
    (2, 64, False, 128, 512, 512),       # W2 g64
    (3, 128, True, 128, 512, 512),       # symmetric, 3-bit (weight-only setting)
    (4, 0, True, 128, 512, 512),         # per-channel symmetric
    (4, 32, False, 96, 200, 480),        # block not a power of two, ragged last block
    (4, 0, False, 50, 64, 130),          # tiny, ragged everything
    (8, 16, False, 16, 1100, 256),       # one row per wavefront, eight wavefronts per workgroup
    (4, 128, False, 128, 2500, 384),     # two rows per wavefront
    (4, 128, False, 128, 5100, 256),     # three
    (3, 0, False, 128, 7000, 128),       # four
    (4, 64, False, 64, 8200, 256),       # six
    (4, 0, False, 128, 16500, 128),      # eight
    (4, 128, False, 128, 19000, 128),    # ten
    (4, 128, False, 128, 22016, 256),    # twelve (gate and up of the Llama-2-7B block stacked)
    (4, 0, False, 128, 26000, 128),      # eight again, more than one round of workgroups
    (4, 8, False, 64, 300, 256),         # group sizes the super-block kernel does not take go block by block
    (3, 24, False, 96, 2100, 240),
    (4, 16, False, 128, 130, 512),       # group = one sub-block of the super-block kernel
    (5, 32, False, 128, 64, 384),
])
def test_quantize_variants(c1, bits, group, sym, blocksize, m, n):
    Hn = c1["H"][:n, :n]; An = c1["A"][:n, :n]
    U, P, _ = O.prepare(Hn, An, 0.01)
    U32, P32 = U.astype(np.float32), P.astype(np.float32)
    W = synth.make_weights(m, n, 3, f"v{m}x{n}")
    got = PU.gpu_quantize(W, dev(U32), dev(P32), bits, group, sym, blocksize)
    PU.check_against_oracle(W, U32.astype(np.float64), P32.astype(np.float64), got, bits, group, sym,
                            label=f"W{bits} g{group} sym{int(sym)} B{blocksize} {m}x{n}")


@pytest.mark.parametrize("bits,group,m,n,k", [
    (4, 0, 200, 2066, 2800),      # 1024 + 1024 + 18 columns: a last sub-block with two valid columns, unaligned rows
    (3, 128, 130, 1920, 2600),    # 1024 + 896
    (4, 64, 70, 2048, 2800),      # exactly two super-blocks
])
def test_quantize_several_super_blocks(bits, group, m, n, k):
    """Layers wider than one super-block: the update of the columns after a super-block goes through the GEMM."""
    Xb, Xtb = synth.make_activations(k, n, 21, "sbs", 3, 20.0)
    H, A = O.accumulate(Xb, Xtb)
    U, P, _ = O.prepare(H, A, 0.01)
    U32, P32 = U.astype(np.float32), P.astype(np.float32)
    W = synth.make_weights(m, n, 21, f"sbs{m}x{n}")
    got = PU.gpu_quantize(W, dev(U32), dev(P32), bits, group, False, 128)
    PU.check_against_oracle(W, U32.astype(np.float64), P32.astype(np.float64), got, bits, group, False,
                            label=f"W{bits} g{group} {m}x{n}")


def test_quantize_does_not_depend_on_blocksize(c1):
    """Step 4: lazy batching only re-associates sums, so every block size must reach the oracle's (unbatched)
    codes; what differs between block sizes is rounding noise, i.e. near-tie flips, which the parity bar bounds."""
    U32, P32 = c1["U"].astype(np.float32), c1["P"].astype(np.float32)
    U64, P64 = U32.astype(np.float64), P32.astype(np.float64)
    W = c1["W"][:256]
    # groups of 8 columns go through the block-by-block kernels, which do use the caller's block size
    outs = {}
    for B in (16, 64, 128):
        outs[B] = PU.gpu_quantize(W, dev(U32), dev(P32), 4, 8, False, B)
        PU.check_against_oracle(W, U64, P64, outs[B], 4, 8, False, label=f"g8 B{B}")
    again = PU.gpu_quantize(W, dev(U32), dev(P32), 4, 8, False, 128)
    assert np.array_equal(again["codes"], outs[128]["codes"]) and np.array_equal(again["What"], outs[128]["What"])
    # the super-block kernel (groups of 16) has its own blocking and ignores the caller's
    sb = PU.gpu_quantize(W, dev(U32), dev(P32), 4, 16, False, 128)
    PU.check_against_oracle(W, U64, P64, sb, 4, 16, False, label="g16 super-block")
    again = PU.gpu_quantize(W, dev(U32), dev(P32), 4, 16, False, 32)
    assert np.array_equal(again["codes"], sb["codes"]) and np.array_equal(again["What"], sb["What"])


def test_quantize_with_dead_input():
    Xb, Xtb = synth.make_activations(600, 128, 8, "deadq", 2, 20.0)
    Xb = Xb.copy(); Xb[:, 70] = 0
    W = synth.make_weights(96, 128, 8, "deadq")
    H, A = O.accumulate(Xb, Xtb)
    U, P, dead = O.prepare(H, A, 0.01)
    Hd, Ad = PU.gpu_accumulate(Xb, Xtb)
    dd, info = PU.gpu_prepare(Hd, Ad, 0.01)
    got = PU.gpu_quantize(W, Hd, Ad, 4, 0, False, 128, dead=dd)
    assert np.all(got["What"][:, 70] == 0)
    PU.check_against_oracle(W, U, P, got, 4, 0, False, dead=dead, Xb=Xb, Xtb=Xtb, label="dead input")


@pytest.mark.parametrize("terms,name", [(1, "GPTQ: E term only"), (2, "P term only"), (0, "round to nearest")])
def test_update_term_ablation(c1, terms, name):
    """Section 5.5: the two terms of the update applied individually (or not at all)."""
    wl = c1["wl"]
    U32, P32 = c1["U"].astype(np.float32), c1["P"].astype(np.float32)
    Pd = dev(P32) if terms & 2 else None
    got = PU.gpu_quantize(c1["W"], dev(U32), Pd, 4, 128, False, 128, terms=terms)
    PU.check_against_oracle(c1["W"], U32.astype(np.float64), P32.astype(np.float64), got, 4, 128, False,
                            Xb=c1["Xb"], Xtb=c1["Xtb"], label=name, terms=terms)


def test_act_order_path():
    """act_order: permutation from the Hessian diagonal, permuted solve, results scattered back."""
    from paper_2504_02692_amd import binding as B
    n, m, k, bits, group = 384, 200, 3000, 3, 128
    Xb, Xtb = synth.make_activations(k, n, 12, "ao", 3, 30.0)
    W = synth.make_weights(m, n, 12, "ao")
    Hd, Ad = PU.gpu_accumulate(Xb, Xtb)
    Hg = upper_to_full(Hd); Ag = Ad.cpu().numpy().astype(np.float64)
    perm = B.gptaq_act_order(Hd)
    ref = O.solve_with_act_order(W, Hg, Ag, 0.1, bits, group, True)     # ViT / weight-only setting: damp 10 %, symmetric
    assert np.array_equal(perm.cpu().numpy(), ref["perm"])
    B.gptaq_permute_hessian(Hd, Ad, perm, B.workspace(B.gptaq_permute_hessian_workspace_bytes(n)))
    torch.cuda.synchronize()
    hp = upper_to_full(Hd)
    assert np.array_equal(hp, Hg[np.ix_(ref["perm"], ref["perm"])])
    assert np.array_equal(Ad.cpu().numpy().astype(np.float64), Ag[np.ix_(ref["perm"], ref["perm"])])
    dead, info = PU.gpu_prepare(Hd, Ad, 0.1)
    Wp = B.gptaq_permute_columns_f32(torch.from_numpy(W).cuda(), perm)
    assert np.array_equal(Wp.cpu().numpy(), W[:, ref["perm"]])
    ws = B.workspace(B.gptaq_quantize_workspace_bytes(m, n))
    codes_p, scales, zeros = B.gptaq_quantize_layer(Wp, Hd, Ad, bits, group, True, 128, ws, dead=dead)
    What = B.gptaq_permute_columns_f32(Wp, perm, inverse=True)
    codes = B.gptaq_permute_columns_u8(codes_p, perm, inverse=True)
    torch.cuda.synchronize()
    # compare in permuted order with the near-tie protocol, and the scatter exactly
    got = dict(What=Wp.cpu().numpy(), codes=codes_p.cpu().numpy(), scales=scales.cpu().numpy(), zeros=zeros.cpu().numpy())
    PU.check_against_oracle(W[:, ref["perm"]], ref["U"], ref["P"], got, bits, group, True, label="act_order")
    assert np.array_equal(codes.cpu().numpy()[:, ref["perm"]], got["codes"])
    assert np.array_equal(What.cpu().numpy()[:, ref["perm"]], got["What"])


@pytest.mark.parametrize("tokens,n,chunks", [(3000, 384, None), (1500, 1096, [0, 700, 1500]), (900, 2304, None)])
def test_act_order_with_the_upper_triangle_accumulation(tokens, n, chunks):
    """The two-pass route: the diagonal of H first, the order from it, then H and the upper triangle of dXXT of the
    reordered inputs directly.  Against the one-pass route (full sums, gptaq_act_order, gptaq_permute_hessian): the same
    order, the same H and dXXT on and above the diagonal bit for bit, hence the same factors."""
    from paper_2504_02692_amd import binding as B
    Xb, Xtb = synth.make_activations(tokens, n, 21, "ao2", 3, 30.0)
    X, Xt = PU.to_dev_bf16(Xb), PU.to_dev_bf16(Xtb)
    bounds = chunks or [0, tokens]
    # one pass
    Hf, Af = PU.gpu_accumulate(Xb, Xtb, chunks=chunks)
    perm1 = B.gptaq_act_order(Hf)
    # two passes
    diag = torch.zeros(n, device="cuda")
    for t0, t1 in zip(bounds[:-1], bounds[1:]):
        B.gptaq_accumulate_diag(X[t0:t1], diag)
    H64, _ = O.accumulate(Xb, Xtb)
    assert PU.rel_fro(diag.cpu().numpy(), np.diag(H64)) <= 1e-6
    perm = B.gptaq_act_order(diag)
    # the order of the fp64 diagonal, up to swaps of inputs whose diagonals agree to fp32 rounding (the two routes sum
    # the diagonal in different orders); from here on both routes use this one
    p = perm.cpu().numpy()
    d64 = np.diag(H64)[p]
    assert sorted(p.tolist()) == list(range(n)) and np.all(d64[:-1] >= d64[1:] * (1 - 1e-5))
    assert np.mean(p == perm1.cpu().numpy()) > 0.99 and np.mean(p == O.act_order_permutation(H64)) > 0.99
    perm1 = perm
    inv = B.gptaq_invert_permutation(perm)
    assert np.array_equal(inv.cpu().numpy()[perm.cpu().numpy()], np.arange(n))
    Hp = torch.zeros((n, n), device="cuda"); Ap = torch.zeros_like(Hp)
    for t0, t1 in zip(bounds[:-1], bounds[1:]):
        B.gptaq_accumulate_upper_permuted(X[t0:t1], Xt[t0:t1], inv, Hp, Ap, B.workspace(B.gptaq_accumulate_workspace_bytes(t1 - t0, n)))
    B.gptaq_permute_hessian(Hf, Af, perm1, B.workspace(B.gptaq_permute_hessian_workspace_bytes(n)))
    torch.cuda.synchronize()
    assert np.array_equal(np.triu(Hp.cpu().numpy()), np.triu(Hf.cpu().numpy()))
    assert np.array_equal(np.triu(Ap.cpu().numpy()), np.triu(Af.cpu().numpy()))
    d1, i1 = PU.gpu_prepare(Hf, Af, 0.1)
    d2, i2 = PU.gpu_prepare(Hp, Ap, 0.1)
    assert i1.cpu().tolist() == [0, 0] and i2.cpu().tolist() == [0, 0]
    assert torch.equal(Hp, Hf) and torch.equal(Ap, Af)                   # U and P


@pytest.mark.parametrize("bits,group,sym", [(4, 128, False), (3, 64, True), (4, 0, False)])
def test_clip_range_search(c1, bits, group, sym):
    """Section 5.1's MSE-searched clipping range (grid 100, 80 steps) against the oracle."""
    U32, P32 = c1["U"].astype(np.float32), c1["P"].astype(np.float32)
    W = c1["W"][:300]
    got = PU.gpu_quantize(W, dev(U32), dev(P32), bits, group, sym, 128, mse=(100, 80))
    plain = PU.gpu_quantize(W, dev(U32), dev(P32), bits, group, sym, 128)
    assert np.mean(got["scales"] < plain["scales"]) > 0.5            # the search does clip
    PU.check_against_oracle(W, U32.astype(np.float64), P32.astype(np.float64), got, bits, group, sym,
                            Xb=c1["Xb"], Xtb=c1["Xtb"], label=f"clip search W{bits} g{group} sym{int(sym)}", mse=(100, 80))


def test_activation_quantiser_and_packing_on_gpu():
    from paper_2504_02692_amd import binding as B
    Xb, _ = synth.make_activations(999, 520, 9, "actq", 3, 20.0)
    for bits, clip in ((4, 0.9), (8, 1.0)):
        Y = B.gptaq_fake_quant_activations(PU.to_dev_bf16(Xb), bits, clip)
        got = Y.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        raw, t, _ = O.fake_quant_activations(Xb, bits, clip)
        ref, _, hints = O.fake_quant_activations(Xb, bits, clip, hint_bits=got, tau=PU.tau_for(bits))
        print(f"activation quantiser A{bits} clip {clip}: raw mismatch {(raw != got).mean():.2e}, near-tie hints {hints} of {got.size}")
        # fp64 oracle: bit-identical outputs apart from near-ties of x / scale (fp32 division in the library)
        assert hints <= PU.MAX_HINT_FRAC * got.size
        assert np.array_equal(ref, got)
        if hints == 0:
            assert np.array_equal(raw, got)
    rng = np.random.default_rng(2)
    for bits, n in ((2, 512), (3, 1000), (4, 130), (8, 77)):
        c = rng.integers(0, 2 ** bits, (300, n)).astype(np.uint8)
        p = B.gptaq_pack_codes(torch.from_numpy(c).cuda(), bits)
        assert np.array_equal(p.cpu().numpy().view(np.uint32), O.pack_codes(c, bits))


def test_mfma_peak_measurement_is_sane():
    # the measured ceiling bench.py quotes beside the vendor peak: a finite loop of MFMAs, a plausible rate and clock
    from paper_2504_02692_amd import binding as B
    tf1, ghz1 = B.gptaq_measure_mfma_peak(False, 5)
    tf2, ghz2 = B.gptaq_measure_mfma_peak(True, 5)
    print(f"pure MFMA loop: all-ones {tf1:.0f} TFLOP/s at {ghz1:.2f} GHz, random operands {tf2:.0f} TFLOP/s at {ghz2:.2f} GHz")
    assert 500.0 < tf2 <= tf1 * 1.05 < 2700.0
    assert 1.0 < ghz2 < 2.6 and 1.0 < ghz1 < 2.6


def test_stacked_layers_equal_separate_calls(c1):
    """Layers that share an input share U and P and their rows are independent (Step 1): quantising them as one
    stacked matrix, as bench.py does for q/k/v and gate/up, gives bit for bit what separate calls give."""
    wl = c1["wl"]
    U32, P32 = dev(c1["U"].astype(np.float32)), dev(c1["P"].astype(np.float32))
    W1, W2 = c1["W"][:300], synth.make_weights(212, 512, 3, "second")
    one = PU.gpu_quantize(np.concatenate([W1, W2]), U32, P32, 4, 128, False, 128)
    a, b = PU.gpu_quantize(W1, U32, P32, 4, 128, False, 128), PU.gpu_quantize(W2, U32, P32, 4, 128, False, 128)
    for key in ("codes", "scales", "zeros", "What"):
        assert np.array_equal(one[key], np.concatenate([a[key], b[key]])), key


def test_tall_matrix_in_two_row_halves_equals_separate_calls():
    """A matrix of 10240 rows or more is quantised as two row halves on two streams (rows are independent, Step 1).
    The result must be bit for bit what two separate calls on those halves give (each short enough to take the
    one-stream route), over several super-blocks and with a ragged last super-block."""
    n, m, k = 2100, 10500, 2600
    Xb, Xtb = synth.make_activations(k, n, 11, "tall", 2, 20.0)
    H, A = O.accumulate(Xb, Xtb)
    U, P, _ = O.prepare(H, A, 0.01)
    U32, P32 = dev(U.astype(np.float32)), dev(P.astype(np.float32))
    W = synth.make_weights(m, n, 12, "tall")
    one = PU.gpu_quantize(W, U32, P32, 4, 0, False, 128)
    half = -(-((m + 1) // 2) // 256) * 256                     # where the library splits
    a, b = PU.gpu_quantize(W[:half], U32, P32, 4, 0, False, 128), PU.gpu_quantize(W[half:], U32, P32, 4, 0, False, 128)
    for key in ("codes", "scales", "zeros", "What"):
        assert np.array_equal(one[key], np.concatenate([a[key], b[key]])), key
    again = PU.gpu_quantize(W, U32, P32, 4, 0, False, 128)
    for key in ("codes", "scales", "zeros", "What"):
        assert np.array_equal(one[key], again[key]), key


def test_bench_line_on_the_small_workload():
    """bench.py end to end on the 512 x 512 layer: one JSON line with the fields the contract names."""
    import json, os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "c1", "--steps", "2", "--warmup", "1",
                          "--no-cpu-baseline"], capture_output=True, text=True, timeout=110, cwd=root)
    assert out.returncode == 0, out.stderr[-2000:]
    line = json.loads(out.stdout.strip().splitlines()[-1])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in line, key
    assert line["n_gpus"] == 1 and line["steps"] == 2 and line["higher_is_better"] is False and line["value"] > 0
    r = line["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9 and 0 < r["frac"] < 1
    assert "workload" in line["config"] and "col >= row" in line["config"]["workload"]
    forms = line["accumulate_ms_per_step_by_form"]
    assert forms["timed_path_uses"] == "dxxt_upper" and forms["dxxt_upper"] > 0 and forms["dxxt_full"] > 0
    # the other form of the accumulation on request
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "c1", "--steps", "1", "--warmup", "1",
                          "--no-cpu-baseline", "--full-dxxt"], capture_output=True, text=True, timeout=110, cwd=root)
    assert out.returncode == 0, out.stderr[-2000:]
    full = json.loads(out.stdout.strip().splitlines()[-1])
    assert full["accumulate_ms_per_step_by_form"]["timed_path_uses"] == "dxxt_full" and "all entries" in full["config"]["workload"]
    # more than one GPU is refused with a message
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=60, cwd=root)
    assert out.returncode != 0 and "one GPU" in out.stderr


def test_path_is_bit_reproducible(c1):
    """No atomics and a fixed summation order everywhere: two runs of the whole path give identical bits (the sweep of
    gptaq_prepare runs on two streams; a missing dependency between them would show up here as a difference)."""
    wl = c1["wl"]
    runs = []
    for rep in range(3):
        Hd, Ad = PU.gpu_accumulate(c1["Xb"], c1["Xtb"], chunks=[0, 1500, 4096])
        h0, a0 = Hd.clone(), Ad.clone()
        dead, info = PU.gpu_prepare(Hd, Ad, wl.damp)
        got = PU.gpu_quantize(c1["W"], Hd, Ad, wl.bits, 128, wl.sym, wl.blocksize)
        runs.append((h0.cpu().numpy(), a0.cpu().numpy(), Hd.cpu().numpy(), Ad.cpu().numpy(), got["codes"], got["What"],
                     got["scales"], got["zeros"]))
    for other in runs[1:]:
        for x, y in zip(runs[0], other):
            assert np.array_equal(x, y)
    # and at a size whose sweep has several outer blocks on both streams
    rng = np.random.default_rng(9)
    Z = rng.standard_normal((3000, 1160))
    H, A = Z.T @ Z, 0.05 * rng.standard_normal((3000, 1160)).T @ Z
    outs = []
    for rep in range(3):
        Ud, Pd, dead, info = run_prepare(H, A, 0.01)
        outs.append((Ud.cpu().numpy(), Pd.cpu().numpy()))
    for u, p in outs[1:]:
        assert np.array_equal(u, outs[0][0]) and np.array_equal(p, outs[0][1])

"""Pins of the fp64 oracle against what the paper and plain mathematics fix.

No test here calls the HIP library.  Each pin states which passage it checks and is
chosen so that a plausible slip in the oracle (a transposed dXXT, a wrong sign, a
dropped term, an off-by-one in the triangular mask, the wrong W column in the P term)
makes it fail; test_planted_mistakes_are_caught shows that for a few such slips.
"""
import os

import numpy as np
import pytest

from oracle import gptaq_oracle as O
from paper_2504_02692_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tiny_problem(n=24, m=10, k=160, seed=1, noise=0.05, outliers=2):
    Xb, Xtb = synth.make_activations(k, n, seed, "tiny", outliers, 20.0, noise)
    W = synth.make_weights(m, n, seed, "tiny").astype(np.float64)
    return W, Xb, Xtb


def solved(n=24, m=10, k=160, seed=1, damp=0.01):
    W, Xb, Xtb = tiny_problem(n, m, k, seed)
    H, A = O.accumulate(Xb, Xtb)
    H_lam, A_f, dead, lam = O.dampen(H, A, damp)
    L = O.inverse_cholesky(H_lam)
    P = O.correction_matrix(A_f, L)
    return dict(W=W, Xb=Xb, Xtb=Xtb, H=H, A=A, H_lam=H_lam, lam=lam, L=L, U=L.T.copy(), P=P)


# ------------------------------------------------------------------ quantiser
def test_quantiser_hand_worked_examples():
    rows = [l for l in open(os.path.join(GOLD, "quantiser_example.txt")) if l[0] != "#" and l.strip()]
    assert len(rows) == 3
    for line in rows:
        head, w, sz, q, what = [p.split() for p in line.split("|")]
        bits, sym = int(head[1]), bool(int(head[2]))
        w = np.array(w, float)[None, :]
        scale, zero = O.quant_params(w.min(1), w.max(1), bits, sym)
        assert scale[0] == pytest.approx(float(sz[0]), rel=1e-7)
        assert zero[0] == float(sz[1])
        for j in range(3):
            c, wh, _ = O.quantize_column(w[:, j], scale, zero, bits)
            assert c[0] == float(q[j])
            assert wh[0] == pytest.approx(float(what[j]), rel=1e-6, abs=1e-9)


def test_quantiser_grid_properties():
    rng = np.random.default_rng(0)
    w = rng.standard_normal((50, 64)) * 0.02
    for bits in (2, 3, 4, 8):
        for sym in (False, True):
            s, z = O.quant_params(w.min(1), w.max(1), bits, sym)
            assert np.all(s == s.astype(np.float32))            # fp32-representable scale
            assert np.all(z == np.rint(z)) and np.all((z >= 0) & (z <= 2 ** bits))
            for j in range(w.shape[1]):
                c, wh, t = O.quantize_column(w[:, j], s, z, bits)
                assert np.all((c >= 0) & (c <= 2 ** bits - 1))
                inside = (np.rint(t) + z >= 0) & (np.rint(t) + z <= 2 ** bits - 1)
                assert np.all(np.abs(wh - w[:, j])[inside] <= 0.5 * s[inside] * (1 + 1e-12))
    # all-zero row: range (-1, 1)
    s, z = O.quant_params(np.zeros(1), np.zeros(1), 4, False)
    assert s[0] == pytest.approx(2.0 / 15.0, rel=1e-6) and z[0] in (7.0, 8.0)   # 1/scale = 7.5: a tie


# ---------------------------------------------------- Algorithm 1 line 2: H, dXXT
def test_accumulate_orientation_by_loops():
    Xb, Xtb = synth.make_activations(7, 4, 3, "loops", 1, 20.0)
    X = synth.bf16_bits_to_f32(Xb).astype(float)
    Xt = synth.bf16_bits_to_f32(Xtb).astype(float)
    H, A = O.accumulate(Xb, Xtb)
    for q in range(4):
        for j in range(4):
            h = sum(X[t, q] * X[t, j] for t in range(7))
            a = sum((Xt[t, q] - X[t, q]) * X[t, j] for t in range(7))   # dX_{q,:} X^T, Eq. 16
            assert H[q, j] == pytest.approx(h, rel=1e-13, abs=1e-13)
            assert A[q, j] == pytest.approx(a, rel=1e-13, abs=1e-13)


def test_dampen_is_one_percent_of_mean_diagonal():
    s = solved()
    assert s["lam"] == pytest.approx(0.01 * np.trace(s["H"]) / s["H"].shape[0], rel=1e-14)
    assert np.allclose(s["H_lam"] - s["H"], s["lam"] * np.eye(s["H"].shape[0]), rtol=0, atol=1e-9)


# --------------------------------------------------------------- Lemma 4.1, Step 3
def test_lemma_4_1_trailing_factor_is_reduced_inverse():
    s = solved()
    L, H_lam = s["L"], s["H_lam"]
    n = L.shape[0]
    assert np.allclose(np.tril(L), L) and np.all(np.diag(L) > 0)
    assert np.allclose(L @ L.T @ H_lam, np.eye(n), atol=1e-9)
    for q in range(n):
        sub = np.linalg.inv(H_lam[q:, q:])          # (X_{-q:} X_{-q:}^T + lam I)^-1
        assert np.allclose(L[q:, q:] @ L[q:, q:].T, sub, rtol=1e-8, atol=1e-12)


def test_gaussian_elimination_equals_reduced_inverse():
    # Eq. 3: eliminating row/column q of H^-1 gives the inverse of H without input q
    s = solved(n=12)
    Hinv = np.linalg.inv(s["H_lam"])
    q = 0
    ge = Hinv - np.outer(Hinv[:, q], Hinv[q, :]) / Hinv[q, q]
    assert np.allclose(ge[1:, 1:], np.linalg.inv(s["H_lam"][1:, 1:]), rtol=1e-8, atol=1e-12)


# -------------------------------------------------------- Theorem 4.2 and Eq. 16
def test_theorem_4_2_fused_P_equals_per_row_form():
    s = solved()
    P, A, L, H_lam = s["P"], s["A"], s["L"], s["H_lam"]
    n = P.shape[0]
    assert np.all(np.tril(P) == 0.0)                 # P_ij = 0 for i >= j (proof of Thm 4.2)
    for q in range(n - 1):
        Lq = L[q + 1:, q + 1:]
        row = (A[q, :][None, q + 1:] @ Lq) @ Lq.T    # Eq. 16 on the columns after q
        assert np.allclose(P[q, q + 1:], row[0], rtol=1e-9, atol=1e-13)
        # the same row without any factor: dX_q X^T_{q+1:} (H_lam)_{q+1:,q+1:}^-1
        row2 = A[q, q + 1:] @ np.linalg.inv(H_lam[q + 1:, q + 1:])
        assert np.allclose(P[q, q + 1:], row2, rtol=1e-8, atol=1e-13)


def test_P_reads_only_the_strictly_upper_triangle_of_dXXT():
    """Eq. 16: row q of P is built from the columns after q of row q of dXXT (and Eq. 17 is the same rows stacked), so
    the diagonal and the lower triangle of dXXT never reach P, and through it never reach a quantised weight.  The
    library's upper-triangle accumulation rests on this; planted here as garbage below the diagonal."""
    s = solved()
    A, L, W = s["A"], s["L"], s["W"]
    n = A.shape[0]
    rng = np.random.default_rng(0)
    low = np.tril(np.ones((n, n), bool))
    for junk in (np.zeros((n, n)), 1e3 * np.abs(A).max() * rng.standard_normal((n, n))):
        A2 = np.where(low, junk, A)
        P2 = O.correction_matrix(A2, L)
        assert np.allclose(P2, s["P"], rtol=1e-12, atol=1e-300)
        U2, P3, _ = O.prepare(s["H"], np.where(low, junk, A), 0.01)
        r0 = O.quantize_layer(W, s["U"], s["P"], 4, group=8)
        r1 = O.quantize_layer(W, U2, P3, 4, group=8)
        assert np.array_equal(r0["codes"], r1["codes"]) and np.allclose(r0["What"], r1["What"], rtol=1e-12)
    # while an entry above the diagonal does
    A3 = A.copy(); A3[2, 5] *= 1.5
    assert not np.allclose(O.correction_matrix(A3, L)[2], s["P"][2], rtol=1e-6)


def test_rows_of_P_are_ridge_regressions():
    """Row q of P regresses dX_q on the inputs after q (objective of Eq. 14 with the
    weight factored out); solved here by a library least-squares on the tokens, with
    the damping as sqrt(lam) * I extra 'tokens'.  Pins sign and orientation of dXXT."""
    s = solved()
    X = O.bf16_bits_to_f64(s["Xb"]).T       # n x k, the paper's X
    dX = O.bf16_bits_to_f64(s["Xtb"]).T - X
    n, k = X.shape
    lam = s["lam"]
    for q in (0, 3, n - 2):
        Xa = np.hstack([X[q + 1:], np.sqrt(lam) * np.eye(n)[q + 1:]])     # (n-q-1) x (k+n)
        ya = np.concatenate([dX[q], np.zeros(n)])
        p, *_ = np.linalg.lstsq(Xa.T, ya, rcond=None)
        assert np.allclose(s["P"][q, q + 1:], p, rtol=1e-7, atol=1e-12)


# ------------------------------------------------------- the column loop itself
@pytest.mark.parametrize("bits,group,sym", [(4, 0, False), (3, 8, False), (3, 8, True), (2, 0, True)])
def test_reduces_to_gptq_when_dX_is_zero(bits, group, sym):
    """With X~ = X the P term vanishes and Algorithm 1 is GPTQ; compare with the
    explicit-inverse OBS update and Gaussian elimination of Eq. 2-3."""
    W, Xb, _ = tiny_problem()
    H, A = O.accumulate(Xb, Xb)
    assert np.all(A == 0.0)
    U, P, dead = O.prepare(H, A, 0.01)
    assert np.all(P == 0.0)
    ours = O.quantize_layer(W, U, P, bits, group, sym)
    H_lam = O.dampen(H, A, 0.01)[0]
    ref = O.gptq_explicit_inverse(W, H_lam, bits, group, sym)
    assert np.array_equal(ours["codes"], ref["codes"])
    assert np.allclose(ours["What"], ref["What"], rtol=0, atol=1e-12)


@pytest.mark.parametrize("bits,group,sym", [(4, 0, False), (3, 8, False), (2, 12, False)])
def test_equals_eq15_with_explicit_inverses(bits, group, sym):
    s = solved()
    ours = O.quantize_layer(s["W"], s["U"], s["P"], bits, group, sym)
    ref = O.gptaq_explicit_inverse(s["W"], s["H_lam"], s["A"], bits, group, sym)
    assert np.array_equal(ours["codes"], ref["codes"])
    assert np.allclose(ours["What"], ref["What"], rtol=0, atol=1e-12)


def test_each_column_update_solves_the_constrained_least_squares():
    """Eq. 14: at column q, with the first q columns fixed and column q forced to its
    quantised value, the change of the later columns minimises
    || dW_{q:} X_{q:} - W_{:,q} dX_q ||^2 (+ damping).  Solve that by lstsq on tokens
    for every q and follow the whole trajectory; no H^-1, L or P involved."""
    n, m, k = 10, 3, 60
    W, Xb, Xtb = tiny_problem(n, m, k, seed=5)
    H, A = O.accumulate(Xb, Xtb)
    H_lam, A_f, dead, lam = O.dampen(H, A, 0.01)
    U, P, _ = O.prepare(H, A, 0.01)
    bits = 3
    ours = O.quantize_layer(W, U, P, bits)
    X = O.bf16_bits_to_f64(Xb).T
    dX = O.bf16_bits_to_f64(Xtb).T - X
    Xa = np.hstack([X, np.sqrt(lam) * np.eye(n)])
    dXa = np.hstack([dX, np.zeros((n, n))])
    Wc = W.copy()
    scale, zero = O.quant_params(Wc.min(1), Wc.max(1), bits, False)
    for q in range(n):
        w_q = Wc[:, q].copy()
        c, w_hat, _ = O.quantize_column(w_q, scale, zero, bits)
        assert np.array_equal(c.astype(np.uint8), ours["codes"][:, q])
        if q + 1 < n:
            # target for the free columns: w_q dX_q - (w_hat - w_q) X_q
            rhs = np.outer(w_q, dXa[q]) - np.outer(w_hat - w_q, Xa[q])
            d, *_ = np.linalg.lstsq(Xa[q + 1:].T, rhs.T, rcond=None)
            Wc[:, q + 1:] += d.T
        Wc[:, q] = w_hat
    assert np.allclose(Wc, ours["What"], rtol=0, atol=1e-10)


def test_identity_quantiser_closed_form():
    """Without quantisation error E = 0 and the recurrence w^_j = w_j + sum_{i<j} w^_i P_ij
    has the closed form What = W (I - P)^-1, P strictly upper (nilpotent)."""
    s = solved()
    out = O.quantize_layer(s["W"], s["U"], s["P"], 4, identity_quantizer=True)
    n = s["P"].shape[0]
    assert np.allclose(out["What"], s["W"] @ np.linalg.inv(np.eye(n) - s["P"]), rtol=1e-10, atol=1e-14)
    # and without the P term nothing moves at all (round-to-nearest limit, Section 5.5)
    out0 = O.quantize_layer(s["W"], s["U"], s["P"], 4, identity_quantizer=True, use_P=False)
    assert np.array_equal(out0["What"], s["W"])


def test_unconstrained_update_is_the_ridge_minimiser():
    """Appendix A.1 with the multiplier set to zero: dW = R X^T H^-1, i.e.
    W + W dXXT H_lam^-1 minimises ||W' X - W X~||^2 + lam ||W' - W||^2.  Checked by
    lstsq on tokens; pins accumulate() and dampen() together."""
    s = solved(n=16, m=5, k=200)
    X = O.bf16_bits_to_f64(s["Xb"]).T
    Xt = O.bf16_bits_to_f64(s["Xtb"]).T
    n = X.shape[0]
    Xa = np.hstack([X, np.sqrt(s["lam"]) * np.eye(n)])
    target = np.hstack([s["W"] @ (Xt - X), np.zeros((s["W"].shape[0], n))])
    dW, *_ = np.linalg.lstsq(Xa.T, target.T, rcond=None)
    assert np.allclose(s["W"] @ s["A"] @ np.linalg.inv(s["H_lam"]), dW.T, rtol=1e-7, atol=1e-12)


def test_first_column_is_round_to_nearest():
    s = solved()
    out = O.quantize_layer(s["W"], s["U"], s["P"], 4)
    W = s["W"]
    scale, zero = O.quant_params(W.min(1), W.max(1), 4, False)
    c, wh, _ = O.quantize_column(W[:, 0], scale, zero, 4)
    assert np.array_equal(out["codes"][:, 0], c.astype(np.uint8))
    # no update at all -> plain RTN of every column
    rtn = O.quantize_layer(W, s["U"], s["P"], 4, use_E=False, use_P=False)
    for j in range(W.shape[1]):
        c, wh, _ = O.quantize_column(W[:, j], scale, zero, 4)
        assert np.array_equal(rtn["codes"][:, j], c.astype(np.uint8))
    assert np.allclose(out["What"], out["scales"][:, :1] * (out["codes"] - out["zeros"][:, :1]))


# ------------------------------------------------------------ Step 4, invariances
@pytest.mark.parametrize("group,sym", [(0, False), (8, False), (8, True)])
def test_lazy_batching_does_not_change_the_result(group, sym):
    s = solved(n=48, m=12, k=300)
    base = O.quantize_layer(s["W"], s["U"], s["P"], 3, group, sym)
    for B in (8, 16, 48, 128) + ((1,) if group <= 0 else ()):
        blk = O.quantize_layer_blocked(s["W"], s["U"], s["P"], 3, group, sym, blocksize=B)
        assert np.array_equal(blk["codes"], base["codes"]), B
        assert np.allclose(blk["What"], base["What"], rtol=0, atol=1e-12)
        assert np.array_equal(blk["zeros"], base["zeros"])


def test_rows_are_independent_and_common_scale_cancels():
    s = solved()
    full = O.quantize_layer(s["W"], s["U"], s["P"], 4)
    part = O.quantize_layer(s["W"][3:7], s["U"], s["P"], 4)
    assert np.array_equal(full["codes"][3:7], part["codes"])
    U2, P2, _ = O.prepare(7.0 * s["H"], 7.0 * s["A"], 0.01)
    scaled = O.quantize_layer(s["W"], U2, P2, 4)
    assert np.array_equal(scaled["codes"], full["codes"])
    assert np.allclose(P2, s["P"], rtol=1e-9, atol=1e-14)


def test_dead_input_equals_problem_without_that_input():
    n, m, k = 12, 4, 80
    W, Xb, Xtb = tiny_problem(n, m, k, seed=9)
    Xb = Xb.copy()
    Xb[:, 5] = 0                                  # input 5 never fires in the quantised model
    H, A = O.accumulate(Xb, Xtb)
    U, P, dead = O.prepare(H, A, 0.01)
    assert dead.tolist() == [i == 5 for i in range(n)]
    out = O.quantize_layer(W, U, P, 4, dead=dead)
    keep = np.arange(n) != 5
    Wr = W[:, keep]
    Hr, Ar = O.accumulate(Xb[:, keep], Xtb[:, keep])
    # same damping constant as the full problem (mean over n entries, dead diagonal = 1)
    lam = 0.01 * (np.trace(Hr) + 1.0) / n
    Hl = Hr + lam * np.eye(n - 1)
    Lr = O.inverse_cholesky(Hl)
    Pr = O.correction_matrix(Ar, Lr)
    # per-channel range of the full row includes the zeroed column (0 is always inside)
    red = O.quantize_layer(Wr, Lr.T, Pr, 4)
    assert np.array_equal(out["codes"][:, keep], red["codes"])
    assert np.all(out["What"][:, 5] == 0.0)


def test_moment_form_of_the_objective():
    s = solved()
    out = O.quantize_layer(s["W"], s["U"], s["P"], 3)
    X = O.bf16_bits_to_f64(s["Xb"])
    dX = O.bf16_bits_to_f64(s["Xtb"]) - X
    direct = O.layer_output_error(s["W"], out["What"], s["Xb"], s["Xtb"])
    mom = O.layer_output_error_from_moments(s["W"], out["What"], s["H"], s["A"], dX.T @ dX)
    assert mom == pytest.approx(direct, rel=1e-9)


def test_loss_ordering_on_the_synthetic_recipe():
    """Direction of Table 5 only: both terms < first term only (GPTQ) < no update (RTN)."""
    W, Xb, Xtb = tiny_problem(n=64, m=48, k=1024, seed=2)
    H, A = O.accumulate(Xb, Xtb)
    U, P, _ = O.prepare(H, A, 0.01)
    err = {}
    for name, (e, p) in dict(gptaq=(True, True), gptq=(True, False), rtn=(False, False)).items():
        out = O.quantize_layer(W, U, P, 3, use_E=e, use_P=p)
        err[name] = O.layer_output_error(W, out["What"], Xb, Xtb)
    assert err["gptaq"] < err["gptq"] < err["rtn"]


def test_upper_factor_route_equals_literal_route():
    """U = L^T is also the inverse of the upper factor V of H_lam = V V^T (unique for a
    positive diagonal); the HIP library factors that way, the oracle does not."""
    s = solved()
    H_lam = s["H_lam"]
    J = np.eye(H_lam.shape[0])[::-1]
    V = J @ np.linalg.cholesky(J @ H_lam @ J) @ J
    assert np.allclose(np.triu(V), V) and np.allclose(V @ V.T, H_lam)
    assert np.allclose(np.linalg.inv(V), s["U"], rtol=1e-9, atol=1e-13)


def test_near_tie_hints_only_act_inside_the_window():
    s = solved()
    base = O.quantize_layer(s["W"], s["U"], s["P"], 4)
    flipped = base["codes"].astype(np.int64) + 1            # a hint that disagrees everywhere
    out = O.quantize_layer(s["W"], s["U"], s["P"], 4, hint_codes=flipped, tau=0.0)
    assert out["hints_used"] == 0 and np.array_equal(out["codes"], base["codes"])
    out = O.quantize_layer(s["W"], s["U"], s["P"], 4, hint_codes=base["codes"], tau=0.5)
    assert out["hints_used"] == 0 and np.array_equal(out["codes"], base["codes"])


# ------------------------------------------------- the pins do catch planted slips
def test_planted_mistakes_are_caught():
    s = solved()
    W, U, P, A, L, H_lam = s["W"], s["U"], s["P"], s["A"], s["L"], s["H_lam"]
    n = P.shape[0]

    # (a) slips in P are seen by the factor-free row formula of Eq. 16
    def p_ok(Pc):
        return all(np.allclose(Pc[q, q + 1:], A[q, q + 1:] @ np.linalg.inv(H_lam[q + 1:, q + 1:]),
                               rtol=1e-8, atol=1e-13) for q in range(n - 1)) and np.all(np.tril(Pc) == 0)

    assert p_ok(P)
    assert not p_ok(O.correction_matrix(A.T, L))              # transposed dXXT
    assert not p_ok(-P)                                       # sign
    assert not p_ok(np.triu(A @ L, 0) @ L.T)                  # mask keeps the diagonal
    assert not p_ok(np.triu(A @ L, 2) @ L.T)                  # mask one too strict
    assert not p_ok(np.triu(A @ L.T, 1) @ L)                  # L and L^T swapped

    # (b) slips in the loop are seen by the closed form of the identity-quantiser run
    closed = W @ np.linalg.inv(np.eye(n) - P)

    def loop_ok(**kw):
        out = O.quantize_layer(W, kw.pop("U", U), kw.pop("P", P), 4, identity_quantizer=True, **kw)
        return np.allclose(out["What"], closed, rtol=1e-10, atol=1e-14)

    assert loop_ok()
    assert not loop_ok(use_P=False)                           # dropped term
    assert not loop_ok(P=P.T)                                 # column instead of row of P
    # (c) and by Eq. 15 with explicit inverses when real quantisation error is fed back
    ref = O.gptaq_explicit_inverse(W, H_lam, A, 3)
    assert np.array_equal(O.quantize_layer(W, U, P, 3)["codes"], ref["codes"])
    assert not np.array_equal(O.quantize_layer(W, U, P, 3, use_E=False)["codes"], ref["codes"])
    assert not np.array_equal(O.quantize_layer(W, L, P, 3)["codes"], ref["codes"])   # L for L^T


def test_act_order_is_the_same_solve_on_permuted_inputs():
    """act_order only reorders the inputs: solving with the permutation equals relabelling the neurons
    of X, X~ and the columns of W beforehand, and the order is by decreasing diagonal, ties by index."""
    W, Xb, Xtb = tiny_problem(n=24, m=6, k=200, seed=4)
    H, A = O.accumulate(Xb, Xtb)
    perm = O.act_order_permutation(H)
    d = np.diag(H)[perm]
    assert np.all(d[:-1] >= d[1:]) and sorted(perm.tolist()) == list(range(24))
    assert O.act_order_permutation(np.diag([3.0, 5.0, 3.0, 7.0])).tolist() == [3, 1, 0, 2]
    out = O.solve_with_act_order(W, H, A, 0.01, 3, group=8)
    Hp, Ap = O.accumulate(Xb[:, perm], Xtb[:, perm])          # relabelled neurons
    U, P, _ = O.prepare(Hp, Ap, 0.01)
    ref = O.quantize_layer(W[:, perm], U, P, 3, 8)
    assert np.array_equal(out["codes"][:, perm], ref["codes"])
    assert np.allclose(out["What"][:, perm], ref["What"], rtol=0, atol=1e-12)


def test_clip_search_properties():
    """The clip-range search: never worse than min-max, exact grids keep p = 1, an outlier row gets
    clipped, power-of-two scaling of the weights scales the result, and the argmin is a true argmin."""
    rng = np.random.default_rng(1)
    bits, grid, steps = 3, 100, 80
    w = rng.standard_normal((40, 64)) * 0.02
    w[0] = 0.3 * rng.uniform(-1, 1, 64); w[0, 7] = 1.0              # a dense body and one outlier
    s0, z0 = O.quant_params(w.min(1), w.max(1), bits, False)
    s1, z1, _ = O.quant_params_mse(w, bits, False, grid, steps)

    def sse(s, z):
        q = np.clip(np.rint(w / s[:, None]) + z[:, None], 0, 2 ** bits - 1)
        return np.sum((s[:, None] * (q - z[:, None]) - w) ** 2, axis=1)

    e0, e1 = sse(s0, z0), sse(s1, z1)
    assert np.all(e1 <= e0 * (1 + 1e-12)) and np.array_equal(z0, z1)
    assert s1[0] < 0.95 * s0[0] and e1[0] < e0[0]                # clipping the outlier pays for the body
    for r in (0, 5, 11):                                              # brute force over the candidate list
        cand = [np.float64(np.float32((1 - i / grid) * (max(w[r].max(), 0) - min(w[r].min(), 0)) / 7)) for i in range(steps)]
        errs = [sse(np.full(40, c), z1)[r] for c in cand]
        assert s1[r] == cand[int(np.argmin(errs))]
    grid_row = (np.arange(8) - 3)[None, :] * 0.25                     # already on a 3-bit grid: error 0 at p = 1
    sg, zg, _ = O.quant_params_mse(grid_row, bits, False, grid, steps)
    assert sg[0] == np.float32(0.25) and zg[0] == 3
    s4, _, _ = O.quant_params_mse(4.0 * w, bits, False, grid, steps)
    assert np.array_equal(s4, 4.0 * s1)
    out = O.quantize_layer(w[:, :32], np.eye(32), np.zeros((32, 32)), bits, 16, False, mse_grid=grid, mse_steps=steps)
    assert np.array_equal(out["scales"][:, 0], O.quant_params_mse(w[:, :16], bits, False, grid, steps)[0])


def test_scale_hints_cannot_hide_a_wrong_candidate_list(monkeypatch):
    """The parity protocol lets the oracle take the library's scale when it is one of the oracle's own candidates with
    an error within 1e-4 of the best (fp32 and fp64 error sums can order two near-equal candidates differently).
    A planted mistake must not slip through that door: an implementation whose candidate list is off by one
    (p = 1 - (i + 1) / grid) is rejected, and so is one that searches the right list with the wrong exponent."""
    from tests import parity_util as PU
    rng = np.random.default_rng(4)
    m, n, bits, group, grid, steps = 48, 64, 4, 32, 100, 80
    W = 0.02 * rng.standard_normal((m, n))
    X = rng.standard_normal((400, n))
    H = X.T @ X
    A = (0.05 * rng.standard_normal((400, n))).T @ X
    U, P, _ = O.prepare(H, A, 0.01)
    good = O.quantize_layer(W, U, P, bits, group, False, mse_grid=grid, mse_steps=steps)
    as_library = lambda r: dict(codes=r["codes"], scales=r["scales"].astype(np.float32), zeros=r["zeros"].astype(np.float32),
                                What=r["What"].astype(np.float32))
    PU.check_against_oracle(W, U, P, as_library(good), bits, group, False, label="unchanged oracle", mse=(grid, steps))
    real = O.quant_params_mse

    def off_by_one(block, bits_, sym, grid_, steps_, hint_scales=None, rel_tol=0.0):
        # candidates p = 1 - (i + 1) / grid: every scale of this list but the last is also in the right list
        s, z, _ = real(block * (1.0 - 1.0 / grid_), bits_, sym, grid_, steps_)
        return s, real(block, bits_, sym, grid_, steps_)[1], 0

    def wrong_exponent(block, bits_, sym, grid_, steps_, hint_scales=None, rel_tol=0.0):
        # minimises the sum of absolute errors instead of squared errors over the right candidate list
        maxq = float(2 ** bits_ - 1)
        lo, hi = np.minimum(block.min(axis=1), 0.0), np.maximum(block.max(axis=1), 0.0)
        base = (hi - lo) / maxq
        zero = np.rint(-lo / base.astype(np.float32).astype(np.float64))
        best_s, best_e = None, None
        for i in range(steps_):
            sc = ((1.0 - i / grid_) * base).astype(np.float32).astype(np.float64)
            q = np.clip(np.rint(block / sc[:, None]) + zero[:, None], 0.0, maxq)
            e = np.sum(np.abs(sc[:, None] * (q - zero[:, None]) - block), axis=1)
            if best_e is None:
                best_s, best_e = sc.copy(), e.copy()
            else:
                take = e < best_e
                best_s, best_e = np.where(take, sc, best_s), np.where(take, e, best_e)
        return best_s, zero, 0

    for mutant in (off_by_one, wrong_exponent):
        monkeypatch.setattr(O, "quant_params_mse", mutant)
        bad = O.quantize_layer(W, U, P, bits, group, False, mse_grid=grid, mse_steps=steps)
        monkeypatch.setattr(O, "quant_params_mse", real)
        assert not np.array_equal(bad["scales"], good["scales"])          # the mistake does change the result
        with pytest.raises(AssertionError):
            PU.check_against_oracle(W, U, P, as_library(bad), bits, group, False, label=mutant.__name__, mse=(grid, steps))


def test_activation_quantiser_hand_worked_example():
    """Pins fake_quant_activations to values worked out by hand from the definition (tests/golden)."""
    for line in open(os.path.join(GOLD, "activation_quantiser_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, xs, sz, qs, ys = [f.split() for f in line.split("|")]
        bits, clip = int(head[1]), float(head[2])
        x = np.array([float(v) for v in xs], np.float32)
        xb = synth.f32_to_bf16_bits(x)[None, :]
        assert np.array_equal(synth.bf16_bits_to_f32(xb)[0], x)           # the fixture is exact in bfloat16
        yb, t, _ = O.fake_quant_activations(xb, bits, clip)
        scale, zero = float(sz[0]), float(sz[1])
        y = synth.bf16_bits_to_f32(yb)[0].astype(np.float64)
        assert np.allclose(y, [float(v) for v in ys], rtol=0, atol=2.0 ** -9 * scale * 4), (head[0], y)
        assert np.allclose(t[0], x.astype(np.float64) / scale, rtol=1e-7, atol=0)
        q = np.rint(y / scale + zero)
        assert np.array_equal(q, [float(v) for v in qs]), (head[0], q)


def test_activation_quantiser_and_packing():
    Xb, _ = synth.make_activations(50, 96, 7, "act", 2, 20.0)
    yb, t, _ = O.fake_quant_activations(Xb, 4, 0.9)
    x = synth.bf16_bits_to_f32(Xb).astype(np.float64)
    y = synth.bf16_bits_to_f32(yb).astype(np.float64)
    for r in (0, 17, 49):                                  # per token: 16 levels, clipped range, error bound
        assert len(np.unique(y[r])) <= 16
        lo, hi = 0.9 * min(x[r].min(), 0), 0.9 * max(x[r].max(), 0)
        step = (hi - lo) / 15
        assert y[r].min() >= lo - step and y[r].max() <= hi + step
        inside = (x[r] > lo + step) & (x[r] < hi - step)
        assert np.all(np.abs(y[r] - x[r])[inside] <= 0.5 * step * 1.02 + 2.0 ** -8 * np.abs(x[r][inside]))
    same, _, _ = O.fake_quant_activations(Xb, 16, 1.0)        # 16 bits, no clipping: (nearly) the identity
    assert np.max(np.abs(synth.bf16_bits_to_f32(same).astype(np.float64) - x)) <= np.abs(x).max() * 2.0 ** -8
    # packing: hand-checked 3-bit stream and a round trip
    assert O.pack_codes(np.array([[1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 3]], np.uint8), 3).tolist() == \
        [[1 | 2 << 3 | 3 << 6 | 4 << 9 | 5 << 12 | 6 << 15 | 7 << 18 | 0 << 21 | 1 << 24 | 2 << 27 | (3 & 3) << 30, 3 >> 2]]
    rng = np.random.default_rng(0)
    for bits in (2, 3, 4, 5, 8):
        c = rng.integers(0, 2 ** bits, (5, 77)).astype(np.uint8)
        p = O.pack_codes(c, bits)
        stream = np.unpackbits(p.view(np.uint8), axis=1, bitorder="little")[:, :77 * bits]
        back = (stream.reshape(5, 77, bits) * (1 << np.arange(bits))).sum(axis=2)
        assert np.array_equal(back, c)

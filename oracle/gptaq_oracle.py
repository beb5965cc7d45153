"""fp64 CPU oracle for the GPTAQ per-layer solve.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module.  It shares no code with the HIP library: numpy in float64, one function per
step of Algorithm 1 of the paper, in the paper's order and notation, unblocked and
unfused so that it can be checked against the paper by eye.

Orientation.  The paper writes X as n x k (neurons x tokens).  Activations arrive
here token-major, shape (k, n), as bfloat16 bit patterns (uint16); Xk below is that
array widened exactly to float64, so the paper's X is Xk.T.

Readings taken where the paper is silent:
  * H and dXXT are plain sums over tokens (Algorithm 1, line 2).
  * the W_{:,j} that multiplies P_{j,:} is the current, error-compensated value of
    column j *before* it is quantised (the W_{:,q} of Eq. 15), both inside the block
    and in the lazy trailing update; this is what makes lazy batching (Step 4) exact.
  * dead inputs (H_qq = 0): H_qq <- 1, row q of dXXT <- 0, column q of W <- 0, then
    lambda = damp * mean(diag H).
  * the weight quantiser is the uniform affine min-max grid with 0 inside the range;
    group parameters are taken from the current weights at the first column of a
    group; rounding is half-to-even; the scale is rounded to fp32 (the library hands
    fp32 scales to its caller, the oracle quantises on that same grid).

Pins (tests/test_oracle_pins.py): Eq. 2-3 explicit-inverse GPTQ when dX = 0, a
per-column constrained least-squares solved by a library lstsq (Eq. 14), Eq. 15 with
explicit inverses, Lemma 4.1, Theorem 4.2 vs Eq. 16, ridge-regression rows of P,
closed form W (I - P)^-1 for the identity quantiser, a hand-worked quantiser example.
Every function in this file has at least one such pin; none is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------- inputs
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 patterns (uint16) to float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ------------------------------------------------ Algorithm 1, line 2: H and dXXT
def accumulate(X_bits: np.ndarray, Xtilde_bits: np.ndarray):
    """H = X X^T and dXXT = (X~ - X) X^T (Algorithm 1, line 2), token-major inputs.

    dXXT[q, j] = sum_t dX[q, t] X[j, t]: row = neuron of dX, column = neuron of X
    (the row vector dX_{q,:} X^T of Eq. 16).
    """
    Xk = bf16_bits_to_f64(X_bits)
    Xtk = bf16_bits_to_f64(Xtilde_bits)
    H = Xk.T @ Xk
    dXXT = (Xtk - Xk).T @ Xk
    return H, dXXT


# ------------------------------------- Algorithm 1, line 3: damping, H^-1 = L L^T
def dampen(H: np.ndarray, dXXT: np.ndarray, damp: float):
    """H + lambda I with lambda = damp * mean(diag H) (damping relative to the mean
    diagonal, end of Section 4.2), after the dead-input rule."""
    H = np.array(H, dtype=np.float64, copy=True)
    A = np.array(dXXT, dtype=np.float64, copy=True)
    dead = np.diag(H) == 0.0
    idx = np.nonzero(dead)[0]
    H[idx, idx] = 1.0
    A[idx, :] = 0.0
    lam = damp * np.mean(np.diag(H))
    H[np.diag_indices_from(H)] += lam
    return H, A, dead, lam


def inverse_cholesky(H_lam: np.ndarray) -> np.ndarray:
    """Lower-triangular L with H_lam^-1 = L L^T (Step 3), by the literal route:
    invert, then factor."""
    Hinv = np.linalg.inv(H_lam)
    Hinv = 0.5 * (Hinv + Hinv.T)
    return np.linalg.cholesky(Hinv)


# ------------------------------------------- Algorithm 1, line 4 / Theorem 4.2: P
def correction_matrix(dXXT: np.ndarray, L: np.ndarray) -> np.ndarray:
    """P = ((dXXT L) (.) M_U) L^T with M_U the strictly-upper 0/1 mask (Eq. 17)."""
    O = np.triu(dXXT @ L, k=1)
    return O @ L.T


def prepare(H: np.ndarray, dXXT: np.ndarray, damp: float):
    """Lines 3-4 of Algorithm 1.  Returns U = L^T (upper), P (strictly upper), dead."""
    H_lam, A, dead, _ = dampen(H, dXXT, damp)
    L = inverse_cholesky(H_lam)
    P = correction_matrix(A, L)
    return L.T.copy(), P, dead


# -------------------------------------------------------------------- quantiser
def quant_params(xmin: np.ndarray, xmax: np.ndarray, bits: int, sym: bool):
    """Scale and zero-point of the uniform affine grid for ranges [xmin, xmax].

    The range always contains 0.  Symmetric: the range is widened to +-max|w| and the
    zero-point sits at mid-grid.  The scale is rounded to fp32 once.
    """
    maxq = float(2 ** bits - 1)
    xmin = np.minimum(np.asarray(xmin, np.float64), 0.0)
    xmax = np.maximum(np.asarray(xmax, np.float64), 0.0)
    if sym:
        xmax = np.maximum(np.abs(xmin), xmax)
        xmin = -xmax
    flat = (xmin == 0.0) & (xmax == 0.0)
    xmin = np.where(flat, -1.0, xmin)
    xmax = np.where(flat, 1.0, xmax)
    scale = ((xmax - xmin) / maxq).astype(np.float32).astype(np.float64)
    if sym:
        zero = np.full_like(scale, (maxq + 1.0) / 2.0)
    else:
        zero = np.rint(-xmin / scale)
    return scale, zero


def quant_params_mse(block: np.ndarray, bits: int, sym: bool, grid: int, steps: int,
                     hint_scales=None, rel_tol=0.0):
    """Clip-range search of Section 5.1 (the clipping range of the weights is the one that minimises the
    squared quantisation error), read as: the candidates p = 1 - i/grid, i = 0..steps-1, shrink the min-max range
    of each row of `block` about its zero-point (scale_i = fp32(p * (xmax - xmin)/maxq), zero-point of
    the full range); the candidate with the smallest sum of squared errors wins, the earlier on ties.
    With `hint_scales`, a hinted scale is accepted for a row if it is (to 1e-5) one of the row's
    candidates and that candidate's error is within rel_tol of the best.  Returns scale, zero, #hints."""
    maxq = float(2 ** bits - 1)
    xmin = np.minimum(block.min(axis=1), 0.0)
    xmax = np.maximum(block.max(axis=1), 0.0)
    if sym:
        xmax = np.maximum(np.abs(xmin), xmax)
        xmin = -xmax
    flat = (xmin == 0.0) & (xmax == 0.0)
    xmin = np.where(flat, -1.0, xmin)
    xmax = np.where(flat, 1.0, xmax)
    base = (xmax - xmin) / maxq
    scale0 = base.astype(np.float32).astype(np.float64)
    zero = np.full_like(base, (maxq + 1.0) / 2.0) if sym else np.rint(-xmin / scale0)
    cand = np.zeros((steps, block.shape[0]))
    errs = np.zeros((steps, block.shape[0]))
    for i in range(steps):
        sc = ((1.0 - i / grid) * base).astype(np.float32).astype(np.float64)
        q = np.clip(np.rint(block / sc[:, None]) + zero[:, None], 0.0, maxq)
        d = sc[:, None] * (q - zero[:, None]) - block
        cand[i], errs[i] = sc, np.sum(d * d, axis=1)
    best = np.argmin(errs, axis=0)                     # first minimum = earlier candidate on ties
    rows = np.arange(block.shape[0])
    hints = 0
    if hint_scales is not None:
        hs = np.asarray(hint_scales, np.float64)
        near = np.abs(cand - hs[None, :]) <= 1e-5 * hs[None, :]
        ok = near & (errs <= errs[best, rows][None, :] * (1.0 + rel_tol) + 1e-300)
        alt = np.argmax(ok, axis=0)
        take = ok.any(axis=0) & (alt != best)
        hints = int(take.sum())
        best = np.where(take, alt, best)
    return cand[best, rows], zero, hints


def quantize_column(w: np.ndarray, scale: np.ndarray, zero: np.ndarray, bits: int):
    """quant(.) for one column.  Returns integer codes, dequantised values and
    t = w / scale (the value whose rounding decides the code)."""
    maxq = float(2 ** bits - 1)
    t = w / scale
    q = np.clip(np.rint(t) + zero, 0.0, maxq)
    return q, scale * (q - zero), t


# ------------------------------- Algorithm 1, lines 5-13 with B = 1 (no batching)
def quantize_layer(W, U, P, bits, group=0, sym=False, dead=None,
                   identity_quantizer=False, use_E=True, use_P=True,
                   hint_codes=None, hint_zeros=None, tau=0.0,
                   mse_grid=0, mse_steps=0, hint_scales=None, mse_rel_tol=0.0):
    """The column loop of Algorithm 1, one column at a time (Eq. 15 with the Cholesky
    rows of Step 3): for each j

        v = W[:, j];  Q[:, j] = quant(v);  e = (v - Q[:, j]) / U[j, j]
        W[:, j:] += - e (x) U[j, j:]  +  v (x) P[j, j:]

    `hint_codes` / `hint_zeros` implement the near-tie protocol of the parity tests:
    where the pre-rounding value lies within `tau` of a rounding boundary and the
    hinted integer is the neighbour on the other side of it, the hinted integer is
    taken.  Returns a dict with codes (uint8), scales, zeros, What (float64), t,
    and the numbers of hints used.
    """
    W = np.array(W, dtype=np.float64, copy=True)
    m, n = W.shape
    maxq = float(2 ** bits - 1)
    if dead is not None:
        W[:, np.asarray(dead, bool)] = 0.0
    G = 1 if group <= 0 else n // group
    if group > 0 and n % group:
        raise ValueError("n must be a multiple of the group size")
    codes = np.zeros((m, n), np.uint8)
    What = np.zeros((m, n))
    T = np.zeros((m, n))
    scales = np.zeros((m, G))
    zeros = np.zeros((m, G))
    hints_used = 0
    zero_hints_used = 0
    scale_hints_used = 0

    def params(block, g):
        nonlocal zero_hints_used, scale_hints_used
        if mse_steps > 0:
            hs = None if hint_scales is None else hint_scales[:, g]
            s, z, nh = quant_params_mse(block, bits, sym, mse_grid, mse_steps, hs, mse_rel_tol)
            scale_hints_used += nh
            return s, z
        s, z = quant_params(block.min(axis=1), block.max(axis=1), bits, sym)
        if hint_zeros is not None and not sym:
            xmin = np.minimum(block.min(axis=1), 0.0)
            r = -xmin / s
            near = np.abs(np.abs(r - np.floor(r)) - 0.5) < tau
            hz = hint_zeros[:, g].astype(np.float64)
            take = near & (np.abs(hz - z) == 1.0)
            zero_hints_used += int(take.sum())
            z = np.where(take, hz, z)
        return s, z

    if group <= 0:
        scale, zero = params(W, 0)
        scales[:, 0], zeros[:, 0] = scale, zero
    for j in range(n):
        if group > 0 and j % group == 0:
            g = j // group
            scale, zero = params(W[:, j:j + group], g)
            scales[:, g], zeros[:, g] = scale, zero
        v = W[:, j].copy()
        if identity_quantizer:
            q, w_hat, t = np.zeros(m), v.copy(), v / scale
        else:
            q, w_hat, t = quantize_column(v, scale, zero, bits)
            if hint_codes is not None:
                frac = t - np.floor(t)
                near = np.abs(frac - 0.5) < tau
                hq = hint_codes[:, j].astype(np.float64)
                take = near & (np.abs(hq - q) == 1.0) & (hq >= 0) & (hq <= maxq)
                hints_used += int(take.sum())
                q = np.where(take, hq, q)
                w_hat = scale * (q - zero)
        codes[:, j] = q.astype(np.uint8)
        What[:, j] = w_hat
        T[:, j] = t
        e = (v - w_hat) / U[j, j]
        if use_E:
            W[:, j:] -= np.outer(e, U[j, j:])
        if use_P:
            W[:, j:] += np.outer(v, P[j, j:])
        W[:, j] = w_hat
    return dict(codes=codes, scales=scales, zeros=zeros, What=What, t=T,
                hints_used=hints_used, zero_hints_used=zero_hints_used, scale_hints_used=scale_hints_used)


# ----------------------------------- Algorithm 1 as printed, block size B (Step 4)
def quantize_layer_blocked(W, U, P, bits, group=0, sym=False, blocksize=128, dead=None):
    """Algorithm 1 with lazy batching: inside a block of B columns the update is
    applied at once, the columns after the block receive it once per block (Eq. 18).
    V keeps each column's value as it stood just before it was quantised."""
    W = np.array(W, dtype=np.float64, copy=True)
    m, n = W.shape
    if dead is not None:
        W[:, np.asarray(dead, bool)] = 0.0
    if group > 0 and (n % group or blocksize % group):
        raise ValueError("group must divide n and the block size")
    G = 1 if group <= 0 else n // group
    codes = np.zeros((m, n), np.uint8)
    What = np.zeros((m, n))
    scales = np.zeros((m, G))
    zeros = np.zeros((m, G))
    if group <= 0:
        scale, zero = quant_params(W.min(axis=1), W.max(axis=1), bits, sym)
        scales[:, 0], zeros[:, 0] = scale, zero
    for i in range(0, n, blocksize):
        i2 = min(i + blocksize, n)
        E = np.zeros((m, i2 - i))
        V = np.zeros((m, i2 - i))
        for j in range(i, i2):
            if group > 0 and j % group == 0:
                g = j // group
                blk = W[:, j:j + group]
                scale, zero = quant_params(blk.min(axis=1), blk.max(axis=1), bits, sym)
                scales[:, g], zeros[:, g] = scale, zero
            v = W[:, j].copy()
            q, w_hat, _ = quantize_column(v, scale, zero, bits)
            codes[:, j] = q.astype(np.uint8)
            What[:, j] = w_hat
            E[:, j - i] = (v - w_hat) / U[j, j]
            V[:, j - i] = v
            W[:, j:i2] += -np.outer(E[:, j - i], U[j, j:i2]) + np.outer(v, P[j, j:i2])
            W[:, j] = w_hat
        W[:, i2:] += -E @ U[i:i2, i2:] + V @ P[i:i2, i2:]
    return dict(codes=codes, scales=scales, zeros=zeros, What=What)


# ------------------------------------- neighbours of the solve in Algorithm 2 (Section 5.1)
def fake_quant_activations(X_bits: np.ndarray, bits: int, clip: float = 0.9, hint_bits=None, tau: float = 0.0):
    """Per-token asymmetric activation quantiser with a clipping ratio (Section 5.1), in float64.

    For every token (row): range = clip * [min(0, min x), max(0, max x)]; scale = range / (2^bits - 1),
    rounded to fp32 once (the grid is the one a user rebuilds from an fp32 scale, as for the weights);
    zero = rint(-clip * min / scale); y = scale * (clamp(rint(x / scale) + zero) - zero), which is exact in
    float64 (24-bit scale times a small integer), rounded once to bfloat16 (nearest, ties to even).
    `clip` is taken as the fp32 number the library receives.
    `hint_bits` / `tau`: near-tie protocol as in quantize_layer: where x / scale lies within tau of a rounding
    boundary and the hinted output is the dequantised neighbouring integer, that integer is taken.
    Returns (y as bf16 bit patterns, t = x / scale before rounding, number of hints used)."""
    x = bf16_bits_to_f64(X_bits)
    maxq = float(2 ** bits - 1)
    c = float(np.float32(clip))
    mn = np.minimum(x.min(axis=1), 0.0) * c
    mx = np.maximum(x.max(axis=1), 0.0) * c
    flat = (mn == 0.0) & (mx == 0.0)
    mn = np.where(flat, -1.0, mn)
    mx = np.where(flat, 1.0, mx)
    scale = ((mx - mn) / maxq).astype(np.float32).astype(np.float64)
    zero = np.rint(-mn / scale)
    t = x / scale[:, None]
    q = np.clip(np.rint(t) + zero[:, None], 0.0, maxq)
    hints = 0
    if hint_bits is not None:
        hy = bf16_bits_to_f64(hint_bits)
        frac = t - np.floor(t)
        near = np.abs(frac - 0.5) < tau
        for dq in (-1.0, 1.0):
            qa = q + dq
            ya = _f64_to_bf16_bits(scale[:, None] * (qa - zero[:, None]))
            take = near & (qa >= 0.0) & (qa <= maxq) & (ya == np.asarray(hint_bits, np.uint16)) & \
                (_f64_to_bf16_bits(scale[:, None] * (q - zero[:, None])) != np.asarray(hint_bits, np.uint16))
            hints += int(take.sum())
            q = np.where(take, qa, q)
        del hy
    y = scale[:, None] * (q - zero[:, None])
    return _f64_to_bf16_bits(y), t, hints


def _f64_to_bf16_bits(y: np.ndarray) -> np.ndarray:
    """float64 -> bfloat16 bit patterns with ONE rounding (nearest, ties to even).  Going through float32 would
    round twice; the float32 value is therefore first made 'sticky' (round to odd), after which the second rounding
    cannot go wrong: bfloat16 keeps 8 significand bits, float32 24."""
    y = np.asarray(y, np.float64)
    f = y.astype(np.float32)                                # nearest
    u = f.view(np.uint32).copy()
    back = f.astype(np.float64)
    inexact = back != y
    # turn the nearest float32 into the truncated one where it was rounded away from zero, then set the sticky bit
    away = inexact & (np.abs(back) > np.abs(y))
    u = np.where(away, u - 1, u)
    u = np.where(inexact, u | 1, u).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """Row-wise little-endian bit stream: code j occupies bits [j*bits, (j+1)*bits) of its row."""
    m, n = codes.shape
    words = (n * bits + 31) // 32
    out = np.zeros((m, words), np.uint64)
    for j in range(n):
        bit = j * bits
        w, sh = bit // 32, bit % 32
        v = codes[:, j].astype(np.uint64) & ((1 << bits) - 1)
        out[:, w] |= (v << sh) & 0xFFFFFFFF
        if sh + bits > 32:
            out[:, w + 1] |= v >> (32 - sh)
    return out.astype(np.uint32)


# ------------------------------------------------ act_order (Sections 5.2 and 5.3)
def act_order_permutation(H: np.ndarray) -> np.ndarray:
    """Inputs in the order of decreasing Hessian diagonal (the act_order option the paper takes from
    GPTQ); equal diagonals keep their index order."""
    return np.argsort(-np.diag(np.asarray(H, np.float64)), kind="stable")


def solve_with_act_order(W, H, dXXT, damp, bits, group=0, sym=False):
    """Algorithm 1 on the permuted problem, results scattered back to the original column order.
    scales/zeros stay indexed by groups of consecutive permuted columns."""
    perm = act_order_permutation(H)
    Hp = np.asarray(H, np.float64)[np.ix_(perm, perm)]
    Ap = np.asarray(dXXT, np.float64)[np.ix_(perm, perm)]
    U, P, dead = prepare(Hp, Ap, damp)
    out = quantize_layer(np.asarray(W, np.float64)[:, perm], U, P, bits, group, sym, dead=dead)
    res = dict(out)
    for key in ("codes", "What"):
        back = np.empty_like(out[key])
        back[:, perm] = out[key]
        res[key] = back
    res["perm"] = perm
    res["U"], res["P"] = U, P
    return res


# --------------------------------------------------------------- Eq. 4 objective
def layer_output_error(W, What, X_bits, Xtilde_bits) -> float:
    """|| What X - W X~ ||_F^2 (Eq. 4), original W, undamped data."""
    Xk = bf16_bits_to_f64(X_bits)
    Xtk = bf16_bits_to_f64(Xtilde_bits)
    D = np.asarray(What, np.float64) @ Xk.T - np.asarray(W, np.float64) @ Xtk.T
    return float(np.sum(D * D))


def layer_output_error_from_moments(W, What, H, dXXT, C) -> float:
    """The same objective without touching tokens:  with D = What - W,
    ||What X - W X~||^2 = tr(D H D^T) - 2 tr(D dXXT^T W^T) + tr(W C W^T),
    H = X X^T, dXXT = dX X^T, C = dX dX^T (all undamped)."""
    W = np.asarray(W, np.float64)
    D = np.asarray(What, np.float64) - W
    return float(np.sum((D @ H) * D) - 2.0 * np.sum((D @ dXXT.T) * W) + np.sum((W @ C) * W))


# ------------------------------------------------------- independent cross-checks
def gptq_explicit_inverse(W, H_lam, bits, group=0, sym=False):
    """Plain GPTQ/OBQ in its original form (Eq. 2-3): explicit inverse Hessian, update
    of the whole row from column q of H^-1, then Gaussian elimination of row/column q.
    No Cholesky factor anywhere.  Used to pin the dX = 0 case."""
    W = np.array(W, dtype=np.float64, copy=True)
    m, n = W.shape
    Hinv = np.linalg.inv(H_lam)
    codes = np.zeros((m, n), np.uint8)
    What = np.zeros((m, n))
    if group <= 0:
        scale, zero = quant_params(W.min(axis=1), W.max(axis=1), bits, sym)
    for q in range(n):
        if group > 0 and q % group == 0:
            blk = W[:, q:q + group]
            scale, zero = quant_params(blk.min(axis=1), blk.max(axis=1), bits, sym)
        c, w_hat, _ = quantize_column(W[:, q], scale, zero, bits)
        codes[:, q] = c.astype(np.uint8)
        What[:, q] = w_hat
        W += np.outer((w_hat - W[:, q]) / Hinv[q, q], Hinv[q, :])
        W[:, q] = w_hat
        Hinv = Hinv - np.outer(Hinv[:, q], Hinv[q, :]) / Hinv[q, q]
        Hinv[q, :] = 0.0
        Hinv[:, q] = 0.0
    return dict(codes=codes, What=What)


def gptaq_explicit_inverse(W, H_lam, dXXT, bits, group=0, sym=False):
    """Eq. 15 taken literally: at column q recompute, from H_lam alone, the inverse of
    the Hessian of the not-yet-quantised inputs (H~^-1) and of the inputs after q
    (H~^-1_{-q}), no factor L and no matrix P."""
    W = np.array(W, dtype=np.float64, copy=True)
    m, n = W.shape
    codes = np.zeros((m, n), np.uint8)
    What = np.zeros((m, n))
    if group <= 0:
        scale, zero = quant_params(W.min(axis=1), W.max(axis=1), bits, sym)
    for q in range(n):
        if group > 0 and q % group == 0:
            blk = W[:, q:q + group]
            scale, zero = quant_params(blk.min(axis=1), blk.max(axis=1), bits, sym)
        w_q = W[:, q].copy()
        c, w_hat, _ = quantize_column(w_q, scale, zero, bits)
        codes[:, q] = c.astype(np.uint8)
        What[:, q] = w_hat
        Ht = np.linalg.inv(H_lam[q:, q:])
        W[:, q:] += np.outer((w_hat - w_q) / Ht[0, 0], Ht[0, :])
        if q + 1 < n:
            Hm = np.linalg.inv(H_lam[q + 1:, q + 1:])
            W[:, q + 1:] += np.outer(w_q, dXXT[q, q + 1:] @ Hm)
        W[:, q] = w_hat
    return dict(codes=codes, What=What)

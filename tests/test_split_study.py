"""Host-side study: which cheaper treatments of dX = X~ - X keep H and dXXT inside the 1e-5 bar (Algorithm 1, line 2).

The library multiplies dX as an exact sum of two bf16 terms (hi + lo), which costs 5 n^2 c executed flop for the
3 n^2 c the sums need.  This test evaluates the alternatives on the synthetic recipe with numpy only (products of
bf16 numbers are exact in fp32, so the operand rounding is the whole story) and pins the facts the design rests on.
"""
import numpy as np

from paper_2504_02692_amd import synth


def _bf16(x):
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))


def _e4m3(x):
    """Round to 4 significant bits with a 4-bit exponent under one power-of-two scale per tensor (an OCP e4m3 model)."""
    x = x.astype(np.float64)
    out = np.zeros_like(x)
    nz = x != 0
    q = 2.0 ** (np.floor(np.log2(np.abs(x[nz]))) - 3)
    out[nz] = np.rint(x[nz] / q) * q
    qmin = 2.0 ** (np.floor(np.log2(np.abs(x).max())) - 8 - 6 - 3)          # quantum of the subnormals
    sub = np.abs(x) < 8 * qmin
    out[sub] = np.rint(x[sub] / qmin) * qmin
    return out


def test_cheaper_treatments_of_the_dx_split():
    n, tokens = 256, 32768
    Xb, Xtb = synth.make_activations(tokens, n, 1)[:2]
    X = synth.bf16_bits_to_f32(Xb)
    Xt = synth.bf16_bits_to_f32(Xtb)
    X64 = X.astype(np.float64)
    ref = (Xt.astype(np.float64) - X64).T @ X64
    err = lambda A: np.linalg.norm(A - ref) / np.linalg.norm(ref)

    dX = Xt - X                                    # exact in fp32: both are bf16 with nearby exponents
    hi = _bf16(dX)
    lo = _bf16(dX - hi)
    assert np.abs(dX.astype(np.float64) - hi - lo).max() == 0.0             # the two-term split loses nothing
    prod = lambda A, B: A.T.astype(np.float64) @ B.astype(np.float64)
    e_split = err(prod(hi, X) + prod(lo, X))
    e_hi = err(prod(hi, X))
    e_fp8 = err(prod(hi, X) + prod(_e4m3(lo), _e4m3(X)))                    # an fp8 product needs both operands in fp8
    e_diff = err((Xt.T @ X).astype(np.float64) - (X.T @ X).astype(np.float64))   # X~X^T - XX^T, fp32 sums
    print(f"exact split {e_split:.1e}  hi only {e_hi:.1e}  hi + fp8 lo {e_fp8:.1e}  difference of products {e_diff:.1e}")
    assert e_split < 1e-9
    assert e_hi > 1e-4                             # one bf16 term: 50x outside the bar
    assert e_diff > 1e-4                           # cancellation of two fp32 sums: outside the bar
    assert e_fp8 > 1e-5                            # lo and X in fp8 (the matrix cores take no bf16 x fp8 pair): just outside the bar
    assert err(prod(hi, X) + prod(_e4m3(lo), X)) < 1e-5      # (with a full-precision X it would pass: the X rounding is what breaks it)
    # fp16 keeps 11 bits of dX: one fp16 product is still outside the bar; with its remainder as an fp8 product it would
    # be inside, at the price of fp16 operands (a range of 65504, against bf16's, for activations of any scale)
    h16 = dX.astype(np.float16).astype(np.float32)
    X16 = X.astype(np.float16).astype(np.float32)
    e_h16 = err(prod(h16, X16))
    e_h16_fp8 = err(prod(h16, X16) + prod(_e4m3(dX - h16), _e4m3(X)))
    print(f"fp16 hi only {e_h16:.1e}  fp16 hi + fp8 remainder {e_h16_fp8:.1e}")
    assert e_h16 > 1e-5 and e_h16_fp8 < 2e-6

"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run the HIP
path through the binding, and compare with the fp64 oracle (near-tie protocol included)."""
import numpy as np
import torch

from oracle import gptaq_oracle as O
from paper_2504_02692_amd import binding as B

MAX_HINT_FRAC = 1e-4


def tau_for(bits: int) -> float:
    """Half-width of the near-tie window, in quantisation steps.

    The weights live in fp32, so the value t = w / scale whose rounding decides a code carries the fp32
    rounding of w: 2^-24 |t| steps per rounding, |t| up to maxq = 2^bits - 1, one rounding per update the
    weight receives.  Measured in steps this noise grows in proportion to the number of levels, so the
    window does too: 5e-5 of a step up to 4 bits (maxq = 15; about 50 roundings of the largest |t|), and
    5e-5 * maxq / 15 above (8.5e-4 at 8 bits, where a single fp32 rounding of w is already 1.5e-5 steps).
    The window only says which entries MAY take the other integer; how many do is bounded separately
    (MAX_HINT_FRAC of the entries)."""
    maxq = 2 ** bits - 1
    return 5e-5 * max(1.0, maxq / 15.0)


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16).copy()).cuda().view(torch.bfloat16)


def rel_fro(a, b) -> float:
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def gpu_accumulate(Xb, Xtb, chunks=None, ws_bytes=None, upper=False):
    tokens, n = Xb.shape
    X, Xt = to_dev_bf16(Xb), to_dev_bf16(Xtb)
    H = torch.zeros((n, n), dtype=torch.float32, device="cuda")
    A = torch.zeros_like(H)
    bounds = [0, tokens] if not chunks else chunks
    for t0, t1 in zip(bounds[:-1], bounds[1:]):
        nb = B.gptaq_accumulate_workspace_bytes(t1 - t0, n) if ws_bytes is None else ws_bytes
        ws = B.workspace(nb)
        (B.gptaq_accumulate_upper if upper else B.gptaq_accumulate)(X[t0:t1], Xt[t0:t1], H, A, ws)
    torch.cuda.synchronize()
    return H, A


def gpu_prepare(H, A, damp):
    n = H.shape[0]
    ws = B.workspace(B.gptaq_prepare_workspace_bytes(n))
    dead, info = B.gptaq_prepare(H, A, damp, ws)
    torch.cuda.synchronize()
    return dead, info


def gpu_quantize(W, U, P, bits, group, sym, blocksize, dead=None, terms=3, mse=(0, 0)):
    Wd = torch.from_numpy(np.asarray(W, np.float32).copy()).cuda()
    m, n = Wd.shape
    ws = B.workspace(B.gptaq_quantize_workspace_bytes(m, n))
    codes, scales, zeros = B.gptaq_quantize_layer(Wd, U, P, bits, group, sym, blocksize, ws, dead=dead, terms=terms,
                                                  mse_grid=mse[0], mse_steps=mse[1])
    torch.cuda.synchronize()
    return dict(What=Wd.cpu().numpy(), codes=codes.cpu().numpy(), scales=scales.cpu().numpy(),
                zeros=zeros.cpu().numpy())


def check_against_oracle(W, U64, P64, got, bits, group, sym, dead=None, Xb=None, Xtb=None, label="", terms=3, mse=(0, 0)):
    """The parity bar.  Codes and zero-points must be bit-exact apart from near-tie flips: the oracle is
    re-run taking the library's integer wherever its own pre-rounding value lies within tau_for(bits) of a
    rounding boundary and the library's integer is the neighbour across it; such hints must number at most
    1e-4 of the entries, and with none used the raw codes must already be equal.  Then every code and
    zero-point must agree, scales to 2 tau / maxq + 2^-24 relative (both ends of the range carry the same
    fp32 noise as a weight near a tie; exact for per-channel grids, which come from the original weights),
    dequantised weights to 1e-4 relative Frobenius, and the layer output error to 0.5 %."""
    W = np.asarray(W, np.float64)
    m, n = W.shape
    tau = tau_for(bits)
    maxq = 2 ** bits - 1
    kw = dict(use_E=bool(terms & 1), use_P=bool(terms & 2), mse_grid=mse[0], mse_steps=mse[1])
    raw = O.quantize_layer(W, U64, P64, bits, group, sym, dead=dead, **kw)
    raw_diff = raw["codes"] != got["codes"]
    raw_mis = float(raw_diff.mean())
    hinted = O.quantize_layer(W, U64, P64, bits, group, sym, dead=dead,
                              hint_codes=got["codes"], hint_zeros=got["zeros"], tau=tau,
                              hint_scales=got["scales"] if mse[1] else None, mse_rel_tol=1e-4, **kw)
    nh = hinted["hints_used"] + hinted["zero_hints_used"] + hinted["scale_hints_used"]
    print(f"[{label}] raw code mismatch {raw_mis:.3e}; hints used {nh} of {m * n} (tau {tau:.1e})")
    diff = hinted["codes"] != got["codes"]
    if diff.any():
        # for every row that still differs: the first differing column and how far the oracle's value was from a tie
        rows = np.nonzero(diff.any(axis=1))[0]
        for r in rows[:8]:
            c = int(np.argmax(diff[r]))
            t = hinted["t"][r, c]
            print(f"[{label}]   row {r} col {c}: oracle t {t:.6f} (distance from a tie {abs(abs(t - np.floor(t)) - 0.5):.2e}), "
                  f"codes oracle {int(hinted['codes'][r, c])} library {int(got['codes'][r, c])}")
    if nh == 0:
        assert raw_mis == 0.0, "codes differ although no entry was near a tie"
    assert nh <= MAX_HINT_FRAC * m * n, f"{nh} near-tie hints on {m * n} entries"
    assert np.array_equal(hinted["zeros"], got["zeros"].astype(np.float64)), "zero points differ"
    ds = float(np.max(np.abs(hinted["scales"] - got["scales"]) / hinted["scales"]))
    ds_tol = 1e-4 if mse[1] else (0.0 if group <= 0 else 2.0 * tau / maxq + 2.0 ** -24)
    print(f"[{label}] largest relative scale difference {ds:.3e} (allowed {ds_tol:.1e})")
    assert ds <= ds_tol, "scales differ"
    mism = int(diff.sum())
    assert mism == 0, f"{mism} codes differ after near-tie hints"
    rf = rel_fro(got["What"], hinted["What"])
    print(f"[{label}] dequantised weights rel. Frobenius error {rf:.3e}")
    assert rf <= 1e-4
    if Xb is not None:
        e_gpu = O.layer_output_error(W, got["What"], Xb, Xtb)
        e_ref = O.layer_output_error(W, raw["What"], Xb, Xtb)
        print(f"[{label}] layer output error gpu {e_gpu:.6e} oracle {e_ref:.6e}")
        assert abs(e_gpu - e_ref) <= 5e-3 * e_ref
    return raw_mis, nh

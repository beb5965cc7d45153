"""gptaq_accumulate_noalloc (the entry point that allocates nothing) against gptaq_accumulate.

Two calls in a row on the same GPU, the second with a smaller input, each compared with the existing
entry point: bit for bit when that one is given a workspace of the built-in array's size (the passes are
then the same), and to the accumulate parity bar (relative Frobenius error <= 1e-5) against both its
default workspace and the fp64 oracle.
"""
import numpy as np
import pytest
import torch

from oracle import gptaq_oracle as O
from paper_2504_02692_amd import binding as B
from paper_2504_02692_amd import synth
from tests.parity_util import rel_fro, to_dev_bf16

pytestmark = pytest.mark.gpu

SCRATCH_BYTES = 32 << 20


def _run_pair(tokens, n, seed):
    Xb, Xtb = synth.make_activations(tokens, n, seed, "x", 4, 20.0, 0.05)
    X, Xt = to_dev_bf16(Xb), to_dev_bf16(Xtb)
    out = {}
    for name in ("noalloc", "same_ws", "default_ws"):
        H = torch.zeros((n, n), dtype=torch.float32, device="cuda")
        A = torch.zeros_like(H)
        if name == "noalloc":
            B.gptaq_accumulate_noalloc(X, Xt, H, A)
        else:
            nb = SCRATCH_BYTES if name == "same_ws" else B.gptaq_accumulate_workspace_bytes(tokens, n)
            B.gptaq_accumulate(X, Xt, H, A, B.workspace(nb))
        torch.cuda.synchronize()
        out[name] = (np.triu(H.cpu().numpy()), A.cpu().numpy())
    H64, A64 = O.accumulate(Xb, Xtb)
    return out, np.triu(H64), A64


def test_noalloc_accumulate_two_calls_in_a_row():
    # first call: several passes (1344 tokens each at n = 1024 + padding) and a ragged last one;
    # second call: smaller in both dimensions, so it reads only part of what the first left behind
    for tokens, n, seed in ((5000, 1000, 11), (700, 328, 12)):
        print(f"noalloc accumulate: tokens {tokens} n {n} seed {seed}", flush=True)
        out, H64, A64 = _run_pair(tokens, n, seed)
        Hn, An = out["noalloc"]
        Hs, As = out["same_ws"]
        Hd, Ad = out["default_ws"]
        assert np.array_equal(Hn, Hs) and np.array_equal(An, As), "differs from gptaq_accumulate on an equal workspace"
        assert rel_fro(Hn, Hd) <= 1e-5 and rel_fro(An, Ad) <= 1e-5
        eh, ea = rel_fro(Hn, H64), rel_fro(An, A64)
        print(f"  vs fp64 oracle: H {eh:.2e} dXXT {ea:.2e}", flush=True)
        assert eh <= 1e-5 and ea <= 1e-5


def test_noalloc_accumulate_rejects_what_does_not_fit():
    n = 16384 + 8
    X = torch.zeros((64, n), dtype=torch.bfloat16, device="cuda")
    H = torch.zeros((8, 8), dtype=torch.float32, device="cuda")          # never touched: the call must fail first
    lib = B.load()
    rc = lib.gptaq_accumulate_noalloc(X.data_ptr(), X.data_ptr(), 64, n, n, H.data_ptr(), H.data_ptr(), n, None)
    assert rc == -6
    assert b"scratch" in lib.gptaq_status_string(rc)

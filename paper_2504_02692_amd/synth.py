"""Seeded synthetic inputs for the GPTAQ per-layer solve.

This module only *draws numbers*: activations X (what the quantised model feeds a
layer), X-tilde (what the full-precision model feeds it) and weights W, shaped like
the transformer layers the paper calibrates (Table 9; Section 4.2 "Step 2" for the
token count k = 128 x 2048).  It contains none of the method's arithmetic, so both
the HIP library and the CPU oracle can be fed from it without sharing code.

Recipe (all seeded):
  * X[t, c] ~ N(0, 1); a few seeded "outlier" channels are multiplied by a constant
    (x20 for the language-model shapes, x30 for the ViT shapes), imitating the
    activation outliers of language transformers (Section 5.3).
  * X-tilde = X + N(0, (0.05 * sigma_c)^2) per channel c, sigma_c the channel's std.
  * both are rounded to bfloat16 (round-to-nearest-even) exactly once; every
    consumer reads the same 16-bit patterns.
  * W ~ N(0, 0.02^2) in fp32.

Layout: activations are token-major, shape (tokens, n), i.e. the transpose of the
paper's n x k matrix X.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Tuple

import numpy as np


# --------------------------------------------------------------------------- bf16
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even); returns the uint16 patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = u + 0x7FFF + lsb
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


# ------------------------------------------------------------------------ configs
@dataclasses.dataclass(frozen=True)
class LayerSpec:
    name: str
    m: int            # output channels (rows of W)
    n: int            # input channels (columns of W)
    input_id: str     # layers with the same input share H, dXXT, U, P


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    tokens: int
    layers: Tuple[LayerSpec, ...]
    n_outliers: int
    outlier_scale: float
    noise: float = 0.05
    bits: int = 4
    group: int = 128       # <= 0 : one scale per output channel
    sym: bool = False
    blocksize: int = 128
    damp: float = 0.01
    seed: int = 0

    def inputs(self) -> Dict[str, int]:
        out: Dict[str, int] = {}
        for l in self.layers:
            out.setdefault(l.input_id, l.n)
        return out


def workload(name: str) -> Workload:
    """The synthetic stand-ins for the layer sets the paper calibrates."""
    if name == "c1":       # small single layer, the full oracle runs in seconds
        return Workload("c1", 4096, (LayerSpec("fc", 512, 512, "x"),), 4, 20.0,
                        bits=4, group=0, sym=False)
    if name == "llama7b":  # Table 9 shapes, 128 x 2048 calibration tokens
        L = (LayerSpec("q_proj", 4096, 4096, "attn_in"),
             LayerSpec("k_proj", 4096, 4096, "attn_in"),
             LayerSpec("v_proj", 4096, 4096, "attn_in"),
             LayerSpec("o_proj", 4096, 4096, "attn_out"),
             LayerSpec("gate_proj", 11008, 4096, "mlp_in"),
             LayerSpec("up_proj", 11008, 4096, "mlp_in"),
             LayerSpec("down_proj", 4096, 11008, "mlp_mid"))
        return Workload("llama7b", 128 * 2048, L, 4, 20.0, bits=4, group=128)
    if name == "llama70b":
        L = (LayerSpec("q_proj", 8192, 8192, "attn_in"),
             LayerSpec("k_proj", 1024, 8192, "attn_in"),
             LayerSpec("v_proj", 1024, 8192, "attn_in"),
             LayerSpec("o_proj", 8192, 8192, "attn_out"),
             LayerSpec("gate_proj", 28672, 8192, "mlp_in"),
             LayerSpec("up_proj", 28672, 8192, "mlp_in"),
             LayerSpec("down_proj", 8192, 28672, "mlp_mid"))
        return Workload("llama70b", 128 * 2048, L, 4, 20.0, bits=3, group=128)
    if name == "llama405b":
        L = (LayerSpec("q_proj", 16384, 16384, "attn_in"),
             LayerSpec("k_proj", 1024, 16384, "attn_in"),
             LayerSpec("v_proj", 1024, 16384, "attn_in"),
             LayerSpec("o_proj", 16384, 16384, "attn_out"),
             LayerSpec("gate_proj", 53248, 16384, "mlp_in"),
             LayerSpec("up_proj", 53248, 16384, "mlp_in"),
             LayerSpec("down_proj", 16384, 53248, "mlp_mid"))
        return Workload("llama405b", 65536, L, 4, 20.0, bits=4, group=128)
    if name == "eva02":
        L = (LayerSpec("qkv", 3072, 1024, "attn_in"),
             LayerSpec("proj", 1024, 1024, "attn_out"),
             LayerSpec("fc1", 4096, 1024, "mlp_in"),
             LayerSpec("fc2", 1024, 4096, "mlp_mid"))
        return Workload("eva02", 128 * 257, L, 2, 30.0, bits=3, group=128, sym=True)
    raise KeyError(name)


# -------------------------------------------------------------------- generators
def _stable_id(s: str) -> int:
    h = 2166136261
    for ch in s.encode():
        h = ((h ^ ch) * 16777619) & 0xFFFFFFFF
    return h


def outlier_channels(n: int, count: int, seed: int, input_id: str = "x") -> np.ndarray:
    rng = np.random.default_rng([seed, _stable_id(input_id), 7])
    return np.sort(rng.choice(n, size=min(count, n), replace=False))


def make_weights(m: int, n: int, seed: int, name: str = "fc") -> np.ndarray:
    rng = np.random.default_rng([seed, _stable_id(name), 11])
    return (0.02 * rng.standard_normal((m, n))).astype(np.float32)


def make_activations(tokens: int, n: int, seed: int, input_id: str = "x",
                     n_outliers: int = 4, outlier_scale: float = 20.0,
                     noise: float = 0.05, empirical_sigma: bool = True
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """CPU generator.  Returns (X_bits, Xtilde_bits), uint16 bf16 patterns, (tokens, n)."""
    rng = np.random.default_rng([seed, _stable_id(input_id), 3])
    x = rng.standard_normal((tokens, n)).astype(np.float32)
    ch = outlier_channels(n, n_outliers, seed, input_id)
    x[:, ch] *= np.float32(outlier_scale)
    if empirical_sigma and tokens > 1:
        sigma = x.std(axis=0, dtype=np.float64).astype(np.float32)
    else:
        sigma = np.ones(n, np.float32)
        sigma[ch] = outlier_scale
    xt = x + (noise * sigma)[None, :] * rng.standard_normal((tokens, n)).astype(np.float32)
    return f32_to_bf16_bits(x), f32_to_bf16_bits(xt)


def make_activations_device(tokens: int, n: int, seed: int, input_id: str, device,
                            n_outliers: int = 4, outlier_scale: float = 20.0,
                            noise: float = 0.05, chunk: int = 16384):
    """Device generator for the full-size workloads (tens of GB do not fit a host
    generator's time budget).  Same recipe with the nominal per-channel sigma
    (1, or the outlier scale), drawn with torch's seeded device generator in token
    chunks.  Returns two torch.bfloat16 tensors (tokens, n) living on `device`;
    a checker copies whatever rows/columns it needs back to the host, so both
    sides still consume identical bit patterns.
    """
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + _stable_id(input_id)) & 0x7FFFFFFF)
    ch = torch.as_tensor(outlier_channels(n, n_outliers, seed, input_id), device=device)
    sigma = torch.ones(n, device=device, dtype=torch.float32)
    sigma[ch] = outlier_scale
    X = torch.empty((tokens, n), device=device, dtype=torch.bfloat16)
    Xt = torch.empty((tokens, n), device=device, dtype=torch.bfloat16)
    for t0 in range(0, tokens, chunk):
        t1 = min(tokens, t0 + chunk)
        x = torch.randn((t1 - t0, n), device=device, dtype=torch.float32, generator=g) * sigma
        e = torch.randn((t1 - t0, n), device=device, dtype=torch.float32, generator=g)
        X[t0:t1] = x.to(torch.bfloat16)
        Xt[t0:t1] = (x + noise * sigma * e).to(torch.bfloat16)
    return X, Xt


def make_weights_device(m: int, n: int, seed: int, name: str, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + _stable_id(name) + 17) & 0x7FFFFFFF)
    return 0.02 * torch.randn((m, n), device=device, dtype=torch.float32, generator=g)

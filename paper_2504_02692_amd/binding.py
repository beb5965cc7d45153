"""Thin ctypes binding of libgptaq.so.  Argument marshalling only: every step of the solve
runs in the library's HIP kernels.  torch is used for device memory and the current stream.

The functions carry the names of the C entry points (include/gptaq.h).  There is no CPU or
PyTorch fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgptaq.so")
_lib: Optional[ctypes.CDLL] = None

_c = ctypes
_SIGS = {
    "gptaq_status_string": (_c.c_char_p, [_c.c_int]),
    "gptaq_last_hip_error": (_c.c_int, []),
    "gptaq_accumulate_workspace_bytes": (_c.c_size_t, [_c.c_int64, _c.c_int64]),
    "gptaq_accumulate": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64,
                                    _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "gptaq_accumulate_upper": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64,
                                          _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "gptaq_accumulate_noalloc": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64,
                                            _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p]),
    "gptaq_accumulate_staged": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_void_p,
                                           _c.c_void_p, _c.c_int64, _c.c_void_p, _c.c_size_t, _c.POINTER(_c.c_int64),
                                           _c.c_int, _c.c_void_p]),
    "gptaq_accumulate_staged_upper": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64,
                                                 _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p, _c.c_size_t,
                                                 _c.POINTER(_c.c_int64), _c.c_int, _c.c_void_p]),
    "gptaq_symmetrize": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_void_p]),
    "gptaq_prepare_workspace_bytes": (_c.c_size_t, [_c.c_int64]),
    "gptaq_prepare": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_float,
                                 _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "gptaq_quantize_workspace_bytes": (_c.c_size_t, [_c.c_int64, _c.c_int64]),
    "gptaq_quantize_layer": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_void_p, _c.c_void_p,
                                        _c.c_int64, _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                        _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_size_t,
                                        _c.c_void_p]),
    "gptaq_quantize_layer_terms": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_void_p, _c.c_void_p,
                                              _c.c_int64, _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                              _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_size_t,
                                              _c.c_void_p, _c.c_int]),
    "gptaq_quantize_layer_ex": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_void_p, _c.c_void_p,
                                           _c.c_int64, _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                           _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_size_t,
                                           _c.c_void_p, _c.c_int, _c.c_int, _c.c_int]),
    "gptaq_act_order": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_void_p, _c.c_void_p]),
    "gptaq_accumulate_diag": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_void_p, _c.c_void_p]),
    "gptaq_invert_permutation": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_void_p, _c.c_void_p]),
    "gptaq_accumulate_upper_permuted": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_void_p,
                                                   _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p, _c.c_size_t,
                                                   _c.c_void_p]),
    "gptaq_permute_hessian_workspace_bytes": (_c.c_size_t, [_c.c_int64]),
    "gptaq_permute_hessian": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_void_p, _c.c_void_p,
                                         _c.c_size_t, _c.c_void_p]),
    "gptaq_permute_columns_f32": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_int64,
                                             _c.c_void_p, _c.c_int, _c.c_void_p]),
    "gptaq_permute_columns_u8": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_int64,
                                            _c.c_void_p, _c.c_int, _c.c_void_p]),
    "gptaq_fake_quant_activations": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_int64,
                                                _c.c_int, _c.c_float, _c.c_void_p]),
    "gptaq_packed_words_per_row": (_c.c_int64, [_c.c_int64, _c.c_int]),
    "gptaq_pack_codes": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_int, _c.c_void_p, _c.c_void_p]),
    "gptaq_profile_enable": (_c.c_int, [_c.c_int]),
    "gptaq_profile_read": (_c.c_int, [_c.c_int, _c.POINTER(_c.c_int64), _c.POINTER(_c.c_double)]),
    "gptaq_measure_mfma_peak": (_c.c_int, [_c.c_int, _c.c_int, _c.c_void_p, _c.c_size_t, _c.POINTER(_c.c_double),
                                           _c.POINTER(_c.c_double), _c.c_void_p]),
    "gptaq_measure_hbm_copy": (_c.c_int, [_c.c_size_t, _c.c_int, _c.c_void_p, _c.c_size_t, _c.POINTER(_c.c_double),
                                          _c.c_void_p]),
}
EXPORTS = tuple(_SIGS)
PROFILE_TAGS = ("accumulate_gemm", "accumulate_split", "factor_sweep", "p_gemm", "column_loop", "trailing_gemm",
                "trailing_split")


class GptaqError(RuntimeError):
    pass


def load() -> ctypes.CDLL:
    """Load libgptaq.so (built by paper_2504_02692_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise GptaqError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_02692_amd.build` "
                             "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(status: int, what: str) -> None:
    if status != 0:
        lib = load()
        msg = lib.gptaq_status_string(status).decode()
        raise GptaqError(f"{what}: {msg} (status {status}, hip error {lib.gptaq_last_hip_error()})")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _need(t: torch.Tensor, dtype, name: str) -> None:
    if not t.is_cuda or t.dtype != dtype or t.dim() != 2 or t.stride(1) != 1:
        raise GptaqError(f"{name}: expected a 2-D row-major {dtype} CUDA tensor")


def _need_vec(t: torch.Tensor, dtype, name: str) -> None:
    if not t.is_cuda or t.dtype != dtype or t.dim() != 1 or not t.is_contiguous():
        raise GptaqError(f"{name}: expected a contiguous 1-D {dtype} CUDA tensor")


def workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def gptaq_accumulate_workspace_bytes(tokens: int, n: int) -> int:
    return load().gptaq_accumulate_workspace_bytes(tokens, n)


def gptaq_prepare_workspace_bytes(n: int) -> int:
    return load().gptaq_prepare_workspace_bytes(n)


def gptaq_quantize_workspace_bytes(m: int, n: int) -> int:
    return load().gptaq_quantize_workspace_bytes(m, n)


def _accumulate(name: str, X: torch.Tensor, Xtilde: torch.Tensor, H: torch.Tensor, dXXT: torch.Tensor,
                ws: torch.Tensor) -> None:
    _need(X, torch.bfloat16, "X"); _need(Xtilde, torch.bfloat16, "Xtilde")
    _need(H, torch.float32, "H"); _need(dXXT, torch.float32, "dXXT")
    tokens, n = X.shape
    if Xtilde.shape != X.shape or Xtilde.stride(0) != X.stride(0) or H.shape != (n, n) or dXXT.shape != (n, n) \
            or H.stride(0) != dXXT.stride(0):
        raise GptaqError(f"{name}: shape mismatch")
    _check(getattr(load(), name)(_ptr(X), _ptr(Xtilde), tokens, n, X.stride(0), _ptr(H), _ptr(dXXT),
                                 H.stride(0), _ptr(ws), ws.numel(), _stream()), name)


def gptaq_accumulate(X: torch.Tensor, Xtilde: torch.Tensor, H: torch.Tensor, dXXT: torch.Tensor,
                     ws: torch.Tensor) -> None:
    """H += X^T X (upper triangle), dXXT += (Xtilde - X)^T X for token-major bf16 X, Xtilde."""
    _accumulate("gptaq_accumulate", X, Xtilde, H, dXXT, ws)


def gptaq_accumulate_upper(X: torch.Tensor, Xtilde: torch.Tensor, H: torch.Tensor, dXXT: torch.Tensor,
                           ws: torch.Tensor) -> None:
    """gptaq_accumulate that maintains only the entries of dXXT with col >= row (natural column order)."""
    _accumulate("gptaq_accumulate_upper", X, Xtilde, H, dXXT, ws)


def gptaq_accumulate_noalloc(X: torch.Tensor, Xtilde: torch.Tensor, H: torch.Tensor, dXXT: torch.Tensor) -> None:
    """gptaq_accumulate on the library's built-in scratch array (no workspace, no allocation; n <= 16384)."""
    _need(X, torch.bfloat16, "X"); _need(Xtilde, torch.bfloat16, "Xtilde")
    _need(H, torch.float32, "H"); _need(dXXT, torch.float32, "dXXT")
    tokens, n = X.shape
    if Xtilde.shape != X.shape or Xtilde.stride(0) != X.stride(0) or H.shape != (n, n) or dXXT.shape != (n, n) \
            or H.stride(0) != dXXT.stride(0):
        raise GptaqError("gptaq_accumulate_noalloc: shape mismatch")
    _check(load().gptaq_accumulate_noalloc(_ptr(X), _ptr(Xtilde), tokens, n, X.stride(0), _ptr(H), _ptr(dXXT),
                                           H.stride(0), _stream()), "gptaq_accumulate_noalloc")


def gptaq_accumulate_staged(X: Optional[torch.Tensor], Xtilde: Optional[torch.Tensor], H: torch.Tensor, dXXT: torch.Tensor,
                            ws: torch.Tensor, pending: int, flush: bool = False, upper: bool = False) -> int:
    """Appends a chunk to the staged operands in `ws` (products run per 32768 pending tokens or on flush);
    returns the new number of pending tokens.  X, Xtilde may be None with flush=True.
    upper=True calls gptaq_accumulate_staged_upper."""
    fn = "gptaq_accumulate_staged_upper" if upper else "gptaq_accumulate_staged"
    _need(H, torch.float32, "H"); _need(dXXT, torch.float32, "dXXT")
    n = H.shape[0]
    tokens, ldx = 0, n
    if X is not None:
        _need(X, torch.bfloat16, "X"); _need(Xtilde, torch.bfloat16, "Xtilde")
        if X.shape != Xtilde.shape or X.shape[1] != n or X.stride(0) != Xtilde.stride(0) or X.stride(1) != 1:
            raise GptaqError("gptaq_accumulate_staged: shape mismatch")
        tokens, ldx = X.shape[0], X.stride(0)
    if dXXT.shape != (n, n) or H.stride(0) != dXXT.stride(0):
        raise GptaqError("gptaq_accumulate_staged: shape mismatch")
    p = _c.c_int64(int(pending))
    _check(getattr(load(), fn)(_ptr(X), _ptr(Xtilde), tokens, n, ldx, _ptr(H), _ptr(dXXT), H.stride(0),
                               _ptr(ws), ws.numel() * ws.element_size(), _c.byref(p), int(bool(flush)),
                               _stream()), fn)
    return p.value


def gptaq_symmetrize(H: torch.Tensor) -> None:
    _need(H, torch.float32, "H")
    _check(load().gptaq_symmetrize(_ptr(H), H.shape[0], H.stride(0), _stream()), "gptaq_symmetrize")


def gptaq_prepare(H: torch.Tensor, dXXT: torch.Tensor, damp: float, ws: torch.Tensor,
                  dead: Optional[torch.Tensor] = None, info: Optional[torch.Tensor] = None):
    """In place: H -> U = L^T (upper), dXXT -> P (strictly upper).  Returns (dead, info) device tensors."""
    _need(H, torch.float32, "H"); _need(dXXT, torch.float32, "dXXT")
    n = H.shape[0]
    if H.shape != (n, n) or dXXT.shape != (n, n) or H.stride(0) != dXXT.stride(0):
        raise GptaqError("gptaq_prepare: shape mismatch")
    if dead is None:
        dead = torch.empty(n, dtype=torch.uint8, device=H.device)
    if info is None:
        info = torch.empty(2, dtype=torch.int32, device=H.device)
    _check(load().gptaq_prepare(_ptr(H), _ptr(dXXT), n, H.stride(0), float(damp), _ptr(dead), _ptr(info),
                                _ptr(ws), ws.numel(), _stream()), "gptaq_prepare")
    return dead, info


def gptaq_quantize_layer(W: torch.Tensor, U: torch.Tensor, P: torch.Tensor, bits: int, group: int, sym: bool,
                         blocksize: int, ws: torch.Tensor, dead: Optional[torch.Tensor] = None,
                         codes: Optional[torch.Tensor] = None, scales: Optional[torch.Tensor] = None,
                         zeros: Optional[torch.Tensor] = None, terms: int = 3, mse_grid: int = 0, mse_steps: int = 0):
    """In place: W -> dequantised quantised weights.  Returns (codes, scales, zeros).
    terms != 3 goes through gptaq_quantize_layer_terms (1: E term only = GPTQ, P may be None)."""
    _need(W, torch.float32, "W"); _need(U, torch.float32, "U")
    m, n = W.shape
    if P is not None:
        _need(P, torch.float32, "P")
        if P.shape != (n, n) or U.stride(0) != P.stride(0):
            raise GptaqError("gptaq_quantize_layer: shape mismatch")
    if U.shape != (n, n):
        raise GptaqError("gptaq_quantize_layer: shape mismatch")
    G = max(1, n // group) if group > 0 else 1
    if codes is None:
        codes = torch.empty((m, n), dtype=torch.uint8, device=W.device)
    if scales is None:
        scales = torch.empty((m, G), dtype=torch.float32, device=W.device)
    if zeros is None:
        zeros = torch.empty((m, G), dtype=torch.float32, device=W.device)
    args = (_ptr(W), m, n, W.stride(0), _ptr(U), _ptr(P), U.stride(0), _ptr(dead), int(bits), int(group),
            int(bool(sym)), int(blocksize), _ptr(codes), _ptr(scales), _ptr(zeros), _ptr(ws), ws.numel(), _stream())
    if mse_steps > 0:
        _check(load().gptaq_quantize_layer_ex(*args, int(terms), int(mse_grid), int(mse_steps)), "gptaq_quantize_layer_ex")
    elif terms == 3:
        _check(load().gptaq_quantize_layer(*args), "gptaq_quantize_layer")
    else:
        _check(load().gptaq_quantize_layer_terms(*args, int(terms)), "gptaq_quantize_layer_terms")
    return codes, scales, zeros


gptaq_quantize_layer_terms = gptaq_quantize_layer
gptaq_quantize_layer_ex = gptaq_quantize_layer


def gptaq_profile_enable(mask: int) -> None:
    """Record the kernels whose tag bit (1 << tag) is set in `mask`; 0 switches recording off."""
    _check(load().gptaq_profile_enable(int(mask)), "gptaq_profile_enable")


def gptaq_profile_read(tag: int):
    """(launches, total milliseconds) of the kernels bracketed under `tag` since profiling was enabled."""
    n, ms = _c.c_int64(0), _c.c_double(0.0)
    _check(load().gptaq_profile_read(int(tag), _c.byref(n), _c.byref(ms)), "gptaq_profile_read")
    return n.value, ms.value


def gptaq_measure_mfma_peak(random_data: bool, millis: int = 50):
    """(TFLOP/s, core clock in GHz) of a pure bf16 MFMA loop on every CU, on all-ones or on random operands."""
    ws = workspace(1 << 20)
    tf, ghz = _c.c_double(0.0), _c.c_double(0.0)
    _check(load().gptaq_measure_mfma_peak(int(bool(random_data)), int(millis), _ptr(ws), ws.numel() * ws.element_size(),
                                          _c.byref(tf), _c.byref(ghz), _stream()), "gptaq_measure_mfma_peak")
    return tf.value, ghz.value


def gptaq_measure_hbm_copy(nbytes: int = 1 << 30, reps: int = 10) -> float:
    """GB/s (read + written) of a plain streaming copy of `nbytes`."""
    ws = workspace(2 * nbytes)
    g = _c.c_double(0.0)
    _check(load().gptaq_measure_hbm_copy(int(nbytes), int(reps), _ptr(ws), ws.numel() * ws.element_size(), _c.byref(g),
                                         _stream()), "gptaq_measure_hbm_copy")
    return g.value


def gptaq_act_order(H: torch.Tensor) -> torch.Tensor:
    """perm (int32, device): inputs in the order of decreasing H[i][i]; a 1-D H is the diagonal itself."""
    if H.dim() == 1:
        _need_vec(H, torch.float32, "H")
    else:
        _need(H, torch.float32, "H")
    n = H.shape[0]
    perm = torch.empty(n, dtype=torch.int32, device=H.device)
    _check(load().gptaq_act_order(_ptr(H), n, H.stride(0) if H.dim() == 2 else 0, _ptr(perm), _stream()), "gptaq_act_order")
    return perm


def gptaq_accumulate_diag(X: torch.Tensor, diag: torch.Tensor) -> None:
    """diag[j] += sum_t X[t][j]^2 (the diagonal of H) for token-major bf16 X."""
    _need(X, torch.bfloat16, "X"); _need_vec(diag, torch.float32, "diag")
    tokens, n = X.shape
    if diag.shape != (n,):
        raise GptaqError("gptaq_accumulate_diag: shape mismatch")
    _check(load().gptaq_accumulate_diag(_ptr(X), tokens, n, X.stride(0), _ptr(diag), _stream()), "gptaq_accumulate_diag")


def gptaq_invert_permutation(perm: torch.Tensor) -> torch.Tensor:
    """inv with inv[perm[r]] = r (int32, device)."""
    if perm.dtype != torch.int32 or perm.dim() != 1 or not perm.is_contiguous():
        raise GptaqError("gptaq_invert_permutation: perm must be a contiguous int32 vector")
    inv = torch.empty_like(perm)
    _check(load().gptaq_invert_permutation(_ptr(perm), perm.numel(), _ptr(inv), _stream()), "gptaq_invert_permutation")
    return inv


def gptaq_accumulate_upper_permuted(X: torch.Tensor, Xtilde: torch.Tensor, inv_perm: torch.Tensor, H: torch.Tensor,
                                    dXXT: torch.Tensor, ws: torch.Tensor) -> None:
    """gptaq_accumulate_upper on the inputs with their channels reordered: input channel j is row / column inv_perm[j]."""
    _need(X, torch.bfloat16, "X"); _need(Xtilde, torch.bfloat16, "Xtilde")
    _need(H, torch.float32, "H"); _need(dXXT, torch.float32, "dXXT")
    tokens, n = X.shape
    if Xtilde.shape != X.shape or Xtilde.stride(0) != X.stride(0) or H.shape != (n, n) or dXXT.shape != (n, n) \
            or H.stride(0) != dXXT.stride(0) or inv_perm.dtype != torch.int32 or inv_perm.shape != (n,) \
            or not inv_perm.is_contiguous():
        raise GptaqError("gptaq_accumulate_upper_permuted: shape mismatch")
    _check(load().gptaq_accumulate_upper_permuted(_ptr(X), _ptr(Xtilde), tokens, n, X.stride(0), _ptr(inv_perm), _ptr(H),
                                                  _ptr(dXXT), H.stride(0), _ptr(ws), ws.numel(), _stream()),
           "gptaq_accumulate_upper_permuted")


def gptaq_permute_hessian_workspace_bytes(n: int) -> int:
    return load().gptaq_permute_hessian_workspace_bytes(n)


def gptaq_permute_hessian(H: torch.Tensor, dXXT: torch.Tensor, perm: torch.Tensor, ws: torch.Tensor) -> None:
    _need(H, torch.float32, "H"); _need(dXXT, torch.float32, "dXXT")
    n = H.shape[0]
    if dXXT.shape != (n, n) or H.stride(0) != dXXT.stride(0) or perm.dtype != torch.int32 or perm.numel() != n:
        raise GptaqError("gptaq_permute_hessian: shape mismatch")
    _check(load().gptaq_permute_hessian(_ptr(H), _ptr(dXXT), n, H.stride(0), _ptr(perm), _ptr(ws), ws.numel(),
                                        _stream()), "gptaq_permute_hessian")


def _permute_columns(fn, name, src: torch.Tensor, perm: torch.Tensor, inverse: bool) -> torch.Tensor:
    if src.dim() != 2 or src.stride(1) != 1 or perm.dtype != torch.int32 or perm.numel() != src.shape[1]:
        raise GptaqError(f"{name}: shape mismatch")
    out = torch.empty_like(src, memory_format=torch.contiguous_format)
    m, n = src.shape
    _check(fn(_ptr(src), _ptr(out), m, n, src.stride(0), out.stride(0), _ptr(perm), int(bool(inverse)), _stream()), name)
    return out


def gptaq_permute_columns_f32(src: torch.Tensor, perm: torch.Tensor, inverse: bool = False) -> torch.Tensor:
    if src.dtype != torch.float32:
        raise GptaqError("gptaq_permute_columns_f32: expected float32")
    return _permute_columns(load().gptaq_permute_columns_f32, "gptaq_permute_columns_f32", src, perm, inverse)


def gptaq_permute_columns_u8(src: torch.Tensor, perm: torch.Tensor, inverse: bool = False) -> torch.Tensor:
    if src.dtype != torch.uint8:
        raise GptaqError("gptaq_permute_columns_u8: expected uint8")
    return _permute_columns(load().gptaq_permute_columns_u8, "gptaq_permute_columns_u8", src, perm, inverse)


def gptaq_fake_quant_activations(X: torch.Tensor, bits: int, clip: float = 0.9) -> torch.Tensor:
    """Per-token asymmetric fake quantisation of bf16 activations (Section 5.1); returns a new tensor."""
    _need(X, torch.bfloat16, "X")
    Y = torch.empty_like(X, memory_format=torch.contiguous_format)
    tokens, n = X.shape
    _check(load().gptaq_fake_quant_activations(_ptr(X), _ptr(Y), tokens, n, X.stride(0), Y.stride(0), int(bits),
                                               float(clip), _stream()), "gptaq_fake_quant_activations")
    return Y


def gptaq_packed_words_per_row(n: int, bits: int) -> int:
    return load().gptaq_packed_words_per_row(n, bits)


def gptaq_pack_codes(codes: torch.Tensor, bits: int) -> torch.Tensor:
    """(m x n) uint8 codes -> (m x ceil(n*bits/32)) int32 words, code j of a row in bits [j*bits, (j+1)*bits)."""
    if codes.dtype != torch.uint8 or codes.dim() != 2 or codes.stride(1) != 1 or not codes.is_cuda:
        raise GptaqError("gptaq_pack_codes: expected a 2-D row-major uint8 CUDA tensor")
    m, n = codes.shape
    out = torch.empty((m, gptaq_packed_words_per_row(n, bits)), dtype=torch.int32, device=codes.device)
    _check(load().gptaq_pack_codes(_ptr(codes), m, n, codes.stride(0), int(bits), _ptr(out), _stream()),
           "gptaq_pack_codes")
    return out

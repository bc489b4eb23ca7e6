"""ctypes binding of include/ec_moe.h.  Same names as the C entry points.

Tensors are torch tensors on the GPU (torch owns device memory and streams,
nothing else); shapes and the storage type are read off the tensors, pointers
are passed as raw addresses, the current torch stream is passed as the HIP
stream.  A non-zero status raises EcMoeError.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_double, c_int, c_int64, c_size_t, c_void_p
from typing import Optional

import torch

EC_F32, EC_BF16, EC_BF16_HILO = 0, 1, 2
EC_ACT_RELU, EC_ACT_GELU, EC_ACT_IDENTITY = 0, 1, 2
EC_MOE_MAX_EXPERTS = 1024

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libec_moe.so"
_lib: Optional[ctypes.CDLL] = None


class EcMoeError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        name = lib().ec_moe_status_string(status).decode()
        extra = f" (hipError {lib().ec_moe_last_hip_error()})" if status == -3 else ""
        super().__init__(f"{fn} failed: {name}{extra}")


def lib_path() -> str:
    return os.path.join(_PKG_DIR, _LIB_NAME)


_P, _I64, _SZ = c_void_p, c_int64, c_size_t
_SIGNATURES = {
    "ec_moe_capacity": (c_int, [_I64, _I64, c_double, ctypes.POINTER(c_int64)]),
    "ec_moe_workspace_bytes": (c_size_t, [_I64, _I64, _I64, _I64, _I64, c_int, c_int]),
    "ec_moe_gate": (c_int, [_P, _P, _P, _P, _I64, _I64, _I64, c_int, _P, _SZ, _P]),
    "ec_moe_topk_tokens": (c_int, [_P, _I64, _I64, _I64, _P, _P, _P, _SZ, _P]),
    "ec_moe_dispatch": (c_int, [_P, _P, _P, _I64, _I64, _I64, _I64, c_int, _P]),
    "ec_moe_expert_ffn": (c_int, [_P, _P, _P, _P, _P, _P, _I64, _I64, _I64, _I64, c_int, c_int, _P, _SZ, _P]),
    "ec_moe_combine": (c_int, [_P, _P, _P, _P, _I64, _I64, _I64, _I64, c_int, _P, _SZ, _P]),
    "ec_moe_combine_static": (c_int, [_P, _P, _P, _P, _I64, _I64, _I64, _I64, c_int, _P]),
    "ec_moe_forward": (c_int, [_P, _P, _P, _P, c_double, _P, _P, _P, _P, _P, _P, _P, _P,
                               _I64, _I64, _I64, _I64, c_int, c_int, _P, _SZ, _P]),
    "ec_moe_topk_tokens_grouped": (c_int, [_P, _I64, _I64, _I64, _I64, _P, _P, _P, _SZ, _P]),
    "ec_moe_forward_grouped": (c_int, [_P, _P, _P, _P, c_double, _I64, _P, _P, _P, _P, _P, _P, _P, _P,
                                       _I64, _I64, _I64, _I64, c_int, c_int, _P, _SZ, _P]),
    "ec_moe_token_choice": (c_int, [_P, _I64, _I64, _I64, _I64, _P, _P, _P, _P, _SZ, _P]),
    "ec_moe_forward_token_choice": (c_int, [_P, _P, _P, _P, c_double, _I64, _P, _P, _P, _P, _P, _P, _P, _P, _P,
                                            _I64, _I64, _I64, _I64, c_int, c_int, _P, _SZ, _P]),
    "ec_moe_capped_workspace_bytes": (c_size_t, [_I64, _I64]),
    "ec_moe_capped_assignment": (c_int, [_P, _I64, _I64, _I64, c_double, c_double, _I64, _P, _P, _SZ, _P]),
    "ec_moe_forward_capped": (c_int, [_P, _P, _P, _P, c_double, c_double, c_double, _I64, _P, _P, _P, _P, _P, _P,
                                      _I64, _I64, _I64, _I64, c_int, c_int, _P, _SZ, _P]),
    "ec_moe_backward": (c_int, [_P] * 16 + [_I64] * 5 + [c_int, c_int, _P, _SZ, _P]),
    "ec_moe_backward_timed": (c_int, [_P] * 16 + [_I64] * 5 + [c_int, c_int, _P, _SZ, _P, ctypes.POINTER(ctypes.c_float)]),
    "ec_moe_backward_stage_name": (c_char_p, [c_int]),
    "ec_moe_last_hip_error": (c_int, []),
    "ec_moe_status_string": (c_char_p, [c_int]),
    "ec_moe_version": (c_char_p, []),
}


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(
                f"{path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
                "There is no fallback path.")
        handle = ctypes.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


# ------------------------------------------------------------------ helpers --
def _dtype_code(t: torch.Tensor, hilo: bool = False) -> int:
    """ec_dtype of a tensor; hilo asks for EC_BF16_HILO (bf16 storage, two-part matrix-core operands)."""
    if t.dtype == torch.float32:
        if hilo:
            raise TypeError("hilo applies to bf16 storage")
        return EC_F32
    if t.dtype == torch.bfloat16:
        return EC_BF16_HILO if hilo else EC_BF16
    raise TypeError(f"unsupported storage type {t.dtype}")


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous and live on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _ws(ws: Optional[torch.Tensor]):
    if ws is None:
        return None, 0
    if ws.dtype != torch.uint8:
        raise TypeError("workspace must be a uint8 tensor")
    return _ptr(ws), ws.numel()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise EcMoeError(fn, status)


# ------------------------------------------------------------- entry points --
def ec_moe_capacity(n: int, e: int, c: float) -> int:
    k = c_int64(0)
    _check("ec_moe_capacity", lib().ec_moe_capacity(n, e, c, ctypes.byref(k)))
    return int(k.value)


def ec_moe_workspace_bytes(n: int, d: int, e: int, k: int, d_ff: int, dtype: int, with_backward: bool = False) -> int:
    return int(lib().ec_moe_workspace_bytes(n, d, e, k, d_ff, dtype, int(with_backward)))


def alloc_workspace(n: int, d: int, e: int, k: int, d_ff: int, dtype: int, with_backward: bool = False,
                    device="cuda") -> torch.Tensor:
    size = ec_moe_workspace_bytes(n, d, e, k, d_ff, dtype, with_backward)
    if size == 0:
        raise ValueError("invalid sizes for a workspace")
    return torch.empty(size, dtype=torch.uint8, device=device)


def ec_moe_gate(X, Wg, S, St, ws) -> None:
    n, d = X.shape
    e = Wg.shape[1]
    wp, wb = _ws(ws)
    _check("ec_moe_gate", lib().ec_moe_gate(_ptr(X), _ptr(Wg, X.dtype), _ptr(S, torch.float32),
                                            _ptr(St, torch.float32), n, d, e, _dtype_code(X), wp, wb, _stream()))


def ec_moe_topk_tokens(St, k: int, G, I, ws) -> None:
    e, n = St.shape
    wp, wb = _ws(ws)
    _check("ec_moe_topk_tokens", lib().ec_moe_topk_tokens(_ptr(St, torch.float32), n, e, k, _ptr(G, torch.float32),
                                                          _ptr(I, torch.int32), wp, wb, _stream()))


def ec_moe_dispatch(X, I, Xin) -> None:
    n, d = X.shape
    e, k = I.shape
    _check("ec_moe_dispatch", lib().ec_moe_dispatch(_ptr(X), _ptr(I, torch.int32), _ptr(Xin, X.dtype), n, d, e, k,
                                                    _dtype_code(X), _stream()))


def ec_moe_expert_ffn(Xin, W1, W2, Xe, act: int, ws, A_save=None, H_save=None, hilo: bool = False) -> None:
    e, k, d = Xin.shape
    d_ff = W1.shape[2]
    wp, wb = _ws(ws)
    dt = Xin.dtype
    _check("ec_moe_expert_ffn", lib().ec_moe_expert_ffn(_ptr(Xin), _ptr(W1, dt), _ptr(W2, dt), _ptr(Xe, dt),
                                                        _ptr(A_save, dt), _ptr(H_save, dt), e, k, d, d_ff, act,
                                                        _dtype_code(Xin, hilo), wp, wb, _stream()))


def ec_moe_combine(Xe, G, I, Xout, ws) -> None:
    e, k, d = Xe.shape
    n = Xout.shape[0]
    wp, wb = _ws(ws)
    _check("ec_moe_combine", lib().ec_moe_combine(_ptr(Xe), _ptr(G, torch.float32), _ptr(I, torch.int32),
                                                  _ptr(Xout, Xe.dtype), n, d, e, k, _dtype_code(Xe), wp, wb,
                                                  _stream()))


def ec_moe_combine_static(Xe, G, I, Xout) -> None:
    e, k, d = Xe.shape
    n = Xout.shape[0]
    _check("ec_moe_combine_static", lib().ec_moe_combine_static(
        _ptr(Xe), _ptr(G, torch.float32), _ptr(I, torch.int32), _ptr(Xout, Xe.dtype), n, d, e, k, _dtype_code(Xe),
        _stream()))


def ec_moe_forward(X, Wg, W1, W2, c: float, Xout, act: int, ws, S_out=None, G_out=None, I_out=None,
                   Xin_out=None, A_out=None, H_out=None, Xe_out=None, hilo: bool = False) -> None:
    n, d = X.shape
    e = Wg.shape[1]
    d_ff = W1.shape[2] if W1 is not None else 0
    wp, wb = _ws(ws)
    dt = X.dtype
    _check("ec_moe_forward", lib().ec_moe_forward(
        _ptr(X), _ptr(Wg, dt), _ptr(W1, dt), _ptr(W2, dt), c, _ptr(Xout, dt), _ptr(S_out, torch.float32),
        _ptr(G_out, torch.float32), _ptr(I_out, torch.int32), _ptr(Xin_out, dt), _ptr(A_out, dt), _ptr(H_out, dt),
        _ptr(Xe_out, dt), n, d, e, d_ff, act, _dtype_code(X, hilo), wp, wb, _stream()))


def ec_moe_topk_tokens_grouped(St, groups: int, k_g: int, G, I, ws=None) -> None:
    e, n = St.shape
    wp, wb = _ws(ws)
    _check("ec_moe_topk_tokens_grouped", lib().ec_moe_topk_tokens_grouped(
        _ptr(St, torch.float32), n, e, groups, k_g, _ptr(G, torch.float32), _ptr(I, torch.int32), wp, wb, _stream()))


def ec_moe_forward_grouped(X, Wg, W1, W2, c: float, groups: int, Xout, act: int, ws, S_out=None, G_out=None,
                           I_out=None, Xin_out=None, A_out=None, H_out=None, Xe_out=None, hilo: bool = False) -> None:
    n, d = X.shape
    e = Wg.shape[1]
    d_ff = W1.shape[2] if W1 is not None else 0
    wp, wb = _ws(ws)
    dt = X.dtype
    _check("ec_moe_forward_grouped", lib().ec_moe_forward_grouped(
        _ptr(X), _ptr(Wg, dt), _ptr(W1, dt), _ptr(W2, dt), c, groups, _ptr(Xout, dt), _ptr(S_out, torch.float32),
        _ptr(G_out, torch.float32), _ptr(I_out, torch.int32), _ptr(Xin_out, dt), _ptr(A_out, dt), _ptr(H_out, dt),
        _ptr(Xe_out, dt), n, d, e, d_ff, act, _dtype_code(X, hilo), wp, wb, _stream()))


def ec_moe_token_choice(S, m: int, cap: int, G, I, load, ws) -> None:
    n, e = S.shape
    wp, wb = _ws(ws)
    _check("ec_moe_token_choice", lib().ec_moe_token_choice(
        _ptr(S, torch.float32), n, e, m, cap, _ptr(G, torch.float32), _ptr(I, torch.int32), _ptr(load, torch.int32),
        wp, wb, _stream()))


def ec_moe_forward_token_choice(X, Wg, W1, W2, c: float, m: int, Xout, act: int, ws, S_out=None, G_out=None,
                                I_out=None, load_out=None, Xin_out=None, A_out=None, H_out=None, Xe_out=None,
                                hilo: bool = False) -> None:
    n, d = X.shape
    e = Wg.shape[1]
    d_ff = W1.shape[2] if W1 is not None else 0
    wp, wb = _ws(ws)
    dt = X.dtype
    _check("ec_moe_forward_token_choice", lib().ec_moe_forward_token_choice(
        _ptr(X), _ptr(Wg, dt), _ptr(W1, dt), _ptr(W2, dt), c, m, _ptr(Xout, dt), _ptr(S_out, torch.float32),
        _ptr(G_out, torch.float32), _ptr(I_out, torch.int32), _ptr(load_out, torch.int32), _ptr(Xin_out, dt),
        _ptr(A_out, dt), _ptr(H_out, dt), _ptr(Xe_out, dt), n, d, e, d_ff, act, _dtype_code(X, hilo), wp, wb, _stream()))


def ec_moe_capped_workspace_bytes(n: int, e: int) -> int:
    return int(lib().ec_moe_capped_workspace_bytes(n, e))


def ec_moe_capped_assignment(St, k: int, b: float, lam: float, iters: int, A, ws) -> None:
    e, n = St.shape
    wp, wb = _ws(ws)
    _check("ec_moe_capped_assignment", lib().ec_moe_capped_assignment(
        _ptr(St, torch.float32), n, e, k, b, lam, iters, _ptr(A, torch.float32), wp, wb, _stream()))


def ec_moe_forward_capped(X, Wg, W1, W2, c: float, b: float, lam: float, iters: int, Xout, act: int, ws,
                          S_out=None, G_out=None, I_out=None, A_out=None, Xe_out=None, hilo: bool = False) -> None:
    n, d = X.shape
    e = Wg.shape[1]
    d_ff = W1.shape[2] if W1 is not None else 0
    wp, wb = _ws(ws)
    dt = X.dtype
    _check("ec_moe_forward_capped", lib().ec_moe_forward_capped(
        _ptr(X), _ptr(Wg, dt), _ptr(W1, dt), _ptr(W2, dt), c, b, lam, iters, _ptr(Xout, dt),
        _ptr(S_out, torch.float32), _ptr(G_out, torch.float32), _ptr(I_out, torch.int32), _ptr(A_out, torch.float32),
        _ptr(Xe_out, dt), n, d, e, d_ff, act, _dtype_code(X, hilo), wp, wb, _stream()))


def ec_moe_backward(dY, X, Wg, W1, W2, S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2, act: int, ws, hilo: bool = False) -> None:
    n, d = X.shape
    e, k = I.shape
    d_ff = W1.shape[2]
    wp, wb = _ws(ws)
    dt = X.dtype
    f32 = torch.float32
    _check("ec_moe_backward", lib().ec_moe_backward(
        _ptr(dY, dt), _ptr(X), _ptr(Wg, dt), _ptr(W1, dt), _ptr(W2, dt), _ptr(S, f32), _ptr(G, f32),
        _ptr(I, torch.int32), _ptr(Xin, dt), _ptr(A, dt), _ptr(H, dt), _ptr(Xe, dt), _ptr(dX, dt), _ptr(dWg, f32),
        _ptr(dW1, f32), _ptr(dW2, f32), n, d, e, k, d_ff, act, _dtype_code(X, hilo), wp, wb, _stream()))


EC_MOE_BWD_STAGES = 9


def ec_moe_backward_timed(dY, X, Wg, W1, W2, S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2, act: int, ws,
                          hilo: bool = False) -> dict:
    """ec_moe_backward with HIP events between its stages; waits, returns {stage name: milliseconds}."""
    n, d = X.shape
    e, k = I.shape
    d_ff = W1.shape[2]
    wp, wb = _ws(ws)
    dt = X.dtype
    f32 = torch.float32
    ms = (ctypes.c_float * EC_MOE_BWD_STAGES)()
    _check("ec_moe_backward_timed", lib().ec_moe_backward_timed(
        _ptr(dY, dt), _ptr(X), _ptr(Wg, dt), _ptr(W1, dt), _ptr(W2, dt), _ptr(S, f32), _ptr(G, f32),
        _ptr(I, torch.int32), _ptr(Xin, dt), _ptr(A, dt), _ptr(H, dt), _ptr(Xe, dt), _ptr(dX, dt), _ptr(dWg, f32),
        _ptr(dW1, f32), _ptr(dW2, f32), n, d, e, k, d_ff, act, _dtype_code(X, hilo), wp, wb, _stream(), ms))
    return {lib().ec_moe_backward_stage_name(i).decode(): float(ms[i]) for i in range(EC_MOE_BWD_STAGES)}


def ec_moe_last_hip_error() -> int:
    return int(lib().ec_moe_last_hip_error())


def ec_moe_status_string(status: int) -> str:
    return lib().ec_moe_status_string(status).decode()


def ec_moe_version() -> str:
    return lib().ec_moe_version().decode()

"""Helpers for the GPU parity tests: host<->device marshalling and error metrics."""
from __future__ import annotations

import numpy as np
import torch

import workloads as wl


def sized(base: wl.Workload, **kw) -> wl.Workload:
    """A resized copy of a workload with k taken from the library's own host function (Eq. 1)."""
    import paper_2202_09368_amd as m
    w = wl.scaled(base, **kw)
    return w if w.k is not None else wl.scaled(w, k=m.ec_moe_capacity(w.n, w.e, w.c))


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy (float32 / int32 / uint16 bf16 bits) -> tensor on cuda:0 (bf16 for uint16)."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    """Tensor -> numpy; bf16 comes back as uint16 bit patterns."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def to_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return wl.bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def max_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max(|ref|, rms(ref)): relative error with an rms floor near zero."""
    got, ref = to_f64(got), np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den)) if ref.size else 0.0


def torch_dtype(w: wl.Workload):
    return torch.bfloat16 if w.dtype == wl.DTYPE_BF16 else torch.float32


# tolerances of the parity bar: fp32 outputs 1e-5, bf16 outputs 2e-2 (vs. a reference
# without intermediate rounding), scores S always fp32
def out_tol(w: wl.Workload) -> float:
    return 2e-2 if w.dtype == wl.DTYPE_BF16 else 1e-5


def score_tolerance(X: np.ndarray, Wg: np.ndarray) -> np.ndarray:
    """Per-token relative tolerance on the fp32 scores S.

    A logit is a length-d sum accumulated in fp32, so its absolute error is bounded to first order
    by a small multiple of u * sum_t |x_t w_t| (u = 2^-24), and a relative error of S equals an
    absolute error of (logit - logsumexp).  The bar is the stated 1e-5 plus 2u * max_i sum_t |x_t||w_ti|:
    about 1.2e-5 for unit-variance tokens, and proportionally more for tokens scaled up to skew the
    routing, whose logits are ten times larger.
    """
    a = np.abs(to_f64(X)) @ np.abs(to_f64(Wg))          # [n,e]
    return 1e-5 + 2.0 * 2.0 ** -24 * a.max(axis=1)


def max_rel_err_rows(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """Row-wise max |got - ref| / max(|ref|, rms(ref)) (rms over the whole tensor)."""
    got, ref = to_f64(got), np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return (np.abs(got - ref) / np.maximum(np.abs(ref), max(rms, 1e-300))).max(axis=1)

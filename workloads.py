"""Seeded synthetic inputs for the expert-choice MoE layer.

This module only draws numbers and converts storage formats.  It contains none
of the layer's arithmetic (no softmax, no top-k, no matmul) so that both the
CPU oracle's tests and the HIP path's tests/bench can consume identical bits
without sharing any of the method's code.

Shapes follow the paper's problem statement (Sec. 3.2): token matrix X[n,d],
expert embeddings W_g[d,e], expert weights W1[e,d,d_ff] and W2[e,d_ff,d];
Table 1 gives the 0.1B/16E layer (d=768, d_ff=3072, 16 experts) that the
"cfg2" workload reproduces.  Everything is i.i.d. Gaussian; the second
parameter of N(., .) in the workload descriptions is a variance.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

ACT_RELU = 0
ACT_GELU = 1
ACT_IDENTITY = 2

DTYPE_F32 = 0
DTYPE_BF16 = 1


@dataclass(frozen=True)
class Workload:
    name: str
    n: int          # tokens (batch x sequence)
    d: int          # model width
    e: int          # experts
    c: float        # capacity factor
    d_ff: int       # expert hidden width (0: identity experts, routing only)
    act: int
    dtype: int
    seed: int
    skew_frac: float = 0.0   # fraction of token rows multiplied by skew_scale
    skew_scale: float = 1.0
    backward: bool = False
    k: Optional[int] = None  # tokens per expert: a number the caller supplies (the workload descriptions print it;
                             # resized copies get it from whichever implementation is under test), never computed here


# The five workloads the build is measured and parity-checked on.
WORKLOADS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", n=256, d=64, e=8, c=2.0, d_ff=256, act=ACT_RELU,
                     dtype=DTYPE_F32, seed=0, k=64),
    "cfg2": Workload("cfg2", n=8192, d=768, e=16, c=2.0, d_ff=3072, act=ACT_GELU,
                     dtype=DTYPE_BF16, seed=2, k=1024),
    "cfg3": Workload("cfg3", n=16384, d=1024, e=64, c=2.0, d_ff=4096, act=ACT_GELU,
                     dtype=DTYPE_BF16, seed=3, k=512),
    "cfg4": Workload("cfg4", n=32768, d=2048, e=128, c=2.0, d_ff=8192, act=ACT_GELU,
                     dtype=DTYPE_BF16, seed=4, backward=True, k=512),
    "cfg5": Workload("cfg5", n=65536, d=4096, e=256, c=1.0, d_ff=0, act=ACT_IDENTITY,
                     dtype=DTYPE_BF16, seed=5, skew_frac=0.01, skew_scale=10.0, k=256),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (reduced parity sizes).  When n, e or c change the
    stored k no longer applies: pass the new k, or it is left unset for the caller to fill in."""
    if "k" not in kw and any(key in kw and kw[key] != getattr(w, key) for key in ("n", "e", "c")):
        kw["k"] = None
    return replace(w, **kw)


# ----------------------------------------------------------------------------
# bf16 storage helpers (numpy has no bfloat16: bf16 tensors travel as uint16).
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


_CHUNKED_ABOVE = 1 << 28  # elements; larger tensors are drawn slice by slice along the first axis


def _normal_stored(rng: np.random.Generator, shape, std: float, bf16: bool) -> np.ndarray:
    """Like _normal, then the storage conversion.  Very large tensors (the 128-expert weights) are drawn
    one leading slice at a time from the same stream, which keeps the temporaries small."""
    count = int(np.prod(shape))
    if count <= _CHUNKED_ABOVE:
        a = _normal(rng, shape, std)
        return f32_to_bf16_bits(a) if bf16 else a
    out = np.empty(shape, dtype=np.uint16 if bf16 else np.float32)
    for i in range(shape[0]):
        a = _normal(rng, shape[1:], std)
        out[i] = f32_to_bf16_bits(a) if bf16 else a
    return out


def make_inputs(w: Workload, with_dy: Optional[bool] = None) -> Dict[str, np.ndarray]:
    """Draw X, Wg, W1, W2 (and dY for backward workloads) for a workload.

    One independent PCG64 stream per tensor, spawned in a fixed order from the
    workload's seed, so a tensor's bits do not depend on the others' shapes.
    Returned arrays are float32 for DTYPE_F32 workloads and uint16 bfloat16 bit
    patterns for DTYPE_BF16 workloads (values drawn in float32, then rounded).
    """
    ss = np.random.SeedSequence(w.seed)
    s_x, s_wg, s_w1, s_w2, s_dy, s_mask = ss.spawn(6)
    out: Dict[str, np.ndarray] = {}

    X = _normal(np.random.default_rng(s_x), (w.n, w.d), 1.0)
    if w.skew_frac > 0.0:
        m = int(round(w.n * w.skew_frac))
        rows = np.random.default_rng(s_mask).choice(w.n, size=m, replace=False)
        X[rows, :] *= np.float32(w.skew_scale)
        out["skew_rows"] = np.sort(rows).astype(np.int64)
    out["X"] = X
    out["Wg"] = _normal(np.random.default_rng(s_wg), (w.d, w.e), (1.0 / w.d) ** 0.5)
    bf16 = w.dtype == DTYPE_BF16
    if w.d_ff > 0:
        out["W1"] = _normal_stored(np.random.default_rng(s_w1), (w.e, w.d, w.d_ff), (1.0 / w.d) ** 0.5, bf16)
        out["W2"] = _normal_stored(np.random.default_rng(s_w2), (w.e, w.d_ff, w.d), (1.0 / w.d_ff) ** 0.5, bf16)
    if with_dy if with_dy is not None else w.backward:
        out["dY"] = _normal(np.random.default_rng(s_dy), (w.n, w.d), 1.0)

    if bf16:
        for key in ("X", "Wg", "dY"):
            if key in out:
                out[key] = f32_to_bf16_bits(out[key])
    return out


def as_float(a: np.ndarray) -> np.ndarray:
    """float32 view of an input tensor whatever its storage (bf16 bits or f32)."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a)
    return np.asarray(a, dtype=np.float32)

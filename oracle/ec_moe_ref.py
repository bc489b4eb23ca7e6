"""CPU oracle for the expert-choice MoE layer (TEST INFRASTRUCTURE ONLY).

A plain, slow, float64 numpy statement of what the layer computes, written
from the paper's definitions: capacity (Sec. 3.2, Eq. 1), gating and TopK over
the token axis (Eq. 2), gather and expert FFN (Eq. 3), gate-weighted combine
(Eq. 4).  The backward pass is not printed in the paper; it is the derivative
of Eq. 2-4 with the TopK indices held constant (Sec. 3.4 says the gate is
trained, so gradient reaches W_g through the selected gate values G).

Only tests, the smoke check and the bench's cpu_baseline leg may import this
module.  It shares no code with the HIP path and must never be used by it.

Conventions (paper notation):
  X[n,d]  tokens;  Wg[d,e] expert embeddings;  S[n,e] affinity scores;
  I[e,k] int32 token index of the j-th selected token of expert i;
  G[e,k] gate weight S[I[i,j], i];  X_in[e,k,d];  W1[e,d,d_ff];  W2[e,d_ff,d]
  (the paper keeps W2[i] as [d,d_ff] and multiplies by its transpose; storing
  [d_ff,d] and multiplying untransposed is the same mathematics);
  X_e[e,k,d];  X_out[n,d].

Readings where the paper is silent (each listed in the design notes too):
  * TopK ties go to the lower token index (a token enters a bucket ahead of any
    token with the same score and a higher index).  The paper does not say in
    which order a bucket lists its k tokens ("the j-th selected token"); here a
    bucket is listed by ascending token index.  X_out does not depend on it.
  * k = floor(n*c/e) evaluated in double.
  * Softmax is over the expert axis (one distribution per token).
  * G is the raw score (no renormalisation per token).
  * GeLU is the exact erf form; no biases; tokens chosen by nobody get 0.
  * S is stored in float32 (the interface type); TopK acts on those float32
    values, so ties are decided on float32 bit patterns.

bfloat16 tensors arrive as uint16 bit patterns and are widened exactly.

parity pins: every function here is pinned by tests/test_oracle_pins.py
(brute-force selection, dense one-hot einsum of Eq. 3/4, closed forms for
degenerate routings, textbook dense FFN for e=1, finite differences and an
autograd restatement for the backward; routing per group against the plain
layer run on each group as a batch of its own and a brute-force selection;
token-choice routing against a hand-worked example, a per-token brute force,
the dense top-m mixture when nothing is dropped, and its priority rule;
the capped assignment of Sec. 3.3 against the linear programme solved by a
library LP solver, the closed-form optimum when the cap is slack, and its
constraints).
parity partly unpinned: capped_assignment.  Its fixed point is pinned to the
programme Sec. 3.3 prints, but the paper gives neither the projections nor
what its "maximum of 100 iterations" return, so the iterate after a fixed
number of sweeps follows this file's reading of the algorithm, not a printed
one (see the section's comment).
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Tuple

import numpy as np
from scipy.special import erf as _erf

ACT_RELU = 0
ACT_GELU = 1
ACT_IDENTITY = 2


def widen(a: np.ndarray) -> np.ndarray:
    """float64 copy of a tensor stored as float32/float64 or as bf16 bits."""
    a = np.asarray(a)
    if a.dtype == np.uint16:  # bfloat16 bit pattern: upper half of a float32
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# ------------------------------------------------------------------ Eq. 1 ---
def capacity(n: int, c: float, e: int) -> int:
    """Bucket size k = n*c/e (Sec. 3.2, Eq. 1), floored when not integral."""
    if n <= 0 or e <= 0 or not (c > 0):
        raise ValueError("n, e and c must be positive")
    k = int(math.floor(float(n) * float(c) / float(e)))
    if k < 1 or k > n:
        raise ValueError(f"capacity k={k} outside [1, n={n}]")
    return k


# ------------------------------------------------------------------ Eq. 2 ---
def gate(X: np.ndarray, Wg: np.ndarray, out_dtype=np.float32) -> np.ndarray:
    """S = Softmax(X . Wg) over the expert axis (Sec. 3.2, Eq. 2; Sec. 3.4).

    Returns S[n,e] rounded to float32, the type the interface carries
    (out_dtype=np.float64 keeps the unrounded scores, for derivative checks).
    """
    Z = widen(X) @ widen(Wg)                       # [n,e] token-to-expert logits
    Z = Z - Z.max(axis=1, keepdims=True)           # shift invariance of softmax
    P = np.exp(Z)
    S = P / P.sum(axis=1, keepdims=True)
    return S.astype(out_dtype)


def topk_tokens(S: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """G, I = TopK(S^T, k): every expert takes its k best tokens (Eq. 2).

    S is float32 [n,e].  For expert i the tokens are ranked by descending
    S[:, i]; equal scores rank by ascending token index (stable sort), which
    settles who is admitted at the k-th place.  The k admitted tokens are then
    listed by ascending token index.
    """
    S = np.asarray(S)
    if S.dtype != np.float32:
        raise TypeError("TopK acts on the float32 scores")
    n, e = S.shape
    if not (1 <= k <= n):
        raise ValueError("k outside [1, n]")
    I = np.empty((e, k), dtype=np.int32)
    G = np.empty((e, k), dtype=np.float32)
    for i in range(e):
        col = S[:, i]
        order = np.argsort(-col, kind="stable")    # descending score, ties: low index first
        chosen = np.sort(order[:k])                # the bucket lists its tokens by ascending index
        I[i, :] = chosen
        G[i, :] = col[chosen]
    return G, I


# ------------------------------------------------------------------ Eq. 3 ---
def dispatch(X: np.ndarray, I: np.ndarray) -> np.ndarray:
    """X_in = P . X with P = Onehot(I): X_in[i,j,:] = X[I[i,j],:] (Eq. 3).

    A pure gather; the storage type of X is kept (so it can be compared
    bit for bit).
    """
    X = np.asarray(X)
    return X[np.asarray(I, dtype=np.int64), :]


def activation(A: np.ndarray, act: int) -> np.ndarray:
    if act == ACT_RELU:
        return np.maximum(A, 0.0)
    if act == ACT_GELU:                              # a * Phi(a), exact erf form
        return 0.5 * A * (1.0 + _erf(A / math.sqrt(2.0)))
    if act == ACT_IDENTITY:
        return A
    raise ValueError("unknown activation")


def activation_grad(A: np.ndarray, act: int) -> np.ndarray:
    if act == ACT_RELU:
        return (A > 0.0).astype(np.float64)
    if act == ACT_GELU:                              # Phi(a) + a * phi(a)
        Phi = 0.5 * (1.0 + _erf(A / math.sqrt(2.0)))
        phi = np.exp(-0.5 * A * A) / math.sqrt(2.0 * math.pi)
        return Phi + A * phi
    if act == ACT_IDENTITY:
        return np.ones_like(A)
    raise ValueError("unknown activation")


def expert_ffn(X_in: np.ndarray, W1: np.ndarray, W2: np.ndarray, act: int,
               return_hidden: bool = False):
    """X_e[i] = act(X_in[i] . W1[i]) . W2[i], no bias (Eq. 3).

    W2 is stored [e,d_ff,d] (the paper's W2[i]^T).  float64 throughout, no
    intermediate rounding.
    """
    X_in = widen(X_in)
    e, k, d = X_in.shape
    d_ff = W1.shape[2]
    X_e = np.empty((e, k, d), dtype=np.float64)
    A_all = np.empty((e, k, d_ff), dtype=np.float64) if return_hidden else None
    for i in range(e):
        A = X_in[i] @ widen(W1[i])                  # [k,d_ff]
        H = activation(A, act)
        X_e[i] = H @ widen(W2[i])                   # [k,d]
        if return_hidden:
            A_all[i] = A
    if return_hidden:
        return X_e, A_all
    return X_e


# ------------------------------------------------------------------ Eq. 4 ---
def combine(X_e: np.ndarray, G: np.ndarray, I: np.ndarray, n: int) -> np.ndarray:
    """X_out[l,:] = sum_{i,j} P[i,j,l] G[i,j] X_e[i,j,:] (Eq. 4).

    Tokens that no expert selected keep a zero row.
    """
    X_e = widen(X_e)
    G = widen(G)
    e, k, d = X_e.shape
    X_out = np.zeros((n, d), dtype=np.float64)
    for i in range(e):                              # experts ascending
        for j in range(k):
            X_out[I[i, j], :] += G[i, j] * X_e[i, j, :]
    return X_out


# ------------------------------------------------------------- whole layer ---
def forward(X, Wg, W1, W2, c: float, act: int) -> Dict[str, np.ndarray]:
    """Gate -> TopK over tokens -> gather -> expert FFN -> combine (Eq. 1-4).

    W1 = W2 = None with act = ACT_IDENTITY gives identity experts (routing
    only): X_e = X_in.
    """
    n, d = np.asarray(X).shape
    e = np.asarray(Wg).shape[1]
    k = capacity(n, c, e)
    S = gate(X, Wg)
    G, I = topk_tokens(S, k)
    X_in = dispatch(X, I)
    if W1 is None:
        if act != ACT_IDENTITY:
            raise ValueError("identity experts need act = ACT_IDENTITY")
        X_e = widen(X_in)
    else:
        X_e = expert_ffn(X_in, W1, W2, act)
    X_out = combine(X_e, G, I, n)
    return {"k": k, "S": S, "G": G, "I": I, "X_in": X_in, "X_e": X_e, "X_out": X_out}


# ------------------------------------------------------- routing per group ---
# Limitations section: expert choice looks at every token of the batch, future ones included; the
# proposed remedy is to cut the batch into groups and let every expert choose inside each group
# separately.  Reading taken here: the n tokens are cut into `groups` equal runs of consecutive
# tokens (the caller lays the batch out so that a run is what must be routed together, e.g. one
# position of many sequences); every (expert, group) pair keeps k_g = floor((n/groups)*c/e) tokens;
# an expert's bucket lists group 0's tokens, then group 1's, and so on, each by ascending index.
def topk_tokens_grouped(S: np.ndarray, k_g: int, groups: int) -> Tuple[np.ndarray, np.ndarray]:
    """Per group g and expert i: the k_g best of S[g*n_g:(g+1)*n_g, i]; ties to the lower index.

    Returns G, I of shape [e, groups*k_g]; I holds indices into the whole batch.
    """
    S = np.asarray(S)
    if S.dtype != np.float32:
        raise TypeError("TopK acts on the float32 scores")
    n, e = S.shape
    if groups < 1 or n % groups != 0:
        raise ValueError("the groups must cut the batch into equal parts")
    n_g = n // groups
    if not (1 <= k_g <= n_g):
        raise ValueError("k_g outside [1, n/groups]")
    I = np.empty((e, groups * k_g), dtype=np.int32)
    G = np.empty((e, groups * k_g), dtype=np.float32)
    for g in range(groups):
        first = g * n_g
        for i in range(e):
            col = S[first:first + n_g, i]
            order = np.lexsort((np.arange(n_g), -col.astype(np.float64)))   # by score descending, then index
            chosen = np.sort(order[:k_g]) + first
            I[i, g * k_g:(g + 1) * k_g] = chosen
            G[i, g * k_g:(g + 1) * k_g] = S[chosen, i]
    return G, I


def forward_grouped(X, Wg, W1, W2, c: float, act: int, groups: int) -> Dict[str, np.ndarray]:
    """The layer of Eq. 1-4 with the TopK of Eq. 2 taken inside each group of tokens."""
    n, d = np.asarray(X).shape
    e = np.asarray(Wg).shape[1]
    if groups < 1 or n % groups != 0:
        raise ValueError("the groups must cut the batch into equal parts")
    k_g = capacity(n // groups, c, e)
    S = gate(X, Wg)
    G, I = topk_tokens_grouped(S, k_g, groups)
    X_in = dispatch(X, I)
    if W1 is None:
        if act != ACT_IDENTITY:
            raise ValueError("identity experts need act = ACT_IDENTITY")
        X_e = widen(X_in)
    else:
        X_e = expert_ffn(X_in, W1, W2, act)
    X_out = combine(X_e, G, I, n)
    return {"k_g": k_g, "S": S, "G": G, "I": I, "X_in": X_in, "X_e": X_e, "X_out": X_out}


# ------------------------------------------- token-choice routing (baseline) ---
# Sec. 3.1: in conventional routing every token independently picks its top-m experts (m = 1 in
# Switch Transformer, m = 2 in GShard, Sec. 3.4), an expert can only take a maximum number of tokens,
# and what is routed to it beyond that is dropped.  The paper states no more than this; the reading
# taken here, chosen so that the result is unique and the layer around it is Eq. 3-4 unchanged:
#   * a token's choices are its m largest S[l,:], ties to the lower expert index;
#   * an expert's buffer has `cap` rows; with cap = floor(n*c/e) (Eq. 1) and c = m the buffers are
#     as large as expert choice's at the same cost (Sec. 3.4 compares c = 2 with top-2 gating);
#   * all first choices are placed before any second choice, and inside one rank of choice tokens
#     are placed by ascending token index; a token that finds the buffer full is dropped there;
#   * gate weight = the raw score S[l,i] (no renormalisation over the m choices), as in Eq. 4;
#   * rows of a buffer that stay empty carry I = -1, G = 0 and contribute nothing.
def token_choice(S: np.ndarray, m: int, cap: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Returns G [e,cap] float32, I [e,cap] int32 (-1: empty row) and load [e] int32, the number of
    tokens that chose each expert before anything is dropped (load / cap - 1 is the over-capacity
    ratio of Sec. 3.1)."""
    S = np.asarray(S)
    if S.dtype != np.float32:
        raise TypeError("routing acts on the float32 scores")
    n, e = S.shape
    if not (1 <= m <= e) or cap < 1:
        raise ValueError("m outside [1, e] or empty buffers")
    choice = np.empty((n, m), dtype=np.int64)
    for l in range(n):
        choice[l] = np.argsort(-S[l], kind="stable")[:m]      # descending score, ties: low expert first
    I = np.full((e, cap), -1, dtype=np.int32)
    G = np.zeros((e, cap), dtype=np.float32)
    fill = np.zeros(e, dtype=np.int64)
    load = np.zeros(e, dtype=np.int32)
    for r in range(m):                                         # first choices, then second choices, ...
        for l in range(n):                                     # by ascending token index
            i = choice[l, r]
            load[i] += 1
            if fill[i] < cap:
                I[i, fill[i]] = l
                G[i, fill[i]] = S[l, i]
                fill[i] += 1
    return G, I, load


def dispatch_padded(X: np.ndarray, I: np.ndarray) -> np.ndarray:
    """Eq. 3's gather for buffers with empty rows: X_in[i,j,:] = X[I[i,j],:], zeros where I[i,j] = -1."""
    X = np.asarray(X)
    out = np.zeros(I.shape + (X.shape[1],), dtype=X.dtype)
    filled = I >= 0
    out[filled] = X[I[filled]]
    return out


def combine_padded(X_e: np.ndarray, G: np.ndarray, I: np.ndarray, n: int) -> np.ndarray:
    """Eq. 4 over the filled rows only; ascending expert order per token as in `combine`."""
    X_e = widen(X_e)
    e, k, d = X_e.shape
    X_out = np.zeros((n, d), dtype=np.float64)
    for i in range(e):
        for j in range(k):
            if I[i, j] >= 0:
                X_out[I[i, j], :] += float(G[i, j]) * X_e[i, j, :]
    return X_out


def forward_token_choice(X, Wg, W1, W2, c: float, m: int, act: int) -> Dict[str, np.ndarray]:
    """Gate -> every token's top-m experts with buffers of floor(n*c/e) rows -> Eq. 3 -> Eq. 4."""
    n, d = np.asarray(X).shape
    e = np.asarray(Wg).shape[1]
    cap = capacity(n, c, e)
    S = gate(X, Wg)
    G, I, load = token_choice(S, m, cap)
    X_in = dispatch_padded(X, I)
    if W1 is None:
        if act != ACT_IDENTITY:
            raise ValueError("identity experts need act = ACT_IDENTITY")
        X_e = widen(X_in)
    else:
        X_e = expert_ffn(X_in, W1, W2, act)
    X_out = combine_padded(X_e, G, I, n)
    return {"cap": cap, "S": S, "G": G, "I": I, "load": load, "X_in": X_in, "X_e": X_e, "X_out": X_out}


# ------------------------------------ expert choice with a cap per token ---
# Sec. 3.3: limit the number of experts a token can get.  A[e,n] >= 0 solves the entropy-regularised
# linear programme
#     max <S^T, A> + lambda H(A),   H(A) = -sum A log A,
#     rows sum to k,  columns sum to at most b,  0 <= A <= 1,
# by Dykstra's algorithm, projecting in turn on the three constraint sets (lambda = 0.001, at most
# 100 iterations), and the buckets are TopK(A, k) instead of TopK(S^T, k).  The paper gives neither
# the projections nor a stopping rule.  Reading taken here: since <S^T,A> + lambda H(A) equals
# -lambda KL(A || exp(S^T/lambda)) up to terms fixed by the row sums, the solution is the KL
# projection of the Gibbs kernel exp(S^T/lambda) on the intersection, and Dykstra's algorithm is run
# with KL projections (iterative Bregman projections), which are scalings:
#   rows sum to k      A[i,:] *= k / sum_j A[i,j]                      (affine set: no correction)
#   columns at most b  A[:,j] *= min(1, b / sum_i A[i,j])              (correction q_col[j])
#   entries at most 1  A = min(A, 1)                                   (correction q_box[i,j])
# with the usual Dykstra corrections for the two inequality sets (multiply the correction in before
# projecting, keep input/output as the new correction).  All in the log domain, float64, because
# exp(S/lambda) overflows.  A fixed number of sweeps is run (`iters`, the paper's maximum 100 by
# default), each sweep = rows, columns, box in this order.  Gate weights stay the scores:
# G[i,j] = S[I[i,j], i] (Sec. 3.3 replaces only the indices).
def _logsumexp(a: np.ndarray, axis: int) -> np.ndarray:
    m = a.max(axis=axis, keepdims=True)
    return (m + np.log(np.exp(a - m).sum(axis=axis, keepdims=True))).squeeze(axis)


def capped_assignment(S: np.ndarray, k: int, b: float, lam: float = 1e-3, iters: int = 100,
                      out_dtype=np.float32) -> np.ndarray:
    """A[e,n] of Sec. 3.3 after `iters` sweeps of rows / columns / box (float32 like S unless asked otherwise)."""
    S = np.asarray(S)
    n, e = S.shape
    if not (1 <= k <= n) or not (b > 0) or not (lam > 0) or iters < 0:
        raise ValueError("bad k, b, lambda or iteration count")
    logA = S.T.astype(np.float64) / lam                 # log of the Gibbs kernel
    lq_col = np.zeros(n)                                # log of the column set's correction (one scale per column)
    lq_box = np.zeros((e, n))                           # log of the box set's correction
    for _ in range(iters):
        logA = logA + (math.log(k) - _logsumexp(logA, axis=1))[:, None]
        B = logA + lq_col[None, :]
        s = np.minimum(0.0, math.log(b) - _logsumexp(B, axis=0))
        logA = B + s[None, :]
        lq_col = -s
        B = logA + lq_box
        logA = np.minimum(B, 0.0)
        lq_box = np.maximum(B, 0.0)
    return np.exp(logA).astype(out_dtype)


def forward_capped(X, Wg, W1, W2, c: float, act: int, b: float, lam: float = 1e-3,
                   iters: int = 100) -> Dict[str, np.ndarray]:
    """Eq. 1-4 with the routing indices taken from TopK(A, k) (Sec. 3.3), weights from S."""
    n, d = np.asarray(X).shape
    e = np.asarray(Wg).shape[1]
    k = capacity(n, c, e)
    S = gate(X, Wg)
    A = capped_assignment(S, k, b, lam, iters)
    _, I = topk_tokens(np.ascontiguousarray(A.T), k)
    G = np.stack([S[I[i], i] for i in range(e)])
    X_in = dispatch(X, I)
    if W1 is None:
        if act != ACT_IDENTITY:
            raise ValueError("identity experts need act = ACT_IDENTITY")
        X_e = widen(X_in)
    else:
        X_e = expert_ffn(X_in, W1, W2, act)
    X_out = combine(X_e, G, I, n)
    return {"k": k, "S": S, "A": A, "G": G, "I": I, "X_in": X_in, "X_e": X_e, "X_out": X_out}


# ---------------------------------------------------------------- backward ---
# The paper prints no backward pass.  These are the derivatives of Eq. 4, Eq. 3 and Eq. 2 in that
# order, with the selection I a constant and the gate values G[i,j] = S[I[i,j], i] differentiable.
# Buffers of token-choice routing may hold empty rows (I = -1): such a row took part in nothing, so
# it receives no gradient and passes none on.
def backward_combine(dY, X_e, G, I) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 4 differentiated: dX_e[i,j,:] = G[i,j] dY[I[i,j],:] and dG[i,j] = <dY[I[i,j],:], X_e[i,j,:]>."""
    dYd, Xed, Gd = widen(dY), widen(X_e), widen(G)
    Ii = np.asarray(I, dtype=np.int64)
    dYsel = dYd[np.maximum(Ii, 0), :]                          # [e,k,d] rows of dY each bucket row fed
    dYsel[Ii < 0] = 0.0                                        # empty rows fed nothing
    dXe = Gd[:, :, None] * dYsel
    dG = np.einsum("ijt,ijt->ij", dYsel, Xed)
    return dXe, dG


def backward_ffn(X_in, W1, W2, act: int, dXe) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Eq. 3 differentiated, expert by expert: returns dX_in [e,k,d], dW1 [e,d,d_ff], dW2 [e,d_ff,d]."""
    X_in = widen(X_in)
    e = X_in.shape[0]
    dXin = np.empty_like(X_in)
    dW1 = np.empty(np.asarray(W1).shape, dtype=np.float64)
    dW2 = np.empty(np.asarray(W2).shape, dtype=np.float64)
    for i in range(e):
        W1i, W2i = widen(W1[i]), widen(W2[i])
        A = X_in[i] @ W1i                                       # [k,d_ff]
        H = activation(A, act)
        dW2[i] = H.T @ dXe[i]
        dH = dXe[i] @ W2i.T
        dA = dH * activation_grad(A, act)
        dW1[i] = X_in[i].T @ dA
        dXin[i] = dA @ W1i.T
    return dXin, dW1, dW2


def backward_gate(X, Wg, S, dG, I) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Eq. 2 differentiated: dS is dG scattered to the selected (token, expert) pairs, the softmax
    backward gives dZ = S * (dS - <dS, S>) row by row, then dWg = X^T dZ and the gate's share of dX."""
    Xd, Wgd, Sd = widen(X), widen(Wg), widen(S)
    n = Xd.shape[0]
    e, k = np.asarray(I).shape
    Ii = np.asarray(I, dtype=np.int64)
    dS = np.zeros((n, e), dtype=np.float64)
    for i in range(e):
        filled = Ii[i] >= 0
        dS[Ii[i][filled], i] = np.asarray(dG[i])[filled]        # each token at most once per expert
    dZ = Sd * (dS - (dS * Sd).sum(axis=1, keepdims=True))
    return Xd.T @ dZ, dZ @ Wgd.T, dZ


def backward(X, Wg, W1, W2, act: int, S: np.ndarray, G: np.ndarray, I: np.ndarray,
             dY: np.ndarray) -> Dict[str, np.ndarray]:
    """Gradients of L = <dY, X_out> w.r.t. X, Wg, W1, W2 (derived from Eq. 2-4).

    S, G, I are the forward's routing tensors (float32 / int32), taken as given so that the same
    selection is differentiated on both sides.
    """
    Ii = np.asarray(I, dtype=np.int64)
    n, d = np.asarray(X).shape
    e, k = Ii.shape
    X_in = widen(X)[np.maximum(Ii, 0), :]
    X_in[Ii < 0] = 0.0                                          # empty rows gathered nothing
    X_e = expert_ffn(X_in, W1, W2, act)
    dXe, dG = backward_combine(dY, X_e, G, I)
    dXin, dW1, dW2 = backward_ffn(X_in, W1, W2, act, dXe)
    dWg, dX, dZ = backward_gate(X, Wg, S, dG, I)
    for i in range(e):
        for j in range(k):                                      # Eq. 3 gather differentiated: scatter-add
            if Ii[i, j] >= 0:
                dX[Ii[i, j], :] += dXin[i, j, :]
    return {"dX": dX, "dWg": dWg, "dW1": dW1, "dW2": dW2, "dZ": dZ, "dG": dG}

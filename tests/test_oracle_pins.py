"""Pins for the CPU oracle: what the paper and the mathematics fix.

Each test checks the oracle against something other than itself: hand-worked
values (tests/golden), closed forms of degenerate routings, brute force in
pure Python on tiny inputs, the dense one-hot einsum form of Eq. 3 / Eq. 4,
textbook routines from an independent library (torch CPU float64), and
finite differences for the derived backward.  No GPU is needed.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import ec_moe_ref as ref


def _sized(base, **kw):
    """A resized copy of a workload with k from the oracle's Eq. 1."""
    w = wl.scaled(base, **kw)
    return w if w.k is not None else wl.scaled(w, k=ref.capacity(w.n, w.c, w.e))


def _rng(seed):
    return np.random.default_rng(seed)


@pytest.fixture(scope="module")
def golden(golden_dir):
    with open(os.path.join(golden_dir, "handworked_routing.json")) as f:
        return json.load(f)


# --------------------------------------------------------------- Eq. 1 ------
def test_capacity_closed_form_and_sum_of_buckets():
    # Eq. 1 on the five workloads: e*k == n*c exactly (c = average experts per token)
    for w in wl.WORKLOADS.values():
        k = ref.capacity(w.n, w.c, w.e)
        assert k == w.k
        assert k * w.e == int(w.n * w.c)
    assert ref.capacity(256, 2.0, 8) == 64
    assert ref.capacity(8192, 2.0, 16) == 1024
    assert ref.capacity(65536, 1.0, 256) == 256
    assert ref.capacity(10, 0.5, 3) == 1        # 1.67 floors to 1
    assert ref.capacity(7, 7.0, 7) == 7         # c = e: every expert takes all tokens
    with pytest.raises(ValueError):
        ref.capacity(4, 0.5, 16)                # k < 1
    with pytest.raises(ValueError):
        ref.capacity(4, 8.0, 2)                 # k > n


# --------------------------------------------------------------- Eq. 2 ------
def test_gate_handworked(golden):
    g = golden["gate_example"]
    X = np.array(g["X"], dtype=np.float64)
    Wg = np.log(np.array(g["Wg_log_of"], dtype=np.float64))
    S = ref.gate(X, Wg, out_dtype=np.float64)
    np.testing.assert_allclose(S, np.array(g["S"]), rtol=1e-14)


def test_gate_rows_are_distributions_and_degenerate_cases():
    r = _rng(1)
    X = r.standard_normal((37, 19)).astype(np.float32)
    Wg = (r.standard_normal((19, 5)) / math.sqrt(19)).astype(np.float32)
    S = ref.gate(X, Wg)
    assert S.dtype == np.float32 and S.shape == (37, 5)
    assert (S >= 0).all()
    np.testing.assert_allclose(S.astype(np.float64).sum(axis=1), 1.0, atol=1e-6)
    # zero embeddings: uniform distribution, exactly 1/e
    S0 = ref.gate(X, np.zeros_like(Wg))
    assert (S0 == np.float32(1.0 / 5)).all()
    # one expert: probability one
    assert (ref.gate(X, Wg[:, :1]) == np.float32(1.0)).all()
    # a constant added to every logit of a token changes nothing
    Xa = np.concatenate([X, np.ones((37, 1), np.float32)], axis=1)
    Wa = np.concatenate([Wg, np.full((1, 5), 3.25, np.float32)], axis=0)
    np.testing.assert_allclose(ref.gate(Xa, Wa, np.float64), ref.gate(X, Wg, np.float64), rtol=1e-12)
    # large logits do not overflow
    Sbig = ref.gate(X * 1000.0, Wg, np.float64)
    assert np.isfinite(Sbig).all()


def test_gate_against_library_softmax():
    r = _rng(2)
    X = r.standard_normal((64, 48))
    Wg = r.standard_normal((48, 7)) / 7.0
    lib = torch.softmax(torch.from_numpy(X) @ torch.from_numpy(Wg), dim=1).numpy()
    np.testing.assert_allclose(ref.gate(X, Wg, np.float64), lib, rtol=1e-12, atol=1e-15)


def test_gate_widens_bf16_exactly():
    r = _rng(3)
    Xf = r.standard_normal((8, 16)).astype(np.float32)
    Wf = r.standard_normal((16, 4)).astype(np.float32)
    Xb, Wb = wl.f32_to_bf16_bits(Xf), wl.f32_to_bf16_bits(Wf)
    S_bits = ref.gate(Xb, Wb, np.float64)
    S_wide = ref.gate(wl.bf16_bits_to_f32(Xb), wl.bf16_bits_to_f32(Wb), np.float64)
    assert (S_bits == S_wide).all()
    # 1.0 and -2.5 have exact bf16 forms
    assert (ref.widen(np.array([0x3F80, 0xC020], np.uint16)) == np.array([1.0, -2.5])).all()


def _brute_topk(col, k):
    """Pure-Python selection: k times, take the largest remaining, lowest index on ties."""
    taken = []
    alive = list(range(len(col)))
    for _ in range(k):
        best = alive[0]
        for t in alive[1:]:
            if col[t] > col[best]:
                best = t
        taken.append(best)
        alive.remove(best)
    return taken


def test_topk_handworked(golden):
    S = np.array(golden["S"], dtype=np.float32)
    G, I = ref.topk_tokens(S, golden["k"])
    assert I.tolist() == golden["I"]
    assert G.tolist() == golden["G"]
    counts = np.bincount(I.ravel(), minlength=golden["n"])
    assert counts.tolist() == golden["experts_per_token"]


@pytest.mark.parametrize("seed,n,e,k,levels", [(0, 17, 3, 5, 0), (1, 32, 4, 32, 0),
                                              (2, 29, 5, 7, 4), (3, 24, 2, 1, 3)])
def test_topk_against_brute_force(seed, n, e, k, levels):
    r = _rng(seed)
    S = r.random((n, e)).astype(np.float32)
    if levels:   # quantise so that many scores tie, also across the k-th place
        S = (np.floor(S * levels) / levels).astype(np.float32)
    G, I = ref.topk_tokens(S, k)
    for i in range(e):
        expect = sorted(_brute_topk(S[:, i].tolist(), k))      # admitted set, listed by token index
        assert I[i].tolist() == expect
        assert (G[i] == S[expect, i]).all()


def test_topk_invariants_and_lexsort():
    r = _rng(5)
    n, e, k = 512, 8, 96
    S = ref.gate(r.standard_normal((n, 24)), r.standard_normal((24, e)))
    S[::7, :] = S[3, :]          # plant ties
    G, I = ref.topk_tokens(S, k)
    assert I.dtype == np.int32 and G.dtype == np.float32
    for i in range(e):
        ids = I[i]
        assert len(set(ids.tolist())) == k and ids.min() >= 0 and ids.max() < n   # k distinct tokens
        assert (G[i] == S[ids, i]).all()                                            # raw scores, bitwise
        unsel = np.setdiff1d(np.arange(n), ids)
        lo = G[i].min()
        assert lo >= S[unsel, i].max()
        # an unselected token tying with the threshold must have a higher index
        # than every selected token at the threshold
        tied_out = unsel[S[unsel, i] == lo]
        tied_in = ids[G[i] == lo]
        if tied_out.size:
            assert tied_out.min() > tied_in.max()
        # independent library ordering: last key is primary in lexsort
        order = np.lexsort((np.arange(n), -S[:, i].astype(np.float64)))
        assert (np.sort(order[:k]) == ids).all()
        assert (np.diff(ids) > 0).all()                                             # listed by ascending token
    assert I.size == e * k                                                          # sum of buckets = n*c


def test_topk_all_ties_and_full_capacity():
    n, e = 40, 4
    S = np.full((n, e), 0.25, np.float32)
    G, I = ref.topk_tokens(S, 10)
    assert (I == np.arange(10)[None, :]).all() and (G == 0.25).all()
    r = _rng(6)
    S = r.random((n, e)).astype(np.float32)
    G, I = ref.topk_tokens(S, n)                  # k = n: every token, in token order
    for i in range(e):
        assert I[i].tolist() == list(range(n))
        assert (G[i] == S[:, i]).all()


# --------------------------------------------------------------- Eq. 3 ------
def _onehot(I, n):
    e, k = I.shape
    P = np.zeros((e, k, n))
    for i in range(e):
        for j in range(k):
            P[i, j, I[i, j]] = 1.0
    return P


def test_dispatch_equals_onehot_einsum():
    r = _rng(7)
    n, d, e, k = 12, 5, 3, 4
    X = r.standard_normal((n, d))
    I = np.stack([r.permutation(n)[:k] for _ in range(e)]).astype(np.int32)
    X_in = ref.dispatch(X, I)
    np.testing.assert_array_equal(X_in, np.einsum("ikn,nd->ikd", _onehot(I, n), X))
    # storage type and bits are kept
    Xb = wl.f32_to_bf16_bits(X.astype(np.float32))
    assert ref.dispatch(Xb, I).dtype == np.uint16
    assert (ref.dispatch(Xb, I)[2, 1] == Xb[I[2, 1]]).all()


def test_ffn_handworked(golden):
    g = golden["ffn_example"]
    for act, expect in [(ref.ACT_GELU, g["X_e"]), (ref.ACT_RELU, 3.0), (ref.ACT_IDENTITY, 3.0)]:
        out = ref.expert_ffn(np.array([[[g["x"]]]]), np.array([[[g["W1"]]]]), np.array([[[g["W2"]]]]), act)
        assert out.shape == (1, 1, 1)
        assert abs(out[0, 0, 0] - expect) < 1e-15
    # negative pre-activation: ReLU clips, GeLU(-1) = -(1 - Phi(1))
    out = ref.expert_ffn(np.array([[[-2.0]]]), np.array([[[0.5]]]), np.array([[[3.0]]]), ref.ACT_RELU)
    assert out[0, 0, 0] == 0.0
    out = ref.expert_ffn(np.array([[[-2.0]]]), np.array([[[0.5]]]), np.array([[[3.0]]]), ref.ACT_GELU)
    assert abs(out[0, 0, 0] + 3.0 * (1.0 - g["gelu_of_1"])) < 1e-15


def test_ffn_against_library_and_shapes():
    r = _rng(8)
    e, k, d, d_ff = 3, 7, 6, 10               # all different: a transposed operand cannot pass
    X_in = r.standard_normal((e, k, d))
    W1 = r.standard_normal((e, d, d_ff))
    W2 = r.standard_normal((e, d_ff, d))
    tX, tW1, tW2 = map(torch.from_numpy, (X_in, W1, W2))
    for act, fn in [(ref.ACT_GELU, lambda a: torch.nn.functional.gelu(a, approximate="none")),
                    (ref.ACT_RELU, torch.relu), (ref.ACT_IDENTITY, lambda a: a)]:
        lib = torch.bmm(fn(torch.bmm(tX, tW1)), tW2).numpy()
        np.testing.assert_allclose(ref.expert_ffn(X_in, W1, W2, act), lib, rtol=1e-12, atol=1e-13)
    # per-element definition on one entry
    i, j, t = 1, 4, 2
    a = [sum(X_in[i, j, u] * W1[i, u, f] for u in range(d)) for f in range(d_ff)]
    h = [0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in a]
    val = sum(h[f] * W2[i, f, t] for f in range(d_ff))
    assert abs(ref.expert_ffn(X_in, W1, W2, ref.ACT_GELU)[i, j, t] - val) < 1e-12
    # identity activation is linear in X_in
    lin = ref.expert_ffn(2.0 * X_in, W1, W2, ref.ACT_IDENTITY)
    np.testing.assert_allclose(lin, 2.0 * ref.expert_ffn(X_in, W1, W2, ref.ACT_IDENTITY), rtol=1e-12)


def test_activation_grad_by_central_difference():
    a = np.linspace(-4.0, 4.0, 41) + 0.013
    h = 1e-6
    for act in (ref.ACT_GELU, ref.ACT_RELU, ref.ACT_IDENTITY):
        fd = (ref.activation(a + h, act) - ref.activation(a - h, act)) / (2 * h)
        np.testing.assert_allclose(ref.activation_grad(a, act), fd, atol=1e-8)


# --------------------------------------------------------------- Eq. 4 ------
def test_combine_equals_dense_einsum_and_counts():
    r = _rng(9)
    n, d, e, k = 14, 4, 5, 6
    X_e = r.standard_normal((e, k, d))
    G = r.random((e, k)).astype(np.float32)
    I = np.stack([r.permutation(n)[:k] for _ in range(e)]).astype(np.int32)
    out = ref.combine(X_e, G, I, n)
    dense = np.einsum("ijl,ij,ijd->ld", _onehot(I, n), G.astype(np.float64), X_e)
    np.testing.assert_allclose(out, dense, rtol=1e-13, atol=1e-14)
    counts = np.bincount(I.ravel(), minlength=n)
    assert counts.sum() == e * k and counts.max() <= e
    assert (np.abs(out[counts == 0]).sum(axis=1) == 0).all()       # unrouted tokens: zero rows


def test_layer_identity_experts_closed_form(golden):
    # hand-worked: X_out[l] = (sum of the selected scores of token l) * X[l]
    S = np.array(golden["S"], dtype=np.float32)
    G, I = ref.topk_tokens(S, golden["k"])
    X = _rng(10).standard_normal((golden["n"], 3))
    out = ref.combine(ref.dispatch(X, I), G, I, golden["n"])
    np.testing.assert_allclose(out, np.array(golden["identity_expert_row_scale"])[:, None] * X, rtol=1e-15)
    # same closed form through forward() on random data
    r = _rng(11)
    n, d, e, c = 48, 8, 6, 2.0
    X = r.standard_normal((n, d)).astype(np.float32)
    Wg = r.standard_normal((d, e)).astype(np.float32)
    f = ref.forward(X, Wg, None, None, c, ref.ACT_IDENTITY)
    scale = np.zeros(n)
    for i in range(e):
        for j in range(f["k"]):
            scale[f["I"][i, j]] += float(f["S"][f["I"][i, j], i])
    np.testing.assert_allclose(f["X_out"], scale[:, None] * X.astype(np.float64), rtol=1e-13, atol=1e-15)
    counts = np.bincount(f["I"].ravel(), minlength=n)
    assert counts.sum() == int(n * c) and 0 <= counts.min() and counts.max() <= e


def _dense_ffn(x, W1, W2, act):
    t = torch.from_numpy(x) @ torch.from_numpy(W1)
    t = torch.nn.functional.gelu(t) if act == ref.ACT_GELU else torch.relu(t)
    return (t @ torch.from_numpy(W2)).numpy()


def test_layer_one_expert_is_dense_ffn():
    # e = 1, c = 1: every token goes through the single expert with weight 1
    r = _rng(12)
    n, d, d_ff = 20, 6, 9
    X = r.standard_normal((n, d))
    Wg = r.standard_normal((d, 1))
    W1 = r.standard_normal((1, d, d_ff))
    W2 = r.standard_normal((1, d_ff, d))
    f = ref.forward(X, Wg, W1, W2, 1.0, ref.ACT_GELU)
    assert f["k"] == n and (f["I"][0] == np.arange(n)).all()       # all scores 1.0: ties by index
    np.testing.assert_allclose(f["X_out"], _dense_ffn(X, W1[0], W2[0], ref.ACT_GELU), rtol=1e-12, atol=1e-13)


def test_layer_full_capacity_is_dense_soft_mixture():
    # c = e: k = n, every expert processes every token; X_out = sum_i S[:,i] * FFN_i(X)
    r = _rng(13)
    n, d, d_ff, e = 10, 5, 7, 3
    X = r.standard_normal((n, d)).astype(np.float32)
    Wg = r.standard_normal((d, e)).astype(np.float32)
    W1 = r.standard_normal((e, d, d_ff)).astype(np.float32)
    W2 = r.standard_normal((e, d_ff, d)).astype(np.float32)
    f = ref.forward(X, Wg, W1, W2, float(e), ref.ACT_RELU)
    S = f["S"].astype(np.float64)
    expect = sum(S[:, i:i + 1] * _dense_ffn(X.astype(np.float64), W1[i].astype(np.float64),
                                            W2[i].astype(np.float64), ref.ACT_RELU) for i in range(e))
    np.testing.assert_allclose(f["X_out"], expect, rtol=1e-12, atol=1e-13)


def test_layer_zero_gate_closed_form():
    # Wg = 0: all scores tie at 1/e, every expert takes tokens 0..k-1;
    # X_out[l] = (1/e) sum_i FFN_i(X[l]) for l < k and 0 beyond
    r = _rng(14)
    n, d, d_ff, e, c = 16, 4, 6, 4, 2.0
    X = r.standard_normal((n, d)).astype(np.float32)
    W1 = r.standard_normal((e, d, d_ff)).astype(np.float32)
    W2 = r.standard_normal((e, d_ff, d)).astype(np.float32)
    f = ref.forward(X, np.zeros((d, e), np.float32), W1, W2, c, ref.ACT_GELU)
    k = f["k"]
    assert k == 8 and (f["I"] == np.arange(k)[None, :]).all()
    mean = sum(_dense_ffn(X[:k].astype(np.float64), W1[i].astype(np.float64), W2[i].astype(np.float64),
                          ref.ACT_GELU) for i in range(e)) * float(np.float32(1.0 / e))
    np.testing.assert_allclose(f["X_out"][:k], mean, rtol=1e-12, atol=1e-13)
    assert (f["X_out"][k:] == 0).all()


def test_layer_expert_permutation_invariance():
    r = _rng(15)
    n, d, d_ff, e = 24, 6, 8, 4
    X = r.standard_normal((n, d)).astype(np.float32)
    Wg = r.standard_normal((d, e)).astype(np.float32)
    W1 = r.standard_normal((e, d, d_ff)).astype(np.float32)
    W2 = r.standard_normal((e, d_ff, d)).astype(np.float32)
    p = np.array([2, 0, 3, 1])
    a = ref.forward(X, Wg, W1, W2, 2.0, ref.ACT_GELU)
    b = ref.forward(X, Wg[:, p], W1[p], W2[p], 2.0, ref.ACT_GELU)
    np.testing.assert_allclose(a["X_out"], b["X_out"], rtol=1e-12, atol=1e-14)
    assert (a["I"][p] == b["I"]).all()


# ------------------------------------------------------------- backward -----
def _loss_fixed_selection(X, Wg, W1, W2, act, I, dY):
    """<dY, X_out> with the selection I held constant, built from the oracle's forward pieces."""
    S = ref.gate(X, Wg, out_dtype=np.float64)
    G = np.stack([S[I[i], i] for i in range(I.shape[0])])
    X_e = ref.expert_ffn(ref.dispatch(X, I), W1, W2, act)
    return float((ref.combine(X_e, G, I, X.shape[0]) * dY).sum())


def _small_problem(seed, act):
    r = _rng(seed)
    n, d, d_ff, e, c = 12, 5, 7, 3, 2.0
    X = r.standard_normal((n, d))
    Wg = r.standard_normal((d, e))
    W1 = r.standard_normal((e, d, d_ff)) / math.sqrt(d)
    W2 = r.standard_normal((e, d_ff, d)) / math.sqrt(d_ff)
    dY = r.standard_normal((n, d))
    S64 = ref.gate(X, Wg, out_dtype=np.float64)
    k = ref.capacity(n, c, e)
    _, I = ref.topk_tokens(S64.astype(np.float32), k)
    G64 = np.stack([S64[I[i], i] for i in range(e)])
    return X, Wg, W1, W2, dY, S64, G64, I


@pytest.mark.parametrize("act", [ref.ACT_GELU, ref.ACT_IDENTITY])
def test_backward_against_central_differences(act):
    X, Wg, W1, W2, dY, S, G, I = _small_problem(21, act)
    g = ref.backward(X, Wg, W1, W2, act, S, G, I, dY)
    h = 1e-6
    r = _rng(22)
    for name, arr in (("dX", X), ("dWg", Wg), ("dW1", W1), ("dW2", W2)):
        for _ in range(12):
            idx = tuple(int(r.integers(0, s)) for s in arr.shape)
            old = arr[idx]
            arr[idx] = old + h
            lp = _loss_fixed_selection(X, Wg, W1, W2, act, I, dY)
            arr[idx] = old - h
            lm = _loss_fixed_selection(X, Wg, W1, W2, act, I, dY)
            arr[idx] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - g[name][idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, g[name][idx])


def test_backward_with_empty_rows_against_central_differences():
    # token-choice buffers: dropped tokens and empty rows; the routing (I) is held constant
    r = _rng(31)
    n, d, d_ff, e, m, cap = 14, 5, 6, 4, 2, 5
    X = r.standard_normal((n, d))
    Wg = r.standard_normal((d, e)) * 1.5
    W1 = r.standard_normal((e, d, d_ff)) / math.sqrt(d)
    W2 = r.standard_normal((e, d_ff, d)) / math.sqrt(d_ff)
    dY = r.standard_normal((n, d))
    S64 = ref.gate(X, Wg, out_dtype=np.float64)
    _, I, load = ref.token_choice(S64.astype(np.float32), m, cap)
    assert (I < 0).any() and (load > cap).any()            # both empty rows and drops occur
    filled = I >= 0
    G64 = np.where(filled, S64[np.maximum(I, 0), np.arange(e)[:, None]], 0.0)

    def loss():
        S = ref.gate(X, Wg, out_dtype=np.float64)
        G = np.where(filled, S[np.maximum(I, 0), np.arange(e)[:, None]], 0.0)
        X_e = ref.expert_ffn(ref.dispatch_padded(X, I), W1, W2, ref.ACT_GELU)
        return float((ref.combine_padded(X_e, G, I, n) * dY).sum())

    g = ref.backward(X, Wg, W1, W2, ref.ACT_GELU, S64, G64, I, dY)
    h = 1e-6
    for name, arr in (("dX", X), ("dWg", Wg), ("dW1", W1), ("dW2", W2)):
        for _ in range(12):
            idx = tuple(int(r.integers(0, s)) for s in arr.shape)
            old = arr[idx]
            arr[idx] = old + h
            lp = loss()
            arr[idx] = old - h
            lm = loss()
            arr[idx] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - g[name][idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, g[name][idx])
    # an expert whose buffer is entirely empty gets no weight gradient at all
    S0 = S64.astype(np.float32).copy()
    S0[:, 3] = 0.0
    _, I0, _ = ref.token_choice(S0, 1, cap)
    assert (I0[3] < 0).all()
    G0 = np.where(I0 >= 0, S0[np.maximum(I0, 0), np.arange(e)[:, None]], 0.0)
    g0 = ref.backward(X, Wg, W1, W2, ref.ACT_GELU, S0, G0, I0, dY)
    assert (g0["dW1"][3] == 0).all() and (g0["dW2"][3] == 0).all()


def test_backward_against_autograd_restatement():
    act = ref.ACT_GELU
    X, Wg, W1, W2, dY, S, G, I = _small_problem(23, act)
    g = ref.backward(X, Wg, W1, W2, act, S, G, I, dY)
    tX, tWg, tW1, tW2 = (torch.tensor(a, requires_grad=True) for a in (X, Wg, W1, W2))
    tS = torch.softmax(tX @ tWg, dim=1)
    out = torch.zeros_like(tX)
    for i in range(I.shape[0]):
        idx = torch.from_numpy(I[i].astype(np.int64))
        xin = tX.index_select(0, idx)
        xe = torch.nn.functional.gelu(xin @ tW1[i]) @ tW2[i]
        out = out.index_add(0, idx, tS[idx, i][:, None] * xe)
    (out * torch.from_numpy(dY)).sum().backward()
    for name, t in (("dX", tX), ("dWg", tWg), ("dW1", tW1), ("dW2", tW2)):
        np.testing.assert_allclose(g[name], t.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_backward_one_expert_is_dense_ffn_gradient():
    r = _rng(24)
    n, d, d_ff = 9, 4, 6
    X = r.standard_normal((n, d))
    Wg = r.standard_normal((d, 1))
    W1 = r.standard_normal((1, d, d_ff))
    W2 = r.standard_normal((1, d_ff, d))
    dY = r.standard_normal((n, d))
    f = ref.forward(X, Wg, W1, W2, 1.0, ref.ACT_RELU)
    g = ref.backward(X, Wg, W1, W2, ref.ACT_RELU, f["S"], f["G"], f["I"], dY)
    tX, tW1, tW2 = (torch.tensor(a, requires_grad=True) for a in (X, W1[0], W2[0]))
    ((torch.relu(tX @ tW1) @ tW2) * torch.from_numpy(dY)).sum().backward()
    np.testing.assert_allclose(g["dX"], tX.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["dW1"][0], tW1.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["dW2"][0], tW2.grad.numpy(), rtol=1e-12, atol=1e-13)
    assert np.abs(g["dWg"]).max() < 1e-12            # a softmax over one expert has no gradient


# ------------------------------------------------------------- workloads ----
# ------------------------------------------------------- routing per group ---
@pytest.mark.parametrize("seed,n,e,groups,k_g,levels", [(0, 24, 3, 4, 2, 0), (1, 30, 2, 3, 10, 0),
                                                        (2, 32, 4, 2, 5, 3), (3, 12, 2, 12, 1, 0)])
def test_grouped_topk_against_brute_force(seed, n, e, groups, k_g, levels):
    r = _rng(seed)
    S = r.random((n, e)).astype(np.float32)
    if levels:
        S = (np.floor(S * levels) / levels).astype(np.float32)
    G, I = ref.topk_tokens_grouped(S, k_g, groups)
    n_g = n // groups
    for i in range(e):
        expect = []
        for g in range(groups):   # pure-Python selection inside the group's own tokens
            expect += [g * n_g + t for t in sorted(_brute_topk(S[g * n_g:(g + 1) * n_g, i].tolist(), k_g))]
        assert I[i].tolist() == expect
        assert (G[i] == S[expect, i]).all()


def test_grouped_topk_special_cases():
    r = _rng(11)
    S = r.random((40, 5)).astype(np.float32)
    # one group is the plain TopK of Eq. 2
    G1, I1 = ref.topk_tokens_grouped(S, 7, 1)
    G0, I0 = ref.topk_tokens(S, 7)
    assert (I1 == I0).all() and (G1 == G0).all()
    # k_g = n_g: every expert takes every token, in order
    G, I = ref.topk_tokens_grouped(S, 10, 4)
    assert (I == np.arange(40)[None, :]).all() and (G == S.T).all()
    # a group's selection does not see the other groups: overwrite group 2, groups 0, 1, 3 keep theirs
    _, Ia = ref.topk_tokens_grouped(S, 3, 4)
    S2 = S.copy()
    S2[20:30] = r.random((10, 5)).astype(np.float32)
    _, Ib = ref.topk_tokens_grouped(S2, 3, 4)
    keep = np.r_[0:6, 9:12]
    assert (Ia[:, keep] == Ib[:, keep]).all()
    # every expert holds exactly k_g tokens of every group
    for g in range(4):
        seg = Ia[:, 3 * g:3 * g + 3]
        assert ((seg >= 10 * g) & (seg < 10 * g + 10)).all()


@pytest.mark.parametrize("act", [wl.ACT_GELU, wl.ACT_IDENTITY])
def test_grouped_layer_is_the_plain_layer_on_every_group(act):
    # routing per group == running Eq. 1-4 on each group as a batch of its own
    w = _sized(wl.WORKLOADS["cfg1"], n=48, d=8, e=4, c=2.0, d_ff=16, act=act, seed=21)
    inp = wl.make_inputs(w)
    groups = 4
    n_g = w.n // groups
    W1, W2 = (inp["W1"], inp["W2"]) if act != wl.ACT_IDENTITY else (None, None)
    out = ref.forward_grouped(inp["X"], inp["Wg"], W1, W2, w.c, act, groups)
    assert out["k_g"] == ref.capacity(n_g, w.c, w.e)
    for g in range(groups):
        sub = ref.forward(inp["X"][g * n_g:(g + 1) * n_g], inp["Wg"], W1, W2, w.c, act)
        np.testing.assert_allclose(out["X_out"][g * n_g:(g + 1) * n_g], sub["X_out"], rtol=1e-12, atol=1e-14)
        seg = out["I"][:, g * out["k_g"]:(g + 1) * out["k_g"]]
        assert (seg == sub["I"] + g * n_g).all()


# ---------------------------------------------------- token-choice routing ---
def test_token_choice_handworked(golden_dir):
    with open(os.path.join(golden_dir, "handworked_token_choice.json")) as f:
        gold = json.load(f)
    S = np.array(gold["S"], dtype=np.float32)
    for case in gold["cases"]:
        G, I, load = ref.token_choice(S, case["m"], case["cap"])
        assert I.tolist() == case["I"]
        assert G.tolist() == case["G"]
        assert load.tolist() == case["load"]


def _brute_token_choice(S, m, cap):
    """Pure Python, token by token: repeated maximum per token, then placement in rank-major order."""
    n, e = len(S), len(S[0])
    picks = []
    for l in range(n):
        alive = list(range(e))
        mine = []
        for _ in range(m):
            best = alive[0]
            for i in alive[1:]:
                if S[l][i] > S[l][best]:
                    best = i
            mine.append(best)
            alive.remove(best)
        picks.append(mine)
    rows = [[] for _ in range(e)]
    load = [0] * e
    for r in range(m):
        for l in range(n):
            i = picks[l][r]
            load[i] += 1
            if len(rows[i]) < cap:
                rows[i].append(l)
    return rows, load


@pytest.mark.parametrize("seed,n,e,m,cap,levels", [(0, 40, 4, 1, 10, 0), (1, 40, 4, 2, 20, 0), (2, 33, 5, 2, 9, 3),
                                                  (3, 16, 3, 3, 16, 0), (4, 25, 6, 1, 2, 2)])
def test_token_choice_against_brute_force(seed, n, e, m, cap, levels):
    r = _rng(seed)
    S = r.random((n, e)).astype(np.float32)
    if levels:
        S = (np.floor(S * levels) / levels).astype(np.float32)
    G, I, load = ref.token_choice(S, m, cap)
    rows, load_b = _brute_token_choice(S.tolist(), m, cap)
    assert load.tolist() == load_b
    for i in range(e):
        assert I[i, :len(rows[i])].tolist() == rows[i]
        assert (I[i, len(rows[i]):] == -1).all() and (G[i, len(rows[i]):] == 0).all()
        assert (G[i, :len(rows[i])] == S[rows[i], i]).all()


def test_token_choice_invariants_and_priority():
    r = _rng(5)
    n, e, m, cap = 200, 8, 2, 50
    S = ref.gate(r.standard_normal((n, 16)).astype(np.float32), 2 * r.standard_normal((16, e)).astype(np.float32))
    G, I, load = ref.token_choice(S, m, cap)
    assert load.sum() == n * m                                   # every token makes m choices
    filled = I >= 0
    assert (filled.sum(axis=1) == np.minimum(load, cap)).all()   # an expert holds min(load, cap) tokens
    per_token = np.bincount(I[filled], minlength=n)
    assert per_token.max() <= m
    for i in range(e):                                           # a token sits at most once in a buffer
        assert len(set(I[i][filled[i]].tolist())) == filled[i].sum()
    # priority: second choices never displace first choices.  Expert 0 is every token's second choice
    # except for the last `cap` tokens, whose first choice it is: those must all be placed.
    n, cap = 30, 5
    S = np.zeros((n, 3), dtype=np.float32)
    S[:, 0], S[:, 1], S[:, 2] = 0.3, 0.6, 0.1
    S[n - cap:, 0], S[n - cap:, 1] = 0.6, 0.3
    _, I, load = ref.token_choice(S, 2, cap)
    assert I[0].tolist() == list(range(n - cap, n)) and load[0] == n


def test_token_choice_layer_without_drops_is_dense_top_m_mixture():
    # buffers as large as the batch: nothing is dropped, X_out[l] = sum over l's top-m experts of S[l,i] FFN_i(x_l)
    w = _sized(wl.WORKLOADS["cfg1"], n=24, d=8, e=4, d_ff=12, act=wl.ACT_GELU, seed=9)
    inp = wl.make_inputs(w)
    m = 2
    out = ref.forward_token_choice(inp["X"], inp["Wg"], inp["W1"], inp["W2"], c=float(w.e), m=m, act=w.act)
    assert out["cap"] == w.n and (out["load"] <= w.n).all()
    S = out["S"].astype(np.float64)
    X = inp["X"].astype(np.float64)
    expect = np.zeros((w.n, w.d))
    for l in range(w.n):
        top = np.argsort(-out["S"][l], kind="stable")[:m]
        for i in top:
            a = X[l] @ inp["W1"][i].astype(np.float64)
            h = np.array([0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0))) for t in a])
            expect[l] += S[l, i] * (h @ inp["W2"][i].astype(np.float64))
    np.testing.assert_allclose(out["X_out"], expect, rtol=1e-12, atol=1e-14)
    # identity experts, m = e: every token keeps the whole of itself (the scores sum to 1)
    out = ref.forward_token_choice(inp["X"], inp["Wg"], None, None, c=float(w.e), m=w.e, act=wl.ACT_IDENTITY)
    np.testing.assert_allclose(out["X_out"], X * S.sum(axis=1, keepdims=True), rtol=1e-12)
    # m = e with full buffers routes every token to every expert, like expert choice at c = e
    ec = ref.forward(inp["X"], inp["Wg"], inp["W1"], inp["W2"], c=float(w.e), act=w.act)
    tc = ref.forward_token_choice(inp["X"], inp["Wg"], inp["W1"], inp["W2"], c=float(w.e), m=w.e, act=w.act)
    np.testing.assert_allclose(tc["X_out"], ec["X_out"], rtol=1e-12, atol=1e-14)


# ----------------------------------------- expert choice with a cap (Sec. 3.3) ---
def _capped_lp(S, k, b):
    """The linear programme of Sec. 3.3 without the entropy term, by a library LP solver."""
    from scipy.optimize import linprog
    n, e = S.shape
    cost = -S.T.ravel().astype(np.float64)
    rows = np.zeros((e, e * n))
    for i in range(e):
        rows[i, i * n:(i + 1) * n] = 1.0
    cols = np.zeros((n, e * n))
    for j in range(n):
        cols[j, j::n] = 1.0
    res = linprog(cost, A_ub=cols, b_ub=np.full(n, float(b)), A_eq=rows, b_eq=np.full(e, float(k)),
                  bounds=(0.0, 1.0), method="highs")
    assert res.status == 0
    return res.x.reshape(e, n), -res.fun


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_capped_assignment_reaches_the_linear_programme(seed):
    r = _rng(seed)
    n, e, k, b, lam = 12, 4, 6, 2, 1e-3
    S = ref.gate(r.standard_normal((n, 8)).astype(np.float32), (0.3 * r.standard_normal((8, e))).astype(np.float32))
    A = ref.capped_assignment(S, k, b, lam, iters=20000, out_dtype=np.float64)
    # feasible ...
    np.testing.assert_allclose(A.sum(axis=1), k, atol=2e-3)
    assert (A.sum(axis=0) <= b + 2e-3).all() and A.max() <= 1.0 and A.min() >= 0.0
    # ... and optimal: the entropy term is worth at most lambda * e * n / exp(1)
    L, best = _capped_lp(S, k, b)
    value = float((S.T.astype(np.float64) * A).sum())
    assert best - value <= lam * e * n / math.e + 1e-3 * float(S.max()) * e
    # where the LP's vertex is clear-cut the near-integer A rounds to it
    if np.abs(L - A).max() < 0.4:
        assert (np.round(A) == np.round(L)).all()


def test_capped_assignment_slack_cap_closed_form():
    # column cap out of reach: per row, a_j = min(1, exp((S_j - mu)/lambda)) with mu set by sum_j a_j = k
    r = _rng(7)
    n, e, k, lam = 40, 3, 9, 0.05
    S = r.random((n, e)).astype(np.float32)
    A = ref.capped_assignment(S, k, b=float(e * k), lam=lam, iters=4000, out_dtype=np.float64)
    for i in range(e):
        x = S[:, i].astype(np.float64) / lam
        lo, hi = x.min() - 50.0, x.max() + 50.0
        for _ in range(200):                       # bisection on mu: the sum decreases with mu
            mu = 0.5 * (lo + hi)
            if np.minimum(1.0, np.exp(x - mu)).sum() > k:
                lo = mu
            else:
                hi = mu
        np.testing.assert_allclose(A[i], np.minimum(1.0, np.exp(x - 0.5 * (lo + hi))), atol=1e-6)


def test_capped_assignment_special_cases():
    # equal scores: one sweep gives the uniform matrix k/n, a fixed point when the cap allows e*k/n per column
    S = np.full((20, 4), 0.25, np.float32)
    A = ref.capped_assignment(S, 5, b=1.0, iters=1, out_dtype=np.float64)
    np.testing.assert_allclose(A, 0.25, rtol=1e-12)
    np.testing.assert_allclose(ref.capped_assignment(S, 5, b=1.0, iters=50, out_dtype=np.float64), 0.25, rtol=1e-12)
    # a binding cap: b = 0.5 halves every column, rows are rescaled next sweep, the cap halves again:
    # the constraints contradict each other (e*k > n*b) and A after the box step is the capped value
    A = ref.capped_assignment(S, 5, b=0.5, iters=30, out_dtype=np.float64)
    np.testing.assert_allclose(A.sum(axis=0), 0.5, rtol=1e-9)
    # zero sweeps: the Gibbs kernel itself (log domain avoids the overflow of exp(S/lambda))
    A0 = ref.capped_assignment(np.array([[0.0, 0.001]], np.float32), 1, 1, lam=1e-3, iters=0, out_dtype=np.float64)
    np.testing.assert_allclose(A0.ravel(), [1.0, math.e], rtol=1e-6)
    # layer: with the cap slack and the solver run to the end, the buckets are those of plain expert choice
    w = _sized(wl.WORKLOADS["cfg1"], n=32, d=8, e=4, d_ff=12, act=wl.ACT_GELU, seed=13)
    inp = wl.make_inputs(w)
    plain = ref.forward(inp["X"], inp["Wg"], inp["W1"], inp["W2"], w.c, w.act)
    capped = ref.forward_capped(inp["X"], inp["Wg"], inp["W1"], inp["W2"], w.c, w.act, b=float(w.e * plain["k"]),
                                lam=1e-3, iters=3000)
    assert (capped["I"] == plain["I"]).all() and (capped["G"] == plain["G"]).all()
    np.testing.assert_allclose(capped["X_out"], plain["X_out"], rtol=1e-12)
    # and with b = 1 no token sits in more than one bucket once the solver has converged
    capped = ref.forward_capped(inp["X"], inp["Wg"], inp["W1"], inp["W2"], 1.0, w.act, b=1.0, lam=1e-3, iters=20000)
    assert np.bincount(capped["I"].ravel(), minlength=w.n).max() == 1


def test_workload_generators_are_seeded_and_shaped():
    w = wl.WORKLOADS["cfg1"]
    a, b = wl.make_inputs(w), wl.make_inputs(w)
    assert all((a[key] == b[key]).all() for key in a)
    assert a["X"].shape == (256, 64) and a["Wg"].shape == (64, 8)
    assert a["W1"].shape == (8, 64, 256) and a["W2"].shape == (8, 256, 64)
    assert abs(a["Wg"].std() - 1 / 8) < 0.01 and abs(a["W2"].std() - 1 / 16) < 0.01
    s = _sized(wl.WORKLOADS["cfg5"], n=2048, d=64, e=8)
    t = wl.make_inputs(s)
    assert t["X"].dtype == np.uint16 and "W1" not in t and len(t["skew_rows"]) == 20
    # bf16 rounding: nearest-even on a few exact cases
    bits = wl.f32_to_bf16_bits(np.array([1.0, 1.00390625, 1.01171875, -2.5], np.float32))
    assert bits.tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020]

"""GPU parity for expert choice with a cap per token (Sec. 3.3 of the paper): the matrix A of the
entropy-regularised programme after a fixed number of Dykstra sweeps against the float64 oracle, and
the layer routed by TopK(A, k)."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import sized, max_rel_err, max_rel_err_rows, out_tol, score_tolerance, to_dev, to_host, torch_dtype

pytestmark = pytest.mark.gpu

# Both sides iterate in float64 and round A to float32 once; they differ in the order of the
# log-sum-exp reductions and in the exp/log routines, a few ulps of float64 per sweep.
A_TOL = 1e-6


@pytest.fixture(scope="module")
def m():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2202_09368_amd as mod
    mod.lib()
    return mod


@pytest.fixture(scope="module")
def ref():
    from oracle import ec_moe_ref
    return ec_moe_ref


def _p(msg):
    print(msg, flush=True)


def _scores(n, e, seed, scale):
    r = np.random.default_rng(seed)
    z = r.standard_normal((n, e)) * scale
    p = np.exp(z - z.max(axis=1, keepdims=True))
    return (p / p.sum(axis=1, keepdims=True)).astype(np.float32)


@pytest.mark.parametrize("n,e,k,b,lam,iters,scale", [
    (64, 4, 16, 1, 1e-3, 100, 1.0), (1000, 8, 250, 2, 1e-3, 100, 1.0), (1000, 8, 250, 2, 1e-3, 1, 1.0),
    (4099, 16, 512, 2, 1e-3, 100, 0.2),        # ragged token count, the paper's lambda and sweep cap
    (2048, 64, 64, 3, 1e-3, 100, 0.1),
    (300, 5, 100, 1, 5e-2, 400, 1.0),          # larger lambda: runs to convergence
    (512, 3, 200, 1000, 1e-2, 50, 1.0),        # cap out of reach
])
def test_capped_assignment(m, ref, n, e, k, b, lam, iters, scale):
    _p(f"[capped] n={n} e={e} k={k} b={b} lambda={lam} iters={iters}")
    S_h = _scores(n, e, n + e + iters, scale)
    St = to_dev(np.ascontiguousarray(S_h.T))
    A = torch.empty((e, n), dtype=torch.float32, device="cuda")
    ws = torch.empty(m.ec_moe_capped_workspace_bytes(n, e), dtype=torch.uint8, device="cuda")
    m.ec_moe_capped_assignment(St, k, float(b), lam, iters, A, ws)
    torch.cuda.synchronize()
    A_h = to_host(A)
    A_o = ref.capped_assignment(S_h, k, float(b), lam, iters)
    err = np.abs(A_h.astype(np.float64) - A_o.astype(np.float64)).max()
    _p(f"[capped] max |A - oracle| = {err:.3e}; row sums {A_h.sum(axis=1).min():.2f}..{A_h.sum(axis=1).max():.2f}")
    assert err <= A_TOL
    assert A_h.max() <= 1.0 and A_h.min() >= 0.0


@pytest.mark.parametrize("base,kw,b,iters", [
    ("cfg1", dict(n=512, d=64, e=8, d_ff=128), 1.0, 100),                # fp32
    ("cfg2", dict(n=2048, d=256, e=16, d_ff=512), 2.0, 100),             # bf16
    ("cfg3", dict(n=2048, d=128, e=64, d_ff=256), 3.0, 60),
    ("cfg5", dict(n=4096, d=128, e=32), 1.0, 100),                       # identity experts
    ("cfg2", dict(), 2.0, 100),                                          # full size, as `bench.py --capped 2` runs it
    ("cfg2", dict(n=2048, d=256, e=16, d_ff=512, hilo=True), 2.0, 100),  # two-part H, unrounded X_e into the sum
])
def test_capped_forward(m, ref, base, kw, b, iters):
    kw = dict(kw)
    hilo = kw.pop("hilo", False)
    w = sized(wl.WORKLOADS[base], **kw)
    inp = wl.make_inputs(w)
    n, d, e = w.n, w.d, w.e
    k = ref.capacity(n, w.c, e)
    lam = 1e-3
    _p(f"[capped forward] {base} n={n} d={d} e={e} k={k} b={b} iters={iters}")
    dt = torch_dtype(w)
    nbytes = m.ec_moe_workspace_bytes(n, d, e, k, w.d_ff, m.EC_BF16_HILO if hilo else w.dtype) \
        + m.ec_moe_capped_workspace_bytes(n, e) + (4 * e * n + 255) // 256 * 256
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    t = {key: to_dev(inp[key]) for key in ("X", "Wg", "W1", "W2") if key in inp}
    Xout = torch.empty((n, d), dtype=dt, device="cuda")
    S = torch.empty((n, e), dtype=torch.float32, device="cuda")
    A = torch.empty((e, n), dtype=torch.float32, device="cuda")
    G = torch.empty((e, k), dtype=torch.float32, device="cuda")
    I = torch.empty((e, k), dtype=torch.int32, device="cuda")
    Xe = torch.empty((e, k, d), dtype=dt, device="cuda") if w.d_ff else None
    m.ec_moe_forward_capped(t["X"], t["Wg"], t.get("W1"), t.get("W2"), w.c, b, lam, iters, Xout, w.act, ws,
                            S_out=S, G_out=G, I_out=I, A_out=A, Xe_out=Xe, hilo=hilo)
    torch.cuda.synchronize()
    S_h, A_h, G_h, I_h = to_host(S), to_host(A), to_host(G), to_host(I)
    S_ref = ref.gate(inp["X"], inp["Wg"])
    assert (max_rel_err_rows(S_h, S_ref) <= score_tolerance(inp["X"], inp["Wg"])).all()
    # the solver on the GPU's own scores
    A_o = ref.capped_assignment(S_h, k, b, lam, iters)
    assert np.abs(A_h.astype(np.float64) - A_o.astype(np.float64)).max() <= A_TOL
    # indices: TopK of the GPU's A, bit for bit; weights: the scores at those indices
    _, I_o = ref.topk_tokens(np.ascontiguousarray(A_h.T), k)
    assert (I_h == I_o).all()
    G_o = np.stack([S_h[I_h[i], i] for i in range(e)])
    assert (G_h.view(np.uint32) == G_o.view(np.uint32)).all()
    per_token = np.bincount(I_h.ravel(), minlength=n)
    _p(f"[capped forward] experts per token: max {per_token.max()}, tokens above the cap {(per_token > b).sum()}")
    X_in = ref.dispatch(inp["X"], I_h)
    if w.d_ff:
        Xe_ref = ref.expert_ffn(X_in, inp["W1"], inp["W2"], w.act)
        assert max_rel_err(to_host(Xe), Xe_ref) <= out_tol(w)
    else:
        Xe_ref = ref.widen(X_in)
    err = max_rel_err(to_host(Xout), ref.combine(Xe_ref, G_h, I_h, n))
    _p(f"[capped forward] X_out max rel err {err:.3e}")
    assert err <= (5e-3 if hilo else out_tol(w))    # two-part intermediates: what is left is the rounding of X_out


@pytest.mark.parametrize("base,kw,b,tol", [
    ("cfg1", dict(n=256, d=64, e=8, c=2.0, d_ff=128, act=wl.ACT_GELU), 1.0, 1e-5),   # fp32
    ("cfg2", dict(n=4096, d=256, e=8, d_ff=512), 2.0, 2e-2),                         # bf16, matrix-core path, k = 1024
])
def test_capped_backward(m, ref, base, kw, b, tol):
    # The capped variant changes only where I comes from (TopK of A instead of TopK of S); G stays S at the chosen
    # indices, so the backward pass of Eq. 2-4 applies unchanged: ec_moe_backward on the capped routing against the
    # oracle's backward on the same routing.
    w = sized(wl.WORKLOADS[base], backward=True, **kw)
    inp = wl.make_inputs(w)
    n, d, e, f = w.n, w.d, w.e, w.d_ff
    k = ref.capacity(n, w.c, e)
    lam, iters = 1e-3, 50
    _p(f"[capped backward] {base} n={n} d={d} e={e} k={k} b={b}")
    dt = torch_dtype(w)
    nbytes = m.ec_moe_workspace_bytes(n, d, e, k, f, w.dtype, True) + m.ec_moe_capped_workspace_bytes(n, e) \
        + (4 * e * n + 255) // 256 * 256
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    t = {key: to_dev(inp[key]) for key in ("X", "Wg", "W1", "W2", "dY")}
    dev = dict(device="cuda")
    f32 = torch.float32
    Xout = torch.empty((n, d), dtype=dt, **dev)
    S = torch.empty((n, e), dtype=f32, **dev)
    G = torch.empty((e, k), dtype=f32, **dev)
    I = torch.empty((e, k), dtype=torch.int32, **dev)
    m.ec_moe_forward_capped(t["X"], t["Wg"], t["W1"], t["W2"], w.c, b, lam, iters, Xout, w.act, ws, S_out=S, G_out=G, I_out=I)
    # the tensors the backward consumes, from the stage-wise entry points on the capped routing
    Xin = torch.empty((e, k, d), dtype=dt, **dev)
    A = torch.empty((e, k, f), dtype=dt, **dev)
    H = torch.empty((e, k, f), dtype=dt, **dev)
    Xe = torch.empty((e, k, d), dtype=dt, **dev)
    m.ec_moe_dispatch(t["X"], I, Xin)
    m.ec_moe_expert_ffn(Xin, t["W1"], t["W2"], Xe, w.act, ws, A_save=A, H_save=H)
    dX = torch.full((n, d), float("nan"), dtype=dt, **dev)
    dWg = torch.full((d, e), float("nan"), dtype=f32, **dev)
    dW1 = torch.full((e, d, f), float("nan"), dtype=f32, **dev)
    dW2 = torch.full((e, f, d), float("nan"), dtype=f32, **dev)
    m.ec_moe_backward(t["dY"], t["X"], t["Wg"], t["W1"], t["W2"], S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2, w.act, ws)
    torch.cuda.synchronize()
    S_h, G_h, I_h = to_host(S), to_host(G), to_host(I)
    per_token = np.bincount(I_h.ravel(), minlength=n)
    plain = np.bincount(ref.topk_tokens(S_h, k)[1].ravel(), minlength=n)
    assert (per_token != plain).any()            # the cap did change the routing this backward runs on
    g = ref.backward(inp["X"], inp["Wg"], inp["W1"], inp["W2"], w.act, S_h, G_h, I_h, inp["dY"])
    for key, got in (("dX", dX), ("dWg", dWg), ("dW1", dW1), ("dW2", dW2)):
        err = max_rel_err(to_host(got), g[key])
        _p(f"[capped backward] {key} max rel err {err:.3e}")
        assert err <= tol

"""GPU parity for expert choice per group of tokens (Limitations section of the paper): the grouped
TopK bit for bit against the oracle on the same scores, and the grouped layer stage by stage."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import sized, max_rel_err, out_tol, score_tolerance, max_rel_err_rows, to_dev, to_host, torch_dtype

pytestmark = pytest.mark.gpu


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


@pytest.mark.parametrize("n,e,groups,k_g,kind", [
    (4096, 3, 4, 100, "rand"), (8192, 16, 8, 128, "rand"), (8192, 2, 2048, 1, "rand"),
    (1200, 5, 3, 400, "rand"),                 # k_g = n_g
    (6000, 2, 5, 300, "levels"),               # exact ties across the cut inside every group
    (4000, 3, 10, 7, "const"),
    (65536 * 2, 2, 2, 300, "rand"),            # longest run the kernel accepts
    (16384, 4, 1, 512, "rand"),                # one group: the plain selection
    (8192, 16, 64, 20, "rand"),                # short runs (128 tokens): one wavefront per (expert, group)
    (4096, 8, 16, 256, "rand"),                # runs of 256 tokens, all of them taken
    (2048, 64, 8, 3, "levels"), (2048, 64, 8, 200, "levels"), (1024, 128, 4, 100, "const"),
    (240, 70, 1, 17, "rand"),                  # one short row per expert, the last lanes idle
])
def test_grouped_topk(m, ref, n, e, groups, k_g, kind):
    _p(f"[grouped topk] n={n} e={e} groups={groups} k_g={k_g} {kind}")
    r = np.random.default_rng(n + 7 * groups + k_g)
    if kind == "rand":
        St_h = r.random((e, n), dtype=np.float32)
    elif kind == "levels":
        St_h = (np.floor(r.random((e, n)) * 4) / 4).astype(np.float32)
    else:
        St_h = np.full((e, n), 0.25, np.float32)
    St = to_dev(St_h)
    G = torch.empty((e, groups * k_g), dtype=torch.float32, device="cuda")
    I = torch.empty((e, groups * k_g), dtype=torch.int32, device="cuda")
    m.ec_moe_topk_tokens_grouped(St, groups, k_g, G, I)
    torch.cuda.synchronize()
    G_o, I_o = ref.topk_tokens_grouped(np.ascontiguousarray(St_h.T), k_g, groups)
    assert (to_host(I) == I_o).all()
    assert (to_host(G).view(np.uint32) == G_o.view(np.uint32)).all()


def test_grouped_topk_rejects_bad_groups(m):
    St = torch.zeros((2, 1000), dtype=torch.float32, device="cuda")
    G = torch.empty((2, 30), dtype=torch.float32, device="cuda")
    I = torch.empty((2, 30), dtype=torch.int32, device="cuda")
    with pytest.raises(m.EcMoeError):           # 1000 tokens do not split into 3 equal runs
        m.ec_moe_topk_tokens_grouped(St, 3, 10, G, I)
    with pytest.raises(m.EcMoeError):           # runs of 250 tokens: not a multiple of 4
        m.ec_moe_topk_tokens_grouped(St, 4, 5, G, I)


@pytest.mark.parametrize("base,kw,groups", [
    ("cfg1", dict(n=512, d=64, e=8, d_ff=128), 4),                     # fp32
    ("cfg2", dict(n=4096, d=256, e=16, d_ff=512), 8),                  # bf16, slot lists in the combine
    ("cfg3", dict(n=4096, d=128, e=64, d_ff=256), 16),                 # bf16, CSR index in the combine
    ("cfg5", dict(n=8192, d=128, e=32), 4),                            # identity experts
    ("cfg2", dict(), 8),                                               # full size, as `bench.py --groups 8` runs it
    ("cfg2", dict(n=4096, d=256, e=16, d_ff=512), 32),                 # runs of 128 tokens: the small-segment kernel
    ("cfg3", dict(n=4096, d=128, e=64, d_ff=256), 64),
    ("cfg2", dict(n=4096, d=256, e=16, d_ff=512, hilo=True), 8),       # two-part H, unrounded X_e into the sum
])
def test_grouped_forward(m, ref, base, kw, groups):
    kw = dict(kw)
    hilo = kw.pop("hilo", False)
    w = sized(wl.WORKLOADS[base], **kw)
    inp = wl.make_inputs(w)
    n, d, e = w.n, w.d, w.e
    k_g = ref.capacity(n // groups, w.c, e)
    k = groups * k_g
    _p(f"[grouped forward] {base} n={n} d={d} e={e} groups={groups} k_g={k_g}")
    dt = torch_dtype(w)
    ws = m.alloc_workspace(n, d, e, k, w.d_ff, m.EC_BF16_HILO if hilo else w.dtype)
    t = {key: to_dev(inp[key]) for key in ("X", "Wg", "W1", "W2") if key in inp}
    Xout = torch.empty((n, d), dtype=dt, device="cuda")
    S = torch.empty((n, e), dtype=torch.float32, device="cuda")
    G = torch.empty((e, k), dtype=torch.float32, device="cuda")
    I = torch.empty((e, k), dtype=torch.int32, device="cuda")
    Xe = torch.empty((e, k, d), dtype=dt, device="cuda") if w.d_ff else None
    m.ec_moe_forward_grouped(t["X"], t["Wg"], t.get("W1"), t.get("W2"), w.c, groups, Xout, w.act, ws,
                             S_out=S, G_out=G, I_out=I, Xe_out=Xe, hilo=hilo)
    torch.cuda.synchronize()
    S_h, G_h, I_h = to_host(S), to_host(G), to_host(I)
    S_ref = ref.gate(inp["X"], inp["Wg"])
    assert (max_rel_err_rows(S_h, S_ref) <= score_tolerance(inp["X"], inp["Wg"])).all()
    G_o, I_o = ref.topk_tokens_grouped(S_h, k_g, groups)      # same scores: bit for bit
    assert (I_h == I_o).all() and (G_h.view(np.uint32) == G_o.view(np.uint32)).all()
    # downstream stages: the oracle fed with the GPU's routing
    X_in = ref.dispatch(inp["X"], I_h)
    if w.d_ff:
        Xe_ref = ref.expert_ffn(X_in, inp["W1"], inp["W2"], w.act)
        assert max_rel_err(to_host(Xe), Xe_ref) <= out_tol(w)
    else:
        Xe_ref = ref.widen(X_in)
    Xout_ref = ref.combine(Xe_ref, G_h, I_h, n)
    err = max_rel_err(to_host(Xout), Xout_ref)
    _p(f"[grouped forward] X_out max rel err {err:.3e}")
    assert err <= (5e-3 if hilo else out_tol(w))    # two-part intermediates: what is left is the rounding of X_out
    # the plain entry point is the one-group case
    if groups > 1 and not hilo:
        Xout1 = torch.empty_like(Xout)
        Xout2 = torch.empty_like(Xout)
        ws1 = m.alloc_workspace(n, d, e, ref.capacity(n, w.c, e), w.d_ff, w.dtype)
        m.ec_moe_forward(t["X"], t["Wg"], t.get("W1"), t.get("W2"), w.c, Xout1, w.act, ws1)
        m.ec_moe_forward_grouped(t["X"], t["Wg"], t.get("W1"), t.get("W2"), w.c, 1, Xout2, w.act, ws1)
        torch.cuda.synchronize()
        assert (to_host(Xout1) == to_host(Xout2)).all()


@pytest.mark.parametrize("base,kw,groups,tol", [
    ("cfg1", dict(n=256, d=64, e=8, c=2.0, d_ff=128, act=wl.ACT_GELU), 4, 1e-5),
    ("cfg2", dict(n=2048, d=256, e=16, d_ff=512), 8, 2e-2),
])
def test_grouped_backward(m, ref, base, kw, groups, tol):
    # the backward pass only sees the buckets (S, G, I and the saved activations), so it serves the
    # grouped routing unchanged: k is the bucket length groups * k_g
    w = sized(wl.WORKLOADS[base], backward=True, **kw)
    inp = wl.make_inputs(w)
    n, d, e, f = w.n, w.d, w.e, w.d_ff
    k = groups * ref.capacity(n // groups, w.c, e)
    _p(f"[grouped backward] {base} n={n} e={e} groups={groups} k={k}")
    dt = torch_dtype(w)
    t = {key: to_dev(inp[key]) for key in ("X", "Wg", "W1", "W2", "dY")}
    ws = m.alloc_workspace(n, d, e, k, f, w.dtype, with_backward=True)
    dev = dict(device="cuda")
    S = torch.empty((n, e), dtype=torch.float32, **dev)
    G = torch.empty((e, k), dtype=torch.float32, **dev)
    I = torch.empty((e, k), dtype=torch.int32, **dev)
    Xin = torch.empty((e, k, d), dtype=dt, **dev)
    A = torch.empty((e, k, f), dtype=dt, **dev)
    H = torch.empty((e, k, f), dtype=dt, **dev)
    Xe = torch.empty((e, k, d), dtype=dt, **dev)
    Xout = torch.empty((n, d), dtype=dt, **dev)
    m.ec_moe_forward_grouped(t["X"], t["Wg"], t["W1"], t["W2"], w.c, groups, Xout, w.act, ws, S_out=S, G_out=G,
                             I_out=I, Xin_out=Xin, A_out=A, H_out=H, Xe_out=Xe)
    dX = torch.empty((n, d), dtype=dt, **dev)
    dWg = torch.empty((d, e), dtype=torch.float32, **dev)
    dW1 = torch.empty((e, d, f), dtype=torch.float32, **dev)
    dW2 = torch.empty((e, f, d), dtype=torch.float32, **dev)
    m.ec_moe_backward(t["dY"], t["X"], t["Wg"], t["W1"], t["W2"], S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2, w.act, ws)
    torch.cuda.synchronize()
    g = ref.backward(inp["X"], inp["Wg"], inp["W1"], inp["W2"], w.act, to_host(S), to_host(G), to_host(I), inp["dY"])
    for key, got in (("dX", dX), ("dWg", dWg), ("dW1", dW1), ("dW2", dW2)):
        err = max_rel_err(to_host(got), g[key])
        _p(f"[grouped backward] {key} max rel err {err:.3e}")
        assert err <= tol

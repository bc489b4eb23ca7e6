"""GPU parity of ec_moe_backward against the oracle's derived backward (Eq. 2-4 differentiated with
the selection held constant), on the routing tensors S, G, I that the GPU forward produced."""
import numpy as np
import pytest
import torch

import workloads as wl
import os
import time

from gpu_util import sized, max_rel_err, max_rel_err_rows, score_tolerance, to_dev, to_f64, to_host, torch_dtype

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


def _forward_backward(m, w, inp, keep_on_device=False):
    n, d, e, k, f = w.n, w.d, w.e, w.k, w.d_ff
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
    m.ec_moe_forward(t["X"], t["Wg"], t["W1"], t["W2"], w.c, Xout, w.act, ws, S_out=S, G_out=G, I_out=I,
                     Xin_out=Xin, A_out=A, H_out=H, Xe_out=Xe)
    dX = torch.full((n, d), float("nan"), dtype=dt, **dev)
    dWg = torch.full((d, e), float("nan"), dtype=torch.float32, **dev)
    dW1 = torch.full((e, d, f), float("nan"), dtype=torch.float32, **dev)
    dW2 = torch.full((e, f, d), float("nan"), dtype=torch.float32, **dev)
    m.ec_moe_backward(t["dY"], t["X"], t["Wg"], t["W1"], t["W2"], S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2, w.act, ws)
    torch.cuda.synchronize()
    if keep_on_device:
        return dict(S=S, G=G, I=I, dX=dX, dWg=dWg, dW1=dW1, dW2=dW2, Xe=Xe, Xout=Xout)
    return dict(S=to_host(S), G=to_host(G), I=to_host(I), dX=to_host(dX), dWg=to_host(dWg), dW1=to_host(dW1),
                dW2=to_host(dW2))


@pytest.mark.parametrize("name,kw,tol", [
    ("cfg1", dict(n=300, d=60, e=5, c=2.0, d_ff=100), 1e-5),                      # fp32, ragged everything
    ("cfg1", dict(n=256, d=64, e=8, c=2.0, d_ff=256, act=wl.ACT_GELU), 1e-5),     # fp32, GeLU
    ("cfg2", dict(n=1000, d=192, e=16, d_ff=320), 2e-2),                          # bf16 matrix-core path, k = 125
    ("cfg2", dict(n=2048, d=256, e=8, d_ff=512, act=wl.ACT_RELU), 2e-2),          # bf16, ReLU
    ("cfg2", dict(n=1000, d=192, e=16, d_ff=328), 2e-2),                          # bf16, d_ff % 64 != 0: plain path
    ("cfg3", dict(n=4096, d=128, e=64, d_ff=256), 2e-2),                          # bf16, 64 experts (CSR lists)
])
def test_backward_reduced(m, ref, name, kw, tol):
    w = sized(wl.WORKLOADS[name], backward=True, **kw)
    inp = wl.make_inputs(w)
    print(f"[bwd {w.name}] n={w.n} d={w.d} e={w.e} k={w.k} d_ff={w.d_ff} act={w.act}", flush=True)
    r = _forward_backward(m, w, inp)
    g = ref.backward(inp["X"], inp["Wg"], inp["W1"], inp["W2"], w.act, r["S"], r["G"], r["I"], inp["dY"])
    errs = {}
    for key in ("dX", "dWg", "dW1", "dW2"):
        err = max_rel_err(r[key], g[key])
        print(f"[bwd {w.name}] {key} max rel err {err:.3e}", flush=True)
        errs[key] = err
    assert all(v <= tol for v in errs.values()), errs


def _progress(msg):
    """Progress of the long full-size test (it runs for most of a minute)."""
    print(f"[cfg4 {time.strftime('%H:%M:%S')}] {msg}", flush=True)


def test_cfg4_full_forward_backward(m, ref):
    """Full size: 32768 tokens, d=2048, 128 experts, d_ff=8192, forward + backward.  The float64 oracle
    runs the expert FFN (forward and backward) on a sample of experts; the gate gradient is checked
    with the oracle's Eq. 4 / Eq. 2 derivatives fed with the GPU's X_e (itself checked on the sample)."""
    w = wl.WORKLOADS["cfg4"]
    n, d, e, k = w.n, w.d, w.e, w.k
    _progress("drawing inputs")
    inp = wl.make_inputs(w)
    _progress("forward + backward on the GPU")
    r = _forward_backward(m, w, inp, keep_on_device=True)
    S, G, I = to_host(r["S"]), to_host(r["G"]), to_host(r["I"])

    _progress("scores and selection")
    S_ref = ref.gate(inp["X"], inp["Wg"])
    s_err = max_rel_err_rows(S, S_ref)
    _progress(f"S max rel err {s_err.max():.3e} (bar 1e-5)")
    assert s_err.max() <= 1e-5
    G_o, I_o = ref.topk_tokens(S, k)
    assert (I_o == I).all() and (G_o.view(np.uint32) == G.view(np.uint32)).all()

    ex = [0, 13, 31, 50, 77, 90, 111, 127]
    _progress(f"oracle FFN forward/backward on experts {ex}")
    Xin_ex = ref.dispatch(inp["X"], I[ex])
    Xe_ref = ref.expert_ffn(Xin_ex, inp["W1"][ex], inp["W2"][ex], w.act)
    Xe_gpu = to_host(r["Xe"])
    err = max_rel_err(Xe_gpu[ex], Xe_ref)
    _progress(f"X_e max rel err {err:.3e}")
    assert err <= 2e-2
    dXe_ref, _ = ref.backward_combine(inp["dY"], Xe_ref, G[ex], I[ex])
    dXin_ref, dW1_ref, dW2_ref = ref.backward_ffn(Xin_ex, inp["W1"][ex], inp["W2"][ex], w.act, dXe_ref)
    idx = torch.tensor(ex, device="cuda")
    for key, want in (("dW1", dW1_ref), ("dW2", dW2_ref)):
        err = max_rel_err(to_host(r[key].index_select(0, idx)), want)
        _progress(f"{key}[sample] max rel err {err:.3e}")
        assert err <= 2e-2, key

    _progress("gate gradient (Eq. 4 and Eq. 2 derivatives on the GPU's X_e)")
    _, dG_t = ref.backward_combine(inp["dY"], Xe_gpu, G, I)
    dWg_ref, dXgate, _ = ref.backward_gate(inp["X"], inp["Wg"], S, dG_t, I)
    err = max_rel_err(to_host(r["dWg"]), dWg_ref)
    _progress(f"dWg max rel err {err:.3e}")
    assert err <= 2e-2

    # dX on the tokens that only the sampled experts selected
    in_sample = np.zeros(e, bool)
    in_sample[ex] = True
    other = np.unique(I[~in_sample].ravel())
    toks = np.setdiff1d(np.unique(I[in_sample].ravel()), other)
    assert toks.size > 0
    dX_ref = dXgate.copy()
    for a, i in enumerate(ex):
        for j in range(k):
            dX_ref[I[i, j], :] += dXin_ref[a, j, :]
    err = max_rel_err(to_f64(to_host(r["dX"]))[toks], dX_ref[toks])
    _progress(f"dX on {toks.size} tokens served only by the sample: max rel err {err:.3e}")
    assert err <= 2e-2

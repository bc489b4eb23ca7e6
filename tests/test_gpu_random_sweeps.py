"""Seeded random sweeps on the GPU: many small routing problems and whole fp32 layers with shapes nobody
picked by hand (unaligned rows, odd expert counts, groups, ties, constant and peaked scores, k = n, ragged
widths), each compared with the oracle -- routing bit for bit, fp32 outputs at 1e-5."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import max_rel_err, max_rel_err_rows, to_dev, to_host

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


def _scores(rng, kind, n, e):
    if kind == 0:
        return rng.random((n, e), dtype=np.float32)
    if kind == 1:                                   # three distinct values: ties everywhere
        return (np.floor(rng.random((n, e)) * 3) / 3).astype(np.float32)
    if kind == 2:                                   # one value: the selection is decided by token order alone
        return np.full((n, e), 0.5, np.float32)
    z = rng.standard_normal((n, e)) * 3             # peaked softmax rows
    p = np.exp(z - z.max(1, keepdims=True))
    return (p / p.sum(1, keepdims=True)).astype(np.float32)


def test_random_long_rows(m, ref):
    """Rows of more than 32768 scores with small buckets: the selection first tries a threshold taken from the
    per-thread maxima and falls back to the radix passes when that keeps too many candidates.  Random row lengths
    (partial register tiles), bucket sizes on both sides of 512, and score layouts that hit both outcomes."""
    rng = np.random.default_rng(77)
    for it in range(24):
        seg = int(rng.integers(32768 // 4 + 1, 65536 // 4 + 1)) * 4
        groups = 2 if it % 6 == 5 else 1
        n, e = seg * groups, int(rng.integers(1, 4))
        k = int(rng.choice([1, 2, 37, 128, 256, 300, 511, 512, 513, 700]))
        kind = it % 6
        if kind in (0, 5):
            S = rng.random((n, e), dtype=np.float32)
        elif kind == 1:                               # gate-like: softmax over 64 experts, the first e kept
            z = rng.standard_normal((n, 64)) * 4
            p = np.exp(z - z.max(1, keepdims=True))
            S = np.ascontiguousarray((p / p.sum(1, keepdims=True)).astype(np.float32)[:, :e])
        elif kind == 2:                               # blocks of 4096 sorted tokens: the large scores sit in few threads
            S = rng.random((n, e), dtype=np.float32)
            for b in range(0, n, 4096):
                S[b:b + 4096] = -np.sort(-S[b:b + 4096], axis=0)
        elif kind == 3:                               # 16 distinct values: ties at every threshold
            S = (np.floor(rng.random((n, e)) * 16) / 16).astype(np.float32)
        else:                                         # a few hundred large scores over a floor of equal ones
            S = np.full((n, e), 0.001, np.float32)
            for i in range(e):
                idx = rng.choice(n, int(rng.integers(1, 2 * k + 2)), replace=False)
                S[idx, i] = 0.5 + 0.5 * rng.random(idx.size, dtype=np.float32)
        print(f"[long rows {it}] layout {kind} n={n} e={e} groups={groups} k_g={k}", flush=True)
        G = torch.empty((e, groups * k), dtype=torch.float32, device="cuda")
        I = torch.empty((e, groups * k), dtype=torch.int32, device="cuda")
        m.ec_moe_topk_tokens_grouped(to_dev(np.ascontiguousarray(S.T)), groups, k, G, I)
        torch.cuda.synchronize()
        G_o, I_o = ref.topk_tokens_grouped(S, k, groups)
        assert (to_host(I) == I_o).all() and (to_host(G).view(np.uint32) == G_o.view(np.uint32)).all()


def test_random_routing_problems(m, ref):
    rng = np.random.default_rng(2024)
    done = 0
    for it in range(90):
        kind = int(rng.integers(0, 4))
        e = int(rng.choice([1, 2, 3, 7, 16, 33, 64, 130]))
        groups = int(rng.choice([1, 1, 2, 4, 8, 16]))
        seg = int(rng.choice([4, 12, 64, 100, 256, 260, 1000, 4096, 5000, 20000]))
        if rng.random() < 0.3:
            seg += int(rng.integers(1, 4))          # rows that are not a multiple of 4 tokens (one group only)
        if seg % 4:
            groups = 1
        n = seg * groups
        if n * e > 3_000_000:
            continue
        k = int(rng.integers(1, seg + 1)) if rng.random() < 0.8 else seg
        S = _scores(rng, kind, n, e)
        print(f"[routing {it}] scores {kind} n={n} e={e} groups={groups} k_g={k}", flush=True)
        G = torch.empty((e, groups * k), dtype=torch.float32, device="cuda")
        I = torch.empty((e, groups * k), dtype=torch.int32, device="cuda")
        m.ec_moe_topk_tokens_grouped(to_dev(np.ascontiguousarray(S.T)), groups, k, G, I)
        torch.cuda.synchronize()
        G_o, I_o = ref.topk_tokens_grouped(S, k, groups)
        assert (to_host(I) == I_o).all() and (to_host(G).view(np.uint32) == G_o.view(np.uint32)).all()
        # token choice on the same scores
        mt, cap = int(rng.integers(1, min(e, 8) + 1)), int(rng.integers(1, n + 1))
        if e * cap < 1_500_000:
            G2 = torch.empty((e, cap), dtype=torch.float32, device="cuda")
            I2 = torch.empty((e, cap), dtype=torch.int32, device="cuda")
            load = torch.empty((e,), dtype=torch.int32, device="cuda")
            ws = torch.empty(32 * n + 256, dtype=torch.uint8, device="cuda")
            m.ec_moe_token_choice(to_dev(S), mt, cap, G2, I2, load, ws)
            torch.cuda.synchronize()
            G_t, I_t, load_t = ref.token_choice(S, mt, cap)
            assert (to_host(I2) == I_t).all() and (to_host(G2).view(np.uint32) == G_t.view(np.uint32)).all()
            assert (to_host(load) == load_t).all()
        done += 1
    assert done >= 60


def test_random_fp32_layers(m, ref):
    rng = np.random.default_rng(7)
    done = 0
    for it in range(60):
        d = int(rng.choice([8, 24, 64, 72, 128, 192, 200])) + int(rng.integers(0, 3))
        d_ff = int(rng.choice([8, 40, 64, 136, 256, 328])) + int(rng.integers(0, 3))
        e = int(rng.choice([1, 2, 4, 8, 16, 24, 64, 72, 128]))
        n = int(rng.choice([16, 100, 256, 1000, 2048, 4100]))
        c = float(rng.choice([0.5, 1.0, 2.0, 3.0]))
        try:
            k = ref.capacity(n, c, e)
        except ValueError:
            continue
        if e * k * max(d, d_ff) > 3_000_000:
            continue
        identity = rng.random() < 0.15
        act = wl.ACT_IDENTITY if identity else int(rng.choice([wl.ACT_RELU, wl.ACT_GELU, wl.ACT_IDENTITY]))
        w = wl.Workload("sweep", n=n, d=d, e=e, c=c, d_ff=0 if identity else d_ff, act=act, dtype=wl.DTYPE_F32,
                        seed=1000 + it, k=k)
        print(f"[layer {it}] n={n} d={d} e={e} c={c} k={k} d_ff={w.d_ff} act={act}", flush=True)
        inp = wl.make_inputs(w)
        t = {key: to_dev(inp[key]) for key in ("X", "Wg", "W1", "W2") if key in inp}
        ws = m.alloc_workspace(n, d, e, k, w.d_ff, w.dtype)
        Xout = torch.full((n, d), float("nan"), dtype=torch.float32, device="cuda")
        S = torch.empty((n, e), dtype=torch.float32, device="cuda")
        G = torch.empty((e, k), dtype=torch.float32, device="cuda")
        I = torch.empty((e, k), dtype=torch.int32, device="cuda")
        m.ec_moe_forward(t["X"], t["Wg"], t.get("W1"), t.get("W2"), c, Xout, act, ws, S_out=S, G_out=G, I_out=I)
        torch.cuda.synchronize()
        S_h, G_h, I_h = to_host(S), to_host(G), to_host(I)
        assert max_rel_err_rows(S_h, ref.gate(inp["X"], inp["Wg"])).max() <= 1e-5
        G_o, I_o = ref.topk_tokens(S_h, k)
        assert (I_h == I_o).all() and (G_h.view(np.uint32) == G_o.view(np.uint32)).all()
        Xin = ref.dispatch(inp["X"], I_h)
        Xe = ref.widen(Xin) if identity else ref.expert_ffn(Xin, inp["W1"], inp["W2"], act)
        assert max_rel_err(to_host(Xout), ref.combine(Xe, G_h, I_h, n)) <= 1e-5
        done += 1
    assert done >= 30

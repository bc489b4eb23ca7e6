"""ec_moe_combine_static (the entry point that allocates nothing: its token-major index lives in a
static device array inside the library) against ec_moe_combine on the same inputs.

Both run the same kernels in the same order of additions, so X_out must be bit-identical.  Two calls
in a row on one GPU, the second with a smaller input, check that what the first call left in the
shared array does not leak into the second; both index forms (slot lists for e <= 16, bitmap + CSR
above) and both storage types are covered, and a problem too large for the array is refused.
"""
import numpy as np
import pytest
import torch

import paper_2202_09368_amd as m
import workloads as wl
from gpu_util import to_dev, to_host

pytestmark = pytest.mark.gpu


def _routing(n, e, k, d, bf16, seed):
    """Seeded bucket contents: every expert holds k distinct tokens in ascending order (any TopK output has this form)."""
    rng = np.random.default_rng(seed)
    I = np.stack([np.sort(rng.choice(n, size=k, replace=False)) for _ in range(e)]).astype(np.int32)
    G = rng.random((e, k), dtype=np.float32)
    Xe = rng.standard_normal((e, k, d), dtype=np.float32)
    return (to_dev(wl.f32_to_bf16_bits(Xe) if bf16 else Xe), to_dev(G), to_dev(I))


def _both(n, e, k, d, bf16, seed):
    Xe, G, I = _routing(n, e, k, d, bf16, seed)
    dt = torch.bfloat16 if bf16 else torch.float32
    ws = m.alloc_workspace(n, d, e, k, 0, m.EC_BF16 if bf16 else m.EC_F32)
    want = torch.full((n, d), 7.0, dtype=dt, device="cuda")
    got = torch.full((n, d), -3.0, dtype=dt, device="cuda")
    m.ec_moe_combine(Xe, G, I, want, ws)
    m.ec_moe_combine_static(Xe, G, I, got)
    torch.cuda.synchronize()
    return to_host(got), to_host(want)


@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("first,second", [
    ((4096, 64, 128, 256), (1000, 24, 60, 64)),     # bitmap + CSR index, then a smaller one
    ((4096, 16, 512, 128), (512, 8, 128, 64)),      # slot lists (16 slots), then 8 slots
    ((2048, 40, 100, 96), (2048, 4, 700, 96)),      # CSR, then slot lists on the same token count
])
def test_static_scratch_combine_matches_workspace_combine(first, second, bf16):
    for seed, (n, e, k, d) in enumerate((first, second)):
        print(f"combine_static n={n} e={e} k={k} d={d} bf16={bf16}", flush=True)
        got, want = _both(n, e, k, d, bf16, 100 + seed)
        assert got.shape == want.shape
        assert (got.view(np.uint16 if bf16 else np.uint32) == want.view(np.uint16 if bf16 else np.uint32)).all()
        # repeat on the array as this call left it
        got2, _ = _both(n, e, k, d, bf16, 100 + seed)
        assert (got2.view(got.dtype) == got).all()


def test_static_scratch_combine_refuses_what_does_not_fit():
    # the index of this problem needs 4*n*ceil(e/32) bytes = 16 MiB > EC_MOE_STATIC_SCRATCH_BYTES
    n, e, k, d = 131072, 1024, 2, 8
    Xe = torch.zeros((e, k, d), dtype=torch.float32, device="cuda")
    G = torch.zeros((e, k), dtype=torch.float32, device="cuda")
    I = torch.zeros((e, k), dtype=torch.int32, device="cuda")
    out = torch.zeros((n, d), dtype=torch.float32, device="cuda")
    with pytest.raises(m.EcMoeError) as ei:
        m.ec_moe_combine_static(Xe, G, I, out)
    assert ei.value.status == -4


def test_static_scratch_combine_under_graph_capture():
    # what the entry point is for: a caller that captures the call in a HIP graph.  The array's address is looked up
    # at the first call on a device, so one call is made before the capture; every replay, with eager work and
    # synchronisations in between, must equal the eager result (the index is cleared by a kernel, not a memset node).
    n, e, k, d = 4096, 64, 128, 256
    Xe, G, I = _routing(n, e, k, d, True, 7)
    out = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    m.ec_moe_combine_static(Xe, G, I, out)
    torch.cuda.synchronize()
    eager = to_host(out)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        m.ec_moe_combine_static(Xe, G, I, out)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        m.ec_moe_combine_static(Xe, G, I, out)
    torch.cuda.synchronize()
    for _ in range(3):
        out.fill_(1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert (to_host(out) == eager).all()

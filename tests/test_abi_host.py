"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before anything reaches a GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def m():
    import paper_2202_09368_amd as mod
    if not os.path.exists(mod.lib_path()):
        import __graft_entry__
        __graft_entry__.build()
    mod.lib()
    return mod


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ec_moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ec_moe_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(m):
    names = _declared_functions()
    assert {"ec_moe_gate", "ec_moe_topk_tokens", "ec_moe_dispatch", "ec_moe_expert_ffn", "ec_moe_combine",
            "ec_moe_forward", "ec_moe_backward", "ec_moe_capacity", "ec_moe_workspace_bytes"} <= set(names)
    raw = ctypes.CDLL(m.lib_path())
    for name in names:
        assert hasattr(raw, name), f"{name} declared in ec_moe.h but not exported"


def test_capacity_and_status_strings(m):
    assert m.ec_moe_capacity(8192, 16, 2.0) == 1024
    assert m.ec_moe_capacity(65536, 256, 1.0) == 256
    assert m.ec_moe_capacity(10, 3, 0.5) == 1
    for bad in [(0, 4, 1.0), (16, 0, 1.0), (16, 4, 0.0), (4, 16, 0.5), (4, 2, 8.0), (4, 2, float("nan"))]:
        with pytest.raises(m.EcMoeError) as ei:
            m.ec_moe_capacity(*bad)
        assert ei.value.status == -1
    assert m.ec_moe_status_string(0) == "EC_OK"
    assert m.ec_moe_status_string(-2) == "EC_ERR_WORKSPACE"
    assert m.ec_moe_status_string(-4) == "EC_ERR_UNSUPPORTED"
    assert re.match(r"\d+\.\d+", m.ec_moe_version())


def test_workspace_sizes(m):
    small = m.ec_moe_workspace_bytes(256, 64, 8, 64, 256, m.EC_F32)
    big = m.ec_moe_workspace_bytes(8192, 768, 16, 1024, 3072, m.EC_BF16)
    assert 0 < small < big and big % 256 == 0
    assert big >= 16 * 1024 * 3072 * 2           # at least the hidden activations
    assert m.ec_moe_workspace_bytes(0, 64, 8, 64, 256, m.EC_F32) == 0
    assert m.ec_moe_workspace_bytes(256, 64, 8, 512, 256, m.EC_F32) == 0      # k > n
    assert m.ec_moe_workspace_bytes(256, 64, 8, 64, 256, 7) == 0             # unknown dtype
    assert m.ec_moe_workspace_bytes(256, 64, 2000, 1, 256, m.EC_F32) == 0    # too many experts
    # two-part intermediates: room for the remainder of H and for the unrounded X_e on top of the bf16 layout; nothing
    # extra for identity experts; no such layer when a width is not a multiple of 64
    hilo = m.ec_moe_workspace_bytes(8192, 768, 16, 1024, 3072, m.EC_BF16_HILO)
    assert hilo >= big + 16 * 1024 * (3072 * 2 + 768 * 4) and hilo % 256 == 0
    assert m.ec_moe_workspace_bytes(8192, 768, 16, 1024, 3072, m.EC_BF16_HILO, True) > \
        m.ec_moe_workspace_bytes(8192, 768, 16, 1024, 3072, m.EC_BF16, True) + (hilo - big)   # and of dX_e
    assert m.ec_moe_workspace_bytes(8192, 768, 16, 1024, 0, m.EC_BF16_HILO) == \
        m.ec_moe_workspace_bytes(8192, 768, 16, 1024, 0, m.EC_BF16)
    assert m.ec_moe_workspace_bytes(256, 72, 4, 64, 136, m.EC_BF16_HILO) == 0
    assert m.ec_moe_workspace_bytes(256, 72, 4, 64, 136, m.EC_BF16) > 0


def test_invalid_arguments_are_rejected_on_the_host(m):
    lib = m.lib()
    P = 0x1000   # non-null, 16- and 256-byte aligned; never dereferenced: validation fails first
    INV, WS = -1, -2
    # gate: null X, bad dtype, both outputs null, misaligned pointer
    assert lib.ec_moe_gate(None, P, P, P, 8, 8, 4, 0, None, 0, None) == INV
    assert lib.ec_moe_gate(P, P, P, P, 8, 8, 4, 9, None, 0, None) == INV
    assert lib.ec_moe_gate(P, P, None, None, 8, 8, 4, 0, None, 0, None) == INV
    assert lib.ec_moe_gate(P + 4, P, P, P, 8, 8, 4, 0, None, 0, None) == INV
    assert lib.ec_moe_gate(P, P, P, P, 8, 8, 5000, 0, None, 0, None) == INV
    # top-k: k outside [1, n]
    assert lib.ec_moe_topk_tokens(P, 8, 2, 0, P, P, None, 0, None) == INV
    assert lib.ec_moe_topk_tokens(P, 8, 2, 9, P, P, None, 0, None) == INV
    assert lib.ec_moe_topk_tokens(None, 8, 2, 4, P, P, None, 0, None) == INV
    # dispatch: bf16 rows must be multiples of 8 elements
    assert lib.ec_moe_dispatch(P, P, P, 8, 12, 2, 4, 1, None) == INV
    assert lib.ec_moe_dispatch(P, None, P, 8, 16, 2, 4, 1, None) == INV
    # expert FFN: bad activation, missing workspace for the hidden buffer
    assert lib.ec_moe_expert_ffn(P, P, P, P, None, None, 2, 4, 16, 32, 5, 1, P, 1 << 20, None) == INV
    assert lib.ec_moe_expert_ffn(P, P, P, P, None, None, 2, 4, 16, 32, 1, 1, None, 0, None) == WS
    assert lib.ec_moe_expert_ffn(P, P, P, P, None, None, 2, 4, 16, 32, 1, 1, P, 16, None) == WS
    # combine: workspace too small / misaligned
    assert lib.ec_moe_combine(P, P, P, P, 8, 16, 2, 4, 1, P, 8, None) == WS
    assert lib.ec_moe_combine(P, P, P, P, 8, 16, 2, 4, 1, P + 16, 1 << 20, None) == WS
    assert lib.ec_moe_combine(P, P, None, P, 8, 16, 2, 4, 1, P, 1 << 20, None) == INV
    # forward: capacity outside [1, n]; identity experts need the identity activation; one weight missing
    fwd = lambda W1, W2, c, act, ws, wsb: lib.ec_moe_forward(P, P, W1, W2, c, P, None, None, None, None, None,
                                                             None, None, 64, 16, 4, 32, act, 1, ws, wsb, None)
    assert fwd(P, P, 0.001, 1, P, 1 << 30) == INV
    assert fwd(None, None, 2.0, 1, P, 1 << 30) == INV
    assert fwd(P, None, 2.0, 1, P, 1 << 30) == INV
    assert fwd(P, P, 2.0, 1, None, 0) == WS
    assert fwd(P, P, 2.0, 1, P, 64) == WS
    # two-part intermediates: widths outside the matrix-core path are refused
    UNS = -4
    assert lib.ec_moe_forward(P, P, P, P, 2.0, P, None, None, None, None, None, None, None, 64, 16, 4, 32, 1,
                              m.EC_BF16_HILO, P, 1 << 30, None) == UNS
    assert lib.ec_moe_expert_ffn(P, P, P, P, None, None, 2, 4, 16, 32, 1, m.EC_BF16_HILO, P, 1 << 20, None) == UNS
    assert lib.ec_moe_forward_token_choice(P, P, P, P, 2.0, 2, P, None, None, None, None, None, None, None, None, 64, 16,
                                           16, 32, 1, m.EC_BF16_HILO, P, 1 << 30, None) == UNS
    assert lib.ec_moe_forward_capped(P, P, P, P, 2.0, 2.0, 1e-3, 10, P, None, None, None, None, None, 64, 16, 4, 32, 1,
                                     m.EC_BF16_HILO, P, 1 << 30, None) == UNS
    assert lib.ec_moe_backward(*([P] * 16 + [64, 16, 4, 32, 32, 1, m.EC_BF16_HILO, P, 1 << 40, None])) == UNS
    # grouped top-k: the groups must cut the tokens into equal runs; k_g within a run
    assert lib.ec_moe_topk_tokens_grouped(P, 10, 2, 3, 1, P, P, None, 0, None) == INV
    assert lib.ec_moe_topk_tokens_grouped(P, 12, 2, 0, 1, P, P, None, 0, None) == INV
    assert lib.ec_moe_topk_tokens_grouped(P, 12, 2, 3, 5, P, P, None, 0, None) == INV
    fwdg = lambda groups, ws, wsb: lib.ec_moe_forward_grouped(P, P, P, P, 2.0, groups, P, None, None, None, None,
                                                              None, None, None, 64, 16, 4, 32, 1, 1, ws, wsb, None)
    assert fwdg(3, P, 1 << 30) == INV           # 64 tokens do not split into 3 runs
    assert fwdg(64, P, 1 << 30) == INV          # runs of one token: k_g = floor(1*2/4) = 0
    assert fwdg(4, None, 0) == WS
    # token choice: m within [1, min(e, 8)], buffers within [1, n], workspace of 32 n bytes
    tc = lambda mm, cap, ws, wsb: lib.ec_moe_token_choice(P, 64, 4, mm, cap, P, P, None, ws, wsb, None)
    assert tc(0, 16, P, 1 << 20) == INV
    assert tc(5, 16, P, 1 << 20) == INV
    assert tc(2, 0, P, 1 << 20) == INV
    assert tc(2, 65, P, 1 << 20) == INV
    assert tc(2, 16, P, 64) == WS
    assert lib.ec_moe_forward_token_choice(P, P, P, P, 2.0, 9, P, None, None, None, None, None, None, None, None, 64, 16,
                                           16, 32, 1, 1, P, 1 << 30, None) == INV
    # capped expert choice: b and lambda positive and finite, a bounded sweep count, its own workspace
    cap = lambda b, lam, iters, ws, wsb: lib.ec_moe_capped_assignment(P, 64, 4, 16, b, lam, iters, P, ws, wsb, None)
    assert cap(0.0, 1e-3, 10, P, 1 << 30) == INV
    assert cap(2.0, 0.0, 10, P, 1 << 30) == INV
    assert cap(2.0, float("inf"), 10, P, 1 << 30) == INV
    assert cap(2.0, 1e-3, -1, P, 1 << 30) == INV
    assert cap(2.0, 1e-3, 10, P, 64) == WS
    assert m.ec_moe_capped_workspace_bytes(0, 4) == 0 and m.ec_moe_capped_workspace_bytes(64, 4) >= 2 * 64 * 4 * 8
    # the combine without a workspace: same argument checks (its size limit needs a GPU: the array's address is looked up first)
    assert lib.ec_moe_combine_static(P, P, None, P, 8, 16, 2, 4, 1, None) == INV
    assert lib.ec_moe_combine_static(P, P, P, P, 8, 12, 2, 4, 1, None) == INV
    # the timed backward: a host pointer for the stage times is required; stage names
    bwd_args = [P] * 16 + [64, 16, 4, 32, 32, 1, 1, P, 1 << 40, None]
    assert lib.ec_moe_backward_timed(*bwd_args, None) == INV
    assert lib.ec_moe_backward(*([None] + bwd_args[1:])) == INV
    assert lib.ec_moe_backward(*(bwd_args[:-3] + [P, 64, None])) == WS
    assert lib.ec_moe_backward_stage_name(0) == b"bwd_rows" and lib.ec_moe_backward_stage_name(8) == b"bwd_scatter"
    assert lib.ec_moe_backward_stage_name(9) is None and lib.ec_moe_backward_stage_name(-1) is None
    assert m.ec_moe_last_hip_error() == 0      # nothing was launched


def test_the_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own (no C++ constructs, no torch types)
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text('#include "ec_moe.h"\nint main(void) { long long k = 0; return ec_moe_capacity(8, 2, 1.0, (int64_t*)&k); }\n')
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr

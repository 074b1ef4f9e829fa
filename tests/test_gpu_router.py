"""a1 on the GPU against the oracle (Eq. 2, Eq. 3; Section 3.3 router paragraph)."""
import numpy as np
import pytest

import oracle
from moe_inputs import get_config, make_layer_inputs, make_logits
from helpers import GATE_ATOL, GATE_RTOL, LOGIT_ATOL, guard_margins, to_dev, to_host

pytestmark = pytest.mark.gpu


def _gpu_topk(logits32, K, renorm, x=None, w=None, bias=None):
    import torch
    import paper_2504_14960_amd as moe
    T, E = logits32.shape
    lg = to_dev(logits32) if x is None else torch.empty((T, E), dtype=torch.float32, device="cuda")
    idx = torch.full((T, K), -7, dtype=torch.int32, device="cuda")
    gate = torch.full((T, K), -7.0, dtype=torch.float32, device="cuda")
    moe.router_topk(None if x is None else to_dev(x), None if w is None else to_dev(w),
                    None if bias is None else to_dev(bias), lg, K, renorm, idx, gate)
    torch.cuda.synchronize()
    return to_host(lg), to_host(idx), to_host(gate)


@pytest.mark.parametrize("kind", ["normal", "ties", "dupcols", "zeros", "tiny", "equal", "onehot"])
@pytest.mark.parametrize("T,E,K", [(1000, 8, 2), (517, 64, 8), (64, 64, 6), (300, 7, 3), (129, 16, 1),
                                   (200, 4, 4), (150, 100, 5), (90, 256, 64), (33, 1, 1)])
@pytest.mark.parametrize("renorm", [False, True])
def test_selection_on_shared_logits_is_bit_exact(kind, T, E, K, renorm):
    l = make_logits(101, T, E, kind)
    want_idx, want_gate = oracle.topk_gates(l, K, renorm)
    _, idx, gate = _gpu_topk(l, K, renorm)
    np.testing.assert_array_equal(idx, want_idx)
    np.testing.assert_allclose(gate, want_gate, rtol=GATE_RTOL, atol=GATE_ATOL)


def test_nan_logits_rank_last_and_never_index_out_of_range():
    l = make_logits(102, 256, 8, "normal")
    l[::3, 2] = np.nan
    l[5, :] = np.nan
    want_idx, _ = oracle.topk_gates(l, 3, False)
    _, idx, _ = _gpu_topk(l, 3, False)
    np.testing.assert_array_equal(idx, want_idx)


@pytest.mark.parametrize("T,H,E,K,bias,renorm", [
    (1000, 512, 8, 2, None, True),
    (777, 1024, 64, 8, None, False),
    (2100, 256, 64, 6, "zipf1.2", False),
    (300, 264, 5, 3, "normal", True),       # H not a multiple of the slice width
    (250, 128, 100, 4, None, False),
    (130, 192, 200, 7, None, True),
    (20000, 128, 8, 2, "normal", True),     # tall tile variant (T >= 16384)
    (33000, 64, 64, 8, None, False),        # tallest tile variant
    (5, 64, 8, 8, None, True),
])
def test_router_bf16_against_oracle(T, H, E, K, bias, renorm):
    cfg = get_config("mixtral8x7b").scaled(T=T, H=H, E=E, K=K, bias=bias, seed=2000 + E)
    inp = make_layer_inputs(cfg, ["x", "w_router", "bias"])
    guard_margins(inp, K)
    l64 = oracle.router_logits(inp["x"], inp["w_router"], inp.bias)
    want_idx, want_gate = oracle.topk_gates(l64.astype(np.float32), K, renorm)
    logits, idx, gate = _gpu_topk(np.zeros((T, E), np.float32), K, renorm, inp["x"], inp["w_router"], inp.bias)
    assert np.abs(logits - l64).max() <= LOGIT_ATOL
    np.testing.assert_array_equal(idx, want_idx)
    np.testing.assert_allclose(gate, want_gate, rtol=GATE_RTOL, atol=2e-5)


def test_router_fp32_tiny_config():
    cfg = get_config("tiny")
    inp = make_layer_inputs(cfg, ["x", "w_router"])
    guard_margins(inp, cfg.K)
    l64 = oracle.router_logits(inp["x"], inp["w_router"], None)
    want_idx, want_gate = oracle.topk_gates(l64.astype(np.float32), cfg.K, True)
    logits, idx, gate = _gpu_topk(np.zeros((cfg.T, cfg.E), np.float32), cfg.K, True, inp["x"], inp["w_router"])
    assert np.abs(logits - l64).max() <= 1e-5
    np.testing.assert_array_equal(idx, want_idx)
    np.testing.assert_allclose(gate, want_gate, rtol=GATE_RTOL, atol=1e-5)


@pytest.mark.parametrize("tile", [1, 2, 4])
@pytest.mark.parametrize("T,H,E,K,bias,renorm", [
    (1000, 512, 8, 2, "normal", True),      # ragged last tile
    (777, 1032, 64, 8, None, False),        # a ragged last slice
    (333, 264, 5, 3, "normal", True),       # fewer slices than waves
    (260, 96, 20, 4, None, False),          # two expert blocks
    (4100, 6144, 8, 2, "normal", True),     # the benchmark's row length
    (130, 40, 40, 7, None, True),           # three expert blocks
])
def test_every_router_tile_height_against_oracle(T, H, E, K, bias, renorm, tile):
    """The router kernel at every tile height (16, 32, 64 tokens per workgroup) on shapes with ragged tiles, rows
    and expert blocks: logits, indices and gates."""
    import paper_2504_14960_amd as moe
    cfg = get_config("mixtral8x7b").scaled(T=T, H=H, E=E, K=K, bias=bias, seed=2100 + E)
    inp = make_layer_inputs(cfg, ["x", "w_router", "bias"])
    guard_margins(inp, K)
    l64 = oracle.router_logits(inp["x"], inp["w_router"], inp.bias)
    want_idx, want_gate = oracle.topk_gates(l64.astype(np.float32), K, renorm)
    moe.set_option("router_tile", tile)
    try:
        logits, idx, gate = _gpu_topk(np.zeros((T, E), np.float32), K, renorm, inp["x"], inp["w_router"], inp.bias)
    finally:
        moe.set_option("router_tile", 0)
    assert np.abs(logits - l64).max() <= LOGIT_ATOL
    np.testing.assert_array_equal(idx, want_idx)
    np.testing.assert_allclose(gate, want_gate, rtol=GATE_RTOL, atol=2e-5)

"""The whole forward (moe_layer_forward) on the GPU against the oracle's layer."""
import numpy as np
import pytest

import oracle
from moe_inputs import get_config, make_layer_inputs
from helpers import (GATE_ATOL, GATE_RTOL, assert_close, capacity_rows, guard_margins, to_dev, to_host)

pytestmark = pytest.mark.gpu


def run_layer(inp, capacity):
    import torch
    import paper_2504_14960_amd as moe
    cfg = inp.cfg
    dt = moe.MOE_BF16 if cfg.dtype == "bf16" else moe.MOE_F32
    d = {k: to_dev(v) for k, v in inp.tensors.items()}
    bias = None if inp.bias is None else to_dev(inp.bias)
    nbytes = moe.layer_workspace_bytes(cfg.T, cfg.H, cfg.E, cfg.K, cfg.F, cfg.shared_F, capacity, dt)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    y = torch.empty_like(d["x"])
    moe.layer_forward(d["x"], d["w_router"], bias, d["w_gate"], d["w_up"], d["w_down"],
                      d.get("ws_gate"), d.get("ws_up"), d.get("ws_down"), cfg.K, cfg.renormalize, capacity, y, ws)
    torch.cuda.synchronize()
    lay = moe.layer_workspace_layout(cfg.T, cfg.H, cfg.E, cfg.K, cfg.F, cfg.shared_F, capacity, dt)
    A = cfg.T * cfg.K

    def view(name, dtype, n):
        return ws[lay[name]:lay[name] + n * torch.empty((), dtype=dtype).element_size()].view(dtype)

    out = {
        "y": to_host(y),
        "topk_idx": to_host(view("topk_idx", torch.int32, A)).reshape(cfg.T, cfg.K),
        "topk_gate": to_host(view("topk_gate", torch.float32, A)).reshape(cfg.T, cfg.K),
        "row_of_assign": to_host(view("row_of_assign", torch.int32, A)),
        "expert_offsets": to_host(view("expert_offsets", torch.int32, cfg.E + 1)),
    }
    return out


def oracle_layer(inp, capacity):
    t = inp.tensors
    return oracle.layer_forward(t["x"], t["w_router"], inp.bias, t["w_gate"], t["w_up"], t["w_down"],
                                K=inp.cfg.K, renormalize=inp.cfg.renormalize, capacity_rows=capacity,
                                ws_gate=t.get("ws_gate"), ws_up=t.get("ws_up"), ws_down=t.get("ws_down"))


def check_layer(cfg):
    inp = make_layer_inputs(cfg)
    guard_margins(inp, cfg.K)
    capacity = capacity_rows(cfg)
    want = oracle_layer(inp, capacity)
    got = run_layer(inp, capacity)
    np.testing.assert_array_equal(got["topk_idx"], want.idx)
    np.testing.assert_array_equal(got["row_of_assign"], want.row_of_assign)
    assert got["expert_offsets"][-1] == want.R
    np.testing.assert_allclose(got["topk_gate"], want.gate, rtol=GATE_RTOL, atol=2e-5)
    assert_close(got["y"], want.y, cfg.dtype == "bf16", f"y ({cfg.name})")
    return inp, got, want


def test_tiny_config_fp32_end_to_end():
    check_layer(get_config("tiny"))


@pytest.mark.parametrize("base,kw", [
    ("mixtral8x7b", dict(T=1500, H=256, F=512)),                       # 3000 rows, ~3 M-tiles per expert
    ("mixtral8x22b", dict(T=1111, H=384, F=256)),                      # skewed load, ragged everywhere
    ("qwen2_57b_a14b", dict(T=600, H=256, F=128, shared_F=512)),       # 64 experts, top-8, shared expert
    ("tokendrop", dict(T=2048, H=128, F=128)),                         # capacity factor 1, Zipf skew
    ("tokendrop", dict(T=999, H=192, F=64, E=16, K=4, capacity_factor=1.25)),
])
def test_scaled_configs_end_to_end(base, kw):
    cfg = get_config(base).scaled(**kw)
    inp, got, want = check_layer(cfg)
    if cfg.capacity_factor is not None:
        dropped = (want.row_of_assign < 0).sum()
        assert dropped > 0, "the drop recipe was meant to drop something"
        all_dropped = (want.row_of_assign.reshape(cfg.T, cfg.K) < 0).all(axis=1)
        if all_dropped.any():
            from helpers import values
            assert (values(got["y"])[all_dropped] == 0).all()


def test_layer_is_bit_reproducible():
    cfg = get_config("mixtral8x22b").scaled(T=700, H=256, F=256)
    inp = make_layer_inputs(cfg)
    a = run_layer(inp, 0)
    b = run_layer(inp, 0)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])

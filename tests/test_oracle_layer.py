"""Pins for the oracle's expert FFN, the combine step and the whole layer (Eq. 1)."""
import numpy as np
import pytest
import torch

import oracle
from moe_inputs import (bf16_bits_to_f32, get_config, make_layer_inputs, make_logits, make_tokens)


def _small_cfg(**kw):
    base = dict(T=16, H=8, E=4, K=2, F=8)
    base.update(kw)
    return get_config("tiny").scaled(**base)


def _torch_swiglu(x, wg, wu, wd):
    x, wg, wu, wd = (torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in (x, wg, wu, wd))
    h = torch.nn.functional.silu(x @ wg.T) * (x @ wu.T)
    return (h @ wd.T).numpy(), h.numpy()


def test_single_expert_reduces_to_a_dense_swiglu_mlp():
    # E = 1, K = 1: the layer is a plain dense MLP; the gate is softmax of one logit = 1
    cfg = _small_cfg(T=40, H=24, E=1, K=1, F=56)
    inp = make_layer_inputs(cfg)
    res = oracle.layer_forward(inp["x"], inp["w_router"], None, inp["w_gate"], inp["w_up"], inp["w_down"],
                               K=1, renormalize=False)
    want, _ = _torch_swiglu(inp["x"], inp["w_gate"][0], inp["w_up"][0], inp["w_down"][0])
    np.testing.assert_allclose(res.gate, 1.0, rtol=0, atol=0)
    np.testing.assert_allclose(res.y, want, rtol=1e-12, atol=1e-15)


def test_expert_ffn_rows_against_library_ops_bf16_and_h():
    x = make_tokens(31, 9, 32, bf16=True)
    wg = make_tokens(32, 48, 32, bf16=True, std=0.3)
    wu = make_tokens(33, 48, 32, bf16=True, std=0.3)
    wd = make_tokens(34, 32, 48, bf16=True, std=0.3)
    y, h = oracle.expert_ffn_rows(x, wg, wu, wd, want_h=True)
    want_y, want_h = _torch_swiglu(*(bf16_bits_to_f32(a) for a in (x, wg, wu, wd)))
    np.testing.assert_allclose(h, want_h, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(y, want_y, rtol=1e-12, atol=1e-13)
    # swapping the gate and up projections must change the result (silu is on the gate)
    y_sw = oracle.expert_ffn_rows(x, wu, wg, wd)
    assert np.abs(y_sw - y).max() > 1e-3 * np.abs(y).max()


def test_expert_output_is_linear_in_w_down():
    cfg = _small_cfg()
    inp = make_layer_inputs(cfg)
    x = inp["x"][:5]
    y1 = oracle.expert_ffn_rows(x, inp["w_gate"][1], inp["w_up"][1], inp["w_down"][1])
    y2 = oracle.expert_ffn_rows(x, inp["w_gate"][1], inp["w_up"][1], (inp["w_down"][1] * np.float32(4.0)))
    np.testing.assert_array_equal(y2, 4.0 * y1)


def test_grouped_experts_use_each_experts_own_weights_and_rows():
    cfg = _small_cfg(T=50, H=16, E=5, K=2, F=24)
    inp = make_layer_inputs(cfg)
    offsets = np.array([0, 7, 7, 30, 31, 50], dtype=np.int32)   # one empty expert, one single-row expert
    xp = make_tokens(35, 50, 16, bf16=False)
    y, h = oracle.experts(xp, offsets, inp["w_gate"], inp["w_up"], inp["w_down"], want_h=True)
    for e in range(5):
        lo, hi = offsets[e], offsets[e + 1]
        wy, wh = _torch_swiglu(xp[lo:hi], inp["w_gate"][e], inp["w_up"][e], inp["w_down"][e])
        np.testing.assert_allclose(y[lo:hi], wy, rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(h[lo:hi], wh, rtol=1e-12, atol=1e-18)


def test_combine_matches_index_add_formulation():
    T, H, K, R = 30, 12, 3, 120
    rng = np.random.default_rng(5)
    y_perm = rng.standard_normal((R, H))
    gate = rng.random((T, K))
    roa = rng.permutation(R)[:T * K].astype(np.int32)
    roa[::7] = -1                                       # some dropped
    addend = rng.standard_normal((T, H))
    got = oracle.combine(y_perm, roa, gate, addend)
    want = torch.from_numpy(addend.copy())
    kept = np.nonzero(roa >= 0)[0]
    want.index_add_(0, torch.from_numpy(kept // K),
                    torch.from_numpy(gate.reshape(-1)[kept, None] * y_perm[roa[kept]]))
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-13, atol=1e-15)
    got0 = oracle.combine(y_perm, roa, gate, None)
    np.testing.assert_allclose(got0, want.numpy() - addend, rtol=1e-12, atol=1e-14)


def test_identity_experts_round_trip_returns_the_input():
    # permute then unpermute with f_e = identity and gates that sum to one gives x back
    T, H, E = 200, 32, 8
    for K in (1, 2, 4):
        l = make_logits(41, T, E, "normal")
        idx, gate = oracle.topk_gates(l, K, renormalize=True)
        x = make_tokens(42, T, H, bf16=False)
        p = oracle.permute(x, idx, E)
        y = oracle.combine(p.x_perm.astype(np.float64), p.row_of_assign, gate)
        if K == 1:
            np.testing.assert_array_equal(y, x.astype(np.float64))
        else:
            np.testing.assert_allclose(y, x.astype(np.float64), rtol=1e-14, atol=1e-15)


@pytest.mark.parametrize("K", [1, 2, 4])
@pytest.mark.parametrize("capacity", [0, 3, 100])
@pytest.mark.parametrize("renorm", [False, True])
def test_dispatcher_path_equals_dense_equation_one(K, capacity, renorm):
    cfg = _small_cfg(K=K)
    inp = make_layer_inputs(cfg)
    bias = np.array([1.0, 0.0, -0.5, 0.25], dtype=np.float32)   # skew so that capacity 3 really drops
    args = (inp["x"], inp["w_router"], bias, inp["w_gate"], inp["w_up"], inp["w_down"])
    res = oracle.layer_forward(*args, K=K, renormalize=renorm, capacity_rows=capacity)
    y_dense, g = oracle.dense_bruteforce(*args, K=K, renormalize=renorm, capacity_rows=capacity)
    scale = np.abs(y_dense).max()
    np.testing.assert_allclose(res.y, y_dense, rtol=0, atol=1e-12 * scale)
    # the dense gate matrix agrees with the sparse routing result
    g2 = np.zeros_like(g)
    kept = res.row_of_assign.reshape(cfg.T, K) >= 0
    for t in range(cfg.T):
        for k in range(K):
            if kept[t, k]:
                g2[t, res.idx[t, k]] = res.gate[t, k]
    np.testing.assert_allclose(g, g2, rtol=1e-14, atol=0)
    if capacity == 3:
        assert (~kept).any(), "capacity 3 was meant to drop something"
        assert res.R == np.minimum(np.bincount(res.idx.reshape(-1), minlength=cfg.E), 3).sum()
    else:
        assert kept.all() and res.R == cfg.T * K


def test_fully_dropped_tokens_output_exactly_zero():
    cfg = _small_cfg(T=32, K=1)
    inp = make_layer_inputs(cfg)
    bias = np.array([30.0, 0, 0, 0], dtype=np.float32)          # every token picks expert 0
    res = oracle.layer_forward(inp["x"], inp["w_router"], bias, inp["w_gate"], inp["w_up"], inp["w_down"],
                               K=1, renormalize=False, capacity_rows=5)
    assert (res.idx == 0).all() and res.R == 5
    assert (res.y[5:] == 0.0).all()
    assert (np.abs(res.y[:5]).max(axis=1) > 0).all()


def test_k_equals_e_without_renormalisation_is_the_soft_mixture():
    cfg = _small_cfg(K=4)
    inp = make_layer_inputs(cfg)
    res = oracle.layer_forward(inp["x"], inp["w_router"], None, inp["w_gate"], inp["w_up"], inp["w_down"],
                               K=4, renormalize=False)
    x64 = inp["x"].astype(np.float64)
    logits32 = (x64 @ inp["w_router"].astype(np.float64).T).astype(np.float32)
    p = torch.softmax(torch.from_numpy(logits32).double(), dim=1).numpy()
    want = np.zeros((cfg.T, cfg.H))
    for e in range(4):
        ye, _ = _torch_swiglu(inp["x"], inp["w_gate"][e], inp["w_up"][e], inp["w_down"][e])
        want += p[:, e:e + 1] * ye
    np.testing.assert_allclose(res.y, want, rtol=1e-11, atol=1e-14 * np.abs(want).max())


def test_dropless_result_does_not_depend_on_how_tokens_are_batched():
    # Section 3.3: dropless assignments are the same under any split of the tokens
    cfg = get_config("tiny")
    inp = make_layer_inputs(cfg)
    w = (inp["w_router"], None, inp["w_gate"], inp["w_up"], inp["w_down"])
    full = oracle.layer_forward(inp["x"], *w, K=cfg.K, renormalize=True)
    a = oracle.layer_forward(np.ascontiguousarray(inp["x"][:100]), *w, K=cfg.K, renormalize=True)
    b = oracle.layer_forward(np.ascontiguousarray(inp["x"][100:]), *w, K=cfg.K, renormalize=True)
    np.testing.assert_array_equal(full.idx, np.concatenate([a.idx, b.idx]))
    np.testing.assert_allclose(full.y, np.concatenate([a.y, b.y]), rtol=1e-13, atol=1e-18)


def test_shared_expert_is_added_ungated():
    cfg = _small_cfg(T=12, H=16, E=4, K=2, F=8).scaled(shared_F=24)
    inp = make_layer_inputs(cfg)
    w = (inp["w_router"], None, inp["w_gate"], inp["w_up"], inp["w_down"])
    base = oracle.layer_forward(inp["x"], *w, K=2, renormalize=False)
    withs = oracle.layer_forward(inp["x"], *w, K=2, renormalize=False,
                                 ws_gate=inp["ws_gate"], ws_up=inp["ws_up"], ws_down=inp["ws_down"])
    ys, _ = _torch_swiglu(inp["x"], inp["ws_gate"], inp["ws_up"], inp["ws_down"])
    np.testing.assert_allclose(withs.y - base.y, ys, rtol=1e-9, atol=1e-13 * np.abs(ys).max() + 1e-18)


def test_tiny_config_against_a_library_formulation():
    # whole layer at cfg "tiny" rebuilt from torch library ops in fp64 (topk is
    # safe here: iid logits are tie-free, checked)
    cfg = get_config("tiny")
    inp = make_layer_inputs(cfg)
    res = oracle.layer_forward(inp["x"], inp["w_router"], None, inp["w_gate"], inp["w_up"], inp["w_down"],
                               K=cfg.K, renormalize=True)
    x = torch.from_numpy(inp["x"]).double()
    logits32 = (x @ torch.from_numpy(inp["w_router"]).double().T).float()
    assert logits32.unique().numel() == logits32.numel()
    np.testing.assert_array_equal(res.logits32, logits32.numpy())
    p = torch.softmax(logits32.double(), dim=1)
    tv, ti = torch.topk(logits32, cfg.K, dim=1)
    g = torch.gather(p, 1, ti)
    g = g / g.sum(dim=1, keepdim=True)
    want = torch.zeros(cfg.T, cfg.H, dtype=torch.float64)
    for e in range(cfg.E):
        ye, _ = _torch_swiglu(inp["x"], inp["w_gate"][e], inp["w_up"][e], inp["w_down"][e])
        w_e = (g * (ti == e)).sum(dim=1, keepdim=True)
        want += w_e * torch.from_numpy(ye)
    assert (res.idx == ti.numpy()).all()
    np.testing.assert_allclose(res.y, want.numpy(), rtol=1e-10, atol=1e-13 * float(want.abs().max()))
    assert res.R == cfg.T * cfg.K

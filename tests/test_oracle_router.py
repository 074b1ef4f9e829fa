"""Pins for the oracle's router: Eq. 2 and Eq. 3 of the paper (Section 3.1.1).

Each test fixes the oracle to something other than itself: a closed form, a
library routine on a special case, or an exhaustive sort.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from moe_inputs import bf16_bits_to_f32, get_config, make_layer_inputs, make_logits, make_tokens


def _sorted_topk(row, K):
    """Exhaustive selection: full sort by (value desc, index asc); NaN last."""
    key = [(-(-math.inf if math.isnan(v) else float(v)), e) for e, v in enumerate(row)]
    return [e for _, e in sorted(key)][:K]


def test_logits_equal_library_matmul_fp32():
    cfg = get_config("tiny")
    inp = make_layer_inputs(cfg, ["x", "w_router"])
    got = oracle.router_logits(inp["x"], inp["w_router"], None)
    want = inp["x"].astype(np.float64) @ inp["w_router"].astype(np.float64).T
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_logits_bf16_inputs_and_bias():
    x = make_tokens(7, 33, 72, bf16=True)
    w = make_tokens(8, 5, 72, bf16=True, std=0.02)
    bias = np.linspace(-1, 1, 5).astype(np.float32)
    got = oracle.router_logits(x, w, bias)
    want = bf16_bits_to_f32(x).astype(np.float64) @ bf16_bits_to_f32(w).astype(np.float64).T + bias.astype(np.float64)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    # a transposed weight operand would not even have the right shape; a
    # dropped bias would miss by up to 1.0
    assert np.abs(got - (want - bias)).max() > 0.5


def test_equal_logits_give_uniform_gates_and_lowest_indices():
    for E, K in ((8, 2), (64, 8), (5, 5)):
        l = make_logits(1, 17, E, "equal")
        idx, gate = oracle.topk_gates(l, K, renormalize=False)
        assert (idx == np.arange(K, dtype=np.int32)[None, :]).all()
        np.testing.assert_allclose(gate, 1.0 / E, rtol=1e-15)
        _, gate_r = oracle.topk_gates(l, K, renormalize=True)
        np.testing.assert_allclose(gate_r, 1.0 / K, rtol=1e-15)


def test_two_expert_softmax_closed_form():
    # E = 2: softmax reduces to the logistic function of the logit difference
    l = np.array([[0.0, 1.0], [2.5, -0.5], [-3.0, -3.0]], dtype=np.float32)
    idx, gate = oracle.topk_gates(l, 2, renormalize=False)
    for t in range(3):
        d = float(l[t, idx[t, 0]]) - float(l[t, idx[t, 1]])
        assert d >= 0
        assert gate[t, 0] == pytest.approx(1.0 / (1.0 + math.exp(-d)), rel=1e-14)
        assert gate[t, 1] == pytest.approx(1.0 / (1.0 + math.exp(d)), rel=1e-14)
    assert idx.tolist() == [[1, 0], [0, 1], [0, 1]]


def test_k_equals_e_gates_are_the_full_softmax():
    l = make_logits(2, 64, 8, "normal")
    idx, gate, probs = oracle.topk_gates(l, 8, renormalize=False, want_probs=True)
    np.testing.assert_allclose(gate.sum(axis=1), 1.0, rtol=1e-14)
    want = torch.softmax(torch.from_numpy(l).double(), dim=1).numpy()
    np.testing.assert_allclose(probs, want, rtol=1e-13)
    np.testing.assert_allclose(gate, np.take_along_axis(want, idx.astype(np.int64), axis=1), rtol=1e-13)
    # slots are ordered by value, descending
    assert (np.diff(np.take_along_axis(l, idx.astype(np.int64), axis=1), axis=1) <= 0).all()


def test_renormalised_gates_sum_to_one_and_keep_ratios():
    l = make_logits(3, 200, 64, "normal")
    idx, g0 = oracle.topk_gates(l, 6, renormalize=False)
    idx1, g1 = oracle.topk_gates(l, 6, renormalize=True)
    assert (idx == idx1).all()
    np.testing.assert_allclose(g1.sum(axis=1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(g1, g0 / g0.sum(axis=1, keepdims=True), rtol=1e-14)


@pytest.mark.parametrize("kind", ["normal", "ties", "dupcols", "zeros", "tiny", "equal", "onehot"])
@pytest.mark.parametrize("E,K", [(8, 2), (64, 8), (7, 3), (16, 1), (4, 4)])
def test_selection_matches_exhaustive_sort(kind, E, K):
    l = make_logits(11, 96, E, kind)
    idx, _ = oracle.topk_gates(l, K, renormalize=False)
    for t in range(l.shape[0]):
        assert idx[t].tolist() == _sorted_topk(l[t], K), (kind, t)


def test_selection_on_tiny_config_every_token_and_torch_topk():
    cfg = get_config("tiny")
    inp = make_layer_inputs(cfg, ["x", "w_router"])
    l = oracle.router_logits(inp["x"], inp["w_router"], None).astype(np.float32)
    idx, gate = oracle.topk_gates(l, cfg.K, renormalize=True)
    for t in range(cfg.T):
        assert idx[t].tolist() == _sorted_topk(l[t], cfg.K)
    # iid normal logits are tie-free, so torch.topk must agree too
    tv, ti = torch.topk(torch.from_numpy(l), cfg.K, dim=1)
    assert len(np.unique(l)) == l.size
    assert (ti.numpy() == idx).all()
    p = torch.softmax(torch.from_numpy(l).double(), dim=1)
    sel = torch.gather(p, 1, ti)
    np.testing.assert_allclose(gate, (sel / sel.sum(dim=1, keepdim=True)).numpy(), rtol=1e-13)


def test_negative_zero_ties_with_positive_zero_and_nan_ranks_last():
    l = np.array([[-0.0, 0.0, -1.0, 0.0],
                  [np.nan, -5.0, np.nan, -6.0],
                  [1.0, np.nan, 1.0, 2.0]], dtype=np.float32)
    idx, _ = oracle.topk_gates(l, 3, renormalize=False)
    assert idx[0].tolist() == [0, 1, 3]
    assert idx[1].tolist() == [1, 3, 0]
    assert idx[2].tolist() == [3, 0, 2]


def test_softmax_is_shift_invariant_and_max_subtracted():
    l = make_logits(5, 32, 8, "normal")
    _, g0 = oracle.topk_gates(l, 2, renormalize=False)
    # shifting by a power of two keeps the fp32 differences exact
    _, g1 = oracle.topk_gates((l + np.float32(64.0)).astype(np.float32) - np.float32(0.0), 2, renormalize=False)
    l64 = (l.astype(np.float64) + 64.0).astype(np.float32)
    want = torch.softmax(torch.from_numpy(l64).double(), dim=1).numpy()
    idx, _ = oracle.topk_gates(l64, 2, renormalize=False)
    np.testing.assert_allclose(g1, np.take_along_axis(want, idx.astype(np.int64), axis=1), rtol=1e-13)
    # huge logits must not overflow
    big = (l * np.float32(1e30)).astype(np.float32)
    _, gb = oracle.topk_gates(big, 2, renormalize=False)
    assert np.isfinite(gb).all() and (gb[:, 0] <= 1.0).all()
    assert g0.shape == g1.shape

"""Pins for the dispatcher's backward in the oracle (Section 3.3: the backward
workflow mirrors the forward): adjoint identities, finite differences in the
gates, a library scatter-add."""
import numpy as np
import pytest
import torch

import oracle
from helpers import oracle_layer_backward


def _routing(T, E, K, capacity, seed):
    rng = np.random.default_rng(seed)
    idx = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32)
    perm = oracle.permute(None, idx, E, capacity)
    return perm, rng


@pytest.mark.parametrize("T,H,E,K,capacity", [(37, 8, 4, 2, 0), (50, 6, 8, 3, 5), (16, 4, 4, 4, 2)])
def test_combine_backward_is_the_adjoint_of_combine(T, H, E, K, capacity):
    perm, rng = _routing(T, E, K, capacity, 1)
    R = perm.R
    y_perm = rng.normal(size=(max(R, 1), H))
    gate = rng.uniform(0.1, 1.0, size=(T, K))
    dy = rng.normal(size=(T, H))
    dy_perm, dgate = oracle.combine_backward(dy, y_perm, perm.row_of_assign, gate)
    y = oracle.combine(y_perm, perm.row_of_assign, gate)
    # linear in y_perm: <combine(Y), dY> = <Y, dY_perm>
    np.testing.assert_allclose((y * dy).sum(), (y_perm * dy_perm).sum(), rtol=1e-12)
    # linear in the gates: the directional derivative is exact at any step
    d = rng.normal(size=(T, K))
    y2 = oracle.combine(y_perm, perm.row_of_assign, gate + 0.5 * d)
    np.testing.assert_allclose(((y2 - y) * dy).sum() / 0.5, (dgate * d).sum(), rtol=1e-10, atol=1e-12)
    # a dropped assignment has no gradient; rows nobody points at stay zero
    roa = perm.row_of_assign.reshape(T, K)
    assert (dgate[roa < 0] == 0).all()
    untouched = np.setdiff1d(np.arange(y_perm.shape[0]), roa[roa >= 0])
    assert (dy_perm[untouched] == 0).all()
    # one entry by hand
    t, k = np.argwhere(roa >= 0)[0]
    np.testing.assert_allclose(dy_perm[roa[t, k]], gate[t, k] * dy[t], rtol=1e-15)
    np.testing.assert_allclose(dgate[t, k], dy[t] @ y_perm[roa[t, k]], rtol=1e-13)


@pytest.mark.parametrize("T,H,E,K,capacity", [(37, 8, 4, 2, 0), (50, 6, 8, 3, 5)])
def test_permute_backward_is_the_adjoint_of_permute_and_a_scatter_add(T, H, E, K, capacity):
    perm, rng = _routing(T, E, K, capacity, 2)
    R = perm.R
    x = rng.normal(size=(T, H)).astype(np.float32)
    # forward permutation as a gather by the oracle's own map
    xp = np.zeros((max(R, 1), H))
    roa = perm.row_of_assign.reshape(T, K)
    for t in range(T):
        for k in range(K):
            if roa[t, k] >= 0:
                xp[roa[t, k]] = x[t]
    dxp = rng.normal(size=xp.shape)
    add = rng.normal(size=(T, H))
    dx = oracle.permute_backward(dxp, perm.row_of_assign, T, K)
    np.testing.assert_allclose((xp * dxp)[:R].sum(), (x * dx).sum(), rtol=1e-12)
    # library formulation: scatter-add of the kept rows onto their tokens
    want = torch.zeros((T, H), dtype=torch.float64)
    rows = torch.from_numpy(perm.assign_of_row[:R].astype(np.int64) // K)
    want.index_add_(0, rows, torch.from_numpy(dxp[:R]))
    np.testing.assert_allclose(dx, want.numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(oracle.permute_backward(dxp, perm.row_of_assign, T, K, addend=add), dx + add, rtol=1e-13)


def test_backward_of_the_round_trip_with_unit_gates_counts_kept_copies():
    # permute then combine with gates 1 maps x to (number of kept copies) * x; so does its backward
    perm, rng = _routing(40, 8, 2, 7, 3)
    T, K, H = 40, 2, 5
    dy = rng.normal(size=(T, H))
    ones = np.ones((T, K))
    dy_perm, _ = oracle.combine_backward(dy, np.zeros((max(perm.R, 1), H)), perm.row_of_assign, ones)
    dx = oracle.permute_backward(dy_perm, perm.row_of_assign, T, K)
    kept = (perm.row_of_assign.reshape(T, K) >= 0).sum(axis=1)
    np.testing.assert_allclose(dx, kept[:, None] * dy, rtol=1e-15)


def _ffn_case(seed, E, H, F, counts):
    rng = np.random.default_rng(seed)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offsets[-1])
    x = rng.normal(0, 1, (R, H)).astype(np.float32)
    wg = rng.normal(0, 0.3, (E, F, H)).astype(np.float32)
    wu = rng.normal(0, 0.3, (E, F, H)).astype(np.float32)
    wd = rng.normal(0, 0.3, (E, H, F)).astype(np.float32)
    dy = rng.normal(0, 1, (R, H))
    return offsets, x, wg, wu, wd, dy


def test_experts_backward_matches_library_autograd():
    """The same layer written with torch fp64 ops, differentiated by autograd."""
    offsets, x, wg, wu, wd, dy = _ffn_case(20, 3, 12, 9, [5, 0, 7])
    dx, dwg, dwu, dwd = oracle.experts_backward(x, offsets, wg, wu, wd, dy)
    tx, twg, twu, twd = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, wg, wu, wd))
    ys = []
    for e in range(3):
        xe = tx[offsets[e]:offsets[e + 1]]
        ys.append((torch.nn.functional.silu(xe @ twg[e].T) * (xe @ twu[e].T)) @ twd[e].T)
    (torch.cat(ys) * torch.tensor(dy)).sum().backward()
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dwg, twg.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dwu, twu.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dwd, twd.grad.numpy(), rtol=1e-11, atol=1e-13)
    assert (dwg[1] == 0).all() and (dwu[1] == 0).all() and (dwd[1] == 0).all()   # the expert without rows


def test_experts_backward_is_the_directional_derivative_of_the_forward_oracle():
    """Central differences of oracle.experts itself along random directions (all inputs at once)."""
    offsets, x, wg, wu, wd, dy = _ffn_case(21, 2, 8, 6, [4, 3])
    dx, dwg, dwu, dwd = oracle.experts_backward(x, offsets, wg, wu, wd, dy)
    rng = np.random.default_rng(22)
    dirs = [rng.normal(size=a.shape).astype(np.float32) for a in (x, wg, wu, wd)]
    h = np.float32(2.0 ** -9)        # exactly representable steps: the perturbed fp32 inputs are exact
    plus = oracle.experts(x + h * dirs[0], offsets, wg + h * dirs[1], wu + h * dirs[2], wd + h * dirs[3])
    minus = oracle.experts(x - h * dirs[0], offsets, wg - h * dirs[1], wu - h * dirs[2], wd - h * dirs[3])
    # the steps actually taken (fp32 rounding of a +- h d)
    steps = [((a + h * d).astype(np.float64) - (a - h * d).astype(np.float64)) / 2 for a, d in zip((x, wg, wu, wd), dirs)]
    numeric = ((plus - minus) * dy).sum() / 2
    analytic = sum((g * s).sum() for g, s in zip((dx, dwg, dwu, dwd), steps))
    np.testing.assert_allclose(numeric, analytic, rtol=2e-5)


@pytest.mark.parametrize("renorm", [False, True])
@pytest.mark.parametrize("T,H,E,K", [(9, 6, 8, 2), (5, 4, 5, 5), (7, 3, 16, 1)])
def test_router_backward_matches_library_autograd(T, H, E, K, renorm):
    rng = np.random.default_rng(30 + T + E)
    x = rng.normal(0, 1, (T, H)).astype(np.float32)
    w = rng.normal(0, 0.5, (E, H)).astype(np.float32)
    bias = rng.normal(0, 0.5, E).astype(np.float32)
    logits32 = oracle.router_logits(x, w, bias).astype(np.float32)
    idx, gate = oracle.topk_gates(logits32, K, renorm)
    dgate = rng.normal(size=(T, K))
    dl, dx, dw, db = oracle.router_backward(x, w, logits32, idx, dgate, renorm)
    # the same gating written with torch fp64 ops on the same fp32 logits, differentiated by autograd
    tl = torch.tensor(logits32.astype(np.float64), requires_grad=True)
    p = torch.softmax(tl, dim=1)
    g = torch.gather(p, 1, torch.tensor(idx.astype(np.int64)))
    if renorm:
        g = g / g.sum(dim=1, keepdim=True)
    np.testing.assert_allclose(g.detach().numpy(), gate, rtol=1e-12)
    (g * torch.tensor(dgate)).sum().backward()
    np.testing.assert_allclose(dl, tl.grad.numpy(), rtol=1e-10, atol=1e-14)
    # logits = x W^T + bias: the two products and the column sums, with numpy
    np.testing.assert_allclose(dx, dl @ w.astype(np.float64), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dw, dl.T @ x.astype(np.float64), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(db, dl.sum(axis=0), rtol=1e-12, atol=1e-15)
    # softmax is shift invariant: the logit gradients of a token sum to zero
    assert np.abs(dl.sum(axis=1)).max() < 1e-14
    if renorm:
        # renormalised gates sum to one: a constant dgate has no effect
        dl0 = oracle.router_backward(x, w, logits32, idx, np.full((T, K), 3.7), True)[0]
        assert np.abs(dl0).max() < 1e-14


def test_router_backward_ignores_out_of_range_indices():
    rng = np.random.default_rng(40)
    T, H, E, K = 4, 3, 6, 3
    x = rng.normal(size=(T, H)).astype(np.float32)
    w = rng.normal(size=(E, H)).astype(np.float32)
    logits32 = rng.normal(size=(T, E)).astype(np.float32)
    idx = np.array([[0, 7, 2], [1, -1, 3], [5, 4, 0], [2, 3, 99]], dtype=np.int32)
    dgate = rng.normal(size=(T, K))
    dl = oracle.router_backward(x, w, logits32, idx, dgate, False)[0]
    idx_ok = idx.copy()
    dg_ok = dgate.copy()
    bad = (idx < 0) | (idx >= E)
    idx_ok[bad] = 0
    dg_ok[bad] = 0.0          # an out-of-range slot behaves like a slot whose gate gradient is zero
    np.testing.assert_allclose(dl, oracle.router_backward(x, w, logits32, idx_ok, dg_ok, False)[0], rtol=1e-13, atol=1e-16)


@pytest.mark.parametrize("K,renorm,capacity", [(2, True, 0), (2, False, 3), (1, True, 0), (3, True, 4)])
def test_chained_backward_matches_autograd_of_the_whole_layer(K, renorm, capacity):
    """Eq. 1 with Top-K gating, capacity drops and SwiGLU experts, written densely with torch fp64 ops (every expert
    on every token, masked by the oracle's own routing decisions) and differentiated by autograd."""
    rng = np.random.default_rng(50 + K)
    T, H, E, F = 11, 6, 4, 5
    x = rng.normal(0, 1, (T, H)).astype(np.float32)
    wr = rng.normal(0, 0.5, (E, H)).astype(np.float32)
    bias = rng.normal(0, 0.3, E).astype(np.float32)
    wg = rng.normal(0, 0.4, (E, F, H)).astype(np.float32)
    wu = rng.normal(0, 0.4, (E, F, H)).astype(np.float32)
    wd = rng.normal(0, 0.4, (E, H, F)).astype(np.float32)
    dy = rng.normal(size=(T, H))
    got = oracle_layer_backward(x, wr, bias, wg, wu, wd, K, renorm, capacity, dy)
    # routing decisions (piecewise constant) from the forward oracle
    logits32 = oracle.router_logits(x, wr, bias).astype(np.float32)
    idx, _ = oracle.topk_gates(logits32, K, renorm)
    perm = oracle.permute(None, idx, E, capacity)
    kept = torch.tensor(perm.row_of_assign.reshape(T, K) >= 0)

    tx, twr, tb, twg, twu, twd = (torch.tensor(a.astype(np.float64), requires_grad=True) for a in (x, wr, bias, wg, wu, wd))
    # the gating acts on the fp32-rounded logits; the gradient flows through the unrounded product
    tl = tx @ twr.T + tb
    tl = tl + (torch.tensor(logits32.astype(np.float64)) - tl).detach()
    p = torch.softmax(tl, dim=1)
    g = torch.gather(p, 1, torch.tensor(idx.astype(np.int64)))
    if renorm:
        g = g / g.sum(dim=1, keepdim=True)
    y = torch.zeros((T, H), dtype=torch.float64)
    for k in range(K):
        for e in range(E):
            sel = (torch.tensor(idx[:, k]) == e) & kept[:, k]
            if sel.any():
                f = (torch.nn.functional.silu(tx @ twg[e].T) * (tx @ twu[e].T)) @ twd[e].T
                y = y + torch.where(sel[:, None], g[:, k:k + 1] * f, torch.zeros_like(f))
    (y * torch.tensor(dy)).sum().backward()
    for name, t in (("dx", tx), ("dw_router", twr), ("dbias", tb), ("dw_gate", twg), ("dw_up", twu), ("dw_down", twd)):
        np.testing.assert_allclose(got[name], t.grad.numpy(), rtol=1e-9, atol=1e-12, err_msg=name)

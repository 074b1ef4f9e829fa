"""Pins for the dispatcher's backward in the oracle (Section 3.3: the backward
workflow mirrors the forward): adjoint identities, finite differences in the
gates, a library scatter-add."""
import numpy as np
import pytest
import torch

import oracle


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

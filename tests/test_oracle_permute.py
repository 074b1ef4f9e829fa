"""Pins for the oracle's dispatcher permutation and capacity rule.

Section 3.1.2 ("Token Dispatching", "Token Restore") and Eq. 4 of the paper.
"""
import os

import numpy as np
import pytest

import oracle
from moe_inputs import make_logits, make_tokens

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "capacity_eq4.txt")


def _random_idx(seed, T, E, K, skew=False):
    """Distinct experts per token via the oracle-independent route: argsort of noise."""
    l = make_logits(seed, T, E, "onehot" if skew else "normal")
    return np.argsort(-l, axis=1, kind="stable")[:, :K].astype(np.int32)


def test_capacity_closed_form_values():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 6
    for cf, T, K, E, C in rows:
        assert oracle.capacity(float(cf), int(T), int(K), int(E)) == int(C), (cf, T, K, E)


@pytest.mark.parametrize("T,E,K", [(256, 8, 2), (1000, 64, 8), (37, 5, 5), (513, 16, 1)])
def test_dropless_permutation_is_a_stable_sort_by_expert(T, E, K):
    idx = _random_idx(21, T, E, K)
    x = make_tokens(22, T, 16, bf16=False)
    p = oracle.permute(x, idx, E)
    flat = idx.reshape(-1)
    order = np.argsort(flat, kind="stable")           # library routine: stable counting order
    assert p.R == T * K
    assert (p.assign_of_row == order).all()
    inv = np.empty_like(order)
    inv[order] = np.arange(T * K)
    assert (p.row_of_assign == inv).all()
    assert (p.counts == np.bincount(flat, minlength=E)).all()
    assert p.counts.sum() == T * K
    assert (p.offsets == np.concatenate([[0], np.cumsum(p.counts)])).all()
    # rows are byte copies of the source tokens
    assert (p.x_perm == x[order // K]).all()


def test_rows_of_an_expert_are_its_assignments_in_ascending_order():
    T, E, K = 300, 8, 2
    idx = _random_idx(23, T, E, K)
    p = oracle.permute(None, idx, E)
    flat = idx.reshape(-1)
    for e in range(E):
        a = p.assign_of_row[p.offsets[e]:p.offsets[e + 1]]
        assert (flat[a] == e).all()
        assert (np.diff(a) > 0).all()
        assert set(a.tolist()) == set(np.nonzero(flat == e)[0].tolist())


@pytest.mark.parametrize("C", [1, 7, 40, 64])
def test_capacity_keeps_the_first_c_assignments_of_each_expert(C):
    T, E, K = 256, 8, 2
    idx = _random_idx(24, T, E, K, skew=True)         # expert 0 chosen by every token
    x = make_tokens(25, T, 8, bf16=True)
    p = oracle.permute(x, idx, E, capacity_rows=C)
    flat = idx.reshape(-1)
    n = np.bincount(flat, minlength=E)
    assert n[0] == T
    assert (p.counts == np.minimum(n, C)).all()
    assert p.R == p.counts.sum() == p.offsets[E]
    for e in range(E):
        all_a = np.nonzero(flat == e)[0]
        kept, dropped = all_a[:C], all_a[C:]
        assert (p.assign_of_row[p.offsets[e]:p.offsets[e + 1]] == kept).all()
        assert (p.row_of_assign[dropped] == -1).all()
        assert (p.row_of_assign[kept] == p.offsets[e] + np.arange(len(kept))).all()
    assert (p.assign_of_row[p.R:] == -1).all()
    kept_a = np.nonzero(p.row_of_assign >= 0)[0]
    assert (p.assign_of_row[p.row_of_assign[kept_a]] == kept_a).all()
    assert (p.x_perm[:p.R] == x[p.assign_of_row[:p.R] // K]).all()


def test_capacity_at_least_t_equals_dropless():
    T, E, K = 128, 8, 2
    idx = _random_idx(26, T, E, K, skew=True)
    a = oracle.permute(None, idx, E)
    b = oracle.permute(None, idx, E, capacity_rows=T, r_max=T * K)
    assert (a.row_of_assign == b.row_of_assign).all()
    assert (a.counts == b.counts).all() and (a.assign_of_row == b.assign_of_row).all()


def test_capacity_one_keeps_first_token_only():
    T, E, K = 64, 4, 2
    idx = _random_idx(27, T, E, K)
    p = oracle.permute(None, idx, E, capacity_rows=1)
    flat = idx.reshape(-1)
    for e in range(E):
        first = np.nonzero(flat == e)[0][0]
        assert p.assign_of_row[p.offsets[e]] == first
    assert (p.counts == 1).all() and p.R == E


def test_empty_experts_and_out_of_range_indices():
    idx = np.array([[3, 1], [3, 9], [-1, 3], [1, 3]], dtype=np.int32)   # experts 0, 2 empty; 9 and -1 invalid
    p = oracle.permute(None, idx, 4)
    assert p.counts.tolist() == [0, 2, 0, 4]
    assert p.offsets.tolist() == [0, 0, 2, 2, 6]
    assert p.row_of_assign.tolist() == [2, 0, 3, -1, -1, 4, 1, 5]
    assert p.assign_of_row.tolist() == [1, 6, 0, 2, 5, 7, -1, -1]

"""Pins of the oracle's dispatch variants (drop by score, pad to capacity): numpy brute force, closed-form special
cases, a hand-worked example, and agreement with the position/packed oracle where the variants coincide."""
import numpy as np
import pytest

import oracle
from moe_inputs import make_tokens


def _case(seed, T, E, K, skew=1.5):
    rng = np.random.default_rng(seed)
    # distinct experts per token, skewed popularity so that some experts overflow
    p = 1.0 / np.arange(1, E + 1) ** skew
    p /= p.sum()
    idx = np.stack([rng.choice(E, size=K, replace=False, p=p) for _ in range(T)]).astype(np.int32)
    scores = rng.random((T, K)).astype(np.float32)
    return idx, scores


def _brute(idx, scores, E, C, by_score):
    """Kept set and rows straight from the definition, with numpy sorts."""
    T, K = idx.shape
    flat = idx.reshape(-1)
    s = scores.reshape(-1)
    roa = np.full(T * K, -1, dtype=np.int64)
    counts = np.zeros(E, dtype=np.int64)
    kept_lists = []
    for e in range(E):
        a = np.nonzero(flat == e)[0]
        if by_score:
            order = np.lexsort((a, -s[a].astype(np.float64)))     # score descending, then index ascending
            a = a[order]
        kept = np.sort(a[:C] if C > 0 else a)
        kept_lists.append(kept)
        counts[e] = kept.size
    return kept_lists, counts


@pytest.mark.parametrize("by_score", [False, True])
@pytest.mark.parametrize("pad", [False, True])
@pytest.mark.parametrize("T,E,K,C", [(64, 4, 2, 9), (200, 8, 3, 20), (33, 5, 5, 4), (50, 6, 1, 1)])
def test_variant_against_numpy_brute_force(T, E, K, C, by_score, pad):
    idx, scores = _case(T + E, T, E, K)
    x = make_tokens(T, T, 8, bf16=False)
    got = oracle.permute_variant(x, idx, scores, E, C, by_score, pad)
    kept_lists, counts = _brute(idx, scores, E, C, by_score)
    np.testing.assert_array_equal(got.counts, counts)
    start = 0
    for e in range(E):
        lo = e * C if pad else start
        assert got.offsets[e] == lo
        rows = np.arange(lo, lo + counts[e])
        np.testing.assert_array_equal(got.assign_of_row[rows], kept_lists[e])
        np.testing.assert_array_equal(got.row_of_assign[kept_lists[e]], rows)
        np.testing.assert_array_equal(got.x_perm[rows], x[kept_lists[e] // K])
        if pad:
            tail = np.arange(lo + counts[e], lo + C)
            assert (got.assign_of_row[tail] == -1).all() and (got.x_perm[tail] == 0).all()
        start += counts[e]
    assert got.offsets[E] == (E * C if pad else counts.sum())
    all_kept = np.concatenate(kept_lists)
    dropped = np.setdiff1d(np.arange(T * K), all_kept)
    assert (got.row_of_assign[dropped] == -1).all()


def test_position_packed_variant_is_the_plain_dispatch():
    idx, scores = _case(5, 120, 8, 2)
    for C in (0, 7, 1000):
        a = oracle.permute_variant(None, idx, scores, 8, C, False, False)
        b = oracle.permute(None, idx, 8, C)
        for f in ("counts", "offsets", "row_of_assign", "assign_of_row"):
            np.testing.assert_array_equal(getattr(a, f), getattr(b, f))


def test_equal_scores_drop_by_position():
    idx, _ = _case(6, 90, 4, 2)
    flat = np.full(idx.shape, 0.25, dtype=np.float32)
    a = oracle.permute_variant(None, idx, flat, 4, 11, True, False)
    b = oracle.permute(None, idx, 4, 11)
    np.testing.assert_array_equal(a.row_of_assign, b.row_of_assign)


def test_capacity_one_keeps_each_experts_best_assignment():
    idx, scores = _case(7, 40, 5, 2)
    got = oracle.permute_variant(None, idx, scores, 5, 1, True, False)
    flat, s = idx.reshape(-1), scores.reshape(-1)
    for e in range(5):
        a = np.nonzero(flat == e)[0]
        if a.size:
            best = a[np.argmax(s[a])]           # argmax returns the first of equal maxima = lowest index
            assert got.assign_of_row[got.offsets[e]] == best and got.counts[e] == 1


def test_no_overflow_means_no_drop_under_either_rule():
    idx, scores = _case(8, 30, 4, 2)
    a = oracle.permute_variant(None, idx, scores, 4, 60, True, False)
    b = oracle.permute(None, idx, 4, 0)
    np.testing.assert_array_equal(a.row_of_assign, b.row_of_assign)


def test_hand_worked_example():
    # 4 tokens, K = 2, E = 3, capacity 2.  Assignments a = 2t + k:
    #   a: 0  1  2  3  4  5  6  7
    #   e: 0  1  0  2  0  1  0  1
    #   s: .1 .9 .8 .5 .8 .2 .3 .7
    idx = np.array([[0, 1], [0, 2], [0, 1], [0, 1]], dtype=np.int32)
    s = np.array([[.1, .9], [.8, .5], [.8, .2], [.3, .7]], dtype=np.float32)
    # expert 0 has a = 0, 2, 4, 6 with scores .1 .8 .8 .3: keeps 2 and 4 (tie: both fit); expert 1 has a = 1, 5, 7
    # with .9 .2 .7: keeps 1 and 7; expert 2 keeps 3.
    got = oracle.permute_variant(None, idx, s, 3, 2, True, False)
    np.testing.assert_array_equal(got.counts, [2, 2, 1])
    np.testing.assert_array_equal(got.offsets, [0, 2, 4, 5])
    np.testing.assert_array_equal(got.row_of_assign, [-1, 2, 0, 4, 1, -1, -1, 3])
    np.testing.assert_array_equal(got.assign_of_row[:5], [2, 4, 1, 7, 3])
    # capacity 1: the tie at .8 goes to the lower assignment index
    got1 = oracle.permute_variant(None, idx, s, 3, 1, True, False)
    np.testing.assert_array_equal(got1.row_of_assign, [-1, 1, 0, 2, -1, -1, -1, -1])
    # padded to capacity 2: expert 2's block has one zero row
    gotp = oracle.permute_variant(None, idx, s, 3, 2, True, True)
    np.testing.assert_array_equal(gotp.offsets, [0, 2, 4, 6])
    np.testing.assert_array_equal(gotp.assign_of_row, [2, 4, 1, 7, 3, -1])
    np.testing.assert_array_equal(gotp.counts, [2, 2, 1])


def test_padded_layout_gives_the_same_layer_output():
    """Zero rows pass through the bias-free SwiGLU FFN as zeros and no assignment points at them."""
    rng = np.random.default_rng(11)
    T, H, E, K, F, C = 40, 8, 4, 2, 6, 12
    idx, scores = _case(12, T, E, K)
    x = make_tokens(13, T, H, bf16=False)
    wg, wu = (rng.normal(0, 0.3, (E, F, H)).astype(np.float32) for _ in range(2))
    wd = rng.normal(0, 0.3, (E, H, F)).astype(np.float32)
    gate = rng.random((T, K))
    ys = []
    for pad in (False, True):
        p = oracle.permute_variant(x, idx, scores, E, C, True, pad)
        y_perm = oracle.experts(p.x_perm, p.offsets, wg, wu, wd)
        if pad:
            assert (y_perm[p.assign_of_row < 0] == 0).all()
        ys.append(oracle.combine(y_perm, p.row_of_assign, gate))
    np.testing.assert_allclose(ys[0], ys[1], rtol=1e-13, atol=1e-15)

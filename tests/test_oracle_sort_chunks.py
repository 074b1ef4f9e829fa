"""Pins of the oracle's chunk gather (the one-GPU step of expert-parallel dispatch, Section 3.3): numpy
split/concatenate, the inverse order, closed-form offsets, the stated edge rules, and a simulated expert-parallel
group whose result must equal the one-GPU layer (itself pinned by the dense brute force of Eq. 1)."""
import numpy as np
import pytest

import oracle
from helpers import ep_chunk_orders, oracle_ep_group_forward
from moe_inputs import get_config, make_layer_inputs, make_tokens


def _sizes(seed, n, hi):
    rng = np.random.default_rng(seed)
    rows = rng.integers(0, hi + 1, size=n).astype(np.int32)
    rows[rng.random(n) < 0.2] = 0                      # empty chunks are common: an expert nobody chose
    return rng, rows


@pytest.mark.parametrize("n,hi,H", [(1, 5, 4), (6, 7, 8), (64, 40, 16), (257, 9, 4)])
def test_against_numpy_split_concatenate(n, hi, H):
    rng, rows = _sizes(n, n, hi)
    src = make_tokens(n, int(rows.sum()), H, bf16=False)
    order = rng.permutation(n).astype(np.int32)
    parts = np.split(src, np.cumsum(rows)[:-1])
    want = np.concatenate([parts[c] for c in order]) if rows.sum() else src[:0]
    dst, rows_out, goff, total = oracle.sort_chunks(src, rows, order, group=1)
    assert total == rows.sum()
    np.testing.assert_array_equal(dst, want)
    np.testing.assert_array_equal(rows_out, rows[order])
    np.testing.assert_array_equal(goff, np.concatenate([[0], np.cumsum(rows[order])]))


def test_inverse_order_restores_the_source():
    rng, rows = _sizes(3, 48, 11)
    src = make_tokens(5, int(rows.sum()), 8, bf16=True)
    order = rng.permutation(48).astype(np.int32)
    dst, rows_out, _, _ = oracle.sort_chunks(src, rows, order)
    inverse = np.argsort(order).astype(np.int32)
    back, rows_back, _, _ = oracle.sort_chunks(dst, rows_out, inverse)
    np.testing.assert_array_equal(back, src)
    np.testing.assert_array_equal(rows_back, rows)


def test_identity_order_is_a_copy_and_group_offsets_are_block_sums():
    _, rows = _sizes(9, 24, 6)
    src = make_tokens(2, int(rows.sum()), 4, bf16=False)
    dst, _, goff, total = oracle.sort_chunks(src, rows, np.arange(24), group=4)
    np.testing.assert_array_equal(dst, src)
    np.testing.assert_array_equal(goff, np.concatenate([[0], np.cumsum(rows.reshape(6, 4).sum(1))]))
    assert total == goff[-1]


def test_hand_worked_example():
    # chunks A (1 row), B (2 rows), C (0 rows), D (3 rows); wanted D, A, C, B
    src = np.arange(6, dtype=np.float32).reshape(6, 1) * 10
    dst, rows_out, goff, total = oracle.sort_chunks(src, [1, 2, 0, 3], [3, 0, 2, 1], group=2)
    np.testing.assert_array_equal(dst[:, 0], [30, 40, 50, 0, 10, 20])
    np.testing.assert_array_equal(rows_out, [3, 1, 0, 2])
    np.testing.assert_array_equal(goff, [0, 4, 6])
    assert total == 6


def test_edge_rules_repeats_out_of_range_negative_and_truncation():
    src = np.arange(5, dtype=np.float32).reshape(5, 1) + 1
    # a chunk named twice is copied twice; index outside the source and a negative count are empty chunks
    dst, rows_out, _, total = oracle.sort_chunks(src, [2, -3, 3], [0, 0, 7, -1, 1, 2])
    np.testing.assert_array_equal(rows_out, [2, 2, 0, 0, 0, 3])
    np.testing.assert_array_equal(dst[:, 0], [1, 2, 1, 2, 3, 4, 5])
    assert total == 7
    # destination shorter than the total: the rows that fit are written, the total is still reported
    dst, _, _, total = oracle.sort_chunks(src, [2, 3], [1, 0], r_dst=4)
    np.testing.assert_array_equal(dst[:, 0], [3, 4, 5, 1])
    assert total == 5
    # source shorter than its chunk sizes claim: rows past its end are not read
    dst, _, _, total = oracle.sort_chunks(src[:3], [2, 3], [1, 0], r_dst=5)
    np.testing.assert_array_equal(dst[:, 0], [3, 0, 0, 1, 2])
    # nothing at all
    dst, rows_out, goff, total = oracle.sort_chunks(src[:0], [], [], group=1)
    assert dst.shape[0] == 0 and rows_out.size == 0 and total == 0 and list(goff) == [0]


def test_ep_orders_are_mutually_inverse():
    for S, El in [(1, 1), (2, 4), (8, 8), (4, 1), (1, 8)]:
        by_expert, by_source = ep_chunk_orders(S, El)
        np.testing.assert_array_equal(by_source[by_expert], np.arange(S * El))
        np.testing.assert_array_equal(by_expert[by_source], np.arange(S * El))


@pytest.mark.parametrize("S,capacity", [(1, 0), (2, 0), (4, 0), (8, 0), (4, 5)])
def test_simulated_ep_group_equals_one_gpu_layer(S, capacity):
    cfg = get_config("tiny")
    inp = make_layer_inputs(cfg)
    x_all, w_router, w_gate, w_up, w_down = (inp[n] for n in ("x", "w_router", "w_gate", "w_up", "w_down"))
    assert cfg.E % S == 0
    # ranks hold different numbers of tokens (ragged split of the batch), one of them possibly few
    T = cfg.T
    cuts = np.linspace(0, T, S + 1).astype(int)
    if S > 1:
        cuts[1] = max(1, cuts[1] // 3)
    xs = [x_all[cuts[s]:cuts[s + 1]] for s in range(S)]
    ys = oracle_ep_group_forward(xs, w_router, inp.bias, w_gate, w_up, w_down, cfg.K, cfg.renormalize, capacity)
    for x, y in zip(xs, ys):
        ref = oracle.layer_forward(x, w_router, inp.bias, w_gate, w_up, w_down, cfg.K, cfg.renormalize, capacity)
        # the same rows through the same per-row arithmetic: identical up to nothing at all
        np.testing.assert_array_equal(y, ref.y)

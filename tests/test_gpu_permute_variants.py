"""Dispatch variants on the GPU (drop by score, pad to capacity) against the oracle, bit for bit."""
import numpy as np
import pytest

import oracle
from moe_inputs import make_logits, make_tokens
from helpers import to_dev, to_host

pytestmark = pytest.mark.gpu


def _routing(seed, T, E, K, kind, renorm=False, quantise=0):
    idx, gate = oracle.topk_gates(make_logits(seed, T, E, kind), K, renorm)
    scores = gate.astype(np.float32)
    if quantise:      # many exactly equal scores: the index tie-break decides
        scores = (np.floor(scores * quantise) / quantise).astype(np.float32)
    return idx, scores


def _gpu(x, idx, scores, E, capacity, by_score, pad, extra_rows=0):
    import torch
    import paper_2504_14960_amd as moe
    T, K = idx.shape
    r_max = (E * capacity if pad else moe.max_rows(T, K, E, capacity)) + extra_rows
    dx = None if x is None else to_dev(x)
    x_perm = None if x is None else torch.full((r_max, x.shape[1]), 3.0, dtype=dx.dtype, device="cuda")
    counts = torch.full((E,), -3, dtype=torch.int32, device="cuda")
    offsets = torch.full((E + 1,), -3, dtype=torch.int32, device="cuda")
    roa = torch.full((T * K,), -3, dtype=torch.int32, device="cuda")
    aor = torch.full((max(r_max, 1),), -3, dtype=torch.int32, device="cuda")
    ws = torch.empty(moe.permute_variant_workspace_bytes(T, K, E) + 16, dtype=torch.uint8, device="cuda")
    moe.permute_variant(dx, to_dev(idx), None if scores is None else to_dev(scores), E, capacity, by_score, pad,
                        x_perm, counts, offsets, roa, aor[:r_max] if r_max else aor[:0], ws, H=8)
    torch.cuda.synchronize()
    return (None if x is None else to_host(x_perm)), to_host(counts), to_host(offsets), to_host(roa), to_host(aor)[:r_max]


def _check(T, H, E, K, capacity, kind, by_score, pad, quantise=0, bf16=True, extra_rows=0, seed=0):
    idx, scores = _routing(700 + T + seed, T, E, K, kind, quantise=quantise)
    x = make_tokens(701 + seed, T, H, bf16=bf16)
    r_max = (E * capacity if pad else min(T * K, E * capacity) if capacity > 0 else T * K) + extra_rows
    want = oracle.permute_variant(x, idx, scores, E, capacity, by_score, pad, r_max=r_max)
    x_perm, counts, offsets, roa, aor = _gpu(x, idx, scores, E, capacity, by_score, pad, extra_rows)
    np.testing.assert_array_equal(counts, want.counts)
    np.testing.assert_array_equal(offsets, want.offsets)
    np.testing.assert_array_equal(roa, want.row_of_assign)
    np.testing.assert_array_equal(aor, want.assign_of_row)
    owned = want.assign_of_row >= 0
    np.testing.assert_array_equal(x_perm[owned], want.x_perm[owned])
    if pad:
        assert (x_perm[: E * capacity][~owned[: E * capacity]] == 0).all(), "padding rows must be zero"
    else:
        rest = x_perm[~owned]
        assert rest.size == 0 or (rest == rest.reshape(-1)[0]).all(), "rows nobody owns must be left untouched"
    return want


@pytest.mark.parametrize("by_score,pad", [(True, False), (False, True), (True, True)])
@pytest.mark.parametrize("T,H,E,K,capacity,kind,quantise", [
    (2048, 256, 16, 4, 512, "onehot", 0),       # heavy drops on expert 0
    (5000, 64, 64, 6, 469, "onehot", 0),
    (40000, 16, 64, 6, 3750, "normal", 0),      # 235 chunks
    (3000, 72, 8, 2, 300, "normal", 16),        # scores on a grid of 16 values: ties everywhere
    (300, 40, 8, 1, 1, "normal", 0),            # capacity 1
    (600, 24, 256, 64, 100, "normal", 0),       # the limits of E and K
    (37, 3072, 5, 5, 40, "normal", 0),          # nothing overflows
    (1, 8, 4, 2, 3, "normal", 0),
])
def test_variants_are_bit_exact(T, H, E, K, capacity, kind, quantise, by_score, pad):
    _check(T, H, E, K, capacity, kind, by_score, pad, quantise=quantise)


def test_every_token_to_one_expert_and_constant_scores():
    import torch  # noqa: F401
    T, E, K, C = 5000, 4, 1, 777
    idx = np.full((T, K), 2, dtype=np.int32)
    x = make_tokens(5, T, 32, bf16=True)
    for scores in (np.full((T, K), 0.5, dtype=np.float32),                       # all equal: first C by index
                   np.linspace(-1, 1, T, dtype=np.float32).reshape(T, K),         # negative scores, best last
                   np.where(np.arange(T) % 2, 0.0, -0.0).astype(np.float32).reshape(T, K)):   # +0 and -0 tie
        want = oracle.permute_variant(x, idx, scores, E, C, True, False)
        x_perm, counts, offsets, roa, aor = _gpu(x, idx, scores, E, C, True, False)
        np.testing.assert_array_equal(counts, want.counts)
        np.testing.assert_array_equal(offsets, want.offsets)
        np.testing.assert_array_equal(roa, want.row_of_assign)
        np.testing.assert_array_equal(aor, want.assign_of_row)
        np.testing.assert_array_equal(x_perm[:C], want.x_perm[:C])


def test_plain_flags_reproduce_moe_permute_and_invalid_indices_are_dropped():
    idx, scores = _routing(9, 700, 8, 2, "normal")
    idx = idx.copy()
    idx[5, 0] = -1
    idx[9, 1] = 8
    idx[11, 0] = 1 << 30
    for by_score, pad in ((False, False), (True, False), (True, True)):
        want = oracle.permute_variant(None, idx, scores, 8, 150, by_score, pad)
        _, counts, offsets, roa, aor = _gpu(None, idx, scores, 8, 150, by_score, pad)
        np.testing.assert_array_equal(roa, want.row_of_assign)
        np.testing.assert_array_equal(aor, want.assign_of_row)
        np.testing.assert_array_equal(counts, want.counts)
        np.testing.assert_array_equal(offsets, want.offsets)
    plain = oracle.permute(None, idx, 8, 150)
    _, counts, offsets, roa, aor = _gpu(None, idx, None, 8, 150, False, False)
    np.testing.assert_array_equal(roa, plain.row_of_assign)
    np.testing.assert_array_equal(aor, plain.assign_of_row)


def test_extra_rows_are_marked_unused_and_left_alone():
    _check(900, 64, 8, 2, 100, "onehot", True, False, extra_rows=37)
    _check(900, 64, 8, 2, 100, "onehot", True, True, extra_rows=37, seed=1)


def test_argument_errors():
    import torch
    import paper_2504_14960_amd as moe
    idx = torch.zeros((4, 2), dtype=torch.int32, device="cuda")
    i32 = dict(dtype=torch.int32, device="cuda")
    counts, offsets, roa, aor = torch.zeros(4, **i32), torch.zeros(5, **i32), torch.zeros(8, **i32), torch.zeros(8, **i32)
    ws = torch.empty(moe.permute_variant_workspace_bytes(4, 2, 4), dtype=torch.uint8, device="cuda")
    with pytest.raises(RuntimeError):     # padded layout without a capacity
        moe.permute_variant(None, idx, None, 4, 0, False, True, None, counts, offsets, roa, aor, ws)
    with pytest.raises(RuntimeError):     # drop by score without scores
        moe.permute_variant(None, idx, None, 4, 1, True, False, None, counts, offsets, roa, aor, ws)
    with pytest.raises(RuntimeError):     # too few rows for the padded layout
        moe.permute_variant(None, idx, None, 4, 3, False, True, None, counts, offsets, roa, aor, ws)


def test_padded_dispatch_through_the_expert_ffn_and_combine():
    """The padded layout end to end: equal groups through the grouped GEMM, zero rows stay zero, same y."""
    import torch
    import paper_2504_14960_amd as moe
    from moe_inputs import get_config, make_layer_inputs
    from helpers import assert_close, guard_margins
    cfg = get_config("tokendrop").scaled(T=1536, H=256, F=256)
    inp = make_layer_inputs(cfg)
    guard_margins(inp, cfg.K)
    t = inp.tensors
    T, H, E, K, F = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F
    C = moe.capacity_from_factor(cfg.capacity_factor, T, K, E)
    l64 = oracle.router_logits(t["x"], t["w_router"], inp.bias)
    idx, gate = oracle.topk_gates(l64.astype(np.float32), K, cfg.renormalize)
    scores = gate.astype(np.float32)
    p = oracle.permute_variant(t["x"], idx, scores, E, C, True, True)
    y_ref = oracle.combine(oracle.experts(p.x_perm, p.offsets, t["w_gate"], t["w_up"], t["w_down"]), p.row_of_assign, gate)

    bf = dict(dtype=torch.bfloat16, device="cuda")
    r_max = E * C
    x_perm, counts, offsets, roa, aor = (torch.empty((r_max, H), **bf), torch.empty(E, dtype=torch.int32, device="cuda"),
                                         torch.empty(E + 1, dtype=torch.int32, device="cuda"),
                                         torch.empty(T * K, dtype=torch.int32, device="cuda"),
                                         torch.empty(r_max, dtype=torch.int32, device="cuda"))
    ws = torch.empty(moe.permute_variant_workspace_bytes(T, K, E), dtype=torch.uint8, device="cuda")
    moe.permute_variant(to_dev(t["x"]), to_dev(idx), to_dev(scores), E, C, True, True, x_perm, counts, offsets, roa, aor, ws)
    h, y_perm, y = torch.empty((r_max, F), **bf), torch.empty((r_max, H), **bf), torch.empty((T, H), **bf)
    moe.grouped_gemm_swiglu(x_perm, offsets, to_dev(t["w_gate"]), to_dev(t["w_up"]), to_dev(t["w_down"]), h, y_perm)
    moe.unpermute_combine(y_perm, roa, to_dev(gate.astype(np.float32)), None, y)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(roa), p.row_of_assign)
    from helpers import values
    assert (values(to_host(y_perm))[p.assign_of_row < 0] == 0).all()
    assert_close(to_host(y), y_ref, True, "y (padded, drop by score)")

"""Backward of the dispatcher's data movements on the GPU against the oracle."""
import numpy as np
import pytest

import oracle
from moe_inputs import make_logits, make_tokens
from helpers import assert_close, to_dev, to_host, values

pytestmark = pytest.mark.gpu


def _setup(T, H, E, K, capacity, bf16, seed):
    logits = make_logits(seed, T, E, "normal")
    idx, gate = oracle.topk_gates(logits, K, True)
    perm = oracle.permute(None, idx, E, capacity)
    r_max = max(perm.R + 5, 1)
    y_perm = make_tokens(seed + 1, r_max, H, bf16=bf16)
    dy = make_tokens(seed + 2, T, H, bf16=bf16)
    return perm, gate.astype(np.float32), y_perm, dy, r_max


@pytest.mark.parametrize("T,H,E,K,capacity,bf16", [
    (300, 256, 8, 2, 0, True), (1000, 136, 16, 4, 150, True), (257, 1032, 64, 8, 0, True), (64, 64, 4, 1, 3, True),
    (90, 128, 64, 33, 0, True), (200, 64, 8, 2, 20, False),
])
def test_combine_backward_against_oracle(T, H, E, K, capacity, bf16):
    import torch
    import paper_2504_14960_amd as moe
    perm, gate, y_perm, dy, r_max = _setup(T, H, E, K, capacity, bf16, 7000 + T)
    want_dyp, want_dg = oracle.combine_backward(values(dy), values(y_perm), perm.row_of_assign, gate)
    d_dy, d_yp = to_dev(dy), to_dev(y_perm)
    dy_perm = torch.zeros_like(d_yp)
    dgate = torch.full((T, K), 123.0, dtype=torch.float32, device="cuda")
    moe.unpermute_combine_backward(d_dy, d_yp, to_dev(perm.row_of_assign), to_dev(gate), dy_perm, dgate)
    torch.cuda.synchronize()
    got = to_host(dy_perm)
    assert_close(got, want_dyp, bf16, "dy_perm")
    assert (values(got)[perm.R:] == 0).all()                      # rows nobody points at are untouched
    got_dg = dgate.cpu().numpy()
    roa = perm.row_of_assign.reshape(T, K)
    assert (got_dg[roa < 0] == 0).all()                           # dropped assignments: exactly zero
    # fp32 dot products over H terms against fp64: relative to the norms of the two rows
    bound = 1e-5 * np.linalg.norm(values(dy), axis=1)[:, None] * np.abs(values(y_perm)).max() * np.sqrt(H) + 1e-30
    assert (np.abs(got_dg - want_dg) <= bound).all()


@pytest.mark.parametrize("T,H,E,K,capacity,bf16,with_addend", [
    (300, 256, 8, 2, 0, True, False), (1000, 136, 16, 4, 150, True, True), (257, 1032, 64, 8, 0, True, False),
    (200, 64, 8, 2, 20, False, True),
])
def test_permute_backward_against_oracle(T, H, E, K, capacity, bf16, with_addend):
    import torch
    import paper_2504_14960_amd as moe
    perm, _, dx_perm, add, r_max = _setup(T, H, E, K, capacity, bf16, 7100 + T)
    addend = add if with_addend else None
    want = oracle.permute_backward(values(dx_perm), perm.row_of_assign, T, K,
                                   None if addend is None else values(addend))
    dx = torch.empty((T, H), dtype=to_dev(dx_perm).dtype, device="cuda")
    moe.permute_backward(to_dev(dx_perm), to_dev(perm.row_of_assign), None if addend is None else to_dev(addend), dx, K)
    torch.cuda.synchronize()
    assert_close(to_host(dx), want, bf16, "dx")
    if not with_addend:
        none_kept = (perm.row_of_assign.reshape(T, K) < 0).all(axis=1)
        assert (values(to_host(dx))[none_kept] == 0).all()

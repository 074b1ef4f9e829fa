"""a2 and a4 on the GPU against the oracle (Section 3.1.2; Eq. 4; Eq. 1's sum)."""
import numpy as np
import pytest

import oracle
from moe_inputs import make_logits, make_tokens
from helpers import assert_close, to_dev, to_host, values

pytestmark = pytest.mark.gpu


def _idx(seed, T, E, K, kind="normal"):
    l = make_logits(seed, T, E, kind)
    return oracle.topk_gates(l, K, True)


def _gpu_permute(x, idx, E, capacity):
    import torch
    import paper_2504_14960_amd as moe
    T, K = idx.shape
    r_max = moe.max_rows(T, K, E, capacity)
    dx = None if x is None else to_dev(x)
    x_perm = None if x is None else torch.zeros((r_max, x.shape[1]), dtype=dx.dtype, device="cuda")
    counts = torch.full((E,), -3, dtype=torch.int32, device="cuda")
    offsets = torch.full((E + 1,), -3, dtype=torch.int32, device="cuda")
    roa = torch.full((T * K,), -3, dtype=torch.int32, device="cuda")
    aor = torch.full((max(r_max, 1),), -3, dtype=torch.int32, device="cuda")
    ws = torch.empty(moe.permute_workspace_bytes(T, K, E) + 16, dtype=torch.uint8, device="cuda")
    moe.permute(dx, to_dev(idx), E, capacity, x_perm, counts, offsets, roa, aor, ws, H=8)
    torch.cuda.synchronize()
    return (None if x is None else to_host(x_perm)), to_host(counts), to_host(offsets), to_host(roa), to_host(aor)[:r_max]


@pytest.mark.parametrize("T,H,E,K,capacity,kind,bf16", [
    (256, 128, 8, 2, 0, "normal", False),
    (1000, 512, 8, 2, 0, "normal", True),
    (3000, 72, 64, 8, 0, "normal", True),        # 144-byte rows, 24 chunks
    (2048, 256, 16, 4, 512, "onehot", True),     # heavy drops on expert 0
    (5000, 64, 64, 6, 469, "onehot", True),
    (40000, 16, 64, 6, 3750, "normal", True),    # 235 chunks
    (37, 3072, 5, 5, 0, "normal", True),         # 6 KiB rows, K = E
    (600, 24, 256, 64, 0, "normal", False),      # the limits of E and K
    (300, 40, 8, 1, 1, "normal", True),          # capacity 1
    (1, 8, 4, 2, 0, "normal", True),
])
def test_permute_maps_and_rows_are_bit_exact(T, H, E, K, capacity, kind, bf16):
    idx, _ = _idx(300 + T, T, E, K, kind)
    x = make_tokens(301, T, H, bf16=bf16)
    want = oracle.permute(x, idx, E, capacity)
    x_perm, counts, offsets, roa, aor = _gpu_permute(x, idx, E, capacity)
    np.testing.assert_array_equal(counts, want.counts)
    np.testing.assert_array_equal(offsets, want.offsets)
    np.testing.assert_array_equal(roa, want.row_of_assign)
    np.testing.assert_array_equal(aor, want.assign_of_row)
    np.testing.assert_array_equal(x_perm[:want.R], want.x_perm[:want.R])
    assert (x_perm[want.R:] == 0).all(), "rows past the kept total must be left untouched"


def test_permute_maps_only_and_invalid_indices_are_dropped():
    idx, _ = _idx(310, 500, 8, 2)
    idx = idx.copy()
    idx[::7, 0] = 8          # one past the last expert
    idx[3::11, 1] = -1
    idx[100, 0] = 2**30
    want = oracle.permute(None, idx, 8, 0)
    _, counts, offsets, roa, aor = _gpu_permute(None, idx, 8, 0)
    np.testing.assert_array_equal(counts, want.counts)
    np.testing.assert_array_equal(offsets, want.offsets)
    np.testing.assert_array_equal(roa, want.row_of_assign)
    np.testing.assert_array_equal(aor, want.assign_of_row)


def test_all_tokens_to_one_expert_and_empty_experts():
    idx = np.zeros((700, 1), dtype=np.int32) + 5
    x = make_tokens(311, 700, 64, bf16=True)
    want = oracle.permute(x, idx, 8, 0)
    x_perm, counts, offsets, roa, aor = _gpu_permute(x, idx, 8, 0)
    np.testing.assert_array_equal(counts, want.counts)
    np.testing.assert_array_equal(offsets, want.offsets)
    np.testing.assert_array_equal(roa, np.arange(700, dtype=np.int32))
    np.testing.assert_array_equal(x_perm, x)
    assert counts.tolist() == [0, 0, 0, 0, 0, 700, 0, 0]


def _gpu_combine(y_perm, roa, gate, addend, T, K):
    import torch
    import paper_2504_14960_amd as moe
    dy = to_dev(y_perm)
    y = torch.empty((T, y_perm.shape[1]), dtype=dy.dtype, device="cuda")
    moe.unpermute_combine(dy, to_dev(roa), to_dev(gate.astype(np.float32)),
                          None if addend is None else to_dev(addend), y)
    torch.cuda.synchronize()
    return to_host(y)


@pytest.mark.parametrize("T,H,E,K,capacity,bf16,with_addend", [
    (256, 128, 8, 2, 0, False, False),
    (1000, 512, 8, 2, 0, True, False),
    (900, 3584, 64, 8, 0, True, True),
    (2048, 264, 16, 4, 300, True, False),     # drops, 528-byte rows
    (700, 72, 64, 6, 40, True, True),
    (50, 1024, 4, 4, 0, False, True),
])
def test_combine_against_oracle(T, H, E, K, capacity, bf16, with_addend):
    idx, gate = _idx(320 + T, T, E, K, "onehot" if capacity else "normal")
    p = oracle.permute(None, idx, E, capacity)
    r_max = len(p.assign_of_row)
    y_perm = make_tokens(321, max(r_max, 1), H, bf16=bf16)
    addend = make_tokens(322, T, H, bf16=bf16) if with_addend else None
    gate32 = gate.astype(np.float32)
    want = oracle.combine(values(y_perm), p.row_of_assign, gate32.astype(np.float64),
                          None if addend is None else values(addend))
    got = _gpu_combine(y_perm, p.row_of_assign, gate32, addend, T, K)
    assert_close(got, want, bf16, "y")
    if not bf16:
        np.testing.assert_allclose(values(got), want, rtol=0, atol=1e-6 * np.abs(want).max())
    dropped_all = (p.row_of_assign.reshape(T, K) < 0).all(axis=1)
    if dropped_all.any() and addend is None:
        assert (values(got)[dropped_all] == 0).all(), "fully dropped tokens must be exactly zero"


def test_round_trip_with_identity_experts_returns_x():
    # permute then combine with y_perm := x_perm and renormalised gates gives x (K = 1: bit-exact)
    for K in (1, 2):
        T, H, E = 1500, 256, 8
        idx, gate = _idx(330, T, E, K)
        x = make_tokens(331, T, H, bf16=True)
        x_perm, _, _, roa, _ = _gpu_permute(x, idx, E, 0)
        y = _gpu_combine(x_perm, roa, gate.astype(np.float32), None, T, K)
        if K == 1:
            np.testing.assert_array_equal(y, x)
        else:
            assert_close(y, values(x), True, "round trip")


@pytest.mark.parametrize("fused", [0, 1, 2, 3], ids=["three_kernels", "one_launch", "one_token_per_wave", "two_tokens_per_wave"])
@pytest.mark.parametrize("T,H,E,K,capacity,kind,bf16", [
    (8192, 64, 8, 2, 0, "normal", True),          # the benchmark's index array (rows kept small for the oracle)
    (8192, 64, 8, 2, 1800, "onehot", True),       # with drops
    (4099, 24, 8, 3, 0, "normal", True),          # T*K odd: the last assignments are not a group of four
    (333, 6144, 7, 2, 0, "normal", True),         # 12 KiB rows, E not a power of two, ragged last workgroup
    (50, 8192, 8, 1, 0, "normal", True),          # 16 KiB rows: one token per wave whatever is asked
    (700, 100, 3, 3, 200, "normal", False),       # fp32 rows of 400 bytes, K = E, capacity
    (32766, 8, 2, 2, 0, "normal", True),          # 65532 assignments: the largest index array the one launch takes
    (16400, 16, 8, 4, 0, "onehot", True),         # 65600 assignments: always three kernels
    (17, 8, 8, 8, 1, "normal", True),             # capacity 1, every expert on every token
])
def test_one_launch_and_three_kernel_dispatch_agree_with_the_oracle(T, H, E, K, capacity, kind, bf16, fused):
    """Layers with at most 8 experts take a dispatch that is ONE kernel (every workgroup counts the index array
    itself); it must give the oracle's maps bit for bit like the three-kernel form, at every token-per-wave setting."""
    import paper_2504_14960_amd as moe
    idx, _ = _idx(900 + T + K, T, E, K, kind)
    idx = idx.copy()
    idx[5 % T, 0] = E            # an index outside [0, E): a dropped assignment
    x = make_tokens(901, T, H, bf16=bf16)
    want = oracle.permute(x, idx, E, capacity)
    moe.set_option("permute_fused", fused)
    try:
        x_perm, counts, offsets, roa, aor = _gpu_permute(x, idx, E, capacity)
    finally:
        moe.set_option("permute_fused", 1)
    np.testing.assert_array_equal(counts, want.counts)
    np.testing.assert_array_equal(offsets, want.offsets)
    np.testing.assert_array_equal(roa, want.row_of_assign)
    np.testing.assert_array_equal(aor, want.assign_of_row)
    np.testing.assert_array_equal(x_perm[:want.R], want.x_perm[:want.R])
    assert (x_perm[want.R:] == 0).all(), "rows past the kept total must be left untouched"

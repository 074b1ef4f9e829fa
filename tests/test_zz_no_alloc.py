"""moe_permute_noalloc (the entry point for callers that cannot allocate or pass a workspace) against
moe_permute: every output bit for bit, on two calls in a row, the second on a smaller input, so that what the
first call left in the library's own scratch array cannot leak into the second."""
import numpy as np
import pytest

from helpers import to_dev, to_host


def _outputs(T, H, E, K, capacity):
    import torch
    import paper_2504_14960_amd as moe
    r_max = moe.max_rows(T, K, E, capacity)
    i32 = dict(dtype=torch.int32, device="cuda")
    return dict(x_perm=torch.full((r_max, H), 7.0, dtype=torch.bfloat16, device="cuda"),
                counts=torch.full((E,), -3, **i32), offsets=torch.full((E + 1,), -3, **i32),
                roa=torch.full((T * K,), -3, **i32), aor=torch.full((r_max,), -3, **i32))


@pytest.mark.gpu
def test_noalloc_permute_equals_permute_on_two_calls_in_a_row():
    import torch
    import paper_2504_14960_amd as moe
    rng = np.random.default_rng(77)
    # (T, H, E, K, capacity): a large skewed call with drops first, then a much smaller dropless one
    for T, H, E, K, capacity in [(20000, 256, 64, 6, 1500), (700, 128, 16, 2, 0)]:
        print(f"moe_permute_noalloc T={T} H={H} E={E} K={K} capacity={capacity}", flush=True)
        p = 1.0 / np.arange(1, E + 1) ** 1.2
        idx = np.stack([rng.choice(E, size=K, replace=False, p=p / p.sum()) for _ in range(T)]).astype(np.int32)
        x = torch.randn((T, H), dtype=torch.bfloat16, device="cuda")
        d_idx = to_dev(idx)
        a, b = _outputs(T, H, E, K, capacity), _outputs(T, H, E, K, capacity)
        ws = torch.empty(moe.permute_workspace_bytes(T, K, E) + 256, dtype=torch.uint8, device="cuda")
        moe.permute(x, d_idx, E, capacity, a["x_perm"], a["counts"], a["offsets"], a["roa"], a["aor"], ws)
        moe.permute_noalloc(x, d_idx, E, capacity, b["x_perm"], b["counts"], b["offsets"], b["roa"], b["aor"])
        torch.cuda.synchronize()
        for k in a:
            ga, gb = to_host(a[k]), to_host(b[k])
            np.testing.assert_array_equal(gb, ga, err_msg=f"{k} (T={T})")
        assert int(to_host(a["counts"]).sum()) > 0


def test_noalloc_permute_refuses_what_its_scratch_cannot_hold():
    """Host-side check, nothing is launched: ceil(T*K/1024) * E ints must fit into 1 MiB."""
    import paper_2504_14960_amd as moe
    L = moe.lib()
    T, K, E = 1 << 21, 2, 256                      # 4096 chunks x 256 experts x 4 B = 4 MiB
    assert moe.permute_workspace_bytes(T, K, E) > (1 << 20)
    st = L.moe_permute_noalloc(None, None, T, 8, E, K, 0, moe.MOE_BF16, None, None, None, None, None, None)
    assert st == 2 and b"scratch" in L.moe_last_error()

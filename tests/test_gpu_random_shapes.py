"""Seeded sweep over odd shapes for the integer-exact stages (dispatch, its variants, combine and the dispatcher's
backward): many small cases, every one compared with the oracle in full."""
import numpy as np
import pytest

import oracle
from moe_inputs import make_tokens
from helpers import assert_close, to_dev, to_host, values

pytestmark = pytest.mark.gpu


def _shapes(seed, n):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        E = int(rng.choice([1, 2, 3, 5, 8, 16, 37, 64, 100, 256]))
        K = int(rng.integers(1, min(E, 64) + 1)) if rng.random() < 0.5 else int(min(E, rng.choice([1, 2, 4, 8])))
        T = int(rng.choice([1, 2, 7, 63, 64, 65, 255, 511, 1000, 1777, 3000]))
        H = int(rng.choice([8, 16, 24, 72, 128, 136, 520]))
        mode = rng.choice(["dropless", "tight", "loose"])
        avg = max(1, T * K // E)
        cap = 0 if mode == "dropless" else max(1, int(avg * (0.4 if mode == "tight" else 1.7)))
        out.append((T, H, E, K, cap, bool(rng.random() < 0.5)))
    return out


def _routing(rng, T, E, K):
    skew = 1.0 / np.arange(1, E + 1) ** rng.choice([0.0, 0.7, 1.5])
    skew /= skew.sum()
    idx = np.stack([rng.choice(E, size=K, replace=False, p=skew) for _ in range(T)]).astype(np.int32)
    scores = (np.floor(rng.random((T, K)) * 64) / 64).astype(np.float32)      # ties on purpose
    return idx, scores


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_dispatch_combine_and_their_backward_on_random_shapes(seed):
    import torch
    import paper_2504_14960_amd as moe
    rng = np.random.default_rng(100 + seed)
    for case, (T, H, E, K, cap, bf16) in enumerate(_shapes(seed, 14)):
        tag = f"case {case}: T={T} H={H} E={E} K={K} capacity={cap} bf16={bf16}"
        idx, scores = _routing(rng, T, E, K)
        x = make_tokens(1000 * seed + case, T, H, bf16=bf16)
        d_x, d_idx = to_dev(x), to_dev(idx)
        i32 = dict(dtype=torch.int32, device="cuda")
        # ---- plain dispatch
        want = oracle.permute(x, idx, E, cap)
        r_max = moe.max_rows(T, K, E, cap)
        x_perm = torch.zeros((max(r_max, 1), H), dtype=d_x.dtype, device="cuda")
        counts, offsets = torch.empty((E,), **i32), torch.empty((E + 1,), **i32)
        roa, aor = torch.empty((T * K,), **i32), torch.empty((max(r_max, 1),), **i32)
        ws = torch.empty(moe.permute_variant_workspace_bytes(T, K, E) + 64, dtype=torch.uint8, device="cuda")
        moe.permute(d_x, d_idx, E, cap, x_perm[:r_max], counts, offsets, roa, aor[:r_max], ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(to_host(roa), want.row_of_assign, err_msg=tag)
        np.testing.assert_array_equal(to_host(aor)[:r_max], want.assign_of_row[:r_max], err_msg=tag)
        np.testing.assert_array_equal(to_host(offsets), want.offsets, err_msg=tag)
        np.testing.assert_array_equal(to_host(x_perm)[:want.R], want.x_perm[:want.R], err_msg=tag)
        # ---- variants (only with a capacity)
        if cap > 0:
            for by_score, pad in ((True, False), (True, True), (False, True)):
                wv = oracle.permute_variant(x, idx, scores, E, cap, by_score, pad)
                rows = E * cap if pad else r_max
                xp = torch.full((max(rows, 1), H), 2.0, dtype=d_x.dtype, device="cuda")
                aor_v = torch.empty((max(rows, 1),), **i32)
                moe.permute_variant(d_x, d_idx, to_dev(scores), E, cap, by_score, pad, xp[:rows], counts, offsets, roa,
                                    aor_v[:rows], ws)
                torch.cuda.synchronize()
                np.testing.assert_array_equal(to_host(roa), wv.row_of_assign, err_msg=f"{tag} score={by_score} pad={pad}")
                np.testing.assert_array_equal(to_host(aor_v)[:rows], wv.assign_of_row[:rows], err_msg=tag)
                np.testing.assert_array_equal(to_host(counts), wv.counts, err_msg=tag)
                owned = wv.assign_of_row[:rows] >= 0
                np.testing.assert_array_equal(to_host(xp)[:rows][owned], wv.x_perm[:rows][owned], err_msg=tag)
            moe.permute(d_x, d_idx, E, cap, x_perm[:r_max], counts, offsets, roa, aor[:r_max], ws)   # maps of the plain dispatch again
        # ---- combine and the two backward movements on the plain maps
        gate = rng.random((T, K)).astype(np.float32)
        y_perm = make_tokens(2000 * seed + case, max(r_max, 1), H, bf16=bf16)
        d_yp, d_gate = to_dev(y_perm), to_dev(gate)
        y = torch.empty((T, H), dtype=d_x.dtype, device="cuda")
        moe.unpermute_combine(d_yp, roa, d_gate, None, y)
        y_ref = oracle.combine(values(y_perm), want.row_of_assign, gate)
        assert_close(to_host(y), y_ref, bf16, f"y {tag}")
        dy = make_tokens(3000 * seed + case, T, H, bf16=bf16)
        dy_perm = torch.zeros((max(r_max, 1), H), dtype=d_x.dtype, device="cuda")
        dgate = torch.empty((T, K), dtype=torch.float32, device="cuda")
        moe.unpermute_combine_backward(to_dev(dy), d_yp, roa, d_gate, dy_perm, dgate)
        dyp_ref, dgate_ref = oracle.combine_backward(values(dy), values(y_perm), want.row_of_assign, gate)
        torch.cuda.synchronize()
        if want.R:
            assert_close(to_host(dy_perm)[:want.R], dyp_ref[:want.R], bf16, f"dy_perm {tag}")
        tol = 1e-5 * np.sqrt(H) * np.linalg.norm(values(dy), axis=1).max() * max(np.abs(values(y_perm)).max(), 1e-30) + 1e-30
        assert np.abs(dgate.cpu().numpy() - dgate_ref).max() <= tol, tag
        dx = torch.empty((T, H), dtype=d_x.dtype, device="cuda")
        moe.permute_backward(dy_perm, roa, None, dx, K)
        torch.cuda.synchronize()
        dx_ref = oracle.permute_backward(values(to_host(dy_perm)), want.row_of_assign, T, K)
        assert_close(to_host(dx), dx_ref, bf16, f"dx {tag}")

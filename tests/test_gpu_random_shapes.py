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


@pytest.mark.parametrize("seed", [11, 12])
def test_expert_ffn_forward_and_backward_on_random_shapes(seed):
    """Odd layer sizes and ragged counts through the default kernels: sizes that are multiples of 128 take the
    persistent MFMA kernels (forward, forward keeping g | u, backward), the others the guarded fallback (forward)."""
    import torch
    import paper_2504_14960_amd as moe
    from moe_inputs import get_config, make_layer_inputs
    rng = np.random.default_rng(seed)
    for case in range(6):
        H = int(rng.choice([64, 72, 128, 256, 320, 384]))
        F = int(rng.choice([64, 136, 128, 256, 384, 448]))
        E = int(rng.choice([1, 3, 8, 40]))
        counts = [int(c) for c in rng.choice([0, 1, 31, 64, 130, 257, 300], size=E)]
        tag = f"case {case}: H={H} F={F} E={E} counts={counts}"
        cfg = get_config("mixtral8x7b").scaled(T=8, H=H, E=E, K=1, F=F, seed=7000 + 10 * seed + case)
        inp = make_layer_inputs(cfg, ["w_gate", "w_up", "w_down"])
        offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        R = int(offsets[-1])
        if R == 0:
            continue
        x = make_tokens(seed * 100 + case, R, H, bf16=True)
        y_ref, h_ref = oracle.experts(x, offsets, inp["w_gate"], inp["w_up"], inp["w_down"], want_h=True)
        bf = dict(dtype=torch.bfloat16, device="cuda")
        d_x, off = to_dev(x), to_dev(offsets)
        wg, wu, wd = to_dev(inp["w_gate"]), to_dev(inp["w_up"]), to_dev(inp["w_down"])
        h, y = torch.zeros((R, F), **bf), torch.zeros((R, H), **bf)
        moe.grouped_gemm_swiglu(d_x, off, wg, wu, wd, h, y)
        torch.cuda.synchronize()
        assert_close(to_host(h), h_ref, True, f"h {tag}")
        assert_close(to_host(y), y_ref, True, f"y_perm {tag}")
        if H % 128 or F % 128:
            continue
        # training forward + backward at the supported sizes
        gu, h2 = torch.zeros((R, 2 * F), **bf), torch.zeros((R, F), **bf)
        moe.expert_gate_up_saving(d_x, off, wg, wu, h2, gu)
        torch.cuda.synchronize()
        assert torch.equal(h2, h), tag
        dy = make_tokens(seed * 100 + 50 + case, R, H, bf16=True)
        want = oracle.experts_backward(x, offsets, inp["w_gate"], inp["w_up"], inp["w_down"], values(dy))
        wgu_t, wd_t = torch.empty((E, H, 2 * F), **bf), torch.empty((E, F, H), **bf)
        moe.expert_weights_transpose(wg, wu, wd, wgu_t, wd_t)
        dxp = torch.zeros((R, H), **bf)
        dwg, dwu, dwd = torch.empty((E, F, H), **bf), torch.empty((E, F, H), **bf), torch.empty((E, H, F), **bf)
        ws = torch.empty(moe.expert_backward_workspace_bytes(R, H, F, E) + 256, dtype=torch.uint8, device="cuda")
        ws.random_(0, 255)
        moe.grouped_gemm_swiglu_backward(d_x, h, gu, to_dev(dy), off, wg, wu, wgu_t, wd_t, dxp, dwg, dwu, dwd, ws)
        torch.cuda.synchronize()
        for got, ref, what in ((dxp, want[0], "dx_perm"), (dwg, want[1], "dw_gate"), (dwu, want[2], "dw_up"), (dwd, want[3], "dw_down")):
            g, r = values(to_host(got)), np.asarray(ref, dtype=np.float64)
            d = g - r
            assert np.isfinite(g).all(), f"{what} {tag}"
            assert np.abs(d).max() <= 3e-2 * np.abs(r).max() + 1e-30, f"{what} {tag}: max|d| {np.abs(d).max():.3e}"
            assert np.linalg.norm(d) <= 1e-2 * np.linalg.norm(r) + 1e-30, f"{what} {tag}"

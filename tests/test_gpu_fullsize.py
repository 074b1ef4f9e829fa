"""Parity at the benchmark's full layer sizes, through the same stage calls and
launch configuration bench.py times.

Routing, maps, counts and offsets are compared in full (bit-exact).  The expert
FFN and the combine are compared on sampled tokens: for every sampled token the
oracle evaluates each of its kept (token, expert) rows one by one and then the
gate-weighted sum, so every sampled output value is an independent full-size
result.  Properties that hold at any size (row copies, exact zeros for fully
dropped tokens) are checked on everything.
"""
import numpy as np
import pytest

import oracle
from moe_inputs import get_config, make_layer_inputs
from helpers import (LOGIT_ATOL, assert_close, capacity_rows, guard_margins, to_dev, to_host, values)

pytestmark = pytest.mark.gpu

N_SAMPLE_TOKENS = 24


def _run_stages(inp, capacity):
    import torch
    import paper_2504_14960_amd as moe
    cfg = inp.cfg
    T, H, E, K, F, Fs = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F, cfg.shared_F
    d = {k: to_dev(v) for k, v in inp.tensors.items()}
    bias = None if inp.bias is None else to_dev(inp.bias)
    r_max = moe.max_rows(T, K, E, capacity)
    tdt = d["x"].dtype
    i32 = dict(dtype=torch.int32, device="cuda")
    o = dict(
        logits=torch.empty((T, E), dtype=torch.float32, device="cuda"),
        idx=torch.empty((T, K), **i32), gate=torch.empty((T, K), dtype=torch.float32, device="cuda"),
        counts=torch.empty((E,), **i32), offsets=torch.empty((E + 1,), **i32),
        roa=torch.empty((T * K,), **i32), aor=torch.empty((r_max,), **i32),
        x_perm=torch.zeros((r_max, H), dtype=tdt, device="cuda"),
        h=torch.zeros((r_max, F), dtype=tdt, device="cuda"),
        y_perm=torch.zeros((r_max, H), dtype=tdt, device="cuda"),
        y=torch.empty((T, H), dtype=tdt, device="cuda"),
    )
    pws = torch.empty((moe.permute_workspace_bytes(T, K, E) + 256,), dtype=torch.uint8, device="cuda")
    moe.router_topk(d["x"], d["w_router"], bias, o["logits"], K, cfg.renormalize, o["idx"], o["gate"])
    moe.permute(d["x"], o["idx"], E, capacity, o["x_perm"], o["counts"], o["offsets"], o["roa"], o["aor"], pws)
    moe.expert_gate_up(o["x_perm"], o["offsets"], d["w_gate"], d["w_up"], o["h"])
    moe.expert_down(o["h"], o["offsets"], d["w_down"], o["y_perm"])
    addend = None
    if Fs:
        s_off = torch.tensor([0, T], **i32)
        s_h = torch.empty((T, Fs), dtype=tdt, device="cuda")
        o["s_y"] = torch.empty((T, H), dtype=tdt, device="cuda")
        moe.grouped_gemm_swiglu(d["x"], s_off, d["ws_gate"].unsqueeze(0), d["ws_up"].unsqueeze(0),
                                d["ws_down"].unsqueeze(0), s_h, o["s_y"])
        addend = o["s_y"]
    moe.unpermute_combine(o["y_perm"], o["roa"], o["gate"], addend, o["y"])
    torch.cuda.synchronize()
    return o, r_max


@pytest.mark.parametrize("name", ["mixtral8x22b", "mixtral8x7b", "qwen2_57b_a14b", "tokendrop",
                                  "mixtral8x22b_g8t8", "llama3_8x70b"])
def test_full_size_layer(name):
    cfg = get_config(name)
    T, H, E, K, F = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F
    bf16 = cfg.dtype == "bf16"
    inp = make_layer_inputs(cfg)
    redrawn = guard_margins(inp, K)
    capacity = capacity_rows(cfg)
    t = inp.tensors
    print(f"\n[{name}] T={T} H={H} E={E} K={K} F={F} capacity={capacity} redrawn rows={redrawn}", flush=True)

    # ---- oracle: router, selection, permutation in full ----
    l64 = oracle.router_logits(t["x"], t["w_router"], inp.bias)
    want_idx, want_gate = oracle.topk_gates(l64.astype(np.float32), K, cfg.renormalize)
    perm = oracle.permute(None, want_idx, E, capacity)

    o, r_max = _run_stages(inp, capacity)

    logits = to_host(o["logits"])
    assert np.abs(logits - l64).max() <= LOGIT_ATOL
    np.testing.assert_array_equal(to_host(o["idx"]), want_idx)
    np.testing.assert_allclose(to_host(o["gate"]), want_gate, rtol=1e-5, atol=2e-5)
    np.testing.assert_array_equal(to_host(o["counts"]), perm.counts)
    np.testing.assert_array_equal(to_host(o["offsets"]), perm.offsets)
    roa = to_host(o["roa"])
    np.testing.assert_array_equal(roa, perm.row_of_assign)
    np.testing.assert_array_equal(to_host(o["aor"]), perm.assign_of_row)
    R = perm.R
    assert R == int(perm.counts.sum()) and R <= r_max
    if capacity:
        assert (perm.counts <= capacity).all() and (perm.row_of_assign < 0).sum() == T * K - R > 0

    # ---- property at full size: every kept row of x_perm is a byte copy of its token ----
    x_perm = to_host(o["x_perm"])
    np.testing.assert_array_equal(x_perm[:R], t["x"][perm.assign_of_row[:R] // K])
    del x_perm

    # ---- sampled tokens: expert rows one by one, then the weighted sum ----
    rng = np.random.default_rng(cfg.seed)
    kept_any = (perm.row_of_assign.reshape(T, K) >= 0).any(axis=1)
    pool = np.nonzero(kept_any)[0]
    tokens = np.sort(rng.choice(pool, size=min(N_SAMPLE_TOKENS, pool.size), replace=False))
    rows = np.unique(perm.row_of_assign.reshape(T, K)[tokens].reshape(-1))
    rows = rows[rows >= 0]
    y_perm_ref = np.zeros((rows.size, H))
    h_ref = np.zeros((rows.size, F))
    expert_of_row = np.searchsorted(perm.offsets, rows, side="right") - 1
    for e in np.unique(expert_of_row):
        sel = np.nonzero(expert_of_row == e)[0]
        xr = np.ascontiguousarray(t["x"][perm.assign_of_row[rows[sel]] // K])
        ye, he = oracle.expert_ffn_rows(xr, t["w_gate"][e], t["w_up"][e], t["w_down"][e], want_h=True)
        y_perm_ref[sel], h_ref[sel] = ye, he
    import torch
    dev_rows = torch.from_numpy(rows.astype(np.int64)).cuda()
    assert_close(to_host(o["h"][dev_rows]), h_ref, bf16, f"h rows ({name})")
    assert_close(to_host(o["y_perm"][dev_rows]), y_perm_ref, bf16, f"y_perm rows ({name})")

    # compact maps for the sampled tokens, then the oracle's combine
    remap = {int(r): i for i, r in enumerate(rows)}
    roa_s = np.array([[remap[int(r)] if r >= 0 else -1 for r in perm.row_of_assign.reshape(T, K)[tk]] for tk in tokens],
                     dtype=np.int32)
    addend = None
    if cfg.shared_F:
        addend = oracle.expert_ffn_rows(np.ascontiguousarray(t["x"][tokens]), t["ws_gate"], t["ws_up"], t["ws_down"])
        dev_tok = torch.from_numpy(tokens.astype(np.int64)).cuda()
        assert_close(to_host(o["s_y"][dev_tok]), addend, bf16, f"shared expert rows ({name})")
    y_ref = oracle.combine(y_perm_ref, roa_s.reshape(-1), want_gate[tokens], addend)
    dev_tok = torch.from_numpy(tokens.astype(np.int64)).cuda()
    assert_close(to_host(o["y"][dev_tok]), y_ref, bf16, f"y rows ({name})")

    # ---- property at full size: fully dropped tokens are exactly zero ----
    if capacity and not cfg.shared_F and (~kept_any).any():
        y = values(to_host(o["y"]))
        assert (y[~kept_any] == 0).all()
        assert np.isfinite(y).all()

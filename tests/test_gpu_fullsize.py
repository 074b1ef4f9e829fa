"""Parity at the benchmark's full layer sizes, through the same stage calls and
launch configuration bench.py times.

Routing, maps, counts and offsets are compared in full (bit-exact).  The expert
FFN and the combine are compared on samples the oracle evaluates one row at a
time, so every sampled output value is an independent full-size result:
  * h and y_perm on the first and the last valid row of EVERY 256-row M-tile of
    every expert, whole rows (all N-tiles), each row judged on its own: a single
    wrong output tile (m, n) of either GEMM fails, whichever workgroup, round or
    remainder share of the persistent schedule it fell into;
  * h, y_perm and y on the rows of 512 random tokens (all their assignments).
Properties that hold at any size (row copies, exact zeros for fully dropped
tokens) are checked on everything.
"""
import numpy as np
import pytest

import oracle
from moe_inputs import get_config, make_layer_inputs
from helpers import (LOGIT_ATOL, assert_close, capacity_rows, guard_margins, to_dev, to_host, values)

pytestmark = pytest.mark.gpu

N_SAMPLE_TOKENS = 512      # tokens whose layer output is compared (all their kept rows go through the oracle)
N_SAMPLE_TOKENS_FP8 = 48   # the FP8 oracle quantises on one core
M_TILE = 256               # rows per output tile of the grouped GEMM kernels


def tile_edge_rows(offsets, counts):
    """First and last valid row of every M_TILE-row block of every expert's row range."""
    rows = []
    for e, n in enumerate(counts):
        lo = int(offsets[e])
        for m0 in range(0, int(n), M_TILE):
            rows += [lo + m0, lo + min(m0 + M_TILE, int(n)) - 1]
    return np.unique(np.array(rows, dtype=np.int64))


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
    edge_rows = tile_edge_rows(perm.offsets, perm.counts)
    assert edge_rows.size >= int(np.ceil(perm.counts / M_TILE).sum())      # at least one row per tile
    rows = np.union1d(rows[rows >= 0], edge_rows)
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
    got_h, got_yp = to_host(o["h"][dev_rows]), to_host(o["y_perm"][dev_rows])
    assert_close(got_h, h_ref, bf16, f"h rows ({name})")
    assert_close(got_yp, y_perm_ref, bf16, f"y_perm rows ({name})")
    # every tile-edge row on its own, so one wrong tile cannot hide in the norm of the whole sample
    for i in np.nonzero(np.isin(rows, edge_rows))[0]:
        assert_close(got_h[i], h_ref[i], bf16, f"h row {rows[i]} ({name})")
        assert_close(got_yp[i], y_perm_ref[i], bf16, f"y_perm row {rows[i]} ({name})")
    print(f"[{name}] compared {rows.size} rows of h / y_perm ({edge_rows.size} tile-edge rows) and {tokens.size} "
          "tokens of y", flush=True)

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


@pytest.mark.parametrize("name", ["mixtral8x22b", "tokendrop"])
def test_full_size_fp8_expert_ffn(name):
    """The FP8 chain bench.py --precision fp8 times (permute fused with quantisation, the two FP8 grouped GEMMs,
    combine), at full size: maps and the E4M3 codes of every kept row in full, FFN rows and layer outputs on
    sampled tokens against the FP8 oracle."""
    import torch
    import paper_2504_14960_amd as moe
    cfg = get_config(name)
    T, H, E, K, F = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F
    inp = make_layer_inputs(cfg)
    guard_margins(inp, K)
    capacity = capacity_rows(cfg)
    t = inp.tensors
    l64 = oracle.router_logits(t["x"], t["w_router"], inp.bias)
    want_idx, want_gate = oracle.topk_gates(l64.astype(np.float32), K, cfg.renormalize)
    perm = oracle.permute(None, want_idx, E, capacity)
    R = perm.R
    token_of_row = perm.assign_of_row[:R] // K

    # scales as a delayed-scaling run would hold them: from amax values slightly above today's
    sc, wq = {}, {}
    for k in ("w_gate", "w_up", "w_down"):
        sc[k] = oracle.fp8_delayed_scale([oracle.fp8_quantize(t[k], 1.0)[1] * 1.05])
        wq[k] = oracle.fp8_quantize(t[k], sc[k])[0]
    sc["x"] = oracle.fp8_delayed_scale([oracle.fp8_quantize(t["x"], 1.0)[1] * 1.05])
    dq_gate, dq_up = 1.0 / (sc["x"] * sc["w_gate"]), 1.0 / (sc["x"] * sc["w_up"])

    # sampled tokens and their kept rows, grouped by expert for the oracle
    rng = np.random.default_rng(cfg.seed + 1)
    kept_any = (perm.row_of_assign.reshape(T, K) >= 0).any(axis=1)
    pool = np.nonzero(kept_any)[0]
    tokens = np.sort(rng.choice(pool, size=min(N_SAMPLE_TOKENS_FP8, pool.size), replace=False))
    rows = np.unique(perm.row_of_assign.reshape(T, K)[tokens].reshape(-1))
    # plus the first and last row of every 256-row block of every expert (the FP8 kernels' tiles are 256 rows too)
    rows = np.union1d(rows[rows >= 0], tile_edge_rows(perm.offsets, perm.counts))   # ascending = grouped by expert
    expert_of_row = np.searchsorted(perm.offsets, rows, side="right") - 1
    sub_offsets = np.concatenate([[0], np.cumsum(np.bincount(expert_of_row, minlength=E))]).astype(np.int32)
    xq_rows = oracle.fp8_quantize(np.ascontiguousarray(t["x"][token_of_row[rows]]), sc["x"])[0]
    probe = oracle.experts_fp8(xq_rows, sub_offsets, wq["w_gate"], wq["w_up"], wq["w_down"], dq_gate, dq_up, 1.0, 1.0)
    scale_h = oracle.fp8_delayed_scale([probe.amax_h * 1.5])
    dq_down = 1.0 / (scale_h * sc["w_down"])
    ref = oracle.experts_fp8(xq_rows, sub_offsets, wq["w_gate"], wq["w_up"], wq["w_down"], dq_gate, dq_up, scale_h,
                             dq_down)

    # ---- GPU: the stage calls of the FP8 bench ----
    r_max = moe.max_rows(T, K, E, capacity)
    i32 = dict(dtype=torch.int32, device="cuda")
    d_x, d_idx, d_gate = to_dev(t["x"]), to_dev(want_idx), to_dev(want_gate.astype(np.float32))
    counts, offsets = torch.empty((E,), **i32), torch.empty((E + 1,), **i32)
    roa, aor = torch.empty((T * K,), **i32), torch.empty((r_max,), **i32)
    pws = torch.empty((moe.permute_workspace_bytes(T, K, E) + 256,), dtype=torch.uint8, device="cuda")
    xq = torch.zeros((r_max, H), dtype=torch.uint8, device="cuda")
    hq = torch.zeros((r_max, F), dtype=torch.uint8, device="cuda")
    y_perm = torch.zeros((r_max, H), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((T, H), dtype=torch.bfloat16, device="cuda")
    amax = torch.zeros(2, dtype=torch.float32, device="cuda")
    dwq = {k: torch.from_numpy(v).cuda() for k, v in wq.items()}
    moe.permute_fp8(d_x, d_idx, E, capacity, sc["x"], xq, counts, offsets, roa, aor, amax[0:1], pws)
    moe.expert_gate_up_fp8(xq, offsets, dwq["w_gate"], dwq["w_up"], dq_gate, dq_up, scale_h, hq, amax[1:2])
    moe.expert_down_fp8(hq, offsets, dwq["w_down"], dq_down, y_perm)
    moe.unpermute_combine(y_perm, roa, d_gate, None, y)
    torch.cuda.synchronize()

    # maps and every kept row's codes, in full
    np.testing.assert_array_equal(to_host(offsets), perm.offsets)
    np.testing.assert_array_equal(to_host(roa), perm.row_of_assign)
    got_xq = xq.cpu().numpy()
    step = 4096
    for lo in range(0, R, step):                            # in slices: the oracle quantises on one core
        hi = min(R, lo + step)
        want = oracle.fp8_quantize(np.ascontiguousarray(t["x"][token_of_row[lo:hi]]), sc["x"])[0]
        np.testing.assert_array_equal(got_xq[lo:hi], want)
    kept_tokens = np.unique(token_of_row)
    assert float(amax[0].item()) == float(np.abs(values(t["x"][kept_tokens])).max())

    # sampled rows: h codes and y_perm; sampled tokens: y
    dev_rows = torch.from_numpy(rows.astype(np.int64)).cuda()
    got_h = hq[dev_rows].cpu().numpy()
    differ = got_h != ref.hq
    assert differ.mean() <= 3e-3
    gv, rv = oracle.fp8_decode(got_h[differ]), oracle.fp8_decode(ref.hq[differ])
    assert (np.abs(gv - rv) <= np.maximum(np.abs(rv) * 2.0 ** -3, 2.0 ** -9)).all()
    assert float(amax[1].item()) >= ref.amax_h * (1 - 1e-5)  # the sample's maximum is a lower bound of the tensor's
    assert_close(to_host(y_perm[dev_rows]), ref.y, True, f"fp8 y_perm rows ({name})")
    remap = {int(r): i for i, r in enumerate(rows)}
    roa_s = np.array([[remap[int(r)] if r >= 0 else -1 for r in perm.row_of_assign.reshape(T, K)[tk]] for tk in tokens],
                     dtype=np.int32)
    y_ref = oracle.combine(ref.y, roa_s.reshape(-1), want_gate[tokens], None)
    dev_tok = torch.from_numpy(tokens.astype(np.int64)).cuda()
    assert_close(to_host(y[dev_tok]), y_ref, True, f"fp8 y rows ({name})")


@pytest.mark.parametrize("name", ["mixtral8x22b", "mixtral8x22b_g8t8", "llama3_8x70b"])
def test_full_size_ffn_backward(name):
    """The expert FFN's backward at full size, launched as bench.py --ffn-backward does.  dx_perm on sampled rows
    (a row's input gradient depends on that row only); weight gradients on sampled features of sampled experts: the
    gradients of gate/up row f and of down column f depend on the other features only through nothing at all, so a
    layer cut down to a few features, with all rows of the expert, gives exactly those entries."""
    import torch
    import paper_2504_14960_amd as moe
    cfg = get_config(name)
    T, H, E, K, F = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F
    inp = make_layer_inputs(cfg)
    capacity = capacity_rows(cfg)
    t = inp.tensors
    l64 = oracle.router_logits(t["x"], t["w_router"], inp.bias)
    idx, _ = oracle.topk_gates(l64.astype(np.float32), K, cfg.renormalize)
    perm = oracle.permute(None, idx, E, capacity)
    R = perm.R
    r_max = R
    token_of_row = perm.assign_of_row[:R] // K
    x_perm = np.ascontiguousarray(t["x"][token_of_row])
    from moe_inputs import make_tokens
    dy = make_tokens(cfg.seed + 77, R, H, bf16=True)

    bf = dict(dtype=torch.bfloat16, device="cuda")
    d_x, d_dy, off = to_dev(x_perm), to_dev(dy), to_dev(perm.offsets)
    wg, wu, wd = to_dev(t["w_gate"]), to_dev(t["w_up"]), to_dev(t["w_down"])
    h = torch.empty((r_max, F), **bf)
    y = torch.empty((r_max, H), **bf)
    gu = torch.empty((r_max, 2 * F), **bf)
    moe.expert_gate_up_saving(d_x, off, wg, wu, h, gu)       # the forward that keeps g | u for the backward
    del y
    wgu_t, wd_t = torch.empty((E, H, 2 * F), **bf), torch.empty((E, F, H), **bf)
    moe.expert_weights_transpose(wg, wu, wd, wgu_t, wd_t)
    dxp = torch.empty((r_max, H), **bf)
    dwg, dwu, dwd = torch.empty((E, F, H), **bf), torch.empty((E, F, H), **bf), torch.empty((E, H, F), **bf)
    ws = torch.empty(moe.expert_backward_workspace_bytes(r_max, H, F, E) + 256, dtype=torch.uint8, device="cuda")
    moe.grouped_gemm_swiglu_backward(d_x, h, gu, d_dy, off, wg, wu, wgu_t, wd_t, dxp, dwg, dwu, dwd, ws)
    torch.cuda.synchronize()

    def close(got, ref, what):     # the gradient bar of tests/test_gpu_backward.py
        g, r = values(got), np.asarray(ref, dtype=np.float64)
        d = g - r
        assert np.isfinite(g).all(), what
        assert np.abs(d).max() <= 3e-2 * np.abs(r).max() + 1e-30, f"{what}: max|d| {np.abs(d).max():.3e}"
        assert np.linalg.norm(d) / np.linalg.norm(r) <= 1e-2, f"{what}: rel-L2 {np.linalg.norm(d) / np.linalg.norm(r):.3e}"

    rng = np.random.default_rng(cfg.seed + 3)
    # ---- dx_perm on sampled rows, with the full weights ----
    rows = np.sort(rng.choice(R, size=16, replace=False))
    expert_of_row = np.searchsorted(perm.offsets, rows, side="right") - 1
    sub_off = np.concatenate([[0], np.cumsum(np.bincount(expert_of_row, minlength=E))]).astype(np.int32)
    dx_ref = oracle.experts_backward(np.ascontiguousarray(x_perm[rows]), sub_off, t["w_gate"], t["w_up"], t["w_down"],
                                     values(dy[rows]))[0]
    dev_rows = torch.from_numpy(rows.astype(np.int64)).cuda()
    close(to_host(dxp[dev_rows]), dx_ref, f"dx_perm rows ({name})")

    # ---- weight gradients of sampled features of sampled experts, over all rows of the expert ----
    nonempty = np.nonzero(perm.counts > 0)[0]
    for e in rng.choice(nonempty, size=min(2, nonempty.size), replace=False):
        lo, hi = int(perm.offsets[e]), int(perm.offsets[e + 1])
        feats = np.sort(rng.choice(F, size=4, replace=False))
        mini_g = np.ascontiguousarray(t["w_gate"][e][feats])[None]          # [1, 4, H]
        mini_u = np.ascontiguousarray(t["w_up"][e][feats])[None]
        mini_d = np.ascontiguousarray(t["w_down"][e][:, feats])[None]       # [1, H, 4]
        one = np.array([0, hi - lo], dtype=np.int32)
        _, rg, ru, rd = oracle.experts_backward(np.ascontiguousarray(x_perm[lo:hi]), one, mini_g, mini_u, mini_d,
                                                values(dy[lo:hi]))
        f_dev = torch.from_numpy(feats.astype(np.int64)).cuda()
        close(to_host(dwg[e][f_dev]), rg[0], f"dw_gate expert {e} ({name})")
        close(to_host(dwu[e][f_dev]), ru[0], f"dw_up expert {e} ({name})")
        close(to_host(dwd[e][:, f_dev].contiguous()), rd[0], f"dw_down expert {e} ({name})")
    for e in np.nonzero(perm.counts == 0)[0]:
        assert (values(to_host(dwd[int(e)])) == 0).all()


@pytest.mark.parametrize("name", ["tokendrop", "mixtral8x22b_g8t8"])
@pytest.mark.parametrize("by_score,pad", [(True, False), (True, True), (False, True)])
def test_full_size_permute_variants(name, by_score, pad):
    """The dispatch variants at full size, as bench.py --permute-variants launches them: maps, counts and offsets
    in full (bit-exact); the rows of x_perm in full too (a row copy is checked by indexing the source)."""
    import torch
    import paper_2504_14960_amd as moe
    cfg = get_config(name)
    T, H, E, K = cfg.T, cfg.H, cfg.E, cfg.K
    inp = make_layer_inputs(cfg, ["x", "w_router"])
    capacity = capacity_rows(cfg)
    l32 = oracle.router_logits(inp["x"], inp["w_router"], inp.bias).astype(np.float32)
    idx, gate = oracle.topk_gates(l32, K, cfg.renormalize)
    scores = gate.astype(np.float32)
    want = oracle.permute_variant(None, idx, scores, E, capacity, by_score, pad)
    r_max = E * capacity if pad else moe.max_rows(T, K, E, capacity)
    i32 = dict(dtype=torch.int32, device="cuda")
    d_x = to_dev(inp["x"])
    x_perm = torch.full((r_max, H), 5.0, dtype=d_x.dtype, device="cuda")
    counts, offsets = torch.empty((E,), **i32), torch.empty((E + 1,), **i32)
    roa, aor = torch.empty((T * K,), **i32), torch.empty((r_max,), **i32)
    ws = torch.empty(moe.permute_variant_workspace_bytes(T, K, E) + 256, dtype=torch.uint8, device="cuda")
    moe.permute_variant(d_x, to_dev(idx), to_dev(scores), E, capacity, by_score, pad, x_perm, counts, offsets, roa, aor, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(counts), want.counts)
    np.testing.assert_array_equal(to_host(offsets), want.offsets)
    np.testing.assert_array_equal(to_host(roa), want.row_of_assign)
    np.testing.assert_array_equal(to_host(aor), want.assign_of_row[:r_max])
    # every owned row is a copy of its token's row; unowned rows are zero (padded) or untouched (packed)
    d_aor = aor.to(torch.int64)
    owned = d_aor >= 0
    src = d_x[(d_aor.clamp(min=0) // K)]
    assert torch.equal(x_perm[owned].view(torch.int16), src[owned].view(torch.int16))
    rest = x_perm[~owned].float()
    assert rest.numel() == 0 or bool((rest == (0.0 if pad else 5.0)).all())


@pytest.mark.parametrize("S,El,H,mean_rows", [(8, 8, 6144, 1024), (8, 1, 6144, 2048), (64, 4, 4096, 96)])
def test_full_size_chunk_gather(S, El, H, mean_rows):
    """The gather of an expert-parallel share at bench size (8 sources x 8 local experts of the G8T8 shape; one local
    expert; many sources).  The oracle runs the same gather on a 16-byte payload that carries each row's number, which
    gives the source row of every destination row; every destination row must be that source row, whole."""
    import torch
    import paper_2504_14960_amd as moe
    rng = np.random.default_rng(S * 1000 + El)
    rows = rng.poisson(mean_rows, size=S * El).astype(np.int32)
    rows[rng.random(S * El) < 0.1] = 0
    R = int(rows.sum())
    order = np.array([s * El + e for e in range(El) for s in range(S)], dtype=np.int32)
    ids = np.zeros((R, 4), dtype=np.int32)
    ids[:, 0] = np.arange(R)
    want_ids, want_rows, want_goff, total = oracle.sort_chunks(ids, rows, order, group=S)
    assert total == R
    src = torch.randn((R, H), dtype=torch.bfloat16, device="cuda")
    dst = torch.zeros((R + 5, H), dtype=torch.bfloat16, device="cuda")
    rows_out = torch.empty(S * El, dtype=torch.int32, device="cuda")
    goff = torch.empty(El + 1, dtype=torch.int32, device="cuda")
    ws = torch.empty(moe.sort_chunks_workspace_bytes(S * El), dtype=torch.uint8, device="cuda")
    moe.sort_chunks(src, to_dev(rows), to_dev(order), S, dst, rows_out, goff, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(rows_out), want_rows)
    np.testing.assert_array_equal(to_host(goff), want_goff)
    from_row = torch.from_numpy(want_ids[:, 0].astype(np.int64)).cuda()
    assert torch.equal(dst[:R].view(torch.int16), src.view(torch.int16)[from_row])
    assert not dst[R:].any(), "rows past the total must be left untouched"
    # and the way back restores the received layout
    inv = np.array([e * S + s for s in range(S) for e in range(El)], dtype=np.int32)
    back = torch.zeros_like(src)
    moe.sort_chunks(dst, rows_out, to_dev(inv), 0, back, None, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(back.view(torch.int16), src.view(torch.int16))

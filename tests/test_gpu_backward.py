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


def _ffn_backward_case(H, F, E, counts, seed):
    from moe_inputs import get_config, make_layer_inputs
    cfg = get_config("mixtral8x7b").scaled(T=8, H=H, E=E, K=1, F=F, seed=seed)
    inp = make_layer_inputs(cfg, ["w_gate", "w_up", "w_down"])
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offsets[-1])
    x = make_tokens(seed + 1, max(R, 1), H, bf16=True)
    dy = make_tokens(seed + 2, max(R, 1), H, bf16=True)
    want = oracle.experts_backward(x, offsets, inp["w_gate"], inp["w_up"], inp["w_down"], values(dy)[:R])
    return inp, offsets, R, x, dy, want


def _run_ffn_backward(inp, offsets, R, x, dy, r_pad=0, saved=False, variant=0):
    import torch
    import paper_2504_14960_amd as moe
    E, F, H = inp["w_gate"].shape
    r_max = R + r_pad
    bf = dict(dtype=torch.bfloat16, device="cuda")
    dx_in = torch.zeros((r_max, H), **bf)
    dy_in = torch.zeros((r_max, H), **bf)
    dx_in[:R] = to_dev(x)[:R]
    dy_in[:R] = to_dev(dy)[:R]
    wg, wu, wd = to_dev(inp["w_gate"]), to_dev(inp["w_up"]), to_dev(inp["w_down"])
    off = to_dev(offsets)
    h = torch.zeros((r_max, F), **bf)
    y = torch.zeros((r_max, H), **bf)
    gu = None
    if saved:
        # the forward that keeps the pre-activations: h must be the plain forward's bit for bit, gu = (g | u)
        gu = torch.zeros((r_max, 2 * F), **bf)
        h_plain = torch.zeros((r_max, F), **bf)
        moe.expert_gate_up(dx_in, off, wg, wu, h_plain)
        moe.expert_gate_up_saving(dx_in, off, wg, wu, h, gu)
        moe.expert_down(h, off, wd, y)
        torch.cuda.synchronize()
        assert torch.equal(h, h_plain)
        got_gu = to_host(gu)
        assert (values(got_gu)[R:] == 0).all()
        for e in range(E):
            lo, hi = int(offsets[e]), int(offsets[e + 1])
            if hi > lo:     # x W^T is the router's linear map with another weight matrix
                assert_close(got_gu[lo:hi, :F], oracle.router_logits(x[lo:hi], inp["w_gate"][e], None), True, f"g of expert {e}")
                assert_close(got_gu[lo:hi, F:], oracle.router_logits(x[lo:hi], inp["w_up"][e], None), True, f"u of expert {e}")
    else:
        moe.grouped_gemm_swiglu(dx_in, off, wg, wu, wd, h, y)          # the forward leaves h behind
    wgu_t = torch.empty((E, H, 2 * F), **bf)
    wd_t = torch.empty((E, F, H), **bf)
    moe.expert_weights_transpose(wg, wu, wd, wgu_t, wd_t)
    dxp = torch.zeros((r_max, H), **bf)
    dwg, dwu, dwd = torch.full((E, F, H), 7.0, **bf), torch.full((E, F, H), 7.0, **bf), torch.full((E, H, F), 7.0, **bf)
    ws = torch.empty(moe.expert_backward_workspace_bytes(r_max, H, F, E) + 256, dtype=torch.uint8, device="cuda")
    # 31: weight gradients by the one-workgroup-per-tile kernel; -1: straight from the row-major activations
    moe.set_option("gemm_variant", max(variant, 0))
    moe.set_option("wgrad_rowmajor", int(variant == -1))
    try:
        moe.grouped_gemm_swiglu_backward(dx_in, h, gu, dy_in, off, wg, wu, wgu_t, wd_t, dxp, dwg, dwu, dwd, ws)
    finally:
        moe.set_option("gemm_variant", 0)
        moe.set_option("wgrad_rowmajor", 0)
    torch.cuda.synchronize()
    # the transposes are plain copies: check them bit for bit against the host
    np.testing.assert_array_equal(to_host(wd_t), np.ascontiguousarray(inp["w_down"].transpose(0, 2, 1)))
    np.testing.assert_array_equal(to_host(wgu_t)[:, :, :F], np.ascontiguousarray(inp["w_gate"].transpose(0, 2, 1)))
    np.testing.assert_array_equal(to_host(wgu_t)[:, :, F:], np.ascontiguousarray(inp["w_up"].transpose(0, 2, 1)))
    return to_host(dxp), to_host(dwg), to_host(dwu), to_host(dwd)


def _assert_grad_close(got, ref, what):
    """Gradients pass through five bf16 roundings (g, u, dh, dg|du, result) instead of the forward's three:
    max |d| <= 3e-2 max|ref|, relative L2 <= 1e-2."""
    g, r = values(got), np.asarray(ref, dtype=np.float64)
    assert np.isfinite(g).all(), what
    d = g - r
    assert np.abs(d).max() <= 3e-2 * np.abs(r).max() + 1e-30, f"{what}: max|d|={np.abs(d).max():.3e} vs {np.abs(r).max():.3e}"
    nr = np.linalg.norm(r)
    assert nr == 0 or np.linalg.norm(d) / nr <= 1e-2, f"{what}: rel-L2={np.linalg.norm(d) / nr:.3e}"


@pytest.mark.parametrize("H,F,E,counts", [
    (256, 384, 6, [700, 0, 1, 300, 513, 86]),      # ragged tiles, an empty expert, a 1-row expert
    (128, 128, 3, [64, 130, 5]),                   # smallest supported sizes
    (384, 256, 64, None),                          # many small experts
    (640, 384, 2, [1300, 77]),                     # several M- and N-tiles per expert, ragged last tiles
])
@pytest.mark.parametrize("saved,variant", [(False, 0), (True, 0), (True, 31), (True, -1)],
                         ids=["recompute", "saved_gu", "saved_gu_tile_per_workgroup", "saved_gu_rowmajor_wgrad"])
def test_expert_ffn_backward_against_oracle(H, F, E, counts, saved, variant):
    if counts is None:
        counts = np.random.default_rng(12).integers(0, 90, size=E).tolist()
    inp, offsets, R, x, dy, want = _ffn_backward_case(H, F, E, counts, 8000 + H + E)
    dx, dwg, dwu, dwd = _run_ffn_backward(inp, offsets, R, x, dy, r_pad=9, saved=saved, variant=variant)
    assert (values(dx)[R:] == 0).all()                     # rows past the kept ones untouched
    _assert_grad_close(dx[:R], want[0], "dx_perm")
    _assert_grad_close(dwg, want[1], "dw_gate")
    _assert_grad_close(dwu, want[2], "dw_up")
    _assert_grad_close(dwd, want[3], "dw_down")
    for e, n in enumerate(counts):
        if n == 0:                                         # experts without rows: exact zeros
            assert (values(dwg)[e] == 0).all() and (values(dwu)[e] == 0).all() and (values(dwd)[e] == 0).all()


def test_expert_ffn_backward_with_no_rows_gives_zero_weight_gradients():
    inp, offsets, R, x, dy, want = _ffn_backward_case(128, 128, 4, [0, 0, 0, 0], 8100)
    dx, dwg, dwu, dwd = _run_ffn_backward(inp, offsets, R, x, dy, r_pad=16)
    assert (values(dx) == 0).all() and (values(dwg) == 0).all() and (values(dwu) == 0).all() and (values(dwd) == 0).all()


@pytest.mark.parametrize("T,H,E,K,renorm,bf16", [
    (300, 256, 8, 2, True, True), (1000, 136, 16, 4, False, True), (257, 1032, 64, 8, False, True),
    (130, 64, 256, 8, True, True), (200, 64, 8, 2, True, False), (33, 8, 1, 1, True, True),
])
def test_router_backward_against_oracle(T, H, E, K, renorm, bf16):
    import torch
    import paper_2504_14960_amd as moe
    rng = np.random.default_rng(9000 + T)
    x = make_tokens(9001 + T, T, H, bf16=bf16)
    w = make_tokens(9002 + T, E, H, bf16=bf16, std=0.05)
    logits32 = oracle.router_logits(x, w, None).astype(np.float32)
    idx, _ = oracle.topk_gates(logits32, K, renorm)
    dgate = rng.normal(size=(T, K)).astype(np.float32)
    dl, dx, dw, db = oracle.router_backward(x, w, logits32, idx, dgate, renorm)
    d_x, d_w = to_dev(x), to_dev(w)
    g_dl = torch.empty((T, E), dtype=torch.float32, device="cuda")
    g_dx = torch.empty_like(d_x)
    g_dw = torch.empty((E, H), dtype=torch.float32, device="cuda")
    g_db = torch.empty((E,), dtype=torch.float32, device="cuda")
    ws = torch.empty(moe.router_backward_workspace_bytes(T, H, E) + 256, dtype=torch.uint8, device="cuda")
    moe.router_backward(d_x, d_w, to_dev(logits32), to_dev(idx), to_dev(dgate), renorm, g_dl, g_dx, g_dw, g_db, ws)
    torch.cuda.synchronize()
    # fp32 softmax Jacobian against fp64
    np.testing.assert_allclose(g_dl.cpu().numpy(), dl, rtol=2e-4, atol=2e-6 * np.abs(dgate).max())
    assert_close(to_host(g_dx), dx, bf16, "dx (router)")
    # fp32 sums over T tokens of products with bf16/fp32 x
    scale = np.abs(dw).max()
    assert np.abs(g_dw.cpu().numpy() - dw).max() <= 2e-4 * scale + 1e-30
    assert np.abs(g_db.cpu().numpy() - db).max() <= 2e-4 * np.abs(db).max() + 1e-6


@pytest.mark.parametrize("base,kw", [
    ("mixtral8x22b", dict(T=640, H=256, F=384)),
    ("tokendrop", dict(T=1536, H=256, F=256)),
    ("mixtral8x7b", dict(T=300, H=128, F=128, K=1)),
])
def test_backward_of_the_whole_layer_chained_on_the_gpu(base, kw):
    """Forward stage by stage (keeping what the backward needs), then the four backward calls in mirrored order,
    against the oracle's chain (itself pinned against autograd of the whole layer)."""
    import torch
    import paper_2504_14960_amd as moe
    from moe_inputs import get_config, make_layer_inputs
    from helpers import capacity_rows, guard_margins, oracle_layer_backward
    cfg = get_config(base).scaled(**kw)
    inp = make_layer_inputs(cfg)
    guard_margins(inp, cfg.K)
    capacity = capacity_rows(cfg)
    t = inp.tensors
    T, H, E, K, F = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F
    dy = make_tokens(cfg.seed + 5, T, H, bf16=True)
    want = oracle_layer_backward(t["x"], t["w_router"], inp.bias, t["w_gate"], t["w_up"], t["w_down"], K,
                                 cfg.renormalize, capacity, values(dy))

    d = {k: to_dev(v) for k, v in t.items()}
    bias = None if inp.bias is None else to_dev(inp.bias)
    r_max = moe.max_rows(T, K, E, capacity)
    bf, i32, f32 = dict(dtype=torch.bfloat16, device="cuda"), dict(dtype=torch.int32, device="cuda"), dict(dtype=torch.float32, device="cuda")
    logits, idx, gate = torch.empty((T, E), **f32), torch.empty((T, K), **i32), torch.empty((T, K), **f32)
    counts, offsets = torch.empty((E,), **i32), torch.empty((E + 1,), **i32)
    roa, aor = torch.empty((T * K,), **i32), torch.empty((r_max,), **i32)
    pws = torch.empty((moe.permute_workspace_bytes(T, K, E) + 256,), dtype=torch.uint8, device="cuda")
    x_perm, h, y_perm = torch.zeros((r_max, H), **bf), torch.zeros((r_max, F), **bf), torch.zeros((r_max, H), **bf)
    y = torch.empty((T, H), **bf)
    moe.router_topk(d["x"], d["w_router"], bias, logits, K, cfg.renormalize, idx, gate)
    moe.permute(d["x"], idx, E, capacity, x_perm, counts, offsets, roa, aor, pws)
    gu = torch.zeros((r_max, 2 * F), **bf)
    moe.expert_gate_up_saving(x_perm, offsets, d["w_gate"], d["w_up"], h, gu)
    moe.expert_down(h, offsets, d["w_down"], y_perm)
    moe.unpermute_combine(y_perm, roa, gate, None, y)
    np.testing.assert_array_equal(to_host(idx), want["idx"])           # same routing on both sides

    # ---- backward, mirrored ----
    d_dy = to_dev(dy)
    dy_perm, dgate = torch.zeros((r_max, H), **bf), torch.empty((T, K), **f32)
    moe.unpermute_combine_backward(d_dy, y_perm, roa, gate, dy_perm, dgate)
    wgu_t, wd_t = torch.empty((E, H, 2 * F), **bf), torch.empty((E, F, H), **bf)
    moe.expert_weights_transpose(d["w_gate"], d["w_up"], d["w_down"], wgu_t, wd_t)
    dx_perm = torch.zeros((r_max, H), **bf)
    dwg, dwu, dwd = torch.empty((E, F, H), **bf), torch.empty((E, F, H), **bf), torch.empty((E, H, F), **bf)
    ws = torch.empty(moe.expert_backward_workspace_bytes(r_max, H, F, E) + 256, dtype=torch.uint8, device="cuda")
    moe.grouped_gemm_swiglu_backward(x_perm, h, gu, dy_perm, offsets, d["w_gate"], d["w_up"], wgu_t, wd_t, dx_perm, dwg, dwu,
                                     dwd, ws)
    dlogits, dx_r = torch.empty((T, E), **f32), torch.empty((T, H), **bf)
    dwr, dbias = torch.empty((E, H), **f32), torch.empty((E,), **f32)
    rws = torch.empty(moe.router_backward_workspace_bytes(T, H, E) + 256, dtype=torch.uint8, device="cuda")
    moe.router_backward(d["x"], d["w_router"], logits, idx, dgate, cfg.renormalize, dlogits, dx_r, dwr, dbias, rws)
    dx = torch.empty((T, H), **bf)
    moe.permute_backward(dx_perm, roa, dx_r, dx, K)
    torch.cuda.synchronize()

    _assert_grad_close(to_host(dx), want["dx"], "dx")
    _assert_grad_close(to_host(dwg), want["dw_gate"], "dw_gate")
    _assert_grad_close(to_host(dwu), want["dw_up"], "dw_up")
    _assert_grad_close(to_host(dwd), want["dw_down"], "dw_down")
    _assert_grad_close(dwr.cpu().numpy(), want["dw_router"], "dw_router")
    if inp.bias is not None:
        _assert_grad_close(dbias.cpu().numpy(), want["dbias"], "dbias")


@pytest.mark.parametrize("base,kw", [
    ("mixtral8x22b", dict(T=640, H=256, F=384)),
    ("tokendrop", dict(T=1536, H=256, F=256)),
])
def test_layer_training_step_in_two_calls(base, kw):
    """moe_layer_forward_train + moe_layer_backward against the oracle's chain of the four backward steps."""
    import torch
    import paper_2504_14960_amd as moe
    from moe_inputs import get_config, make_layer_inputs
    from helpers import capacity_rows, guard_margins, oracle_layer_backward
    cfg = get_config(base).scaled(**kw)
    inp = make_layer_inputs(cfg)
    guard_margins(inp, cfg.K)
    capacity = capacity_rows(cfg)
    t = inp.tensors
    T, H, E, K, F = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F
    dy = make_tokens(cfg.seed + 5, T, H, bf16=True)
    want = oracle_layer_backward(t["x"], t["w_router"], inp.bias, t["w_gate"], t["w_up"], t["w_down"], K,
                                 cfg.renormalize, capacity, values(dy))
    d = {k: to_dev(v) for k, v in t.items()}
    bias = None if inp.bias is None else to_dev(inp.bias)
    bf, f32 = dict(dtype=torch.bfloat16, device="cuda"), dict(dtype=torch.float32, device="cuda")
    r_max = moe.max_rows(T, K, E, capacity)
    fws = torch.empty(moe.layer_workspace_bytes(T, H, E, K, F, 0, capacity, moe.MOE_BF16), dtype=torch.uint8, device="cuda")
    bws = torch.empty(moe.layer_backward_workspace_bytes(T, H, E, K, F, capacity), dtype=torch.uint8, device="cuda")
    y, gu = torch.empty((T, H), **bf), torch.zeros((r_max, 2 * F), **bf)
    moe.layer_forward_train(d["x"], d["w_router"], bias, d["w_gate"], d["w_up"], d["w_down"], K, cfg.renormalize,
                            capacity, y, gu, fws)
    y_plain = torch.empty((T, H), **bf)
    fws2 = torch.empty_like(fws)
    moe.layer_forward(d["x"], d["w_router"], bias, d["w_gate"], d["w_up"], d["w_down"], None, None, None, K,
                      cfg.renormalize, capacity, y_plain, fws2)
    wgu_t, wd_t = torch.empty((E, H, 2 * F), **bf), torch.empty((E, F, H), **bf)
    moe.expert_weights_transpose(d["w_gate"], d["w_up"], d["w_down"], wgu_t, wd_t)
    dx = torch.empty((T, H), **bf)
    dwr, dbias = torch.empty((E, H), **f32), torch.empty((E,), **f32)
    dwg, dwu, dwd = torch.empty((E, F, H), **bf), torch.empty((E, F, H), **bf), torch.empty((E, H, F), **bf)
    moe.layer_backward(d["x"], d["w_router"], d["w_gate"], d["w_up"], wgu_t, wd_t, to_dev(dy), K, cfg.renormalize,
                       capacity, fws, gu, dx, dwr, dbias, dwg, dwu, dwd, bws)
    torch.cuda.synchronize()
    assert torch.equal(y, y_plain)          # keeping g | u does not change the forward's result
    _assert_grad_close(to_host(dx), want["dx"], "dx")
    _assert_grad_close(to_host(dwg), want["dw_gate"], "dw_gate")
    _assert_grad_close(to_host(dwu), want["dw_up"], "dw_up")
    _assert_grad_close(to_host(dwd), want["dw_down"], "dw_down")
    _assert_grad_close(dwr.cpu().numpy(), want["dw_router"], "dw_router")
    if inp.bias is not None:
        _assert_grad_close(dbias.cpu().numpy(), want["dbias"], "dbias")
    # every sum over tokens has a fixed order: a second backward on a dirtied workspace gives the same bits
    grads = (dx, dwr, dbias, dwg, dwu, dwd)
    first = [g.clone() for g in grads]
    bws.fill_(0x5a)
    for g in grads:
        g.fill_(float("nan"))
    moe.layer_backward(d["x"], d["w_router"], d["w_gate"], d["w_up"], wgu_t, wd_t, to_dev(dy), K, cfg.renormalize,
                       capacity, fws, gu, dx, dwr, dbias, dwg, dwu, dwd, bws)
    torch.cuda.synchronize()
    for name, a, b in zip(("dx", "dw_router", "dbias", "dw_gate", "dw_up", "dw_down"), first, grads):
        bits = torch.int16 if a.dtype == torch.bfloat16 else torch.int32
        assert torch.equal(a.view(bits), b.view(bits)), f"{name} differs between two runs"

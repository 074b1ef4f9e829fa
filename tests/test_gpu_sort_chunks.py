"""Chunk gather on the GPU (one GPU's step of expert-parallel dispatch, Section 3.3) against the oracle, bit for bit,
and a whole expert-parallel group run rank after rank on the one GPU (the All-to-All-V stood in for by device
slicing) against the oracle's one-GPU layer."""
import numpy as np
import pytest

import oracle
from helpers import assert_close, ep_chunk_orders, guard_margins, to_dev, to_host, values
from moe_inputs import get_config, make_layer_inputs, make_tokens

pytestmark = pytest.mark.gpu

SENTINEL = 7.0


def _gpu(src, rows, order, group, r_dst, want_rows=True):
    import torch
    import paper_2504_14960_amd as moe
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    order = np.ascontiguousarray(order, dtype=np.int32)
    d_src = None if src is None else to_dev(src)
    dst = None if src is None else torch.full((r_dst, src.shape[1]), SENTINEL, dtype=d_src.dtype, device="cuda")
    rows_out = torch.full((max(order.size, 1),), -3, dtype=torch.int32, device="cuda") if want_rows else None
    n_groups = (order.size + group - 1) // group + 1 if group > 0 else 0
    goff = torch.full((n_groups,), -3, dtype=torch.int32, device="cuda") if group > 0 else None
    ws = torch.empty(moe.sort_chunks_workspace_bytes(order.size) + 16, dtype=torch.uint8, device="cuda")
    moe.sort_chunks(d_src, to_dev(rows) if rows.size else torch.empty(0, dtype=torch.int32, device="cuda"),
                    to_dev(order) if order.size else torch.empty(0, dtype=torch.int32, device="cuda"),
                    group, dst, rows_out, goff, ws, H=8)
    torch.cuda.synchronize()
    return (None if dst is None else to_host(dst), to_host(rows_out)[:order.size] if want_rows else None,
            None if goff is None else to_host(goff))


def _check(src, rows, order, group, r_dst):
    want_dst, want_rows, want_goff, _ = oracle.sort_chunks(src, rows, order, group=group, r_dst=r_dst)
    # which rows the definition writes: the same gather over a payload of ones leaves the others at zero
    ones = np.ones((src.shape[0], 4), dtype=np.float32)
    written = oracle.sort_chunks(ones, rows, order, r_dst=r_dst)[0][:, 0] == 1.0
    dst, rows_out, goff = _gpu(src, rows, order, group, r_dst)
    np.testing.assert_array_equal(rows_out, want_rows)
    if group > 0:
        np.testing.assert_array_equal(goff, want_goff)
    np.testing.assert_array_equal(dst[written], want_dst[written])
    rest = values(dst[~written])
    assert (rest == SENTINEL).all(), "rows the gather does not own must be left untouched"


@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("n,hi,H,group", [
    (1, 300, 64, 1),
    (6, 70, 8, 2),
    (64, 400, 256, 8),          # 8 sources x 8 local experts
    (257, 30, 3072, 0),         # a row longer than one pass of the copy loop
    (4096, 5, 16, 64),          # the chunk limit
    (512, 0, 16, 8),            # every chunk empty
])
def test_gather_is_bit_exact(n, hi, H, group, bf16):
    rng = np.random.default_rng(1000 + n)
    rows = rng.integers(0, hi + 1, size=n).astype(np.int32)
    rows[rng.random(n) < 0.2] = 0
    src = make_tokens(n, max(int(rows.sum()), 1), H, bf16=bf16)[: int(rows.sum())]
    order = rng.permutation(n).astype(np.int32)
    _check(src, rows, order, group, int(rows.sum()) + 3)


def test_edge_rules():
    src = make_tokens(3, 50, 24, bf16=True)
    # repeats, an index outside the source, a negative index, a negative count
    _check(src, [20, -3, 30], [0, 0, 7, -1, 1, 2], 2, 80)
    # destination shorter than the total; source shorter than its chunk sizes claim
    _check(src, [20, 30], [1, 0], 1, 33)
    _check(src[:25], [20, 30], [1, 0], 1, 50)
    # fewer and more destination chunks than source chunks
    _check(src, [10, 10, 10, 10, 10], [4, 2], 1, 20)
    _check(src, [25, 25], [1, 0, 1, 0, 1], 5, 125)


def test_nothing_to_do_and_outputs_only():
    import torch
    import paper_2504_14960_amd as moe
    src = make_tokens(4, 8, 16, bf16=True)
    dst, rows_out, goff = _gpu(src, [], [], 1, 8)
    assert (values(dst) == SENTINEL).all() and list(goff) == [0]
    # no payload at all: sizes and offsets only
    _, rows_out, goff = _gpu(None, [3, 0, 5], [2, 1, 0], 1, 0)
    assert list(rows_out) == [5, 0, 3] and list(goff) == [0, 5, 5, 8]
    # zero-row destination with a payload
    ws = torch.empty(moe.sort_chunks_workspace_bytes(2) + 16, dtype=torch.uint8, device="cuda")
    moe.sort_chunks(to_dev(src), to_dev(np.array([4, 4], np.int32)), to_dev(np.array([1, 0], np.int32)), 0,
                    to_dev(src)[:0].clone(), None, None, ws)
    torch.cuda.synchronize()


def test_argument_errors():
    import torch
    import paper_2504_14960_amd as moe
    a = torch.zeros((8, 16), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((8, 16), dtype=torch.bfloat16, device="cuda")
    rows = torch.tensor([4, 4], dtype=torch.int32, device="cuda")
    order = torch.tensor([1, 0], dtype=torch.int32, device="cuda")
    ws = torch.empty(moe.sort_chunks_workspace_bytes(2), dtype=torch.uint8, device="cuda")
    goff = torch.zeros(3, dtype=torch.int32, device="cuda")
    with pytest.raises(moe.MoeError, match="overlap"):
        moe.sort_chunks(a, rows, order, 0, a[2:], None, None, ws)
    with pytest.raises(moe.MoeError, match="group"):
        moe.sort_chunks(a, rows, order, 0, b, None, goff, ws)
    with pytest.raises(moe.MoeError, match="workspace"):
        moe.sort_chunks(a, rows, order, 0, b, None, None, ws[:4])
    with pytest.raises(moe.MoeError, match="multiple of 16"):
        moe.sort_chunks(a[:, :4].contiguous(), rows, order, 0, b[:, :4].contiguous(), None, None, ws)
    many = torch.zeros(4097, dtype=torch.int32, device="cuda")
    assert moe.sort_chunks_workspace_bytes(4097) == 0
    with pytest.raises(moe.MoeError, match="limit"):
        moe.sort_chunks(a, many, order, 0, b, None, None, ws)
    torch.cuda.synchronize()


def _ep_group_on_gpu(xs, inp, cfg, capacity):
    """Every rank of the group in turn on the one GPU; the two All-to-All-Vs are slices and concatenations of
    device tensors (plumbing standing in for the collective), everything else runs in the library."""
    import torch
    import paper_2504_14960_amd as moe
    S, E, K, H, F = len(xs), cfg.E, cfg.K, cfg.H, cfg.F
    El = E // S
    dev = {n: to_dev(inp[n]) for n in ("w_router", "w_gate", "w_up", "w_down")}
    bias = None if inp.bias is None else to_dev(inp.bias)
    by_expert, by_source = (to_dev(o) for o in ep_chunk_orders(S, El))
    sent = []
    for x in xs:                                           # a1 + a2 on every rank's own tokens
        T = x.shape[0]
        dx = to_dev(x)
        logits = torch.empty((T, E), dtype=torch.float32, device="cuda")
        idx = torch.empty((T, K), dtype=torch.int32, device="cuda")
        gate = torch.empty((T, K), dtype=torch.float32, device="cuda")
        moe.router_topk(dx, dev["w_router"], bias, logits, K, cfg.renormalize, idx, gate)
        r_max = moe.max_rows(T, K, E, capacity)
        x_perm = torch.zeros((r_max, H), dtype=dx.dtype, device="cuda")
        counts = torch.empty(E, dtype=torch.int32, device="cuda")
        offsets = torch.empty(E + 1, dtype=torch.int32, device="cuda")
        roa = torch.empty(T * K, dtype=torch.int32, device="cuda")
        aor = torch.empty(max(r_max, 1), dtype=torch.int32, device="cuda")
        ws = torch.empty(moe.permute_workspace_bytes(T, K, E), dtype=torch.uint8, device="cuda")
        moe.permute(dx, idx, E, capacity, x_perm, counts, offsets, roa, aor[:r_max], ws)
        sent.append(dict(T=T, gate=gate, roa=roa, x_perm=x_perm, counts=counts, offsets=offsets.cpu().numpy(),
                         y_perm=torch.zeros_like(x_perm), r_max=r_max))
    for d in range(S):                                     # what rank d does with what it receives
        lo, hi = d * El, (d + 1) * El
        recv = torch.cat([p["x_perm"][p["offsets"][lo]:p["offsets"][hi]] for p in sent])
        chunk_rows = torch.cat([p["counts"][lo:hi] for p in sent])
        R = recv.shape[0]
        grouped = torch.zeros((R, H), dtype=recv.dtype, device="cuda")
        rows_by_expert = torch.empty(S * El, dtype=torch.int32, device="cuda")
        goff = torch.empty(El + 1, dtype=torch.int32, device="cuda")
        ws = torch.empty(moe.sort_chunks_workspace_bytes(S * El), dtype=torch.uint8, device="cuda")
        moe.sort_chunks(recv, chunk_rows, by_expert, S, grouped, rows_by_expert, goff, ws)
        h = torch.empty((R, F), dtype=recv.dtype, device="cuda")
        y_rows = torch.zeros((R, H), dtype=recv.dtype, device="cuda")
        moe.grouped_gemm_swiglu(grouped, goff, dev["w_gate"][lo:hi], dev["w_up"][lo:hi], dev["w_down"][lo:hi],
                                h, y_rows)
        back = torch.zeros((R, H), dtype=recv.dtype, device="cuda")
        moe.sort_chunks(y_rows, rows_by_expert, by_source, 0, back, None, None, ws)
        at = 0
        for p in sent:                                     # second All-to-All-V
            n = int(p["offsets"][hi] - p["offsets"][lo])
            p["y_perm"][p["offsets"][lo]:p["offsets"][hi]] = back[at:at + n]
            at += n
    ys = []
    for p in sent:                                         # a4 on every rank
        y = torch.empty((p["T"], H), dtype=p["x_perm"].dtype, device="cuda")
        moe.unpermute_combine(p["y_perm"], p["roa"], p["gate"], None, y)
        ys.append(to_host(y))
    torch.cuda.synchronize()
    return ys


@pytest.mark.parametrize("name,scale,S,capacity", [
    ("tiny", {}, 4, 0),
    ("tiny", {}, 8, 5),
    ("mixtral8x22b_g8t8", dict(T=1500, H=256, F=128, capacity_factor=None), 8, 0),     # 8 sources x 8 local experts
    ("qwen2_57b_a14b", dict(T=900, H=128, F=96, shared_F=0), 2, 0),                    # 2 sources x 32 local experts
])
def test_ep_group_rank_by_rank_equals_the_one_gpu_layer(name, scale, S, capacity):
    cfg = get_config(name).scaled(**scale)
    inp = make_layer_inputs(cfg)
    guard_margins(inp, cfg.K)     # no token whose top-k choice hangs on fp32 summation order
    cuts = np.linspace(0, cfg.T, S + 1).astype(int)
    cuts[1] = max(1, cuts[1] // 3)                         # ragged: one rank holds few tokens
    xs = [inp["x"][cuts[s]:cuts[s + 1]] for s in range(S)]
    ys = _ep_group_on_gpu(xs, inp, cfg, capacity)
    for x, y in zip(xs, ys):
        ref = oracle.layer_forward(x, inp["w_router"], inp.bias, inp["w_gate"], inp["w_up"], inp["w_down"], cfg.K,
                                   cfg.renormalize, capacity)
        assert_close(values(y), ref.y, inp.is_bf16, f"{name} S={S}")

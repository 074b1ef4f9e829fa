"""The layer under HIP graph capture: every entry point only enqueues kernels on
the caller's stream (no allocation, no synchronisation, no memset nodes), so a
captured forward must replay to the eager result every time."""
import numpy as np
import pytest

from moe_inputs import get_config, make_layer_inputs
from helpers import assert_close, capacity_rows, guard_margins, to_dev, to_host
from test_gpu_layer import oracle_layer

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("base,kw", [
    ("mixtral8x22b", dict(T=640, H=256, F=512)),
    ("tokendrop", dict(T=1536, H=256, F=256)),
])
def test_captured_layer_replays_to_the_eager_result(base, kw):
    import torch
    import paper_2504_14960_amd as moe
    cfg = get_config(base).scaled(**kw)
    inp = make_layer_inputs(cfg)
    guard_margins(inp, cfg.K)
    capacity = capacity_rows(cfg)
    want = oracle_layer(inp, capacity)
    d = {k: to_dev(v) for k, v in inp.tensors.items()}
    bias = None if inp.bias is None else to_dev(inp.bias)
    nbytes = moe.layer_workspace_bytes(cfg.T, cfg.H, cfg.E, cfg.K, cfg.F, 0, capacity, moe.MOE_BF16)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    y = torch.zeros_like(d["x"])

    def forward():
        moe.layer_forward(d["x"], d["w_router"], bias, d["w_gate"], d["w_up"], d["w_down"], None, None, None,
                          cfg.K, cfg.renormalize, capacity, y, ws)

    # eager first (also sets the kernels' one-time attributes outside the capture)
    forward()
    torch.cuda.synchronize()
    eager = to_host(y).copy()
    assert_close(eager, want.y, True, "eager y")

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            forward()
    torch.cuda.synchronize()
    scratch = torch.empty(1 << 20, device="cuda")
    for replay in range(4):
        # the program's own eager work between replays: dirty the outputs and the workspace
        y.fill_(float("nan"))
        ws.random_(0, 255)
        scratch.normal_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(to_host(y), eager, err_msg=f"replay {replay}")


def test_captured_forward_and_backward_replay_to_the_eager_result():
    """The training step stage by stage (forward keeping g | u, then the four backward calls) under capture:
    every replay must give the eager gradients bit for bit (fixed summation orders, no atomics on floats)."""
    import torch
    import paper_2504_14960_amd as moe
    from moe_inputs import make_tokens
    cfg = get_config("mixtral8x22b").scaled(T=640, H=256, F=384)
    inp = make_layer_inputs(cfg)
    guard_margins(inp, cfg.K)
    T, H, E, K, F = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F
    d = {k: to_dev(v) for k, v in inp.tensors.items()}
    bias = None if inp.bias is None else to_dev(inp.bias)
    dy = to_dev(make_tokens(77, T, H, bf16=True))
    r_max = moe.max_rows(T, K, E, 0)
    bf, i32, f32 = (dict(dtype=torch.bfloat16, device="cuda"), dict(dtype=torch.int32, device="cuda"),
                    dict(dtype=torch.float32, device="cuda"))
    b = dict(logits=torch.empty((T, E), **f32), idx=torch.empty((T, K), **i32), gate=torch.empty((T, K), **f32),
             counts=torch.empty((E,), **i32), offsets=torch.empty((E + 1,), **i32), roa=torch.empty((T * K,), **i32),
             aor=torch.empty((r_max,), **i32), x_perm=torch.empty((r_max, H), **bf), h=torch.empty((r_max, F), **bf),
             gu=torch.empty((r_max, 2 * F), **bf), y_perm=torch.empty((r_max, H), **bf), y=torch.empty((T, H), **bf),
             dy_perm=torch.empty((r_max, H), **bf), dgate=torch.empty((T, K), **f32),
             wgu_t=torch.empty((E, H, 2 * F), **bf), wd_t=torch.empty((E, F, H), **bf),
             dx_perm=torch.empty((r_max, H), **bf), dwg=torch.empty((E, F, H), **bf), dwu=torch.empty((E, F, H), **bf),
             dwd=torch.empty((E, H, F), **bf), dlogits=torch.empty((T, E), **f32), dx_r=torch.empty((T, H), **bf),
             dwr=torch.empty((E, H), **f32), dbias=torch.empty((E,), **f32), dx=torch.empty((T, H), **bf))
    pws = torch.empty(moe.permute_workspace_bytes(T, K, E) + 256, dtype=torch.uint8, device="cuda")
    ews = torch.empty(moe.expert_backward_workspace_bytes(r_max, H, F, E) + 256, dtype=torch.uint8, device="cuda")
    rws = torch.empty(moe.router_backward_workspace_bytes(T, H, E) + 256, dtype=torch.uint8, device="cuda")
    outs = ("y", "dx", "dwg", "dwu", "dwd", "dwr", "dbias")

    def step():
        moe.router_topk(d["x"], d["w_router"], bias, b["logits"], K, cfg.renormalize, b["idx"], b["gate"])
        moe.permute(d["x"], b["idx"], E, 0, b["x_perm"], b["counts"], b["offsets"], b["roa"], b["aor"], pws)
        moe.expert_gate_up_saving(b["x_perm"], b["offsets"], d["w_gate"], d["w_up"], b["h"], b["gu"])
        moe.expert_down(b["h"], b["offsets"], d["w_down"], b["y_perm"])
        moe.unpermute_combine(b["y_perm"], b["roa"], b["gate"], None, b["y"])
        moe.expert_weights_transpose(d["w_gate"], d["w_up"], d["w_down"], b["wgu_t"], b["wd_t"])
        moe.unpermute_combine_backward(dy, b["y_perm"], b["roa"], b["gate"], b["dy_perm"], b["dgate"])
        moe.grouped_gemm_swiglu_backward(b["x_perm"], b["h"], b["gu"], b["dy_perm"], b["offsets"], d["w_gate"],
                                         d["w_up"], b["wgu_t"], b["wd_t"], b["dx_perm"], b["dwg"], b["dwu"], b["dwd"], ews)
        moe.router_backward(d["x"], d["w_router"], b["logits"], b["idx"], b["dgate"], cfg.renormalize, b["dlogits"],
                            b["dx_r"], b["dwr"], b["dbias"], rws)
        moe.permute_backward(b["dx_perm"], b["roa"], b["dx_r"], b["dx"], K)

    step()
    torch.cuda.synchronize()
    eager = {k: b[k].clone() for k in outs}
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    scratch = torch.empty(1 << 20, device="cuda")
    for replay in range(3):
        for k, t in b.items():          # dirty every intermediate and output
            if t.dtype == torch.int32:
                t.fill_(-7)
            else:
                t.fill_(float("nan"))
        for w in (pws, ews, rws):
            w.random_(0, 255)
        scratch.normal_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(b[k].view(torch.int16 if b[k].dtype == torch.bfloat16 else torch.int32),
                               eager[k].view(torch.int16 if eager[k].dtype == torch.bfloat16 else torch.int32)), \
                f"{k} differs on replay {replay}"

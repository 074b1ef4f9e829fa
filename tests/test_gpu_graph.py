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

"""Edge cases of the C ABI on the GPU: guard bytes around every output stay
untouched, repeated calls are bit-identical, empty inputs are legal."""
import numpy as np
import pytest

import oracle
from moe_inputs import get_config, make_layer_inputs, make_logits, make_tokens
from helpers import to_dev, to_host

pytestmark = pytest.mark.gpu

GUARD = 4096  # bytes of canary on each side of every output buffer


class Guarded:
    """A device buffer of `nbytes` (rounded up to 256) with canaries on both sides."""

    def __init__(self, nbytes, dtype):
        import torch
        self.nbytes = (nbytes + 255) // 256 * 256
        self.raw = torch.full((self.nbytes + 2 * GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
        self.dtype = dtype

    def view(self, *shape):
        import torch
        n = int(np.prod(shape)) * torch.empty((), dtype=self.dtype).element_size()
        return self.raw[GUARD:GUARD + n].view(self.dtype).view(*shape)

    def intact(self):
        return bool((self.raw[:GUARD] == 0xA5).all().item() and (self.raw[GUARD + self.nbytes:] == 0xA5).all().item())


def test_no_stage_writes_outside_its_outputs():
    import torch
    import paper_2504_14960_amd as moe
    cfg = get_config("tokendrop").scaled(T=1111, H=192, F=128, E=16, K=4, capacity_factor=1.25)
    inp = make_layer_inputs(cfg)
    T, H, E, K, F = cfg.T, cfg.H, cfg.E, cfg.K, cfg.F
    cap = moe.capacity_from_factor(cfg.capacity_factor, T, K, E)
    r_max = moe.max_rows(T, K, E, cap)
    d = {k: to_dev(v) for k, v in inp.tensors.items()}
    bf = torch.bfloat16
    g = dict(
        logits=Guarded(T * E * 4, torch.float32), idx=Guarded(T * K * 4, torch.int32),
        gate=Guarded(T * K * 4, torch.float32), counts=Guarded(E * 4, torch.int32),
        offsets=Guarded((E + 1) * 4, torch.int32), roa=Guarded(T * K * 4, torch.int32),
        aor=Guarded(r_max * 4, torch.int32), x_perm=Guarded(r_max * H * 2, bf), h=Guarded(r_max * F * 2, bf),
        y_perm=Guarded(r_max * H * 2, bf), y=Guarded(T * H * 2, bf),
        pws=Guarded(moe.permute_workspace_bytes(T, K, E), torch.uint8),
    )
    logits, idx, gate = g["logits"].view(T, E), g["idx"].view(T, K), g["gate"].view(T, K)
    counts, offsets = g["counts"].view(E), g["offsets"].view(E + 1)
    roa, aor = g["roa"].view(T * K), g["aor"].view(r_max)
    x_perm, h, y_perm, y = g["x_perm"].view(r_max, H), g["h"].view(r_max, F), g["y_perm"].view(r_max, H), g["y"].view(T, H)
    pws = g["pws"].view(moe.permute_workspace_bytes(T, K, E))
    moe.router_topk(d["x"], d["w_router"], to_dev(inp.bias), logits, K, cfg.renormalize, idx, gate)
    moe.permute(d["x"], idx, E, cap, x_perm, counts, offsets, roa, aor, pws)
    moe.grouped_gemm_swiglu(x_perm, offsets, d["w_gate"], d["w_up"], d["w_down"], h, y_perm)
    moe.unpermute_combine(y_perm, roa, gate, None, y)
    torch.cuda.synchronize()
    for name, buf in g.items():
        assert buf.intact(), f"{name}: bytes outside the buffer were written"
    R = int(offsets[E].item())
    assert 0 < R < T * K
    # rows past the kept total are untouched as well
    assert (x_perm[R:].view(torch.int16) == torch.tensor(-23131, dtype=torch.int16)).all()   # 0xA5A5
    assert (y_perm[R:].view(torch.int16) == torch.tensor(-23131, dtype=torch.int16)).all()


def test_twenty_repeats_are_bit_identical():
    import torch
    import paper_2504_14960_amd as moe
    cfg = get_config("qwen2_57b_a14b").scaled(T=700, H=256, F=128, shared_F=256)
    inp = make_layer_inputs(cfg)
    d = {k: to_dev(v) for k, v in inp.tensors.items()}
    dt = moe.MOE_BF16
    nbytes = moe.layer_workspace_bytes(cfg.T, cfg.H, cfg.E, cfg.K, cfg.F, cfg.shared_F, 0, dt)
    ref_y = ref_ws = None
    for i in range(20):
        ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(d["x"])
        moe.layer_forward(d["x"], d["w_router"], None, d["w_gate"], d["w_up"], d["w_down"], d["ws_gate"],
                          d["ws_up"], d["ws_down"], cfg.K, cfg.renormalize, 0, y, ws)
        torch.cuda.synchronize()
        if ref_y is None:
            ref_y, ref_ws = y.clone(), ws.clone()
        else:
            assert torch.equal(y.view(torch.int16), ref_y.view(torch.int16)), f"output differs on repeat {i}"
            assert torch.equal(ws, ref_ws), f"intermediates differ on repeat {i}"


def test_empty_batch_and_single_token():
    import torch
    import paper_2504_14960_amd as moe
    E, K, H, F = 8, 2, 64, 64
    cfg = get_config("mixtral8x7b").scaled(T=1, H=H, F=F)
    inp = make_layer_inputs(cfg)
    d = {k: to_dev(v) for k, v in inp.tensors.items()}
    # T = 0: every entry point returns OK and launches nothing that could fault
    z = torch.empty((0, H), dtype=torch.bfloat16, device="cuda")
    counts = torch.full((E,), 7, dtype=torch.int32, device="cuda")
    offsets = torch.full((E + 1,), 7, dtype=torch.int32, device="cuda")
    dummy_i = torch.zeros((4,), dtype=torch.int32, device="cuda")
    dummy_f = torch.zeros((4,), dtype=torch.float32, device="cuda")
    L = moe.lib()
    assert L.moe_router_topk(None, None, None, None, 0, H, E, K, 1, moe.MOE_BF16, None, None, None) == 0
    assert L.moe_permute(None, None, 0, H, E, K, 0, moe.MOE_BF16, None, counts.data_ptr(), offsets.data_ptr(),
                         None, None, None, 0, None) == 0
    torch.cuda.synchronize()
    assert counts.tolist() == [0] * E and offsets.tolist() == [0] * (E + 1)
    assert L.moe_unpermute_combine(None, None, None, None, 0, H, K, 0, moe.MOE_BF16, None, None) == 0
    assert L.moe_grouped_gemm_swiglu(None, None, 0, H, F, E, None, None, None, moe.MOE_BF16, None, None, None) == 0
    # T = 1 end to end against the oracle
    want = oracle.layer_forward(inp["x"], inp["w_router"], None, inp["w_gate"], inp["w_up"], inp["w_down"],
                                K=K, renormalize=True)
    nbytes = moe.layer_workspace_bytes(1, H, E, K, F, 0, 0, moe.MOE_BF16)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    y = torch.empty((1, H), dtype=torch.bfloat16, device="cuda")
    moe.layer_forward(d["x"], d["w_router"], None, d["w_gate"], d["w_up"], d["w_down"], None, None, None, K, True, 0, y, ws)
    torch.cuda.synchronize()
    from helpers import assert_close
    assert_close(to_host(y), want.y, True, "single token")
    del z, dummy_i, dummy_f

"""The bare-MFMA probe of bench.py's roofline note: it must really multiply what it is given."""
import numpy as np
import pytest

from helpers import to_dev, values
from moe_inputs import make_tokens

pytestmark = pytest.mark.gpu


def test_probe_accumulates_the_products_of_its_operand_image():
    import torch
    import paper_2504_14960_amd as moe
    a = make_tokens(91, 256, 64, True, 1.0)
    b = make_tokens(92, 256, 64, True, 0.5)
    image = to_dev(np.ascontiguousarray(np.concatenate([a, b])))
    iters, nwg = 3, 5
    sink = torch.zeros(nwg * 256, dtype=torch.float32, device="cuda")
    ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
    moe.probe_mfma_bf16(image, iters, nwg, sink, ticks)
    torch.cuda.synchronize()
    # the image is read as the GEMM's LDS tiles are laid out: the 16-byte piece p of row r sits at piece p ^ ((r >> 1) & 7)
    def logical(m):
        v = values(m).reshape(256, 8, 8)
        r = np.arange(256)[:, None]
        return v[r, np.arange(8)[None, :] ^ ((r >> 1) & 7)].reshape(256, 64)
    la, lb = logical(a), logical(b)
    # the four waves cover the 256 x 256 block of dot products once per iteration
    want = iters * float(la.sum(axis=0) @ lb.sum(axis=0))
    scale = iters * float(np.abs(la).sum(axis=0) @ np.abs(lb).sum(axis=0))
    got = sink.cpu().numpy().astype(np.float64).reshape(nwg, 256).sum(axis=1)
    assert np.abs(got - want).max() <= 1e-5 * scale
    tk = ticks.cpu().tolist()
    assert tk[0] > 0 and tk[1] > 0


def test_probe_rejects_bad_arguments():
    import torch
    import paper_2504_14960_amd as moe
    image = torch.zeros(32768, dtype=torch.int16, device="cuda")
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    with pytest.raises(RuntimeError):
        moe.probe_mfma_bf16(image, 0, 1, sink, None)


def test_fp8_probe_accumulates_the_products_of_its_operand_image():
    import torch
    import paper_2504_14960_amd as moe
    rng = np.random.default_rng(93)
    # small integers are exact in E4M3: the expected sum is exact integer arithmetic
    vals = rng.integers(-4, 5, size=(2, 256, 128)).astype(np.float32)
    codes = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    iters, nwg = 2, 3
    sink = torch.zeros(nwg * 256, dtype=torch.float32, device="cuda")
    ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
    moe.probe_mfma_fp8(to_dev(np.ascontiguousarray(codes.reshape(-1))), iters, nwg, sink, ticks)
    torch.cuda.synchronize()

    def logical(m):     # 16-byte piece p of row r sits at piece p ^ ((r >> 1) & 7)
        v = m.reshape(256, 8, 16)
        r = np.arange(256)[:, None]
        return v[r, np.arange(8)[None, :] ^ ((r >> 1) & 7)].reshape(256, 128)
    la, lb = logical(vals[0]).astype(np.float64), logical(vals[1]).astype(np.float64)
    want = iters * float(la.sum(axis=0) @ lb.sum(axis=0))
    got = sink.cpu().numpy().astype(np.float64).reshape(nwg, 256).sum(axis=1)
    np.testing.assert_array_equal(got, np.full(nwg, want))
    assert min(ticks.cpu().tolist()) > 0

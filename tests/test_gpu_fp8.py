"""FP8 (E4M3, delayed scaling) variant of the expert FFN on the GPU against its
oracle: quantisation codes bit-exact, h codes equal up to rounding-boundary
flips, y within the bf16 bar."""
import numpy as np
import pytest

import oracle
from moe_inputs import f32_to_bf16_bits, get_config, make_layer_inputs, make_tokens
from helpers import assert_close, to_dev, to_host, values

pytestmark = pytest.mark.gpu


def _quantize_gpu(src, scale, amax0=0.0):
    import torch
    import paper_2504_14960_amd as moe
    d = to_dev(src)
    dst = torch.zeros(d.numel(), dtype=torch.uint8, device="cuda")
    amax = torch.tensor([amax0], dtype=torch.float32, device="cuda")
    moe.fp8_quantize(d, scale, dst, amax)
    torch.cuda.synchronize()
    return dst.cpu().numpy().reshape(src.shape), float(amax.item())


@pytest.mark.parametrize("n", [1, 15, 16, 17, 4096 + 5, 1 << 20])
@pytest.mark.parametrize("bf16", [True, False])
def test_quantize_codes_and_amax_are_bit_exact(n, bf16):
    rng = np.random.default_rng(n + bf16)
    x = (rng.normal(0, 1, n) * np.exp(rng.normal(0, 3, n))).astype(np.float32)
    special = np.array([0.0, -0.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 15 * 2.0 ** -10, 448, 449, 463.9, 464, 1e30,
                        -1e30, np.inf, -np.inf, 1.0625, 1.1875, -1.0625], dtype=np.float32)
    x[:min(n, special.size)] = special[:min(n, special.size)]
    src = f32_to_bf16_bits(x) if bf16 else x
    for scale in (1.0, 37.3):
        want, want_amax = oracle.fp8_quantize(src, scale, amax_in=0.25)
        got, got_amax = _quantize_gpu(src, scale, amax0=0.25)
        np.testing.assert_array_equal(got, want)
        finite = np.abs(x[np.isfinite(x)]).max() if np.isfinite(x).any() else 0.0
        assert got_amax == want_amax or (not np.isfinite(want_amax) and got_amax >= finite)


def test_quantize_keeps_nan_and_host_scale_matches_oracle():
    import paper_2504_14960_amd as moe
    x = np.array([np.nan, 1.0, -np.nan, 2.0] * 4, dtype=np.float32)
    got, amax = _quantize_gpu(x, 1.0)
    assert (got[0::4] & 0x7F == 0x7F).all() and (got[2::4] & 0x7F == 0x7F).all()
    assert got[1] == 0x38 and got[3] == 0x40 and amax == 2.0
    for hist, margin in (([1.0, 2.0, 0.5], 0), ([1.0, 2.0, 0.5], 1), ([0.0], 0), ([np.inf, 4.0], 0), ([7.0], 2), ([], 0)):
        assert moe.fp8_delayed_scale(hist, margin) == oracle.fp8_delayed_scale(hist, margin)


def _case(H, F, E, counts, seed):
    """bf16 layer tensors, quantised by the oracle with scales as a delayed-scaling run would hold them."""
    cfg = get_config("mixtral8x7b").scaled(T=8, H=H, E=E, K=1, F=F, seed=seed)
    inp = make_layer_inputs(cfg, ["w_gate", "w_up", "w_down"])
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offsets[-1])
    x = make_tokens(seed + 1, max(R, 1), H, bf16=True)
    sc = {}
    q = {}
    for k, a in (("x", x), ("w_gate", inp["w_gate"]), ("w_up", inp["w_up"]), ("w_down", inp["w_down"])):
        _, amax = oracle.fp8_quantize(a, 1.0)
        sc[k] = oracle.fp8_delayed_scale([amax * 1.07])      # an earlier step saw slightly larger values
        q[k], _ = oracle.fp8_quantize(a, sc[k])
    dq_gate, dq_up = 1.0 / (sc["x"] * sc["w_gate"]), 1.0 / (sc["x"] * sc["w_up"])
    probe = oracle.experts_fp8(q["x"], offsets, q["w_gate"], q["w_up"], q["w_down"], dq_gate, dq_up, 1.0, 1.0)
    scale_h = oracle.fp8_delayed_scale([probe.amax_h * 1.2]) if probe.amax_h > 0 else 1.0
    dq_down = 1.0 / (scale_h * sc["w_down"])
    ref = oracle.experts_fp8(q["x"], offsets, q["w_gate"], q["w_up"], q["w_down"], dq_gate, dq_up, scale_h, dq_down,
                             want_h=True)
    return dict(q=q, offsets=offsets, R=R, dq=(dq_gate, dq_up, scale_h, dq_down), ref=ref, H=H, F=F, E=E)


def _run(c, r_pad=0, h_codes=None):
    import torch
    import paper_2504_14960_amd as moe
    q, R = c["q"], c["R"]
    dq_gate, dq_up, scale_h, dq_down = c["dq"]
    xq = torch.zeros((R + r_pad, c["H"]), dtype=torch.uint8, device="cuda")
    xq[:R] = torch.from_numpy(q["x"][:R]).cuda()
    h = torch.zeros((R + r_pad, c["F"]), dtype=torch.uint8, device="cuda")
    y = torch.zeros((R + r_pad, c["H"]), dtype=torch.bfloat16, device="cuda")
    amax = torch.zeros(1, dtype=torch.float32, device="cuda")
    off = to_dev(c["offsets"])
    wg, wu, wd = (torch.from_numpy(q[k]).cuda() for k in ("w_gate", "w_up", "w_down"))
    if h_codes is None:
        moe.grouped_gemm_swiglu_fp8(xq, off, wg, wu, wd, dq_gate, dq_up, scale_h, dq_down, h, amax, y)
    else:
        h[:R] = torch.from_numpy(h_codes).cuda()
        moe.expert_down_fp8(h, off, wd, dq_down, y)
    torch.cuda.synchronize()
    return h.cpu().numpy(), to_host(y), float(amax.item())


def _check_h_codes(got, ref_codes, what):
    """Codes agree except where h sat within rounding noise of a rounding boundary: then they are neighbours."""
    gv, rv = oracle.fp8_decode(got), oracle.fp8_decode(ref_codes)
    differ = got != ref_codes
    frac = differ.mean() if differ.size else 0.0
    assert frac <= 3e-3, f"{what}: {frac:.2e} of the h codes differ"
    step = np.maximum(np.abs(rv) * 2.0 ** -3, 2.0 ** -9)       # never more than one spacing apart
    assert (np.abs(gv - rv)[differ] <= step[differ]).all(), f"{what}: h codes differ by more than one step"


RAGGED = dict(H=256, F=384, E=6, counts=[700, 0, 1, 300, 513, 86])


@pytest.fixture(scope="module")
def ragged_fp8():
    return _case(seed=5000, **RAGGED)


def test_ffn_fp8_on_ragged_experts(ragged_fp8):
    c = ragged_fp8
    h, y, amax = _run(c, r_pad=19)
    R = c["R"]
    _check_h_codes(h[:R], c["ref"].hq, "ragged")
    assert (h[R:] == 0).all() and (y[R:] == 0).all()           # rows past the last expert untouched
    assert abs(amax - c["ref"].amax_h) <= 1e-5 * c["ref"].amax_h
    assert_close(y[:R], c["ref"].y, True, "y_perm (fp8 chain)")


def test_down_fp8_on_the_oracles_h_codes(ragged_fp8):
    c = ragged_fp8
    _, y, _ = _run(c, h_codes=c["ref"].hq)
    # identical operands on both sides: what remains is the bf16 output rounding (half an ulp, 2^-9 relative;
    # 2^-8 allowed) and fp32 accumulation over F terms that partly cancel (absolute, 1e-3 of the largest output)
    ref = np.asarray(c["ref"].y)
    d = np.abs(ref - values(y[:c["R"]]))
    assert (d <= np.abs(ref) * 2.0 ** -8 + 1e-3 * np.abs(ref).max()).all()
    assert np.linalg.norm(d) / np.linalg.norm(ref) <= 2.5e-3


@pytest.mark.parametrize("workgroups", [8, 24, 13])
def test_ffn_fp8_with_many_tiles_per_workgroup(ragged_fp8, workgroups):
    import paper_2504_14960_amd as moe
    c = ragged_fp8
    moe.set_option("gemm_workgroups", workgroups)
    try:
        h, y, amax = _run(c)
    finally:
        moe.set_option("gemm_workgroups", 0)
    _check_h_codes(h, c["ref"].hq, f"{workgroups} workgroups")
    assert_close(y, c["ref"].y, True, f"y_perm ({workgroups} workgroups)")


def test_ffn_fp8_deep_contraction_and_many_small_experts():
    c = _case(H=1536, F=256, E=3, counts=[130, 257, 40], seed=5100)
    h, y, _ = _run(c)
    _check_h_codes(h, c["ref"].hq, "deep")
    assert_close(y, c["ref"].y, True, "y deep")
    counts = np.random.default_rng(11).integers(0, 90, size=64).tolist()
    c = _case(H=256, F=256, E=64, counts=counts, seed=5200)
    h, y, _ = _run(c)
    _check_h_codes(h, c["ref"].hq, "fine-grained")
    assert_close(y, c["ref"].y, True, "y fine-grained")


def test_ffn_fp8_is_reproducible_and_handles_empty_input():
    import torch
    import paper_2504_14960_amd as moe
    c = _case(H=256, F=256, E=4, counts=[100, 50, 0, 270], seed=5300)
    h1, y1, a1 = _run(c)
    h2, y2, a2 = _run(c)
    np.testing.assert_array_equal(h1, h2)
    np.testing.assert_array_equal(y1, y2)
    assert a1 == a2
    e = _case(H=256, F=256, E=4, counts=[0, 0, 0, 0], seed=5400)
    h, y, amax = _run(e, r_pad=16)
    assert (h == 0).all() and (y == 0).all() and amax == 0.0
    # shapes outside the FP8 kernel's reach are refused on the host, nothing is enqueued
    z = torch.zeros((8, 192), dtype=torch.uint8, device="cuda")
    w = torch.zeros((2, 256, 192), dtype=torch.uint8, device="cuda")
    wd = torch.zeros((2, 192, 256), dtype=torch.uint8, device="cuda")
    off = torch.tensor([0, 4, 8], dtype=torch.int32, device="cuda")
    with pytest.raises(moe.MoeError):
        moe.grouped_gemm_swiglu_fp8(z, off, w, w, wd, 1.0, 1.0, 1.0, 1.0, torch.zeros((8, 256), dtype=torch.uint8, device="cuda"),
                                    None, torch.zeros((8, 192), dtype=torch.bfloat16, device="cuda"))


# fused: the "permute_fused" option (0 = the maps from the three-kernel path, 1 = default dispatch, 2 / 3 = the maps from
# the one-launch kernel with one / two tokens per wave); the quantising copy follows in either case.  Shapes with at
# most 8 experts take the one-launch kernel: rows of 272 bytes up to 16 KiB, drops that leave whole tokens without a row
@pytest.mark.parametrize("fused", [0, 1, 2, 3])
@pytest.mark.parametrize("T,H,E,K,capacity", [(300, 256, 8, 2, 0), (1000, 136, 16, 4, 150), (257, 1032, 64, 8, 0),
                                              (64, 64, 4, 1, 3), (700, 6144, 8, 2, 0), (513, 4096, 8, 2, 40),
                                              (130, 8192, 8, 2, 0), (1000, 136, 8, 4, 150)])
def test_permute_fp8_writes_the_codes_of_the_permuted_rows(T, H, E, K, capacity, fused):
    import torch
    import paper_2504_14960_amd as moe
    if fused and E > 8:
        pytest.skip("more than 8 experts: the dispatch is the three-kernel path whatever the option says")
    rng = np.random.default_rng(T + H)
    x = make_tokens(6000 + T, T, H, bf16=True)
    idx = np.stack([rng.permutation(E)[:K] for _ in range(T)]).astype(np.int32)
    perm = oracle.permute(x, idx, E, capacity)
    R = perm.R
    scale = 23.7
    want_codes, want_amax = oracle.fp8_quantize(perm.x_perm[:R], scale)
    r_max = moe.max_rows(T, K, E, capacity)
    i32 = dict(dtype=torch.int32, device="cuda")
    xq = torch.full((r_max + 3, H), 0xAA, dtype=torch.uint8, device="cuda")
    counts, offsets = torch.empty((E,), **i32), torch.empty((E + 1,), **i32)
    roa, aor = torch.empty((T * K,), **i32), torch.empty((r_max,), **i32)
    ws = torch.empty((moe.permute_workspace_bytes(T, K, E) + 256,), dtype=torch.uint8, device="cuda")
    amax = torch.zeros(1, dtype=torch.float32, device="cuda")
    moe.set_option("permute_fused", fused)
    try:
        moe.permute_fp8(to_dev(x), to_dev(idx), E, capacity, scale, xq[:r_max], counts, offsets, roa, aor, amax, ws)
        torch.cuda.synchronize()
    finally:
        moe.set_option("permute_fused", 1)
    np.testing.assert_array_equal(counts.cpu().numpy(), perm.counts)
    np.testing.assert_array_equal(offsets.cpu().numpy(), perm.offsets)
    np.testing.assert_array_equal(roa.cpu().numpy(), perm.row_of_assign)
    np.testing.assert_array_equal(aor.cpu().numpy(), perm.assign_of_row)
    got = xq.cpu().numpy()
    np.testing.assert_array_equal(got[:R], want_codes)
    assert (got[R:] == 0xAA).all()          # rows past the kept ones are untouched
    assert float(amax.item()) == want_amax

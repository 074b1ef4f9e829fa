"""a3 on the GPU against the oracle: grouped SwiGLU expert FFN over ragged rows."""
import numpy as np
import pytest

import oracle
from moe_inputs import get_config, make_layer_inputs, make_tokens
from helpers import assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu

ALL_VARIANTS = [0, 30, 31, 40, 41, 42, 43, 99]


def _offsets(counts):
    return np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)


def _run(x_perm, offsets, inp, variant, r_max=None):
    import torch
    import paper_2504_14960_amd as moe
    R = int(offsets[-1])
    r_max = R if r_max is None else r_max
    E, F, H = inp["w_gate"].shape
    dx = to_dev(x_perm)
    h = torch.zeros((r_max, F), dtype=dx.dtype, device="cuda")
    y = torch.zeros((r_max, H), dtype=dx.dtype, device="cuda")
    moe.set_option("gemm_variant", variant)
    try:
        moe.grouped_gemm_swiglu(dx, to_dev(offsets), to_dev(inp["w_gate"]), to_dev(inp["w_up"]),
                                to_dev(inp["w_down"]), h, y)
        torch.cuda.synchronize()
    finally:
        moe.set_option("gemm_variant", 0)
    return to_host(h), to_host(y)


def _case(H, F, E, counts, bf16=True, seed=4000, r_pad=0):
    cfg = get_config("mixtral8x7b").scaled(T=8, H=H, E=E, K=1, F=F, seed=seed, dtype="bf16" if bf16 else "f32")
    inp = make_layer_inputs(cfg, ["w_gate", "w_up", "w_down"])
    offsets = _offsets(counts)
    R = int(offsets[-1])
    x_perm = make_tokens(seed + 1, R + r_pad, H, bf16=bf16)
    y_ref, h_ref = oracle.experts(x_perm, offsets, inp["w_gate"], inp["w_up"], inp["w_down"], want_h=True)
    return inp, x_perm, offsets, h_ref, y_ref


@pytest.fixture(scope="module")
def ragged_case():
    # spans several 256-row tiles, ragged tails, an empty expert, a 1-row expert
    return _case(H=256, F=384, E=6, counts=[700, 0, 1, 300, 513, 86])


@pytest.mark.parametrize("variant", ALL_VARIANTS)
def test_every_kernel_variant_on_ragged_experts(ragged_case, variant):
    inp, x_perm, offsets, h_ref, y_ref = ragged_case
    h, y = _run(x_perm, offsets, inp, variant)
    assert_close(h, h_ref, True, f"h (variant {variant})")
    assert_close(y, y_ref, True, f"y_perm (variant {variant})")


@pytest.mark.parametrize("variant", [0, 30, 31, 40, 41, 42, 43])
def test_deep_contraction_and_fine_grained_experts(variant):
    # long K loops (many k-tiles) and many small experts
    inp, x_perm, offsets, h_ref, y_ref = _case(H=1536, F=128, E=3, counts=[130, 257, 40], seed=4100)
    h, y = _run(x_perm, offsets, inp, variant)
    assert_close(h, h_ref, True, "h deep")
    assert_close(y, y_ref, True, "y deep")
    rng = np.random.default_rng(7)
    counts = rng.integers(0, 90, size=64).tolist()
    inp, x_perm, offsets, h_ref, y_ref = _case(H=128, F=192, E=64, counts=counts, seed=4200)
    h, y = _run(x_perm, offsets, inp, variant)
    assert_close(h, h_ref, True, "h fine-grained")
    assert_close(y, y_ref, True, "y fine-grained")


@pytest.mark.parametrize("variant", [0, 30, 31, 40, 41, 42, 43])
def test_experts_with_more_m_tiles_than_one_scheduler_group(variant):
    # 2400 rows = 10 (or 19) M-tiles: the scheduler cuts them into balanced groups
    inp, x_perm, offsets, h_ref, y_ref = _case(H=128, F=128, E=3, counts=[2400, 130, 4500], seed=4150)
    h, y = _run(x_perm, offsets, inp, variant)
    assert_close(h, h_ref, True, "h many tiles")
    assert_close(y, y_ref, True, "y many tiles")


@pytest.mark.parametrize("variant", [40, 41, 42, 43])
@pytest.mark.parametrize("workgroups", [8, 24, 13, 64])
def test_persistent_kernel_walks_many_tiles_per_workgroup(ragged_case, variant, workgroups):
    # few workgroups => each one streams through several tiles (tile boundaries,
    # ragged tails and the end of its list all inside one kernel instance)
    import paper_2504_14960_amd as moe
    inp, x_perm, offsets, h_ref, y_ref = ragged_case
    moe.set_option("gemm_workgroups", workgroups)
    try:
        h, y = _run(x_perm, offsets, inp, variant)
    finally:
        moe.set_option("gemm_workgroups", 0)
    assert_close(h, h_ref, True, f"h (variant {variant}, {workgroups} workgroups)")
    assert_close(y, y_ref, True, f"y_perm (variant {variant}, {workgroups} workgroups)")


@pytest.mark.parametrize("variant", [40, 41, 42, 43])
@pytest.mark.parametrize("idle_skip", [0, 1])
def test_waves_without_valid_rows_may_skip_their_multiplications(variant, idle_skip):
    # experts whose last tile holds at most 128 rows (half of the waves idle), exactly 128, one row, and full tiles
    import paper_2504_14960_amd as moe
    inp, x_perm, offsets, h_ref, y_ref = _case(H=256, F=384, E=7, counts=[300, 128, 1, 513, 0, 256, 90], seed=4500)
    moe.set_option("gemm_idle_skip", idle_skip)
    try:
        h, y = _run(x_perm, offsets, inp, variant)
    finally:
        moe.set_option("gemm_idle_skip", -1)
    assert_close(h, h_ref, True, f"h (variant {variant}, idle_skip {idle_skip})")
    assert_close(y, y_ref, True, f"y_perm (variant {variant}, idle_skip {idle_skip})")


def test_rows_past_the_last_expert_are_untouched_and_result_is_reproducible():
    inp, x_perm, offsets, h_ref, y_ref = _case(H=128, F=256, E=4, counts=[100, 50, 0, 270], seed=4300, r_pad=37)
    R = int(offsets[-1])
    h1, y1 = _run(x_perm, offsets, inp, 0, r_max=R + 37)
    h2, y2 = _run(x_perm, offsets, inp, 0, r_max=R + 37)
    assert (y1[R:] == 0).all() and (h1[R:] == 0).all()
    np.testing.assert_array_equal(y1, y2)
    np.testing.assert_array_equal(h1, h2)
    assert_close(y1[:R], y_ref, True, "y_perm")


def test_shapes_outside_the_mfma_fast_path_use_the_plain_kernel():
    inp, x_perm, offsets, h_ref, y_ref = _case(H=72, F=40, E=3, counts=[65, 3, 130], seed=4400)
    h, y = _run(x_perm, offsets, inp, 0)
    assert_close(h, h_ref, True, "h odd shape")
    assert_close(y, y_ref, True, "y odd shape")


def test_fp32_experts():
    inp, x_perm, offsets, h_ref, y_ref = _case(H=128, F=256, E=8, counts=[64, 70, 1, 0, 129, 33, 90, 125],
                                               bf16=False, seed=4500)
    h, y = _run(x_perm, offsets, inp, 0)
    assert_close(h, h_ref, False, "h fp32")
    assert_close(y, y_ref, False, "y fp32")


def test_all_experts_empty_is_a_no_op():
    inp, x_perm, offsets, h_ref, y_ref = _case(H=128, F=128, E=4, counts=[0, 0, 0, 0], seed=4600, r_pad=16)
    h, y = _run(x_perm, offsets, inp, 0, r_max=16)
    assert (y == 0).all() and (h == 0).all()


def test_clock_sample_reports_a_plausible_shader_clock_and_leaves_the_results_alone(ragged_case):
    """moe_gemm_clock_sample: workgroup 0 of a persistent GEMM launch writes its shader-clock and 100 MHz ticks."""
    import torch
    import paper_2504_14960_amd as moe
    inp, x_perm, offsets, h_ref, y_ref = ragged_case
    E, F, H = inp["w_gate"].shape
    dx, doff = to_dev(x_perm), to_dev(offsets)
    wg, wu, wd = to_dev(inp["w_gate"]), to_dev(inp["w_up"]), to_dev(inp["w_down"])
    h = torch.zeros((x_perm.shape[0], F), dtype=dx.dtype, device="cuda")
    y = torch.zeros((x_perm.shape[0], H), dtype=dx.dtype, device="cuda")
    ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
    moe.gemm_clock_sample(ticks)
    try:
        moe.expert_gate_up(dx, doff, wg, wu, h)
        torch.cuda.synchronize()
        t_gu = ticks.cpu().tolist()
        moe.expert_down(h, doff, wd, y)
        torch.cuda.synchronize()
        t_dn = ticks.cpu().tolist()
    finally:
        moe.gemm_clock_sample(None)
    for tk in (t_gu, t_dn):
        assert tk[0] > 0 and tk[1] > 0
        mhz = 100.0 * tk[0] / tk[1]
        assert 100.0 < mhz < 3000.0, mhz          # the part's clock range, generously
    assert t_gu != t_dn                            # the second launch wrote its own sample
    # sampling off again: the cells keep their last values, and the results are the oracle's either way
    ticks.zero_()
    moe.expert_gate_up(dx, doff, wg, wu, h)
    moe.expert_down(h, doff, wd, y)
    torch.cuda.synchronize()
    assert ticks.cpu().tolist() == [0, 0]
    assert_close(to_host(h), h_ref, True, "h after sampling")
    assert_close(to_host(y), y_ref, True, "y_perm after sampling")

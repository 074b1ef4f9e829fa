"""Pins for the FP8 (E4M3, delayed scaling) oracle, oracle/moe_oracle_fp8.c.

Each test checks the oracle against something other than itself: a library's
E4M3 table and cast, hand-worked values of the format, exact integer
arithmetic, and the bf16/fp64 expert oracle on the dequantised operands.
"""
import numpy as np
import pytest
import torch

import oracle
from moe_inputs import bf16_bits_to_f32, f32_to_bf16_bits

ALL_CODES = np.arange(256, dtype=np.uint8)


def _lib_decode(codes):
    return torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def test_decode_matches_library_table_for_all_256_codes():
    got = oracle.fp8_decode(ALL_CODES)
    want = _lib_decode(ALL_CODES)
    nan = np.isnan(want)
    assert nan.sum() == 2 and np.isnan(got[nan]).all()
    np.testing.assert_array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_decode_hand_worked_values_of_the_format():
    d = lambda c: float(oracle.fp8_decode(np.array([c], dtype=np.uint8))[0])
    assert d(0x7E) == 448.0                 # largest finite: 1.75 * 2^8
    assert d(0x38) == 1.0                   # exponent field 7 = bias
    assert d(0x08) == 2.0 ** -6             # smallest normal
    assert d(0x01) == 2.0 ** -9             # smallest subnormal
    assert d(0x07) == 7 * 2.0 ** -9
    assert d(0xC0) == -2.0


def test_encode_inverts_decode_on_every_finite_code():
    finite = ALL_CODES[(ALL_CODES & 0x7F) != 0x7F]
    vals = oracle.fp8_decode(finite).astype(np.float32)
    np.testing.assert_array_equal(oracle.fp8_encode(vals), finite)


def test_encode_matches_library_cast_in_range():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 100, 20000), rng.uniform(-2.0 ** -6, 2.0 ** -6, 5000),
                        rng.uniform(-448, 448, 5000)]).astype(np.float32)
    x = x[np.abs(x) <= 448]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = oracle.fp8_encode(x)
    # the library may encode a result of zero without the sign; values must agree exactly
    np.testing.assert_array_equal(oracle.fp8_decode(got), _lib_decode(want))


def test_encode_ties_go_to_the_even_mantissa():
    e = lambda v: int(oracle.fp8_encode(np.array([v], dtype=np.float32))[0])
    assert e(1.0625) == 0x38        # halfway 1.0 (mantissa 000) / 1.125 (001) -> 000
    assert e(1.1875) == 0x3A        # halfway 1.125 (001) / 1.25 (010) -> 010
    assert e(2.0 ** -10) == 0x00    # halfway 0 / 2^-9 -> 0
    assert e(3 * 2.0 ** -10) == 0x02  # halfway 1 / 2 subnormal steps -> 2
    assert e(15 * 2.0 ** -10) == 0x08  # halfway 7 * 2^-9 / 2^-6 -> the normal 2^-6 (even)
    assert e(-1.0625) == 0xB8


def test_encode_saturates_and_keeps_nan():
    e = lambda v: int(oracle.fp8_encode(np.array([v], dtype=np.float32))[0])
    assert e(448.0) == 0x7E and e(449.0) == 0x7E and e(464.0) == 0x7E and e(1e30) == 0x7E
    assert e(np.inf) == 0x7E and e(-np.inf) == 0xFE
    assert e(np.nan) & 0x7F == 0x7F
    assert e(447.0) == 0x7E and e(431.9) == 0x7D   # 416 | 432 (midpoint) | 448


def test_encode_is_monotone():
    x = np.sort(np.random.default_rng(6).normal(0, 50, 50000).astype(np.float32))
    v = oracle.fp8_decode(oracle.fp8_encode(x))
    assert (np.diff(v) >= 0).all()
    # and never further away than half a step of the local spacing
    assert np.all(np.abs(v - np.clip(x, -448, 448)) <= np.maximum(np.abs(x) * 2.0 ** -4, 2.0 ** -10))


def test_quantize_applies_scale_in_fp32_and_reports_amax():
    rng = np.random.default_rng(7)
    x32 = rng.normal(0, 3, 4096).astype(np.float32)
    xb = f32_to_bf16_bits(x32)
    scale = np.float32(37.3)
    codes, amax = oracle.fp8_quantize(xb, float(scale), amax_in=0.5)
    xv = bf16_bits_to_f32(xb)
    want = torch.from_numpy(np.clip(xv * scale, -448, 448).astype(np.float32)).to(torch.float8_e4m3fn)
    np.testing.assert_array_equal(oracle.fp8_decode(codes), want.to(torch.float64).numpy())
    assert amax == max(0.5, float(np.abs(xv).max()))
    _, amax2 = oracle.fp8_quantize(xb, 1.0, amax_in=1e9)
    assert amax2 == np.float32(1e9)


def test_delayed_scale_closed_forms():
    assert oracle.fp8_delayed_scale([1.0, 2.0, 0.5]) == 224.0            # 448 / max
    assert oracle.fp8_delayed_scale([1.0, 2.0, 0.5], margin=1) == 112.0  # 448 / (max * 2)
    assert oracle.fp8_delayed_scale([0.0, 0.0]) == 1.0                   # nothing seen yet
    assert oracle.fp8_delayed_scale([np.inf, 4.0]) == 112.0              # non-finite entries ignored
    assert oracle.fp8_delayed_scale([7.0]) == np.float32(448.0 / 7.0)


def _small_int_case(seed=8, E=3, H=16, F=8, counts=(5, 0, 7)):
    rng = np.random.default_rng(seed)
    R = sum(counts)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    enc = lambda a: oracle.fp8_encode(a.astype(np.float32))
    x = rng.integers(-3, 4, size=(R, H))
    wg = rng.integers(-2, 3, size=(E, F, H))
    wu = rng.integers(-2, 3, size=(E, F, H))
    wd = rng.integers(-2, 3, size=(E, H, F))
    return offsets, x, wg, wu, wd, enc


def test_experts_fp8_with_small_integers_is_exact_integer_arithmetic():
    offsets, x, wg, wu, wd, enc = _small_int_case()
    res = oracle.experts_fp8(enc(x), offsets, enc(wg), enc(wu), enc(wd), 1.0, 1.0, 1.0, 1.0, want_h=True)
    for e in range(3):
        lo, hi = offsets[e], offsets[e + 1]
        g = (x[lo:hi] @ wg[e].T).astype(np.float64)
        u = (x[lo:hi] @ wu[e].T).astype(np.float64)
        h = g / (1.0 + np.exp(-g)) * u
        np.testing.assert_allclose(res.h_val[lo:hi], h, rtol=1e-14, atol=0)
        hq_val = oracle.fp8_decode(res.hq[lo:hi])
        # h is quantised with scale 1: every value is the nearest E4M3 number (saturating)
        want_q = torch.from_numpy(np.clip(h, -448, 448).astype(np.float32)).to(torch.float8_e4m3fn).to(torch.float64).numpy()
        np.testing.assert_array_equal(hq_val, want_q)
        np.testing.assert_allclose(res.y[lo:hi], hq_val @ wd[e].T.astype(np.float64), rtol=1e-14, atol=1e-12)
    assert res.amax_h == np.abs(res.h_val).max()


def test_experts_fp8_h_equals_the_bf16_oracle_on_dequantised_operands_and_scales_divide_out():
    rng = np.random.default_rng(9)
    E, H, F, counts = 2, 32, 24, (9, 6)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offsets[-1])
    sx, sw, sh = 16.0, 512.0, 64.0   # powers of two: scaling is exact, so it must divide out exactly
    x = rng.normal(0, 1, (R, H)).astype(np.float32)
    w = [rng.normal(0, 0.05, s).astype(np.float32) for s in ((E, F, H), (E, F, H), (E, H, F))]
    xq, _ = oracle.fp8_quantize(x, sx)
    wq = [oracle.fp8_quantize(a, sw)[0] for a in w]
    res = oracle.experts_fp8(xq, offsets, wq[0], wq[1], wq[2], 1.0 / (sx * sw), 1.0 / (sx * sw), sh, 1.0 / (sh * sw),
                             want_h=True)
    # every E4M3 value (and its power-of-two multiple) is a bf16 number: hand the
    # dequantised operands to the other oracle
    deq = lambda q, s: f32_to_bf16_bits((oracle.fp8_decode(q) / s).astype(np.float32))
    y_ref, h_ref = oracle.experts(deq(xq, sx), offsets, deq(wq[0], sw), deq(wq[1], sw), deq(wq[2], sw), want_h=True)
    np.testing.assert_allclose(res.h_val, h_ref, rtol=1e-12, atol=1e-300)
    # the recorded amax is that of h itself, not of h times its scale (the next step's scale is 448 / amax)
    assert res.amax_h == np.abs(res.h_val).max() and sh != 1.0
    # second GEMM runs on the quantised h
    hq_val = oracle.fp8_decode(res.hq) / sh
    for e in range(E):
        lo, hi = offsets[e], offsets[e + 1]
        wd = oracle.fp8_decode(wq[2][e]) / sw
        np.testing.assert_allclose(res.y[lo:hi], hq_val[lo:hi] @ wd.T, rtol=1e-12, atol=1e-15)
    # and quantising h costs at most half an E4M3 step
    assert np.all(np.abs(hq_val - res.h_val) <= np.maximum(np.abs(res.h_val) * 2.0 ** -4, 2.0 ** -10 / sh))


def test_experts_fp8_gate_and_up_are_not_interchangeable_and_experts_use_their_own_weights():
    offsets, x, wg, wu, wd, enc = _small_int_case(seed=10)
    a = oracle.experts_fp8(enc(x), offsets, enc(wg), enc(wu), enc(wd), 1.0, 1.0, 1.0, 1.0, want_h=True)
    b = oracle.experts_fp8(enc(x), offsets, enc(wu), enc(wg), enc(wd), 1.0, 1.0, 1.0, 1.0, want_h=True)
    assert np.abs(a.h_val - b.h_val).max() > 0.1          # silu is applied to the gate only
    c = oracle.experts_fp8(enc(x), offsets, enc(wg[::-1].copy()), enc(wu[::-1].copy()), enc(wd[::-1].copy()),
                           1.0, 1.0, 1.0, 1.0, want_h=True)
    assert np.abs(a.y - c.y).max() > 0.1                  # expert 0 and expert 2 swapped
    # dequantisation factors act where they should
    d = oracle.experts_fp8(enc(x), offsets, enc(wg), enc(wu), enc(wd), 1.0, 0.5, 1.0, 4.0, want_h=True)
    np.testing.assert_allclose(d.h_val, 0.5 * a.h_val, rtol=1e-14)

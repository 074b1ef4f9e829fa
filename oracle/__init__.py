"""ctypes access to the CPU oracle (oracle/moe_oracle.c, oracle/moe_oracle_fp8.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()``
and by ``bench.py``'s cpu_baseline leg, never by the product package.

Arrays holding layer tensors are float32 (fp32 configs) or uint16 bf16 bit
patterns (bf16 configs); the C side widens either exactly to double.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np

from .build import build as _build

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        # MOE_ORACLE_LIB: another build of the same sources, used only by tests/test_oracle_mutations.py to show
        # that the pins reject an oracle with a planted mistake
        L = C.CDLL(os.environ.get("MOE_ORACLE_LIB") or _build())
        L.oracle_num_threads.restype = C.c_int
        L.oracle_capacity.restype = C.c_int
        L.oracle_capacity.argtypes = [C.c_double, C.c_int, C.c_int, C.c_int]
        L.oracle_permute.restype = C.c_int
        L.oracle_permute_variant.restype = C.c_int
        L.oracle_layer_forward.restype = C.c_int
        L.oracle_sort_chunks.restype = C.c_longlong
        L.oracle_fp8_decode.restype = C.c_double
        L.oracle_fp8_decode.argtypes = [C.c_uint8]
        L.oracle_fp8_encode.restype = C.c_uint8
        L.oracle_fp8_encode.argtypes = [C.c_float]
        L.oracle_fp8_delayed_scale.restype = C.c_float
        L.oracle_fp8_delayed_scale.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.oracle_fp8_quantize.argtypes = [C.c_void_p, C.c_int, C.c_size_t, C.c_float, C.c_void_p, C.c_void_p]
        L.oracle_experts_fp8.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_double, C.c_double, C.c_float, C.c_double, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"layer tensors must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"], "oracle needs C-contiguous arrays"
    return a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def capacity(cf: float, T: int, K: int, E: int) -> int:
    return int(lib().oracle_capacity(float(cf), T, K, E))


def router_logits(x: np.ndarray, w_router: np.ndarray, bias: Optional[np.ndarray]) -> np.ndarray:
    T, H = x.shape
    E = w_router.shape[0]
    assert w_router.shape == (E, H) and _dt(x) == _dt(w_router)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.shape == (E,)
    out = np.empty((T, E), dtype=np.float64)
    lib().oracle_router_logits(_p(x), _p(w_router), _p(bias), T, H, E, _dt(x), _p(out))
    return out


def topk_gates(logits32: np.ndarray, K: int, renormalize: bool,
               want_probs: bool = False):
    logits32 = np.ascontiguousarray(logits32)
    assert logits32.dtype == np.float32
    T, E = logits32.shape
    assert 1 <= K <= E
    idx = np.empty((T, K), dtype=np.int32)
    gate = np.empty((T, K), dtype=np.float64)
    probs = np.empty((T, E), dtype=np.float64) if want_probs else None
    lib().oracle_topk_gates(_p(logits32), T, E, K, int(bool(renormalize)), _p(idx), _p(gate), _p(probs))
    return (idx, gate, probs) if want_probs else (idx, gate)


class Permutation:
    """Result of oracle_permute."""
    def __init__(self, R, x_perm, counts, offsets, row_of_assign, assign_of_row):
        self.R = R
        self.x_perm = x_perm
        self.counts = counts
        self.offsets = offsets
        self.row_of_assign = row_of_assign
        self.assign_of_row = assign_of_row


def permute(x: Optional[np.ndarray], idx: np.ndarray, E: int, capacity_rows: int = 0,
            r_max: Optional[int] = None, H: Optional[int] = None) -> Permutation:
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, K = idx.shape
    if x is not None:
        assert x.shape[0] == T
        H = x.shape[1]
        dt = _dt(x)
    else:
        H = H or 1
        dt = 0
    if r_max is None:
        r_max = T * K if capacity_rows <= 0 else min(T * K, E * capacity_rows)
    x_perm = None
    if x is not None:
        x_perm = np.zeros((r_max, H), dtype=x.dtype)
    counts = np.empty(E, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    roa = np.empty(T * K, dtype=np.int32)
    aor = np.empty(max(r_max, 1), dtype=np.int32)
    R = lib().oracle_permute(_p(x), _p(idx), T, H, E, K, int(capacity_rows), dt, r_max,
                             _p(x_perm), _p(counts), _p(offsets), _p(roa), _p(aor))
    return Permutation(int(R), x_perm, counts, offsets, roa, aor[:r_max])


def permute_variant(x: Optional[np.ndarray], idx: np.ndarray, scores: Optional[np.ndarray], E: int,
                    capacity_rows: int, by_score: bool, pad: bool, r_max: Optional[int] = None,
                    H: Optional[int] = None) -> Permutation:
    """Dispatch with the drop rule (position or score) and layout (packed or padded to capacity) chosen."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, K = idx.shape
    if scores is not None:
        scores = np.ascontiguousarray(scores, dtype=np.float32)
        assert scores.shape == (T, K)
    assert not by_score or scores is not None
    assert not pad or capacity_rows > 0
    if x is not None:
        assert x.shape[0] == T
        H = x.shape[1]
        dt = _dt(x)
    else:
        H = H or 1
        dt = 0
    if r_max is None:
        if pad:
            r_max = E * capacity_rows
        else:
            r_max = T * K if capacity_rows <= 0 else min(T * K, E * capacity_rows)
    x_perm = np.zeros((r_max, H), dtype=x.dtype) if x is not None else None
    counts = np.empty(E, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    roa = np.empty(T * K, dtype=np.int32)
    aor = np.empty(max(r_max, 1), dtype=np.int32)
    R = lib().oracle_permute_variant(_p(x), _p(idx), _p(scores), T, H, E, K, int(capacity_rows), int(by_score),
                                     int(pad), dt, r_max, _p(x_perm), _p(counts), _p(offsets), _p(roa), _p(aor))
    assert R >= 0
    return Permutation(int(R), x_perm, counts, offsets, roa, aor[:r_max])


def expert_ffn_rows(x_rows: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray,
                    want_h: bool = False):
    """One expert's SwiGLU FFN over the given rows; returns y (and h) in double."""
    n, H = x_rows.shape
    F = w_gate.shape[0]
    assert w_gate.shape == (F, H) and w_up.shape == (F, H) and w_down.shape == (H, F)
    dt = _dt(x_rows)
    assert dt == _dt(w_gate) == _dt(w_up) == _dt(w_down)
    x_rows = np.ascontiguousarray(x_rows)
    y = np.zeros((n, H), dtype=np.float64)
    h = np.zeros((n, F), dtype=np.float64) if want_h else None
    lib().oracle_expert_ffn_rows(_p(x_rows), n, H, F, _p(w_gate), _p(w_up), _p(w_down), dt, _p(h), _p(y))
    return (y, h) if want_h else y


def experts(x_perm: np.ndarray, offsets: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray,
            w_down: np.ndarray, want_h: bool = False):
    E, F, H = w_gate.shape
    assert w_up.shape == (E, F, H) and w_down.shape == (E, H, F)
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    assert offsets.shape == (E + 1,)
    R = int(offsets[E])
    assert x_perm.shape[0] >= R and x_perm.shape[1] == H
    dt = _dt(x_perm)
    y = np.zeros((R, H), dtype=np.float64)
    h = np.zeros((R, F), dtype=np.float64) if want_h else None
    lib().oracle_experts(_p(x_perm), _p(offsets), E, H, F, _p(w_gate), _p(w_up), _p(w_down), dt, _p(h), _p(y))
    return (y, h) if want_h else y


def combine(y_perm: np.ndarray, row_of_assign: np.ndarray, gate: np.ndarray,
            addend: Optional[np.ndarray] = None) -> np.ndarray:
    y_perm = np.ascontiguousarray(y_perm, dtype=np.float64)
    gate = np.ascontiguousarray(gate, dtype=np.float64)
    T, K = gate.shape
    H = y_perm.shape[1]
    roa = np.ascontiguousarray(row_of_assign, dtype=np.int32).reshape(T * K)
    if addend is not None:
        addend = np.ascontiguousarray(addend, dtype=np.float64)
        assert addend.shape == (T, H)
    y = np.empty((T, H), dtype=np.float64)
    lib().oracle_combine(_p(y_perm), _p(roa), _p(gate), _p(addend), T, H, K, _p(y))
    return y


def router_backward(x: np.ndarray, w_router: np.ndarray, logits32: np.ndarray, idx: np.ndarray, dgate: np.ndarray,
                    renormalize: bool):
    """Backward of the router: returns (dlogits [T,E], dx [T,H], dw_router [E,H], dbias [E]) in double."""
    T, H = x.shape
    E = w_router.shape[0]
    logits32 = np.ascontiguousarray(logits32, dtype=np.float32)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    dgate = np.ascontiguousarray(dgate, dtype=np.float64)
    K = idx.shape[1]
    assert logits32.shape == (T, E) and dgate.shape == (T, K) and _dt(x) == _dt(w_router)
    dl = np.zeros((T, E), dtype=np.float64)
    dx = np.zeros((T, H), dtype=np.float64)
    dw = np.zeros((E, H), dtype=np.float64)
    db = np.zeros(E, dtype=np.float64)
    lib().oracle_router_backward(_p(np.ascontiguousarray(x)), _p(np.ascontiguousarray(w_router)), _p(logits32), _p(idx),
                                 _p(dgate), T, H, E, K, int(bool(renormalize)), _dt(x), _p(dl), _p(dx), _p(dw), _p(db))
    return dl, dx, dw, db


def experts_backward(x_perm: np.ndarray, offsets: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray,
                     w_down: np.ndarray, dy: np.ndarray):
    """Backward of experts(): returns (dx [R,H], dw_gate [E,F,H], dw_up [E,F,H], dw_down [E,H,F]) in double."""
    E, F, H = w_gate.shape
    assert w_up.shape == (E, F, H) and w_down.shape == (E, H, F)
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    R = int(offsets[E])
    assert x_perm.shape[0] >= R and x_perm.shape[1] == H
    dt = _dt(x_perm)
    assert dt == _dt(w_gate) == _dt(w_up) == _dt(w_down)
    dy = np.ascontiguousarray(dy, dtype=np.float64)
    assert dy.shape[0] >= R and dy.shape[1] == H
    dx = np.zeros((R, H), dtype=np.float64)
    dwg = np.zeros((E, F, H), dtype=np.float64)
    dwu = np.zeros((E, F, H), dtype=np.float64)
    dwd = np.zeros((E, H, F), dtype=np.float64)
    lib().oracle_experts_backward(_p(np.ascontiguousarray(x_perm)), _p(offsets), E, H, F, _p(w_gate), _p(w_up),
                                  _p(w_down), dt, _p(dy), _p(dx), _p(dwg), _p(dwu), _p(dwd))
    return dx, dwg, dwu, dwd


def combine_backward(dy: np.ndarray, y_perm: np.ndarray, row_of_assign: np.ndarray, gate: np.ndarray):
    """Backward of combine(): returns (dy_perm [R,H], dgate [T,K]); rows of dy_perm that no kept
    assignment points at stay zero."""
    dy = np.ascontiguousarray(dy, dtype=np.float64)
    y_perm = np.ascontiguousarray(y_perm, dtype=np.float64)
    gate = np.ascontiguousarray(gate, dtype=np.float64)
    T, K = gate.shape
    H = dy.shape[1]
    roa = np.ascontiguousarray(row_of_assign, dtype=np.int32).reshape(-1)
    assert roa.size == T * K and dy.shape == (T, H) and y_perm.shape[1] == H
    assert roa.max(initial=-1) < y_perm.shape[0]
    dy_perm = np.zeros_like(y_perm)
    dgate = np.zeros((T, K), dtype=np.float64)
    lib().oracle_combine_backward(_p(dy), _p(y_perm), _p(roa), _p(gate), T, H, K, _p(dy_perm), _p(dgate))
    return dy_perm, dgate


def permute_backward(dx_perm: np.ndarray, row_of_assign: np.ndarray, T: int, K: int,
                     addend: Optional[np.ndarray] = None) -> np.ndarray:
    """Backward of permute(): dx [T,H]."""
    dx_perm = np.ascontiguousarray(dx_perm, dtype=np.float64)
    H = dx_perm.shape[1]
    roa = np.ascontiguousarray(row_of_assign, dtype=np.int32).reshape(-1)
    assert roa.size == T * K and roa.max(initial=-1) < dx_perm.shape[0]
    if addend is not None:
        addend = np.ascontiguousarray(addend, dtype=np.float64)
        assert addend.shape == (T, H)
    dx = np.zeros((T, H), dtype=np.float64)
    lib().oracle_permute_backward(_p(dx_perm), _p(roa), _p(addend), T, H, K, _p(dx))
    return dx


def sort_chunks(src: Optional[np.ndarray], chunk_rows, order, group: int = 0, r_dst: Optional[int] = None):
    """Gather of ragged row chunks: dst = chunks order[0], order[1], ... of src.

    Returns (dst [r_dst, H] or None, rows of each dst chunk, group offsets or None, total rows)."""
    chunk_rows = np.ascontiguousarray(chunk_rows, dtype=np.int32).reshape(-1)
    order = np.ascontiguousarray(order, dtype=np.int32).reshape(-1)
    n_src, n_dst = chunk_rows.size, order.size
    rows_out = np.zeros(n_dst, dtype=np.int32)
    goff = np.zeros((n_dst + group - 1) // group + 1, dtype=np.int32) if group > 0 else None
    if src is not None:
        src = np.ascontiguousarray(src)
        r_src, row_bytes = src.shape[0], src.shape[1] * src.itemsize
    else:
        r_src, row_bytes = 0, 0
    if r_dst is None:
        valid = (order >= 0) & (order < n_src)
        r_dst = int(np.maximum(chunk_rows, 0)[order[valid]].sum())
    dst = np.zeros((r_dst, src.shape[1]), dtype=src.dtype) if src is not None else None
    total = lib().oracle_sort_chunks(_p(src), C.c_longlong(r_src), _p(chunk_rows), n_src, _p(order), n_dst,
                                     int(group), C.c_size_t(row_bytes), _p(dst), C.c_longlong(r_dst),
                                     _p(rows_out), _p(goff))
    return dst, rows_out, goff, int(total)


class LayerResult:
    def __init__(self, R, logits32, idx, gate, row_of_assign, y):
        self.R = R
        self.logits32 = logits32
        self.idx = idx
        self.gate = gate
        self.row_of_assign = row_of_assign
        self.y = y


def layer_forward(x, w_router, bias, w_gate, w_up, w_down, K: int, renormalize: bool,
                  capacity_rows: int = 0, ws_gate=None, ws_up=None, ws_down=None) -> LayerResult:
    T, H = x.shape
    E, F, _ = w_gate.shape
    dt = _dt(x)
    Fs = 0 if ws_gate is None else ws_gate.shape[0]
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    logits32 = np.empty((T, E), dtype=np.float32)
    idx = np.empty((T, K), dtype=np.int32)
    gate = np.empty((T, K), dtype=np.float64)
    roa = np.empty(T * K, dtype=np.int32)
    y = np.empty((T, H), dtype=np.float64)
    R = lib().oracle_layer_forward(_p(x), _p(w_router), _p(bias), _p(w_gate), _p(w_up), _p(w_down),
                                   _p(ws_gate), _p(ws_up), _p(ws_down), T, H, E, K, F, Fs,
                                   int(bool(renormalize)), int(capacity_rows), dt,
                                   _p(logits32), _p(idx), _p(gate), _p(roa), _p(y))
    return LayerResult(int(R), logits32, idx, gate, roa, y)


def dense_bruteforce(x, w_router, bias, w_gate, w_up, w_down, K: int, renormalize: bool,
                     capacity_rows: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 1 with every expert evaluated on every token; returns (y, dense gates)."""
    T, H = x.shape
    E, F, _ = w_gate.shape
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    g = np.empty((T, E), dtype=np.float64)
    y = np.empty((T, H), dtype=np.float64)
    lib().oracle_dense_bruteforce(_p(x), _p(w_router), _p(bias), _p(w_gate), _p(w_up), _p(w_down),
                                  T, H, E, K, F, int(bool(renormalize)), int(capacity_rows), _dt(x),
                                  _p(g), _p(y))
    return y, g


# ---------------------------------------------------------------- FP8 (E4M3) variant
def fp8_decode(codes: np.ndarray) -> np.ndarray:
    """Values (float64) of E4M3 codes (uint8), element by element."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    f = lib().oracle_fp8_decode
    return np.array([f(int(c)) for c in codes.ravel()], dtype=np.float64).reshape(codes.shape)


def fp8_encode(values: np.ndarray) -> np.ndarray:
    """Nearest E4M3 codes (ties to even, saturating) of float32 values, element by element."""
    values = np.ascontiguousarray(values, dtype=np.float32)
    f = lib().oracle_fp8_encode
    return np.array([f(float(v)) for v in values.ravel()], dtype=np.uint8).reshape(values.shape)


def fp8_quantize(src: np.ndarray, scale: float, amax_in: float = 0.0) -> Tuple[np.ndarray, float]:
    """codes = encode(fp32(src * scale)); returns (codes, max(amax_in, max |src|))."""
    src = np.ascontiguousarray(src)
    dst = np.empty(src.shape, dtype=np.uint8)
    amax = np.array([amax_in], dtype=np.float32)
    lib().oracle_fp8_quantize(_p(src), _dt(src), src.size, float(scale), _p(dst), _p(amax))
    return dst, float(amax[0])


def fp8_delayed_scale(amax_history, margin: int = 0) -> float:
    h = np.ascontiguousarray(amax_history, dtype=np.float32)
    return float(lib().oracle_fp8_delayed_scale(_p(h), int(h.size), int(margin)))


class Fp8Experts:
    def __init__(self, hq, h_val, amax_h, y):
        self.hq = hq          # [R, F] uint8 E4M3 codes of h * scale_h
        self.h_val = h_val    # [R, F] float64, h before quantisation (or None)
        self.amax_h = amax_h  # max |h|
        self.y = y            # [R, H] float64


def experts_fp8(xq: np.ndarray, offsets: np.ndarray, wg: np.ndarray, wu: np.ndarray, wd: np.ndarray,
                dq_gate: float, dq_up: float, scale_h: float, dq_down: float,
                want_h: bool = False) -> Fp8Experts:
    E, F, H = wg.shape
    assert wu.shape == (E, F, H) and wd.shape == (E, H, F)
    for a in (xq, wg, wu, wd):
        assert a.dtype == np.uint8
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    R = int(offsets[E])
    assert xq.shape[0] >= R and xq.shape[1] == H
    hq = np.zeros((R, F), dtype=np.uint8)
    h_val = np.zeros((R, F), dtype=np.float64) if want_h else None
    y = np.zeros((R, H), dtype=np.float64)
    amax = np.zeros(1, dtype=np.float64)
    lib().oracle_experts_fp8(_p(np.ascontiguousarray(xq)), _p(offsets), E, H, F, _p(np.ascontiguousarray(wg)),
                             _p(np.ascontiguousarray(wu)), _p(np.ascontiguousarray(wd)), float(dq_gate),
                             float(dq_up), float(scale_h), float(dq_down), _p(hq), _p(h_val), _p(amax), _p(y))
    return Fp8Experts(hq, h_val, float(amax[0]), y)

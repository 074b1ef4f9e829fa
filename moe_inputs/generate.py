"""Seeded tensor generation for one MoE layer.

Every tensor is drawn in independent row blocks, each from its own PCG64 stream
keyed by (config seed, tensor id, expert, block), so that

* generation is reproducible regardless of thread count,
* a test can build only the tensors (or experts) it needs, and
* the CPU oracle and the HIP path receive identical bytes.

For the bf16 configurations the fp32 draws are rounded to bf16
(round-to-nearest-even) here, once; both sides then read the same 16-bit
patterns.  Nothing in this file evaluates any part of the layer.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Iterable, Optional, Sequence

import numpy as np

from .configs import LayerConfig

# tensor ids used as the second word of the seed sequence
_TID = {
    "x": 0, "w_router": 1, "bias": 2, "w_gate": 3, "w_up": 4, "w_down": 5,
    "ws_gate": 6, "ws_up": 7, "ws_down": 8, "redraw": 9, "logits": 10, "rows": 11,
}
_ROW_BLOCK = 1024          # rows per independently seeded block
_WEIGHT_STD = 0.02
ALL_TENSORS = ("x", "w_router", "bias", "w_gate", "w_up", "w_down",
               "ws_gate", "ws_up", "ws_down")


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _stream(seed: int, tid: int, a: int = 0, b: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tid, a, b])))


def _workers() -> int:
    return max(1, min(16, (os.cpu_count() or 1)))


def _normal_rows(seed: int, tid: int, idx: int, rows: int, cols: int, std: float,
                 bf16: bool, pool: Optional[ThreadPoolExecutor]) -> np.ndarray:
    """[rows, cols] ~ N(0, std^2), drawn per block of _ROW_BLOCK rows."""
    out = np.empty((rows, cols), dtype=np.uint16 if bf16 else np.float32)

    def fill(blk: int) -> None:
        lo = blk * _ROW_BLOCK
        hi = min(rows, lo + _ROW_BLOCK)
        v = _stream(seed, tid, idx, blk).standard_normal((hi - lo, cols), dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        out[lo:hi] = f32_to_bf16_bits(v) if bf16 else v

    nblk = (rows + _ROW_BLOCK - 1) // _ROW_BLOCK
    if pool is None or nblk == 1:
        for b in range(nblk):
            fill(b)
    else:
        list(pool.map(fill, range(nblk)))
    return out


@dataclass
class LayerInputs:
    """Host copies of one layer's tensors in their storage type.

    fp32 configs hold float32 arrays; bf16 configs hold uint16 bit patterns.
    ``bias`` is always float32 (it is added to fp32 logits) or None.
    """
    cfg: LayerConfig
    tensors: Dict[str, np.ndarray] = field(default_factory=dict)
    bias: Optional[np.ndarray] = None

    @property
    def is_bf16(self) -> bool:
        return self.cfg.dtype == "bf16"

    def __getitem__(self, name: str) -> np.ndarray:
        return self.tensors[name]

    def __contains__(self, name: str) -> bool:
        return name in self.tensors

    def f32(self, name: str) -> np.ndarray:
        """The tensor's values as float32 (exact for both storage types)."""
        t = self.tensors[name]
        return bf16_bits_to_f32(t) if t.dtype == np.uint16 else t


def make_bias(cfg: LayerConfig) -> Optional[np.ndarray]:
    """Per-expert additive logit bias that skews the load (None = balanced)."""
    if cfg.bias is None:
        return None
    g = _stream(cfg.seed, _TID["bias"])
    if cfg.bias == "normal":
        return g.standard_normal(cfg.E, dtype=np.float32)
    if cfg.bias.startswith("zipf"):
        s = float(cfg.bias[4:])
        rank = g.permutation(cfg.E) + 1          # a random expert gets rank 1, another rank 2, ...
        return (-s * np.log(rank.astype(np.float64))).astype(np.float32)
    raise ValueError(f"unknown bias recipe {cfg.bias!r}")


def make_layer_inputs(cfg: LayerConfig, tensors: Optional[Iterable[str]] = None) -> LayerInputs:
    """Draw the tensors of one layer (all of them, or the named subset)."""
    want = set(ALL_TENSORS if tensors is None else tensors)
    bf16 = cfg.dtype == "bf16"
    T, H, E, F, Fs = cfg.T, cfg.H, cfg.E, cfg.F, cfg.shared_F
    out = LayerInputs(cfg)
    with ThreadPoolExecutor(_workers()) as pool:
        if "x" in want:
            out.tensors["x"] = _normal_rows(cfg.seed, _TID["x"], 0, T, H, 1.0, bf16, pool)
        if "w_router" in want:
            out.tensors["w_router"] = _normal_rows(cfg.seed, _TID["w_router"], 0, E, H, _WEIGHT_STD, bf16, pool)
        if "bias" in want:
            out.bias = make_bias(cfg)
        for name, rows, cols in (("w_gate", F, H), ("w_up", F, H), ("w_down", H, F)):
            if name in want:
                w = np.empty((E, rows, cols), dtype=np.uint16 if bf16 else np.float32)
                for e in range(E):
                    w[e] = _normal_rows(cfg.seed, _TID[name], e, rows, cols, _WEIGHT_STD, bf16, pool)
                out.tensors[name] = w
        if Fs > 0:
            for name, rows, cols in (("ws_gate", Fs, H), ("ws_up", Fs, H), ("ws_down", H, Fs)):
                if name in want:
                    out.tensors[name] = _normal_rows(cfg.seed, _TID[name], 0, rows, cols, _WEIGHT_STD, bf16, pool)
    return out


def redraw_token_rows(inp: LayerInputs, rows: Sequence[int], round_no: int) -> None:
    """Replace the given rows of ``x`` by fresh N(0,1) draws (in place).

    Tests use this to move a token whose K-th and (K+1)-th router logits are
    closer than the summation-order noise of fp32; which rows those are is the
    test's business (it asks the oracle), not this module's.
    """
    rows = np.asarray(sorted(int(r) for r in rows), dtype=np.int64)
    if rows.size == 0:
        return
    H = inp.cfg.H
    v = _stream(inp.cfg.seed, _TID["redraw"], round_no).standard_normal((rows.size, H), dtype=np.float32)
    inp.tensors["x"][rows] = f32_to_bf16_bits(v) if inp.is_bf16 else v


def make_tokens(seed: int, rows: int, cols: int, bf16: bool, std: float = 1.0) -> np.ndarray:
    """A free-standing [rows, cols] activation-like tensor (stage tests)."""
    return _normal_rows(seed, _TID["rows"], 0, rows, cols, std, bf16, None)


def make_logits(seed: int, T: int, E: int, kind: str = "normal") -> np.ndarray:
    """fp32 router logits for selection tests that bypass the router product.

    kinds: "normal" (iid N(0,1.5^2)), "equal" (all one value), "ties" (values
    from a 4-symbol alphabet, so most rows hold exact ties), "dupcols" (every
    odd column repeats the column before it), "zeros" (a mix of +0.0 and -0.0),
    "tiny" (subnormal magnitudes), "onehot" (every token prefers expert 0).
    """
    g = _stream(seed, _TID["logits"], T, E)
    if kind == "normal":
        return (1.5 * g.standard_normal((T, E), dtype=np.float32)).astype(np.float32)
    if kind == "equal":
        return np.full((T, E), 0.375, dtype=np.float32)
    if kind == "ties":
        return g.integers(0, 4, size=(T, E)).astype(np.float32) * np.float32(0.5) - np.float32(0.75)
    if kind == "dupcols":
        a = g.standard_normal((T, E), dtype=np.float32)
        a[:, 1::2] = a[:, 0:(E // 2) * 2:2]
        return a
    if kind == "zeros":
        sign = g.integers(0, 2, size=(T, E)).astype(np.uint32) << np.uint32(31)
        return sign.view(np.float32)
    if kind == "tiny":
        return (g.integers(-40, 41, size=(T, E)).astype(np.float32) * np.float32(1e-42)).astype(np.float32)
    if kind == "onehot":
        a = g.standard_normal((T, E), dtype=np.float32)
        a[:, 0] += np.float32(50.0)
        return a
    raise ValueError(f"unknown logits kind {kind!r}")


def expected_bytes(cfg: LayerConfig) -> int:
    """Host bytes make_layer_inputs(cfg) allocates (for sizing tests)."""
    s = 2 if cfg.dtype == "bf16" else 4
    n = cfg.T * cfg.H + cfg.E * cfg.H + 3 * cfg.E * cfg.H * cfg.F + 3 * cfg.H * cfg.shared_F
    return n * s + (4 * cfg.E if cfg.bias else 0)

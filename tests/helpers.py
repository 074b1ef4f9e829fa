"""Shared test plumbing: host<->device conversion, tolerances, margin guard.

Nothing here computes any part of the layer; expected values always come from
``oracle`` and GPU values always come through the C ABI binding.
"""
from __future__ import annotations

import numpy as np

import oracle
from moe_inputs import LayerInputs, bf16_bits_to_f32, redraw_token_rows

# acceptance bars: bf16 max|d| <= 2e-2 max|ref| and relative L2 <= 5e-3 (three bf16 roundings at 2^-9 each give ~3e-3);
# fp32: accumulation over <= 256 terms has relative error <~ sqrt(256) * 6e-8 ~ 1e-6, taken with a 10x margin
BF16_MAXABS, BF16_RELL2 = 2e-2, 5e-3
F32_MAXABS, F32_RELL2 = 1e-4, 1e-5
GATE_ATOL, GATE_RTOL = 1e-6, 1e-5
LOGIT_ATOL = 1e-4


def to_dev(a: np.ndarray):
    """numpy (float32 / int32 / uint16 bf16 bits) -> cuda tensor of the matching dtype."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t) -> np.ndarray:
    """cuda tensor -> numpy; bf16 comes back as uint16 bit patterns."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def values(a: np.ndarray) -> np.ndarray:
    """float64 values of a float32 array or of bf16 bit patterns."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def assert_close(got: np.ndarray, ref: np.ndarray, bf16: bool, what: str = "") -> None:
    """max|d| <= a * max|ref| and ||d||_2 / ||ref||_2 <= b."""
    got, ref = values(got), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    a, b = (BF16_MAXABS, BF16_RELL2) if bf16 else (F32_MAXABS, F32_RELL2)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    d = got - ref
    scale = np.abs(ref).max()
    nref = np.linalg.norm(ref)
    maxabs = np.abs(d).max()
    rel = np.linalg.norm(d) / nref if nref > 0 else np.linalg.norm(d)
    assert maxabs <= a * scale + 1e-30, f"{what}: max|d|={maxabs:.3e} > {a}*max|ref|={a * scale:.3e}"
    assert rel <= b, f"{what}: rel-L2={rel:.3e} > {b}"


def fragile_rows(logits64: np.ndarray, K: int, margin: float) -> np.ndarray:
    """Tokens whose selection could flip under fp32 summation-order noise: the
    gap between any two neighbouring logits among the K+1 largest is < margin."""
    T, E = logits64.shape
    top = -np.sort(-logits64, axis=1)[:, :min(K + 1, E)]
    gaps = top[:, :-1] - top[:, 1:]
    if gaps.shape[1] == 0:
        return np.zeros(0, dtype=np.int64)
    return np.nonzero(gaps.min(axis=1) < margin)[0]


def guard_margins(inp: LayerInputs, K: int, margin: float = 1e-3, max_rounds: int = 12) -> int:
    """Re-draw token rows until no token's top-(K+1) logits are closer than
    `margin` (the oracle says which).  Returns how many rows were re-drawn."""
    total = 0
    for rnd in range(max_rounds):
        l = oracle.router_logits(inp["x"], inp["w_router"], inp.bias)
        rows = fragile_rows(l, K, margin)
        if rows.size == 0:
            return total
        total += rows.size
        redraw_token_rows(inp, rows, rnd)
    raise AssertionError("margin guard did not converge")


def capacity_rows(cfg) -> int:
    if cfg.capacity_factor is None:
        return 0
    return oracle.capacity(cfg.capacity_factor, cfg.T, cfg.K, cfg.E)


def oracle_layer_backward(x, w_router, bias, w_gate, w_up, w_down, K, renorm, capacity, dy):
    """The four backward functions chained in the order the backward workflow runs them (Section 3.3, mirrored)."""
    E = w_router.shape[0]
    T, H = x.shape
    logits32 = oracle.router_logits(x, w_router, bias).astype(np.float32)
    idx, gate = oracle.topk_gates(logits32, K, renorm)
    perm = oracle.permute(x, idx, E, capacity)
    R = perm.R
    y_perm = oracle.experts(perm.x_perm, perm.offsets, w_gate, w_up, w_down)
    dy_perm, dgate = oracle.combine_backward(dy, y_perm if R else np.zeros((1, H)), perm.row_of_assign, gate)
    dx_perm, dwg, dwu, dwd = oracle.experts_backward(perm.x_perm, perm.offsets, w_gate, w_up, w_down, dy_perm)
    dl, dx_r, dw_r, db = oracle.router_backward(x, w_router, logits32, idx, dgate, renorm)
    dx = oracle.permute_backward(dx_perm if R else np.zeros((1, H)), perm.row_of_assign, T, K, addend=dx_r)
    return dict(dx=dx, dw_router=dw_r, dbias=db, dw_gate=dwg, dw_up=dwu, dw_down=dwd, idx=idx)


def ep_chunk_orders(S: int, El: int):
    """Chunk orders of one GPU of an expert-parallel group of S ranks with El local experts: received chunks lie
    source-major (chunk s*El+e); `by_expert` lists them expert-major, `by_source` is the way back."""
    by_expert = np.array([s * El + e for e in range(El) for s in range(S)], dtype=np.int32)
    by_source = np.array([e * S + s for s in range(S) for e in range(El)], dtype=np.int32)
    return by_expert, by_source


def oracle_ep_group_forward(xs, w_router, bias, w_gate, w_up, w_down, K, renorm, capacity=0):
    """The layer over an expert-parallel group simulated on the CPU with the oracle's pieces (Section 3.3 forward
    workflow): every rank routes and permutes its own tokens, the All-to-All-V is a slicing of host arrays, each
    rank gathers what it received by expert (oracle.sort_chunks), runs its local experts, gathers back by source,
    the second All-to-All-V returns the rows, and every rank combines.  Returns one y [T_s, H] (double) per rank."""
    S = len(xs)
    E = w_gate.shape[0]
    assert E % S == 0
    El = E // S
    perms, gates = [], []
    for x in xs:
        logits32 = oracle.router_logits(x, w_router, bias).astype(np.float32)
        idx, gate = oracle.topk_gates(logits32, K, renorm)
        perms.append(oracle.permute(x, idx, E, capacity))
        gates.append(gate)
    by_expert, by_source = ep_chunk_orders(S, El)
    returned = [[None] * S for _ in range(S)]          # returned[s][d]: rows rank s gets back from rank d
    for d in range(S):
        lo, hi = d * El, (d + 1) * El
        recv = np.concatenate([p.x_perm[p.offsets[lo]:p.offsets[hi]] for p in perms])
        chunk_rows = np.concatenate([p.counts[lo:hi] for p in perms])
        grouped, rows_by_expert, goff, total = oracle.sort_chunks(recv, chunk_rows, by_expert, group=S)
        assert total == recv.shape[0]
        y_rows = oracle.experts(grouped, goff, w_gate[lo:hi], w_up[lo:hi], w_down[lo:hi])
        back, rows_by_source, _, _ = oracle.sort_chunks(y_rows, rows_by_expert, by_source)
        np.testing.assert_array_equal(rows_by_source, chunk_rows)
        bounds = np.concatenate([[0], np.cumsum([p.offsets[hi] - p.offsets[lo] for p in perms])])
        for s in range(S):
            returned[s][d] = back[bounds[s]:bounds[s + 1]]
    ys = []
    for s in range(S):
        y_perm = np.concatenate(returned[s])
        ys.append(oracle.combine(y_perm, perms[s].row_of_assign, gates[s]))
    return ys

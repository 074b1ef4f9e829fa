"""ctypes binding of include/moe.h: argument marshalling only.

Functions take torch tensors that already live on the GPU, pass their device
pointers and the current stream to the C ABI and return nothing that was
computed on the host.  There is no fallback: if the HIP library is missing the
import of a symbol raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

MOE_F32 = 0
MOE_BF16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")
_lib = None


class MoeError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"moe status {status}: {message}")
        self.status = status


def lib_path() -> str:
    return _LIB_PATH


def lib() -> C.CDLL:
    """Load libmoe_hip.so (built by ``python -m paper_2504_14960_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2504_14960_amd.build` "
            "(there is no non-HIP fallback)")
    L = C.CDLL(_LIB_PATH)
    vp, i, f, sz = C.c_void_p, C.c_int, C.c_double, C.c_size_t
    L.moe_last_error.restype = C.c_char_p
    L.moe_last_error.argtypes = []
    L.moe_version.restype = C.c_char_p
    L.moe_version.argtypes = []
    L.moe_capacity_from_factor.restype = i
    L.moe_capacity_from_factor.argtypes = [f, i, i, i]
    L.moe_max_rows.restype = i
    L.moe_max_rows.argtypes = [i, i, i, i]
    L.moe_permute_workspace_bytes.restype = sz
    L.moe_permute_workspace_bytes.argtypes = [i, i, i]
    L.moe_router_topk.restype = i
    L.moe_router_topk.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp, vp, vp]
    L.moe_permute.restype = i
    L.moe_permute.argtypes = [vp, vp, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp, sz, vp]
    L.moe_permute_noalloc.restype = i
    L.moe_permute_noalloc.argtypes = [vp, vp, i, i, i, i, i, i, vp, vp, vp, vp, vp, vp]
    L.moe_grouped_gemm_swiglu.restype = i
    L.moe_grouped_gemm_swiglu.argtypes = [vp, vp, i, i, i, i, vp, vp, vp, i, vp, vp, vp]
    L.moe_expert_gate_up.restype = i
    L.moe_expert_gate_up.argtypes = [vp, vp, i, i, i, i, vp, vp, i, vp, vp]
    L.moe_expert_down.restype = i
    L.moe_expert_down.argtypes = [vp, vp, i, i, i, i, vp, i, vp, vp]
    L.moe_unpermute_combine.restype = i
    L.moe_unpermute_combine.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, vp]
    L.moe_unpermute_combine_backward.restype = i
    L.moe_unpermute_combine_backward.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, vp, vp]
    L.moe_permute_backward.restype = i
    L.moe_permute_backward.argtypes = [vp, vp, vp, i, i, i, i, i, vp, vp]
    L.moe_router_backward_workspace_bytes.restype = sz
    L.moe_router_backward_workspace_bytes.argtypes = [i, i, i]
    L.moe_router_backward.restype = i
    L.moe_router_backward.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, vp, vp, vp, vp, vp, sz, vp]
    L.moe_expert_backward_workspace_bytes.restype = sz
    L.moe_expert_backward_workspace_bytes.argtypes = [i, i, i, i]
    L.moe_expert_weights_transpose.restype = i
    L.moe_expert_weights_transpose.argtypes = [vp, vp, vp, i, i, i, vp, vp, vp]
    L.moe_grouped_gemm_swiglu_backward.restype = i
    L.moe_grouped_gemm_swiglu_backward.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.moe_permute_variant_workspace_bytes.restype = sz
    L.moe_permute_variant_workspace_bytes.argtypes = [i, i, i]
    L.moe_sort_chunks_workspace_bytes.restype = sz
    L.moe_sort_chunks_workspace_bytes.argtypes = [i]
    L.moe_sort_chunks.restype = i
    L.moe_sort_chunks.argtypes = [vp, i, vp, i, vp, i, i, i, i, vp, i, vp, vp, vp, sz, vp]
    L.moe_permute_variant.restype = i
    L.moe_permute_variant.argtypes = [vp, vp, vp, i, i, i, i, i, i, i, i, vp, vp, vp, vp, vp, i, vp, sz, vp]
    L.moe_layer_forward_train.restype = i
    L.moe_layer_forward_train.argtypes = [vp] * 6 + [i] * 7 + [vp, vp, vp, sz, vp]
    L.moe_layer_backward_workspace_bytes.restype = sz
    L.moe_layer_backward_workspace_bytes.argtypes = [i] * 6
    L.moe_layer_backward.restype = i
    L.moe_layer_backward.argtypes = [vp] * 7 + [i] * 7 + [vp] * 9 + [sz, vp]
    L.moe_probe_mfma_fp8.restype = i
    L.moe_probe_mfma_fp8.argtypes = [vp, i, i, vp, vp, vp]
    L.moe_probe_mfma_bf16.restype = i
    L.moe_probe_mfma_bf16.argtypes = [vp, i, i, vp, vp, vp]
    L.moe_expert_gate_up_saving.restype = i
    L.moe_expert_gate_up_saving.argtypes = [vp, vp, i, i, i, i, vp, vp, vp, vp, vp]
    L.moe_layer_workspace_bytes.restype = sz
    L.moe_layer_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i]
    L.moe_workspace_bytes.restype = sz
    L.moe_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    L.moe_gemm_clock_sample.restype = i
    L.moe_gemm_clock_sample.argtypes = [vp]
    L.moe_layer_workspace_layout.restype = i
    L.moe_layer_workspace_layout.argtypes = [i, i, i, i, i, i, i, i, C.POINTER(sz), i]
    L.moe_layer_forward.restype = i
    L.moe_layer_forward.argtypes = [vp] * 9 + [i] * 9 + [vp, vp, sz, vp]
    L.moe_set_option.restype = i
    L.moe_set_option.argtypes = [C.c_char_p, i]
    f = C.c_float
    L.moe_fp8_delayed_scale.restype = f
    L.moe_fp8_delayed_scale.argtypes = [C.POINTER(f), i, i]
    L.moe_fp8_quantize.restype = i
    L.moe_fp8_quantize.argtypes = [vp, i, sz, f, vp, vp, vp]
    L.moe_permute_fp8.restype = i
    L.moe_permute_fp8.argtypes = [vp, vp, i, i, i, i, i, f, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.moe_grouped_gemm_swiglu_fp8.restype = i
    L.moe_grouped_gemm_swiglu_fp8.argtypes = [vp, vp, i, i, i, i, vp, vp, vp, f, f, f, f, vp, vp, vp, vp]
    L.moe_expert_gate_up_fp8.restype = i
    L.moe_expert_gate_up_fp8.argtypes = [vp, vp, i, i, i, i, vp, vp, f, f, f, vp, vp, vp]
    L.moe_expert_down_fp8.restype = i
    L.moe_expert_down_fp8.argtypes = [vp, vp, i, i, i, i, vp, f, vp, vp]
    _lib = L
    return L


def _check(status: int) -> None:
    if status != 0:
        raise MoeError(status, lib().moe_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("the MoE hot path takes device tensors only")
    if not t.is_contiguous():
        raise ValueError("tensors must be contiguous")
    return t.data_ptr()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    if t.dtype == torch.float32:
        return MOE_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream():
    return torch.cuda.current_stream().cuda_stream


def version() -> str:
    return lib().moe_version().decode()


def set_option(name: str, value: int) -> None:
    _check(lib().moe_set_option(name.encode(), int(value)))


def capacity_from_factor(cf: float, T: int, K: int, E: int) -> int:
    return int(lib().moe_capacity_from_factor(float(cf), T, K, E))


def max_rows(T: int, K: int, E: int, capacity: int) -> int:
    return int(lib().moe_max_rows(T, K, E, capacity))


def permute_workspace_bytes(T: int, K: int, E: int) -> int:
    return int(lib().moe_permute_workspace_bytes(T, K, E))


def router_topk(x: Optional[torch.Tensor], w_router: Optional[torch.Tensor],
                logit_bias: Optional[torch.Tensor], logits: torch.Tensor, K: int, renormalize: bool,
                topk_idx: torch.Tensor, topk_gate: torch.Tensor, dtype: Optional[int] = None) -> None:
    T, E = logits.shape
    H = x.shape[1] if x is not None else 0
    dt = _dt(x) if x is not None else (MOE_BF16 if dtype is None else dtype)
    _check(lib().moe_router_topk(_ptr(x), _ptr(w_router), _ptr(logit_bias), _ptr(logits), T, H, E, K,
                                 int(bool(renormalize)), dt, _ptr(topk_idx), _ptr(topk_gate), _stream()))


def permute(x: Optional[torch.Tensor], topk_idx: torch.Tensor, E: int, capacity: int,
            x_perm: Optional[torch.Tensor], expert_counts: torch.Tensor, expert_offsets: torch.Tensor,
            row_of_assign: torch.Tensor, assign_of_row: torch.Tensor, workspace: torch.Tensor,
            H: Optional[int] = None, dtype: int = MOE_BF16) -> None:
    T, K = topk_idx.shape
    if x is not None:
        H, dtype = x.shape[1], _dt(x)
    elif H is None:
        H = 8
    _check(lib().moe_permute(_ptr(x), _ptr(topk_idx), T, H, E, K, int(capacity), dtype, _ptr(x_perm),
                             _ptr(expert_counts), _ptr(expert_offsets), _ptr(row_of_assign),
                             _ptr(assign_of_row), _ptr(workspace), workspace.numel() * workspace.element_size(),
                             _stream()))


def permute_noalloc(x: Optional[torch.Tensor], topk_idx: torch.Tensor, E: int, capacity: int,
                    x_perm: Optional[torch.Tensor], expert_counts: torch.Tensor, expert_offsets: torch.Tensor,
                    row_of_assign: torch.Tensor, assign_of_row: torch.Tensor, H: Optional[int] = None,
                    dtype: int = MOE_BF16) -> None:
    T, K = topk_idx.shape
    if x is not None:
        H, dtype = x.shape[1], _dt(x)
    elif H is None:
        H = 8
    _check(lib().moe_permute_noalloc(_ptr(x), _ptr(topk_idx), T, H, E, K, int(capacity), dtype, _ptr(x_perm),
                                     _ptr(expert_counts), _ptr(expert_offsets), _ptr(row_of_assign),
                                     _ptr(assign_of_row), _stream()))


def grouped_gemm_swiglu(x_perm: torch.Tensor, expert_offsets: torch.Tensor, w_gate: torch.Tensor,
                        w_up: torch.Tensor, w_down: torch.Tensor, h_workspace: torch.Tensor,
                        y_perm: torch.Tensor) -> None:
    R_max, H = x_perm.shape
    E, F, _ = w_gate.shape
    _check(lib().moe_grouped_gemm_swiglu(_ptr(x_perm), _ptr(expert_offsets), R_max, H, F, E, _ptr(w_gate),
                                         _ptr(w_up), _ptr(w_down), _dt(x_perm), _ptr(h_workspace),
                                         _ptr(y_perm), _stream()))


def expert_gate_up(x_perm: torch.Tensor, expert_offsets: torch.Tensor, w_gate: torch.Tensor,
                   w_up: torch.Tensor, h: torch.Tensor) -> None:
    R_max, H = x_perm.shape
    E, F, _ = w_gate.shape
    _check(lib().moe_expert_gate_up(_ptr(x_perm), _ptr(expert_offsets), R_max, H, F, E, _ptr(w_gate),
                                    _ptr(w_up), _dt(x_perm), _ptr(h), _stream()))


def expert_down(h: torch.Tensor, expert_offsets: torch.Tensor, w_down: torch.Tensor,
                y_perm: torch.Tensor) -> None:
    R_max, F = h.shape
    E, H, _ = w_down.shape
    _check(lib().moe_expert_down(_ptr(h), _ptr(expert_offsets), R_max, H, F, E, _ptr(w_down), _dt(h),
                                 _ptr(y_perm), _stream()))


def unpermute_combine(y_perm: torch.Tensor, row_of_assign: torch.Tensor, topk_gate: torch.Tensor,
                      addend: Optional[torch.Tensor], y: torch.Tensor) -> None:
    T, K = topk_gate.shape
    R_max, H = y_perm.shape
    _check(lib().moe_unpermute_combine(_ptr(y_perm), _ptr(row_of_assign), _ptr(topk_gate), _ptr(addend),
                                       T, H, K, R_max, _dt(y), _ptr(y), _stream()))


# ---- FP8 (E4M3) variant of the expert FFN; E4M3 tensors are torch.uint8 (codes) ----
def fp8_delayed_scale(amax_history, margin: int = 0) -> float:
    h = [float(v) for v in amax_history]
    arr = (C.c_float * max(len(h), 1))(*h)
    return float(lib().moe_fp8_delayed_scale(arr, len(h), int(margin)))


def fp8_quantize(src: torch.Tensor, scale: float, dst: torch.Tensor, amax: Optional[torch.Tensor] = None) -> None:
    if dst.dtype != torch.uint8 or dst.numel() != src.numel():
        raise ValueError("dst must be a uint8 tensor with as many elements as src")
    _check(lib().moe_fp8_quantize(_ptr(src), _dt(src), src.numel(), float(scale), _ptr(dst), _ptr(amax), _stream()))


def permute_fp8(x: torch.Tensor, topk_idx: torch.Tensor, E: int, capacity: int, scale: float,
                x_perm_fp8: torch.Tensor, expert_counts: torch.Tensor, expert_offsets: torch.Tensor,
                row_of_assign: torch.Tensor, assign_of_row: torch.Tensor, amax: Optional[torch.Tensor],
                workspace: torch.Tensor) -> None:
    T, K = topk_idx.shape
    if x.dtype != torch.bfloat16 or x_perm_fp8.dtype != torch.uint8:
        raise TypeError("permute_fp8 takes a bf16 x and writes uint8 E4M3 codes")
    _check(lib().moe_permute_fp8(_ptr(x), _ptr(topk_idx), T, x.shape[1], E, K, int(capacity), float(scale),
                                 _ptr(x_perm_fp8), _ptr(expert_counts), _ptr(expert_offsets), _ptr(row_of_assign),
                                 _ptr(assign_of_row), _ptr(amax), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream()))


def grouped_gemm_swiglu_fp8(x_perm: torch.Tensor, expert_offsets: torch.Tensor, w_gate: torch.Tensor,
                            w_up: torch.Tensor, w_down: torch.Tensor, dq_gate: float, dq_up: float,
                            scale_h: float, dq_down: float, h: torch.Tensor, amax_h: Optional[torch.Tensor],
                            y_perm: torch.Tensor) -> None:
    R_max, H = x_perm.shape
    E, F, _ = w_gate.shape
    _check(lib().moe_grouped_gemm_swiglu_fp8(_ptr(x_perm), _ptr(expert_offsets), R_max, H, F, E, _ptr(w_gate),
                                             _ptr(w_up), _ptr(w_down), float(dq_gate), float(dq_up), float(scale_h),
                                             float(dq_down), _ptr(h), _ptr(amax_h), _ptr(y_perm), _stream()))


def expert_gate_up_fp8(x_perm: torch.Tensor, expert_offsets: torch.Tensor, w_gate: torch.Tensor, w_up: torch.Tensor,
                       dq_gate: float, dq_up: float, scale_h: float, h: torch.Tensor,
                       amax_h: Optional[torch.Tensor]) -> None:
    R_max, H = x_perm.shape
    E, F, _ = w_gate.shape
    _check(lib().moe_expert_gate_up_fp8(_ptr(x_perm), _ptr(expert_offsets), R_max, H, F, E, _ptr(w_gate), _ptr(w_up),
                                        float(dq_gate), float(dq_up), float(scale_h), _ptr(h), _ptr(amax_h),
                                        _stream()))


def expert_down_fp8(h: torch.Tensor, expert_offsets: torch.Tensor, w_down: torch.Tensor, dq_down: float,
                    y_perm: torch.Tensor) -> None:
    R_max, F = h.shape
    E, H, _ = w_down.shape
    _check(lib().moe_expert_down_fp8(_ptr(h), _ptr(expert_offsets), R_max, H, F, E, _ptr(w_down), float(dq_down),
                                     _ptr(y_perm), _stream()))


def router_backward_workspace_bytes(T: int, H: int, E: int) -> int:
    return int(lib().moe_router_backward_workspace_bytes(T, H, E))


def router_backward(x: torch.Tensor, w_router: torch.Tensor, logits: torch.Tensor, topk_idx: torch.Tensor,
                    dgate: torch.Tensor, renormalize: bool, dlogits: torch.Tensor, dx: Optional[torch.Tensor],
                    dw_router: Optional[torch.Tensor], dbias: Optional[torch.Tensor],
                    workspace: Optional[torch.Tensor]) -> None:
    T, E = logits.shape
    K = topk_idx.shape[1]
    H = x.shape[1]
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().moe_router_backward(_ptr(x), _ptr(w_router), _ptr(logits), _ptr(topk_idx), _ptr(dgate), T, H, E, K,
                                     int(bool(renormalize)), _dt(x), _ptr(dlogits), _ptr(dx), _ptr(dw_router),
                                     _ptr(dbias), _ptr(workspace), nbytes, _stream()))


def expert_backward_workspace_bytes(R_max: int, H: int, F: int, E: int) -> int:
    return int(lib().moe_expert_backward_workspace_bytes(R_max, H, F, E))


def expert_weights_transpose(w_gate: torch.Tensor, w_up: torch.Tensor, w_down: torch.Tensor, wgu_t: torch.Tensor,
                             wd_t: torch.Tensor) -> None:
    E, F, H = w_gate.shape
    _check(lib().moe_expert_weights_transpose(_ptr(w_gate), _ptr(w_up), _ptr(w_down), H, F, E, _ptr(wgu_t), _ptr(wd_t),
                                              _stream()))


def expert_gate_up_saving(x_perm: torch.Tensor, expert_offsets: torch.Tensor, w_gate: torch.Tensor,
                          w_up: torch.Tensor, h: torch.Tensor, gu: torch.Tensor) -> None:
    R_max, H = x_perm.shape
    E, F, _ = w_gate.shape
    _check(lib().moe_expert_gate_up_saving(_ptr(x_perm), _ptr(expert_offsets), R_max, H, F, E, _ptr(w_gate),
                                           _ptr(w_up), _ptr(h), _ptr(gu), _stream()))


def grouped_gemm_swiglu_backward(x_perm: torch.Tensor, h: torch.Tensor, gu: Optional[torch.Tensor],
                                 dy_perm: torch.Tensor, expert_offsets: torch.Tensor, w_gate: torch.Tensor, w_up: torch.Tensor,
                                 wgu_t: torch.Tensor, wd_t: torch.Tensor, dx_perm: torch.Tensor, dw_gate: torch.Tensor,
                                 dw_up: torch.Tensor, dw_down: torch.Tensor, workspace: torch.Tensor) -> None:
    R_max, H = x_perm.shape
    E, F, _ = w_gate.shape
    _check(lib().moe_grouped_gemm_swiglu_backward(_ptr(x_perm), _ptr(h), _ptr(gu), _ptr(dy_perm), _ptr(expert_offsets), R_max, H,
                                                  F, E, _ptr(w_gate), _ptr(w_up), _ptr(wgu_t), _ptr(wd_t),
                                                  _ptr(dx_perm), _ptr(dw_gate), _ptr(dw_up), _ptr(dw_down),
                                                  _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                  _stream()))


def unpermute_combine_backward(dy: torch.Tensor, y_perm: torch.Tensor, row_of_assign: torch.Tensor,
                               topk_gate: torch.Tensor, dy_perm: torch.Tensor, dgate: torch.Tensor) -> None:
    T, K = topk_gate.shape
    R_max, H = y_perm.shape
    _check(lib().moe_unpermute_combine_backward(_ptr(dy), _ptr(y_perm), _ptr(row_of_assign), _ptr(topk_gate), T, H, K,
                                                R_max, _dt(dy), _ptr(dy_perm), _ptr(dgate), _stream()))


def permute_backward(dx_perm: torch.Tensor, row_of_assign: torch.Tensor, addend: Optional[torch.Tensor],
                     dx: torch.Tensor, K: int) -> None:
    T, H = dx.shape
    _check(lib().moe_permute_backward(_ptr(dx_perm), _ptr(row_of_assign), _ptr(addend), T, H, K, dx_perm.shape[0],
                                      _dt(dx), _ptr(dx), _stream()))


def permute_variant_workspace_bytes(T: int, K: int, E: int) -> int:
    return int(lib().moe_permute_variant_workspace_bytes(T, K, E))


def permute_variant(x: Optional[torch.Tensor], topk_idx: torch.Tensor, scores: Optional[torch.Tensor], E: int,
                    capacity: int, drop_by_score: bool, pad_to_capacity: bool, x_perm: Optional[torch.Tensor],
                    expert_counts: torch.Tensor, expert_offsets: torch.Tensor, row_of_assign: torch.Tensor,
                    assign_of_row: torch.Tensor, workspace: torch.Tensor, H: Optional[int] = None,
                    dtype: Optional[int] = None) -> None:
    T, K = topk_idx.shape
    if x is not None:
        H, dtype = x.shape[1], _dt(x)
    _check(lib().moe_permute_variant(_ptr(x), _ptr(topk_idx), _ptr(scores), T, H or 8, E, K, capacity,
                                     int(drop_by_score), int(pad_to_capacity), MOE_BF16 if dtype is None else dtype,
                                     _ptr(x_perm), _ptr(expert_counts), _ptr(expert_offsets), _ptr(row_of_assign),
                                     _ptr(assign_of_row), assign_of_row.numel(), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream()))


def sort_chunks_workspace_bytes(n_dst: int) -> int:
    return int(lib().moe_sort_chunks_workspace_bytes(n_dst))


def sort_chunks(src: Optional[torch.Tensor], chunk_rows: torch.Tensor, order: torch.Tensor, group: int,
                dst: Optional[torch.Tensor], chunk_rows_out: Optional[torch.Tensor],
                group_offsets: Optional[torch.Tensor], workspace: torch.Tensor, H: Optional[int] = None,
                dtype: Optional[int] = None) -> None:
    ref = src if src is not None else dst
    if ref is not None:
        H, dtype = ref.shape[1], _dt(ref)
    _check(lib().moe_sort_chunks(_ptr(src), 0 if src is None else src.shape[0], _ptr(chunk_rows), chunk_rows.numel(),
                                 _ptr(order), order.numel(), group, H or 8, MOE_BF16 if dtype is None else dtype,
                                 _ptr(dst), 0 if dst is None else dst.shape[0], _ptr(chunk_rows_out),
                                 _ptr(group_offsets), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream()))


def probe_mfma_bf16(image: torch.Tensor, iters: int, workgroups: int, sink: torch.Tensor,
                    ticks: Optional[torch.Tensor]) -> None:
    assert image.numel() * image.element_size() == 65536 and sink.numel() >= workgroups * 256
    _check(lib().moe_probe_mfma_bf16(_ptr(image), iters, workgroups, _ptr(sink), _ptr(ticks), _stream()))


def layer_forward_train(x: torch.Tensor, w_router: torch.Tensor, logit_bias: Optional[torch.Tensor],
                        w_gate: torch.Tensor, w_up: torch.Tensor, w_down: torch.Tensor, K: int, renormalize: bool,
                        capacity: int, y: torch.Tensor, gu: torch.Tensor, workspace: torch.Tensor) -> None:
    T, H = x.shape
    E, F, _ = w_gate.shape
    _check(lib().moe_layer_forward_train(_ptr(x), _ptr(w_router), _ptr(logit_bias), _ptr(w_gate), _ptr(w_up),
                                         _ptr(w_down), T, H, E, K, F, int(renormalize), int(capacity), _ptr(y), _ptr(gu),
                                         _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def layer_backward_workspace_bytes(T: int, H: int, E: int, K: int, F: int, capacity: int) -> int:
    return int(lib().moe_layer_backward_workspace_bytes(T, H, E, K, F, capacity))


def layer_backward(x: torch.Tensor, w_router: torch.Tensor, w_gate: torch.Tensor, w_up: torch.Tensor,
                   wgu_t: torch.Tensor, wd_t: torch.Tensor, dy: torch.Tensor, K: int, renormalize: bool, capacity: int,
                   forward_workspace: torch.Tensor, gu: Optional[torch.Tensor], dx: torch.Tensor,
                   dw_router: Optional[torch.Tensor], dbias: Optional[torch.Tensor], dw_gate: torch.Tensor,
                   dw_up: torch.Tensor, dw_down: torch.Tensor, workspace: torch.Tensor) -> None:
    T, H = x.shape
    E, F, _ = w_gate.shape
    _check(lib().moe_layer_backward(_ptr(x), _ptr(w_router), _ptr(w_gate), _ptr(w_up), _ptr(wgu_t), _ptr(wd_t),
                                    _ptr(dy), T, H, E, K, F, int(renormalize), int(capacity), _ptr(forward_workspace),
                                    _ptr(gu), _ptr(dx), _ptr(dw_router), _ptr(dbias), _ptr(dw_gate), _ptr(dw_up),
                                    _ptr(dw_down), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream()))


def probe_mfma_fp8(image: torch.Tensor, iters: int, workgroups: int, sink: torch.Tensor,
                   ticks: Optional[torch.Tensor]) -> None:
    assert image.numel() * image.element_size() == 65536 and sink.numel() >= workgroups * 256
    _check(lib().moe_probe_mfma_fp8(_ptr(image), iters, workgroups, _ptr(sink), _ptr(ticks), _stream()))


def layer_workspace_bytes(T: int, H: int, E: int, K: int, F: int, Fs: int, capacity: int, dtype: int) -> int:
    return int(lib().moe_layer_workspace_bytes(T, H, E, K, F, Fs, capacity, dtype))


def workspace_bytes(T: int, H: int, E: int, K: int, F: int, capacity: int, dtype: int) -> int:
    return int(lib().moe_workspace_bytes(T, H, E, K, F, capacity, dtype))


def gemm_clock_sample(ticks: Optional[torch.Tensor]) -> None:
    """ticks: int64 device tensor of 2 elements that the following grouped bf16 GEMM launches fill, or None."""
    if ticks is not None and (ticks.dtype != torch.int64 or ticks.numel() < 2):
        raise ValueError("ticks must be an int64 tensor with at least 2 elements")
    _check(lib().moe_gemm_clock_sample(_ptr(ticks)))


_LAYOUT_NAMES = ("logits", "topk_idx", "topk_gate", "expert_counts", "expert_offsets", "row_of_assign",
                 "assign_of_row", "x_perm", "h", "y_perm", "shared_y")


def layer_workspace_layout(T: int, H: int, E: int, K: int, F: int, Fs: int, capacity: int, dtype: int) -> dict:
    arr = (C.c_size_t * 11)()
    _check(lib().moe_layer_workspace_layout(T, H, E, K, F, Fs, capacity, dtype, arr, 11))
    return dict(zip(_LAYOUT_NAMES, (int(v) for v in arr)))


def layer_forward(x: torch.Tensor, w_router: torch.Tensor, logit_bias: Optional[torch.Tensor],
                  w_gate: torch.Tensor, w_up: torch.Tensor, w_down: torch.Tensor,
                  ws_gate: Optional[torch.Tensor], ws_up: Optional[torch.Tensor],
                  ws_down: Optional[torch.Tensor], K: int, renormalize: bool, capacity: int,
                  y: torch.Tensor, workspace: torch.Tensor) -> None:
    T, H = x.shape
    E, F, _ = w_gate.shape
    Fs = 0 if ws_gate is None else ws_gate.shape[0]
    _check(lib().moe_layer_forward(_ptr(x), _ptr(w_router), _ptr(logit_bias), _ptr(w_gate), _ptr(w_up),
                                   _ptr(w_down), _ptr(ws_gate), _ptr(ws_up), _ptr(ws_down), T, H, E, K, F,
                                   Fs, int(bool(renormalize)), int(capacity), _dt(x), _ptr(y),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))

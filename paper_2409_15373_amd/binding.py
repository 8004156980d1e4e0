"""ctypes binding of libjfa.so: argument marshalling only -- every step runs in the HIP kernels.

Functions mirror the C ABI of include/jfa.h.  Tensors are torch CUDA (ROCm) tensors used purely as
device memory; work is enqueued on torch's current stream.  A missing library raises: there is no
CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libjfa.so")
_lib = None

JFA_OK = 0
JFA_ERR_INVALID_ARG = -1
JFA_ERR_UNSUPPORTED = -2
JFA_ERR_ALLOC = -3
JFA_ERR_HIP = -4

EXPORTS = (
    "jfa_forward", "jfa_forward_f32", "jfa_backward", "jfa_backward_f32", "jfa_build_schedule",
    "jfa_check_offsets", "jfa_workspace_bytes", "jfa_last_error", "jfa_version", "jfa_timing_enable",
    "jfa_timing_read", "jfa_square_offsets", "jfa_unfused_scores", "jfa_unfused_softmax", "jfa_unfused_apply",
    "jfa_jagged_to_dense", "jfa_dense_to_jagged", "jfa_jagged_dense_bmm", "jfa_jagged_jagged_bmm",
    "jfa_jagged_softmax", "jfa_jagged_softmax_backward", "jfa_forward_cross", "jfa_forward_cross_f32",
    "jfa_backward_cross", "jfa_backward_cross_f32", "jfa_forward_causal", "jfa_forward_causal_f32",
    "jfa_backward_causal", "jfa_backward_causal_f32", "jfa_unfused_product", "jfa_unfused_softmax_backward",
    "jfa_unfused_apply_transposed", "jfa_forward_noalloc",
)


class JfaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libjfa status {status}: {message}")
        self.status = status


def load() -> ctypes.CDLL:
    """Load libjfa.so (built by ``python -m paper_2409_15373_amd.build``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2409_15373_amd.build` "
                          "(hipcc, gfx950). There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    lib.jfa_forward.restype = i32
    lib.jfa_forward.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, vp, vp]
    lib.jfa_forward_f32.restype = i32
    lib.jfa_forward_f32.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, vp, vp]
    lib.jfa_forward_noalloc.restype = i32
    lib.jfa_forward_noalloc.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, vp, vp]
    lib.jfa_backward.restype = i32
    lib.jfa_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i32, i32, vp, vp, vp, vp, vp]
    lib.jfa_backward_f32.restype = i32
    lib.jfa_backward_f32.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i32, i32, vp, vp, vp, vp, vp]
    for name in ("jfa_forward_cross", "jfa_forward_cross_f32"):
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, vp, vp, vp]
    for name in ("jfa_backward_cross", "jfa_backward_cross_f32"):
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp]
    for name in ("jfa_forward_causal", "jfa_forward_causal_f32"):
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = lib.jfa_forward.argtypes
    for name in ("jfa_backward_causal", "jfa_backward_causal_f32"):
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = lib.jfa_backward.argtypes
    lib.jfa_build_schedule.restype = i32
    lib.jfa_build_schedule.argtypes = [vp, i64, i32, vp, vp, vp]
    lib.jfa_check_offsets.restype = i32
    lib.jfa_check_offsets.argtypes = [vp, i64, i64, vp, ctypes.POINTER(ctypes.c_int)]
    lib.jfa_workspace_bytes.restype = sz
    lib.jfa_workspace_bytes.argtypes = [i64, i64, i32, i32, i32]
    lib.jfa_last_error.restype = ctypes.c_char_p
    lib.jfa_last_error.argtypes = []
    lib.jfa_version.restype = i32
    lib.jfa_version.argtypes = []
    lib.jfa_timing_enable.restype = i32
    lib.jfa_timing_enable.argtypes = [i32]
    lib.jfa_timing_read.restype = i32
    lib.jfa_timing_read.argtypes = [i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_float),
                                    ctypes.POINTER(ctypes.c_int)]
    lib.jfa_square_offsets.restype = i32
    lib.jfa_square_offsets.argtypes = [vp, i64, vp, vp]
    lib.jfa_unfused_scores.restype = i32
    lib.jfa_unfused_scores.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, vp]
    lib.jfa_unfused_softmax.restype = i32
    lib.jfa_unfused_softmax.argtypes = [vp, vp, i64, i64, i32, vp, vp]
    lib.jfa_unfused_apply.restype = i32
    lib.jfa_unfused_apply.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, vp]
    lib.jfa_unfused_product.restype = i32
    lib.jfa_unfused_product.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, ctypes.c_float, vp, vp]
    lib.jfa_unfused_softmax_backward.restype = i32
    lib.jfa_unfused_softmax_backward.argtypes = [vp, vp, vp, i64, i64, i32, ctypes.c_float, vp, vp]
    lib.jfa_unfused_apply_transposed.restype = i32
    lib.jfa_unfused_apply_transposed.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, vp]
    lib.jfa_jagged_to_dense.restype = i32
    lib.jfa_jagged_to_dense.argtypes = [vp, vp, i64, i64, i64, ctypes.c_uint32, vp, vp]
    lib.jfa_dense_to_jagged.restype = i32
    lib.jfa_dense_to_jagged.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    lib.jfa_jagged_dense_bmm.restype = i32
    lib.jfa_jagged_dense_bmm.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp, vp]
    lib.jfa_jagged_jagged_bmm.restype = i32
    lib.jfa_jagged_jagged_bmm.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp, vp]
    lib.jfa_jagged_softmax.restype = i32
    lib.jfa_jagged_softmax.argtypes = [vp, vp, i64, i64, i32, vp, vp]
    lib.jfa_jagged_softmax_backward.restype = i32
    lib.jfa_jagged_softmax_backward.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != JFA_OK:
        raise JfaError(status, load().jfa_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _pick(dtype: torch.dtype, bf16_name: str):
    lib = load()
    if dtype == torch.bfloat16:
        return getattr(lib, bf16_name)
    if dtype == torch.float32:
        return getattr(lib, bf16_name + "_f32")
    raise TypeError(f"unsupported dtype {dtype}: bf16 or fp32")


def jfa_forward(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, offsets: torch.Tensor, max_len: int,
                out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None, causal: bool = False
                ) -> Tuple[torch.Tensor, torch.Tensor]:
    """out [sum_B, H, D] (dtype of q) and lse fp32 [H, sum_B]; dispatches on q.dtype (bf16 / fp32).
    causal: row i of a sample attends to rows 0 .. i only (jfa_forward_causal)."""
    sum_B, H, D = q.shape
    assert k.shape == q.shape and v.shape == q.shape and k.dtype == q.dtype and v.dtype == q.dtype
    assert offsets.dtype == torch.int64 and offsets.is_cuda and offsets.dim() == 1
    B = offsets.numel() - 1
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((H, sum_B), dtype=torch.float32, device=q.device)
    fn = _pick(q.dtype, "jfa_forward_causal" if causal else "jfa_forward")
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(offsets), B, max_len, H, D, _ptr(out), _ptr(lse), _stream()))
    return out, lse


def jfa_forward_noalloc(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, offsets: torch.Tensor, max_len: int,
                        out: torch.Tensor, lse: torch.Tensor) -> None:
    """jfa_forward (bf16) with the library's work table in a fixed device array: the call allocates nothing, so `out`
    [sum_B, H, D] and `lse` fp32 [H, sum_B] have to be given.  At most JFA_NOALLOC_MAX_B samples; calls that overlap
    on one GPU race on the shared table."""
    _, H, D = q.shape
    assert q.dtype == torch.bfloat16 and k.dtype == q.dtype and v.dtype == q.dtype
    _check(load().jfa_forward_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(offsets), offsets.numel() - 1, max_len, H, D,
                                      _ptr(out), _ptr(lse), _stream()))


def jfa_backward(q, k, v, out, dout, lse, offsets, max_len: int, dq=None, dk=None, dv=None, delta=None,
                 causal: bool = False):
    """dq, dk, dv [sum_B, H, D] (dtype of q) and delta fp32 [H, sum_B].

    The statistics buffer handed to the library is fp32 [H, sum_B] for fp32 inputs and fp32 [2, H, sum_B] for
    bf16 inputs (plane 0: delta, plane 1: -lse * sqrt(D), which the gradient kernels' score products start from).  A caller-provided `delta` must
    have that size and is returned as it is; otherwise one is allocated here and plane 0 is returned.
    """
    sum_B, H, D = q.shape
    B = offsets.numel() - 1
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(q) if dk is None else dk
    dv = torch.empty_like(q) if dv is None else dv
    planes = 2 if q.dtype == torch.bfloat16 else 1
    stats = torch.empty((planes, H, sum_B), dtype=torch.float32, device=q.device) if delta is None else delta
    fn = _pick(q.dtype, "jfa_backward_causal" if causal else "jfa_backward")
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(dout), _ptr(lse), _ptr(offsets), B, max_len, H, D,
              _ptr(dq), _ptr(dk), _ptr(dv), _ptr(stats), _stream()))
    return dq, dk, dv, (stats[0] if delta is None else delta)


def jfa_forward_cross(q, k, v, offsets_q, offsets_kv, max_len_q: int, max_len_kv: int, out=None, lse=None):
    """Cross attention: out [sum_Bq, H, D] and lse fp32 [H, sum_Bq]; q rows follow offsets_q, k and v rows offsets_kv."""
    sum_Bq, H, D = q.shape
    assert k.shape == v.shape and k.shape[1:] == q.shape[1:] and k.dtype == q.dtype == v.dtype
    assert offsets_q.numel() == offsets_kv.numel()
    B = offsets_q.numel() - 1
    out = torch.empty_like(q) if out is None else out
    lse = torch.empty((H, sum_Bq), dtype=torch.float32, device=q.device) if lse is None else lse
    fn = _pick(q.dtype, "jfa_forward_cross")
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(offsets_q), _ptr(offsets_kv), B, max_len_q, max_len_kv, H, D,
              _ptr(out), _ptr(lse), _stream()))
    return out, lse


def jfa_backward_cross(q, k, v, out, dout, lse, offsets_q, offsets_kv, max_len_q: int, max_len_kv: int,
                       dq=None, dk=None, dv=None, delta=None):
    """dq [sum_Bq, H, D], dk, dv [sum_Bkv, H, D] and delta fp32 [H, sum_Bq] (statistics buffer as in jfa_backward)."""
    sum_Bq, H, D = q.shape
    B = offsets_q.numel() - 1
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    planes = 2 if q.dtype == torch.bfloat16 else 1
    stats = torch.empty((planes, H, sum_Bq), dtype=torch.float32, device=q.device) if delta is None else delta
    fn = _pick(q.dtype, "jfa_backward_cross")
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(dout), _ptr(lse), _ptr(offsets_q), _ptr(offsets_kv), B,
              max_len_q, max_len_kv, H, D, _ptr(dq), _ptr(dk), _ptr(dv), _ptr(stats), _stream()))
    return dq, dk, dv, (stats[0] if delta is None else delta)


def jfa_build_schedule(offsets: torch.Tensor, block_rows: int):
    """(order int32 [B], tile_start int32 [B+1]) as computed on the device."""
    B = offsets.numel() - 1
    order = torch.empty((max(B, 1),), dtype=torch.int32, device=offsets.device)
    tile_start = torch.empty((B + 1,), dtype=torch.int32, device=offsets.device)
    _check(load().jfa_build_schedule(_ptr(offsets), B, block_rows, _ptr(order), _ptr(tile_start), _stream()))
    return order[:B], tile_start


def jfa_square_offsets(offsets: torch.Tensor) -> torch.Tensor:
    """int64 [B+1] on the device: offsets of the jagged square array, sq[b] = sum of L_c^2 over c < b."""
    B = offsets.numel() - 1
    sq = torch.empty((B + 1,), dtype=torch.int64, device=offsets.device)
    _check(load().jfa_square_offsets(_ptr(offsets), B, _ptr(sq), _stream()))
    return sq


def jfa_unfused_scores(q, k, offsets, sq_offsets, max_len: int, scores: torch.Tensor):
    """scores fp32 [H, sq[B]] = q k^T / sqrt(D) per sample and head (the caller sizes `scores` from its lengths)."""
    _, H, D = q.shape
    _check(load().jfa_unfused_scores(_ptr(q), _ptr(k), _ptr(offsets), _ptr(sq_offsets), offsets.numel() - 1, max_len,
                                     H, D, _ptr(scores), _stream()))
    return scores


def jfa_unfused_softmax(offsets, sq_offsets, max_len: int, H: int, scores: torch.Tensor):
    """Row softmax of every L_b x L_b block of `scores`, in place."""
    _check(load().jfa_unfused_softmax(_ptr(offsets), _ptr(sq_offsets), offsets.numel() - 1, max_len, H,
                                      _ptr(scores), _stream()))
    return scores


def jfa_unfused_apply(probs, v, offsets, sq_offsets, max_len: int, out: Optional[torch.Tensor] = None):
    """out [sum_B, H, D] (bf16) = P v per sample and head."""
    _, H, D = v.shape
    out = torch.empty_like(v) if out is None else out
    _check(load().jfa_unfused_apply(_ptr(probs), _ptr(v), _ptr(offsets), _ptr(sq_offsets), offsets.numel() - 1,
                                    max_len, H, D, _ptr(out), _stream()))
    return out


def jfa_unfused_product(a, b, offsets, sq_offsets, max_len: int, scale: float, out: torch.Tensor):
    """out fp32 [H, sq[B]] = scale * a b^T per sample and head (the scaled product behind scores and dP)."""
    _, H, D = a.shape
    _check(load().jfa_unfused_product(_ptr(a), _ptr(b), _ptr(offsets), _ptr(sq_offsets), offsets.numel() - 1, max_len,
                                      H, D, scale, _ptr(out), _stream()))
    return out


def jfa_unfused_softmax_backward(probs, offsets, sq_offsets, max_len: int, H: int, scale: float, dprobs: torch.Tensor):
    """dprobs <- scale * P o (dprobs - rowsum(P o dprobs)), row by row, in place."""
    _check(load().jfa_unfused_softmax_backward(_ptr(probs), _ptr(offsets), _ptr(sq_offsets), offsets.numel() - 1, max_len,
                                               H, scale, _ptr(dprobs), _stream()))
    return dprobs


def jfa_unfused_apply_transposed(array, x, offsets, sq_offsets, max_len: int, out: Optional[torch.Tensor] = None):
    """out [sum_B, H, D] (bf16): out_j = sum_i array[i, j] x_i per sample and head."""
    _, H, D = x.shape
    out = torch.empty_like(x) if out is None else out
    _check(load().jfa_unfused_apply_transposed(_ptr(array), _ptr(x), _ptr(offsets), _ptr(sq_offsets), offsets.numel() - 1,
                                               max_len, H, D, _ptr(out), _stream()))
    return out


def _row_bytes(t: torch.Tensor, lead: int) -> int:
    assert t.is_contiguous()
    n = t.element_size()
    for d in t.shape[lead:]:
        n *= d
    return n


def _pad_pattern(dtype: torch.dtype, pad: float) -> int:
    """The 32-bit pattern that fills padded rows: the pad value's bits, twice for 16-bit types."""
    one = torch.tensor([pad], dtype=dtype)
    if one.element_size() == 4:
        return int(one.view(torch.int32).item()) & 0xFFFFFFFF
    if one.element_size() == 2:
        bits = int(one.view(torch.int16).item()) & 0xFFFF
        return bits | (bits << 16)
    raise ValueError(f"pad value for {dtype}: only 2- and 4-byte element types")


def jfa_jagged_to_dense(values: torch.Tensor, offsets: torch.Tensor, max_len: int, pad: float = 0.0,
                        dense: Optional[torch.Tensor] = None) -> torch.Tensor:
    """dense [B, max_len, ...] from values [sum_B, ...]: rows i >= L_b of each sample hold `pad`."""
    B = offsets.numel() - 1
    if dense is None:
        dense = torch.empty((B, max_len) + tuple(values.shape[1:]), dtype=values.dtype, device=values.device)
    _check(load().jfa_jagged_to_dense(_ptr(values), _ptr(offsets), B, max_len, _row_bytes(values, 1),
                                      _pad_pattern(values.dtype, pad), _ptr(dense), _stream()))
    return dense


def jfa_dense_to_jagged(dense: torch.Tensor, offsets: torch.Tensor, values: torch.Tensor) -> torch.Tensor:
    """values[offsets[b] + i] = dense[b, i] for i < L_b; `values` [sum_B, ...] is caller-provided (the host does not know sum_B)."""
    B, max_len = dense.shape[0], dense.shape[1]
    assert offsets.numel() - 1 == B and _row_bytes(dense, 2) == _row_bytes(values, 1)
    _check(load().jfa_dense_to_jagged(_ptr(dense), _ptr(offsets), B, max_len, _row_bytes(dense, 2), _ptr(values), _stream()))
    return values


def jfa_jagged_dense_bmm(x: torch.Tensor, w: torch.Tensor, offsets: torch.Tensor, max_len: int,
                         out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out [sum_B, T] = x [sum_B, D] times w [B, D, T], sample by sample (bf16)."""
    B, D, T = w.shape
    assert offsets.numel() - 1 == B and x.shape[1] == D
    out = torch.empty((x.shape[0], T), dtype=x.dtype, device=x.device) if out is None else out
    _check(load().jfa_jagged_dense_bmm(_ptr(x), _ptr(w), _ptr(offsets), B, max_len, D, T, _ptr(out), _stream()))
    return out


def jfa_jagged_jagged_bmm(x: torch.Tensor, y: torch.Tensor, offsets: torch.Tensor, max_len: int,
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out [B, D, T] = per-sample x^T y for x [sum_B, D], y [sum_B, T] (bf16)."""
    B, D, T = offsets.numel() - 1, x.shape[1], y.shape[1]
    out = torch.empty((B, D, T), dtype=x.dtype, device=x.device) if out is None else out
    _check(load().jfa_jagged_jagged_bmm(_ptr(x), _ptr(y), _ptr(offsets), B, max_len, D, T, _ptr(out), _stream()))
    return out


def jfa_jagged_softmax(x: torch.Tensor, offsets: torch.Tensor, max_len: int, y: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Softmax along each sample's rows, per column, of x [sum_B, D] (bf16)."""
    y = torch.empty_like(x) if y is None else y
    _check(load().jfa_jagged_softmax(_ptr(x), _ptr(offsets), offsets.numel() - 1, max_len, x.shape[1], _ptr(y), _stream()))
    return y


def jfa_jagged_softmax_backward(y: torch.Tensor, dy: torch.Tensor, offsets: torch.Tensor, max_len: int,
                                dx: Optional[torch.Tensor] = None) -> torch.Tensor:
    dx = torch.empty_like(y) if dx is None else dx
    _check(load().jfa_jagged_softmax_backward(_ptr(y), _ptr(dy), _ptr(offsets), offsets.numel() - 1, max_len, y.shape[1],
                                              _ptr(dx), _stream()))
    return dx


def jfa_check_offsets(offsets: torch.Tensor, max_len: int) -> int:
    flags = ctypes.c_int(-1)
    _check(load().jfa_check_offsets(_ptr(offsets), offsets.numel() - 1, max_len, _stream(), ctypes.byref(flags)))
    return flags.value


def jfa_workspace_bytes(B: int, max_len: int, H: int, D: int, backward: bool = False) -> int:
    return int(load().jfa_workspace_bytes(B, max_len, H, D, 1 if backward else 0))


def jfa_timing_enable(on: bool) -> None:
    _check(load().jfa_timing_enable(1 if on else 0))


def jfa_timing_read(capacity: int = 16):
    """{kernel name: (total milliseconds, launches)} since the last read; waits for the recorded events."""
    names = (ctypes.c_char_p * capacity)()
    ms = (ctypes.c_float * capacity)()
    cnt = (ctypes.c_int * capacity)()
    n = load().jfa_timing_read(capacity, names, ms, cnt)
    if n < 0:
        _check(n)
    return {names[i].decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}


def jfa_version() -> int:
    return int(load().jfa_version())


def jfa_last_error() -> str:
    return load().jfa_last_error().decode()

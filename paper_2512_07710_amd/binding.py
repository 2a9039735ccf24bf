"""ctypes binding of libmoe355.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see
include/moe355.h); tensors are torch CUDA tensors used purely as device
memory.  There is no CPU fallback: if the shared library is missing or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe355.so")
_lib: Optional[ctypes.CDLL] = None

EXPORTS = ("moe_create", "moe_destroy", "moe_strerror", "moe_route", "moe_route_replay", "moe_route_replay_noalloc",
           "moe_route_replay_ids",
           "moe_check_ids", "moe_quantize_fp8", "moe_quantize_weights_fp8", "moe_linear_fp8", "moe_expert_ffn_fp8",
           "moe_expert_ffn_fp8_gather", "moe_combine", "moe_balance_lengths", "moe_debug_copy_hidden",
           "moe_probe_copy", "moe_probe_fp8_mfma", "moe_profile_enable", "moe_profile_read", "moe_version")


class MoEError(RuntimeError):
    pass


class _Dims(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("E", ctypes.c_int32),
                ("k", ctypes.c_int32), ("F", ctypes.c_int32)]


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libmoe355.so (built by paper_2512_07710_amd.build); raises if it is not there."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise MoEError(f"{p} not found: build it with `python -m paper_2512_07710_amd.build` "
                       "(there is no fallback implementation)")
    lib = ctypes.CDLL(p)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.moe_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(_Dims), vp]
    lib.moe_destroy.argtypes = [vp]
    lib.moe_strerror.argtypes = [ctypes.c_int]
    lib.moe_strerror.restype = ctypes.c_char_p
    lib.moe_version.restype = ctypes.c_char_p
    lib.moe_route.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.moe_route_replay.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.moe_route_replay_ids.argtypes = [vp] * 9
    lib.moe_route_replay_noalloc.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.moe_check_ids.argtypes = [vp]
    lib.moe_quantize_weights_fp8.argtypes = [vp, vp, i64, i32, vp, vp]
    lib.moe_linear_fp8.argtypes = [vp, vp, vp, i32, i32, vp, vp, i32, vp]
    lib.moe_quantize_fp8.argtypes = [vp, vp, i64, i32, i32, vp, i32, vp, vp]
    lib.moe_expert_ffn_fp8.argtypes = [vp] * 11
    lib.moe_expert_ffn_fp8_gather.argtypes = [vp] * 12
    lib.moe_combine.argtypes = [vp] * 6
    lib.moe_balance_lengths.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp]
    lib.moe_debug_copy_hidden.argtypes = [vp, vp, vp]
    lib.moe_probe_copy.argtypes = [vp, vp, vp, i64]
    lib.moe_probe_fp8_mfma.argtypes = [vp, i32, i32, i32, vp]
    lib.moe_profile_enable.argtypes = [vp, i32]
    lib.moe_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
    for name in EXPORTS:
        if name not in ("moe_strerror", "moe_version"):
            getattr(lib, name).restype = ctypes.c_int
    if path is None:
        _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise MoEError(f"{what} failed: {load_library().moe_strerror(rc).decode()} ({rc})")


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise MoEError("expected a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise MoEError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def moe_create(T: int, d: int, E: int, k: int, F: int, stream: Optional[torch.cuda.Stream] = None) -> int:
    """Returns an opaque context handle bound to `stream` (default: torch's current stream)."""
    lib = load_library()
    s = stream if stream is not None else torch.cuda.current_stream()
    dims = _Dims(T, d, E, k, F)
    h = ctypes.c_void_p()
    _check(lib.moe_create(ctypes.byref(h), ctypes.byref(dims), ctypes.c_void_p(s.cuda_stream)), "moe_create")
    return h.value


def moe_destroy(ctx: int) -> None:
    _check(load_library().moe_destroy(ctx), "moe_destroy")


def moe_version() -> str:
    return load_library().moe_version().decode()


def moe_route(ctx, x, W_router, sel_bias, k, topk_idx, topk_w, offsets, perm, inv_perm) -> None:
    _check(load_library().moe_route(ctx, _ptr(x, torch.bfloat16), _ptr(W_router, torch.float32),
                                    _ptr(sel_bias, torch.float32), k, _ptr(topk_idx, torch.int32),
                                    _ptr(topk_w, torch.float32), _ptr(offsets, torch.int32),
                                    _ptr(perm, torch.int32), _ptr(inv_perm, torch.int32)), "moe_route")


def moe_route_replay(ctx, x, logged_idx, logged_w, topk_idx, topk_w, offsets, perm, inv_perm) -> None:
    _check(load_library().moe_route_replay(ctx, _ptr(x), _ptr(logged_idx, torch.int32),
                                           _ptr(logged_w, torch.float32), _ptr(topk_idx, torch.int32),
                                           _ptr(topk_w, torch.float32), _ptr(offsets, torch.int32),
                                           _ptr(perm, torch.int32), _ptr(inv_perm, torch.int32)),
           "moe_route_replay")


def moe_route_replay_noalloc(stream, T, E, k, logged_idx, logged_w, topk_idx, topk_w, offsets, perm, inv_perm,
                             id_flags=None) -> None:
    """`stream`: a torch.cuda.Stream or None for torch's current stream."""
    s = stream if stream is not None else torch.cuda.current_stream()
    i32 = torch.int32
    _check(load_library().moe_route_replay_noalloc(ctypes.c_void_p(s.cuda_stream), T, E, k, _ptr(logged_idx, i32),
                                                   _ptr(logged_w, torch.float32), _ptr(topk_idx, i32),
                                                   _ptr(topk_w, torch.float32), _ptr(offsets, i32), _ptr(perm, i32),
                                                   _ptr(inv_perm, i32), _ptr(id_flags, i32)),
           "moe_route_replay_noalloc")


def moe_check_ids(ctx) -> int:
    """Returns the raw status (0 or MOE_EBADIDS) after synchronising the context's stream."""
    return load_library().moe_check_ids(ctx)


def moe_route_replay_ids(ctx, x, W_router, logged_idx, topk_idx, topk_w, offsets, perm, inv_perm) -> None:
    i32 = torch.int32
    _check(load_library().moe_route_replay_ids(ctx, _ptr(x, torch.bfloat16), _ptr(W_router, torch.float32),
                                               _ptr(logged_idx, i32), _ptr(topk_idx, i32),
                                               _ptr(topk_w, torch.float32), _ptr(offsets, i32), _ptr(perm, i32),
                                               _ptr(inv_perm, i32)), "moe_route_replay_ids")


def moe_quantize_weights_fp8(ctx, w, rows, cols, q, scales) -> None:
    _check(load_library().moe_quantize_weights_fp8(ctx, _ptr(w, torch.bfloat16), rows, cols, _ptr(q, torch.uint8),
                                                   _ptr(scales, torch.float32)), "moe_quantize_weights_fp8")


def moe_linear_fp8(ctx, xq, xs, rows, K, Wq, ws, NOUT, y) -> None:
    u8, f32 = torch.uint8, torch.float32
    _check(load_library().moe_linear_fp8(ctx, _ptr(xq, u8), _ptr(xs, f32), rows, K, _ptr(Wq, u8), _ptr(ws, f32),
                                         NOUT, _ptr(y, f32)), "moe_linear_fp8")


def moe_quantize_fp8(ctx, x, rows_in, cols, block, dst_rows, fanout, q, scales) -> None:
    _check(load_library().moe_quantize_fp8(ctx, _ptr(x, torch.bfloat16), rows_in, cols, block,
                                           _ptr(dst_rows, torch.int32), fanout, _ptr(q, torch.uint8),
                                           _ptr(scales, torch.float32)), "moe_quantize_fp8")


def moe_expert_ffn_fp8(ctx, xq_perm, xs_perm, offsets, W1, W3, W2, s1, s3, s2, y_perm) -> None:
    u8, f32 = torch.uint8, torch.float32
    _check(load_library().moe_expert_ffn_fp8(ctx, _ptr(xq_perm, u8), _ptr(xs_perm, f32),
                                             _ptr(offsets, torch.int32), _ptr(W1, u8), _ptr(W3, u8),
                                             _ptr(W2, u8), _ptr(s1, f32), _ptr(s3, f32), _ptr(s2, f32),
                                             _ptr(y_perm, f32)), "moe_expert_ffn_fp8")


def moe_expert_ffn_fp8_gather(ctx, xq_tok, xs_tok, perm, offsets, W1, W3, W2, s1, s3, s2, y_perm) -> None:
    u8, f32 = torch.uint8, torch.float32
    _check(load_library().moe_expert_ffn_fp8_gather(ctx, _ptr(xq_tok, u8), _ptr(xs_tok, f32),
                                                    _ptr(perm, torch.int32),
                                                    _ptr(offsets, torch.int32), _ptr(W1, u8), _ptr(W3, u8),
                                                    _ptr(W2, u8), _ptr(s1, f32), _ptr(s3, f32), _ptr(s2, f32),
                                                    _ptr(y_perm, f32)), "moe_expert_ffn_fp8_gather")


def moe_combine(ctx, y_perm, inv_perm, topk_w, y, y_f32=None) -> None:
    _check(load_library().moe_combine(ctx, _ptr(y_perm, torch.float32), _ptr(inv_perm, torch.int32),
                                      _ptr(topk_w, torch.float32), _ptr(y, torch.bfloat16),
                                      _ptr(y_f32, torch.float32)), "moe_combine")


def moe_balance_lengths(pred_len, n_groups: int, equal_count: bool = True):
    """Host-side length-based load balancing: pred_len is a CPU int64 tensor [n]; returns CPU tensors
    (group_of int32 [n], order int64 [n], bounds int64 [n_groups+1], totals int64 [n_groups])."""
    if pred_len.is_cuda or pred_len.dtype != torch.int64 or not pred_len.is_contiguous() or pred_len.dim() != 1:
        raise MoEError("expected a contiguous 1-D CPU int64 tensor")
    if n_groups < 1:
        raise MoEError("n_groups must be at least 1")
    n = pred_len.numel()
    group_of = torch.empty(n, dtype=torch.int32)
    order = torch.empty(n, dtype=torch.int64)
    bounds = torch.empty(n_groups + 1, dtype=torch.int64)
    totals = torch.empty(n_groups, dtype=torch.int64)
    _check(load_library().moe_balance_lengths(pred_len.data_ptr(), n, n_groups, 1 if equal_count else 0,
                                              group_of.data_ptr(), order.data_ptr(), bounds.data_ptr(),
                                              totals.data_ptr()), "moe_balance_lengths")
    return group_of, order, bounds, totals


def moe_debug_copy_hidden(ctx, hq_out, hs_out) -> None:
    _check(load_library().moe_debug_copy_hidden(ctx, _ptr(hq_out, torch.uint8), _ptr(hs_out, torch.float32)),
           "moe_debug_copy_hidden")


def moe_probe_copy(ctx, src, dst, nbytes: int) -> None:
    _check(load_library().moe_probe_copy(ctx, _ptr(src), _ptr(dst), nbytes), "moe_probe_copy")


def moe_probe_fp8_mfma(ctx, blocks: int, steps: int, scaled: bool, sink) -> None:
    _check(load_library().moe_probe_fp8_mfma(ctx, blocks, steps, 1 if scaled else 0, _ptr(sink, torch.float32)),
           "moe_probe_fp8_mfma")


def moe_profile_enable(ctx, on: bool) -> None:
    _check(load_library().moe_profile_enable(ctx, 1 if on else 0), "moe_profile_enable")


def moe_profile_read(ctx):
    """(mean ms of the gate/up GEMM, mean ms of the down GEMM, recorded calls); synchronises."""
    ms = (ctypes.c_float * 2)()
    n = ctypes.c_int32()
    _check(load_library().moe_profile_read(ctx, ms, ctypes.byref(n)), "moe_profile_read")
    return float(ms[0]), float(ms[1]), int(n.value)

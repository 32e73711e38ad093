"""Thin Python binding of include/moe_train.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C

import torch

from .binding import (MoeError, Shape, _check, _ptr, _stream, lib, moe_max_rows,
                      moe_workspace_bytes)

_ready = False


def _lib():
    global _ready
    L = lib()
    if not _ready:
        sp, vp, i32 = C.POINTER(Shape), C.c_void_p, C.c_int32
        L.moe_backward_workspace_bytes.restype = C.c_size_t
        L.moe_backward_workspace_bytes.argtypes = [sp]
        L.moe_layer_backward.restype = C.c_int
        L.moe_layer_backward.argtypes = [sp, vp, vp, vp, i32] + [vp] * 20
        L.moe_layer_backward_chunked.restype = C.c_int
        L.moe_layer_backward_chunked.argtypes = [sp, i32, vp, vp, vp, i32] + [vp] * 20
        L.moe_layer_forward_keep.restype = C.c_int
        L.moe_layer_forward_keep.argtypes = [sp, vp, vp, vp, i32] + [vp] * 17
        _ready = True
    return L


def moe_backward_workspace_bytes(s: Shape) -> int:
    return int(_lib().moe_backward_workspace_bytes(C.byref(s)))


def _need(t: torch.Tensor, dtype, numel: int, name: str) -> None:
    if t.dtype != dtype or t.numel() < numel:
        raise MoeError(f"{name}: need {numel} elements of {dtype}, got {t.numel()} of {t.dtype}")


def moe_layer_forward_keep(s: Shape, x, Wgp, gate_bias, bias_token_stride, W1p, b1, W2p, b2, expert_idx,
                           gate, counts, offsets, slot_of, src_of, xe, ye, pre, hid, y, workspace,
                           stream=None) -> None:
    rows = moe_max_rows(s)
    T, d, E, h, k = s.T, s.d_model, s.E, s.d_ff, s.k
    _need(x, torch.bfloat16, T * d, "x")
    _need(expert_idx, torch.int32, T * k, "expert_idx")
    _need(gate, torch.float32, T * k, "gate")
    _need(counts, torch.int32, E, "counts")
    _need(offsets, torch.int32, E + 1, "offsets")
    _need(slot_of, torch.int32, T * k, "slot_of")
    _need(src_of, torch.int32, rows, "src_of")
    _need(xe, torch.bfloat16, rows * d, "xe")
    _need(ye, s.ye_dtype, rows * d, "ye")
    _need(pre, torch.float16, rows * h, "pre")
    _need(hid, torch.float16, rows * h, "hid")
    _need(y, torch.float32, T * d, "y")
    _need(workspace, torch.uint8, moe_workspace_bytes(s, 1), "workspace")
    _check(_lib().moe_layer_forward_keep(C.byref(s), _ptr(x), _ptr(Wgp), _ptr(gate_bias),
                                         bias_token_stride, _ptr(W1p), _ptr(b1), _ptr(W2p), _ptr(b2),
                                         _ptr(expert_idx), _ptr(gate), _ptr(counts), _ptr(offsets),
                                         _ptr(slot_of), _ptr(src_of), _ptr(xe), _ptr(ye), _ptr(pre),
                                         _ptr(hid), _ptr(y), _ptr(workspace), _stream(stream)))


def moe_layer_backward(s: Shape, x, Wgp, gate_bias, bias_token_stride, W1, W2, W1p, expert_idx, gate,
                       offsets, slot_of, src_of, xe, ye, pre, hid, dy, dx, dWg, dW1, dW2, dgate, workspace,
                       stream=None, n_chunks: int = 1) -> None:
    """n_chunks = 1: moe_layer_backward; otherwise moe_layer_backward_chunked."""
    rows = moe_max_rows(s)
    T, d, E, h, k = s.T, s.d_model, s.E, s.d_ff, s.k
    _need(x, torch.bfloat16, T * d, "x")
    _need(W1, torch.bfloat16, E * d * h, "W1")
    _need(W2, torch.bfloat16, E * d * h, "W2")
    _need(expert_idx, torch.int32, T * k, "expert_idx")
    _need(gate, torch.float32, T * k, "gate")
    _need(offsets, torch.int32, E + 1, "offsets")
    _need(slot_of, torch.int32, T * k, "slot_of")
    _need(src_of, torch.int32, rows, "src_of")
    _need(xe, torch.bfloat16, rows * d, "xe")
    _need(ye, s.ye_dtype, rows * d, "ye")
    if pre is not None:
        _need(pre, torch.float16, rows * h, "pre")
    if hid is not None:
        _need(hid, torch.float16, rows * h, "hid")
    _need(dy, torch.float32, T * d, "dy")
    _need(dx, torch.float32, T * d, "dx")
    _need(dWg, torch.float32, d * E, "dWg")
    _need(dW1, torch.float32, E * d * h, "dW1")
    _need(dW2, torch.float32, E * d * h, "dW2")
    _need(dgate, torch.float32, T * k, "dgate")
    _need(workspace, torch.uint8, moe_backward_workspace_bytes(s), "workspace")
    tail = (_ptr(x), _ptr(Wgp), _ptr(gate_bias), bias_token_stride, _ptr(W1), _ptr(W2), _ptr(W1p),
            _ptr(expert_idx), _ptr(gate), _ptr(offsets), _ptr(slot_of), _ptr(src_of), _ptr(xe), _ptr(ye),
            _ptr(pre), _ptr(hid), _ptr(dy), _ptr(dx), _ptr(dWg), _ptr(dW1), _ptr(dW2), _ptr(dgate),
            _ptr(workspace), _stream(stream))
    if n_chunks == 1:
        _check(_lib().moe_layer_backward(C.byref(s), *tail))
    else:
        _check(_lib().moe_layer_backward_chunked(C.byref(s), n_chunks, *tail))

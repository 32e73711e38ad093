"""Thin Python binding of include/moe_comm.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional

import torch

from .binding import MoeError, Shape, _check, _ptr, _stream, lib

ALL_TO_ALL, ALLREDUCE = 0, 1
ARRIVAL_ORDER, PRIORITY = 0, 1

_ready = False


class CommRecord(C.Structure):
    """moe_comm_record."""
    _fields_ = [("op", C.c_int64), ("micro", C.c_int32), ("kind", C.c_int32), ("bytes", C.c_int64),
                ("ready_seq", C.c_int64), ("issue_seq", C.c_int64), ("posted_ns", C.c_int64),
                ("launched_ns", C.c_int64), ("done_ns", C.c_int64)]


def _lib():
    global _ready
    L = lib()
    if not _ready:
        sp, vp, i32, i64 = C.POINTER(Shape), C.c_void_p, C.c_int32, C.c_int64
        L.moe_comm_create.restype = C.c_int
        L.moe_comm_create.argtypes = [C.POINTER(vp), i32, i32, i32]
        L.moe_comm_destroy.restype = C.c_int
        L.moe_comm_destroy.argtypes = [vp]
        L.moe_comm_submit.restype = C.c_int
        L.moe_comm_submit.argtypes = [vp, i32, vp, vp, i64, i64, i64, i32, C.POINTER(i64)]
        L.moe_comm_post.restype = C.c_int
        L.moe_comm_post.argtypes = [vp, i64, i32, i32, vp]
        L.moe_comm_wait.restype = C.c_int
        L.moe_comm_wait.argtypes = [vp, i64, i32, vp, i32]
        for name in ("moe_comm_hold", "moe_comm_pause"):
            getattr(L, name).restype = C.c_int
            getattr(L, name).argtypes = [vp, i32]
        L.moe_comm_release.restype = C.c_int
        L.moe_comm_release.argtypes = [vp, i64]
        L.moe_comm_finish.restype = C.c_int
        L.moe_comm_finish.argtypes = [vp, i64, i32, C.POINTER(C.c_float)]
        L.moe_comm_log.restype = i32
        L.moe_comm_log.argtypes = [vp, C.POINTER(CommRecord), i32]
        L.moe_padded_workspace_bytes.restype = C.c_size_t
        L.moe_padded_workspace_bytes.argtypes = [sp, i32]
        L.moe_layer_padded.restype = C.c_int
        L.moe_layer_padded.argtypes = [sp, i32, vp, i32, vp, vp, vp, i32] + [vp] * 16
        _ready = True
    return L


def moe_comm_create(policy: int, link_blocks: int, depth: int = 1) -> C.c_void_p:
    h = C.c_void_p()
    _check(_lib().moe_comm_create(C.byref(h), policy, link_blocks, depth))
    return h


def moe_comm_destroy(c) -> None:
    _check(_lib().moe_comm_destroy(c))


def moe_comm_submit(c, kind: int, src: torch.Tensor, dst: torch.Tensor, slabs: int, rows: int,
                    row_bytes: int, n_micro: int) -> int:
    nbytes = slabs * rows * row_bytes
    for t, name in ((src, "src"), (dst, "dst")):
        if not t.is_cuda or not t.is_contiguous() or t.numel() * t.element_size() < nbytes:
            raise MoeError(f"{name}: need a contiguous device tensor of {nbytes} bytes")
    op = C.c_int64()
    _check(_lib().moe_comm_submit(c, kind, _ptr(src), _ptr(dst), slabs, rows, row_bytes, n_micro,
                                  C.byref(op)))
    return int(op.value)


def moe_comm_post(c, op: int, first: int, count: int, producer_stream=None) -> None:
    _check(_lib().moe_comm_post(c, op, first, count, _stream(producer_stream)))


def moe_comm_wait(c, op: int, micro: int = -1, consumer_stream=None, timeout_ms: int = 20000) -> None:
    _check(_lib().moe_comm_wait(c, op, micro, _stream(consumer_stream), timeout_ms))


def moe_comm_hold(c, on: bool) -> None:
    _check(_lib().moe_comm_hold(c, 1 if on else 0))


def moe_comm_pause(c, on: bool) -> None:
    _check(_lib().moe_comm_pause(c, 1 if on else 0))


def moe_comm_release(c, op: int) -> None:
    _check(_lib().moe_comm_release(c, op))


def moe_comm_finish(c, op: int, timeout_ms: int = 20000) -> float:
    """Returns the operation's completion time on the device in milliseconds."""
    ms = C.c_float()
    _check(_lib().moe_comm_finish(c, op, timeout_ms, C.byref(ms)))
    return float(ms.value)


def moe_comm_log(c, cap: int = 65536) -> List[dict]:
    buf = (CommRecord * cap)()
    n = _lib().moe_comm_log(c, buf, cap)
    return [dict(op=r.op, micro=r.micro, kind=r.kind, bytes=r.bytes, ready_seq=r.ready_seq,
                 issue_seq=r.issue_seq, posted_ns=r.posted_ns, launched_ns=r.launched_ns,
                 done_ns=r.done_ns) for r in buf[:n]]


def moe_padded_workspace_bytes(s: Shape, n_micro: int) -> int:
    return int(_lib().moe_padded_workspace_bytes(C.byref(s), n_micro))


def _need(t: torch.Tensor, dtype, numel: int, name: str) -> None:
    if t.dtype != dtype or t.numel() < numel:
        raise MoeError(f"{name}: need {numel} elements of {dtype}, got {t.numel()} of {t.dtype}")


def moe_layer_padded(s: Shape, n_micro: int, link: Optional[C.c_void_p], link_blocks: int, x, Wgp,
                     gate_bias, bias_token_stride, W1p, b1, W2p, b2, expert_idx, gate, counts, slot_of,
                     src_of, xs, xr, ys, yr, y, workspace, stream=None) -> None:
    slots = s.E * s.capacity
    _need(x, s.torch_dtype, s.T * s.d_model, "x")
    _need(expert_idx, torch.int32, s.T * s.k, "expert_idx")
    _need(gate, torch.float32, s.T * s.k, "gate")
    _need(counts, torch.int32, s.E, "counts")
    _need(slot_of, torch.int32, s.T * s.k, "slot_of")
    _need(src_of, torch.int32, slots, "src_of")
    _need(xs, s.torch_dtype, slots * s.d_model, "xs")
    _need(xr, s.torch_dtype, slots * s.d_model, "xr")
    _need(ys, s.ye_dtype, slots * s.d_model, "ys")
    _need(yr, s.ye_dtype, slots * s.d_model, "yr")
    _need(y, torch.float32, s.T * s.d_model, "y")
    _need(workspace, torch.uint8, moe_padded_workspace_bytes(s, n_micro), "workspace")
    _check(_lib().moe_layer_padded(C.byref(s), n_micro, link, link_blocks, _ptr(x), _ptr(Wgp),
                                   _ptr(gate_bias), bias_token_stride, _ptr(W1p), _ptr(b1), _ptr(W2p),
                                   _ptr(b2), _ptr(expert_idx), _ptr(gate), _ptr(counts), _ptr(slot_of),
                                   _ptr(src_of), _ptr(xs), _ptr(xr), _ptr(ys), _ptr(yr), _ptr(y),
                                   _ptr(workspace), _stream(stream)))

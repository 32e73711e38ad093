"""Thin Python binding of include/moe_sched.h (argument marshalling only).

Device calls take torch tensors (int32 / uint32-as-int32 / uint64-as-int64 storage);
host calls take numpy arrays or sequences and return numpy arrays.
"""
from __future__ import annotations

import ctypes as C
from typing import Sequence, Tuple

import numpy as np
import torch

from .binding import MoeError, _check, _ptr, _stream, lib

_ready = False


class PathShape(C.Structure):
    _fields_ = [("L", C.c_int32), ("E", C.c_int32), ("k", C.c_int32), ("l", C.c_int32)]


def _lib():
    global _ready
    L = lib()
    if not _ready:
        i32, vp, u64 = C.c_int32, C.c_void_p, C.c_uint64
        ps = C.POINTER(PathShape)
        L.moe_path_count.restype = C.c_int64
        L.moe_path_count.argtypes = [ps]
        L.moe_path_profile.restype = C.c_int
        L.moe_path_profile.argtypes = [ps, vp, i32, vp, vp]
        L.moe_path_finalize.restype = C.c_int
        L.moe_path_finalize.argtypes = [ps, vp, vp, vp, vp]
        L.moe_popularity_estimate.restype = C.c_int
        L.moe_popularity_estimate.argtypes = [ps, vp, i32, vp, vp, vp, vp]
        L.moe_devices_for_expert.restype = C.c_double
        L.moe_devices_for_expert.argtypes = [u64, i32, i32]
        L.moe_schedule_experts.restype = C.c_int
        L.moe_schedule_experts.argtypes = [i32, i32, vp, u64, vp, i32, vp, vp, vp, vp]
        L.moe_top_lists_identical.restype = i32
        L.moe_top_lists_identical.argtypes = [i32, i32, vp, vp]
        L.moe_schedule_layer.restype = C.c_int
        L.moe_schedule_layer.argtypes = [i32, i32, i32, i32, vp, vp, i32, vp, vp, vp, vp, vp]
        _ready = True
    return L


def _need(t: torch.Tensor, dtype, numel: int, name: str) -> None:
    if t.dtype != dtype or t.numel() < numel:
        raise MoeError(f"{name}: need {numel} elements of {dtype}, got {t.numel()} of {t.dtype}")


def moe_path_count(s: PathShape) -> int:
    return int(_lib().moe_path_count(C.byref(s)))


def moe_path_profile(s: PathShape, sel: torch.Tensor, T: int, counts: torch.Tensor, stream=None) -> None:
    _need(sel, torch.int32, s.L * T * s.k, "sel")
    _need(counts, torch.int32, (s.L - s.l) * moe_path_count(s) * s.E, "counts")
    _check(_lib().moe_path_profile(C.byref(s), _ptr(sel), T, _ptr(counts), _stream(stream)))


def moe_path_finalize(s: PathShape, counts: torch.Tensor, top_expert: torch.Tensor,
                      top_prob: torch.Tensor, stream=None) -> None:
    rows = (s.L - s.l) * moe_path_count(s)
    _need(counts, torch.int32, rows * s.E, "counts")
    _need(top_expert, torch.int32, rows * s.k, "top_expert")
    _need(top_prob, torch.int64, rows * s.k, "top_prob")
    _check(_lib().moe_path_finalize(C.byref(s), _ptr(counts), _ptr(top_expert), _ptr(top_prob),
                                    _stream(stream)))


def moe_popularity_estimate(s: PathShape, sel_hist: torch.Tensor, N_t: int, top_expert: torch.Tensor,
                            top_prob: torch.Tensor, S: torch.Tensor, stream=None) -> None:
    rows = moe_path_count(s)
    _need(sel_hist, torch.int32, s.l * N_t * s.k, "sel_hist")
    _need(top_expert, torch.int32, rows * s.k, "top_expert")
    _need(top_prob, torch.int64, rows * s.k, "top_prob")
    _need(S, torch.int64, s.E, "S")
    _check(_lib().moe_popularity_estimate(C.byref(s), _ptr(sel_hist), N_t, _ptr(top_expert),
                                          _ptr(top_prob), _ptr(S), _stream(stream)))


def moe_devices_for_expert(S_e: int, N_t: int, N: int) -> float:
    return float(_lib().moe_devices_for_expert(int(S_e), N_t, N))


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=dtype))


def _hp(a: np.ndarray) -> C.c_void_p:
    return C.c_void_p(a.ctypes.data)


def moe_schedule_experts(N: int, E: int, w: Sequence[int], W: int, has: Sequence[bool],
                         max_pack: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """-> (replicas[E], dev_count[N], dev_experts[N,E], devices_used)."""
    wa, ha = _host(w, np.uint64), _host(has, np.uint8)
    if wa.size != E or ha.size != E:
        raise MoeError("w and has need E entries")
    rep, cnt = np.empty(E, np.int32), np.empty(max(N, 1), np.int32)
    dev, used = np.empty(max(N, 1) * E, np.int32), np.zeros(1, np.int32)
    _check(_lib().moe_schedule_experts(N, E, _hp(wa), int(W), _hp(ha), max_pack, _hp(rep), _hp(cnt),
                                       _hp(dev), _hp(used)))
    return rep, cnt, dev.reshape(N, E), int(used[0])


def moe_top_lists_identical(E: int, k: int, S: Sequence[int], counts: Sequence[int]) -> bool:
    Sa, ca = _host(S, np.uint64), _host(counts, np.int32)
    if Sa.size != E or ca.size != E:
        raise MoeError("S and counts need E entries")
    return bool(_lib().moe_top_lists_identical(E, k, _hp(Sa), _hp(ca)))


def moe_schedule_layer(N: int, E: int, k: int, N_t: int, S: Sequence[int], counts: Sequence[int],
                       max_pack: int):
    """-> (replicas[E], dev_count[N], dev_experts[N,E], devices_used, rescheduled)."""
    Sa, ca = _host(S, np.uint64), _host(counts, np.int32)
    if Sa.size != E or ca.size != E:
        raise MoeError("S and counts need E entries")
    rep, cnt = np.empty(E, np.int32), np.empty(max(N, 1), np.int32)
    dev, used, re_ = np.empty(max(N, 1) * E, np.int32), np.zeros(1, np.int32), np.zeros(1, np.int32)
    _check(_lib().moe_schedule_layer(N, E, k, N_t, _hp(Sa), _hp(ca), max_pack, _hp(rep), _hp(cnt),
                                     _hp(dev), _hp(used), _hp(re_)))
    return rep, cnt, dev.reshape(N, E), int(used[0]), bool(re_[0])

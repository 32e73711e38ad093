"""ctypes binding of libmoe.so: one Python function per C entry point, same names.

Argument marshalling only -- every step of the layer runs in the HIP kernels.
Tensors are torch CUDA tensors (device memory); `stream` defaults to torch's
current stream.  There is no CPU fallback: if the library is missing it is built
once with hipcc, and if that fails the import error is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmoe.so")

DTYPE = {"f32": 0, "bf16": 1}
ACT = {"gelu": 0, "gelu_erf": 0, "gelu_tanh": 1, "relu": 2, "identity": 3}


class MoeError(RuntimeError):
    pass


class Shape(C.Structure):
    """Mirror of moe_shape in include/moe.h."""
    _fields_ = [("T", C.c_int32), ("d_model", C.c_int32), ("E", C.c_int32),
                ("d_ff", C.c_int32), ("k", C.c_int32), ("capacity", C.c_int32),
                ("dtype", C.c_int32), ("act", C.c_int32), ("renorm_topk", C.c_int32)]

    @classmethod
    def make(cls, T, d_model, E, d_ff, k, capacity, dtype="bf16", act="gelu", renorm_topk=False):
        return cls(T, d_model, E, d_ff, k, capacity, DTYPE[dtype], ACT[act], int(renorm_topk))

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == DTYPE["bf16"] else torch.float32

    @property
    def ye_dtype(self):
        """Stored type of the expert outputs ye: fp16 for bf16 layers, fp32 for fp32 layers."""
        return torch.float16 if self.dtype == DTYPE["bf16"] else torch.float32


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib() -> C.CDLL:
    """The loaded library (built first if no build exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from .build import build
            build()
        L = C.CDLL(_LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        sp = C.POINTER(Shape)
        L.moe_capacity.restype = C.c_int64
        L.moe_capacity.argtypes = [i32, i32, i32, C.c_double]
        L.moe_max_rows.restype = C.c_int64
        L.moe_max_rows.argtypes = [sp]
        L.moe_workspace_bytes.restype = sz
        L.moe_workspace_bytes.argtypes = [sp, i32]
        L.moe_last_error.restype = C.c_char_p
        L.moe_last_error.argtypes = []
        L.moe_packed_weight_bytes.restype = sz
        L.moe_packed_weight_bytes.argtypes = [sp]
        L.moe_packed_gate_bytes.restype = sz
        L.moe_packed_gate_bytes.argtypes = [sp]
        L.moe_pack_weights.argtypes = [sp, vp, vp, vp, vp, vp]
        L.moe_pack_gate.argtypes = [sp, vp, vp, vp]
        L.moe_route.argtypes = [sp, vp, vp, vp, i32, vp, vp, vp]
        L.moe_dispatch.argtypes = [sp] + [vp] * 9
        L.moe_dispatch_static.argtypes = [sp] + [vp] * 8
        L.moe_dispatch_static.restype = C.c_int
        L.moe_dispatch_static_limit.restype = sz
        L.moe_expert_gemm_kernel.argtypes = [sp, i32, C.c_char_p, sz]
        L.moe_dispatch_static_limit.argtypes = []
        L.moe_expert_ffn.argtypes = [sp] + [vp] * 9
        L.moe_combine.argtypes = [sp] + [vp] * 6
        L.moe_layer_chunked.argtypes = [sp, i32, vp, vp, vp, i32] + [vp] * 16
        L.moe_calib_copy.argtypes = [vp, vp, sz, vp]
        L.moe_calib_copy.restype = C.c_int
        L.moe_calib_gemm.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]
        L.moe_calib_gemm.restype = C.c_int
        L.moe_calib_mfma.argtypes = [vp, i32, i32, i32, vp]
        L.moe_calib_mfma.restype = C.c_int
        L.moe_calib_mfma_flops.argtypes = [i32, i32]
        L.moe_calib_mfma_flops.restype = C.c_double
        L.moe_tune_ffn_group_rows.argtypes = [i32]
        L.moe_tune_ffn_group_rows.restype = i32
        L.moe_profile_enable.restype = C.c_int
        L.moe_profile_enable.argtypes = [C.c_uint32, i32]
        L.moe_profile_read.restype = i32
        L.moe_profile_read.argtypes = [i32, C.POINTER(C.c_float), i32]
        for name in ("moe_pack_weights", "moe_pack_gate", "moe_route", "moe_dispatch",
                     "moe_expert_ffn", "moe_combine", "moe_layer_chunked"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise MoeError("libmoe takes contiguous device tensors")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status: int) -> None:
    if status != 0:
        raise MoeError(f"libmoe status {status}: {moe_last_error()}")


def _need(t: torch.Tensor, dtype, numel: int, name: str) -> None:
    if t.dtype != dtype or t.numel() < numel:
        raise MoeError(f"{name}: expected >= {numel} elements of {dtype}, got {t.numel()} of {t.dtype}")


def moe_last_error() -> str:
    return lib().moe_last_error().decode()


def moe_capacity(T: int, E: int, k: int, cf: float) -> int:
    return int(lib().moe_capacity(T, E, k, float(cf)))


def moe_max_rows(s: Shape) -> int:
    return int(lib().moe_max_rows(C.byref(s)))


def moe_workspace_bytes(s: Shape, n_chunks: int = 1) -> int:
    return int(lib().moe_workspace_bytes(C.byref(s), n_chunks))


def moe_packed_weight_bytes(s: Shape) -> int:
    return int(lib().moe_packed_weight_bytes(C.byref(s)))


def moe_packed_gate_bytes(s: Shape) -> int:
    return int(lib().moe_packed_gate_bytes(C.byref(s)))


def moe_pack_weights(s: Shape, W1, W2, W1p, W2p, stream=None) -> None:
    n = s.E * s.d_model * s.d_ff
    _need(W1, s.torch_dtype, n, "W1")
    _need(W2, s.torch_dtype, n, "W2")
    _check(lib().moe_pack_weights(C.byref(s), _ptr(W1), _ptr(W2), _ptr(W1p), _ptr(W2p),
                                  _stream(stream)))


def moe_pack_gate(s: Shape, Wg, Wgp, stream=None) -> None:
    _need(Wg, s.torch_dtype, s.d_model * s.E, "Wg")
    _check(lib().moe_pack_gate(C.byref(s), _ptr(Wg), _ptr(Wgp), _stream(stream)))


def moe_route(s: Shape, x, Wgp, gate_bias, bias_token_stride, expert_idx, gate, stream=None) -> None:
    _need(x, s.torch_dtype, s.T * s.d_model, "x")
    _need(expert_idx, torch.int32, s.T * s.k, "expert_idx")
    _need(gate, torch.float32, s.T * s.k, "gate")
    if gate_bias is not None:
        _need(gate_bias, torch.float32, s.E if bias_token_stride == 0 else s.T * s.E, "gate_bias")
    _check(lib().moe_route(C.byref(s), _ptr(x), _ptr(Wgp), _ptr(gate_bias), bias_token_stride,
                           _ptr(expert_idx), _ptr(gate), _stream(stream)))


def moe_dispatch(s: Shape, x, expert_idx, counts, offsets, slot_of, src_of, xe, workspace,
                 stream=None) -> None:
    rows = moe_max_rows(s)
    _need(x, s.torch_dtype, s.T * s.d_model, "x")
    _need(expert_idx, torch.int32, s.T * s.k, "expert_idx")
    _need(counts, torch.int32, s.E, "counts")
    _need(offsets, torch.int32, s.E + 1, "offsets")
    _need(slot_of, torch.int32, s.T * s.k, "slot_of")
    _need(src_of, torch.int32, rows, "src_of")
    _need(xe, s.torch_dtype, rows * s.d_model, "xe")
    _need(workspace, torch.uint8, moe_workspace_bytes(s, 1), "workspace")
    _check(lib().moe_dispatch(C.byref(s), _ptr(x), _ptr(expert_idx), _ptr(counts), _ptr(offsets),
                              _ptr(slot_of), _ptr(src_of), _ptr(xe), _ptr(workspace),
                              _stream(stream)))


def moe_calib_copy(dst, src, nbytes: int, stream=None) -> None:
    _check(lib().moe_calib_copy(_ptr(dst), _ptr(src), int(nbytes), _stream(stream)))


def moe_calib_gemm(A, W, Cout, items, n_items, N: int, K: int, variant: int, gelu: bool, stream=None) -> None:
    _check(lib().moe_calib_gemm(_ptr(A), _ptr(W), _ptr(Cout), _ptr(items), _ptr(n_items), items.numel() // 4,
                                N, K, variant, int(gelu), _stream(stream)))


def moe_expert_gemm_kernel(s: Shape, which: int) -> str:
    """Name and tile of the kernel an unchunked bf16 layer launches for expert GEMM `which`."""
    buf = C.create_string_buffer(96)
    _check(lib().moe_expert_gemm_kernel(C.byref(s), int(which), buf, C.sizeof(buf)))
    return buf.value.decode()


def moe_calib_mfma(sink, waves_per_simd: int, iters: int, random_operands: bool, stream=None) -> float:
    """Enqueues the matrix-core calibration loop; returns the launch's flops."""
    _need(sink, torch.float32, 256 * waves_per_simd * 256, "sink")
    _check(lib().moe_calib_mfma(_ptr(sink), waves_per_simd, iters, int(random_operands), _stream(stream)))
    return float(lib().moe_calib_mfma_flops(waves_per_simd, iters))


def moe_tune_ffn_group_rows(rows: int = 0) -> int:
    """Sets (rows >= 1) or reads the rows per expert an FFN launch of a chunked layer must
    hold on average; returns the previous value."""
    return int(lib().moe_tune_ffn_group_rows(int(rows)))


def moe_dispatch_static_limit() -> int:
    return int(lib().moe_dispatch_static_limit())


def moe_dispatch_static(s: Shape, x, expert_idx, counts, offsets, slot_of, src_of, xe,
                        stream=None) -> None:
    rows = moe_max_rows(s)
    _need(x, s.torch_dtype, s.T * s.d_model, "x")
    _need(expert_idx, torch.int32, s.T * s.k, "expert_idx")
    _need(counts, torch.int32, s.E, "counts")
    _need(offsets, torch.int32, s.E + 1, "offsets")
    _need(slot_of, torch.int32, s.T * s.k, "slot_of")
    _need(src_of, torch.int32, rows, "src_of")
    _need(xe, s.torch_dtype, rows * s.d_model, "xe")
    _check(lib().moe_dispatch_static(C.byref(s), _ptr(x), _ptr(expert_idx), _ptr(counts),
                                     _ptr(offsets), _ptr(slot_of), _ptr(src_of), _ptr(xe),
                                     _stream(stream)))


def moe_expert_ffn(s: Shape, xe, offsets, W1p, b1, W2p, b2, ye, workspace, stream=None) -> None:
    rows = moe_max_rows(s)
    _need(xe, s.torch_dtype, rows * s.d_model, "xe")
    _need(offsets, torch.int32, s.E + 1, "offsets")
    _need(ye, s.ye_dtype, rows * s.d_model, "ye")
    _need(workspace, torch.uint8, moe_workspace_bytes(s, 1), "workspace")
    _check(lib().moe_expert_ffn(C.byref(s), _ptr(xe), _ptr(offsets), _ptr(W1p), _ptr(b1),
                                _ptr(W2p), _ptr(b2), _ptr(ye), _ptr(workspace), _stream(stream)))


def moe_combine(s: Shape, ye, slot_of, gate, y, y_act=None, stream=None) -> None:
    _need(ye, s.ye_dtype, moe_max_rows(s) * s.d_model, "ye")
    _need(slot_of, torch.int32, s.T * s.k, "slot_of")
    _need(gate, torch.float32, s.T * s.k, "gate")
    _need(y, torch.float32, s.T * s.d_model, "y")
    if y_act is not None:
        _need(y_act, s.torch_dtype, s.T * s.d_model, "y_act")
    _check(lib().moe_combine(C.byref(s), _ptr(ye), _ptr(slot_of), _ptr(gate), _ptr(y),
                             _ptr(y_act), _stream(stream)))


def moe_layer_chunked(s: Shape, n_chunks: int, x, Wgp, gate_bias, bias_token_stride, W1p, b1,
                      W2p, b2, expert_idx, gate, counts, offsets, slot_of, src_of, xe, ye, y,
                      y_act, workspace, stream=None) -> None:
    rows = moe_max_rows(s)
    _need(x, s.torch_dtype, s.T * s.d_model, "x")
    _need(expert_idx, torch.int32, s.T * s.k, "expert_idx")
    _need(gate, torch.float32, s.T * s.k, "gate")
    _need(counts, torch.int32, s.E, "counts")
    _need(offsets, torch.int32, s.E + 1, "offsets")
    _need(slot_of, torch.int32, s.T * s.k, "slot_of")
    _need(src_of, torch.int32, rows, "src_of")
    _need(xe, s.torch_dtype, rows * s.d_model, "xe")
    _need(ye, s.ye_dtype, rows * s.d_model, "ye")
    _need(y, torch.float32, s.T * s.d_model, "y")
    _need(workspace, torch.uint8, moe_workspace_bytes(s, max(1, n_chunks)), "workspace")
    if gate_bias is not None:
        _need(gate_bias, torch.float32, s.E if bias_token_stride == 0 else s.T * s.E, "gate_bias")
    if y_act is not None:
        _need(y_act, s.torch_dtype, s.T * s.d_model, "y_act")
    _check(lib().moe_layer_chunked(
        C.byref(s), n_chunks, _ptr(x), _ptr(Wgp), _ptr(gate_bias), bias_token_stride,
        _ptr(W1p), _ptr(b1), _ptr(W2p), _ptr(b2), _ptr(expert_idx), _ptr(gate), _ptr(counts),
        _ptr(offsets), _ptr(slot_of), _ptr(src_of), _ptr(xe), _ptr(ye), _ptr(y), _ptr(y_act),
        _ptr(workspace), _stream(stream)))


STAGES = ("route", "plan", "tiles", "scatter", "gemm1", "gemm2", "combine",
          "bwd_recompute", "bwd_dP", "bwd_dxe", "bwd_wgrad2", "bwd_wgrad1", "bwd_other")


def moe_profile_enable(stage_mask: int, max_samples: int) -> None:
    _check(lib().moe_profile_enable(stage_mask, max_samples))


def moe_profile_read(stage: int, cap: int = 4096):
    buf = (C.c_float * cap)()
    n = lib().moe_profile_read(stage, buf, cap)
    return [float(buf[i]) for i in range(n)]


def alloc_buffers(s: Shape, n_chunks: int = 1, device="cuda:0", y_act: bool = False) -> Dict[str, torch.Tensor]:
    """Device buffers for every output and the workspace of one layer (plumbing)."""
    rows = moe_max_rows(s)
    dev = torch.device(device)
    b = dict(
        Wgp=torch.empty(moe_packed_gate_bytes(s) // 4, dtype=torch.float32, device=dev),
        W1p=torch.empty(moe_packed_weight_bytes(s), dtype=torch.uint8, device=dev),
        W2p=torch.empty(moe_packed_weight_bytes(s), dtype=torch.uint8, device=dev),
        expert_idx=torch.empty(s.T * s.k, dtype=torch.int32, device=dev),
        gate=torch.empty(s.T * s.k, dtype=torch.float32, device=dev),
        counts=torch.empty(s.E, dtype=torch.int32, device=dev),
        offsets=torch.empty(s.E + 1, dtype=torch.int32, device=dev),
        slot_of=torch.empty(s.T * s.k, dtype=torch.int32, device=dev),
        src_of=torch.empty(rows, dtype=torch.int32, device=dev),
        xe=torch.empty(rows * s.d_model, dtype=s.torch_dtype, device=dev),
        ye=torch.empty(rows * s.d_model, dtype=s.ye_dtype, device=dev),
        y=torch.empty(s.T * s.d_model, dtype=torch.float32, device=dev),
        workspace=torch.empty(moe_workspace_bytes(s, n_chunks), dtype=torch.uint8, device=dev),
    )
    b["y_act"] = torch.empty(s.T * s.d_model, dtype=s.torch_dtype, device=dev) if y_act else None
    return b

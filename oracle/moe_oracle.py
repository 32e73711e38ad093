"""ctypes front end of the C oracle (oracle/moe_oracle.c) -- test infrastructure only.

Argument marshalling plus `moe_layer`, which strings the oracle steps together in
the order the paper gives for one MoE layer (Sec. 2.1; Sec. 2.2 forward-pass
timeline: gate, first all-to-all, expert FFN, second all-to-all, combine).
No arithmetic of the method happens in this file.
"""
from __future__ import annotations

import ctypes as C
import dataclasses
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")

ACT = {"gelu": 0, "gelu_erf": 0, "gelu_tanh": 1, "relu": 2, "identity": 3}

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc.  FP contraction is off so that every
    multiply-add the source spells separately stays separate."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-mavx2", "-mfma", "-ffp-contract=off",
               "-fopenmp", "-fPIC", "-shared", "-std=gnu11", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_plan.restype = C.c_int
        _lib.oracle_act.restype = C.c_double
        _lib.oracle_act.argtypes = [C.c_double, C.c_int]
        _lib.oracle_capacity.restype = C.c_int64
        _lib.oracle_capacity.argtypes = [C.c_int, C.c_int, C.c_int, C.c_double]
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def threads() -> int:
    return int(_load().oracle_threads())


def capacity(T: int, E: int, k: int, cf: Optional[float]) -> int:
    """Slots per expert; cf=None means no dropping (every expert can hold all T tokens)."""
    if cf is None:
        return int(T)
    return int(_load().oracle_capacity(int(T), int(E), int(k), float(cf)))


def act_value(v: float, act: str) -> float:
    return float(_load().oracle_act(float(v), ACT[act]))


def gate_logits(x, Wg, bias=None, bias_stride: int = 0) -> np.ndarray:
    x, Wg = _f32(x), _f32(Wg)
    T, d = x.shape
    E = Wg.shape[1]
    assert Wg.shape[0] == d
    if bias is not None:
        bias = _f32(bias)
        assert bias.size == (E if bias_stride == 0 else T * E) and bias_stride in (0, E)
    z = np.empty((T, E), np.float32)
    _load().oracle_gate_logits(_p(x), _p(Wg), _p(bias), C.c_int(bias_stride),
                               C.c_int(T), C.c_int(d), C.c_int(E), _p(z))
    return z


def topk_softmax(z, k: int, renorm: bool = False):
    z = _f32(z)
    T, E = z.shape
    assert 1 <= k <= E <= 64
    idx = np.empty((T, k), np.int32)
    gate = np.empty((T, k), np.float32)
    _load().oracle_topk_softmax(_p(z), C.c_int(T), C.c_int(E), C.c_int(k),
                                C.c_int(int(renorm)), _p(idx), _p(gate))
    return idx, gate


def plan(expert_idx, E: int, capacity: int):
    idx = _i32(expert_idx)
    T, k = idx.shape
    count = np.empty(E, np.int32)
    off = np.empty(E + 1, np.int32)
    slot_of = np.empty(T * k, np.int32)
    src_full = np.full(max(T * k, 1), -1, np.int32)
    A = _load().oracle_plan(_p(idx), C.c_int(T), C.c_int(k), C.c_int(E),
                            C.c_int(capacity), _p(count), _p(off), _p(slot_of), _p(src_full))
    return count, off, slot_of, src_full[:A].copy()


def scatter(x, slot_of, k: int, A: int) -> np.ndarray:
    x = _f32(x)
    T, d = x.shape
    slot_of = _i32(slot_of)
    xe = np.zeros((A, d), np.float32)
    _load().oracle_scatter(_p(x), _p(slot_of), C.c_int(T), C.c_int(k), C.c_int(d), _p(xe))
    return xe


def ffn_rows(xe, off, W1, W2, rows: Sequence[int], act: str = "gelu",
             b1=None, b2=None) -> np.ndarray:
    xe, W1, W2, off = _f32(xe), _f32(W1), _f32(W2), _i32(off)
    E, d, h = W1.shape
    assert W2.shape == (E, h, d) and xe.shape[1] == d and off.size == E + 1
    rows = _i32(rows)
    assert rows.size == 0 or (rows.min() >= 0 and rows.max() < xe.shape[0])
    b1 = None if b1 is None else _f32(b1)
    b2 = None if b2 is None else _f32(b2)
    out = np.empty((rows.size, d), np.float64)
    _load().oracle_ffn_rows(_p(xe), _p(off), C.c_int(E), C.c_int(d), C.c_int(h),
                            _p(W1), _p(b1), _p(W2), _p(b2), C.c_int(ACT[act]),
                            _p(rows), C.c_int(rows.size), _p(out))
    return out


def combine(ye, slot_of, gate, T: int, k: int) -> np.ndarray:
    ye = np.ascontiguousarray(ye, np.float64)
    d = ye.shape[1]
    slot_of, gate = _i32(slot_of), _f32(gate)
    y = np.empty((T, d), np.float32)
    _load().oracle_combine(_p(ye), _p(slot_of), _p(gate), C.c_int(T), C.c_int(k),
                           C.c_int(d), _p(y))
    return y


@dataclasses.dataclass
class OracleOut:
    z: np.ndarray            # [T,E] fp32 logits
    expert_idx: np.ndarray   # [T,k] int32
    gate: np.ndarray         # [T,k] fp32
    count: np.ndarray        # [E]
    off: np.ndarray          # [E+1]
    slot_of: np.ndarray      # [T*k], -1 = dropped
    src_of: np.ndarray       # [A]
    xe: np.ndarray           # [A,d]
    tokens: np.ndarray       # tokens whose output rows were computed
    y: np.ndarray            # [len(tokens), d] fp32 (all T tokens when tokens is None)

    @property
    def A(self) -> int:
        return int(self.off[-1])


def moe_layer(x, Wg, W1, W2, *, k: int, capacity: int, act: str = "gelu",
              bias=None, bias_stride: int = 0, b1=None, b2=None, renorm: bool = False,
              tokens: Optional[Sequence[int]] = None) -> OracleOut:
    """One MoE layer forward.  With `tokens` given, the FFN and combine run only for
    those tokens (the layer is per token once the plan is fixed), which is how
    outputs are sampled at sizes where the full fp64 FFN would take minutes."""
    x = _f32(x)
    T, d = x.shape
    E = np.shape(W1)[0]
    z = gate_logits(x, Wg, bias, bias_stride)
    idx, gate = topk_softmax(z, k, renorm)
    count, off, slot_of, src_of = plan(idx, E, capacity)
    A = int(off[-1])
    xe = scatter(x, slot_of, k, A)
    tok = np.arange(T, dtype=np.int32) if tokens is None else _i32(tokens)
    so = slot_of.reshape(T, k)[tok]                      # slots of the sampled tokens
    rows = np.unique(so[so >= 0]).astype(np.int32)
    ye_rows = ffn_rows(xe, off, W1, W2, rows, act, b1, b2)
    # place the computed rows in a sparse [A,d] view indexed by slot for combine
    local = np.full(max(A, 1), -1, np.int32)
    local[rows] = np.arange(rows.size, dtype=np.int32)
    so_local = np.where(so >= 0, local[np.maximum(so, 0)], -1).astype(np.int32)
    y = combine(ye_rows if rows.size else np.zeros((1, d)), so_local.reshape(-1),
                gate.reshape(T, k)[tok].reshape(-1), tok.size, k)
    return OracleOut(z=z, expert_idx=idx, gate=gate, count=count, off=off,
                     slot_of=slot_of, src_of=src_of, xe=xe, tokens=tok, y=y)

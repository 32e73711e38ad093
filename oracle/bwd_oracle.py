"""CPU oracle of the MoE layer's backward pass -- test infrastructure only.

The paper trains the layer of Sec. 2.1 (Sec. 2.2 and Sec. 4 schedule the backward
pass's all-to-all against allreduce); it does not spell the gradients out because they
are the chain rule of the forward definition.  This file writes that chain rule down in
fp64 with numpy matmuls as steps, in the forward's notation, for a loss whose gradient
with respect to the layer output y is the given dy.  Routing (which experts, which
slots) is piecewise constant and carries no gradient; the gate weights do, through the
softmax over all E logits.  Nothing in the product path imports this file, and it
shares no code with the HIP side.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np
from scipy.special import erf

from . import moe_oracle as fo


def act_and_derivative(P: np.ndarray, act: str):
    """phi(P) and phi'(P) for the expert activation."""
    if act == "relu":
        return np.maximum(P, 0.0), (P > 0).astype(np.float64)
    if act == "identity":
        return P.copy(), np.ones_like(P)
    if act == "gelu":                       # 0.5 v (1 + erf(v / sqrt 2)); derivative Phi + v phi
        Phi = 0.5 * (1.0 + erf(P / np.sqrt(2.0)))
        pdf = np.exp(-0.5 * P * P) / np.sqrt(2.0 * np.pi)
        return P * Phi, Phi + P * pdf
    if act == "gelu_tanh":
        c, a = np.sqrt(2.0 / np.pi), 0.044715
        u = c * (P + a * P ** 3)
        th = np.tanh(u)
        return 0.5 * P * (1.0 + th), 0.5 * (1.0 + th) + 0.5 * P * (1.0 - th * th) * c * (1.0 + 3 * a * P * P)
    raise ValueError(act)


@dataclasses.dataclass
class Grads:
    dx: np.ndarray        # [T,d]
    dWg: np.ndarray       # [d,E]
    dW1: np.ndarray       # [E,d,h]
    dW2: np.ndarray       # [E,h,d]
    dgate: np.ndarray     # [T,k]  dL/d(gate weight), 0 for dropped assignments
    dye: np.ndarray       # [A,d]  dL/d(expert output rows)
    dxe: np.ndarray       # [A,d]  dL/d(packed rows)
    dP: np.ndarray        # [A,h]  dL/d(pre-activation)
    y: np.ndarray         # forward output (fp64)
    fwd: "fo.OracleOut"   # the forward's integers (routing, plan)


def moe_layer_backward(x, Wg, W1, W2, dy, *, k: int, capacity: int, act: str = "gelu",
                       bias=None, bias_stride: int = 0,
                       experts: Optional[np.ndarray] = None) -> Grads:
    """Gradients of the layer y = sum_j g[t,j] * FFN_{e(t,j)}(x[t]) (kept assignments only)
    given dy = dL/dy.  `experts`, if given, restricts dW1/dW2 to those experts (the others
    are returned as zeros) so that full-size layers can be sampled."""
    x = np.asarray(x, np.float64)
    Wg64, W1, W2 = np.asarray(Wg, np.float64), np.asarray(W1), np.asarray(W2)
    dy = np.asarray(dy, np.float64)
    T, d = x.shape
    E, _, h = W1.shape
    # ---- forward, keeping what the chain rule needs
    z = fo.gate_logits(x.astype(np.float32), np.asarray(Wg, np.float32), bias, bias_stride)
    idx, gate32 = fo.topk_softmax(z, k)
    count, off, slot_of, src_of = fo.plan(idx, E, capacity)
    A = int(off[-1])
    z64 = z.astype(np.float64)
    p = np.exp(z64 - z64.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)                        # softmax over all E experts
    gate = np.take_along_axis(p, idx.astype(np.int64), 1)   # g[t,j] = p[t, e(t,j)]
    tok = src_of // k                                   # token of each slot
    xe = x[tok]
    P = np.empty((A, h))
    H = np.empty((A, h))
    dphi = np.empty((A, h))
    ye = np.empty((A, d))
    for e in range(E):
        r = slice(off[e], off[e + 1])
        P[r] = xe[r] @ W1[e].astype(np.float64)
        H[r], dphi[r] = act_and_derivative(P[r], act)
        ye[r] = H[r] @ W2[e].astype(np.float64)
    slot = slot_of.reshape(T, k)
    y = np.zeros((T, d))
    for j in range(k):
        kept = slot[:, j] >= 0
        y[kept] += gate[kept, j, None] * ye[slot[kept, j]]
    # ---- backward
    dye = np.zeros((A, d))
    dgate = np.zeros((T, k))
    for j in range(k):
        kept = slot[:, j] >= 0
        s = slot[kept, j]
        dye[s] = gate[kept, j, None] * dy[kept]         # each slot has exactly one source
        dgate[kept, j] = np.einsum("td,td->t", ye[s], dy[kept])
    dP = np.empty((A, h))
    dxe = np.empty((A, d))
    dW1 = np.zeros(W1.shape)
    dW2 = np.zeros(W2.shape)
    want = range(E) if experts is None else [int(e) for e in experts]
    for e in range(E):
        r = slice(off[e], off[e + 1])
        dH = dye[r] @ W2[e].astype(np.float64).T
        dP[r] = dH * dphi[r]
        dxe[r] = dP[r] @ W1[e].astype(np.float64).T
        if e in want:
            dW2[e] = H[r].T @ dye[r]
            dW1[e] = xe[r].T @ dP[r]
    dx = np.zeros((T, d))
    np.add.at(dx, tok, dxe)                             # a token's kept slots add up
    # gate: g = p[e] for the chosen experts, p = softmax(z), z = x Wg (+ bias)
    dgfull = np.zeros((T, E))
    np.put_along_axis(dgfull, idx.astype(np.int64), dgate, 1)
    dz = p * (dgfull - (p * dgfull).sum(1, keepdims=True))
    dx += dz @ Wg64.T
    dWg = x.T @ dz
    fwd = fo.OracleOut(z=z, expert_idx=idx, gate=gate32, count=count, off=off, slot_of=slot_of,
                       src_of=src_of, xe=xe.astype(np.float32), tokens=np.arange(T, dtype=np.int32),
                       y=y.astype(np.float32))
    return Grads(dx=dx, dWg=dWg, dW1=dW1, dW2=dW2, dgate=dgate, dye=dye, dxe=dxe, dP=dP, y=y, fwd=fwd)

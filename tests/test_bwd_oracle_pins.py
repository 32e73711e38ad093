"""Pins of the backward oracle: central finite differences of the (separately pinned)
forward oracle, automatic differentiation of a forward typed in torch fp64, the dense
special case, and structural properties (linearity in dy, dropped tokens)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import bwd_oracle as bo
import workloads as wl


def tiny(seed, T=14, d=6, E=3, h=5, k=2, cf=0.8, dtype="f32"):
    cfg = dict(T=T, d=d, E=E, h=h, k=k, cf=cf, dtype=dtype, skew=None, layers=1)
    li = wl.make_layer(cfg, seed=seed)
    # larger weights than the workload's N(0, 0.02) so that every gradient path is visible
    prng = np.random.Generator(np.random.PCG64(seed + 100))
    li.Wg = prng.standard_normal(li.Wg.shape).astype(np.float32)
    li.W1 = (0.7 * prng.standard_normal(li.W1.shape)).astype(np.float32)
    li.W2 = (0.7 * prng.standard_normal(li.W2.shape)).astype(np.float32)
    dy = prng.standard_normal((T, d))
    return li, dy


def loss(li, dy, x=None, Wg=None, W1=None, W2=None, act="gelu"):
    o = oracle.moe_layer(li.x if x is None else x, li.Wg if Wg is None else Wg,
                         li.W1 if W1 is None else W1, li.W2 if W2 is None else W2,
                         k=li.k, capacity=li.C, act=act)
    return float((o.y.astype(np.float64) * dy).sum()), o.expert_idx.copy()


@pytest.mark.parametrize("act", ["gelu", "relu", "gelu_tanh", "identity"])
def test_finite_differences_of_the_forward_oracle(act):
    li, dy = tiny(1)
    g = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy, k=li.k, capacity=li.C, act=act)
    assert (g.fwd.slot_of < 0).any()                      # some assignments are dropped
    base_idx = loss(li, dy, act=act)[1]
    eps = 2e-3
    checked = 0
    rng = np.random.Generator(np.random.PCG64(9))
    for name, grad in (("x", g.dx), ("Wg", g.dWg), ("W1", g.dW1), ("W2", g.dW2)):
        ref = getattr(li, name)
        scale = np.abs(grad).max()
        for _ in range(40):
            pos = tuple(int(rng.integers(0, n)) for n in ref.shape)
            up, dn = ref.copy(), ref.copy()
            up[pos] += eps
            dn[pos] -= eps
            lu, iu = loss(li, dy, act=act, **{name: up})
            ld, idn = loss(li, dy, act=act, **{name: dn})
            if not (np.array_equal(iu, base_idx) and np.array_equal(idn, base_idx)):
                continue                                   # the step crossed a routing boundary
            if act == "relu":
                # skip entries whose step crosses a kink: second difference must be small
                l0 = loss(li, dy, act=act)[0]
                if abs(lu - 2 * l0 + ld) > 1e-3 * scale * eps:
                    continue
            fd = (lu - ld) / (2 * eps)
            assert abs(fd - grad[pos]) <= 2e-3 * scale + 1e-4, (name, pos, fd, grad[pos])
            checked += 1
    assert checked >= 100


def test_forward_inside_the_backward_oracle_is_the_forward_oracle():
    li, dy = tiny(2, T=40, d=8, E=4, h=12)
    g = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy, k=li.k, capacity=li.C)
    o = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, k=li.k, capacity=li.C)
    assert np.array_equal(g.fwd.slot_of, o.slot_of) and np.array_equal(g.fwd.expert_idx, o.expert_idx)
    np.testing.assert_allclose(g.y, o.y, rtol=2e-6, atol=1e-6)


def test_single_expert_is_a_dense_mlp_under_autograd():
    li, dy = tiny(3, T=20, d=7, E=1, h=9, k=1, cf=None)
    g = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy, k=1, capacity=li.T)
    x = torch.tensor(li.x, dtype=torch.float64, requires_grad=True)
    W1 = torch.tensor(li.W1[0], dtype=torch.float64, requires_grad=True)
    W2 = torch.tensor(li.W2[0], dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.gelu(x @ W1) @ W2             # the gate weight of a lone expert is 1
    (y * torch.tensor(dy)).sum().backward()
    np.testing.assert_allclose(g.dx, x.grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(g.dW1[0], W1.grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(g.dW2[0], W2.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.abs(g.dWg).max() < 1e-12


@pytest.mark.parametrize("k,cf", [(1, 1.0), (2, 0.7), (2, None)])
def test_whole_layer_under_autograd_with_the_oracle_routing(k, cf):
    li, dy = tiny(4, T=30, d=6, E=4, h=8, k=k, cf=cf)
    g = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy, k=k, capacity=li.C)
    f = g.fwd
    t64 = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    x, Wg, W1, W2 = t64(li.x), t64(li.Wg), t64(li.W1), t64(li.W2)
    p = torch.softmax(x @ Wg, dim=1)
    y = torch.zeros(li.T, li.d, dtype=torch.float64)
    rows = []
    for t in range(li.T):
        acc = torch.zeros(li.d, dtype=torch.float64)
        for j in range(k):
            if f.slot_of[t * k + j] < 0:
                continue                                   # dropped: no contribution
            e = int(f.expert_idx[t, j])
            acc = acc + p[t, e] * (torch.nn.functional.gelu(x[t] @ W1[e]) @ W2[e])
        rows.append(acc)
    y = torch.stack(rows)
    (y * torch.tensor(dy)).sum().backward()
    for got, want in ((g.dx, x.grad), (g.dWg, Wg.grad), (g.dW1, W1.grad), (g.dW2, W2.grad)):
        # the oracle's logits are fp32 by definition (torch's here are fp64): 1e-7-level gates
        w = want.numpy()
        np.testing.assert_allclose(got, w, rtol=1e-5, atol=2e-6 * np.abs(w).max())


def test_structure_linearity_and_dropped_tokens():
    li, dy = tiny(5, T=50, d=6, E=3, h=5, k=1, cf=0.5)
    g1 = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy, k=1, capacity=li.C)
    g3 = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, 3.0 * dy, k=1, capacity=li.C)
    for a, b in ((g1.dx, g3.dx), (g1.dWg, g3.dWg), (g1.dW1, g3.dW1), (g1.dW2, g3.dW2)):
        np.testing.assert_allclose(3.0 * a, b, rtol=1e-12, atol=1e-15)
    dropped = g1.fwd.slot_of < 0
    assert dropped.any()
    assert not g1.dx[dropped].any() and not g1.dgate[dropped].any()      # y_t is constant 0
    # restricting the weight gradients to some experts leaves those experts' values unchanged
    gs = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy, k=1, capacity=li.C, experts=[1])
    assert np.array_equal(gs.dW1[1], g1.dW1[1]) and not gs.dW1[0].any() and not gs.dW2[2].any()
    assert np.array_equal(gs.dx, g1.dx)

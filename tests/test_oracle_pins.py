"""Pins of the CPU oracle against things other than itself: a hand-worked example,
closed forms, brute force on tiny inputs, invariants, and library routines on the
special cases that reduce to them.  None of these tests needs a GPU."""
import itertools
import json
import math
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle
import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


# ---------------------------------------------------------------- hand example
def test_hand_worked_example():
    g = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    x, Wg = np.array(g["x"], np.float32), np.array(g["Wg"], np.float32)
    W1, W2 = np.array(g["W1"], np.float32), np.array(g["W2"], np.float32)
    o = oracle.moe_layer(x, Wg, W1, W2, k=g["k"], capacity=g["capacity"], act=g["act"])
    assert o.expert_idx.reshape(-1).tolist() == g["expert_idx"]
    assert o.count.tolist() == g["count"]
    assert o.off.tolist() == g["off"]
    assert o.slot_of.tolist() == g["slot_of"]
    assert o.src_of.tolist() == g["src_of"]
    assert o.xe.tolist() == g["xe"]
    np.testing.assert_allclose(o.gate.reshape(-1), g["gate"], rtol=1e-7)
    np.testing.assert_allclose(o.y, np.array(g["y"]), rtol=1e-7, atol=0)
    ye = oracle.ffn_rows(o.xe, o.off, W1, W2, [0, 1, 2], act="relu")
    assert ye.tolist() == g["ye"]


# ---------------------------------------------------------------- capacity
def test_capacity_closed_forms():
    want = {"tiny_fp32": 128, "gpt2s_moe": 640, "skewed": 1280,
            "large_chunked": 1024, "infer_stack": 256}
    for name, c in wl.CONFIGS.items():
        assert oracle.capacity(c["T"], c["E"], c["k"], c["cf"]) == want[name]
        assert c["C"] == want[name]                  # the literal the generator hands to both sides
    # exact quotients stay, anything above an integer rounds up -- also by one part in 2^52
    assert oracle.capacity(8, 4, 1, 1.0) == 2
    assert oracle.capacity(10, 4, 1, 1.0) == 3
    assert oracle.capacity(10, 4, 1, 1.2) == 3       # 1.2*10 is exactly 12.0 in double
    assert oracle.capacity(100, 8, 2, 1.1) == 28     # 27.5...
    assert oracle.capacity(3, 1, 1, 1.1) == 4        # 3.3000000000000003
    assert oracle.capacity(1 << 20, 1 << 20, 1, 1.0 + 2.0 ** -52) == 2
    assert oracle.capacity(7, 7, 1, 1.0) == 1
    assert oracle.capacity(256, 8, 2, None) == 256
    # integer cross-check where cf is a ratio of small integers: ceil(p*k*T / (q*E))
    for T, E, k, p, q in [(4096, 16, 2, 5, 4), (1000, 7, 2, 3, 2), (333, 5, 1, 1, 1), (96, 4, 2, 1, 1)]:
        assert oracle.capacity(T, E, k, p / q) == -((-p * k * T) // (q * E))


# ---------------------------------------------------------------- gate logits
def test_logits_sequential_order_and_fma():
    # (2^24 + 1) rounds back to 2^24 in fp32, so ascending order gives 0, any
    # order that adds 1 after the cancellation gives 1.
    x = np.array([[2.0 ** 24, 1.0, -(2.0 ** 24)]], np.float32)
    W = np.ones((3, 1), np.float32)
    assert oracle.gate_logits(x, W)[0, 0] == 0.0
    x = np.array([[2.0 ** 24, -(2.0 ** 24), 1.0]], np.float32)
    assert oracle.gate_logits(x, W)[0, 0] == 1.0
    # fused multiply-add: (1+2^-12)^2 = 1 + 2^-11 + 2^-24 keeps its last term only
    # if the product is not rounded before the addition.
    a = np.float32(1 + 2.0 ** -12)
    x = np.array([[-(1 + 2.0 ** -11), a]], np.float32)
    W = np.array([[1.0], [a]], np.float32)
    assert oracle.gate_logits(x, W)[0, 0] == np.float32(2.0 ** -24)


def test_logits_exact_on_small_integers_and_bias():
    rng = np.random.default_rng(3)
    x = rng.integers(-8, 9, size=(37, 50)).astype(np.float32)
    W = rng.integers(-8, 9, size=(50, 5)).astype(np.float32)
    b = rng.integers(-4, 5, size=(5,)).astype(np.float32)
    z = oracle.gate_logits(x, W, b, 0)
    assert np.array_equal(z, (x.astype(np.int64) @ W.astype(np.int64) + b).astype(np.float32))
    bt = rng.integers(-4, 5, size=(37, 5)).astype(np.float32)
    z = oracle.gate_logits(x, W, bt, 5)
    assert np.array_equal(z, (x.astype(np.int64) @ W.astype(np.int64) + bt).astype(np.float32))


def test_logits_close_to_fp64_dot():
    li = wl.make_layer(wl.scaled("gpt2s_moe", T=256), weights=False)
    z = oracle.gate_logits(li.x, li.Wg)
    ref = li.x.astype(np.float64) @ li.Wg.astype(np.float64)
    bound = li.d * 2.0 ** -24 * (np.abs(li.x).astype(np.float64) @ np.abs(li.Wg).astype(np.float64))
    assert np.all(np.abs(z - ref) <= bound)
    assert np.abs(z - ref).max() > 0  # it is an fp32 chain, not an fp64 one


# ---------------------------------------------------------------- top-k / softmax
@pytest.mark.parametrize("k", [1, 2, 3])
def test_topk_and_gate_against_library(k):
    rng = np.random.default_rng(5)
    z = rng.standard_normal((500, 16)).astype(np.float32)
    z[::7, 3] = z[::7, 9]                     # plant exact ties
    z[::11] = 0.25                            # rows where everything ties
    idx, gate = oracle.topk_softmax(z, k)
    order = np.argsort(-z.astype(np.float64), axis=1, kind="stable")[:, :k]
    assert np.array_equal(idx, order.astype(np.int32))
    assert np.array_equal(idx[:, 0], np.argmax(z, axis=1))
    p = sp_softmax(z.astype(np.float64), axis=1)
    np.testing.assert_allclose(gate, np.take_along_axis(p, order, 1), rtol=2e-7)
    assert np.all(gate > 0) and np.all(gate <= 1)
    for t in range(z.shape[0]):
        assert len(set(idx[t].tolist())) == k
    _, gr = oracle.topk_softmax(z, k, renorm=True)
    pk = np.take_along_axis(p, order, 1)
    np.testing.assert_allclose(gr, pk / pk.sum(1, keepdims=True), rtol=2e-7)


def test_softmax_full_row_sums_to_one():
    rng = np.random.default_rng(6)
    z = (rng.standard_normal((64, 8)) * 5).astype(np.float32)
    _, gate = oracle.topk_softmax(z, 8)
    np.testing.assert_allclose(gate.astype(np.float64).sum(1), 1.0, atol=1e-6)


def test_all_tie_closed_form():
    T, d, E, k, C = 40, 16, 8, 2, 12
    x = np.random.default_rng(0).standard_normal((T, d)).astype(np.float32)
    z = oracle.gate_logits(x, np.zeros((d, E), np.float32))
    assert not z.any()
    idx, gate = oracle.topk_softmax(z, k)
    assert np.array_equal(idx, np.tile(np.arange(k, dtype=np.int32), (T, 1)))
    np.testing.assert_allclose(gate, 1.0 / E, rtol=1e-7)
    count, off, slot_of, src_of = oracle.plan(idx, E, C)
    assert count.tolist() == [T, T] + [0] * (E - 2)
    assert off.tolist() == [0, C, 2 * C] + [2 * C] * (E - 2)
    so = slot_of.reshape(T, k)
    assert np.array_equal(so[:C, 0], np.arange(C)) and np.array_equal(so[:C, 1], C + np.arange(C))
    assert np.all(so[C:] == -1)


def test_round_robin_closed_form():
    # the balanced gate: token t goes to expert t mod E
    T, E = 96, 8
    bias = np.zeros((T, E), np.float32)
    bias[np.arange(T), np.arange(T) % E] = 10.0
    x = np.zeros((T, 4), np.float32)
    z = oracle.gate_logits(x, np.zeros((4, E), np.float32), bias, E)
    idx, _ = oracle.topk_softmax(z, 1)
    count, off, slot_of, src_of = oracle.plan(idx, E, T // E)
    assert np.all(count == T // E)
    t = np.arange(T)
    assert np.array_equal(slot_of, (t % E) * (T // E) + t // E)


# ---------------------------------------------------------------- plan
def plan_by_definition(idx, E, C):
    """O(n^2) restatement: position = number of earlier assignments to the same expert."""
    flat = [int(v) for v in np.asarray(idx).reshape(-1)]
    n = len(flat)
    count = [sum(1 for v in flat if v == e) for e in range(E)]
    off = [0]
    for e in range(E):
        off.append(off[-1] + min(count[e], C))
    slot_of, src_of = [], {}
    for i in range(n):
        pos = sum(1 for ii in range(i) if flat[ii] == flat[i])
        if not 0 <= flat[i] < E:              # names no expert: dispatched nowhere
            slot_of.append(-1)
        elif pos < C:
            slot_of.append(off[flat[i]] + pos)
            src_of[off[flat[i]] + pos] = i
        else:
            slot_of.append(-1)
    return count, off, slot_of, [src_of[s] for s in range(off[-1])]


@pytest.mark.parametrize("T,E,k", [(6, 3, 1), (4, 4, 1), (4, 3, 2), (3, 4, 2)])
def test_plan_brute_force_every_assignment(T, E, k):
    choices = list(itertools.permutations(range(E), k))
    for assign in itertools.product(choices, repeat=T):
        idx = np.array(assign, np.int32).reshape(T, k)
        for C in range(1, T + 1):
            got = oracle.plan(idx, E, C)
            want = plan_by_definition(idx, E, C)
            assert got[0].tolist() == want[0] and got[1].tolist() == want[1]
            assert got[2].tolist() == want[2] and got[3].tolist() == want[3]


def test_plan_skips_indices_that_name_no_expert():
    """Every assignment vector of 5 entries over {-1, 0, 1, 2 (= E, out of range)} with E = 2:
    entries outside [0, E) are in no count and take no slot; the rest are planned as if the
    others were absent."""
    E = 2
    for assign in itertools.product((-1, 0, 1, 2), repeat=5):
        idx = np.array(assign, np.int32).reshape(5, 1)
        for C in (1, 2, 5):
            count, off, slot_of, src_of = oracle.plan(idx, E, C)
            want = plan_by_definition(idx, E, C)
            assert count.tolist() == want[0] and off.tolist() == want[1]
            assert slot_of.tolist() == want[2] and src_of.tolist() == want[3]
            # the same plan as for the valid entries alone
            keep = [i for i, v in enumerate(assign) if 0 <= v < E]
            sub = oracle.plan(idx[keep], E, C) if keep else None
            if sub is not None:
                assert count.tolist() == sub[0].tolist() and off.tolist() == sub[1].tolist()
                assert slot_of[keep].tolist() == sub[2].tolist()
                assert [keep.index(i) for i in src_of.tolist()] == sub[3].tolist()
            assert all(slot_of[i] == -1 for i, v in enumerate(assign) if not 0 <= v < E)
    # a hand-worked case: E = 3, C = 1
    count, off, slot_of, src_of = oracle.plan(np.array([[2], [-1], [2], [0], [7]], np.int32), 3, 1)
    assert count.tolist() == [1, 0, 2] and off.tolist() == [0, 1, 1, 2]
    assert slot_of.tolist() == [1, -1, -1, 0, -1] and src_of.tolist() == [3, 0]


def test_plan_brute_force_through_the_gate():
    # every top-1 routing of 5 tokens over 3 experts, imposed by a one-hot bias
    T, E, d = 5, 3, 4
    x = np.random.default_rng(1).standard_normal((T, d)).astype(np.float32)
    Wg = (np.random.default_rng(2).standard_normal((d, E)) * 0.02).astype(np.float32)
    for assign in itertools.product(range(E), repeat=T):
        bias = np.zeros((T, E), np.float32)
        bias[np.arange(T), assign] = 50.0
        z = oracle.gate_logits(x, Wg, bias, E)
        idx, _ = oracle.topk_softmax(z, 1)
        assert idx.reshape(-1).tolist() == list(assign)
        got = oracle.plan(idx, E, 2)
        want = plan_by_definition(idx, E, 2)
        assert got[2].tolist() == want[2] and got[3].tolist() == want[3]


@pytest.mark.parametrize("name,T", [("tiny_fp32", 512), ("skewed", 2048), ("large_chunked", 4096)])
def test_plan_invariants(name, T):
    cfg = wl.scaled(name, T=T)
    li = wl.make_layer(cfg, weights=False)
    z = oracle.gate_logits(li.x, li.Wg, li.gate_bias, li.bias_token_stride)
    idx, gate = oracle.topk_softmax(z, li.k)
    count, off, slot_of, src_of = oracle.plan(idx, li.E, li.C)
    n = li.T * li.k
    assert count.sum() == n
    assert np.array_equal(count, np.bincount(idx.reshape(-1), minlength=li.E))
    kept = np.minimum(count, li.C)
    assert np.array_equal(np.diff(off), kept) and off[0] == 0
    A = off[-1]
    assert (slot_of >= 0).sum() == A == src_of.size
    assert np.array_equal(slot_of[src_of], np.arange(A))          # slot_of o src_of = id
    flat = idx.reshape(-1)
    for e in range(li.E):
        seg = src_of[off[e]:off[e + 1]]
        assert np.all(np.diff(seg) > 0)                           # stable, token order
        assert np.all(flat[seg] == e)
        mine = np.flatnonzero(flat == e)
        assert np.array_equal(seg, mine[:li.C])                   # exactly the first C
        assert np.all(slot_of[mine[li.C:]] == -1)
    so = slot_of.reshape(li.T, li.k)
    assert np.all((so >= 0).sum(1) <= li.k)
    if name == "skewed":
        assert (slot_of < 0).mean() > 0.2                          # the skew really overflows


# ---------------------------------------------------------------- scatter
def test_scatter_is_a_bitwise_row_copy():
    li = wl.make_layer(wl.scaled("skewed", T=1024, d=64), weights=False)
    z = oracle.gate_logits(li.x, li.Wg, li.gate_bias, 0)
    idx, _ = oracle.topk_softmax(z, li.k)
    count, off, slot_of, src_of = oracle.plan(idx, li.E, li.C)
    xe = oracle.scatter(li.x, slot_of, li.k, int(off[-1]))
    assert np.array_equal(xe.view(np.uint32), li.x[src_of // li.k].view(np.uint32))


# ---------------------------------------------------------------- activation
def test_activations():
    for v in np.linspace(-6, 6, 49):
        assert oracle.act_value(v, "gelu") == pytest.approx(
            0.5 * v * (1 + math.erf(v / math.sqrt(2))), rel=1e-15, abs=1e-300)
        assert oracle.act_value(v, "relu") == max(v, 0.0)
        assert oracle.act_value(v, "identity") == v
        assert oracle.act_value(v, "gelu_tanh") == pytest.approx(
            0.5 * v * (1 + math.tanh(math.sqrt(2 / math.pi) * (v + 0.044715 * v ** 3))), rel=1e-14)
    assert oracle.act_value(0.0, "gelu") == 0.0
    assert oracle.act_value(30.0, "gelu") == 30.0
    assert abs(oracle.act_value(-30.0, "gelu")) < 1e-100
    # standard normal CDF at 1 is 0.841344746...
    assert oracle.act_value(1.0, "gelu") == pytest.approx(0.8413447460685429, rel=1e-14)


# ---------------------------------------------------------------- FFN
def test_single_expert_is_a_dense_mlp():
    rng = np.random.default_rng(11)
    T, d, h = 33, 24, 40
    x = rng.standard_normal((T, d)).astype(np.float32)
    W1 = rng.standard_normal((1, d, h)).astype(np.float32) * 0.2
    W2 = rng.standard_normal((1, h, d)).astype(np.float32) * 0.2
    b1 = rng.standard_normal((1, h)).astype(np.float32)
    b2 = rng.standard_normal((1, d)).astype(np.float32)
    Wg = rng.standard_normal((d, 1)).astype(np.float32)
    o = oracle.moe_layer(x, Wg, W1, W2, k=1, capacity=T, act="gelu", b1=b1, b2=b2)
    assert np.all(o.gate == 1.0) and np.array_equal(o.slot_of, np.arange(T))
    pre = x.astype(np.float64) @ W1[0].astype(np.float64) + b1[0]
    H = 0.5 * pre * (1 + np.vectorize(math.erf)(pre / math.sqrt(2)))
    ref = H @ W2[0].astype(np.float64) + b2[0]
    np.testing.assert_allclose(o.y, ref, rtol=2e-7, atol=1e-7)


def test_multi_expert_ffn_rows_against_library_matmul():
    li = wl.make_layer(wl.scaled("tiny_fp32", T=200, d=24, h=56, E=5, k=2))
    z = oracle.gate_logits(li.x, li.Wg)
    idx, gate = oracle.topk_softmax(z, 2)
    count, off, slot_of, src_of = oracle.plan(idx, li.E, 60)
    xe = oracle.scatter(li.x, slot_of, 2, int(off[-1]))
    rows = np.arange(off[-1], dtype=np.int32)[::-1].copy()         # any order of rows
    ye = oracle.ffn_rows(xe, off, li.W1, li.W2, rows, act="relu")
    for e in range(li.E):
        sl = slice(off[e], off[e + 1])
        H = np.maximum(xe[sl].astype(np.float64) @ li.W1[e].astype(np.float64), 0)
        ref = H @ li.W2[e].astype(np.float64)
        got = ye[np.isin(rows, np.arange(off[e], off[e + 1]))][::-1]
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-15)


# ---------------------------------------------------------------- whole layer
def _identity_experts(E, d):
    eye = np.tile(np.eye(d, dtype=np.float32), (E, 1, 1))
    return eye, eye.copy()


def test_identity_experts_give_gate_times_x():
    rng = np.random.default_rng(13)
    T, d, E = 64, 16, 4
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = rng.standard_normal((d, E)).astype(np.float32) * 0.5
    W1, W2 = _identity_experts(E, d)
    o = oracle.moe_layer(x, Wg, W1, W2, k=1, capacity=T, act="identity")
    np.testing.assert_allclose(o.y, o.gate * x, rtol=2e-7)
    o2 = oracle.moe_layer(x, Wg, W1, W2, k=2, capacity=T, act="identity")
    np.testing.assert_allclose(o2.y, o2.gate.astype(np.float64).sum(1, keepdims=True) * x, rtol=2e-7)
    o3 = oracle.moe_layer(x, Wg, W1, W2, k=2, capacity=T, act="identity", renorm=True)
    np.testing.assert_allclose(o3.y, x, rtol=2e-7)
    # a dropped token's output is zero
    o4 = oracle.moe_layer(x, Wg, W1, W2, k=1, capacity=3, act="identity")
    dropped = o4.slot_of < 0
    assert dropped.any() and not o4.y[dropped].any()
    np.testing.assert_allclose(o4.y[~dropped], (o4.gate * x)[~dropped], rtol=2e-7)


def test_permutation_equivariance_and_linearity():
    li = wl.make_layer(wl.scaled("tiny_fp32", T=96, d=32, h=48, E=4, k=2))
    kw = dict(k=2, capacity=li.T, act="gelu")
    o = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, **kw)
    perm = np.random.default_rng(0).permutation(li.T)
    op = oracle.moe_layer(li.x[perm], li.Wg, li.W1, li.W2, **kw)
    assert np.array_equal(op.y, o.y[perm])
    assert np.array_equal(op.expert_idx, o.expert_idx[perm])
    o2 = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2 * np.float32(4.0), **kw)
    assert np.array_equal(o2.y, o.y * np.float32(4.0))


def test_token_sampling_matches_full_run():
    li = wl.make_layer(wl.scaled("skewed", T=512, d=64, h=96, E=8))
    kw = dict(k=li.k, capacity=li.C, bias=li.gate_bias, bias_stride=0)
    full = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, **kw)
    toks = np.array([0, 5, 17, 100, 101, 300, 511], np.int32)
    part = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, tokens=toks, **kw)
    assert np.array_equal(part.y, full.y[toks])
    assert (full.slot_of < 0).any()
    fully_dropped = np.flatnonzero((full.slot_of.reshape(-1, li.k) < 0).all(1))
    assert fully_dropped.size and not full.y[fully_dropped].any()

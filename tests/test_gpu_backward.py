"""Parity of the layer's backward pass with the backward oracle: every gradient within
3e-2 of the oracle gradient's RMS (max-abs); dgate much tighter (it is an fp32 dot product
of fp32 rows).  The forward's bound is 2e-2 with ONE 16-bit operand rounding on the path
(the hidden activation); the input and first-layer weight gradients pass through TWO
chained bf16 operand roundings (dye, then dP), each of relative RMS 2^-9/sqrt(3): the
expected error grows by sqrt(2), and so does the bound (2.8e-2, rounded to 3e-2)."""
import numpy as np
import pytest
import torch

import paper_2210_17223_amd as moe
import workloads as wl
from gpu_util import DEV, DeviceLayer, rel_rms_err, shape_of, upload
from oracle import bwd_oracle as bo

pytestmark = pytest.mark.gpu
TOL = 3e-2

CASES = {
    "small": wl.scaled("gpt2s_moe", T=1000, d=256, h=512),
    "ragged_dims": wl.scaled("gpt2s_moe", T=333, d=72, h=200, E=5, k=2, cf=0.8),
    "k1_e6": wl.scaled("gpt2s_moe", T=700, d=192, h=320, E=6, k=1, cf=1.0),
    "k3": wl.scaled("gpt2s_moe", T=512, d=128, h=264, E=8, k=3, cf=1.1),
    "skewed": wl.scaled("skewed", T=2048, d=256, h=384),
    "stack_layer": wl.scaled("infer_stack", T=256, d=256, h=512),
}


def run_backward(li, act="gelu", keep=False, n_chunks=1, with_oracle=True):
    """keep: the forward is moe_layer_forward_keep and hands its pre-activations to the
    backward pass; else the plain layer call, and the backward pass computes them again."""
    s = shape_of(li, act=act)
    L = DeviceLayer(li, s)
    L.layer(1)
    b = L.b
    pre = hid = None
    if keep:
        plain = {n: b[n].clone() for n in ("expert_idx", "gate", "counts", "offsets", "slot_of", "y")}
        A = int(b["offsets"][-1])
        plain["src_of"], plain["ye"] = b["src_of"][:A].clone(), b["ye"][:A * li.d].clone()
        for n in ("expert_idx", "gate", "counts", "offsets", "slot_of", "src_of", "y", "ye"):
            b[n].fill_(-3)
        pre = torch.full((moe.moe_max_rows(s) * li.h,), 9.0, dtype=torch.float16, device=DEV)
        hid = torch.full_like(pre, 5.0)
        moe.moe_layer_forward_keep(s, L.x, b["Wgp"], L.bias, L.bias_stride, b["W1p"], None, b["W2p"], None,
                                   b["expert_idx"], b["gate"], b["counts"], b["offsets"], b["slot_of"],
                                   b["src_of"], b["xe"], b["ye"], pre, hid, b["y"], b["workspace"])
        torch.cuda.synchronize()
        # same outputs as the plain layer call, bit for bit
        for n, want in plain.items():
            got = b[n][:want.numel()]
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), n
        # kept pre-activations: fp16 roundings of xe W1 (bf16 products, fp32 accumulation)
        o_pre = _oracle_pre(li, b, A)
        got_pre = pre[:A * li.h].float().cpu().numpy().reshape(A, li.h)
        rms = float(np.sqrt(np.mean(o_pre ** 2)))
        assert np.abs(got_pre - o_pre).max() <= 2.0 ** -10 * np.abs(o_pre).max() + 1e-4 * rms
        assert (pre[A * li.h:] == 9.0).all()              # rows beyond offsets[E] untouched
        # kept hidden activations: act of the fp32 accumulator, rounded to fp16
        from oracle import bwd_oracle as _bo
        o_hid = _bo.act_and_derivative(o_pre, act)[0]
        got_hid = hid[:A * li.h].float().cpu().numpy().reshape(A, li.h)
        assert np.abs(got_hid - o_hid).max() <= 2.0 ** -10 * np.abs(o_hid).max() + 1e-4 * rms
        assert (hid[A * li.h:] == 5.0).all()
    prng = np.random.Generator(np.random.PCG64(77))
    dy = prng.standard_normal((li.T, li.d)).astype(np.float32)
    W1, W2 = upload(li.W1, "bf16"), upload(li.W2, "bf16")
    f32 = lambda *shape: torch.full(shape, 7.0, dtype=torch.float32, device=DEV)
    g = dict(dx=f32(li.T * li.d), dWg=f32(li.d * li.E), dW1=f32(li.E * li.d * li.h),
             dW2=f32(li.E * li.d * li.h), dgate=f32(li.T * li.k))
    ws = torch.empty(moe.moe_backward_workspace_bytes(s), dtype=torch.uint8, device=DEV)
    moe.moe_layer_backward(s, L.x, b["Wgp"], L.bias, L.bias_stride, W1, W2, b["W1p"], b["expert_idx"],
                           b["gate"], b["offsets"], b["slot_of"], b["src_of"], b["xe"], b["ye"], pre, hid,
                           torch.from_numpy(dy).to(DEV), g["dx"], g["dWg"], g["dW1"], g["dW2"],
                           g["dgate"], ws, n_chunks=n_chunks)
    torch.cuda.synchronize()
    if not with_oracle:
        return {n: t.cpu().numpy() for n, t in g.items()}, None
    o = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy, k=li.k, capacity=li.C, act=act,
                              bias=li.gate_bias, bias_stride=li.bias_token_stride)
    assert np.array_equal(b["slot_of"].cpu().numpy(), o.fwd.slot_of)
    return {n: t.cpu().numpy() for n, t in g.items()}, o


def _oracle_pre(li, b, A):
    """xe W1 per expert in fp64 from the host inputs and the (already checked) plan."""
    off = b["offsets"].cpu().numpy()
    tok = b["src_of"][:A].cpu().numpy() // li.k
    xe = li.x.astype(np.float64)[tok]
    P = np.empty((A, li.h))
    for e in range(li.E):
        P[off[e]:off[e + 1]] = xe[off[e]:off[e + 1]] @ li.W1[e].astype(np.float64)
    return P


@pytest.mark.parametrize("keep", [False, True], ids=["recompute", "keep"])
@pytest.mark.parametrize("name", list(CASES))
def test_backward_matches_the_oracle(name, keep):
    li = wl.make_layer(CASES[name], seed=0)
    got, o = run_backward(li, keep=keep)
    T, d, E, h, k = li.T, li.d, li.E, li.h, li.k
    assert rel_rms_err(got["dgate"].reshape(T, k), o.dgate) <= 5e-3
    assert rel_rms_err(got["dx"].reshape(T, d), o.dx) <= TOL
    assert rel_rms_err(got["dWg"].reshape(d, E), o.dWg) <= TOL
    assert rel_rms_err(got["dW1"].reshape(E, d, h), o.dW1) <= TOL
    assert rel_rms_err(got["dW2"].reshape(E, h, d), o.dW2) <= TOL
    # per expert too: a wrong row range would hide in the layer-wide RMS
    for e in range(E):
        if o.fwd.count[e] == 0:
            assert not got["dW1"].reshape(E, d, h)[e].any() and not got["dW2"].reshape(E, h, d)[e].any()
        else:
            # An expert with a handful of rows has gradients that are (sums of few) outer
            # products of two bf16-rounded factors: the error of an element is relative to
            # that element (up to 2 x 2^-9 per product), and the largest elements of an
            # outer product are ~20 x its RMS.  Hence relative plus absolute bound here.
            for got_e, ref_e in ((got["dW1"].reshape(E, d, h)[e], o.dW1[e]),
                                 (got["dW2"].reshape(E, h, d)[e], o.dW2[e])):
                rms = float(np.sqrt(np.mean(ref_e ** 2)))
                assert (np.abs(got_e - ref_e) <= 2.0 ** -7 * np.abs(ref_e) + TOL * rms).all(), e
    # a fully dropped token has a zero input gradient
    dropped = (o.fwd.slot_of.reshape(T, k) < 0).all(1)
    assert not got["dx"].reshape(T, d)[dropped].any()


def test_backward_is_bitwise_reproducible():
    # fixed-order sums everywhere (no floating-point atomics): two runs, the same bits
    li = wl.make_layer(CASES[list(CASES)[0]], seed=3)
    a, _ = run_backward(li, keep=True)
    b, _ = run_backward(li, keep=True)
    for name in a:
        assert np.array_equal(a[name].view(np.uint32), b[name].view(np.uint32)), name


@pytest.mark.parametrize("keep", [False, True], ids=["recompute", "keep"])
@pytest.mark.parametrize("name", ["skewed", "k3"])
def test_chunked_backward_changes_no_bit(name, keep):
    """moe_layer_backward_chunked: every gradient is the same bits for every n_chunks, with one
    group of GEMMs per chunk (all side streams and events in use), with a few chunks per group,
    and with the default grouping (one group at these sizes)."""
    li = wl.make_layer(CASES[name], seed=2)
    ref, _ = run_backward(li, keep=keep, with_oracle=False)
    for group_rows, chunks in ((1, (2, 3, 8, 64)), (64, (4, 8)), (0, (4,))):
        before = moe.moe_tune_ffn_group_rows(group_rows)
        try:
            for n_chunks in chunks:
                got, _ = run_backward(li, keep=keep, n_chunks=n_chunks, with_oracle=False)
                for n in ref:
                    assert np.array_equal(got[n].view(np.uint32), ref[n].view(np.uint32)), (n, n_chunks, group_rows)
        finally:
            moe.moe_tune_ffn_group_rows(before)


@pytest.mark.parametrize("act", ["relu", "gelu_tanh", "identity"])
def test_backward_other_activations(act):
    li = wl.make_layer(wl.scaled("gpt2s_moe", T=400, d=128, h=256, E=4), seed=3)
    got, o = run_backward(li, act=act, keep=act != "relu")
    for n, shape in (("dx", (li.T, li.d)), ("dWg", (li.d, li.E)), ("dW1", li.W1.shape), ("dW2", li.W2.shape)):
        assert rel_rms_err(got[n].reshape(shape), getattr(o, n)) <= TOL, n


@pytest.mark.parametrize("d,h,E,T,C", [(128, 256, 8, 600, 400), (768, 1024, 64, 700, 300)],
                         ids=["small", "weight_gradient_in_256_tiles"])
def test_backward_with_empty_experts_and_gate_bias(d, h, E, T, C):
    """Two experts take every token, up to their capacity; the others stay empty and get zero
    weight gradients.  The second shape has enough 256 x 256 weight-gradient tiles (64 experts) for
    the four-wavefront kernel: experts without rows, and a contraction that ends inside a stage."""
    cfg = wl.scaled("gpt2s_moe", T=T, d=d, h=h, E=E, k=2, cf=None)
    li = wl.make_layer(cfg, seed=5)
    bias = np.zeros(li.E, np.float32)
    bias[[1, 6]] = 30.0                                  # every token picks experts 1 and 6
    li.gate_bias, li.bias_token_stride, li.C = bias, 0, C
    got, o = run_backward(li)
    assert set(np.nonzero(o.fwd.count)[0]) == {1, 6}
    for n, shape in (("dx", (li.T, li.d)), ("dWg", (li.d, li.E))):
        assert rel_rms_err(got[n].reshape(shape), getattr(o, n)) <= TOL, n
    for e in (1, 6):          # against the expert's own RMS: the empty experts' zeros tell nothing
        assert rel_rms_err(got["dW1"].reshape(li.W1.shape)[e], o.dW1[e]) <= TOL
        assert rel_rms_err(got["dW2"].reshape(li.W2.shape)[e], o.dW2[e]) <= TOL
    for e in range(E):
        if e not in (1, 6):
            assert not got["dW1"].reshape(li.W1.shape)[e].any() and not got["dW2"].reshape(li.W2.shape)[e].any()


def test_kept_buffers_come_together():
    li = wl.make_layer(wl.scaled("gpt2s_moe", T=64, d=64, h=64, E=4), seed=0)
    s = shape_of(li)
    L = DeviceLayer(li, s)
    L.layer(1)
    b = L.b
    pre = torch.zeros(moe.moe_max_rows(s) * li.h, dtype=torch.float16, device=DEV)
    W1, W2 = upload(li.W1, "bf16"), upload(li.W2, "bf16")
    f32 = lambda n: torch.zeros(n, dtype=torch.float32, device=DEV)
    ws = torch.empty(moe.moe_backward_workspace_bytes(s), dtype=torch.uint8, device=DEV)
    for keep in ((pre, None), (None, pre)):
        with pytest.raises(moe.MoeError):
            moe.moe_layer_backward(s, L.x, b["Wgp"], None, 0, W1, W2, b["W1p"], b["expert_idx"], b["gate"],
                                   b["offsets"], b["slot_of"], b["src_of"], b["xe"], b["ye"], keep[0], keep[1],
                                   f32(li.T * li.d), f32(li.T * li.d), f32(li.d * li.E), f32(li.E * li.d * li.h),
                                   f32(li.E * li.d * li.h), f32(li.T * li.k), ws)


def test_refusals():
    li = wl.make_layer(wl.CONFIGS["tiny_fp32"], seed=0)
    assert moe.moe_backward_workspace_bytes(shape_of(li)) == 0          # fp32 layers: unsupported
    s = shape_of(wl.make_layer(wl.scaled("gpt2s_moe", T=64, d=64, h=64, E=4), seed=0), renorm=True)
    assert moe.moe_backward_workspace_bytes(s) == 0

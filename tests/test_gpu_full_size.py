"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.
Integers (expert choice, counts, offsets, slots, sources) are compared in full and
bit-exactly; packed rows in full and bit-exactly; layer outputs element by element for
EVERY token (the oracle's fp64 FFN over all kept rows takes seconds to tens of seconds on
the machine's host cores), plus properties that hold at any size."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_17223_amd as moe
import workloads as wl
from gpu_util import DeviceLayer, assert_ints_equal, download, rel_rms_err, shape_of, upload

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def oracle_routing(li):
    z = oracle.gate_logits(li.x, li.Wg, li.gate_bias, li.bias_token_stride)
    idx, gate = oracle.topk_softmax(z, li.k)
    count, off, slot_of, src_of = oracle.plan(idx, li.E, li.C)
    return idx, gate, count, off, slot_of, src_of


@pytest.mark.parametrize("name,chunk_list", [("gpt2s_moe", (1,)), ("skewed", (1, 4)),
                                             ("large_chunked", (1, 4, 8))])
def test_full_size_layer(name, chunk_list):
    li = wl.make_layer(wl.CONFIGS[name], seed=0, threads=16)
    idx, gate, count, off, slot_of, src_of = oracle_routing(li)
    A = int(off[-1])
    print(f"{name}: oracle over all {li.T} tokens ({A} rows) ...", flush=True)
    o = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, k=li.k, capacity=li.C, bias=li.gate_bias,
                         bias_stride=li.bias_token_stride)
    assert np.array_equal(o.slot_of, slot_of) and o.y.shape == (li.T, li.d)
    rms = float(np.sqrt(np.mean(np.square(o.y.astype(np.float64)))))
    fully_dropped = (slot_of.reshape(li.T, li.k) < 0).all(1)

    s = shape_of(li)
    L = DeviceLayer(li, s, n_chunks=max(chunk_list))
    li.W1 = li.W2 = None                     # the device holds the packed copies now
    ref = []
    for n_chunks in chunk_list:
        # the first chunked run of the large layer with one FFN launch per chunk, the others
        # with the default grouping (two FFN launches at this size)
        before = moe.moe_tune_ffn_group_rows(1 if n_chunks == 4 else 0)
        try:
            _run_and_check(L, li, o, name, n_chunks, A, gate, src_of, rms, fully_dropped, ref)
        finally:
            moe.moe_tune_ffn_group_rows(before)
    if name == "skewed":
        assert (slot_of < 0).mean() > 0.4                  # the Zipf bias really overflows
        assert count.max() > li.C > count.min()


def _run_and_check(L, li, o, name, n_chunks, A, gate, src_of, rms, fully_dropped, ref):
    L.b["y"].fill_(float("nan"))
    L.b["xe"].zero_()
    L.layer(n_chunks)
    assert_ints_equal(L.ints(), o)
    np.testing.assert_allclose(L.b["gate"].cpu().numpy().reshape(li.T, li.k), gate, rtol=1e-6)
    xe = download(L.b["xe"]).reshape(-1, li.d)
    assert np.array_equal(xe[:A].view(np.uint32), li.x[src_of // li.k].view(np.uint32))
    y = L.b["y"].cpu().numpy().reshape(li.T, li.d)
    assert np.isfinite(y).all()
    err = float(np.abs(y - o.y).max() / rms)          # every element of every token
    print(f"{name} n_chunks={n_chunks}: max-abs err / RMS = {err:.3e}", flush=True)
    assert err <= TOL_BF16, f"{name} n_chunks={n_chunks}: max-abs err / RMS = {err}"
    assert not y[fully_dropped].any()                 # dropped tokens give zeros
    if not ref:
        ref.append(y.view(np.uint32).copy())
    else:                                              # chunking changes no output bit
        assert np.array_equal(y.view(np.uint32), ref[0]), f"n_chunks={n_chunks}"


def canon(expert_idx, slot_of, gate, T, k):
    """Per-token (expert, slot, gate) triples sorted by expert: what is unique about a
    token's routing when the order of its two choices is a near-tie."""
    e = expert_idx.reshape(T, k)
    order = np.argsort(e, axis=1, kind="stable")
    take = lambda a: np.take_along_axis(a.reshape(T, k), order, 1)
    return take(e), take(slot_of), take(gate)


def test_inference_stack():
    cfg = wl.CONFIGS["infer_stack"]
    layers = wl.make_stack(cfg, seed=0, threads=16)
    T, d, E, k = cfg["T"], cfg["d"], cfg["E"], cfg["k"]

    # oracle chain: layer l+1 reads layer l's output rounded to the activation dtype
    x_l = layers[0].x
    oracle_in, oracle_out = [], []
    for li in layers:
        li.x = x_l
        o = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, k=k, capacity=li.C, bias=li.gate_bias,
                             bias_stride=li.bias_token_stride)
        # the bias decides which two experts, the gate only their order
        assert np.array_equal(np.sort(o.expert_idx, 1), np.sort(li.forced_experts, 1))
        assert (o.slot_of >= 0).all()
        oracle_in.append(x_l)
        oracle_out.append(o)
        x_l = wl.bf16_round(o.y)

    s = shape_of(layers[0])
    dev = []
    for li in layers:
        dev.append(DeviceLayer(li, s, y_act=True))
        li.W1 = li.W2 = None

    # (a) every layer on the oracle chain's input: bit-exact routing, toleranced output
    for l, (L, o) in enumerate(zip(dev, oracle_out)):
        L.x = upload(oracle_in[l], "bf16")
        L.layer(1)
        assert_ints_equal(L.ints(), o)
        y = L.b["y"].cpu().numpy().reshape(T, d)
        assert rel_rms_err(y, o.y) <= TOL_BF16, f"layer {l}"
        y_act = download(L.b["y_act"]).reshape(T, d)
        assert np.array_equal(y_act.view(np.uint32), wl.bf16_round(y).view(np.uint32))

    # (b) the free-running stack on the device: layer l+1 reads layer l's y_act
    x_dev = upload(oracle_in[0], "bf16")
    for l, (L, o) in enumerate(zip(dev, oracle_out)):
        L.x = x_dev
        L.layer(1)
        got = L.ints()
        assert np.array_equal(got["count"], o.count) and np.array_equal(got["off"], o.off)
        ge, gs, gg = canon(got["expert_idx"], got["slot_of"], L.b["gate"].cpu().numpy(), T, k)
        we, ws, wg = canon(o.expert_idx, o.slot_of, o.gate, T, k)
        assert np.array_equal(ge, we) and np.array_equal(gs, ws)
        # the two chains' inputs differ by accumulated rounding, and a gate weight is a
        # softmax of logits: compare it absolutely
        np.testing.assert_allclose(gg, wg, rtol=0, atol=3e-2)
        # Layer 0 reads the same input on both sides: it meets the layer tolerance, max-abs,
        # exactly as in (a).  From layer 1 on the two chains' inputs differ by accumulated
        # rounding; there is no normalisation between the layers, so the activations double
        # per layer and the gate's sensitivity to an input ulp doubles with them, and the
        # output is linear in the gate weights: the max-abs bound doubles per layer, and the
        # drift of the whole output stays within the layer tolerance in the mean.
        y = L.b["y"].cpu().numpy().reshape(T, d).astype(np.float64)
        err = rel_rms_err(y, o.y)
        drift = np.linalg.norm(y - o.y) / np.linalg.norm(o.y)
        print(f"free-running layer {l}: max-abs err / RMS = {err:.3e}, Frobenius drift = {drift:.3e}", flush=True)
        assert err <= TOL_BF16 * 2 ** l, f"layer {l}: max-abs err / RMS = {err}"
        assert drift <= TOL_BF16, f"layer {l}: relative Frobenius drift {drift}"
        x_dev = L.b["y_act"].view(T, d)


def test_backward_at_the_bench_configuration():
    """Forward + backward of configuration 2 at full size, as the bench runs them (the forward
    keeps its pre-activations), against the backward oracle (every gradient, every expert)."""
    from oracle import bwd_oracle as bo
    cfg = wl.CONFIGS["gpt2s_moe"]
    li = wl.make_layer(cfg, seed=0, threads=16)
    T, d, E, h, k = li.T, li.d, li.E, li.h, li.k
    s = shape_of(li)
    L = DeviceLayer(li, s)
    b = L.b
    pre = torch.empty(moe.moe_max_rows(s) * h, dtype=torch.float16, device="cuda:0")
    hid = torch.empty_like(pre)
    moe.moe_layer_forward_keep(s, L.x, b["Wgp"], None, 0, b["W1p"], None, b["W2p"], None, b["expert_idx"],
                               b["gate"], b["counts"], b["offsets"], b["slot_of"], b["src_of"], b["xe"],
                               b["ye"], pre, hid, b["y"], b["workspace"])
    dy = np.random.Generator(np.random.PCG64(31)).standard_normal((T, d)).astype(np.float32)
    W1, W2 = upload(li.W1, "bf16"), upload(li.W2, "bf16")
    f32 = lambda n: torch.full((n,), 3.0, dtype=torch.float32, device="cuda:0")
    g = dict(dx=f32(T * d), dWg=f32(d * E), dW1=f32(E * d * h), dW2=f32(E * d * h), dgate=f32(T * k))
    ws = torch.empty(moe.moe_backward_workspace_bytes(s), dtype=torch.uint8, device="cuda:0")
    moe.moe_layer_backward(s, L.x, b["Wgp"], None, 0, W1, W2, b["W1p"], b["expert_idx"], b["gate"],
                           b["offsets"], b["slot_of"], b["src_of"], b["xe"], b["ye"], pre, hid,
                           torch.from_numpy(dy).to("cuda:0"), g["dx"], g["dWg"], g["dW1"], g["dW2"],
                           g["dgate"], ws)
    torch.cuda.synchronize()
    o = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy, k=k, capacity=li.C)
    assert np.array_equal(b["slot_of"].cpu().numpy(), o.fwd.slot_of)
    tol = 3e-2          # two chained bf16 operand roundings (see the backward parity tests)
    assert rel_rms_err(g["dgate"].cpu().numpy().reshape(T, k), o.dgate) <= 5e-3
    assert rel_rms_err(g["dx"].cpu().numpy().reshape(T, d), o.dx) <= tol
    assert rel_rms_err(g["dWg"].cpu().numpy().reshape(d, E), o.dWg) <= tol
    dW1, dW2 = g["dW1"].cpu().numpy().reshape(E, d, h), g["dW2"].cpu().numpy().reshape(E, h, d)
    for e in range(E):
        assert rel_rms_err(dW1[e], o.dW1[e]) <= tol, e
        assert rel_rms_err(dW2[e], o.dW2[e]) <= tol, e


@pytest.mark.parametrize("name,n_chunks,keep", [("skewed", 4, True), ("skewed", 1, False), ("large_chunked", 1, True)],
                         ids=["skewed-4", "skewed-recompute", "large_chunked-1"])
def test_backward_at_full_size_sampled_experts(name, n_chunks, keep):
    """Forward (keeping its pre-activations) + backward of configurations 3 and 4 at full size
    against the backward oracle: dx, dgate and dWg in full (every token), dW1 / dW2 for a sample
    of experts -- the fullest, the emptiest, and four in between -- since the oracle holds each
    expert's weight gradient in fp64.  Configuration 3 runs the chunked backward pass with two
    groups of GEMMs per pass, and once more without the kept buffers (the backward pass then
    computes the pre-activations again, with the 256 x 256 tile kernel at this size)."""
    from oracle import bwd_oracle as bo
    li = wl.make_layer(wl.CONFIGS[name], seed=0, threads=16)
    T, d, E, h, k = li.T, li.d, li.E, li.h, li.k
    s = shape_of(li)
    L = DeviceLayer(li, s)
    b = L.b
    dev = "cuda:0"
    pre = hid = None
    if keep:
        pre = torch.empty(moe.moe_max_rows(s) * h, dtype=torch.float16, device=dev)
        hid = torch.empty_like(pre)
        moe.moe_layer_forward_keep(s, L.x, b["Wgp"], L.bias, L.bias_stride, b["W1p"], None, b["W2p"], None,
                                   b["expert_idx"], b["gate"], b["counts"], b["offsets"], b["slot_of"],
                                   b["src_of"], b["xe"], b["ye"], pre, hid, b["y"], b["workspace"])
    else:
        L.layer(1)
    dy = np.random.Generator(np.random.PCG64(31)).standard_normal((T, d)).astype(np.float32)
    W1, W2 = upload(li.W1, "bf16"), upload(li.W2, "bf16")
    f32 = lambda n: torch.full((n,), 3.0, dtype=torch.float32, device=dev)
    g = dict(dx=f32(T * d), dWg=f32(d * E), dW1=f32(E * d * h), dW2=f32(E * d * h), dgate=f32(T * k))
    ws = torch.empty(moe.moe_backward_workspace_bytes(s), dtype=torch.uint8, device=dev)
    before = moe.moe_tune_ffn_group_rows(512 if n_chunks > 1 else 0)
    try:
        moe.moe_layer_backward(s, L.x, b["Wgp"], L.bias, L.bias_stride, W1, W2, b["W1p"], b["expert_idx"],
                               b["gate"], b["offsets"], b["slot_of"], b["src_of"], b["xe"], b["ye"], pre, hid,
                               torch.from_numpy(dy).to(dev), g["dx"], g["dWg"], g["dW1"], g["dW2"],
                               g["dgate"], ws, n_chunks=n_chunks)
        torch.cuda.synchronize()
    finally:
        moe.moe_tune_ffn_group_rows(before)
    counts = b["counts"].cpu().numpy()
    order = np.argsort(counts)
    experts = np.unique(np.concatenate([order[:1], order[-1:], order[np.linspace(1, E - 2, 4).astype(int)]]))
    print(f"{name}: backward oracle, weight gradients of experts {experts.tolist()} ...", flush=True)
    o = bo.moe_layer_backward(li.x, li.Wg, li.W1, li.W2, dy, k=k, capacity=li.C, bias=li.gate_bias,
                              bias_stride=li.bias_token_stride, experts=experts)
    assert np.array_equal(b["slot_of"].cpu().numpy(), o.fwd.slot_of)
    tol = 3e-2          # two chained bf16 operand roundings (see the backward parity tests)
    dx = g["dx"].cpu().numpy().reshape(T, d)
    dropped = (o.fwd.slot_of.reshape(T, k) < 0).all(1)
    assert not dx[dropped].any()
    # dx: with a skewed gate a third of the tokens are dropped outright (rows of exact zeros,
    # which lower the RMS over all rows without telling anything) and the kept rows' norms
    # spread widely (the largest 4.5 x the RMS over all): the same two roundings, applied to
    # the oracle's own fp64 values on the CPU, already give max-abs err / RMS = 4.0e-2 at
    # configuration 3.  A row's error scales with that row, so each row is held to the
    # tolerance times its own RMS (or the RMS over all rows, where that is larger), and the
    # error's RMS to 4e-3 of the gradient's (two roundings of 2^-9/sqrt(3) each: 1.6e-3, plus
    # the fp16 pre-activations' part; 2.1e-3 in that CPU emulation).
    err = dx - o.dx
    rms = float(np.sqrt(np.mean(o.dx ** 2)))
    row_scale = np.maximum(np.sqrt(np.mean(o.dx ** 2, axis=1)), rms)
    errs = dict(dgate=rel_rms_err(g["dgate"].cpu().numpy().reshape(T, k), o.dgate),
                dx_max_over_rms=float(np.abs(err).max() / rms),
                dx_max_over_row_scale=float((np.abs(err).max(1) / row_scale).max()),
                dx_rms=float(np.sqrt(np.mean(err ** 2)) / rms),
                dWg=rel_rms_err(g["dWg"].cpu().numpy().reshape(d, E), o.dWg))
    print(f"{name}: errors relative to the gradient's RMS: {errs}", flush=True)
    assert errs["dgate"] <= 5e-3 and errs["dWg"] <= tol
    assert errs["dx_max_over_row_scale"] <= tol and errs["dx_rms"] <= 4e-3
    for e in experts.tolist():
        for got_t, ref in ((g["dW1"].view(E, d, h)[e], o.dW1[e]), (g["dW2"].view(E, h, d)[e], o.dW2[e])):
            got = got_t.cpu().numpy()
            rms = float(np.sqrt(np.mean(ref ** 2)))
            # few-row experts: error relative to the element plus the layer tolerance of the RMS
            assert (np.abs(got - ref) <= 2.0 ** -7 * np.abs(ref) + tol * rms).all(), e

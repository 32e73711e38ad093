"""Parity of the HIP path against the CPU oracle, entry point by entry point and as
a whole layer, at sizes the oracle finishes in seconds.  Integers bit-exact; gate
weights within 1e-6 relative; row copies bit-exact; floating-point outputs within
2e-2 (bf16) / 1e-5 (fp32) of the oracle's output RMS, max-abs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_17223_amd as moe
import workloads as wl
from gpu_util import (DEV, DeviceLayer, assert_ints_equal, download, rel_rms_err, shape_of,
                      upload)

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "f32": 1e-5}

SMALL = {
    "tiny_fp32": wl.CONFIGS["tiny_fp32"],
    "tiny_fp32_ragged": wl.scaled("tiny_fp32", T=333, d=72, h=100, E=5, k=2, cf=0.8),
    "gpt2s_small": wl.scaled("gpt2s_moe", T=1000, d=256, h=512),
    "gpt2s_k1_e6": wl.scaled("gpt2s_moe", T=700, d=192, h=320, E=6, k=1, cf=1.0),
    "gpt2s_k3": wl.scaled("gpt2s_moe", T=512, d=128, h=264, E=8, k=3, cf=1.1),
    "skewed_small": wl.scaled("skewed", T=2048, d=256, h=384),
    "chunked_small": wl.scaled("large_chunked", T=2048, d=128, h=256),
    "stack_layer": wl.scaled("infer_stack", T=256, d=256, h=512),
}


def run_oracle(li, act="gelu", renorm=False, b1=None, b2=None, capacity=None):
    return oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, k=li.k,
                            capacity=li.C if capacity is None else capacity, act=act,
                            bias=li.gate_bias, bias_stride=li.bias_token_stride, b1=b1, b2=b2,
                            renorm=renorm)


@pytest.mark.parametrize("name", list(SMALL))
def test_entry_points_one_by_one(name):
    li = wl.make_layer(SMALL[name], seed=0)
    o = run_oracle(li)
    s = shape_of(li)
    L = DeviceLayer(li, s)
    b = L.b
    # --- gate
    moe.moe_route(s, L.x, b["Wgp"], L.bias, L.bias_stride, b["expert_idx"], b["gate"])
    torch.cuda.synchronize()
    assert np.array_equal(b["expert_idx"].cpu().numpy().reshape(li.T, li.k), o.expert_idx)
    np.testing.assert_allclose(b["gate"].cpu().numpy().reshape(li.T, li.k), o.gate, rtol=1e-6)
    # --- dispatch, fed with the oracle's expert choice
    idx = torch.from_numpy(o.expert_idx.reshape(-1)).to(DEV)
    b["xe"].zero_()
    moe.moe_dispatch(s, L.x, idx, b["counts"], b["offsets"], b["slot_of"], b["src_of"], b["xe"],
                     b["workspace"])
    torch.cuda.synchronize()
    got = L.ints()
    got["expert_idx"] = o.expert_idx
    assert_ints_equal(got, o)
    xe = download(b["xe"]).reshape(-1, li.d)
    assert np.array_equal(xe[:o.A].view(np.uint32), o.xe.view(np.uint32))
    assert not xe[o.A:].any()                         # rows past offsets[E] untouched
    # --- expert FFN on the oracle's buffer
    rows = np.arange(o.A, dtype=np.int32)
    ye_ref = oracle.ffn_rows(o.xe, o.off, li.W1, li.W2, rows)
    b["ye"].zero_()
    moe.moe_expert_ffn(s, b["xe"], b["offsets"], b["W1p"], None, b["W2p"], None, b["ye"],
                       b["workspace"])
    torch.cuda.synchronize()
    ye = b["ye"].float().cpu().numpy().reshape(-1, li.d)
    assert rel_rms_err(ye[:o.A], ye_ref) <= TOL[li.dtype]
    assert not ye[o.A:].any()
    # --- combine: both sides are handed the same expert outputs, the oracle's rounded to the
    # type the library stores them in (fp16 for bf16 layers, fp32 for fp32 layers)
    ye_in = ye_ref.astype(np.float16 if li.dtype == "bf16" else np.float32)
    ye_dev = torch.zeros_like(b["ye"])
    ye_dev[:o.A * li.d] = torch.from_numpy(ye_in.reshape(-1)).to(DEV)
    slot = torch.from_numpy(o.slot_of).to(DEV)
    gate = torch.from_numpy(o.gate.reshape(-1)).to(DEV)
    moe.moe_combine(s, ye_dev, slot, gate, b["y"])
    torch.cuda.synchronize()
    y = b["y"].cpu().numpy().reshape(li.T, li.d)
    y_ref = oracle.combine(ye_in.astype(np.float64), o.slot_of, o.gate, li.T, li.k)
    assert rel_rms_err(y, y_ref) <= 1e-5
    dropped = (o.slot_of.reshape(li.T, li.k) < 0).all(1)
    assert not y[dropped].any()


@pytest.mark.parametrize("name", ["gpt2s_small", "tiny_fp32_ragged", "skewed_small"])
def test_dispatch_skips_indices_that_name_no_expert(name):
    """moe_dispatch with padding markers (-1, E, a large value) in expert_idx: those
    assignments are in no count and take no slot; everything else as the oracle plans it."""
    li = wl.make_layer(SMALL[name], seed=6)
    z = oracle.gate_logits(li.x, li.Wg, li.gate_bias, li.bias_token_stride)
    idx, _ = oracle.topk_softmax(z, li.k)
    prng = np.random.Generator(np.random.PCG64(99))
    flat = idx.reshape(-1).copy()
    hit = prng.random(flat.size) < 0.15
    flat[hit] = prng.choice(np.array([-1, li.E, li.E + 5, -7, 2 ** 30], np.int32), size=int(hit.sum()))
    flat[:3] = (-1, li.E, -1)                             # a whole wavefront's first lanes
    idx = flat.reshape(li.T, li.k)
    count, off, slot_of, src_of = oracle.plan(idx, li.E, li.C)
    A = int(off[-1])
    xe_ref = oracle.scatter(li.x, slot_of, li.k, A)
    s = shape_of(li)
    L = DeviceLayer(li, s)
    b = L.b
    b["xe"].zero_()
    b["slot_of"].fill_(12345)
    moe.moe_dispatch(s, L.x, torch.from_numpy(flat).to(DEV), b["counts"], b["offsets"], b["slot_of"],
                     b["src_of"], b["xe"], b["workspace"])
    torch.cuda.synchronize()
    assert np.array_equal(b["counts"].cpu().numpy(), count)
    assert np.array_equal(b["offsets"].cpu().numpy(), off)
    assert np.array_equal(b["slot_of"].cpu().numpy(), slot_of)
    assert np.array_equal(b["src_of"].cpu().numpy()[:A], src_of)
    xe = download(b["xe"]).reshape(-1, li.d)
    assert np.array_equal(xe[:A].view(np.uint32), xe_ref.view(np.uint32))
    assert not xe[A:].any()


@pytest.mark.parametrize("group_rows", [1, 16, 512], ids=["ffn_per_chunk", "ffn_groups_of_16_rows", "default_groups"])
@pytest.mark.parametrize("name", list(SMALL))
def test_whole_layer_and_chunk_invariance(name, group_rows):
    """Every n_chunks gives the oracle's integers and the same output bits.  group_rows sets how
    many rows per expert an FFN launch must hold: 1 = one FFN launch per chunk (every side
    stream and event in use), 16 = a few chunks per FFN launch, 512 = the default (these small
    layers then run their FFN in one launch)."""
    li = wl.make_layer(SMALL[name], seed=1)
    o = run_oracle(li)
    s = shape_of(li)
    L = DeviceLayer(li, s, n_chunks=64, y_act=True)
    ref_bits = None
    before = moe.moe_tune_ffn_group_rows(group_rows)
    try:
        for n_chunks in (1, 2, 3, 4, 8, 64):
            for key in ("y", "ye", "xe"):
                L.b[key].zero_()
            L.layer(n_chunks)
            assert_ints_equal(L.ints(), o)
            np.testing.assert_allclose(L.b["gate"].cpu().numpy().reshape(li.T, li.k), o.gate, rtol=1e-6)
            y = L.b["y"].cpu().numpy().reshape(li.T, li.d)
            assert rel_rms_err(y, o.y) <= TOL[li.dtype], f"n_chunks={n_chunks}"
            if ref_bits is None:
                ref_bits = y.view(np.uint32).copy()
            else:                                          # chunking changes no bit of the output
                assert np.array_equal(y.view(np.uint32), ref_bits), f"n_chunks={n_chunks}"
            y_act = download(L.b["y_act"]).reshape(li.T, li.d)
            want = wl.bf16_round(y) if li.dtype == "bf16" else y
            assert np.array_equal(y_act.view(np.uint32), want.view(np.uint32))
    finally:
        moe.moe_tune_ffn_group_rows(before)


@pytest.mark.parametrize("T,d,E,k", [(600, 128, 16, 2), (9000, 64, 32, 2), (700, 72, 5, 3)],
                         ids=["chain_kernel", "register_blocks", "odd_shape"])
def test_gate_ties_go_to_the_lowest_index(T, d, E, k):
    # inputs on a coarse grid (token values in {-1, 0, 1}, matrix entries multiples of 1/2):
    # every logit is exact in fp32 whatever the order of its sum, and equal logits abound; the
    # first third of the tokens is all zeros, so all their logits tie and experts 0..k-1 win
    cfg = wl.scaled("gpt2s_moe", T=T, d=d, h=64, E=E, k=k, cf=1.0)
    li = wl.make_layer(cfg, seed=2)
    prng = np.random.Generator(np.random.PCG64(123))
    li.x = prng.integers(-1, 2, size=(T, d)).astype(np.float32)
    li.x[:T // 3] = 0.0
    li.Wg = (prng.integers(-2, 3, size=(d, E)) * 0.5).astype(np.float32)
    o = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, k=li.k, capacity=li.C)
    assert (o.expert_idx[:T // 3] == np.arange(k)).all()          # the oracle's own tie rule
    ties = 0
    z = li.x.astype(np.float64) @ li.Wg.astype(np.float64)
    for t in range(T // 3, T):
        ties += len(np.unique(z[t])) < E
    assert ties > (T - T // 3) // 10                               # ties really are common
    s = shape_of(li)
    L = DeviceLayer(li, s)
    b = L.b
    moe.moe_route(s, L.x, b["Wgp"], L.bias, L.bias_stride, b["expert_idx"], b["gate"])
    torch.cuda.synchronize()
    assert np.array_equal(b["expert_idx"].cpu().numpy().reshape(T, k), o.expert_idx)
    np.testing.assert_allclose(b["gate"].cpu().numpy().reshape(T, k), o.gate, rtol=1e-6)
    np.testing.assert_allclose(b["gate"].cpu().numpy().reshape(T, k)[:T // 3], 1.0 / E, rtol=1e-6)


@pytest.mark.parametrize("d,h,act,keep", [(384, 3072, "gelu", False), (3072, 256, "relu", False),
                                          (320, 3072, "gelu_tanh", True)],
                         ids=["first_gemm_256_tiles", "second_gemm_256_tiles", "first_gemm_kept_preactivations"])
def test_large_tile_kernel(d, h, act, keep):
    """Shapes whose expert GEMMs take the 256 x 256 tile kernel (four wavefronts of 128 x 128,
    accumulators in AGPRs, tile stored through LDS) at sizes the oracle still finishes in seconds: ragged
    row tiles, overflowing and near-empty experts (Zipf gate bias), FFN biases, and the variant
    that also keeps the pre-activations."""
    cfg = wl.scaled("skewed", T=8192, d=d, h=h, E=8, k=2, cf=1.1)
    li = wl.make_layer(cfg, seed=21, threads=8)
    prng = np.random.Generator(np.random.PCG64(5))
    b1 = (prng.standard_normal((li.E, li.h)) * 0.05).astype(np.float32)
    b2 = (prng.standard_normal((li.E, li.d)) * 0.05).astype(np.float32)
    if keep:
        b1 = b2 = None                  # the training forward takes no FFN biases
    o = run_oracle(li, act=act, b1=b1, b2=b2)
    assert (o.slot_of < 0).any() and o.count.min() < li.C // 2          # overflow and small experts
    s = shape_of(li, act=act)
    L = DeviceLayer(li, s, b1=b1, b2=b2)
    b = L.b
    if keep:
        pre = torch.full((moe.moe_max_rows(s) * li.h,), 9.0, dtype=torch.float16, device=DEV)
        hid = torch.full_like(pre, 5.0)
        moe.moe_layer_forward_keep(s, L.x, b["Wgp"], L.bias, L.bias_stride, b["W1p"], None, b["W2p"], None,
                                   b["expert_idx"], b["gate"], b["counts"], b["offsets"], b["slot_of"],
                                   b["src_of"], b["xe"], b["ye"], pre, hid, b["y"], b["workspace"])
        torch.cuda.synchronize()
        got_pre = pre[:o.A * li.h].float().cpu().numpy().reshape(o.A, li.h)
        want_pre = np.empty_like(got_pre, dtype=np.float64)
        for e in range(li.E):
            want_pre[o.off[e]:o.off[e + 1]] = o.xe[o.off[e]:o.off[e + 1]].astype(np.float64) @ li.W1[e].astype(np.float64)
        assert np.abs(got_pre - want_pre).max() <= 2.0 ** -10 * np.abs(want_pre).max() + 1e-4 * float(np.sqrt(np.mean(want_pre ** 2)))
        assert (pre[o.A * li.h:] == 9.0).all() and (hid[o.A * li.h:] == 5.0).all()
    else:
        L.layer(1)
    assert_ints_equal(L.ints(), o)
    y = b["y"].cpu().numpy().reshape(li.T, li.d)
    assert rel_rms_err(y, o.y) <= TOL["bf16"]
    rows = np.arange(o.A, dtype=np.int32)
    ye_ref = oracle.ffn_rows(o.xe, o.off, li.W1, li.W2, rows, act, b1, b2)
    ye = b["ye"].float().cpu().numpy().reshape(-1, li.d)
    assert rel_rms_err(ye[:o.A], ye_ref) <= TOL["bf16"]
    # the stand-alone FFN on the packed buffer (no gather) gives the same bits
    ye2 = torch.zeros_like(b["ye"])
    moe.moe_expert_ffn(s, b["xe"], b["offsets"], b["W1p"], L.b1, b["W2p"], L.b2, ye2, b["workspace"])
    torch.cuda.synchronize()
    assert torch.equal(ye2[:o.A * li.d].view(torch.int16), b["ye"][:o.A * li.d].view(torch.int16))
    assert not ye2[o.A * li.d:].any()


@pytest.mark.parametrize("d,h,which", [(64, 4096, 0), (128, 4096, 0), (2048, 192, 1)],
                         ids=["one_stage", "two_stages", "three_stages"])
def test_large_tile_kernel_with_a_short_contraction(d, h, which):
    """The 256 x 256 tile kernel keeps two stages of loads in flight and pairs its stages: a
    contraction of one, two or three 64-deep stages (GEMM `which` of these layers) must still come
    out right -- the loads past the last stage fetch the last stage again and are never used."""
    cfg = wl.scaled("gpt2s_moe", T=16384, d=d, h=h, E=8, k=1 if which == 0 else 2, cf=1.0)
    li = wl.make_layer(cfg, seed=33, threads=8)
    s = shape_of(li)
    assert moe.moe_expert_gemm_kernel(s, which).startswith("grouped_gemm_w4_kernel")
    o = run_oracle(li)
    L = DeviceLayer(li, s)
    L.layer(1)
    assert_ints_equal(L.ints(), o)
    y = L.b["y"].cpu().numpy().reshape(li.T, li.d)
    assert rel_rms_err(y, o.y) <= TOL["bf16"]
    rows = np.arange(o.A, dtype=np.int32)
    ye_ref = oracle.ffn_rows(o.xe, o.off, li.W1, li.W2, rows, "gelu", None, None)
    ye = L.b["ye"].float().cpu().numpy().reshape(-1, li.d)
    assert rel_rms_err(ye[:o.A], ye_ref) <= TOL["bf16"]


def test_layer_is_bitwise_reproducible():
    # no floating-point atomics on the path: the same call gives the same bits, also when
    # the output buffers hold other values beforehand and other work ran in between
    li = wl.make_layer(wl.scaled("skewed", T=3000, d=256, h=512), seed=9)
    s = shape_of(li)
    L = DeviceLayer(li, s, n_chunks=4)
    keys = ("expert_idx", "gate", "counts", "offsets", "slot_of", "xe", "ye", "y")
    ref = None
    for run, n_chunks in enumerate((1, 1, 4, 1)):
        for key in ("y", "ye", "xe", "gate"):
            L.b[key].fill_(float(run) + 0.5)
        L.layer(n_chunks)
        got = {key: L.b[key].clone() for key in keys}
        if ref is None:
            ref = got
        else:
            A = int(ref["offsets"][-1])
            for key in keys:
                a, b = got[key], ref[key]
                if key in ("xe", "ye"):                 # rows past offsets[E] belong to nobody
                    a, b = a[:A * li.d], b[:A * li.d]
                assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (run, key)


@pytest.mark.parametrize("act", ["gelu", "gelu_tanh", "relu", "identity"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_activations_biases_and_renorm(act, dtype):
    cfg = wl.scaled("gpt2s_moe", T=300, d=64, h=136, E=4, k=2, cf=1.5, dtype=dtype)
    li = wl.make_layer(cfg, seed=2)
    rng = np.random.default_rng(5)
    b1 = (rng.standard_normal((li.E, li.h)) * 0.1).astype(np.float32)
    b2 = (rng.standard_normal((li.E, li.d)) * 0.1).astype(np.float32)
    o = run_oracle(li, act=act, renorm=True, b1=b1, b2=b2)
    s = shape_of(li, act=act, renorm=True)
    L = DeviceLayer(li, s, b1=b1, b2=b2)
    L.layer(1)
    assert_ints_equal(L.ints(), o)
    np.testing.assert_allclose(L.b["gate"].cpu().numpy().reshape(li.T, li.k), o.gate, rtol=1e-6)
    assert rel_rms_err(L.b["y"].cpu().numpy().reshape(li.T, li.d), o.y) <= TOL[dtype]


def test_identity_experts_return_gate_times_x():
    # the layer-level invariant: with identity experts and k = 1 the output is gate * x
    cfg = wl.scaled("tiny_fp32", T=256, d=64, h=64, E=4, k=1, cf=None)
    li = wl.make_layer(cfg, seed=3)
    eye = np.tile(np.eye(li.d, dtype=np.float32), (li.E, 1, 1))
    li.W1, li.W2 = eye, eye.copy()
    s = shape_of(li, act="identity")
    L = DeviceLayer(li, s)
    L.layer(1)
    y = L.b["y"].cpu().numpy().reshape(li.T, li.d)
    g = L.b["gate"].cpu().numpy().reshape(li.T, 1)
    np.testing.assert_allclose(y, g * li.x, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("T,E,k,C", [(1, 1, 1, 1), (1, 4, 2, 1), (65, 3, 2, 7), (130, 64, 8, 3),
                                     (513, 2, 1, 600), (64, 8, 8, 64)])
def test_edge_shapes(T, E, k, C):
    cfg = dict(T=T, d=64, E=E, h=72, k=k, cf=None, dtype="bf16", skew=None, layers=1)
    li = wl.make_layer(cfg, seed=4)
    li.C = C
    o = run_oracle(li)
    s = shape_of(li)
    L = DeviceLayer(li, s, n_chunks=4)
    for n_chunks in (1, 4):
        L.layer(n_chunks)
        assert_ints_equal(L.ints(), o)
        assert rel_rms_err(L.b["y"].cpu().numpy().reshape(li.T, li.d), o.y) <= TOL["bf16"]


def test_everything_to_one_expert_and_empty_experts():
    # a bias that sends every token to expert 2: the other experts own no rows
    cfg = wl.scaled("gpt2s_moe", T=700, d=128, h=256, E=8, k=1, cf=None)
    li = wl.make_layer(cfg, seed=5)
    bias = np.zeros(li.E, np.float32)
    bias[2] = 40.0
    li.gate_bias, li.bias_token_stride, li.C = bias, 0, 300
    o = run_oracle(li)
    assert o.count[2] == li.T and o.A == 300
    s = shape_of(li)
    L = DeviceLayer(li, s, n_chunks=8)
    for n_chunks in (1, 8):                             # the later chunks are fully dropped
        L.b["y"].fill_(7.0)
        L.layer(n_chunks)
        assert_ints_equal(L.ints(), o)
        y = L.b["y"].cpu().numpy().reshape(li.T, li.d)
        assert rel_rms_err(y, o.y) <= TOL["bf16"]
        assert not y[300:].any()


# Shapes that select each register block of the gate kernel (tokens x experts per lane,
# chosen from T x E), few experts (lanes that only stage tiles), E not a power of two,
# a model dimension that is no multiple of the 64-column stage, both dtypes and strides of
# the bias.  The layer call also takes its plan histogram from the gate kernel, in
# segments of the gate block's tokens.
GATE_SHAPES = [
    # name,            base,        T,     d,   E,  k, cf
    ("block_1x2",      "gpt2s_moe", 8192,  128, 32, 2, 1.0),
    ("block_2x2",      "skewed",    16384, 128, 32, 2, 1.25),
    ("block_2x4",      "gpt2s_moe", 16384, 64,  64, 2, 1.0),
    ("block_4x4",      "gpt2s_moe", 32768, 64,  64, 1, 1.25),
    ("block_1x2_e3",   "gpt2s_moe", 65536, 72,  3,  2, 0.5),
    ("block_1x2_f32",  "tiny_fp32", 8192,  100, 32, 2, 1.0),
    ("e64_few_tokens", "gpt2s_moe", 100,   200, 64, 2, 2.0),
    ("e2",             "gpt2s_moe", 3000,  136, 2,  1, 0.75),
    # one chain per lane, operands streamed through the LDS ring (d a multiple of 64):
    # 32 tokens x 8 experts (one padded), 16 x 16 in fp32 (three padded), 16 x 16 ragged
    ("chain_32x8_e7",  "gpt2s_moe", 9000,  128, 7,  2, 1.0),
    ("chain_16x16_f32", "tiny_fp32", 5000, 320, 13, 2, 1.0),
    ("chain_16x16",    "gpt2s_moe", 4100,  192, 16, 1, 1.25),
    ("chain_one_stage", "gpt2s_moe", 4096, 64,  16, 2, 1.0),
]


@pytest.mark.parametrize("name,base,T,d,E,k,cf", GATE_SHAPES, ids=[g[0] for g in GATE_SHAPES])
def test_gate_register_blocks_and_segments(name, base, T, d, E, k, cf):
    cfg = wl.scaled(base, T=T, d=d, h=64, E=E, k=k, cf=cf)
    li = wl.make_layer(cfg, seed=11, threads=8)
    if name in ("block_4x4", "chain_16x16"):    # per-token bias
        prng = np.random.Generator(np.random.PCG64(5))
        li.gate_bias = (0.05 * prng.standard_normal((T, E))).astype(np.float32)
        li.bias_token_stride = E
    sample = np.unique(np.concatenate([np.arange(48), np.arange(T - 48, T),
                                       np.arange(0, T, max(1, T // 64))])).astype(np.int32)
    o = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, k=li.k, capacity=li.C, bias=li.gate_bias,
                         bias_stride=li.bias_token_stride, tokens=sample)
    s = shape_of(li)
    L = DeviceLayer(li, s, n_chunks=2)
    b = L.b
    # the gate alone
    moe.moe_route(s, L.x, b["Wgp"], L.bias, L.bias_stride, b["expert_idx"], b["gate"])
    torch.cuda.synchronize()
    assert np.array_equal(b["expert_idx"].cpu().numpy().reshape(T, k), o.expert_idx)
    np.testing.assert_allclose(b["gate"].cpu().numpy().reshape(T, k), o.gate, rtol=1e-6)
    # the layer: plan from the gate kernel's per-block histogram
    for n_chunks in (1, 2):
        b["expert_idx"].zero_()
        L.layer(n_chunks)
        assert_ints_equal(L.ints(), o)
        y = b["y"].cpu().numpy().reshape(T, d)[sample]
        assert rel_rms_err(y, o.y) <= TOL[li.dtype if li.dtype == "bf16" else "f32"]

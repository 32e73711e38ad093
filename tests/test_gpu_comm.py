"""The padded equal-split layer and the communication scheduler against their oracle
(oracle/comm_oracle.py): integers and copied rows bit for bit, y within the forward's
tolerance and bit-identical to the compact layer's, launch order exactly the policy's when
the order depends on the policy alone, and the policy's invariants on live traffic."""
import time

import numpy as np
import pytest
import torch

import paper_2210_17223_amd as moe
import workloads as wl
from gpu_util import DEV, DeviceLayer, download, rel_rms_err, shape_of
from oracle import comm_oracle as co
from oracle import moe_oracle as fo
from paper_2210_17223_amd import comm

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2

CASES = {
    "small": wl.scaled("gpt2s_moe", T=1000, d=256, h=512),
    "ragged_dims": wl.scaled("gpt2s_moe", T=333, d=72, h=200, E=5, k=2, cf=0.8),
    "k3": wl.scaled("gpt2s_moe", T=512, d=128, h=264, E=8, k=3, cf=1.1),
    "skewed": wl.scaled("skewed", T=2048, d=256, h=384),
    "fp32": wl.CONFIGS["tiny_fp32"],
}


def padded_buffers(s, n_micro):
    slots = s.E * s.capacity
    i32 = lambda n: torch.full((n,), -7, dtype=torch.int32, device=DEV)
    return dict(expert_idx=i32(s.T * s.k), gate=torch.zeros(s.T * s.k, device=DEV), counts=i32(s.E),
                slot_of=i32(s.T * s.k), src_of=i32(slots),
                xs=torch.full((slots * s.d_model,), 3.0, dtype=s.torch_dtype, device=DEV),
                xr=torch.full((slots * s.d_model,), 5.0, dtype=s.torch_dtype, device=DEV),
                ys=torch.full((slots * s.d_model,), 11.0, dtype=s.ye_dtype, device=DEV),
                yr=torch.full((slots * s.d_model,), 13.0, dtype=s.ye_dtype, device=DEV),
                y=torch.full((s.T * s.d_model,), 17.0, device=DEV),
                ws=torch.empty(moe.moe_padded_workspace_bytes(s, n_micro), dtype=torch.uint8, device=DEV))


def run_padded(L, s, n_micro, link=None, link_blocks=8):
    p = padded_buffers(s, n_micro)
    b = L.b
    moe.moe_layer_padded(s, n_micro, link, link_blocks, L.x, b["Wgp"], L.bias, L.bias_stride, b["W1p"],
                         None, b["W2p"], None, p["expert_idx"], p["gate"], p["counts"], p["slot_of"],
                         p["src_of"], p["xs"], p["xr"], p["ys"], p["yr"], p["y"], p["ws"])
    torch.cuda.synchronize()
    return p


def check_padded(li, L, s, p):
    T, d, E, k, C = li.T, li.d, li.E, li.k, li.C
    o = fo.moe_layer(li.x, li.Wg, li.W1, li.W2, k=k, capacity=C, bias=li.gate_bias,
                     bias_stride=li.bias_token_stride)
    counts, slot_of, src_of = co.padded_plan(o.expert_idx, E, C)
    assert np.array_equal(p["expert_idx"].cpu().numpy().reshape(T, k), o.expert_idx)
    assert np.array_equal(p["counts"].cpu().numpy(), counts)
    assert np.array_equal(p["slot_of"].cpu().numpy(), slot_of)
    got_src = p["src_of"].cpu().numpy()
    held = src_of >= 0
    assert np.array_equal(got_src[held], src_of[held])
    assert (got_src[~held] == -7).all()                       # empty slots: never written
    want_xs = co.pack_padded(li.x, src_of, k)
    got_xs = download(p["xs"]).reshape(E * C, d)
    assert np.array_equal(got_xs.view(np.uint32), want_xs.astype(np.float32).view(np.uint32))
    assert torch.equal(p["xr"].view(torch.int16 if li.dtype == "bf16" else torch.int32),
                       p["xs"].view(torch.int16 if li.dtype == "bf16" else torch.int32))
    # the second all-to-all carried every slot row as it was
    assert torch.equal(p["yr"].view(torch.int16), p["ys"].view(torch.int16))
    ys = p["ys"].float().cpu().numpy().reshape(E * C, d)
    assert (ys[~held] == 11.0).all()                          # rows without a token: not computed
    tol = TOL_BF16 if li.dtype == "bf16" else 1e-5
    assert rel_rms_err(p["y"].cpu().numpy().reshape(T, d), o.y) <= tol
    # the layout does not change what is computed: same bits as the compact layer
    L.layer(1)
    assert torch.equal(p["y"].view(torch.int32), L.b["y"].view(torch.int32))
    assert torch.equal(p["gate"].view(torch.int32), L.b["gate"].view(torch.int32))


@pytest.mark.parametrize("n_micro", [1, 3, 4])
@pytest.mark.parametrize("name", list(CASES))
def test_padded_layer_matches_the_oracle(name, n_micro):
    li = wl.make_layer(CASES[name], seed=0)
    s = shape_of(li)
    L = DeviceLayer(li, s)
    p = run_padded(L, s, n_micro)
    check_padded(li, L, s, p)


def test_padded_layer_with_empty_experts_and_overflowing_ones():
    cfg = wl.scaled("gpt2s_moe", T=600, d=128, h=256, E=8, k=2, cf=None)
    li = wl.make_layer(cfg, seed=5)
    bias = np.zeros(li.E, np.float32)
    bias[[1, 6]] = 30.0                                  # every token picks experts 1 and 6 ...
    li.gate_bias, li.bias_token_stride, li.C = bias, 0, 400      # ... which hold 400 of the 600
    s = shape_of(li)
    L = DeviceLayer(li, s)
    for n_micro in (1, 5):
        p = run_padded(L, s, n_micro)
        check_padded(li, L, s, p)
        counts = p["counts"].cpu().numpy()
        assert sorted(np.nonzero(counts)[0]) == [1, 6] and (counts[[1, 6]] == 600).all()
        assert (p["slot_of"].cpu().numpy() < 0).sum() == 2 * 200


def test_padded_layer_with_as_many_micro_ops_as_slots_and_a_wide_link():
    li = wl.make_layer(wl.scaled("gpt2s_moe", T=96, d=64, h=128, E=4, k=2, cf=1.0), seed=2)
    s = shape_of(li)
    assert li.C == 48
    L = DeviceLayer(li, s)
    check_padded(li, L, s, run_padded(L, s, 48, link_blocks=64))
    with pytest.raises(moe.MoeError):
        run_padded(L, s, 49)


def test_padded_layer_through_a_scheduler_that_also_carries_allreduce_traffic():
    li = wl.make_layer(CASES["small"], seed=1)
    s = shape_of(li)
    L = DeviceLayer(li, s)
    grad = torch.randn(8 << 20, device=DEV)                   # 32 MiB "gradient"
    out = torch.zeros_like(grad)
    for policy in (comm.ARRIVAL_ORDER, comm.PRIORITY):
        c = comm.moe_comm_create(policy, 8, 2)
        try:
            out.zero_()
            ar = comm.moe_comm_submit(c, comm.ALLREDUCE, grad, out, 1, grad.numel() // 4, 16, 16)
            comm.moe_comm_post(c, ar, 0, 16)
            p = run_padded(L, s, 4, link=c)
            comm.moe_comm_finish(c, ar)
            check_padded(li, L, s, p)
            assert torch.equal(out, grad)
            log = comm.moe_comm_log(c)
            co.check_log(log, policy)
            a2a = [(r["op"], r["micro"]) for r in log if r["kind"] == comm.ALL_TO_ALL]
            assert len(a2a) == 8 and len([r for r in log if r["kind"] == comm.ALLREDUCE]) == 16
        finally:
            comm.moe_comm_destroy(c)


def _submit_batch(c, bufs):
    """Three operations handed over while the scheduler is paused: allreduce A (6 micro-ops),
    all-to-all B (3), allreduce C (2), posted in that order."""
    ids = []
    for (kind, n), (src, dst) in zip(((comm.ALLREDUCE, 6), (comm.ALL_TO_ALL, 3), (comm.ALLREDUCE, 2)), bufs):
        op = comm.moe_comm_submit(c, kind, src, dst, 2, src.numel() * 4 // 32, 16, n)
        comm.moe_comm_post(c, op, 0, n)
        ids.append(op)
    return ids


@pytest.mark.parametrize("policy", [comm.ARRIVAL_ORDER, comm.PRIORITY])
@pytest.mark.parametrize("depth", [1, 2])
def test_launch_order_of_a_batch_is_the_oracles(policy, depth):
    bufs = [(torch.randn(n, device=DEV), torch.zeros(n, device=DEV)) for n in (6000, 12000, 4096)]
    c = comm.moe_comm_create(policy, 4, depth)
    try:
        comm.moe_comm_pause(c, True)
        ids = _submit_batch(c, bufs)
        with pytest.raises(moe.MoeError):                      # nothing leaves while paused
            comm.moe_comm_wait(c, ids[1], 0, timeout_ms=50)
        comm.moe_comm_pause(c, False)
        for op in ids:
            assert comm.moe_comm_finish(c, op) >= 0.0
        log = comm.moe_comm_log(c)
    finally:
        comm.moe_comm_destroy(c)
    for src, dst in bufs:
        assert torch.equal(src, dst)
    # the oracle on the same batch: everything posted at time 0 in the same order
    micros = []
    for op, (kind, n) in zip(ids, ((co.ALLREDUCE, 6), (co.ALL_TO_ALL, 3), (co.ALLREDUCE, 2))):
        micros += [co.Micro(op, m, kind, 0, 0, 1) for m in range(n)]
    want = [(m.op, m.micro) for m in co.simulate(micros, policy, depth)]
    assert [(r["op"], r["micro"]) for r in log] == want
    co.check_log(log, policy)
    # a micro-op's bytes: rows [m*R/n, (m+1)*R/n) of both slabs
    for r in log:
        n = {ids[0]: 6, ids[1]: 3, ids[2]: 2}[r["op"]]
        rows = {ids[0]: 750, ids[1]: 1500, ids[2]: 512}[r["op"]]
        assert r["bytes"] == 2 * ((r["micro"] + 1) * rows // n - r["micro"] * rows // n) * 16


def test_all_to_all_completion_time_with_and_without_priority():
    """A 256 MiB allreduce is on a (narrow) link when a 4 MiB all-to-all becomes ready.
    Handed to the link in arrival order and uncut, the all-to-all waits for all of it; cut
    into micro-ops and prioritised it waits for at most the micro-ops already on the link."""
    grad, gout = torch.randn(64 << 20, device=DEV), torch.empty(64 << 20, device=DEV)
    tok, tout = torch.randn(1 << 20, device=DEV), torch.empty(1 << 20, device=DEV)
    side = torch.cuda.Stream()         # (a wait on the posting stream would delay the post itself)
    times = {}
    for policy, n_ar in ((comm.ARRIVAL_ORDER, 1), (comm.PRIORITY, 64)):
        c = comm.moe_comm_create(policy, 4, 1)
        try:
            warm = comm.moe_comm_submit(c, comm.ALLREDUCE, tok, tout, 1, 64, 16, 1)   # first launch: code load
            comm.moe_comm_post(c, warm, 0, 1)
            comm.moe_comm_wait(c, warm, 0, side)               # (and the side stream's first use)
            comm.moe_comm_finish(c, warm)
            torch.cuda.synchronize()
            ar = comm.moe_comm_submit(c, comm.ALLREDUCE, grad, gout, 1, grad.numel() // 4, 16, n_ar)
            comm.moe_comm_post(c, ar, 0, n_ar)
            comm.moe_comm_wait(c, ar, 0, side)                 # the allreduce has the link
            a2a = comm.moe_comm_submit(c, comm.ALL_TO_ALL, tok, tout, 1, tok.numel() // 4, 16, 2)
            comm.moe_comm_post(c, a2a, 0, 2)
            times[policy] = (comm.moe_comm_finish(c, a2a), comm.moe_comm_finish(c, ar))
            log = comm.moe_comm_log(c)
            co.check_log(log, policy)
            for r in log:                                    # the host's clock tells the same story
                assert 0 < r["posted_ns"] <= r["launched_ns"] <= r["done_ns"]
        finally:
            comm.moe_comm_destroy(c)
        assert torch.equal(gout, grad) and torch.equal(tout, tok)
    (a2a_fifo, ar_fifo), (a2a_prio, ar_prio) = times[comm.ARRIVAL_ORDER], times[comm.PRIORITY]
    print("completion times (ms): all-to-all, allreduce:", times)
    # link time is proportional to bytes: 256 MiB ahead against at most 4 MiB ahead
    assert a2a_prio < 0.5 * a2a_fifo, times
    assert ar_prio < 3.0 * ar_fifo, times                      # and the allreduce is not starved


def test_hold_keeps_allreduce_micro_ops_back():
    grad, gout = torch.randn(1 << 20, device=DEV), torch.zeros(1 << 20, device=DEV)
    c = comm.moe_comm_create(comm.PRIORITY, 4, 1)
    try:
        comm.moe_comm_hold(c, True)
        ar = comm.moe_comm_submit(c, comm.ALLREDUCE, grad, gout, 1, grad.numel() // 4, 16, 4)
        comm.moe_comm_post(c, ar, 0, 4)
        time.sleep(0.05)
        assert not [r for r in comm.moe_comm_log(c) if r["kind"] == comm.ALLREDUCE]
        with pytest.raises(moe.MoeError):
            comm.moe_comm_wait(c, ar, 0, timeout_ms=20)
        comm.moe_comm_hold(c, False)
        comm.moe_comm_finish(c, ar)
        log = comm.moe_comm_log(c)
        co.check_log(log, comm.PRIORITY)
        assert [r["kind"] for r in log] == [2, 2, 1, 1, 1, 1]
    finally:
        comm.moe_comm_destroy(c)
    assert torch.equal(gout, grad)


def test_scheduler_refusals():
    a, b = torch.zeros(1024, device=DEV), torch.zeros(1024, device=DEV)
    for bad in ((2, 4, 1), (0, 0, 1), (0, 2000, 1), (1, 4, 0), (1, 4, 5)):
        with pytest.raises(moe.MoeError):
            comm.moe_comm_create(*bad)
    c = comm.moe_comm_create(comm.PRIORITY, 4, 1)
    try:
        for slabs, rows, row_bytes, n in ((0, 4, 16, 1), (1, 0, 16, 1), (1, 4, 24, 1), (1, 4, 16, 5), (1, 4, 16, 0)):
            with pytest.raises(moe.MoeError):
                comm.moe_comm_submit(c, comm.ALLREDUCE, a, b, slabs, rows, row_bytes, n)
        with pytest.raises(moe.MoeError):
            comm.moe_comm_submit(c, comm.ALLREDUCE, a, b, 1, 4096, 16, 1)    # larger than the tensors
        op = comm.moe_comm_submit(c, comm.ALLREDUCE, a, b, 1, 256, 16, 4)
        with pytest.raises(moe.MoeError):
            comm.moe_comm_post(c, op, 3, 2)
        with pytest.raises(moe.MoeError):
            comm.moe_comm_release(c, op)                       # not fully posted
        comm.moe_comm_post(c, op, 0, 2)
        with pytest.raises(moe.MoeError):
            comm.moe_comm_post(c, op, 1, 1)                    # posted before
        comm.moe_comm_post(c, op, 2, 2)
        comm.moe_comm_release(c, op)
        with pytest.raises(moe.MoeError):
            comm.moe_comm_finish(c, op)                        # the handle is gone
        with pytest.raises(moe.MoeError):
            comm.moe_comm_wait(c, 12345, 0)
    finally:
        comm.moe_comm_destroy(c)

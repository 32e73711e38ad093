"""The layer call only enqueues kernels (and, chunked, forks and joins its side streams with
events), so it can be captured into a HIP graph and replayed: every replay must reproduce
the eager outputs bit for bit, with the program's own eager work between the replays."""
import pytest
import torch

import paper_2210_17223_amd as moe
import workloads as wl
from gpu_util import DEV, DeviceLayer, shape_of

pytestmark = pytest.mark.gpu

OUTPUTS = ("expert_idx", "gate", "counts", "offsets", "slot_of", "y")


def call(L, n_chunks):
    b = L.b
    moe.moe_layer_chunked(L.s, n_chunks, L.x, b["Wgp"], L.bias, L.bias_stride, b["W1p"], None, b["W2p"],
                          None, b["expert_idx"], b["gate"], b["counts"], b["offsets"], b["slot_of"],
                          b["src_of"], b["xe"], b["ye"], b["y"], b["y_act"], b["workspace"])


@pytest.mark.parametrize("n_chunks", [1, 4])
def test_layer_call_replays_from_a_graph(n_chunks):
    li = wl.make_layer(wl.scaled("gpt2s_moe", T=1500, d=256, h=512), seed=4)
    s = shape_of(li)
    L = DeviceLayer(li, s, n_chunks=n_chunks)
    before = moe.moe_tune_ffn_group_rows(32)   # 187 rows per expert: the 4 chunks keep 4 FFN launches
    try:
        _replay(L, li, n_chunks)
    finally:
        moe.moe_tune_ffn_group_rows(before)


def _replay(L, li, n_chunks):
    call(L, n_chunks)                       # eager: the reference, and the side streams exist
    torch.cuda.synchronize()
    want = {n: L.b[n].clone() for n in OUTPUTS}
    A = int(L.b["offsets"][-1])
    want_ye = L.b["ye"][:A * li.d].clone()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(L, n_chunks)
    for rep in range(3):
        for n in OUTPUTS:                   # eager work between the replays: spoil every output
            L.b[n].fill_(-5)
        L.b["ye"].fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in OUTPUTS:
            assert torch.equal(L.b[n].view(torch.int32), want[n].view(torch.int32)), (rep, n)
        assert torch.equal(L.b["ye"][:A * li.d].view(torch.int16), want_ye.view(torch.int16)), rep

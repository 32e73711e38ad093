"""The expert FFN with host-resident weights must give the resident expert FFN's output bit
for bit (same kernels and tiles, experts launched one after the other), for any number of
resident slots; and through it the oracle's output within the layer's tolerance."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_17223_amd as moe
import workloads as wl
from gpu_util import DEV, DeviceLayer, rel_rms_err, shape_of

pytestmark = pytest.mark.gpu

CASES = {
    "small": wl.scaled("gpt2s_moe", T=1000, d=256, h=512),
    "ragged": wl.scaled("gpt2s_moe", T=333, d=72, h=200, E=5, k=2, cf=0.8),
    "skewed": wl.scaled("skewed", T=2048, d=256, h=384),
    "stack_layer_tall": wl.scaled("infer_stack", T=256, d=512, h=2048),
}


@pytest.mark.parametrize("name", list(CASES))
def test_offloaded_ffn_equals_resident_ffn(name):
    li = wl.make_layer(CASES[name], seed=0)
    s = shape_of(li)
    L = DeviceLayer(li, s)
    L.layer(1)
    b = L.b
    want = b["ye"].clone()
    A = int(b["offsets"].cpu().numpy()[-1])
    W1h, W2h = b["W1p"].cpu().pin_memory(), b["W2p"].cpu().pin_memory()
    ws = torch.empty(moe.moe_offload_workspace_bytes(s), dtype=torch.uint8, device=DEV)
    for resident in (1, 2, 3, li.E, li.E + 5):
        staging = torch.empty(moe.moe_offload_staging_bytes(s, resident), dtype=torch.uint8, device=DEV)
        ye = torch.full_like(want, 5.0)
        for _ in range(2):                         # twice: slots and events are reused
            moe.moe_expert_ffn_offloaded(s, b["xe"], b["offsets"], W1h, W2h, None, None, ye, staging,
                                         resident, ws)
        torch.cuda.synchronize()
        assert torch.equal(ye[:A * li.d].view(torch.int16), want[:A * li.d].view(torch.int16)), resident
        got = ye.float().cpu().numpy().reshape(-1, li.d)[:A]
    # and against the oracle, on its own packed rows
    o = oracle.moe_layer(li.x, li.Wg, li.W1, li.W2, k=li.k, capacity=li.C, bias=li.gate_bias,
                         bias_stride=li.bias_token_stride)
    ref = oracle.ffn_rows(o.xe, o.off, li.W1, li.W2, np.arange(o.A, dtype=np.int32))
    assert rel_rms_err(got, ref) <= 2e-2


def test_sizes_and_refusals():
    li = wl.make_layer(wl.scaled("gpt2s_moe", T=64, d=64, h=128, E=4), seed=0)
    s = shape_of(li)
    per = 64 * 128 * 2
    assert moe.moe_offload_staging_bytes(s, 2) == 2 * 2 * per
    assert moe.moe_offload_staging_bytes(s, 9) == 4 * 2 * per          # never more slots than experts
    assert moe.moe_offload_staging_bytes(s, 0) == 0
    f32 = shape_of(wl.make_layer(wl.CONFIGS["tiny_fp32"], seed=0))
    assert moe.moe_offload_staging_bytes(f32, 2) == 0 and moe.moe_offload_workspace_bytes(f32) == 0

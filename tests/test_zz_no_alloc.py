"""moe_dispatch_static (the entry point that allocates nothing: its scratch is a static device
array) against moe_dispatch, through the raw C-ABI, bit for bit: two calls in a row on the same
GPU, the second with a smaller input, so that the shared array still holds the first call's
contents when the second one runs."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import paper_2210_17223_amd as moe
import workloads as wl
from gpu_util import DEV, upload

pytestmark = pytest.mark.gpu


def routed(cfg, seed):
    li = wl.make_layer(cfg, seed=seed, weights=False)
    z = oracle.gate_logits(li.x, li.Wg, li.gate_bias, li.bias_token_stride)
    idx, _ = oracle.topk_softmax(z, li.k)
    return li, idx


def run_both(li, idx):
    """Both entry points on the same inputs through ctypes; returns their outputs."""
    L = moe.lib()
    s = moe.Shape.make(li.T, li.d, li.E, li.h, li.k, li.C, dtype="bf16" if li.dtype == "bf16" else "f32")
    rows = moe.moe_max_rows(s)
    x = upload(li.x, li.dtype)
    e = torch.from_numpy(np.ascontiguousarray(idx.reshape(-1))).to(DEV)
    ws = torch.empty(moe.moe_workspace_bytes(s, 1), dtype=torch.uint8, device=DEV)
    out = []
    for static in (False, True):
        i32 = lambda n, fill: torch.full((n,), fill, dtype=torch.int32, device=DEV)
        b = dict(counts=i32(s.E, -5), offsets=i32(s.E + 1, -5), slot_of=i32(s.T * s.k, -5),
                 src_of=i32(rows, -5), xe=torch.zeros(rows * s.d_model, dtype=s.torch_dtype, device=DEV))
        p = lambda t: C.c_void_p(t.data_ptr())
        st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        if static:
            rc = L.moe_dispatch_static(C.byref(s), p(x), p(e), p(b["counts"]), p(b["offsets"]),
                                       p(b["slot_of"]), p(b["src_of"]), p(b["xe"]), st)
        else:
            rc = L.moe_dispatch(C.byref(s), p(x), p(e), p(b["counts"]), p(b["offsets"]),
                                p(b["slot_of"]), p(b["src_of"]), p(b["xe"]), p(ws), st)
        assert rc == 0, moe.moe_last_error()
        torch.cuda.synchronize()
        A = int(b["offsets"][-1].item())
        out.append({k: (v.view(torch.int16) if v.dtype == torch.bfloat16 else v).cpu().numpy() for k, v in b.items()})
        out[-1]["src_of"] = out[-1]["src_of"][:A]
    return out


CASES = [
    # first call large (many plan segments, separate pack kernel), second call smaller
    (wl.scaled("skewed", T=20000, d=2048, h=64), wl.scaled("gpt2s_moe", T=1000, d=256, h=64)),
    (wl.scaled("large_chunked", T=4096, d=256, h=64), wl.scaled("tiny_fp32", T=333, d=72, h=100, E=5, k=2, cf=0.8)),
]


@pytest.mark.parametrize("big,small", CASES, ids=["bf16_big_then_small", "mixed_then_fp32_ragged"])
def test_static_dispatch_equals_dispatch_twice_in_a_row(big, small):
    for cfg, seed in ((big, 3), (small, 4)):
        li, idx = routed(cfg, seed)
        ref, got = run_both(li, idx)
        for key in ("counts", "offsets", "slot_of", "src_of", "xe"):
            assert np.array_equal(ref[key], got[key]), f"{key} differs (T={li.T})"
        # and both equal the oracle's plan
        count, off, slot_of, src_of = oracle.plan(idx, li.E, li.C)
        assert np.array_equal(got["counts"], count) and np.array_equal(got["offsets"], off)
        assert np.array_equal(got["slot_of"], slot_of) and np.array_equal(got["src_of"], src_of)

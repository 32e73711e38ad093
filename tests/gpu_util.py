"""Helpers of the GPU parity tests: upload seeded inputs, run the library, fetch results."""
from __future__ import annotations

import numpy as np
import torch

import paper_2210_17223_amd as moe
import workloads as wl

DEV = "cuda:0"


def upload(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Host fp32 array -> device tensor in the layer's storage dtype (exact for bf16
    configurations because the generators already rounded the values)."""
    if dtype == "bf16":
        bits = wl.bf16_bits(a).view(np.int16).reshape(a.shape)
        return torch.from_numpy(bits).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV)


def download(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return wl.from_bf16_bits(bits).reshape(t.shape)
    return t.cpu().numpy()


def shape_of(li: wl.LayerInputs, act="gelu", renorm=False, capacity=None) -> moe.Shape:
    return moe.Shape.make(li.T, li.d, li.E, li.h, li.k, li.C if capacity is None else capacity,
                          dtype=li.dtype if li.dtype == "bf16" else "f32", act=act,
                          renorm_topk=renorm)


class DeviceLayer:
    """One layer's inputs on the device plus freshly allocated outputs and packed weights."""

    def __init__(self, li: wl.LayerInputs, s: moe.Shape, n_chunks: int = 1, y_act: bool = False,
                 b1=None, b2=None, x_dev=None):
        self.s, self.li = s, li
        self.x = upload(li.x, li.dtype) if x_dev is None else x_dev
        self.Wg = upload(li.Wg, li.dtype)
        self.bias = None if li.gate_bias is None else torch.from_numpy(li.gate_bias).to(DEV)
        self.bias_stride = li.bias_token_stride
        self.b = moe.alloc_buffers(s, n_chunks, DEV, y_act=y_act)
        self.b1 = None if b1 is None else torch.from_numpy(b1).to(DEV)
        self.b2 = None if b2 is None else torch.from_numpy(b2).to(DEV)
        moe.moe_pack_gate(s, self.Wg, self.b["Wgp"])
        if li.W1.size:
            W1, W2 = upload(li.W1, li.dtype), upload(li.W2, li.dtype)
            moe.moe_pack_weights(s, W1, W2, self.b["W1p"], self.b["W2p"])
            torch.cuda.synchronize()
            del W1, W2

    def layer(self, n_chunks: int = 1):
        b = self.b
        moe.moe_layer_chunked(self.s, n_chunks, self.x, b["Wgp"], self.bias, self.bias_stride,
                              b["W1p"], self.b1, b["W2p"], self.b2, b["expert_idx"], b["gate"],
                              b["counts"], b["offsets"], b["slot_of"], b["src_of"], b["xe"],
                              b["ye"], b["y"], b["y_act"], b["workspace"])
        torch.cuda.synchronize()

    def ints(self):
        b = self.b
        off = b["offsets"].cpu().numpy()
        A = int(off[-1])
        return dict(expert_idx=b["expert_idx"].cpu().numpy().reshape(self.s.T, self.s.k),
                    count=b["counts"].cpu().numpy(), off=off,
                    slot_of=b["slot_of"].cpu().numpy(), src_of=b["src_of"].cpu().numpy()[:A])


def rel_rms_err(got: np.ndarray, want: np.ndarray) -> float:
    """max |got - want| relative to the RMS of `want`."""
    rms = float(np.sqrt(np.mean(np.square(want.astype(np.float64)))))
    if rms == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got.astype(np.float64) - want.astype(np.float64)).max() / rms)


def assert_ints_equal(got: dict, o) -> None:
    assert np.array_equal(got["expert_idx"], o.expert_idx), "expert_idx differs"
    assert np.array_equal(got["count"], o.count), "counts differ"
    assert np.array_equal(got["off"], o.off), "offsets differ"
    assert np.array_equal(got["slot_of"], o.slot_of), "slot_of differs"
    assert np.array_equal(got["src_of"], o.src_of), "src_of differs"

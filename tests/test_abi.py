"""CPU-side checks of the C-ABI library: it loads, exports every declared entry
point, its pure host functions are right, and bad arguments are refused before
anything is enqueued (so none of this needs a GPU)."""
import ctypes as C
import os
import re

import pytest

import paper_2210_17223_amd as moe
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    syms = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not name.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        syms |= set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text))
    return sorted(syms)


def test_library_exports_every_declared_symbol():
    syms = declared_symbols()
    assert {"moe_route", "moe_dispatch", "moe_expert_ffn", "moe_combine",
            "moe_layer_chunked", "moe_path_profile", "moe_popularity_estimate",
            "moe_schedule_experts"} <= set(syms)
    L = moe.lib()
    for name in syms:
        assert hasattr(L, name), f"{name} is declared under include/ but not exported"


def test_capacity_literals_and_rounding():
    want = {"tiny_fp32": 128, "gpt2s_moe": 640, "skewed": 1280, "large_chunked": 1024,
            "infer_stack": 256}
    for name, c in wl.CONFIGS.items():
        assert moe.moe_capacity(c["T"], c["E"], c["k"], c["cf"] or 0.0) == want[name] == c["C"]
    assert moe.moe_capacity(10, 4, 1, 1.0) == 3
    assert moe.moe_capacity(8, 4, 1, 1.0) == 2
    assert moe.moe_capacity(3, 1, 1, 1.1) == 4                       # 3.3000000000000003 rounds up
    assert moe.moe_capacity(1 << 20, 1 << 20, 1, 1.0 + 2.0 ** -52) == 2
    assert moe.moe_capacity(100, 8, 2, 1.1) == 28


def test_capacity_agrees_with_the_oracle_on_a_grid():
    import oracle
    for T in (1, 7, 96, 1000, 4096, 32768):
        for E in (1, 3, 8, 64):
            for k in (1, 2, 4):
                for cf in (0.5, 1.0, 1.1, 1.2, 1.25, 2.0, 1.0 / 3.0):
                    assert moe.moe_capacity(T, E, k, cf) == max(1, oracle.capacity(T, E, k, cf)), (T, E, k, cf)


def test_sizes():
    s = moe.Shape.make(4096, 768, 16, 3072, 2, 640)
    assert moe.moe_max_rows(s) == 8192
    assert moe.moe_packed_weight_bytes(s) == 16 * 768 * 3072 * 2
    assert moe.moe_packed_gate_bytes(s) == 768 * 16 * 4
    assert moe.moe_workspace_bytes(s, 1) >= 8192 * 3072 * 2
    assert moe.moe_workspace_bytes(s, 8) >= moe.moe_workspace_bytes(s, 1) - (1 << 16)
    s2 = moe.Shape.make(100, 64, 6, 128, 2, 5, dtype="f32")
    assert moe.moe_max_rows(s2) == 30
    assert moe.moe_packed_gate_bytes(s2) == 128 * 8 * 4      # d padded to 128, E to a power of two


@pytest.mark.parametrize("kw,frag", [
    (dict(E=65), "at most 64"),
    (dict(k=9, E=16), "at most 8"),
    (dict(k=5, E=4), "exceeds"),
    (dict(d_model=100), "multiples of 16"),
    (dict(T=0), ">= 1"),
    (dict(capacity=0), ">= 1"),
])
def test_bad_shapes_are_refused(kw, frag):
    base = dict(T=64, d_model=64, E=4, d_ff=128, k=2, capacity=32)
    base.update(kw)
    s = moe.Shape.make(**base)
    assert moe.moe_workspace_bytes(s, 1) == 0
    assert frag in moe.moe_last_error()


def test_null_and_misaligned_pointers_are_refused_before_any_launch():
    s = moe.Shape.make(64, 64, 4, 128, 2, 32)
    L = moe.lib()
    z = C.c_void_p(0)
    ok = C.c_void_p(4096)
    odd = C.c_void_p(4100)
    assert L.moe_route(C.byref(s), z, ok, z, 0, ok, ok, z) == 1
    assert "x is NULL" in moe.moe_last_error()
    assert L.moe_route(C.byref(s), odd, ok, z, 0, ok, ok, z) == 1
    assert L.moe_route(C.byref(s), ok, ok, ok, 3, ok, ok, z) == 1
    assert "bias_token_stride" in moe.moe_last_error()
    assert L.moe_combine(C.byref(s), ok, ok, ok, z, z, z) == 1
    assert L.moe_dispatch(C.byref(s), ok, ok, ok, ok, ok, ok, ok, z, z) == 1
    assert L.moe_expert_ffn(C.byref(s), ok, ok, z, z, ok, z, ok, ok, z) == 1
    args = [ok] * 16
    assert L.moe_layer_chunked(C.byref(s), 0, ok, ok, z, 0, *args) == 1
    assert "n_chunks" in moe.moe_last_error()
    assert L.moe_layer_chunked(C.byref(s), 65, ok, ok, z, 0, *args) == 1
    assert L.moe_route(None, ok, ok, z, 0, ok, ok, z) == 1


def test_static_dispatch_refuses_what_does_not_fit_its_array():
    """The entry point that allocates nothing rejects a plan larger than its static scratch
    array before anything is enqueued (so this needs no GPU)."""
    L = moe.lib()
    assert moe.moe_dispatch_static_limit() == 4 << 20
    s = moe.Shape.make(1 << 21, 64, 4, 64, 1, 1 << 21, dtype="bf16")   # 32768 segments of 256 bytes
    buf = (C.c_char * 64)()
    p = C.c_void_p((C.addressof(buf) + 15) // 16 * 16)
    rc = L.moe_dispatch_static(C.byref(s), p, p, p, p, p, p, p, None)
    assert rc == 2 and "static array holds" in moe.moe_last_error()
    rc = L.moe_dispatch_static(C.byref(s), None, p, p, p, p, p, p, None)
    assert rc == 1


def test_expert_gemm_kernel_names_the_kernel_and_its_tile():
    """moe_expert_gemm_kernel is host logic only: the large layer takes the 256 x 256 four-wavefront
    kernel for both GEMMs, the GPT-2-small layer the 128-row tiles of the general kernel."""
    big = wl.CONFIGS["large_chunked"]
    s = moe.Shape.make(big["T"], big["d"], big["E"], big["h"], big["k"], big["C"], dtype="bf16", act="gelu")
    assert moe.moe_expert_gemm_kernel(s, 0) == "grouped_gemm_w4_kernel 256x256"
    assert moe.moe_expert_gemm_kernel(s, 1) == "grouped_gemm_w4_kernel 256x256"
    small = wl.CONFIGS["gpt2s_moe"]
    s2 = moe.Shape.make(small["T"], small["d"], small["E"], small["h"], small["k"], small["C"], dtype="bf16", act="gelu")
    assert moe.moe_expert_gemm_kernel(s2, 0).startswith("grouped_gemm_mfma_kernel 128x")
    tiny = wl.CONFIGS["tiny_fp32"]
    s3 = moe.Shape.make(tiny["T"], tiny["d"], tiny["E"], tiny["h"], tiny["k"], tiny["C"], dtype="f32", act="gelu")
    with pytest.raises(moe.MoeError):
        moe.moe_expert_gemm_kernel(s3, 0)
    with pytest.raises(moe.MoeError):
        moe.moe_expert_gemm_kernel(s, 2)

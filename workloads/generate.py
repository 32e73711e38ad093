"""Input recipes for the five benchmark configurations.

Every buffer is drawn in fp32 from numpy's PCG64 and, for bf16 configurations,
rounded to nearest-even bf16 and kept as fp32 holding exactly those bits, so the
CPU oracle (fp32 arrays) and the GPU path (bf16 arrays) see identical values.

Expert weights are drawn per expert from child seeds so that generation can run
on several threads and still be independent of the thread count.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional

import numpy as np

# Paper context: MoE layer = gating network + E expert FFNs (Sec. 2.1); training
# uses top-2 and inference top-1/2 gates (Sec. 7.1).  The sizes below are the
# benchmark's own synthetic shapes.
CONFIGS: Dict[str, dict] = {
    "tiny_fp32": dict(T=512, d=128, E=4, h=256, k=1, cf=1.0, C=128, dtype="f32",
                      skew=None, layers=1),
    "gpt2s_moe": dict(T=4096, d=768, E=16, h=3072, k=2, cf=1.25, C=640, dtype="bf16",
                      skew=None, layers=1),
    "skewed": dict(T=16384, d=1024, E=32, h=4096, k=2, cf=1.25, C=1280, dtype="bf16",
                   skew=("zipf_bias", 1.2), layers=1),
    "large_chunked": dict(T=32768, d=2048, E=64, h=8192, k=2, cf=1.0, C=1024,
                          dtype="bf16", skew=None, layers=1),
    "infer_stack": dict(T=256, d=4096, E=8, h=14336, k=2, cf=None, C=256, dtype="bf16",
                        skew=("markov", 1.0, 0.7), layers=4),
}
# `C`, the slots per expert, is an INPUT of both the library and the oracle (each also has a
# capacity function of its own, tested against these literals and against each other).


def scaled(name: str, **over) -> dict:
    """A copy of a named configuration with some sizes overridden (test sizes).  Unless the
    caller passes `C`, the copy's slot count is re-sized for its new shape."""
    cfg = dict(CONFIGS[name])
    cfg.update(over)
    if "C" not in over:
        cfg["C"] = test_slots(cfg["T"], cfg["E"], cfg["k"], cfg.get("cf"))
    return cfg


def test_slots(T: int, E: int, k: int, cf: Optional[float]) -> int:
    """Sizes the slot count of a scaled-down test input: about cf times an even share of
    the T*k assignments per expert, rounded up; cf=None gives every expert room for all
    tokens.  This only picks an input; what a capacity factor MEANS is stated, and pinned,
    by the oracle's and the library's own capacity functions."""
    if cf is None:
        return int(T)
    return int(math.ceil(cf * k * T / E))


test_slots.__test__ = False     # not a pytest case, whatever module imports it


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32 values."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 values rounded to bf16 precision, returned as fp32."""
    return from_bf16_bits(bf16_bits(a)).reshape(np.shape(a))


@dataclasses.dataclass
class LayerInputs:
    cfg: dict
    T: int
    d: int
    E: int
    h: int
    k: int
    C: int
    dtype: str
    x: np.ndarray            # [T, d]
    Wg: np.ndarray           # [d, E]
    W1: np.ndarray           # [E, d, h]
    W2: np.ndarray           # [E, h, d]
    gate_bias: Optional[np.ndarray] = None   # [E] (stride 0) or [T, E] (stride E)
    bias_token_stride: int = 0
    forced_experts: Optional[np.ndarray] = None  # [T, k] experts the bias imposes


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    return bf16_round(a) if dtype == "bf16" else np.ascontiguousarray(a, np.float32)


def _expert_weights(seed: int, tag: int, E: int, rows: int, cols: int,
                    dtype: str, threads: int) -> np.ndarray:
    out = np.empty((E, rows, cols), dtype=np.float32)

    def one(e: int) -> None:
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tag, e])))
        rng.standard_normal(out[e].shape, dtype=np.float32, out=out[e])
        out[e] *= np.float32(0.02)
        if dtype == "bf16":
            out[e] = bf16_round(out[e])

    if threads > 1 and E > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(one, range(E)))
    else:
        for e in range(E):
            one(e)
    return out


def zipf_bias(rng: np.random.Generator, E: int, d: int, alpha: float) -> np.ndarray:
    """Per-expert logit offset that makes expert popularity follow Zipf(alpha).

    Logits of iid N(0, sigma^2) noise behave like Gumbel noise of scale
    sigma*sqrt(6)/pi near the maximum; adding scale*ln(p_e) makes expert e win
    with probability close to p_e.
    """
    ranks = rng.permutation(E) + 1
    p = ranks.astype(np.float64) ** (-alpha)
    p /= p.sum()
    sigma = 0.02 * math.sqrt(d)
    scale = sigma * math.sqrt(6.0) / math.pi
    return (scale * np.log(p)).astype(np.float32)


def markov_experts(rng: np.random.Generator, layers: int, T: int, E: int, k: int,
                   alpha: float, stay: float) -> np.ndarray:
    """[layers, T, k] forced experts: each choice slot keeps its previous-layer
    expert with probability `stay`, otherwise draws Zipf(alpha) over a seeded
    permutation of the experts; a token's k experts are kept distinct."""
    perm = rng.permutation(E)
    p = (np.arange(E) + 1.0) ** (-alpha)
    p /= p.sum()
    out = np.empty((layers, T, k), dtype=np.int32)
    def fresh() -> int:
        return int(perm[rng.choice(E, p=p)])

    for l in range(layers):
        for t in range(T):
            for j in range(k):
                e = int(out[l - 1, t, j]) if (l > 0 and rng.random() < stay) else fresh()
                while e in out[l, t, :j]:
                    e = fresh()
                out[l, t, j] = e
    return out


def make_layer(cfg: dict, seed: int = 0, threads: int = 8,
               weights: bool = True) -> LayerInputs:
    """Draw one layer's inputs.  Draw order: x, Wg, (W1, W2 from child seeds), extras."""
    T, d, E, h, k = cfg["T"], cfg["d"], cfg["E"], cfg["h"], cfg["k"]
    dtype = cfg["dtype"]
    rng = np.random.Generator(np.random.PCG64(seed))
    x = _store(rng.standard_normal((T, d), dtype=np.float32), dtype)
    Wg = _store(rng.standard_normal((d, E), dtype=np.float32) * np.float32(0.02), dtype)
    if weights:
        W1 = _expert_weights(seed, 1, E, d, h, dtype, threads)
        W2 = _expert_weights(seed, 2, E, h, d, dtype, threads)
    else:
        W1 = np.zeros((E, 0, 0), np.float32)
        W2 = np.zeros((E, 0, 0), np.float32)
    C = int(cfg["C"]) if "C" in cfg else test_slots(T, E, k, cfg.get("cf"))
    li = LayerInputs(cfg=cfg, T=T, d=d, E=E, h=h, k=k, C=C, dtype=dtype,
                     x=x, Wg=Wg, W1=W1, W2=W2)
    skew = cfg.get("skew")
    if skew and skew[0] == "zipf_bias":
        li.gate_bias = zipf_bias(rng, E, d, skew[1])
        li.bias_token_stride = 0
    elif skew and skew[0] == "markov":
        forced = markov_experts(rng, 1, T, E, k, skew[1], skew[2])[0]
        li.gate_bias, li.forced_experts = _forced_bias(forced, E), forced
        li.bias_token_stride = E
    return li


def _forced_bias(forced: np.ndarray, E: int) -> np.ndarray:
    T, k = forced.shape
    b = np.zeros((T, E), dtype=np.float32)
    b[np.arange(T)[:, None], forced] = 64.0
    return b


def make_stack(cfg: dict, seed: int = 0, threads: int = 8) -> List[LayerInputs]:
    """Inputs of an L-layer stack (inference-shaped configuration).  Layer 0 carries
    the token embeddings; later layers' `x` is empty because their input is the
    previous layer's output.  The expert pattern is drawn before any layer runs."""
    L = cfg["layers"]
    T, E, k = cfg["T"], cfg["E"], cfg["k"]
    skew = cfg["skew"]
    prng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 77])))
    forced = markov_experts(prng, L, T, E, k, skew[1], skew[2])
    layers = []
    for l in range(L):
        c = dict(cfg)
        c["skew"] = None
        li = make_layer(c, seed=seed * 1000 + l, threads=threads)
        if l > 0:
            li.x = np.zeros((0, cfg["d"]), np.float32)
        li.gate_bias = _forced_bias(forced[l], E)
        li.bias_token_stride = E
        li.forced_experts = forced[l]
        li.cfg = cfg
        layers.append(li)
    return layers

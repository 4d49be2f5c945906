"""Seeded synthetic stand-ins for the paper's workloads.

The paper calibrates and evaluates on activations captured from real language
models (Section 4 "Implementation", Appendix D); none of those are available
here, so every input is drawn from a law with the shape the paper shows for the
three activation families of Section 3's distribution figure:

* ``prenorm``  -- post-normalisation input of Up/Gate/QKV/O: N(0,1) times a fixed
  per-channel scale ~ U(0.5, 2);
* ``swiglu``   -- input of Down in a SwiGLU block: SiLU(g)*u with g,u ~ N(0,1), a sharp
  mode at zero;
* ``laplace``  -- input with an off-zero mode (the GELU-fed Down projection the
  mode-centring section is about): Laplace(loc, scale).

Arrays are generated with ``numpy.random.default_rng(seed)``, cast once to the
16-bit storage type with round-to-nearest-even, and returned as raw ``uint16``
bit patterns so that the CPU oracle and the GPU library receive the very same
bits.  Nothing in this module centres, thresholds or multiplies activations.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

# storage dtype codes (same numbering as the C ABI and the oracle, by convention only)
F16 = 0
BF16 = 1
I8 = 2

DTYPE_NAME = {F16: "f16", BF16: "bf16", I8: "i8"}

__all__ = [
    "F16", "BF16", "I8", "DTYPE_NAME", "encode", "decode", "weights", "laplace", "prenorm",
    "swiglu", "draw_inputs", "quantize_i8", "router_logits", "top2_route", "Site", "sites",
    "SEED_W", "SEED_CALIB", "SEED_TEST",
]

SEED_W = 1000
SEED_CALIB = 2000
SEED_TEST = 3000


# --------------------------------------------------------------------------- storage casts
def _f32_to_bf16_bits(a32: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit pattern, round-to-nearest-even, NaN kept quiet."""
    u = np.ascontiguousarray(a32, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    out = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x0040), rounded)
    return out.astype(np.uint16)


def encode(a: np.ndarray, dtype: int) -> np.ndarray:
    """Cast a float array to 16-bit storage and return the raw bits (uint16)."""
    a32 = np.asarray(a, dtype=np.float32)
    if dtype == BF16:
        return _f32_to_bf16_bits(a32).reshape(a32.shape)
    if dtype == F16:
        return a32.astype(np.float16).view(np.uint16).reshape(a32.shape)
    raise ValueError(f"encode: unsupported storage dtype {dtype}")


def decode(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Raw 16-bit storage -> float32 (exact widening)."""
    b = np.asarray(bits, dtype=np.uint16)
    if dtype == BF16:
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(b.shape)
    if dtype == F16:
        return b.view(np.float16).astype(np.float32).reshape(b.shape)
    raise ValueError(f"decode: unsupported storage dtype {dtype}")


# --------------------------------------------------------------------------- draws
def weights(K: int, N: int, seed: int, dtype: int, std: float = 0.02) -> np.ndarray:
    """K-major weight matrix [K, N] ~ N(0, std^2), as 16-bit storage bits."""
    rng = np.random.default_rng(seed)
    out = np.empty((K, N), dtype=np.uint16)
    step = max(1, (1 << 24) // max(N, 1))
    for r0 in range(0, K, step):
        r1 = min(K, r0 + step)
        blk = rng.standard_normal((r1 - r0, N), dtype=np.float32) * np.float32(std)
        out[r0:r1] = encode(blk, dtype)
    return out


def laplace(n: int, K: int, seed: int, dtype: int, loc: float = 0.1, scale: float = 0.5) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return encode(rng.laplace(loc, scale, size=(n, K)), dtype)


def channel_scales(K: int, chan_seed: int) -> np.ndarray:
    """Per-channel scale c ~ U(0.5, 2), drawn once per site and then fixed."""
    return np.random.default_rng(chan_seed).uniform(0.5, 2.0, size=K)


def prenorm(n: int, K: int, seed: int, dtype: int, chan_seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    c = channel_scales(K, chan_seed)
    return encode(rng.standard_normal((n, K)) * c[None, :], dtype)


def swiglu(n: int, K: int, seed: int, dtype: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((n, K))
    u = rng.standard_normal((n, K))
    return encode(g / (1.0 + np.exp(-g)) * u, dtype)


def quantize_i8(K: int, N: int, seed: int, std: float = 0.02) -> Tuple[np.ndarray, np.ndarray]:
    """Symmetric per-output-channel int8 weights: returns (q int8 [K,N], scale fp16 bits [N]).

    scale[o] = max_i |W[i,o]| / 127 rounded to fp16; q = rne(W / scale) clipped to +-127.
    """
    rng = np.random.default_rng(seed)
    Wf = rng.standard_normal((K, N), dtype=np.float32) * np.float32(std)
    scale = (np.abs(Wf).max(axis=0) / np.float32(127.0)).astype(np.float16)
    scale = np.maximum(scale, np.float16(6e-8))
    q = np.clip(np.rint(Wf / scale.astype(np.float32)[None, :]), -127, 127).astype(np.int8)
    return q, scale.view(np.uint16)


def router_logits(n_tokens: int, n_experts: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).standard_normal((n_tokens, n_experts))


def top2_route(logits: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Top-2 experts per token (ties -> lower index) and softmax gate weights over the two."""
    order = np.argsort(-logits, axis=1, kind="stable")[:, :2]
    sel = np.take_along_axis(logits, order, axis=1)
    e = np.exp(sel - sel.max(axis=1, keepdims=True))
    return order.astype(np.int64), e / e.sum(axis=1, keepdims=True)


# --------------------------------------------------------------------------- layer sites
@dataclass
class Site:
    """One fully-connected layer of a benchmark configuration."""
    name: str
    K: int
    N: int
    wdt: int
    xdt: int
    kind: str                      # "laplace" | "prenorm" | "swiglu"
    n_calib: int
    seed_w: int
    seed_calib: int
    seed_test: int
    targets: Tuple[float, ...] = (0.5,)
    est: str = "median"            # mode estimator used at calibration: "zero" | "mean" | "median"
    extra: Dict[str, float] = field(default_factory=dict)

    def draw(self, n: int, seed: int) -> np.ndarray:
        return draw_inputs(self.kind, n, self.K, seed, self.xdt, chan_seed=self.seed_w + 500, **self.extra)

    def calib(self) -> np.ndarray:
        return self.draw(self.n_calib, self.seed_calib)

    def test_vectors(self, n: int = 64) -> np.ndarray:
        return self.draw(n, self.seed_test)

    def make_weights(self) -> np.ndarray:
        return weights(self.K, self.N, self.seed_w, self.wdt)


def draw_inputs(kind: str, n: int, K: int, seed: int, dtype: int, chan_seed: int = 0, **kw) -> np.ndarray:
    if kind == "laplace":
        return laplace(n, K, seed, dtype, **kw)
    if kind == "prenorm":
        return prenorm(n, K, seed, dtype, chan_seed)
    if kind == "swiglu":
        return swiglu(n, K, seed, dtype)
    raise ValueError(kind)


def sites(cfg: int) -> List[Site]:
    """Layer list of benchmark configuration ``cfg`` (1-based, as the configurations are numbered)."""
    w, c, t = SEED_W + cfg, SEED_CALIB + cfg, SEED_TEST + cfg
    s3 = (0.5, 0.7, 0.9)
    if cfg == 1:
        return [Site("fc_1024x4096", 1024, 4096, F16, F16, "laplace", 256, w, c, t, (0.5,), "median",
                     {"loc": 0.1, "scale": 0.5})]
    if cfg == 2:
        return [
            Site("llama_gate_up", 4096, 11008, BF16, BF16, "prenorm", 512, w, c, t, s3, "median"),
            Site("llama_down", 11008, 4096, BF16, BF16, "swiglu", 512, w + 10, c + 10, t + 10, s3, "median"),
        ]
    if cfg == 3:
        return [
            Site("mistral_qkv", 4096, 6144, BF16, BF16, "prenorm", 512, w, c, t),
            Site("mistral_o", 4096, 4096, BF16, BF16, "prenorm", 512, w + 10, c + 10, t + 10),
            Site("mistral_gate_up", 4096, 28672, BF16, BF16, "prenorm", 512, w + 20, c + 20, t + 20),
            Site("mistral_down", 14336, 4096, BF16, BF16, "swiglu", 512, w + 30, c + 30, t + 30),
        ]
    if cfg == 4:
        return [
            Site("mistral_up", 4096, 14336, BF16, BF16, "prenorm", 512, w, c, t, s3),
            Site("mistral_down", 14336, 4096, BF16, BF16, "swiglu", 512, w + 10, c + 10, t + 10, s3),
        ]
    if cfg == 5:
        out = []
        for e in range(8):
            out.append(Site(f"expert{e}_gate_up", 4096, 28672, I8, BF16, "prenorm", 512,
                            w + 100 + e, c + 100 + e, t + 100 + e, (0.4,)))
            out.append(Site(f"expert{e}_down", 14336, 4096, I8, BF16, "swiglu", 512,
                            w + 200 + e, c + 200 + e, t + 200 + e, (0.7,)))
        return out
    raise ValueError(f"unknown configuration {cfg}")

"""Deterministic generators for every buffer the tests and the benchmark use.

Random stream: numpy's counter-based Philox generator, keyed by
(seed, crc32(tensor name)); each named tensor has a stream of its own, so a
tensor's bytes do not depend on which other tensors were generated, or in what
order.  Values are drawn in float32.  For the bf16 model shapes the float32
draw is rounded to bfloat16 (round to nearest even) and handed out as uint16
bit patterns: both consumers widen the same bits.

Shapes follow the paper's two models (Section 3.1: Mistral 7B, 32 layers,
hidden 4096; Mistral NeMo 12B, 40 layers, hidden 5120, grouped-query attention
with 8 KV heads against 32 query heads, 131K vocabulary) plus small shapes for
tests.  The paper's trained weights and its prompts are not available; random
N(0, 0.02) weights and synthetic prompts stand in for them.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float
    rope_theta: float
    dtype: str  # "f32", "bf16" or "f16"

    def with_layers(self, n_layers: int) -> "ModelShape":
        return replace(self, n_layers=n_layers)

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim


SHAPES = {
    # BASELINE config 1: tiny decoder, fp32.
    "tiny_f32": ModelShape("tiny_f32", 2, 256, 4, 2, 64, 688, 1024, 1e-5, 1e4, "f32"),
    # small bf16 shapes for parity tests: several tiles, ragged splits
    "small_bf16": ModelShape("small_bf16", 3, 512, 8, 2, 128, 1408, 2048, 1e-5, 1e6, "bf16"),
    "small64_bf16": ModelShape("small64_bf16", 2, 384, 6, 2, 64, 1056, 1536, 1e-5, 1e4, "bf16"),
    # the same two shapes stored as IEEE half (the paper's own storage type, Section 6.1)
    "small_f16": ModelShape("small_f16", 3, 512, 8, 2, 128, 1408, 2048, 1e-5, 1e6, "f16"),
    "small64_f16": ModelShape("small64_f16", 2, 384, 6, 2, 64, 1056, 1536, 1e-5, 1e4, "f16"),
    # Mistral-7B shape (32 layers in full; tests and bench pick a layer count)
    "mistral7b": ModelShape("mistral7b", 32, 4096, 32, 8, 128, 14336, 32768, 1e-5, 1e6, "bf16"),
    # Mistral-NeMo-12B shape
    "nemo12b": ModelShape("nemo12b", 40, 5120, 32, 8, 128, 14336, 131072, 1e-5, 1e6, "bf16"),
}


def _rng(seed: int, name: str) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), zlib.crc32(name.encode())]))


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 values (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal(seed: int, name: str, shape, std: float = 1.0, dtype: str = "f32") -> np.ndarray:
    """N(0, std) tensor.  dtype "f32" -> float32 array; "bf16" -> uint16 bits; "f16" -> float16 array."""
    x = _rng(seed, name).standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if dtype == "f16":
        return x.astype(np.float16)
    return bf16_bits(x) if dtype == "bf16" else x


def _gain(seed: int, name: str, n: int, unit: bool) -> np.ndarray:
    # Norm gains: 1.0 for the performance configs, U(0.5, 1.5) for parity tests
    # (so that a dropped gain shows).  Gains are always float32.
    if unit:
        return np.ones(n, dtype=np.float32)
    return (0.5 + _rng(seed, name).random(n, dtype=np.float32)).astype(np.float32)


def layer_weights(shape: ModelShape, layer: int, seed: int = 0, unit_gains: bool = False) -> dict:
    """One transformer layer's weights, all matrices row-major [in, out].

    Keys: wq [d, Hq*dh], wk, wv [d, Hkv*dh], wo [Hq*dh, d], wgate, wup [d, F],
    wdown [F, d] (storage dtype of the shape), g_attn, g_mlp [d] float32.
    """
    d, F = shape.d_model, shape.d_ffn
    p = f"{shape.name}/L{layer}/"
    t = shape.dtype
    return {
        "wq": normal(seed, p + "wq", (d, shape.q_dim), 0.02, t),
        "wk": normal(seed, p + "wk", (d, shape.kv_dim), 0.02, t),
        "wv": normal(seed, p + "wv", (d, shape.kv_dim), 0.02, t),
        "wo": normal(seed, p + "wo", (shape.q_dim, d), 0.02, t),
        "wgate": normal(seed, p + "wgate", (d, F), 0.02, t),
        "wup": normal(seed, p + "wup", (d, F), 0.02, t),
        "wdown": normal(seed, p + "wdown", (F, d), 0.02, t),
        "g_attn": _gain(seed, p + "g_attn", d, unit_gains),
        "g_mlp": _gain(seed, p + "g_mlp", d, unit_gains),
    }


def head_weights(shape: ModelShape, seed: int = 0, unit_gains: bool = False,
                 embed: bool = True, unembed: bool = True) -> dict:
    """Embedding table [V, d], final norm gain [d], unembedding [d, V]."""
    out = {"g_final": _gain(seed, shape.name + "/g_final", shape.d_model, unit_gains)}
    if embed:
        out["embed"] = normal(seed, shape.name + "/embed", (shape.vocab, shape.d_model), 0.02, shape.dtype)
    if unembed:
        out["unembed"] = normal(seed, shape.name + "/unembed", (shape.d_model, shape.vocab), 0.02, shape.dtype)
    return out


def kv_fill(shape: ModelShape, layer: int, n: int, seed: int = 0):
    """Pre-filled cache rows 0..n-1 of one layer: K, V ~ N(0,1), [n, Hkv, dh]."""
    p = f"{shape.name}/L{layer}/"
    k = normal(seed, p + "kfill", (n, shape.n_kv_heads, shape.head_dim), 1.0, shape.dtype)
    v = normal(seed, p + "vfill", (n, shape.n_kv_heads, shape.head_dim), 1.0, shape.dtype)
    return k, v


def hidden_block(shape: ModelShape, rows: int, seed: int = 0) -> np.ndarray:
    """Input residual-stream block [rows, d] ~ N(0,1), float32."""
    return normal(seed, shape.name + "/hidden", (rows, shape.d_model), 1.0, "f32")


def uniform_prompt(vocab: int, n: int, seed: int = 0) -> np.ndarray:
    return _rng(seed, "prompt/uniform").integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def _mix64(*vals: int) -> int:
    # splitmix64-style integer mixer used to define the Markov chain implicitly
    h = 0x9E3779B97F4A7C15
    for v in vals:
        h = (h ^ (v & 0xFFFFFFFFFFFFFFFF)) & 0xFFFFFFFFFFFFFFFF
        h = (h + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
        h ^= h >> 30
        h = (h * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        h ^= h >> 27
        h = (h * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        h ^= h >> 31
    return h


def markov_prompt(vocab: int, n: int, rho: float, seed: int = 0) -> np.ndarray:
    """Code-like synthetic prompt: an order-3 Markov chain with verbatim repeats.

    For a context (a, b, c) the four possible successors are
    mix(seed, a, b, c, i) mod vocab, i = 0..3, taken with probabilities
    (0.55, 0.25, 0.12, 0.08).  Segments alternate: with probability rho (and
    once 64 tokens exist) a verbatim copy of an earlier span of length U[8, 64]
    is appended, else U[8, 64] fresh chain tokens.  Stands in for the paper's
    code / structured prompts (Section 6.4), whose repetitiveness is what
    n-gram speculation feeds on.
    """
    rng = _rng(seed, f"prompt/markov/{vocab}/{rho}")
    cum = np.cumsum([0.55, 0.25, 0.12, 0.08])
    toks = [int(t) for t in rng.integers(0, vocab, size=3)]
    while len(toks) < n:
        span = int(rng.integers(8, 65))
        if len(toks) >= 64 and rng.random() < rho:
            start = int(rng.integers(0, len(toks) - span + 1))
            toks.extend(toks[start:start + span])
        else:
            for _ in range(span):
                i = int(np.searchsorted(cum, rng.random(), side="right"))
                i = min(i, 3)
                toks.append(_mix64(seed, toks[-3], toks[-2], toks[-1], i) % vocab)
    return np.asarray(toks[:n], dtype=np.int32)

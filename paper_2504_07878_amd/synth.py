"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws numbers and names shapes; it contains none of the method's
arithmetic and is the one thing the CPU oracle's tests and the GPU path share.

The paper (Section 4, Section 4.2) runs a Qwen2.5-0.5B small model with an MLP router on
CommonsenseQA prompts and a larger Qwen2.5 model for routed tokens. Neither the weights,
the trained router nor the dataset items are reproduced here: every tensor is drawn from a
counter-based generator keyed by (base_seed, tensor name), with the shapes of those models.

Storage conventions
  * fp32 tensors are ``np.float32`` arrays.
  * bf16 tensors are ``np.uint16`` arrays holding the bf16 bit pattern (values are drawn in
    fp32 and rounded to nearest-even bf16 once, here, before either side sees them).
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, asdict, replace

import numpy as np

F32 = 0
BF16 = 1


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
    dtype: int
    kv_dtype: int
    tie_lm_head: int
    router_hidden: int
    threshold: float = 0.5

    def asdict(self):
        return asdict(self)

    def with_(self, **kw):
        return replace(self, **kw)


# Shapes of the three model classes the workloads use.
TINY = ModelShape("tiny", 2, 256, 4, 2, 64, 1024, 4096, 1e-6, 1e4, F32, F32, 1, 64)
SLM_0P5B = ModelShape("slm-0.5b", 24, 896, 14, 2, 64, 4864, 151936, 1e-6, 1e6, BF16, BF16, 1, 256)
LLM_7B = ModelShape("llm-7b", 28, 3584, 28, 4, 128, 18944, 152064, 1e-6, 1e6, BF16, BF16, 0, 0)
SHAPES = {s.name: s for s in (TINY, SLM_0P5B, LLM_7B)}


def _key(base_seed: int, name: str) -> int:
    h = hashlib.blake2b(f"{base_seed}:{name}".encode(), digest_size=16).digest()
    return int.from_bytes(h, "little")


def rng(base_seed: int, name: str) -> np.random.Generator:
    """Independent Philox stream for one named tensor."""
    return np.random.Generator(np.random.Philox(key=_key(base_seed, name) & ((1 << 128) - 1)))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to nearest-even bf16; returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal(base_seed: int, name: str, shape, std: float, dtype: int, mean: float = 0.0) -> np.ndarray:
    """N(mean, std^2) tensor in the given storage type (chunked so that big tensors stay cheap)."""
    g = rng(base_seed, name)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32 if dtype == F32 else np.uint16)
    step = 1 << 24
    for i in range(0, n, step):
        c = g.standard_normal(min(step, n - i), dtype=np.float32)
        if std != 1.0:
            c *= np.float32(std)
        if mean != 0.0:
            c += np.float32(mean)
        out[i:i + c.size] = c if dtype == F32 else f32_to_bf16_bits(c)
    return out.reshape(shape)


def const(shape, value: float, dtype: int) -> np.ndarray:
    a = np.full(shape, value, dtype=np.float32)
    return a if dtype == F32 else f32_to_bf16_bits(a)


def make_weights(s: ModelShape, base_seed: int, std: float = 0.02, bias_std: float = 0.0, gain_std: float = 0.0,
                 qkv_bias: bool = True, workers: int = 1) -> dict:
    """All weight tensors of a model, by name.

    Matrices ~ N(0, std^2) in [out][in] layout; RMSNorm gains = 1 (+ N(0, gain_std^2) when asked); biases = 0
    (N(0, bias_std^2) when asked). Per-layer tensors are named ``l{i}.wq`` etc. Every tensor has its own stream, so
    drawing the matrices on several threads (``workers``) gives the same values as drawing them one by one.
    """
    d, qw, kvw, F, V = s.d_model, s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim, s.d_ffn, s.vocab
    dt = s.dtype
    w = {}
    todo = []

    def mat(name, shape):
        w[name] = None          # keeps the insertion order
        todo.append((name, shape))

    def gain(name, n):
        w[name] = normal(base_seed, name, (n,), gain_std, dt, mean=1.0) if gain_std else const((n,), 1.0, dt)

    def bias(name, n):
        w[name] = normal(base_seed, name, (n,), bias_std, dt) if bias_std else const((n,), 0.0, dt)

    mat("tok_emb", (V, d))
    if not s.tie_lm_head:
        mat("lm_head", (V, d))
    gain("final_norm", d)
    for i in range(s.n_layers):
        p = f"l{i}."
        gain(p + "ln1", d)
        mat(p + "wq", (qw, d)); mat(p + "wk", (kvw, d)); mat(p + "wv", (kvw, d))
        if qkv_bias:
            bias(p + "bq", qw); bias(p + "bk", kvw); bias(p + "bv", kvw)
        mat(p + "wo", (d, qw))
        gain(p + "ln2", d)
        mat(p + "wg", (F, d)); mat(p + "wu", (F, d)); mat(p + "wd", (d, F))
    if s.router_hidden:
        mat("r_w1", (s.router_hidden, d)); bias("r_b1", s.router_hidden)
        mat("r_w2", (s.router_hidden,)); bias("r_b2", 1)
    if workers > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(workers) as pool:
            for (name, _), a in zip(todo, pool.map(lambda t: normal(base_seed, t[0], t[1], std, dt), todo)):
                w[name] = a
    else:
        for name, shape in todo:
            w[name] = normal(base_seed, name, shape, std, dt)
    return w


def prompt_tokens(base_seed: int, name: str, n: int, vocab: int) -> np.ndarray:
    """n token ids uniform on [0, vocab)."""
    return rng(base_seed, name).integers(0, vocab, size=n, dtype=np.int32)


def prompt_lengths(base_seed: int, name: str, n: int, lo: int, hi: int) -> np.ndarray:
    """n prompt lengths uniform on [lo, hi] inclusive."""
    return rng(base_seed, name).integers(lo, hi + 1, size=n, dtype=np.int32)


def bernoulli_flags(base_seed: int, name: str, shape, p: float) -> np.ndarray:
    return (rng(base_seed, name).random(shape) < p).astype(np.int32)


def hidden_rows(base_seed: int, name: str, n: int, d: int, to_bf16_values: bool) -> np.ndarray:
    """n rows ~ N(0,1) as fp32; with to_bf16_values the values are first rounded to bf16-representable ones."""
    a = normal(base_seed, name, (n, d), 1.0, F32)
    return bf16_bits_to_f32(f32_to_bf16_bits(a)) if to_bf16_values else a


def kv_fill(base_seed: int, name: str, s: ModelShape, length: int) -> tuple[np.ndarray, np.ndarray]:
    """Synthetic K and V cache contents ~ N(0,1), layout [layer][kv_head][length][head_dim], in the cache storage type."""
    shape = (s.n_layers, s.n_kv_heads, length, s.head_dim)
    return normal(base_seed, name + ".k", shape, 1.0, s.kv_dtype), normal(base_seed, name + ".v", shape, 1.0, s.kv_dtype)

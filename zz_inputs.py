"""Seeded synthetic inputs for the ZigzagAttention hot path.

Shared by the CPU oracle's tests, the GPU parity tests and the benchmark.  This
module only *draws* numbers and describes workload shapes; it holds none of the
method's arithmetic (no softmax, no masks, no cache-slot rules).

Workload shapes follow the paper's evaluation model (Section 3.1: a Llama-3-8B
long-context model; Section 3.3: 50 % of the KV budget streaming) with N(0,1)
activations standing in for real ones.
"""
from __future__ import annotations

import random
from dataclasses import dataclass, field

import numpy as np


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even) and return
    them as float32.  Input preparation only: both the oracle and the GPU path
    consume the *same* already-rounded values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-exact float32 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def make_qkv(seed: int, batch: int, n_tokens: int, n_q_heads: int, n_kv_heads: int,
             head_dim: int, q_gain: float = 1.0, bf16: bool = True):
    """Q [B,T,Hq,D], K,V [B,T,Hkv,D] ~ N(0,1) as float32 (bf16-exact if bf16)."""
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((batch, n_tokens, n_q_heads, head_dim), dtype=np.float32) * np.float32(q_gain)
    k = rng.standard_normal((batch, n_tokens, n_kv_heads, head_dim), dtype=np.float32)
    v = rng.standard_normal((batch, n_tokens, n_kv_heads, head_dim), dtype=np.float32)
    if bf16:
        q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
    return q, k, v


def draw_layer_mask(seed: int, n_layers: int, n_streaming: int) -> np.ndarray:
    """uint8[L]: which layers are all-streaming (exactly n_streaming of them)."""
    chosen = random.Random(seed).sample(range(n_layers), n_streaming)
    m = np.zeros(n_layers, dtype=np.uint8)
    m[chosen] = 1
    return m


def draw_kvhead_mask(seed: int, n_layers: int, n_kv_heads: int, n_streaming_per_layer: int) -> np.ndarray:
    """uint8[L, Hkv]: mixed-head layout, the same number of streaming KV heads in
    every layer, which ones drawn per layer."""
    r = random.Random(seed)
    m = np.zeros((n_layers, n_kv_heads), dtype=np.uint8)
    for l in range(n_layers):
        m[l, r.sample(range(n_kv_heads), n_streaming_per_layer)] = 1
    return m


def draw_head_importances(seed: int, n_layers: int, n_kv_heads: int) -> np.ndarray:
    """float32[L, Hkv] in [0, 1]: synthetic stand-ins for converged head importances (Section 2.1),
    bimodal as trained gates are - about half the heads near 0 (below 0.2), the rest above 0.6."""
    rng = np.random.default_rng(seed)
    low = rng.random((n_layers, n_kv_heads)) < 0.5
    a = np.where(low, 0.2 * rng.random((n_layers, n_kv_heads)), 0.6 + 0.4 * rng.random((n_layers, n_kv_heads)))
    return a.astype(np.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    batch: int
    context: int          # tokens in the cache when decode attention runs
    sink: int
    window: int
    n_streaming_layers: int
    chunk: int = 0        # prefill chunk length (0: not a prefill workload)
    decode_steps: int = 0
    note: str = ""
    extra: dict = field(default_factory=dict)


# The five configurations the build is measured / checked on.
WORKLOADS = {
    "c1_tiny": Workload("c1_tiny", 2, 4, 2, 64, 1, 1024, 16, 64, 1, chunk=1024, decode_steps=8,
                        note="layer0 retrieval, layer1 streaming; prefill 1024 then 8 decode steps"),
    "c2_llama8b_32k_b1": Workload("c2_llama8b_32k_b1", 32, 32, 8, 128, 1, 32768, 64, 256, 16),
    "c3_llama8b_128k_b4": Workload("c3_llama8b_128k_b4", 32, 32, 8, 128, 4, 131072, 64, 256, 16),
    "c4_prefill_64k": Workload("c4_prefill_64k", 32, 32, 8, 128, 1, 65536, 64, 256, 16, chunk=4096),
    "c5_mha7b_32k_b8": Workload("c5_mha7b_32k_b8", 32, 32, 32, 128, 8, 32768, 64, 256, 24),
}

"""Seeded synthetic inputs for the attention workloads (numpy only).

This module holds none of the method's arithmetic: it draws standard-normal fp32
tensors from ``numpy.random.default_rng(seed)`` in the order Q, K, V and rounds them to
bf16 (round-to-nearest-even) on the host, so that the CPU oracle and the GPU path see
bit-identical inputs.  bf16 tensors are returned as ``uint16`` bit patterns.

The shapes are the Llama-2-7B attention shapes the paper measures (32 heads of size 128,
prompt lengths 2048 and 4096, section 3.2) plus a small parity case, a batched decode
step and a long-context GQA case; the tensors stand in for real activations.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str          # "prefill" | "decode"
    batch: int
    q_heads: int
    kv_heads: int
    seq_len: int       # prefill: S (queries == keys); decode: T cached tokens, one query
    head_dim: int
    causal: bool
    kv_int8: bool
    out_f32: bool
    seed: int

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(np.float64(self.head_dim)))

    @property
    def q_rows(self) -> int:
        return 1 if self.kind == "decode" else self.seq_len


WORKLOADS = {
    "C1": Workload("C1", "prefill", 1, 8, 8, 512, 64, True, False, True, 1),
    "C2": Workload("C2", "prefill", 1, 32, 32, 2048, 128, True, False, False, 2),
    "C3": Workload("C3", "prefill", 1, 32, 32, 4096, 128, True, True, False, 3),
    "C4": Workload("C4", "decode", 16, 32, 32, 8192, 128, False, True, False, 4),
    "C5": Workload("C5", "prefill", 1, 64, 8, 32768, 128, True, True, False, 5),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    xf, of = x.reshape(-1), out.reshape(-1)
    step = 1 << 24
    for s in range(0, xf.size, step):
        u = xf[s:s + step].view(np.uint32)
        r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        of[s:s + step] = (r >> np.uint32(16)).astype(np.uint16)
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    """One tensor of N(0,1) draws, fp32 then bf16 RNE, as uint16 bit patterns."""
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(-1)
    step = 1 << 24
    for s in range(0, flat.size, step):
        n = min(step, flat.size - s)
        flat[s:s + n] = f32_to_bf16_bits(rng.standard_normal(n, dtype=np.float32))
    return out


def make_qkv(w: Workload, seed=None):
    """(q, k, v) bf16 bit patterns: q [B,Hq,Sq,D], k and v [B,Hkv,S,D]; drawn Q, K, V."""
    rng = np.random.default_rng(w.seed if seed is None else seed)
    q = normal_bf16(rng, (w.batch, w.q_heads, w.q_rows, w.head_dim))
    k = normal_bf16(rng, (w.batch, w.kv_heads, w.seq_len, w.head_dim))
    v = normal_bf16(rng, (w.batch, w.kv_heads, w.seq_len, w.head_dim))
    return q, k, v


def make_shape(kind, batch, q_heads, kv_heads, seq_len, head_dim, causal, kv_int8, out_f32, seed,
               name="custom") -> Workload:
    return Workload(name, kind, batch, q_heads, kv_heads, seq_len, head_dim, causal, kv_int8, out_f32, seed)

"""Python face of the CPU oracle (test infrastructure; see ``slim_oracle.c``).

Two independent routes to the same definitions:

* the C library (fp64 scalar loops, OpenMP over independent rows) for sizes up to the
  benchmark shapes, and
* numpy fp64 full-matrix forms for small shapes: ``attn_full_matrix_np`` is
  softmax(Q K^T * scale + mask) V written out, ``slim_attn_rowblocks_np`` follows the
  computation order of the paper's section 2.1 (a horizontal score block over ALL keys,
  softmax over it, times V gives a slice of the output, then the next block reuses the
  same score buffer).

Inputs are numpy arrays: bf16 tensors travel as ``uint16`` bit patterns, INT8 codes as
``int8``, scales as ``float32``.
"""
import ctypes
import os

import numpy as np

from .build_oracle import LIB, build

_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        lib = ctypes.CDLL(LIB)
        c_p = ctypes.c_void_p
        lib.oracle_kv_quant_int8.argtypes = [c_p, c_p, c_p, ctypes.c_long, ctypes.c_int]
        lib.oracle_kv_quant_int8.restype = ctypes.c_int
        lib.oracle_quant_division_sweep.argtypes = [c_p, ctypes.c_int]
        lib.oracle_quant_division_sweep.restype = ctypes.c_int
        lib.oracle_attn.argtypes = [c_p, c_p, c_p, c_p, c_p, c_p] + [ctypes.c_int] * 7 + [
            ctypes.c_double, ctypes.c_int, c_p, ctypes.c_int]
        lib.oracle_attn.restype = ctypes.c_int
        lib.oracle_attn_row_probs.argtypes = [c_p] * 7 + [ctypes.c_int] * 7 + [
            ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_attn_row_probs.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ------------------------------------------------------------------ quantiser

def kv_quant_int8(x_bits: np.ndarray):
    """C oracle quantiser (section 2.2).  x_bits: [..., D] uint16 bf16 patterns.
    Returns (codes int8 [..., D], scales float32 [...])."""
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
    D = x_bits.shape[-1]
    n_rows = x_bits.size // D
    codes = np.empty(x_bits.shape, dtype=np.int8)
    scales = np.empty(x_bits.shape[:-1], dtype=np.float32)
    rc = _load().oracle_kv_quant_int8(_ptr(x_bits), _ptr(codes), _ptr(scales), n_rows, D)
    assert rc == 0
    return codes, scales


def kv_quant_int8_np(x_bits: np.ndarray):
    """The same definition in numpy float32 arithmetic (IEEE division, ``np.rint`` is
    ties-to-even)."""
    x = (np.ascontiguousarray(x_bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
    amax = np.max(np.abs(x), axis=-1)
    scale = (amax / np.float32(127.0)).astype(np.float32)
    safe = np.where(scale == 0, np.float32(1.0), scale)[..., None]
    quo = (x / safe).astype(np.float32)
    codes = np.clip(np.rint(quo), -127, 127).astype(np.int8)
    codes = np.where((scale == 0)[..., None], np.int8(0), codes)
    return codes, scale


def quant_division_sweep(amax_step: int = 1):
    """(scale mismatches, quotient mismatches, pairs visited): fp32 division against the
    fp64 quotient narrowed to fp32, over every bf16 amax and every bf16 |x| <= amax."""
    out = np.zeros(3, dtype=np.int64)
    rc = _load().oracle_quant_division_sweep(_ptr(out), int(amax_step))
    assert rc == 0
    return int(out[0]), int(out[1]), int(out[2])


def dequant_np(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """k^ = code * scale, exact in float64."""
    return codes.astype(np.float64) * scales.astype(np.float64)[..., None]


# ------------------------------------------------------------------ attention

def _kv_args(k, v, k_scale, v_scale):
    is_int8 = k.dtype == np.int8
    if is_int8:
        assert v.dtype == np.int8 and k_scale is not None and v_scale is not None
        k_scale = np.ascontiguousarray(k_scale, dtype=np.float32)
        v_scale = np.ascontiguousarray(v_scale, dtype=np.float32)
        assert k_scale.shape == k.shape[:-1] and v_scale.shape == v.shape[:-1]
    else:
        assert k.dtype == np.uint16 and v.dtype == np.uint16
        k_scale = v_scale = None
    return np.ascontiguousarray(k), np.ascontiguousarray(v), k_scale, v_scale, int(is_int8)


def attn(q_bits, k, v, softmax_scale, causal, k_scale=None, v_scale=None, rows=None):
    """C oracle attention (section 2.1).  q_bits [B,Hq,Sq,D] uint16; k, v [B,Hkv,Skv,D]
    uint16 (bf16) or int8 with k_scale/v_scale [B,Hkv,Skv] float32.  Returns float64
    [B,Hq,Sq,D], or [B,Hq,len(rows),D] when a list of query rows is given."""
    q_bits = np.ascontiguousarray(q_bits, dtype=np.uint16)
    k, v, k_scale, v_scale, is_int8 = _kv_args(k, v, k_scale, v_scale)
    B, Hq, Sq, D = q_bits.shape
    Bk, Hkv, Skv, Dk = k.shape
    assert (B, D) == (Bk, Dk) and v.shape == k.shape
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        assert rows.ndim == 1 and rows.size > 0 and rows.min() >= 0 and rows.max() < Sq
        R = rows.size
    else:
        R = Sq
    out = np.empty((B, Hq, R, D), dtype=np.float64)
    rc = _load().oracle_attn(_ptr(q_bits), _ptr(k), _ptr(v), _ptr(k_scale), _ptr(v_scale), _ptr(out),
                             B, Hq, Hkv, Sq, Skv, D, int(bool(causal)), float(softmax_scale), is_int8,
                             _ptr(rows), 0 if rows is None else int(rows.size))
    if rc != 0:
        raise RuntimeError("oracle_attn failed with status %d" % rc)
    return out


def attn_row_probs(q_bits, k, v, softmax_scale, causal, b, h, i, k_scale=None, v_scale=None):
    """Probabilities p_j / l (Skv values, 0 where masked) and output of one query row."""
    q_bits = np.ascontiguousarray(q_bits, dtype=np.uint16)
    k, v, k_scale, v_scale, is_int8 = _kv_args(k, v, k_scale, v_scale)
    B, Hq, Sq, D = q_bits.shape
    _, Hkv, Skv, _ = k.shape
    probs = np.empty(Skv, dtype=np.float64)
    o = np.empty(D, dtype=np.float64)
    rc = _load().oracle_attn_row_probs(_ptr(q_bits), _ptr(k), _ptr(v), _ptr(k_scale), _ptr(v_scale),
                                       _ptr(probs), _ptr(o), B, Hq, Hkv, Sq, Skv, D, int(bool(causal)),
                                       float(softmax_scale), is_int8, int(b), int(h), int(i))
    if rc != 0:
        raise RuntimeError("oracle_attn_row_probs failed with status %d" % rc)
    return probs, o


def _visible(Sq, Skv, causal):
    i = np.arange(Sq)[:, None] + (Skv - Sq)
    j = np.arange(Skv)[None, :]
    return (j <= i) if causal else np.ones((Sq, Skv), dtype=bool)


def attn_full_matrix_np(q, k, v, softmax_scale, causal):
    """softmax(Q K^T * scale + mask) V with the whole score matrix, numpy float64.
    q [B,Hq,Sq,D], k/v [B,Hkv,Skv,D] float64 (already widened / dequantised)."""
    B, Hq, Sq, D = q.shape
    Hkv, Skv = k.shape[1], k.shape[2]
    G = Hq // Hkv
    vis = _visible(Sq, Skv, causal)
    out = np.empty((B, Hq, Sq, D), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            s = softmax_scale * (q[b, h] @ k[b, g].T)
            s = np.where(vis, s, -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            out[b, h] = (p @ v[b, g]) / p.sum(axis=1, keepdims=True)
    return out


def slim_attn_rowblocks_np(q, k, v, softmax_scale, causal, block_rows):
    """The computation sequence of section 2.1: per block of query rows one horizontal
    score buffer over all keys, softmax over it, times V -> that block's slice of the
    output; the next block reuses the buffer."""
    B, Hq, Sq, D = q.shape
    Hkv, Skv = k.shape[1], k.shape[2]
    G = Hq // Hkv
    vis = _visible(Sq, Skv, causal)
    out = np.empty((B, Hq, Sq, D), dtype=np.float64)
    score = np.empty((block_rows, Skv), dtype=np.float64)  # the one buffer
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for i0 in range(0, Sq, block_rows):
                n = min(block_rows, Sq - i0)
                buf = score[:n]
                np.matmul(q[b, h, i0:i0 + n], k[b, g].T, out=buf)
                buf *= softmax_scale
                buf[~vis[i0:i0 + n]] = -np.inf
                buf -= buf.max(axis=1, keepdims=True)
                np.exp(buf, out=buf)
                buf /= buf.sum(axis=1, keepdims=True)
                out[b, h, i0:i0 + n] = buf @ v[b, g]
    return out

"""ctypes binding of the C-ABI library (``include/slimattn.h``): argument marshalling only.

Tensors are torch tensors on the GPU (PyTorch supplies device memory and the HIP stream);
every step of the path runs in the library's kernels.  There is no CPU fallback: if the
built library is missing, the first call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslimattn.so")

SLIM_OK = 0
SLIM_BF16, SLIM_F32, SLIM_I8 = 0, 1, 2

_lib = None


class SlimError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("slimattn status %d: %s" % (status, text))
        self.status = status


def load():
    """Loads ``libslimattn.so``; raises if it has not been built (``build.build()``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -m paper_2407_07304_amd.build` (hipcc, gfx950) first; "
                              "there is no fallback path" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        p, i, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        lib.kv_quant_int8.argtypes = [p, p, p, i, i, i, i, i, i, f, p]
        lib.kv_quant_int8.restype = i
        lib.kv_quant_int8_pair.argtypes = [p, p, p, p, p, p, i, i, i, i, i, i, f, p]
        lib.kv_quant_int8_pair.restype = i
        lib.kv_quant_int8_append.argtypes = [p, p, p, p, i, i, i, i, i, i, f, p]
        lib.kv_quant_int8_append.restype = i
        lib.slim_attn_prefill.argtypes = [p, p, p, p, p, p, i, i, i, i, i, i, f, i, i, p]
        lib.slim_attn_prefill.restype = i
        lib.slim_attn_prefill_emit_int8.argtypes = [p, p, p, p, p, p, p, p, i, i, i, i, i, i, f, i, p]
        lib.slim_attn_prefill_emit_int8.restype = i
        lib.slim_attn_prefill_two_sweep_workspace_bytes.argtypes = [i, i, i, i, i]
        lib.slim_attn_prefill_two_sweep_workspace_bytes.restype = ctypes.c_size_t
        lib.slim_attn_prefill_two_sweep.argtypes = [p, p, p, p, p, ctypes.c_size_t, i, i, i, i, i, i, f, i, p]
        lib.slim_attn_prefill_two_sweep.restype = i
        lib.slim_attn_prefill_strip_max_seq_len.argtypes = []
        lib.slim_attn_prefill_strip_max_seq_len.restype = i
        lib.slim_attn_prefill_strip.argtypes = [p, p, p, p, i, i, i, i, i, i, f, i, p]
        lib.slim_attn_prefill_strip.restype = i
        lib.slim_attn_decode_int8_workspace_bytes.argtypes = [i, i, i, i, i]
        lib.slim_attn_decode_int8_workspace_bytes.restype = ctypes.c_size_t
        lib.slim_attn_decode_int8.argtypes = [p, p, p, p, p, p, p, ctypes.c_size_t, i, i, i, i, i, i, f, p]
        lib.slim_attn_decode_int8.restype = i
        lib.slim_attn_decode_int8_static_max_bytes.argtypes = []
        lib.slim_attn_decode_int8_static_max_bytes.restype = ctypes.c_size_t
        lib.slim_attn_decode_int8_static.argtypes = [p, p, p, p, p, p, i, i, i, i, i, i, f, p]
        lib.slim_attn_decode_int8_static.restype = i
        lib.slim_attn_decode_int8_varlen.argtypes = [p, p, p, p, p, p, p, p, ctypes.c_size_t, i, i, i, i, i, i, f, p]
        lib.slim_attn_decode_int8_varlen.restype = i
        lib.slim_status_string.argtypes = [i]
        lib.slim_status_string.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().slim_status_string(int(status)).decode()


def _check(status):
    if status != SLIM_OK:
        raise SlimError(status, status_string(status))


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors, densely packed"
    if dtype is not None:
        assert t.dtype == dtype, "expected %s, got %s" % (dtype, t.dtype)
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def kv_quant_int8(x, codes=None, scales=None):
    """x [B,Hkv,S,D] bf16 -> (codes int8 [B,Hkv,S,D], scales fp32 [B,Hkv,S])."""
    B, Hkv, S, D = x.shape
    if codes is None:
        codes = torch.empty((B, Hkv, S, D), dtype=torch.int8, device=x.device)
    if scales is None:
        scales = torch.empty((B, Hkv, S), dtype=torch.float32, device=x.device)
    _check(load().kv_quant_int8(_ptr(x, torch.bfloat16), _ptr(codes, torch.int8), _ptr(scales, torch.float32),
                                B, Hkv, Hkv, S, D, 0, 1.0, _stream()))
    return codes, scales


def kv_quant_int8_pair(k, v, k_codes=None, k_scale=None, v_codes=None, v_scale=None):
    """kv_quant_int8 on k and v [B,Hkv,S,D] bf16 in one launch -> (k_codes, k_scale, v_codes, v_scale)."""
    B, Hkv, S, D = k.shape
    assert v.shape == k.shape
    outs = []
    for codes, scales in ((k_codes, k_scale), (v_codes, v_scale)):
        if codes is None:
            codes = torch.empty((B, Hkv, S, D), dtype=torch.int8, device=k.device)
        if scales is None:
            scales = torch.empty((B, Hkv, S), dtype=torch.float32, device=k.device)
        assert codes.shape == (B, Hkv, S, D) and scales.shape == (B, Hkv, S)
        outs += [codes, scales]
    _check(load().kv_quant_int8_pair(_ptr(k, torch.bfloat16), _ptr(v, torch.bfloat16), _ptr(outs[0], torch.int8),
                                     _ptr(outs[1], torch.float32), _ptr(outs[2], torch.int8), _ptr(outs[3], torch.float32),
                                     B, Hkv, Hkv, S, D, 0, 1.0, _stream()))
    return tuple(outs)


def slim_attn_prefill(q, k, v, softmax_scale, causal=True, k_scale=None, v_scale=None, out=None,
                      out_dtype=torch.bfloat16):
    """q [B,Hq,S,D] bf16; k, v [B,Hkv,S,D] bf16, or int8 with k_scale/v_scale [B,Hkv,S] fp32."""
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, S, D) and v.shape == k.shape
    kv_dtype = SLIM_I8 if k.dtype == torch.int8 else SLIM_BF16
    assert v.dtype == k.dtype and k.dtype in (torch.int8, torch.bfloat16)
    if kv_dtype == SLIM_I8:
        assert k_scale.shape == (B, Hkv, S) and v_scale.shape == (B, Hkv, S)
    if out is None:
        out = torch.empty((B, Hq, S, D), dtype=out_dtype, device=q.device)
    assert out.shape == (B, Hq, S, D) and out.dtype in (torch.bfloat16, torch.float32)
    od = SLIM_F32 if out.dtype == torch.float32 else SLIM_BF16
    _check(load().slim_attn_prefill(_ptr(q, torch.bfloat16), _ptr(k), _ptr(v), _ptr(k_scale, torch.float32),
                                    _ptr(v_scale, torch.float32), _ptr(out), B, Hq, Hkv, S, D, int(bool(causal)),
                                    float(softmax_scale), kv_dtype, od, _stream()))
    return out


def slim_attn_decode_int8_workspace_bytes(batch, q_heads, kv_heads, kv_len, head_dim) -> int:
    return int(load().slim_attn_decode_int8_workspace_bytes(batch, q_heads, kv_heads, kv_len, head_dim))


def slim_attn_decode_int8(q, k_codes, k_scale, v_codes, v_scale, softmax_scale, causal=False, out=None,
                          workspace=None):
    """q [B,Hq,1,D] bf16; codes [B,Hkv,T,D] int8; scales [B,Hkv,T] fp32 -> out [B,Hq,1,D] bf16."""
    B, Hq, one, D = q.shape
    assert one == 1
    Hkv, T = k_codes.shape[1], k_codes.shape[2]
    assert k_codes.shape == (B, Hkv, T, D) and v_codes.shape == k_codes.shape
    assert k_scale.shape == (B, Hkv, T) and v_scale.shape == (B, Hkv, T)
    if out is None:
        out = torch.empty((B, Hq, 1, D), dtype=torch.bfloat16, device=q.device)
    need = slim_attn_decode_int8_workspace_bytes(B, Hq, Hkv, T, D)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=q.device)
    _check(load().slim_attn_decode_int8(_ptr(q, torch.bfloat16), _ptr(k_codes, torch.int8), _ptr(k_scale, torch.float32),
                                        _ptr(v_codes, torch.int8), _ptr(v_scale, torch.float32),
                                        _ptr(out, torch.bfloat16), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                        B, Hq, Hkv, T, D, int(bool(causal)), float(softmax_scale), _stream()))
    return out


def slim_attn_decode_int8_static_max_bytes() -> int:
    return int(load().slim_attn_decode_int8_static_max_bytes())


def slim_attn_decode_int8_static(q, k_codes, k_scale, v_codes, v_scale, softmax_scale, out, causal=False):
    """slim_attn_decode_int8 with the library's own static scratch array: no workspace argument, and nothing is
    allocated here either, so the caller passes ``out`` [B,Hq,1,D] bf16."""
    B, Hq, one, D = q.shape
    assert one == 1
    Hkv, T = k_codes.shape[1], k_codes.shape[2]
    assert k_codes.shape == (B, Hkv, T, D) and v_codes.shape == k_codes.shape
    assert k_scale.shape == (B, Hkv, T) and v_scale.shape == (B, Hkv, T) and out.shape == (B, Hq, 1, D)
    _check(load().slim_attn_decode_int8_static(_ptr(q, torch.bfloat16), _ptr(k_codes, torch.int8),
                                               _ptr(k_scale, torch.float32), _ptr(v_codes, torch.int8),
                                               _ptr(v_scale, torch.float32), _ptr(out, torch.bfloat16), B, Hq, Hkv, T, D,
                                               int(bool(causal)), float(softmax_scale), _stream()))
    return out


def slim_attn_decode_int8_varlen(q, k_codes, k_scale, v_codes, v_scale, kv_lens, softmax_scale, causal=False, out=None,
                                 workspace=None):
    """As slim_attn_decode_int8, sequence b attending to its first kv_lens[b] cached tokens (kv_lens [B] int32,
    on the device)."""
    B, Hq, one, D = q.shape
    assert one == 1
    Hkv, T = k_codes.shape[1], k_codes.shape[2]
    assert k_codes.shape == (B, Hkv, T, D) and v_codes.shape == k_codes.shape
    assert k_scale.shape == (B, Hkv, T) and v_scale.shape == (B, Hkv, T)
    assert kv_lens.shape == (B,)
    if out is None:
        out = torch.empty((B, Hq, 1, D), dtype=torch.bfloat16, device=q.device)
    need = slim_attn_decode_int8_workspace_bytes(B, Hq, Hkv, T, D)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=q.device)
    _check(load().slim_attn_decode_int8_varlen(_ptr(q, torch.bfloat16), _ptr(k_codes, torch.int8),
                                               _ptr(k_scale, torch.float32), _ptr(v_codes, torch.int8),
                                               _ptr(v_scale, torch.float32), _ptr(kv_lens, torch.int32),
                                               _ptr(out, torch.bfloat16), _ptr(workspace),
                                               workspace.numel() * workspace.element_size(), B, Hq, Hkv, T, D,
                                               int(bool(causal)), float(softmax_scale), _stream()))
    return out


def kv_quant_int8_append(x_new, codes, scales, positions):
    """Quantises x_new [B,Hkv,1,D] bf16 into token positions[b] of the cache (codes [B,Hkv,T,D] int8, scales
    [B,Hkv,T] fp32, both updated in place); positions [B] int32 on the device."""
    B, Hkv, one, D = x_new.shape
    assert one == 1
    T = codes.shape[2]
    assert codes.shape == (B, Hkv, T, D) and scales.shape == (B, Hkv, T) and positions.shape == (B,)
    _check(load().kv_quant_int8_append(_ptr(x_new, torch.bfloat16), _ptr(codes, torch.int8), _ptr(scales, torch.float32),
                                       _ptr(positions, torch.int32), B, Hkv, Hkv, T, D, 0, 1.0, _stream()))


def slim_attn_prefill_emit_int8(q, k, v, softmax_scale, causal=True, out=None, out_dtype=torch.bfloat16):
    """Prefill on bf16 K/V that also writes their INT8 cache: returns (out, k_codes, k_scale, v_codes, v_scale)."""
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, S, D) and v.shape == k.shape and k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16
    if out is None:
        out = torch.empty((B, Hq, S, D), dtype=out_dtype, device=q.device)
    kc = torch.empty((B, Hkv, S, D), dtype=torch.int8, device=q.device)
    vc = torch.empty_like(kc)
    ks = torch.empty((B, Hkv, S), dtype=torch.float32, device=q.device)
    vs = torch.empty_like(ks)
    _check(load().slim_attn_prefill_emit_int8(_ptr(q, torch.bfloat16), _ptr(k, torch.bfloat16), _ptr(v, torch.bfloat16),
                                              _ptr(out), _ptr(kc, torch.int8), _ptr(ks, torch.float32),
                                              _ptr(vc, torch.int8), _ptr(vs, torch.float32), B, Hq, Hkv, S, D,
                                              int(bool(causal)), float(softmax_scale),
                                              SLIM_F32 if out.dtype == torch.float32 else SLIM_BF16, _stream()))
    return out, kc, ks, vc, vs


def slim_attn_prefill_two_sweep(q, k, v, softmax_scale, causal=True, out=None, out_dtype=torch.bfloat16, workspace=None):
    """The two-sweep comparison variant of the bf16 prefill (row maxima first, then everything else)."""
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, S, D) and v.shape == k.shape and k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16
    if out is None:
        out = torch.empty((B, Hq, S, D), dtype=out_dtype, device=q.device)
    need = int(load().slim_attn_prefill_two_sweep_workspace_bytes(B, Hq, Hkv, S, D))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(load().slim_attn_prefill_two_sweep(_ptr(q, torch.bfloat16), _ptr(k, torch.bfloat16), _ptr(v, torch.bfloat16),
                                              _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                              B, Hq, Hkv, S, D, int(bool(causal)), float(softmax_scale),
                                              SLIM_F32 if out.dtype == torch.float32 else SLIM_BF16, _stream()))
    return out


def slim_attn_prefill_strip_max_seq_len() -> int:
    return int(load().slim_attn_prefill_strip_max_seq_len())


def slim_attn_prefill_strip(q, k, v, softmax_scale, causal=True, out=None, out_dtype=torch.bfloat16):
    """The comparison variant of the bf16 prefill that keeps a row block's whole score strip on chip."""
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, S, D) and v.shape == k.shape and k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16
    if out is None:
        out = torch.empty((B, Hq, S, D), dtype=out_dtype, device=q.device)
    _check(load().slim_attn_prefill_strip(_ptr(q, torch.bfloat16), _ptr(k, torch.bfloat16), _ptr(v, torch.bfloat16), _ptr(out),
                                          B, Hq, Hkv, S, D, int(bool(causal)), float(softmax_scale),
                                          SLIM_F32 if out.dtype == torch.float32 else SLIM_BF16, _stream()))
    return out

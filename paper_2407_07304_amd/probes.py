"""ctypes binding of the measurement kernels (``include/slimprobe.h``): argument marshalling only."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslimprobe.so")
_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -m paper_2407_07304_amd.build` (hipcc, gfx950) first" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        p, i = ctypes.c_void_p, ctypes.c_int
        lib.slim_probe_stream_read.argtypes = [p, ctypes.c_size_t, p, p]
        lib.slim_probe_stream_read.restype = i
        lib.slim_probe_quant_traffic.argtypes = [p, p, p, ctypes.c_long, i, p]
        lib.slim_probe_quant_traffic.restype = i
        lib.slim_probe_mfma_bf16.argtypes = [p, p, i, p, i, i, p]
        lib.slim_probe_mfma_bf16.restype = i
        lib.slim_probe_gqa_decode_traffic.argtypes = [p, p, p, p, p, p, ctypes.c_size_t, i, i, i, i, i, p]
        lib.slim_probe_gqa_decode_traffic.restype = i
        _lib = lib
    return _lib


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError("%s failed with status %d" % (what, rc))


def slim_probe_stream_read(src, sink):
    """src: any contiguous device tensor whose size in bytes is a multiple of 16; sink: >= 16 bytes."""
    nbytes = src.numel() * src.element_size()
    _check(load().slim_probe_stream_read(ctypes.c_void_p(src.data_ptr()), nbytes, ctypes.c_void_p(sink.data_ptr()), _stream()),
           "slim_probe_stream_read")


def slim_probe_quant_traffic(x, codes, scales):
    """x [..., D] bf16, codes [..., D] int8, scales [...] fp32."""
    D = x.shape[-1]
    _check(load().slim_probe_quant_traffic(ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(codes.data_ptr()),
                                           ctypes.c_void_p(scales.data_ptr()), x.numel() // D, D, _stream()),
           "slim_probe_quant_traffic")


def slim_probe_mfma_bf16(a, b, out, workgroups, iters):
    """a, b: bf16 device tensors of slices * 512 values each; out: fp32, workgroups * 8 values."""
    slices = a.numel() // 512
    assert a.numel() == slices * 512 and b.numel() == a.numel() and out.numel() >= workgroups * 8
    _check(load().slim_probe_mfma_bf16(ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(b.data_ptr()), slices,
                                       ctypes.c_void_p(out.data_ptr()), workgroups, iters, _stream()),
           "slim_probe_mfma_bf16")


def slim_probe_gqa_decode_traffic(q, k_codes, k_scale, v_codes, v_scale, workspace):
    """Shapes as for slim_attn_decode_int8; workspace: a uint8 tensor of at least the decode's workspace size."""
    B, Hq, _, D = q.shape
    Hkv, T = k_codes.shape[1], k_codes.shape[2]
    _check(load().slim_probe_gqa_decode_traffic(ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(k_codes.data_ptr()),
                                                ctypes.c_void_p(k_scale.data_ptr()), ctypes.c_void_p(v_codes.data_ptr()),
                                                ctypes.c_void_p(v_scale.data_ptr()), ctypes.c_void_p(workspace.data_ptr()),
                                                workspace.numel() * workspace.element_size(), B, Hq, Hkv, T, D, _stream()),
           "slim_probe_gqa_decode_traffic")

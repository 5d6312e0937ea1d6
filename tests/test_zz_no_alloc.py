"""The decode entry point that allocates nothing (static device scratch) against the one that takes a workspace.

Same kernels, so the outputs must agree bit for bit; both are also held to the oracle's tolerance.  Two calls in a
row share the static array, the second with a smaller input, so stale partial results of the first call lie behind
the second call's.
"""
import ctypes
import math

import numpy as np
import pytest
import torch

from paper_2407_07304_amd.inputs import normal_bf16

from _gpu_util import dev, dev_bf16, host_f64, check_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sa():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2407_07304_amd import slimattn
    slimattn.load()
    return slimattn


def _case(sa, oracle, B, Hq, Hkv, T, D, seed):
    rng = np.random.default_rng(seed)
    q = normal_bf16(rng, (B, Hq, 1, D))
    kc, ks = oracle.kv_quant_int8(normal_bf16(rng, (B, Hkv, T, D)))
    vc, vs = oracle.kv_quant_int8(normal_bf16(rng, (B, Hkv, T, D)))
    scale = 1.0 / math.sqrt(D)
    dq, dkc, dks, dvc, dvs = dev_bf16(q), dev(kc), dev(ks), dev(vc), dev(vs)
    want = oracle.attn(q, kc, vc, scale, False, k_scale=ks, v_scale=vs)
    ref = sa.slim_attn_decode_int8(dq, dkc, dks, dvc, dvs, scale)
    out = torch.full((B, Hq, 1, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    return (dq, dkc, dks, dvc, dvs, scale, out), ref, want


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 8, 128), (16, 2, 128), (6, 3, 64)])
def test_static_scratch_decode_matches_the_workspace_decode(sa, oracle, Hq, Hkv, D):
    # first a cache with many key-axis splits, then a smaller one: the second call's records overwrite a part of the
    # first call's, and what lies behind them must not reach its result
    print("static-scratch decode", Hq, Hkv, D, flush=True)
    assert sa.slim_attn_decode_int8_static_max_bytes() == 16 << 20
    for B, T, seed in ((3, 5000, 11), (2, 700, 12), (1, 1, 13)):
        assert 0 < sa.slim_attn_decode_int8_workspace_bytes(B, Hq, Hkv, T, D) <= sa.slim_attn_decode_int8_static_max_bytes()
        args, ref, want = _case(sa, oracle, B, Hq, Hkv, T, D, seed + Hq)
        n_allocs = torch.cuda.memory_stats()["allocation.all.allocated"]
        got = sa.slim_attn_decode_int8_static(*args)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == n_allocs   # (torch's allocator saw no request)
        torch.cuda.synchronize()
        assert torch.equal(got, ref), "static-scratch decode differs from the workspace decode (B=%d T=%d)" % (B, T)
        check_close(host_f64(got), want, "static-scratch decode B%d Hq%d Hkv%d T%d D%d" % (B, Hq, Hkv, T, D))


def test_static_scratch_decode_rejects_what_does_not_fit(sa):
    # a shape whose partial results exceed the static array is refused before anything is enqueued
    B, Hq, Hkv, T, D = 256, 64, 8, 8192, 128
    assert sa.slim_attn_decode_int8_workspace_bytes(B, Hq, Hkv, T, D) > sa.slim_attn_decode_int8_static_max_bytes()
    lib = sa.load()
    A = ctypes.c_void_p(0x1000)   # never dereferenced: the size check comes first
    st = lib.slim_attn_decode_int8_static(A, A, A, A, A, A, B, Hq, Hkv, T, D, 0, 0.1, None)
    assert st == 5 and "workspace" in sa.status_string(st).lower()
    assert lib.slim_attn_decode_int8_static(None, A, A, A, A, A, 1, 2, 2, 10, D, 0, 0.1, None) == 1
    assert lib.slim_attn_decode_int8_static(A, A, A, A, A, A, 1, 2, 2, 10, 96, 0, 0.1, None) == 3


def test_static_scratch_decode_under_graph_capture(sa, oracle):
    # what the entry point is for: a decode step recorded into a HIP graph (nothing may allocate while a stream is
    # being captured) and replayed; every replay, with eager work and synchronisations in between, must give the
    # eager call's bits.  The first call on the device (which looks the scratch array's address up) comes before.
    B, Hq, Hkv, T, D = 2, 16, 4, 3000, 128
    args, ref, want = _case(sa, oracle, B, Hq, Hkv, T, D, 21)
    eager = sa.slim_attn_decode_int8_static(*args).clone()
    torch.cuda.synchronize()
    assert torch.equal(eager, ref)
    args[-1].zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sa.slim_attn_decode_int8_static(*args)
    for rep in range(4):
        args[-1].fill_(float(rep))                       # eager work between the replays
        other = sa.slim_attn_decode_int8(*args[:6])      # ... including the decode that takes a workspace
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(args[-1], ref), "replay %d differs from the eager result" % rep
        assert torch.equal(other, ref)
    check_close(host_f64(args[-1]), want, "static-scratch decode replayed from a graph")

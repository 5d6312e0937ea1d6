"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and
rejects bad arguments before anything is launched (no GPU is touched)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "slimattn.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2407_07304_amd import slimattn, build
    if not os.path.exists(slimattn.LIB_PATH):
        build.build()
    return slimattn.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"})


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"kv_quant_int8", "slim_attn_prefill", "slim_attn_decode_int8", "slim_attn_decode_int8_varlen",
            "kv_quant_int8_append", "kv_quant_int8_pair", "slim_attn_prefill_emit_int8", "slim_attn_decode_int8_workspace_bytes", "slim_status_string",
            "slim_attn_prefill_two_sweep", "slim_attn_prefill_two_sweep_workspace_bytes", "slim_attn_prefill_strip",
            "slim_attn_prefill_strip_max_seq_len", "slim_attn_decode_int8_static", "slim_attn_decode_int8_static_max_bytes"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    seen = set()
    for code in range(7):
        s = lib.slim_status_string(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert lib.slim_status_string(99).decode() == "unknown status"


P = ctypes.c_void_p
A = 0x1000   # a fake, aligned, never dereferenced address: every case below fails validation first


def prefill(lib, q=A, k=A, v=A, ks=None, vs=None, out=A, B=1, Hq=2, Hkv=2, S=16, D=128, causal=1, scale=0.1,
            kvd=0, od=0):
    return lib.slim_attn_prefill(P(q), P(k), P(v), P(ks), P(vs), P(out), B, Hq, Hkv, S, D, causal, scale, kvd, od, None)


def test_prefill_rejects_bad_arguments(lib):
    NULL, SHAPE, UNSUP, ALIGN = 1, 2, 3, 4
    assert prefill(lib, q=None) == NULL
    assert prefill(lib, out=None) == NULL
    assert prefill(lib, kvd=2) == NULL                 # INT8 without scales
    assert prefill(lib, ks=A, vs=A) == NULL            # bf16 with scales
    assert prefill(lib, kvd=1) == UNSUP and prefill(lib, od=2) == UNSUP
    assert prefill(lib, D=96) == UNSUP
    assert prefill(lib, S=0) == SHAPE and prefill(lib, B=-1) == SHAPE
    assert prefill(lib, Hq=3, Hkv=2) == SHAPE
    assert prefill(lib, causal=2) == SHAPE
    assert prefill(lib, scale=0.0) == SHAPE and prefill(lib, scale=float("nan")) == SHAPE
    assert prefill(lib, scale=float("inf")) == SHAPE
    assert prefill(lib, k=A + 8) == ALIGN
    assert prefill(lib, kvd=2, ks=A + 4, vs=A) == ALIGN
    assert prefill(lib, B=65536, Hq=65536, Hkv=65536, S=4096) == SHAPE   # not indexable


def test_quant_rejects_bad_arguments(lib):
    f = lib.kv_quant_int8
    assert f(P(None), P(A), P(A), 1, 1, 1, 4, 128, 0, 1.0, None) == 1
    assert f(P(A), P(A), P(A), 1, 1, 1, 0, 128, 0, 1.0, None) == 2
    assert f(P(A), P(A), P(A), 1, 1, 1, 4, 100, 0, 1.0, None) == 3
    assert f(P(A), P(A + 1), P(A), 1, 1, 1, 4, 128, 0, 1.0, None) == 4
    # the scalars of the common tail that the quantiser does not use are still checked for range
    assert f(P(A), P(A), P(A), 1, 0, 1, 4, 128, 0, 1.0, None) == 2
    assert f(P(A), P(A), P(A), 1, 3, 2, 4, 128, 0, 1.0, None) == 2
    assert f(P(A), P(A), P(A), 1, 1, 1, 4, 128, 2, 1.0, None) == 2
    assert f(P(A), P(A), P(A), 1, 1, 1, 4, 128, 0, 0.0, None) == 2
    assert f(P(A), P(A), P(A), 1, 1, 1, 4, 128, 0, float("nan"), None) == 2


def test_decode_rejects_bad_arguments_and_reports_workspace(lib):
    ws = lib.slim_attn_decode_int8_workspace_bytes
    per_row = lambda D: (D + 2) * 4   # one (max, sum, accumulator[D]) record per split
    assert ws(16, 32, 32, 8192, 128) % (16 * 32 * per_row(128)) == 0 and ws(16, 32, 32, 8192, 128) > 0
    assert ws(1, 1, 1, 1, 64) == per_row(64)
    assert ws(2, 4, 4, 100000, 64) >= ws(2, 4, 4, 1000, 64) > 0
    assert ws(1, 3, 2, 10, 128) == 0 and ws(1, 1, 1, 10, 96) == 0
    f = lib.slim_attn_decode_int8

    def call(q=A, kc=A, ks=A, vc=A, vs=A, out=A, wsp=A, wsb=1 << 30, B=1, Hq=2, Hkv=2, T=100, D=128, causal=0, scale=0.1):
        return f(P(q), P(kc), P(ks), P(vc), P(vs), P(out), P(wsp), wsb, B, Hq, Hkv, T, D, causal, scale, None)

    assert call(vs=None) == 1 and call(wsp=None) == 1
    assert call(T=0) == 2 and call(Hq=4, Hkv=3) == 2 and call(scale=-1.0) == 2
    assert call(D=32) == 3
    assert call(out=A + 2) == 4
    assert call(wsb=ws(1, 2, 2, 100, 128) - 1) == 5


def test_decode_workspace_is_a_whole_number_of_split_records_for_every_geometry(lib):
    """Host logic only: whatever split geometry the library picks (per-head or grouped-query kernel), the workspace
    is n_split records of (max, sum, accumulator[D]) per (batch, query head), with at least one split and never
    more splits than the cache has 32-token tiles (plus the one a two-wave workgroup may leave empty)."""
    ws = lib.slim_attn_decode_int8_workspace_bytes
    for D in (64, 128):
        for (B, Hq, Hkv) in ((1, 1, 1), (1, 32, 32), (16, 32, 32), (16, 64, 8), (3, 40, 1), (64, 8, 8), (2, 64, 2), (1, 8, 4)):
            for T in (1, 31, 32, 33, 100, 2048, 8191, 8192, 32768, 100000):
                n, rec = ws(B, Hq, Hkv, T, D), B * Hq * (D + 2) * 4
                assert n > 0 and n % rec == 0, (B, Hq, Hkv, T, D, n)
                splits = n // rec
                assert 1 <= splits <= (T + 31) // 32 + 1, (B, Hq, Hkv, T, D, splits)


def test_varlen_decode_rejects_bad_arguments(lib):
    f = lib.slim_attn_decode_int8_varlen

    def call(lens=A, q=A, wsp=A, wsb=1 << 30, T=100, D=128):
        return f(P(q), P(A), P(A), P(A), P(A), P(lens), P(A), P(wsp), wsb, 1, 2, 2, T, D, 0, 0.1, None)

    assert call(lens=None) == 1 and call(q=None) == 1
    assert call(lens=A + 2) == 4 and call(q=A + 4) == 4
    assert call(T=0) == 2 and call(D=96) == 3
    assert call(wsb=8) == 5


def test_quant_pair_rejects_bad_arguments(lib):
    f = lib.kv_quant_int8_pair

    def call(k=A, v=A, kc=A, ks=A, vc=A, vs=A, B=2, Hq=2, Hkv=2, S=100, D=128, causal=0, scale=1.0):
        return f(P(k), P(v), P(kc), P(ks), P(vc), P(vs), B, Hq, Hkv, S, D, causal, scale, None)

    assert call(k=None) == 1 and call(v=None) == 1 and call(vs=None) == 1 and call(kc=None) == 1
    assert call(S=0) == 2 and call(B=-1) == 2
    assert call(D=96) == 3
    assert call(v=A + 8) == 4 and call(vc=A + 4) == 4
    assert call(Hq=3) == 2 and call(causal=2) == 2 and call(scale=0.0) == 2


def test_append_rejects_bad_arguments(lib):
    f = lib.kv_quant_int8_append

    def call(x=A, codes=A, scales=A, pos=A, B=2, Hq=2, Hkv=2, T=100, D=128, causal=0, scale=1.0):
        return f(P(x), P(codes), P(scales), P(pos), B, Hq, Hkv, T, D, causal, scale, None)

    assert call(x=None) == 1 and call(pos=None) == 1 and call(scales=None) == 1
    assert call(T=0) == 2 and call(B=0) == 2
    assert call(D=100) == 3
    assert call(codes=A + 8) == 4 and call(pos=A + 1) == 4
    assert call(Hq=3) == 2 and call(causal=-1) == 2 and call(scale=float("inf")) == 2


def test_prefill_two_sweep_rejects_bad_arguments(lib):
    f = lib.slim_attn_prefill_two_sweep
    need = lib.slim_attn_prefill_two_sweep_workspace_bytes(1, 4, 2, 100, 128)
    assert need == 1 * 4 * 100 * 2 * 4
    assert lib.slim_attn_prefill_two_sweep_workspace_bytes(1, 4, 3, 100, 128) == 0

    def call(q=A, k=A, v=A, out=A, ws=A, wb=need, S=100, D=128, od=0):
        return f(P(q), P(k), P(v), P(out), P(ws), wb, 1, 4, 2, S, D, 1, 0.1, od, None)

    assert call(ws=None) == 1 and call(v=None) == 1
    assert call(S=0) == 2
    assert call(D=96) == 3 and call(od=7) == 3
    assert call(ws=A + 4) == 4
    assert call(wb=need - 1) == 5


def test_prefill_strip_rejects_bad_arguments(lib):
    f = lib.slim_attn_prefill_strip
    assert lib.slim_attn_prefill_strip_max_seq_len() == 2048

    def call(q=A, k=A, v=A, out=A, S=100, D=128, od=0, Hq=4, Hkv=2, causal=1, scale=0.1):
        return f(P(q), P(k), P(v), P(out), 1, Hq, Hkv, S, D, causal, scale, od, None)

    assert call(q=None) == 1 and call(out=None) == 1
    assert call(S=0) == 2 and call(Hq=3) == 2 and call(causal=3) == 2 and call(scale=-1.0) == 2
    assert call(D=96) == 3 and call(od=7) == 3
    assert call(v=A + 4) == 4


def test_probe_library_exports_what_its_header_declares():
    from paper_2407_07304_amd import probes
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "slimprobe.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(slim_probe_[a-z_0-9]+)\s*\(", text)))
    assert names == ["slim_probe_gqa_decode_traffic", "slim_probe_mfma_bf16", "slim_probe_quant_traffic", "slim_probe_stream_read"]
    lib = probes.load()
    for n in names:
        assert getattr(lib, n) is not None
    # bad arguments are refused before anything is enqueued (no GPU is touched)
    assert lib.slim_probe_stream_read(P(None), 1024, P(A), None) == 1
    assert lib.slim_probe_stream_read(P(A), 1000, P(A), None) == 1
    assert lib.slim_probe_quant_traffic(P(A), P(A), P(A), 10, 96, None) == 1
    assert lib.slim_probe_mfma_bf16(P(A), P(A), 0, P(A), 1, 1, None) == 1
    assert lib.slim_probe_gqa_decode_traffic(P(A), P(A), P(A), P(A), P(A), P(A), 16, 2, 64, 8, 8192, 128, None) == 1   # workspace too small
    assert lib.slim_probe_gqa_decode_traffic(P(A), P(A), P(A), P(A), P(A), P(A), 1 << 30, 1, 4, 4, 100, 128, None) == 1     # not a grouped shape


def test_prefill_emit_rejects_bad_arguments(lib):
    f = lib.slim_attn_prefill_emit_int8

    def call(q=A, k=A, v=A, out=A, kc=A, ks=A, vc=A, vs=A, S=100, D=128, od=0):
        return f(P(q), P(k), P(v), P(out), P(kc), P(ks), P(vc), P(vs), 1, 4, 2, S, D, 1, 0.1, od, None)

    assert call(kc=None) == 1 and call(vs=None) == 1 and call(q=None) == 1
    assert call(S=0) == 2
    assert call(D=96) == 3 and call(od=7) == 3
    assert call(vc=A + 4) == 4 and call(k=A + 2) == 4


def test_binding_fails_loudly_without_the_library(tmp_path, monkeypatch):
    # no CPU fallback: a missing library is an error, not a slower path
    from paper_2407_07304_amd import slimattn
    monkeypatch.setattr(slimattn, "LIB_PATH", str(tmp_path / "libslimattn.so"))
    monkeypatch.setattr(slimattn, "_lib", None, raising=False)
    with pytest.raises(ImportError, match="no fallback"):
        slimattn.load()


def test_product_code_does_not_touch_the_oracle():
    # the oracle is test infrastructure: nothing under the package imports or loads it
    pkg = os.path.join(os.path.dirname(HEADER), "..", "paper_2407_07304_amd")
    for root, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(root, f)).read()
                assert not re.search(r"import\s+oracle|from\s+oracle|oracle[/.]|libslim_oracle|slim_oracle\.", text), f

#!/usr/bin/env python3
"""Benchmark of the SlimAttention hot path on one MI355X.

One step = one pass of the whole path over seeded synthetic inputs already resident in HBM:
  1. slim_attn_prefill   causal prefill, Llama-2-7B shape (B=1, 32 heads, S=2048, D=128, bf16)
  2. kv_quant_int8       the prompt's K and V -> INT8 cache (+ one fp32 scale per token per head)
  3. slim_attn_decode_int8  one decode step, B=16, 32 heads, D=128, INT8 cache of 8192 tokens

`value` is the prefill throughput in TFLOP/s (causal flop count) and `decode.value` the
decode throughput in GB/s (algorithmic bytes), each from HIP-event timing of its own
kernel(s) inside the timed steps.  Prints ONE JSON line.

`--probe ceilings` runs the measurement kernels of include/slimprobe.h instead (streaming read, the quantiser's
traffic without arithmetic, back-to-back MFMAs and the prefill kernel on operands of different bit activity) and
prints their JSON line: the machine's practical ceilings, measured by the harness that measures the kernels.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
TRAFFIC_PROFILE = os.path.join("profiles", "traffic_fetch_write_c2_c4.txt")


def paper_table3_ms():
    """SlimAttention column of the paper's Table 3 (1 socket Xeon 8563C), from the golden fixture; context only."""
    out = {}
    try:
        for ln in open(os.path.join(ROOT, "tests", "golden", "table3_slimattention_ms.txt")):
            if ln.strip() and not ln.startswith("#"):
                s, _, slim = ln.split()
                out[int(s)] = float(slim)
    except OSError:
        pass
    return out


def kernel_sources_sha256():
    """Hash of the HIP sources the loaded library was built from (the tree's, built in place)."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2407_07304_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def profiled_traffic():
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary.  The counters are not
    read in this run: the figures are those of the profile, and they are only passed on while the profile names
    the kernel sources this tree holds."""
    out = {"bytes": {}, "sha": None}
    try:
        for ln in open(os.path.join(ROOT, TRAFFIC_PROFILE)):
            if ln.startswith("traffic_bytes "):
                _, key, val = ln.split()
                out["bytes"][key] = int(float(val))
            elif ln.startswith("sources_sha256 "):
                out["sha"] = ln.split()[1]
    except OSError:
        pass
    out["current"] = out["sha"] is not None and out["sha"] == kernel_sources_sha256()
    return out


def traffic_fields(prof, key):
    return {"traffic": prof["bytes"].get(key) if prof["current"] else None,
            "traffic_source": {"file": TRAFFIC_PROFILE, "measured_in_this_run": False,
                               "profile_matches_these_kernel_sources": prof["current"],
                               "profiled_bytes": prof["bytes"].get(key)}}


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.startswith("model name"):
                    return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _sample_rows(S, n, seed):
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 127, 128, S // 2, S - 129, S - 1]
    return np.array(sorted(set(fixed + rng.integers(0, S, n).tolist())), dtype=np.int32)


def median_ms(torch, fn, iters, warm=3, between=None):
    """Median and mean HIP-event time of fn() over iters launches on the current stream."""
    for _ in range(warm):
        fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in evs:
        if between is not None:
            between()
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    t = np.array([a.elapsed_time(b) for a, b in evs])
    return float(np.median(t)), float(t.mean()), float(t.min())


def probe_ceilings(args):
    import torch
    from paper_2407_07304_amd import probes, slimattn as sa
    from paper_2407_07304_amd import accounting as acct
    from paper_2407_07304_amd.inputs import normal_bf16
    sa.load()
    probes.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    rng = np.random.default_rng(7)
    out = {"probe": "ceilings", "device": torch.cuda.get_device_name(0),
           "peaks": {"bf16_mfma_TFLOPs": PEAK_BF16_TFLOPS, "hbm_GBps": PEAK_HBM_GBPS}}

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    # ---- 1. plain streaming read of 1 GiB (about the bytes of one C4 decode step)
    src = torch.randint(0, 255, (1 << 30,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    med, mean, mn = median_ms(torch, lambda: probes.slim_probe_stream_read(src, sink), 30)
    out["stream_read"] = {"bytes": 1 << 30, "ms_median": round(med, 4), "ms_min": round(mn, 4),
                          "GBps": round((1 << 30) / med / 1e6, 1), "frac_of_hbm_peak": round((1 << 30) / med / 1e6 / PEAK_HBM_GBPS, 4)}
    del src

    # ---- 2. the quantiser's stream (K of the C4 cache before quantisation: 1.07 GB in, 0.54 GB out) without and
    # with its arithmetic
    x = torch.randn((16, 32, 8192, 128), device="cuda", dtype=torch.float32).to(torch.bfloat16)
    codes = torch.empty(x.shape, dtype=torch.int8, device="cuda")
    scales = torch.empty(x.shape[:-1], dtype=torch.float32, device="cuda")
    qbytes = acct.kv_quant_bytes(x.numel() // 128, 128)
    med, _, mn = median_ms(torch, lambda: probes.slim_probe_quant_traffic(x, codes, scales), 30)
    out["quant_traffic_only"] = {"bytes": qbytes, "ms_median": round(med, 4), "ms_min": round(mn, 4), "GBps": round(qbytes / med / 1e6, 1)}
    med, _, mn = median_ms(torch, lambda: sa.kv_quant_int8(x, codes, scales), 30)
    out["kv_quant_int8_same_stream"] = {"bytes": qbytes, "ms_median": round(med, 4), "ms_min": round(mn, 4), "GBps": round(qbytes / med / 1e6, 1),
                                        "frac_of_hbm_peak": round(qbytes / med / 1e6 / PEAK_HBM_GBPS, 4)}
    del x, codes, scales

    # ---- 3. back-to-back bf16 MFMAs (one wave per SIMD, nothing else in the loop) on operands of different bit activity
    slices, iters, wgs = 1024, 4096, 256
    operands = {
        "zeros": (np.zeros((slices, 512), dtype=np.uint16), np.zeros((slices, 512), dtype=np.uint16)),
        "ones": (np.full((slices, 512), 0x3f80, dtype=np.uint16), np.full((slices, 512), 0x3f80, dtype=np.uint16)),
        "normal": (normal_bf16(rng, (slices, 512)), normal_bf16(rng, (slices, 512))),
    }
    res = torch.zeros(wgs * 8, dtype=torch.float32, device="cuda")
    flops = wgs * 4 * iters * 16 * 32768
    out["mfma_bf16_32x32x16"] = {}
    for name, (ah, bh) in operands.items():
        a, b = dev_bf16(ah), dev_bf16(bh)
        med, _, mn = median_ms(torch, lambda: probes.slim_probe_mfma_bf16(a, b, res, wgs, iters), 40, warm=20)
        cyc = float(res.view(-1, 2)[:, 1].mean())
        out["mfma_bf16_32x32x16"][name] = {
            "ms_median": round(med, 4), "TFLOPs": round(flops / med / 1e9, 1), "frac_of_bf16_mfma_peak": round(flops / med / 1e9 / PEAK_BF16_TFLOPS, 4),
            "cycles_per_wave_loop": round(cyc), "cycles_per_mfma": round(cyc / (iters * 16), 2),
            "effective_clock_GHz": round(cyc / (med * 1e6), 3)}

    # ---- 4. the prefill kernel itself on the same three kinds of operands
    out["prefill"] = {}
    for label, (B, H, S, causal) in (("C2 causal", (1, 32, 2048, True)), ("S=8192 non-causal", (1, 32, 8192, False))):
        fl = acct.prefill_flops(B, H, S, 128, causal)
        rec = {}
        for name in ("zeros", "ones", "normal"):
            shape = (B, H, S, 128)
            if name == "normal":
                q, k, v = (dev_bf16(normal_bf16(rng, shape)) for _ in range(3))
            else:
                fill = 0.0 if name == "zeros" else 1.0
                q, k, v = (torch.full(shape, fill, dtype=torch.bfloat16, device="cuda") for _ in range(3))
            o = torch.empty_like(q)
            scale = 1.0 / float(np.sqrt(128.0))
            med, _, mn = median_ms(torch, lambda: sa.slim_attn_prefill(q, k, v, scale, causal, out=o), 40 if S == 2048 else 15, warm=20)
            rec[name] = {"ms_median": round(med, 4), "ms_min": round(mn, 4), "TFLOPs": round(fl / med / 1e9, 1)}
            del q, k, v, o
        out["prefill"][label] = rec
    print(json.dumps(out))


def only_gqa_decode(args):
    """The grouped-query decode alone (for profiling): `steps` launches, each after a 1 GiB streaming read."""
    import torch
    from paper_2407_07304_amd import probes, slimattn as sa
    from paper_2407_07304_amd import accounting as acct
    from paper_2407_07304_amd.inputs import make_qkv, make_shape
    sa.load()
    probes.load()
    torch.cuda.set_device(0)

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    B, Hq, Hkv, T, D = 16, 64, 8, 8192, 128
    w = make_shape("decode", B, Hq, Hkv, T, D, False, True, False, 6, name="GQA decode")
    qh, kh, vh = make_qkv(w)
    q = dev_bf16(qh)
    kc, ks = sa.kv_quant_int8(dev_bf16(kh))
    vc, vs = sa.kv_quant_int8(dev_bf16(vh))
    out = torch.empty_like(q)
    ws = torch.empty((sa.slim_attn_decode_int8_workspace_bytes(B, Hq, Hkv, T, D),), dtype=torch.uint8, device="cuda")
    flush = torch.randint(0, 255, (1 << 30,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    # (as in the full bench: the GPU leaves its idle clocks only after some tens of milliseconds of load)
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(10):
            probes.slim_probe_stream_read(flush, sink)
            sa.slim_attn_decode_int8(q, kc, ks, vc, vs, w.softmax_scale, out=out, workspace=ws)
        torch.cuda.synchronize()
    med, mean, mn = median_ms(torch, lambda: sa.slim_attn_decode_int8(q, kc, ks, vc, vs, w.softmax_scale, out=out, workspace=ws),
                              args.steps, warm=args.warmup, between=lambda: probes.slim_probe_stream_read(flush, sink))
    by = acct.decode_bytes(B, Hq, Hkv, T, D)
    # the same loads without the arithmetic (and without the combine launch): what the memory system charges for this
    # access pattern on this shape
    tmed, tmean, tmn = median_ms(torch, lambda: probes.slim_probe_gqa_decode_traffic(q, kc, ks, vc, vs, ws), args.steps, warm=args.warmup,
                                 between=lambda: probes.slim_probe_stream_read(flush, sink))
    print(json.dumps({"metric": "INT8-KV decode HBM GB/s, grouped query heads", "value": round(by / mean / 1e6, 1), "unit": "GB/s",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(mean, 4), "ms_median": round(med, 4),
                      "ms_min": round(mn, 4), "higher_is_better": True, "dtype": "bf16", "data": "synthetic", "bytes": by,
                      "frac_of_hbm_peak": round(by / mean / 1e6 / PEAK_HBM_GBPS, 4),
                      "loads_only": {"ms": round(tmean, 4), "ms_median": round(tmed, 4), "ms_min": round(tmn, 4),
                                     "GBps": round(by / tmean / 1e6, 1), "frac_of_hbm_peak": round(by / tmean / 1e6 / PEAK_HBM_GBPS, 4)},
                      "config": {"workload": "decode B=16 Hq=64 Hkv=8 T=8192 D=128 INT8 KV", "only": "gqa-decode"}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="before the warm-up steps, run untimed steps for this long: the GPU clocks take about 40 ms of "
                         "load to leave their idle state (the first ~160 steps run up to 1.5x slower)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the workloads reported beside the headline")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="before the steps, run one plain 256 MiB device copy (a kernel of known HBM traffic) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command can be scaled")
    ap.add_argument("--only", choices=["all", "prefill", "decode", "quant", "gqa-decode"], default="all",
                    help="run only one kernel per step (for profiling); the JSON line then carries only its fields.  "
                         "gqa-decode: the grouped-query decode of the other workloads (B=16, 64 query heads on 8 KV heads, "
                         "T=8192), a 1 GiB streaming read before every launch so that the cache comes from HBM")
    ap.add_argument("--probe", choices=["ceilings"], default=None,
                    help="run the measurement kernels instead of the path and print their JSON line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (nothing on the path needs a second); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if args.probe == "ceilings":
        probe_ceilings(args)
        return
    if args.only == "gqa-decode":
        only_gqa_decode(args)
        return

    import torch
    from paper_2407_07304_amd import slimattn as sa
    from paper_2407_07304_amd import accounting as acct
    from paper_2407_07304_amd.inputs import WORKLOADS, make_qkv, make_shape

    sa.load()   # raises if the HIP library has not been built: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    dev_name = torch.cuda.get_device_name(0)
    table3 = paper_table3_ms()
    prof = profiled_traffic()

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    c2, c4 = WORKLOADS["C2"], WORKLOADS["C4"]
    do_prefill = args.only in ("all", "prefill")
    do_quant = args.only in ("all", "quant")
    do_decode = args.only in ("all", "decode")
    do_extras = args.only == "all" and not args.no_extras

    # ---- inputs (host-seeded, then resident in HBM)
    q2h, k2h, v2h = make_qkv(c2)
    q2, k2, v2 = dev_bf16(q2h), dev_bf16(k2h), dev_bf16(v2h)
    o2 = torch.empty_like(q2)
    kc2 = torch.empty(k2.shape, dtype=torch.int8, device="cuda")
    vc2 = torch.empty_like(kc2)
    ks2 = torch.empty(k2.shape[:-1], dtype=torch.float32, device="cuda")
    vs2 = torch.empty_like(ks2)
    if do_decode:
        q4h, k4h, v4h = make_qkv(c4)
        q4 = dev_bf16(q4h)
        k4 = dev_bf16(k4h)
        del k4h
        kc4, ks4 = sa.kv_quant_int8(k4)
        if not do_extras:
            del k4
        vc4, vs4 = sa.kv_quant_int8(dev_bf16(v4h))
        del v4h
        o4 = torch.empty_like(q4)
        ws4 = torch.empty((sa.slim_attn_decode_int8_workspace_bytes(c4.batch, c4.q_heads, c4.kv_heads, c4.seq_len,
                                                                    c4.head_dim),), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()

    def step(ev=None):
        if ev is not None:
            ev[0].record()
        if do_prefill:
            sa.slim_attn_prefill(q2, k2, v2, c2.softmax_scale, True, out=o2)
        if ev is not None:
            ev[1].record()
        if do_quant:
            sa.kv_quant_int8_pair(k2, v2, kc2, ks2, vc2, vs2)
        if ev is not None:
            ev[2].record()
        if do_decode:
            sa.slim_attn_decode_int8(q4, kc4, ks4, vc4, vs4, c4.softmax_scale, out=o4, workspace=ws4)
        if ev is not None:
            ev[3].record()

    if args.traffic_probe:
        src = torch.empty((256 << 20,), dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)        # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    seg = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in events])   # ms: prefill, quant of K and V, decode
    pre_ms, quant_ms, dec_ms = seg.mean(axis=0)
    pre_min, quant_min, dec_min = seg.min(axis=0)
    pre_med, quant_med, dec_med = np.median(seg, axis=0)

    line = {
        "metric": "prefill attn TFLOP/s + INT8-KV decode HBM GB/s, % of MI355X peak",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "device": dev_name,
    }

    pre_flops = acct.prefill_flops(c2.batch, c2.q_heads, c2.seq_len, c2.head_dim, True)
    if do_prefill:
        tfl = pre_flops / (pre_ms * 1e-3) / 1e12
        roof = {"kernel": "slim_prefill_kernel<128,bf16 kv,bf16 out>", "bound": "mfma", "achieved": round(tfl, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tfl / PEAK_BF16_TFLOPS, 4),
                "target_frac": 0.5, "target_met": bool(tfl / PEAK_BF16_TFLOPS >= 0.5)}
        roof.update(traffic_fields(prof, "prefill_c2"))
        line.update({
            "value": round(tfl, 2), "unit": "TFLOP/s",
            "prefill": {"workload": "C2", "ms": round(float(pre_ms), 4), "ms_min": round(float(pre_min), 4),
                        "ms_median": round(float(pre_med), 4), "tflops": round(tfl, 2), "frac_of_bf16_mfma_peak": round(tfl / PEAK_BF16_TFLOPS, 4),
                        "flops": pre_flops,
                        "paper_cpu_ms_context": table3.get(c2.seq_len)},
            "roofline": roof,
        })
    if do_decode:
        dbytes = acct.decode_bytes(c4.batch, c4.q_heads, c4.kv_heads, c4.seq_len, c4.head_dim)
        gbps = dbytes / (dec_ms * 1e-3) / 1e9
        line["decode"] = {"workload": "C4", "value": round(gbps, 1), "unit": "GB/s", "ms": round(float(dec_ms), 4),
                          "ms_min": round(float(dec_min), 4), "ms_median": round(float(dec_med), 4), "bytes": dbytes,
                          "frac_of_hbm_peak": round(gbps / PEAK_HBM_GBPS, 4)}
        roof = {"kernel": "slim_decode_int8_split_kernel<128> + slim_decode_combine_kernel<128>",
                "bound": "hbm", "achieved": round(gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "frac": round(gbps / PEAK_HBM_GBPS, 4), "target_frac": 0.7, "target_met": bool(gbps / PEAK_HBM_GBPS >= 0.7)}
        roof.update(traffic_fields(prof, "decode_c4"))
        line["roofline_decode"] = roof
        if not do_prefill:
            line.update({"value": round(gbps, 1), "unit": "GB/s"})
    if do_quant:
        qbytes = 2 * acct.kv_quant_bytes(c2.batch * c2.kv_heads * c2.seq_len, c2.head_dim)
        qg = qbytes / (quant_ms * 1e-3) / 1e9
        line["kv_quant"] = {"workload": "K and V of C2 (kv_quant_int8_pair: one launch)", "ms": round(float(quant_ms), 4),
                            "ms_median": round(float(quant_med), 4), "GBps": round(qg, 1),
                            "bytes": qbytes, "frac_of_hbm_peak": round(qg / PEAK_HBM_GBPS, 4)}
        if not (do_prefill or do_decode):
            line.update({"value": round(qg, 1), "unit": "GB/s"})
    line["config"] = {
        "workload": "C2 causal prefill B=1 Hq=Hkv=32 S=2048 D=128 bf16 (value); then K,V -> INT8 cache; then "
                    "C4 decode B=16 H=32 D=128 T=8192 INT8 KV (decode.value)",
        "only": args.only, "seeds": {"C2": c2.seed, "C4": c4.seed},
        "settle_ms": args.settle_ms,   # untimed steps before the warm-up steps, until the clocks have left idle
    }

    # ---- the other workloads, beside the headline.  Inputs from the same host generator; K/V quantised by the
    # library's quantiser (the parity tests hold it bit for bit to the oracle's on these very tensors).
    kept = {}   # what the CPU leg below compares: host inputs and sampled GPU output rows of C3 and C5
    if do_extras:
        extras = []
        for name, iters in (("C3", 30), ("C5", 20)):
            w = WORKLOADS[name]
            qh, kh, vh = make_qkv(w)
            qx = dev_bf16(qh)
            kcx, ksx = sa.kv_quant_int8(dev_bf16(kh))
            vcx, vsx = sa.kv_quant_int8(dev_bf16(vh))
            ox = torch.empty_like(qx)
            med, mean, mn = median_ms(torch, lambda: sa.slim_attn_prefill(qx, kcx, vcx, w.softmax_scale, True, k_scale=ksx,
                                                                           v_scale=vsx, out=ox), iters)
            fl = acct.prefill_flops(w.batch, w.q_heads, w.seq_len, w.head_dim, True)
            tf = fl / (mean * 1e-3) / 1e12
            rec = {"workload": name + " causal prefill, INT8 K/V", "launches": iters, "ms": round(mean, 4), "ms_median": round(med, 4),
                   "ms_min": round(mn, 4), "tflops": round(tf, 2), "frac_of_bf16_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4),
                   "paper_cpu_ms_context": table3.get(w.seq_len)}
            rows = _sample_rows(w.seq_len, 57 if name == "C3" else 9, w.seed)
            kept[name] = (w, qh, kh, vh, rows, ox[:, :, torch.from_numpy(rows).long().cuda()].double().cpu().numpy(),
                          kcx.cpu().numpy(), ksx.cpu().numpy(), vcx.cpu().numpy(), vsx.cpu().numpy())
            if name == "C3":
                # information only: what the INT8 cache costs in accuracy (the paper gives no bound): the same
                # attention on the unquantised bf16 K/V, both from this library's kernels
                ob = sa.slim_attn_prefill(qx, dev_bf16(kh), dev_bf16(vh), w.softmax_scale, True)
                torch.cuda.synchronize()
                diff = (ox.float() - ob.float()).abs()
                rec["int8_kv_vs_bf16_kv_output"] = {"max_abs": round(float(diff.max()), 5),
                                                    "mean_abs": round(float(diff.mean()), 6)}
                del ob, diff
            extras.append(rec)
            del qx, kcx, vcx, ksx, vsx, ox

        # ---- C2 prefill that also writes the INT8 cache, against the step's own prefill + two quantiser launches
        med, mean, _ = median_ms(torch, lambda: sa.slim_attn_prefill_emit_int8(q2, k2, v2, c2.softmax_scale, True, out=o2),
                                 50, warm=10, between=step)
        extras.append({"workload": "C2 causal prefill that also emits the INT8 K/V cache (one launch)",
                       "ms": round(mean, 4), "ms_median": round(med, 4),
                       "separate_launches_ms": round(float(pre_ms + quant_ms), 4)})

        # ---- K and V of C2 quantised by two single calls, beside the pair call the step times
        if do_quant:
            def two_calls():
                sa.kv_quant_int8(k2, kc2, ks2)
                sa.kv_quant_int8(v2, vc2, vs2)
            med, mean, _ = median_ms(torch, two_calls, 50, warm=10, between=step)
            qb = 2 * acct.kv_quant_bytes(c2.batch * c2.kv_heads * c2.seq_len, c2.head_dim)
            extras.append({"workload": "kv_quant_int8 on K, then on V of C2 (two launches)", "ms": round(mean, 4),
                           "ms_median": round(med, 4), "GBps": round(qb / (mean * 1e-3) / 1e9, 1), "bytes": qb,
                           "pair_ms": round(float(quant_ms), 4)})

        # ---- the two full-row orders of section 2.1 on C2, beside the streamed one-sweep kernel the step times
        ws2 = torch.empty((c2.batch * c2.q_heads * c2.seq_len * 2,), dtype=torch.float32, device="cuda")
        med, mean, _ = median_ms(torch, lambda: sa.slim_attn_prefill_two_sweep(q2, k2, v2, c2.softmax_scale, True, out=o2,
                                                                                workspace=ws2), 50, warm=10, between=step)
        extras.append({"workload": "C2 causal prefill in two sweeps over K (comparison variant, two launches)",
                       "ms": round(mean, 4), "ms_median": round(med, 4), "one_sweep_ms": round(float(pre_ms), 4)})
        del ws2
        if hasattr(sa, "slim_attn_prefill_strip"):
            med, mean, _ = median_ms(torch, lambda: sa.slim_attn_prefill_strip(q2, k2, v2, c2.softmax_scale, True, out=o2),
                                     50, warm=10, between=step)
            fl = acct.prefill_flops(c2.batch, c2.q_heads, c2.seq_len, c2.head_dim, True)
            extras.append({"workload": "C2 causal prefill with the whole score strip of a row block on chip (comparison "
                                       "variant, one launch)", "ms": round(mean, 4), "ms_median": round(med, 4),
                           "tflops": round(fl / (mean * 1e-3) / 1e12, 2), "one_sweep_ms": round(float(pre_ms), 4)})

        # ---- decode on the grouped-query shape of the paper's larger model (64 query heads on 8 KV heads)
        Bg, Hqg, Hkvg, Tg, Dg = 16, 64, 8, 8192, 128
        wg = make_shape("decode", Bg, Hqg, Hkvg, Tg, Dg, False, True, False, 6, name="GQA decode")
        qgh, kgh, vgh = make_qkv(wg)
        qg_ = dev_bf16(qgh)
        kcg, ksg = sa.kv_quant_int8(dev_bf16(kgh))
        vcg, vsg = sa.kv_quant_int8(dev_bf16(vgh))
        del kgh, vgh
        og = torch.empty_like(qg_)
        wsg = torch.empty((sa.slim_attn_decode_int8_workspace_bytes(Bg, Hqg, Hkvg, Tg, Dg),), dtype=torch.uint8, device="cuda")
        # (the C4 decode of a step streams 1.1 GB: this cache, 277 MB, is out of the caches again before every launch)
        med, mean, _ = median_ms(torch, lambda: sa.slim_attn_decode_int8(qg_, kcg, ksg, vcg, vsg, wg.softmax_scale, out=og,
                                                                          workspace=wsg), 50, warm=10, between=step)
        gbytes = acct.decode_bytes(Bg, Hqg, Hkvg, Tg, Dg)
        # The same launch with a memory-bound neighbour, as in a decode loop: after a 1 GiB streaming read instead of
        # after a whole step (whose prefill leaves the chip at a lower clock under its power cap).
        from paper_2407_07304_amd import probes
        probes.load()
        flush = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda").random_(0, 255)
        sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
        t_settle = time.perf_counter()   # (a decode loop runs for seconds: let the clocks settle on this load first)
        while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
            for _ in range(10):
                probes.slim_probe_stream_read(flush, sink)
                sa.slim_attn_decode_int8(qg_, kcg, ksg, vcg, vsg, wg.softmax_scale, out=og, workspace=wsg)
            torch.cuda.synchronize()
        med_s, mean_s, _ = median_ms(torch, lambda: sa.slim_attn_decode_int8(qg_, kcg, ksg, vcg, vsg, wg.softmax_scale, out=og,
                                                                              workspace=wsg), 50, warm=10,
                                     between=lambda: probes.slim_probe_stream_read(flush, sink))
        extras.append({"workload": "decode B=16 Hq=64 Hkv=8 T=8192 D=128 INT8 KV (grouped query heads)",
                       "ms": round(mean, 4), "ms_median": round(med, 4),
                       "GBps": round(gbytes / (mean * 1e-3) / 1e9, 1), "bytes": gbytes,
                       "frac_of_hbm_peak": round(gbytes / (mean * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                       "after_a_streaming_read": {"ms": round(mean_s, 4), "ms_median": round(med_s, 4),
                                                  "GBps": round(gbytes / (mean_s * 1e-3) / 1e9, 1),
                                                  "frac_of_hbm_peak": round(gbytes / (mean_s * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)}})
        del kcg, ksg, vcg, vsg, wsg
        # the same head layout over caches four times as long (1.07 GB of codes, the bytes of C4): the launch is no
        # longer over in forty microseconds, so this is the kernel's own streaming rate.  Timing only: codes and scales
        # are drawn on the device, nothing is compared.
        Tl = 4 * Tg
        gen = torch.Generator(device="cuda").manual_seed(7)
        kcl = torch.randint(-127, 128, (Bg, Hkvg, Tl, Dg), dtype=torch.int8, device="cuda", generator=gen)
        vcl = torch.randint(-127, 128, (Bg, Hkvg, Tl, Dg), dtype=torch.int8, device="cuda", generator=gen)
        ksl = torch.rand((Bg, Hkvg, Tl), dtype=torch.float32, device="cuda", generator=gen) * 0.02 + 0.02
        vsl = torch.rand((Bg, Hkvg, Tl), dtype=torch.float32, device="cuda", generator=gen) * 0.02 + 0.02
        wsl = torch.empty((sa.slim_attn_decode_int8_workspace_bytes(Bg, Hqg, Hkvg, Tl, Dg),), dtype=torch.uint8, device="cuda")
        med, mean, _ = median_ms(torch, lambda: sa.slim_attn_decode_int8(qg_, kcl, ksl, vcl, vsl, wg.softmax_scale, out=og,
                                                                          workspace=wsl), 20, warm=5, between=step)
        lbytes = acct.decode_bytes(Bg, Hqg, Hkvg, Tl, Dg)
        t_settle = time.perf_counter()   # (and as a decode loop, as above)
        while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
            for _ in range(5):
                probes.slim_probe_stream_read(flush, sink)
                sa.slim_attn_decode_int8(qg_, kcl, ksl, vcl, vsl, wg.softmax_scale, out=og, workspace=wsl)
            torch.cuda.synchronize()
        med_s, mean_s, _ = median_ms(torch, lambda: sa.slim_attn_decode_int8(qg_, kcl, ksl, vcl, vsl, wg.softmax_scale, out=og,
                                                                              workspace=wsl), 20, warm=5,
                                     between=lambda: probes.slim_probe_stream_read(flush, sink))
        extras.append({"workload": "decode B=16 Hq=64 Hkv=8 T=32768 D=128 INT8 KV (grouped query heads, long caches; "
                                   "device-drawn codes, timing only)",
                       "ms": round(mean, 4), "ms_median": round(med, 4),
                       "GBps": round(lbytes / (mean * 1e-3) / 1e9, 1), "bytes": lbytes,
                       "frac_of_hbm_peak": round(lbytes / (mean * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                       "after_a_streaming_read": {"ms": round(mean_s, 4), "ms_median": round(med_s, 4),
                                                  "GBps": round(lbytes / (mean_s * 1e-3) / 1e9, 1),
                                                  "frac_of_hbm_peak": round(lbytes / (mean_s * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)}})
        del qg_, og, kcl, vcl, ksl, vsl, wsl, flush

        # ---- the quantiser on a stream that no cache holds: K of the C4 cache (1.07 GB in, 0.54 GB out)
        if do_decode:
            med, mean, _ = median_ms(torch, lambda: sa.kv_quant_int8(k4, kc4, ks4), 20)   # (the same codes again)
            sbytes = acct.kv_quant_bytes(c4.batch * c4.kv_heads * c4.seq_len, c4.head_dim)
            extras.append({"workload": "kv_quant_int8 on K of C4 (B=16, 32 heads, 8192 tokens: 1.07 GB bf16 in, 0.55 GB out)",
                           "ms": round(mean, 4), "ms_median": round(med, 4), "GBps": round(sbytes / (mean * 1e-3) / 1e9, 1),
                           "bytes": sbytes, "frac_of_hbm_peak": round(sbytes / (mean * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)})
            del k4
        line["other_workloads"] = extras

    # ---- the CPU oracle on this host's cores, beside the GPU numbers (a baseline, not a target), and the GPU
    # outputs held against it
    if not args.no_cpu_baseline and do_prefill:
        import oracle
        sa.slim_attn_prefill(q2, k2, v2, c2.softmax_scale, True, out=o2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        want = oracle.attn(q2h, k2h, v2h, c2.softmax_scale, True)   # the whole C2 tensor: under a second on the box
        dt = time.perf_counter() - t0
        err = np.abs(o2.double().cpu().numpy() - want)
        fl = acct.prefill_flops(c2.batch, c2.q_heads, c2.seq_len, c2.head_dim, True)
        line["cpu_baseline"] = {"value": round(fl / dt / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
                                "cpu_model": _cpu_model(), "kind": "oracle", "seconds": round(dt, 3),
                                "sample": "the whole C2 tensor: 32 heads, 2048 rows (fp64 scalar C, OpenMP)",
                                "gpu_vs_oracle": {"max_abs": float("%.3e" % err.max()), "mean_abs": float("%.3e" % err.mean())}}
        del want, err
        if do_decode:
            kc, ks, vc, vs = (t.cpu().numpy() for t in (kc4, ks4, vc4, vs4))
            t0 = time.perf_counter()
            want = oracle.attn(q4h, kc, vc, c4.softmax_scale, False, k_scale=ks, v_scale=vs)
            dt = time.perf_counter() - t0
            err = np.abs(o4.double().cpu().numpy() - want)
            by = acct.decode_bytes(c4.batch, c4.q_heads, c4.kv_heads, c4.seq_len, c4.head_dim)
            line["cpu_baseline_decode"] = {"value": round(by / dt / 1e9, 3), "unit": "GB/s",
                                           "cores": oracle.num_threads(), "kind": "oracle", "seconds": round(dt, 3),
                                           "sample": "the whole C4 step: 16 sequences, 32 heads, 8192 tokens",
                                           "gpu_vs_oracle": {"max_abs": float("%.3e" % err.max()), "mean_abs": float("%.3e" % err.mean())}}
            del kc, ks, vc, vs, want
        others = []
        for name, (w, qh, kh, vh, rows, got, gkc, gks, gvc, gvs) in kept.items():
            okc, oks = oracle.kv_quant_int8(kh)
            ovc, ovs = oracle.kv_quant_int8(vh)
            exact = bool(np.array_equal(okc, gkc) and np.array_equal(ovc, gvc) and
                         np.array_equal(oks.view(np.uint32), gks.view(np.uint32)) and np.array_equal(ovs.view(np.uint32), gvs.view(np.uint32)))
            t0 = time.perf_counter()
            want = oracle.attn(qh, okc, ovc, w.softmax_scale, True, k_scale=oks, v_scale=ovs, rows=rows)
            dt = time.perf_counter() - t0
            err = np.abs(got - want)
            others.append({"workload": name, "kind": "oracle", "sample": "%d query rows of every head" % rows.size,
                           "seconds": round(dt, 3), "int8_cache_bit_exact": exact,
                           "gpu_vs_oracle": {"max_abs": float("%.3e" % err.max()), "mean_abs": float("%.3e" % err.mean())}})
        if others:
            line["cpu_baseline_other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()

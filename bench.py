#!/usr/bin/env python3
"""Benchmark of the SlimAttention hot path on one MI355X.

One step = one pass of the whole path over seeded synthetic inputs already resident in HBM:
  1. slim_attn_prefill   causal prefill, Llama-2-7B shape (B=1, 32 heads, S=2048, D=128, bf16)
  2. kv_quant_int8       the prompt's K and V -> INT8 cache (+ one fp32 scale per token per head)
  3. slim_attn_decode_int8  one decode step, B=16, 32 heads, D=128, INT8 cache of 8192 tokens

`value` is the prefill throughput in TFLOP/s (causal flop count) and `decode.value` the
decode throughput in GB/s (algorithmic bytes), each from HIP-event timing of its own
kernel(s) inside the timed steps.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E

PAPER_TABLE3_MS = {2048: 96.65, 4096: 392.80}   # SlimAttention, 1 socket Xeon 8563C (paper Table 3); context only


def measured_traffic():
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary, or {}."""
    path = os.path.join(ROOT, "profiles", "traffic_fetch_write_c2_c4.txt")
    out = {}
    try:
        for ln in open(path):
            if ln.startswith("traffic_bytes "):
                _, key, val = ln.split()
                out[key] = int(float(val))
    except OSError:
        pass
    return out


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.startswith("model name"):
                    return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="before the warm-up steps, run untimed steps for this long: the GPU clocks take about 40 ms of "
                         "load to leave their idle state (the first ~160 steps run up to 1.5x slower)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the INT8 prefill workloads reported beside the headline")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="before the steps, run one plain 256 MiB device copy (a kernel of known HBM traffic) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command can be scaled")
    ap.add_argument("--only", choices=["all", "prefill", "decode", "quant"], default="all",
                    help="run only one kernel per step (for profiling); the JSON line then carries only its fields")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (nothing on the path needs a second); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2407_07304_amd import slimattn as sa
    from paper_2407_07304_amd import accounting as acct
    from paper_2407_07304_amd.inputs import WORKLOADS, make_qkv

    sa.load()   # raises if the HIP library has not been built: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    dev_name = torch.cuda.get_device_name(0)

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    c2, c4 = WORKLOADS["C2"], WORKLOADS["C4"]
    do_prefill = args.only in ("all", "prefill")
    do_quant = args.only in ("all", "quant")
    do_decode = args.only in ("all", "decode")

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
        kc4, ks4 = sa.kv_quant_int8(dev_bf16(k4h))
        del k4h
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
            sa.kv_quant_int8(k2, kc2, ks2)
            sa.kv_quant_int8(v2, vc2, vs2)
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
    seg = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in events])   # ms: prefill, quant x2, decode
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
        line.update({
            "value": round(tfl, 2), "unit": "TFLOP/s",
            "prefill": {"workload": "C2", "ms": round(float(pre_ms), 4), "ms_min": round(float(pre_min), 4),
                        "ms_median": round(float(pre_med), 4), "tflops": round(tfl, 2), "frac_of_bf16_mfma_peak": round(tfl / PEAK_BF16_TFLOPS, 4),
                        "flops": pre_flops,
                        "paper_cpu_ms_context": PAPER_TABLE3_MS[2048]},
            "roofline": {"kernel": "slim_prefill_kernel<128,bf16 kv,bf16 out>", "bound": "mfma", "achieved": round(tfl, 2),
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tfl / PEAK_BF16_TFLOPS, 4),
                         "traffic": measured_traffic().get("prefill_c2")},
        })
    if do_decode:
        dbytes = acct.decode_bytes(c4.batch, c4.q_heads, c4.kv_heads, c4.seq_len, c4.head_dim)
        gbps = dbytes / (dec_ms * 1e-3) / 1e9
        line["decode"] = {"workload": "C4", "value": round(gbps, 1), "unit": "GB/s", "ms": round(float(dec_ms), 4),
                          "ms_min": round(float(dec_min), 4), "ms_median": round(float(dec_med), 4), "bytes": dbytes,
                          "frac_of_hbm_peak": round(gbps / PEAK_HBM_GBPS, 4)}
        line["roofline_decode"] = {"kernel": "slim_decode_int8_split_kernel<128> + slim_decode_combine_kernel<128>",
                                   "bound": "hbm", "achieved": round(gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                   "frac": round(gbps / PEAK_HBM_GBPS, 4),
                                   "traffic": measured_traffic().get("decode_c4")}
        if not do_prefill:
            line.update({"value": round(gbps, 1), "unit": "GB/s"})
    if do_quant:
        qbytes = 2 * acct.kv_quant_bytes(c2.batch * c2.kv_heads * c2.seq_len, c2.head_dim)
        qg = qbytes / (quant_ms * 1e-3) / 1e9
        line["kv_quant"] = {"workload": "K and V of C2", "ms": round(float(quant_ms), 4),
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

    # ---- INT8-KV prefill workloads beside the headline (device-seeded N(0,1); a few launches each)
    if args.only == "all" and not args.no_extras:
        extras = []
        for name, iters in (("C3", 10), ("C5", 3)):
            w = WORKLOADS[name]
            g = torch.Generator(device="cuda")
            g.manual_seed(w.seed)
            qx = torch.randn((w.batch, w.q_heads, w.seq_len, w.head_dim), generator=g, device="cuda",
                             dtype=torch.float32).to(torch.bfloat16)
            kx = torch.randn((w.batch, w.kv_heads, w.seq_len, w.head_dim), generator=g, device="cuda",
                             dtype=torch.float32).to(torch.bfloat16)
            vx = torch.randn((w.batch, w.kv_heads, w.seq_len, w.head_dim), generator=g, device="cuda",
                             dtype=torch.float32).to(torch.bfloat16)
            kcx, ksx = sa.kv_quant_int8(kx)
            vcx, vsx = sa.kv_quant_int8(vx)
            ox = torch.empty_like(qx)
            for _ in range(2):
                sa.slim_attn_prefill(qx, kcx, vcx, w.softmax_scale, True, k_scale=ksx, v_scale=vsx, out=ox)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                sa.slim_attn_prefill(qx, kcx, vcx, w.softmax_scale, True, k_scale=ksx, v_scale=vsx, out=ox)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / iters
            fl = acct.prefill_flops(w.batch, w.q_heads, w.seq_len, w.head_dim, True)
            tf = fl / (ms * 1e-3) / 1e12
            rec = {"workload": name + " causal prefill, INT8 K/V", "ms": round(ms, 4), "tflops": round(tf, 2),
                   "frac_of_bf16_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4),
                   "paper_cpu_ms_context": PAPER_TABLE3_MS.get(w.seq_len)}
            if name == "C3":
                # information only: what the INT8 cache costs in accuracy (the paper gives no bound): the same
                # attention on the unquantised bf16 K/V, both from this library's kernels
                ob = sa.slim_attn_prefill(qx, kx, vx, w.softmax_scale, True)
                torch.cuda.synchronize()
                diff = (ox.float() - ob.float()).abs()
                rec["int8_kv_vs_bf16_kv_output"] = {"max_abs": round(float(diff.max()), 5),
                                                    "mean_abs": round(float(diff.mean()), 6)}
                del ob, diff
            extras.append(rec)
            del qx, kx, vx, kcx, vcx, ksx, vsx, ox
        # ---- C2 prefill that also writes the INT8 cache, against the step's own prefill + two quantiser launches
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
        for i in range(60):
            step()
            if i >= 10:
                evs[i - 10][0].record()
            sa.slim_attn_prefill_emit_int8(q2, k2, v2, c2.softmax_scale, True, out=o2)
            if i >= 10:
                evs[i - 10][1].record()
        torch.cuda.synchronize()
        te = np.array([a.elapsed_time(b) for a, b in evs])
        extras.append({"workload": "C2 causal prefill that also emits the INT8 K/V cache (one launch)",
                       "ms": round(float(te.mean()), 4), "ms_median": round(float(np.median(te)), 4),
                       "separate_launches_ms": round(float(pre_ms + quant_ms), 4)})

        # ---- C2 in the two-sweep order (row maxima first, then the exponentials against them), beside the
        # one-sweep kernel the step times
        ws2 = torch.empty((c2.batch * c2.q_heads * c2.seq_len * 2,), dtype=torch.float32, device="cuda")
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
        for i in range(60):
            step()
            if i >= 10:
                evs[i - 10][0].record()
            sa.slim_attn_prefill_two_sweep(q2, k2, v2, c2.softmax_scale, True, out=o2, workspace=ws2)
            if i >= 10:
                evs[i - 10][1].record()
        torch.cuda.synchronize()
        tt = np.array([a.elapsed_time(b) for a, b in evs])
        extras.append({"workload": "C2 causal prefill in two sweeps over K (comparison variant, two launches)",
                       "ms": round(float(tt.mean()), 4), "ms_median": round(float(np.median(tt)), 4),
                       "one_sweep_ms": round(float(pre_ms), 4)})
        del ws2

        # ---- decode on the grouped-query shape of the paper's larger model (64 query heads on 8 KV heads)
        Bg, Hqg, Hkvg, Tg, Dg = 16, 64, 8, 8192, 128
        g = torch.Generator(device="cuda")
        g.manual_seed(6)
        qg = torch.randn((Bg, Hqg, 1, Dg), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        caches = []
        for _ in range(2):
            x = torch.randn((Bg, Hkvg, Tg, Dg), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
            caches.append(sa.kv_quant_int8(x))
            del x
        (kcg, ksg), (vcg, vsg) = caches
        og = torch.empty_like(qg)
        wsg = torch.empty((sa.slim_attn_decode_int8_workspace_bytes(Bg, Hqg, Hkvg, Tg, Dg),), dtype=torch.uint8, device="cuda")
        sg = 1.0 / float(np.sqrt(Dg))
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
        for i in range(60):
            step()   # the C4 decode of a step streams 1.1 GB: this cache (277 MB) is out of the caches again
            if i >= 10:
                evs[i - 10][0].record()
            sa.slim_attn_decode_int8(qg, kcg, ksg, vcg, vsg, sg, out=og, workspace=wsg)
            if i >= 10:
                evs[i - 10][1].record()
        torch.cuda.synchronize()
        tg = np.array([a.elapsed_time(b) for a, b in evs])
        gbytes = acct.decode_bytes(Bg, Hqg, Hkvg, Tg, Dg)
        extras.append({"workload": "decode B=16 Hq=64 Hkv=8 T=8192 D=128 INT8 KV (grouped query heads)",
                       "ms": round(float(tg.mean()), 4), "ms_median": round(float(np.median(tg)), 4),
                       "GBps": round(gbytes / (tg.mean() * 1e-3) / 1e9, 1), "bytes": gbytes,
                       "frac_of_hbm_peak": round(gbytes / (tg.mean() * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)})
        del qg, kcg, ksg, vcg, vsg, og, wsg
        line["other_workloads"] = extras

    # ---- the CPU oracle on this host's cores, beside the GPU number (a baseline, not a target)
    if not args.no_cpu_baseline and do_prefill:
        import oracle
        n_heads = c2.q_heads                          # the whole C2 tensor: under a second of CPU work on the box
        t0 = time.perf_counter()
        oracle.attn(q2h[:, :n_heads], k2h[:, :n_heads], v2h[:, :n_heads], c2.softmax_scale, True)
        dt = time.perf_counter() - t0
        fl = acct.prefill_flops(c2.batch, n_heads, c2.seq_len, c2.head_dim, True)
        line["cpu_baseline"] = {"value": round(fl / dt / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
                                "cpu_model": _cpu_model(), "kind": "oracle", "seconds": round(dt, 3),
                                "sample": "the whole C2 tensor: 32 heads, 2048 rows (fp64 scalar C, OpenMP)"}
        if do_decode:
            nb = c4.batch
            kc, ks, vc, vs = (t[:nb].cpu().numpy() for t in (kc4, ks4, vc4, vs4))
            t0 = time.perf_counter()
            oracle.attn(q4h[:nb], kc, vc, c4.softmax_scale, False, k_scale=ks, v_scale=vs)
            dt = time.perf_counter() - t0
            by = acct.decode_bytes(nb, c4.q_heads, c4.kv_heads, c4.seq_len, c4.head_dim)
            line["cpu_baseline_decode"] = {"value": round(by / dt / 1e9, 3), "unit": "GB/s",
                                           "cores": oracle.num_threads(), "kind": "oracle", "seconds": round(dt, 3),
                                           "sample": "the whole C4 step: 16 sequences, 32 heads, 8192 tokens"}
    print(json.dumps(line))


if __name__ == "__main__":
    main()

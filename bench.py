#!/usr/bin/env python3
"""Benchmark of the PASA attention-forward hot path on one MI355X.

A step is one pass of the whole path (key pre-processing kernel + main attention kernel, through the
C ABI) over the Qwen2-7B-shaped GQA prefill workload (B=1, Hq=28, Hkv=4, d=128, N=8192, causal) with
synthetic seeded inputs already resident in HBM.  Prints ONE JSON line.

  value      counted FLOPs (4*B*Hq*N^2*d, halved for causal) / wall time per step, TFLOP/s
  roofline   the main kernel alone: counted FLOPs per launch / its mean duration between HIP events
             recorded on the launch stream inside the timed region, against the dense fp16 MFMA peak
  variants   the same launch timed for PASA_STRICT16 (every quantity Algorithm 1 marks is rounded to fp16), outside
             the timed region of the headline figure
  overflow   counts from instrumented calls (not timed): score-tile entries beyond 65504 where they would be stored
             as fp16 and non-finite outputs, for PASA and for the unshifted fp16-score FlashAttention, on this
             workload and on the large-bias workload
  cpu_baseline  the numpy fp64 oracle timed on this machine's host cores on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0      # MI355X dense fp16 MFMA, published
WORKLOAD = "qwen2_gqa_n8192"
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "pasa_fwd_qwen2_gqa_n8192_hbm_traffic.txt")


def kernel_source_hash():
    """Hash of the kernel source as the compiler sees it: `//` comments and blank space do not count."""
    import hashlib
    h = hashlib.sha256()
    with open(os.path.join(ROOT, "paper_2503_01873_amd", "csrc", "pasa_kernels.hip"), "r") as f:
        for line in f:
            code = " ".join(line.split("//")[0].split())
            if code:
                h.update(code.encode() + b"\n")
    return h.hexdigest()[:16]


def read_traffic(source_hash=None):
    """HBM bytes per main-kernel launch from the committed rocprofv3 --pmc summary -- only if that summary was
    measured on the kernel source that is in the tree now (it names the source's hash); otherwise None."""
    traffic = stamp = None
    try:
        for line in open(TRAFFIC_FILE):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
            if line.startswith("kernel_source_sha256_16:"):
                stamp = line.split(":")[1].strip()
        if source_hash is None:
            source_hash = kernel_source_hash()
    except OSError:
        return None
    return traffic if (stamp is not None and stamp == source_hash) else None


def cpu_baseline(w, q_heads, kv_heads, scale, budget_s=12.0):
    """Time the oracle's plain-definition attention on sampled (head, 128-row block) units."""
    import numpy as np
    from oracle import pasa_oracle as po
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    rng = np.random.default_rng(123)
    nblk = w.N // 128
    # first and last block of every head first, then the remaining blocks in a seeded random order
    units = [(h, b) for h in range(w.Hq) for b in (0, nblk - 1)]
    rest = [(h, b) for h in range(w.Hq) for b in range(1, nblk - 1)]
    rng.shuffle(rest)
    units += [tuple(int(x) for x in u) for u in rest]
    pairs = 0
    done = 0
    t0 = time.perf_counter()
    for h, blk in units:
        r0 = blk * 128
        nk = r0 + 128 if w.causal else w.N
        kk, vv = kv_heads[h // w.group]
        po.attention_fp64(q_heads[h][r0:r0 + 128], kk[:nk], vv[:nk], scale, w.causal, r0)
        # same convention as the GPU figure: N^2/2 pairs per head when causal
        pairs += 128 * (r0 + 64) if w.causal else 128 * w.N
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    flops = 4.0 * w.d * pairs
    return {
        "value": flops / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": int(cores),
        "kind": "oracle",
        "sample": f"{done} of {len(units)} (head, 128-row block) units of {w.name}, first and last block of every "
                  f"head included, {dt:.1f} s wall, numpy fp64 plain-definition attention; the whole workload "
                  f"extrapolates to {w.flops / (flops / dt):.0f} s",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--settle-ms", type=float, default=500.0,
                    help="before the warmup steps, run untimed steps for this long: an idle GPU takes some hundred "
                         "steps of this size to reach its sustained clock, and steps timed before that run 9 %% slower")
    ap.add_argument("--variant", default="mixed", choices=["mixed", "strict16", "s16", "naive16", "direct"])
    ap.add_argument("--workload", default=WORKLOAD,
                    help="another of the five configurations by name (for profiles of the other shapes; no accuracy check "
                         "or CPU baseline then, and the committed HBM-traffic figure is not attached).  The default is the "
                         "configuration the metric's target is quoted on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-accuracy", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the STRICT16 timing and the overflow counts")
    ap.add_argument("--extra-steps", type=int, default=300, help="timed steps of the STRICT16 leg")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (a known-size reference for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding or collectives are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2503_01873_amd as P
    from workloads import workload, gen_q_head, gen_kv_head

    variant = {"mixed": P.MIXED, "strict16": P.STRICT16, "s16": P.S16, "naive16": P.NAIVE16,
               "direct": P.DIRECT}[args.variant]
    w = workload(args.workload)
    if args.workload != WORKLOAD:
        args.no_accuracy = args.no_cpu_baseline = args.no_extras = True
    scale = float(np.float32(w.scale))
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    q_heads = [gen_q_head(w, 0, h) for h in range(w.Hq)]          # batch 0 is kept on the host for the accuracy sample
    kv_heads = [gen_kv_head(w, 0, hk) for hk in range(w.Hkv)]
    tq = torch.empty((w.B, w.Hq, w.N, w.d), dtype=torch.float16, device=dev)
    tk = torch.empty((w.B, w.Hkv, w.N, w.d), dtype=torch.float16, device=dev)
    tv = torch.empty_like(tk)
    for b in range(w.B):
        for h in range(w.Hq):
            tq[b, h].copy_(torch.from_numpy(q_heads[h] if b == 0 else gen_q_head(w, b, h)))
        for hk in range(w.Hkv):
            kk, vv = kv_heads[hk] if b == 0 else gen_kv_head(w, b, hk)
            tk[b, hk].copy_(torch.from_numpy(kk))
            tv[b, hk].copy_(torch.from_numpy(vv))
    to = torch.full_like(tq, float("nan"))
    wsb = P.pasa_attn_fwd_workspace(w.B, w.Hq, w.Hkv, w.N, w.d)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    dims = (w.B, w.Hq, w.Hkv, w.N, w.d)

    def step(ev=None):
        P.pasa_prepare_kv(tk, tv, w.B, w.Hkv, w.N, w.d, scale, ws, wsb, stream, variant=variant)
        if ev is not None:
            ev[0].record(stream)
        P.pasa_attn_fwd_prepared(tq, to, *dims, w.causal, scale, ws, wsb, stream, variant=variant)
        if ev is not None:
            ev[1].record(stream)

    if args.copy_calibration_mib > 0:
        src = torch.ones(args.copy_calibration_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    settle_steps = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
        settle_steps += 20
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    kern_all = np.array([a.elapsed_time(b) for a, b in events])
    kern_ms = float(kern_all.mean())
    prop = torch.cuda.get_device_properties(dev)
    tflops = w.flops / (ms_per_step * 1e-3) / 1e12
    kern_tflops = w.flops / (kern_ms * 1e-3) / 1e12

    out = {
        "metric": "pasa_fp16_attn_fwd_tflops",
        "value": tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_steps": settle_steps,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "N": w.N, "d": w.d, "causal": w.causal,
                   "variant": args.variant, "beta": "63.5/64.5", "shift_tile": 128,
                   "mfma_accumulate": "fp32 (hardware); fp16 roundings applied where Algorithm 1 marks them"},
        "frac_of_fp16_mfma_peak": tflops / PEAK_FP16_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": "pasa_fwd", "achieved": kern_tflops, "peak": PEAK_FP16_TFLOPS,
                     "unit": "TFLOP/s", "frac": kern_tflops / PEAK_FP16_TFLOPS,
                     "traffic": read_traffic() if args.workload == WORKLOAD else None,
                     "kernel_ms": kern_ms, "kernel_ms_median": float(np.median(kern_all)),
                     "kernel_ms_min": float(kern_all.min()), "flops_per_launch": w.flops},
        "device": {"name": prop.name, "arch": getattr(prop, "gcnArchName", ""), "compute_units": prop.multi_processor_count,
                   "peak_used": "2500 TFLOP/s dense fp16 MFMA (256 CUs x 4 SIMDs x 1024 FLOP/clk x 2.4 GHz)"},
    }

    if not args.no_extras:
        o_keep = to.clone()                      # the headline variant's output, for the accuracy leg below

        # ---- the fp16-rounded variant Algorithm 1 defines, same launch, timed on its own
        def step_v(var, ev=None):
            P.pasa_prepare_kv(tk, tv, w.B, w.Hkv, w.N, w.d, scale, ws, wsb, stream, variant=var)
            if ev is not None:
                ev[0].record(stream)
            P.pasa_attn_fwd_prepared(tq, to, *dims, w.causal, scale, ws, wsb, stream, variant=var)
            if ev is not None:
                ev[1].record(stream)

        out["variants"] = {}
        for name, var in (("strict16", P.STRICT16),):
            for _ in range(100):
                step_v(var)
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                   for _ in range(args.extra_steps)]
            t1 = time.perf_counter()
            for i in range(args.extra_steps):
                step_v(var, evs[i])
            torch.cuda.synchronize()
            dt1 = time.perf_counter() - t1
            kms = float(np.mean([a.elapsed_time(b) for a, b in evs]))
            out["variants"][name] = {"kernel_ms": kms, "ms_per_step": dt1 * 1e3 / args.extra_steps,
                                     "tflops": w.flops / (kms * 1e-3) / 1e12,
                                     "frac": w.flops / (kms * 1e-3) / 1e12 / PEAK_FP16_TFLOPS, "steps": args.extra_steps}

        # ---- overflow counts (instrumented builds of the same kernels, one call each, not timed)
        def counts(wl, q_, k_, v_, o_, ws_, wsb_, var):
            cnt = torch.zeros(2, dtype=torch.int64, device=dev)
            P.pasa_attn_fwd_ex(q_, k_, v_, o_, wl.B, wl.Hq, wl.Hkv, wl.N, wl.d, wl.causal, float(np.float32(wl.scale)),
                               ws_, wsb_, stream, variant=var, overflow_s=cnt[0:1], nonfinite_o=cnt[1:2])
            torch.cuda.synchronize()
            c = cnt.tolist()
            return int(c[0]), int(c[1])

        w2 = workload("overflow_bias")
        q2 = torch.empty((w2.B, w2.Hq, w2.N, w2.d), dtype=torch.float16, device=dev)
        k2 = torch.empty((w2.B, w2.Hkv, w2.N, w2.d), dtype=torch.float16, device=dev)
        v2 = torch.empty_like(k2)
        for h in range(w2.Hq):
            q2[0, h].copy_(torch.from_numpy(gen_q_head(w2, 0, h)))
        for hk in range(w2.Hkv):
            kk, vv = gen_kv_head(w2, 0, hk)
            k2[0, hk].copy_(torch.from_numpy(kk))
            v2[0, hk].copy_(torch.from_numpy(vv))
        o2 = torch.empty_like(q2)
        wsb2 = P.pasa_attn_fwd_workspace(w2.B, w2.Hq, w2.Hkv, w2.N, w2.d)
        ws2 = torch.empty(wsb2, dtype=torch.uint8, device=dev)
        ov = {}
        for wl, args_ in ((w, (tq, tk, tv, to, ws, wsb)), (w2, (q2, k2, v2, o2, ws2, wsb2))):
            entries = wl.B * wl.Hq * wl.N * wl.N // (2 if wl.causal else 1)
            row = {"score_entries_counted_convention": entries}
            for name, var in (("pasa_mixed", P.MIXED), ("pasa_strict16", P.STRICT16), ("naive16", P.NAIVE16)):
                s_over, o_bad = counts(wl, *args_, var)
                row[name] = {"s_over_65504": s_over, "nonfinite_o": o_bad}
            ov[wl.name] = row
        out["overflow"] = ov
        to.copy_(o_keep)

    if not args.no_accuracy:
        from oracle import pasa_oracle as po
        pol = {P.MIXED: po.MIXED, P.STRICT16: po.STRICT16, P.S16: po.PARTIAL16}.get(variant)
        o_host = to.cpu().numpy()
        num = den = 0.0
        maxabs = 0.0
        for h, r0 in ((0, 0), (9, 2048), (18, 6016), (27, w.N - 128)):
            kk, vv = kv_heads[h // w.group]
            gold = po.attention_fp64(q_heads[h][r0:r0 + 128], kk[:r0 + 128], vv[:r0 + 128], scale, True, r0)
            got = o_host[0, h, r0:r0 + 128].astype(np.float64)
            num += ((got - gold) ** 2).sum()
            den += (gold ** 2).sum()
            if variant == P.DIRECT:      # the recovery that is not the paper's: its own oracle function
                ref = po.direct_rows(q_heads[h][r0:r0 + 128], kk[:r0 + 128], vv[:r0 + 128], scale, True,
                                     po.default_beta(), 128, po.MIXED, r0).astype(np.float64)
                maxabs = max(maxabs, float(np.abs(got - ref).max()))
            elif pol is not None:
                ref = po.pasa_rows(q_heads[h][r0:r0 + 128], kk[:r0 + 128], vv[:r0 + 128], scale, True,
                                   po.default_beta(), 128, pol, r0).astype(np.float64)
                maxabs = max(maxabs, float(np.abs(got - ref).max()))
        out["accuracy"] = {"rmse_vs_fp64": float((num / den) ** 0.5), "maxabs_vs_oracle": maxabs,
                           "nonfinite_outputs": int((~np.isfinite(o_host)).sum()),
                           "sample": "4 (head, 128-row block) units"}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, q_heads, kv_heads, scale)

    print(json.dumps(out))


if __name__ == "__main__":
    main()

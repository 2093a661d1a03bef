#!/usr/bin/env python3
"""Benchmark of the cascaded-reduction hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic
input: every entry point of the library on its benchmark workload
  w0  rf_cascade_attention         fp32  Q[128,64] K,V[512,64]
  w1  rf_safe_softmax              bf16  X[32768,4096]
  w2  rf_cascade_attention         bf16  B4 H32 L2048 d128, non-causal and causal
  w3  rf_cascade_attention_splitk + rf_merge_states   bf16 B16 Hq32 Hkv8 Lk32768 d128, S=64
  w4  rf_rmsnorm_gemm              bf16  4096 x 4096 x 4096
After the timed steps the paper's further cascades are timed one kernel at a time
(``further_cascades``; they are not part of a step):
  x0  rf_cascade_attention         fp32  workload 0's shape batched over 16 x 32 heads (labelled extension)
  x1  rf_variance                  f32   X[1024,32768]
  x2  rf_moe_routing               bf16  tokens 2048; hd 8192 x 64 experts, hd 4096 x 128 experts; top 8
  x3  rf_fp8_quant_gemm            bf16 tokens x FP8 weights  4096 x 3584 x 8192 and 4096 x 8192 x 3584
Inputs are generated on the device from fixed seeds before the timed region.
The memory-bound workloads (w1, w3) rotate over three buffer sets so that the
last-level cache cannot serve repeated reads.

Prints ONE JSON line.  ``value`` is the fused-attention throughput of the
prefill workload (non-causal), from the HIP-event time of that kernel inside
the timed region, and ``roofline`` describes that same kernel; ``workloads``
and ``rooflines`` carry every workload's time, throughput and roofline
fraction; ``cpu_baseline`` times the fp64 oracle on a bounded sample of the
prefill workload on the host cores and ``cpu_baselines`` does the same for each
of the five workloads (seconds and the workload's own unit); ``device`` holds
the compute-unit count and clock the box reports.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0      # dense bf16 MFMA, published
PEAK_F32_TFLOPS = 157.3        # fp32 matrix / vector, published
N_ROT = 3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--only", type=str, default="",
                    help="comma list of w0..w4 and x1.. (profiling aid); default all")
    ap.add_argument("--settle-ms", type=float, default=250.0,
                    help="untimed run-in before the warmup steps: a launch takes up to 35 %% longer during the "
                         "first ~100 ms of load on an idle GPU than in the steady state (clock / power management)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay leg")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch one plain 256 MiB -> 256 MiB copy kernel before the warmup "
                         "(reference dispatch for scaling the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2603_10026_amd import binding as rf
    from paper_2603_10026_amd import inputs as I

    rf.load_library()                      # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    only = set(args.only.split(",")) if args.only else {"w0", "w1", "w2", "w3", "w4", "x0", "x1", "x2", "x3"}
    W = I.WORKLOADS
    seed = lambda i: I.SEED_BASE + i

    # ---------------------------------------------------------------- inputs
    state = {}
    if "w0" in only:
        c = W[0]
        q, k, v = I.attention_inputs_device(seed(0), c["B"], c["Hq"], c["Hkv"], c["Lq"], c["Lk"], c["d"], "f32", dev)
        state["w0"] = dict(q=q, k=k, v=v, o=torch.empty_like(q), scale=I.default_scale(c["d"]))
    if "w1" in only:
        c = W[1]
        xs = [I.softmax_inputs_device(seed(1) + 100 * r, c["rows"], c["n"], c["sigma"], "bf16", dev) for r in range(N_ROT)]
        state["w1"] = dict(x=xs, y=[torch.empty_like(x) for x in xs])
    if "w2" in only:
        c = W[2]
        q, k, v = I.attention_inputs_device(seed(2), c["B"], c["Hq"], c["Hkv"], c["Lq"], c["Lk"], c["d"], "bf16", dev)
        state["w2"] = dict(q=q, k=k, v=v, o=torch.empty_like(q), oc=torch.empty_like(q), scale=I.default_scale(c["d"]))
    if "w3" in only:
        c = W[3]
        sets = []
        for r in range(N_ROT):
            q, k, v = I.attention_inputs_device(seed(3) + 100 * r, c["B"], c["Hq"], c["Hkv"], c["Lq"], c["Lk"], c["d"], "bf16", dev)
            pm, pl, pacc = rf.alloc_partial_states(q, c["num_splits"])
            sets.append(dict(q=q, k=k, v=v, pm=pm, pl=pl, pacc=pacc, o=torch.empty_like(q)))
        state["w3"] = dict(sets=sets, scale=I.default_scale(c["d"]), S=c["num_splits"])
    if "w4" in only:
        c = W[4]
        x, g, w = I.rmsnorm_gemm_inputs_device(seed(4), c["M"], c["K"], c["N"], c["w_sigma"], "bf16", dev)
        state["w4"] = dict(x=x, g=g, w=w, y=torch.empty((c["M"], c["N"]), dtype=torch.bfloat16, device=dev), eps=c["eps"])
    torch.cuda.synchronize()

    # kernels of one step, in launch order: (label, callable(step_index))
    launches = []
    if "w0" in only:
        s0 = state["w0"]
        launches.append(("w0_attention_f32", lambda i: rf.rf_cascade_attention(s0["q"], s0["k"], s0["v"], s0["scale"], False, o=s0["o"])))
    if "w1" in only:
        s1 = state["w1"]
        launches.append(("w1_softmax", lambda i: rf.rf_safe_softmax(s1["x"][i % N_ROT], s1["y"][i % N_ROT])))
    if "w2" in only:
        s2 = state["w2"]
        launches.append(("w2_attention_prefill", lambda i: rf.rf_cascade_attention(s2["q"], s2["k"], s2["v"], s2["scale"], False, o=s2["o"])))
        launches.append(("w2_attention_prefill_causal", lambda i: rf.rf_cascade_attention(s2["q"], s2["k"], s2["v"], s2["scale"], True, o=s2["oc"])))
    if "w3" in only:
        s3 = state["w3"]

        def splitk(i):
            t = s3["sets"][i % N_ROT]
            rf.rf_cascade_attention_splitk(t["q"], t["k"], t["v"], s3["S"], t["pm"], t["pl"], t["pacc"], s3["scale"], False)

        def merge(i):
            t = s3["sets"][i % N_ROT]
            rf.rf_merge_states(t["pm"], t["pl"], t["pacc"], t["o"])

        launches.append(("w3_decode_splitk", splitk))
        launches.append(("w3_decode_merge", merge))
    if "w4" in only:
        s4 = state["w4"]
        launches.append(("w4_rmsnorm_gemm", lambda i: rf.rf_rmsnorm_gemm(s4["x"], s4["g"], s4["w"], s4["eps"], y=s4["y"])))

    def run_step(i, events=None):
        for j, (_, fn) in enumerate(launches):
            if events is not None:
                events[j][0].record()
            fn(i)
            if events is not None:
                events[j][1].record()

    if args.calib_copy:
        # plain copy kernel of known size: reads 256 MiB, writes 256 MiB
        src = torch.ones(1 << 26, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # Run-in.  On an idle GPU the first launches run at boost clocks, the next ones up to 35 %
    # slower, and the steady state is only reached after ~100 launches (prefill: 285, 350, then
    # 260 us per launch, one softmax pass between launches): whole steps are run, untimed, until
    # that transient is over, then the W warmup steps, then the K timed ones.
    def settle(fn, ms):
        if ms <= 0:
            return 0
        t_end = time.perf_counter() + ms * 1e-3
        done = 0
        while time.perf_counter() < t_end:
            fn(done)
            done += 1
            if done % 4 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        return done

    settle_steps = settle(run_step, args.settle_ms) if launches else 0
    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()

    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in launches]
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_step(args.warmup + i, ev[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # The same steps captured once in a HIP graph and replayed: what a serving loop that cannot
    # afford per-launch host work would run.  Reported next to, never instead of, ms_per_step.
    graph_replay = None
    if not args.no_graph and launches:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            run_step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            for i in range(N_ROT):
                run_step(i)
        graph.replay()
        torch.cuda.synchronize()
        reps = max(1, args.steps // N_ROT)
        g0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        graph_replay = dict(ms_per_step=round((g1 - g0) * 1e3 / (reps * N_ROT), 4), steps_per_graph=N_ROT, replays=reps)
        del graph

    # average kernel duration per launch over the timed region (HIP events on the launch stream)
    dur_us = {}
    for j, (label, _) in enumerate(launches):
        ts = [ev[i][j][0].elapsed_time(ev[i][j][1]) * 1e3 for i in range(args.steps)]
        dur_us[label] = dict(avg=float(np.mean(ts)), med=float(np.median(ts)), min=float(np.min(ts)))

    # ---------------------------------------------- algorithmic work per launch
    def attn_flops(c, causal):
        pairs = c["Lq"] * (c["Lq"] + 1) // 2 if causal else c["Lq"] * c["Lk"]
        return 4.0 * c["B"] * c["Hq"] * pairs * c["d"]

    work = {}
    c = W[0]
    work["w0_attention_f32"] = dict(bound="latency", flops=attn_flops(c, False),
                                    bytes=4.0 * (2 * c["Lq"] * c["d"] + 2 * c["Lk"] * c["d"]))
    c = W[1]
    work["w1_softmax"] = dict(bound="hbm", bytes=2.0 * c["rows"] * c["n"] * 2)
    c = W[2]
    work["w2_attention_prefill"] = dict(bound="mfma", flops=attn_flops(c, False))
    work["w2_attention_prefill_causal"] = dict(bound="mfma", flops=attn_flops(c, True))
    c = W[3]
    kv_bytes = 2.0 * c["B"] * c["Hkv"] * c["Lk"] * c["d"] * 2
    part_bytes = 1.0 * c["B"] * c["Hq"] * c["Lq"] * c["num_splits"] * (c["d"] + 2) * 4
    qo_bytes = 2.0 * c["B"] * c["Hq"] * c["Lq"] * c["d"] * 2
    work["w3_decode_splitk"] = dict(bound="hbm", bytes=kv_bytes + part_bytes + qo_bytes / 2)
    work["w3_decode_merge"] = dict(bound="hbm", bytes=part_bytes + qo_bytes / 2)
    c = W[4]
    work["w4_rmsnorm_gemm"] = dict(bound="mfma", flops=2.0 * c["M"] * c["K"] * c["N"],
                                   bytes=2.0 * (c["M"] * c["K"] + c["K"] * c["N"] + c["M"] * c["N"] + c["K"]))

    # HBM-side traffic per launch, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and
    # scaled by a plain copy kernel (recorded in profiles/).  The record names the kernel sources
    # it was measured on (a digest of csrc/); if they have changed since, no traffic is reported
    # rather than a stale figure.
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2603_10026_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    kernel_sources = h.hexdigest()[:16]
    traffic, traffic_sources = {}, None
    tpath = os.path.join(ROOT, "profiles", "bench_all_workloads_hbm_traffic.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            f = line.split()
            if len(f) == 4 and f[0] == "TRAFFIC":
                traffic[f[1]] = float(f[2]) + float(f[3])
            if len(f) == 2 and f[0] == "SOURCES":
                traffic_sources = f[1]
    traffic_current = traffic_sources == kernel_sources
    if not traffic_current:
        traffic = {}

    workloads = {}
    rooflines = []
    for label, _ in launches:
        wk, d = work[label], dur_us[label]
        sec = d["avg"] * 1e-6
        entry = dict(us_avg=round(d["avg"], 2), us_med=round(d["med"], 2), us_min=round(d["min"], 2), bound=wk["bound"])
        if wk["bound"] == "hbm":
            ach = wk["bytes"] / sec / 1e9
            entry.update(GBps=round(ach, 1), frac=round(ach / PEAK_HBM_GBS, 4), algorithmic_bytes=wk["bytes"])
            rooflines.append(dict(kernel=label, bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                                  frac=round(ach / PEAK_HBM_GBS, 4), traffic=traffic.get(label), us=round(d["avg"], 2)))
        elif wk["bound"] == "mfma":
            ach = wk["flops"] / sec / 1e12
            entry.update(TFLOPs=round(ach, 1), frac=round(ach / PEAK_BF16_TFLOPS, 4), algorithmic_flops=wk["flops"])
            rooflines.append(dict(kernel=label, bound="mfma", achieved=round(ach, 1), peak=PEAK_BF16_TFLOPS,
                                  unit="TFLOP/s", frac=round(ach / PEAK_BF16_TFLOPS, 4), traffic=traffic.get(label),
                                  us=round(d["avg"], 2)))
        else:
            entry.update(TFLOPs=round(wk["flops"] / sec / 1e12, 3), note="launch-latency bound; time is the figure of merit")
        workloads[label] = entry
    # decode = split kernel + merge kernel together
    if "w3" in only:
        tot = (dur_us["w3_decode_splitk"]["avg"] + dur_us["w3_decode_merge"]["avg"]) * 1e-6
        b = work["w3_decode_splitk"]["bytes"] + work["w3_decode_merge"]["bytes"]
        workloads["w3_decode_total"] = dict(us_avg=round(tot * 1e6, 2), GBps=round(b / tot / 1e9, 1),
                                            frac=round(b / tot / 1e9 / PEAK_HBM_GBS, 4), bound="hbm", algorithmic_bytes=b)

    headline = next((r for r in rooflines if r["kernel"] == "w2_attention_prefill"), None)

    # ------------------------------------------------ further cascades of the paper
    # Timed after the step loop, each kernel alone: `steps` launches bracketed by HIP
    # events one by one, inputs rotating over N_ROT buffer sets.
    def time_launches(fn, n, warm):
        settle(fn, min(args.settle_ms, 60.0))   # (the GPU has idled while the inputs were made)
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        # A kernel of ~20 us ends before the host has issued the next launch and its two event
        # records; on an empty queue the first event of a pair is then stamped before the kernel
        # has been submitted and the pair times the host.  A lead of untimed launches goes first,
        # with no synchronisation after it, so that the timed launches are queued behind GPU work
        # and each pair spans one kernel as the GPU runs it.
        # The average is taken over the n launches between ONE pair of events (the two event
        # markers between consecutive kernels of the per-launch pairs cost about 2 us a launch,
        # which is not kernel time); the per-launch pairs that follow give the median and minimum.
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(64 + 2 * n):
            fn(i)
        g0.record()
        for i in range(n):
            fn(warm + i)
        g1.record()
        for i in range(n):
            evs[i][0].record()
            fn(warm + i)
            evs[i][1].record()
        torch.cuda.synchronize()
        ts = [a.elapsed_time(b) * 1e3 for a, b in evs]
        return dict(avg=g0.elapsed_time(g1) * 1e3 / n, med=float(np.median(ts)), min=float(np.min(ts)),
                    avg_pairs=float(np.mean(ts)))

    further = {}
    if "x0" in only:
        # labelled extension of workload 0: the same fp32 shape batched over 512 heads, so that
        # an fp32 TFLOP/s figure means something (one head alone is a launch-latency measurement)
        c = W[0]
        nb, nh = 16, 32
        qb, kb_, vb_ = I.attention_inputs_device(seed(0) + 50, nb, nh, nh, c["Lq"], c["Lk"], c["d"], "f32", dev)
        ob = torch.empty_like(qb)
        d = time_launches(lambda i: rf.rf_cascade_attention(qb, kb_, vb_, I.default_scale(c["d"]), False, o=ob),
                          args.steps, args.warmup)
        fl = 4.0 * nb * nh * c["Lq"] * c["Lk"] * c["d"]
        ach = fl / (d["avg"] * 1e-6) / 1e12
        further["x0_attention_f32_batched"] = dict(workload=f"attn_fp32_B{nb}_H{nh}_Lq{c['Lq']}_Lk{c['Lk']}_d{c['d']}",
                                                   us_avg=round(d["avg"], 2), us_med=round(d["med"], 2), us_avg_pairs=round(d["avg_pairs"], 2), us_min=round(d["min"], 2),
                                                   bound="mfma", TFLOPs=round(ach, 2), frac=round(ach / PEAK_F32_TFLOPS, 4),
                                                   algorithmic_flops=fl,
                                                   note="fraction of the published fp32 matrix peak (157.3 TFLOP/s); extension of workload 0, not one of the five configurations")
        rooflines.append(dict(kernel="x0_attention_f32_batched", bound="mfma", achieved=round(ach, 2), peak=PEAK_F32_TFLOPS,
                              unit="TFLOP/s", frac=round(ach / PEAK_F32_TFLOPS, 4), traffic=traffic.get("x0_attention_f32_batched"),
                              us=round(d["avg"], 2)))
        del qb, kb_, vb_, ob
    if "x1" in only:
        c = I.EXTRA_WORKLOADS["variance_v8"]
        xs = [I.variance_inputs_device(seed(6) + 100 * r, c["bs"], c["l"], c["dtype"], c["mu"], c["sigma"], dev)
              for r in range(N_ROT)]
        mv = [(torch.empty(c["bs"], dtype=torch.float32, device=dev), torch.empty(c["bs"], dtype=torch.float32, device=dev))
              for _ in range(N_ROT)]
        d = time_launches(lambda i: rf.rf_variance(xs[i % N_ROT], *mv[i % N_ROT]), args.steps, args.warmup)
        b = 4.0 * c["bs"] * c["l"] + 8.0 * c["bs"]
        ach = b / (d["avg"] * 1e-6) / 1e9
        further["x1_variance"] = dict(workload=c["name"], us_avg=round(d["avg"], 2), us_med=round(d["med"], 2), us_avg_pairs=round(d["avg_pairs"], 2),
                                      us_min=round(d["min"], 2), bound="hbm", GBps=round(ach, 1),
                                      frac=round(ach / PEAK_HBM_GBS, 4), algorithmic_bytes=b)
        rooflines.append(dict(kernel="x1_variance", bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                              frac=round(ach / PEAK_HBM_GBS, 4), traffic=traffic.get("x1_variance"), us=round(d["avg"], 2)))
        del xs, mv
    if "x2" in only:
        for key in ("moe_routing_r5", "moe_routing_r8"):
            c = I.EXTRA_WORKLOADS[key]
            sets = []
            for r in range(N_ROT):
                xx, ww = I.moe_routing_inputs_device(seed(5) + 100 * r, c["S"], c["hd"], c["E"], c["score_sigma"], "bf16", dev)
                sets.append(dict(x=xx, w=ww, p=torch.empty((c["S"], c["topk"]), dtype=torch.float32, device=dev),
                                 i=torch.empty((c["S"], c["topk"]), dtype=torch.int32, device=dev)))
            ws = torch.empty(rf.moe_routing_workspace_bytes(c["S"], c["hd"], c["E"]), dtype=torch.uint8, device=dev)

            def route(i, sets=sets, ws=ws, c=c):
                t = sets[i % N_ROT]
                rf.rf_moe_routing(t["x"], t["w"], c["topk"], prob=t["p"], idx=t["i"], workspace=ws)

            d = time_launches(route, args.steps, args.warmup)
            # algorithmic bytes: tokens and router weights read once, results written once
            b = 2.0 * c["S"] * c["hd"] + 2.0 * c["hd"] * c["E"] + 8.0 * c["S"] * c["topk"]
            ach = b / (d["avg"] * 1e-6) / 1e9
            label = "x2_" + key
            further[label] = dict(workload=c["name"], us_avg=round(d["avg"], 2), us_med=round(d["med"], 2), us_avg_pairs=round(d["avg_pairs"], 2),
                                  us_min=round(d["min"], 2), bound="hbm", GBps=round(ach, 1),
                                  frac=round(ach / PEAK_HBM_GBS, 4), algorithmic_bytes=b,
                                  workspace_bytes=ws.numel(),
                                  note="two launches (scores, cascade) timed together; latency-bound at this size")
            rooflines.append(dict(kernel=label, bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                                  frac=round(ach / PEAK_HBM_GBS, 4), traffic=traffic.get(label), us=round(d["avg"], 2)))
            del sets, ws
    if "x3" in only:
        PEAK_FP8_TFLOPS = 5000.0      # dense fp8 MFMA, published
        for key in ("fp8_quant_gemm_q3", "fp8_quant_gemm_q4"):
            c = I.EXTRA_WORKLOADS[key]
            aa, ww = I.fp8_quant_gemm_inputs_device(seed(7), c["M"], c["K"], c["N"], dev)
            cc = torch.empty((c["M"], c["N"]), dtype=torch.bfloat16, device=dev)
            d = time_launches(lambda i, aa=aa, ww=ww, cc=cc: rf.rf_fp8_quant_gemm(aa, ww, c=cc), args.steps, args.warmup)
            fl = 2.0 * c["M"] * c["K"] * c["N"]
            ach = fl / (d["avg"] * 1e-6) / 1e12
            label = "x3_" + key
            further[label] = dict(workload=c["name"], us_avg=round(d["avg"], 2), us_med=round(d["med"], 2), us_avg_pairs=round(d["avg_pairs"], 2),
                                  us_min=round(d["min"], 2), bound="mfma", TFLOPs=round(ach, 1),
                                  frac=round(ach / PEAK_FP8_TFLOPS, 4), algorithmic_flops=fl,
                                  note="fraction of the published dense fp8 peak (5 PFLOP/s)")
            rooflines.append(dict(kernel=label, bound="mfma", achieved=round(ach, 1), peak=PEAK_FP8_TFLOPS,
                                  unit="TFLOP/s", frac=round(ach / PEAK_FP8_TFLOPS, 4), traffic=traffic.get(label),
                                  us=round(d["avg"], 2)))
            del aa, ww, cc

    # -------------------------------------------- measured ceilings (context, not the peaks)
    def timed(fn, n):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn(0)
        torch.cuda.synchronize()
        a.record()
        for i in range(n):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / n

    nbytes = 256 << 20
    srcs = [torch.ones(nbytes // 4, dtype=torch.float32, device=dev) for _ in range(N_ROT)]
    dsts = [torch.empty_like(t) for t in srcs]
    t_copy = timed(lambda i: rf.rf_diag_copy(srcs[i % N_ROT], dsts[i % N_ROT]), 12)
    del srcs, dsts
    rbytes = 1 << 30
    rsrc = [torch.ones(rbytes // 4, dtype=torch.float32, device=dev) for _ in range(2)]
    rsink = torch.empty(rf.DIAG_READ_SINK_BYTES // 4, dtype=torch.int32, device=dev)
    t_read = timed(lambda i: rf.rf_diag_read(rsrc[i % 2], rsink), 8)
    del rsrc, rsink
    sink = torch.empty(512 * 256, dtype=torch.float32, device=dev)
    fl = 512 * 4 * 300 * 32 * 32768.0
    t_rand = timed(lambda i: rf.rf_diag_mfma(sink, 512, 300, True), 5)
    t_const = timed(lambda i: rf.rf_diag_mfma(sink, 512, 300, False), 5)
    ceilings = dict(hbm_copy_GBps=round(2 * nbytes / t_copy / 1e9, 1),
                    hbm_read_only_GBps=round(rbytes / t_read / 1e9, 1),
                    mfma_bf16_random_operands_TFLOPs=round(fl / t_rand / 1e12, 1),
                    mfma_bf16_constant_operands_TFLOPs=round(fl / t_const / 1e12, 1),
                    note="plain 256 MiB copy kernel and 1 GiB read-only kernel (non-temporal accesses); MFMA-only 32x32x16 bf16 loop, 512 workgroups x 4 wavefronts")
    for r in rooflines:
        if r["bound"] == "mfma" and r["peak"] != PEAK_BF16_TFLOPS:
            continue            # no measured ceiling for the fp8 and fp32 matrix pipes
        if r["bound"] == "hbm":
            # kernels that almost only read are put next to the read-only ceiling, the softmax
            # (as many bytes written as read) next to the copy ceiling
            ceil = ceilings["hbm_copy_GBps"] if r["kernel"] == "w1_softmax" else ceilings["hbm_read_only_GBps"]
        else:
            ceil = ceilings["mfma_bf16_random_operands_TFLOPs"]
        r["frac_of_measured_ceiling"] = round(r["achieved"] / ceil, 4)

    # ------------------------------------------------------------ cpu baseline
    # The fp64 oracle as it stands, on the host cores of this machine, on a bounded sample of each
    # workload (about ten seconds in all; the prefill workloads are small enough to run whole),
    # next to the GPU result for the same sample.
    cpu, cpus = None, {}
    if not args.no_cpu_baseline:
        from oracle import rf_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1

        def rel_err(got, ref):
            return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) / np.max(np.abs(ref)))

        if "w0" in only:
            c, s0 = W[0], state["w0"]
            qh, kh, vh = (I.to_numpy(t) for t in (s0["q"], s0["k"], s0["v"]))
            tc0 = time.perf_counter(); ref = O.attention(qh, kh, vh, s0["scale"], False); tc1 = time.perf_counter()
            cpus["w0_attention_f32"] = dict(seconds=round(tc1 - tc0, 4), value=round(attn_flops(c, False) / (tc1 - tc0) / 1e12, 6),
                                            unit="TFLOP/s", sample="the whole workload",
                                            gpu_vs_oracle_max_err_over_max_ref=rel_err(I.to_numpy(s0["o"]), ref))
        if "w1" in only:
            c, s1 = W[1], state["w1"]
            nrows = c["rows"]
            last = (args.warmup + args.steps - 1) % N_ROT          # the buffer set of the last step
            xh = I.to_numpy(s1["x"][last][:nrows])
            tc0 = time.perf_counter(); ref = O.safe_softmax(xh); tc1 = time.perf_counter()
            cpus["w1_softmax"] = dict(seconds=round(tc1 - tc0, 4), value=round(2.0 * nrows * c["n"] * 2 / (tc1 - tc0) / 1e9, 3),
                                      unit="GB/s", sample=f"{nrows} of {c['rows']} rows",
                                      gpu_vs_oracle_max_err_over_max_ref=rel_err(I.to_numpy(s1["y"][last][:nrows]), ref))
        if "w2" in only:
            c, s2 = W[2], state["w2"]
            nb, nh = c["B"], c["Hq"]                # every (batch, head) pair: a few seconds on the host cores
            qh, kh, vh = (I.to_numpy(t[:nb]) for t in (s2["q"], s2["k"], s2["v"]))
            tc0 = time.perf_counter(); ref = O.attention(qh, kh, vh, s2["scale"], False); tc1 = time.perf_counter()
            fl = 4.0 * nb * nh * c["Lq"] * c["Lk"] * c["d"]
            err = rel_err(I.to_numpy(s2["o"][:nb]), ref)
            cpu = dict(value=round(fl / (tc1 - tc0) / 1e12, 5), unit="TFLOP/s", cores=int(cores), kind="oracle",
                       sample=f"{nb * nh} of {c['B'] * c['Hq']} (batch, head) pairs of the non-causal prefill workload, "
                              f"fp64 numpy oracle, {tc1 - tc0:.1f} s wall",
                       gpu_vs_oracle_max_err_over_max_ref=err)
            cpus["w2_attention_prefill"] = dict(seconds=round(tc1 - tc0, 4), value=cpu["value"], unit="TFLOP/s",
                                                sample=f"{nb * nh} of {c['B'] * c['Hq']} (batch, head) pairs",
                                                gpu_vs_oracle_max_err_over_max_ref=err)
            nbc = c["B"]
            tc0 = time.perf_counter(); ref = O.attention(qh[:nbc], kh[:nbc], vh[:nbc], s2["scale"], True); tc1 = time.perf_counter()
            flc = 4.0 * nbc * nh * (c["Lq"] * (c["Lq"] + 1) // 2) * c["d"]
            cpus["w2_attention_prefill_causal"] = dict(seconds=round(tc1 - tc0, 4), value=round(flc / (tc1 - tc0) / 1e12, 5),
                                                       unit="TFLOP/s (visible pairs only)",
                                                       sample=f"{nbc * nh} of {c['B'] * c['Hq']} (batch, head) pairs",
                                                       gpu_vs_oracle_max_err_over_max_ref=rel_err(I.to_numpy(s2["oc"][:nbc]), ref))
            del qh, kh, vh, ref
        if "w3" in only:
            c, s3 = W[3], state["w3"]
            t = s3["sets"][(args.warmup + args.steps - 1) % N_ROT]
            grp = c["Hq"] // c["Hkv"]
            pairs = [(b_, h_) for b_ in range(0, c["B"], 2) for h_ in range(0, c["Hkv"], 2)]
            secs, worst = 0.0, 0.0
            for (b, hk) in pairs:
                kh, vh = (I.to_numpy(x[b, hk])[None, None] for x in (t["k"], t["v"]))
                qh = I.to_numpy(t["q"][b, hk * grp:(hk + 1) * grp])[None]
                tc0 = time.perf_counter(); ref = O.attention(qh, kh, vh, s3["scale"], False); tc1 = time.perf_counter()
                secs += tc1 - tc0
                worst = max(worst, rel_err(I.to_numpy(t["o"][b, hk * grp:(hk + 1) * grp])[None], ref))
            by = len(pairs) * 2.0 * c["Lk"] * c["d"] * 2
            cpus["w3_decode_total"] = dict(seconds=round(secs, 4), value=round(by / secs / 1e9, 3), unit="GB/s",
                                           sample=f"{len(pairs)} of {c['B'] * c['Hkv']} (batch, KV head) pairs, 4 query heads each, whole key axis",
                                           gpu_vs_oracle_max_err_over_max_ref=worst)
        if "w4" in only:
            c, s4 = W[4], state["w4"]
            nrows = c["M"]
            xh, gh, wh = I.to_numpy(s4["x"][:nrows]), I.to_numpy(s4["g"]), I.to_numpy(s4["w"])
            tc0 = time.perf_counter(); ref = O.rmsnorm_gemm(xh, gh, wh, s4["eps"]); tc1 = time.perf_counter()
            cpus["w4_rmsnorm_gemm"] = dict(seconds=round(tc1 - tc0, 4), value=round(2.0 * nrows * c["K"] * c["N"] / (tc1 - tc0) / 1e12, 5),
                                           unit="TFLOP/s", sample=f"{nrows} of {c['M']} rows",
                                           gpu_vs_oracle_max_err_over_max_ref=rel_err(I.to_numpy(s4["y"][:nrows]), ref))
        for v_ in cpus.values():
            v_.update(cores=int(cores), kind="oracle")

    props = torch.cuda.get_device_properties(0)
    device = dict(name=props.name, compute_units=int(props.multi_processor_count), max_clock_mhz=None,
                  hbm_bytes=int(props.total_memory), arch=getattr(props, "gcnArchName", None))
    try:        # the GPU agent's own report of its clock and compute units (a child process; nothing is re-executed)
        import subprocess
        txt = subprocess.run(["/opt/rocm/bin/rocminfo"], capture_output=True, text=True, timeout=30).stdout
        agent = txt[txt.index("gfx950"):]
        for line in agent.splitlines():
            if "Max Clock Freq. (MHz)" in line and device["max_clock_mhz"] is None:
                device["max_clock_mhz"] = float(line.split(":")[1])
            if line.strip().startswith("Compute Unit:") and "rocminfo_compute_units" not in device:
                device["rocminfo_compute_units"] = int(line.split(":")[1])
    except Exception:
        pass

    primary = workloads.get("w2_attention_prefill")
    out = {
        "metric": "fused-attention TFLOP/s (bf16 prefill, non-causal); softmax/decode GB/s and % of roofline per workload in `workloads`",
        "value": primary["TFLOPs"] if primary else None,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "run_in": {"ms": args.settle_ms, "steps": settle_steps,
                   "note": "untimed whole steps before the warmup steps, until the clock / power transient of an idle GPU is over"},
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "attn_prefill_bf16_B4_H32_L2048_d128_noncausal (value); one step = all five workloads: "
                               "attn_f32_128x512x64, softmax_bf16_32768x4096, prefill non-causal + causal, "
                               "decode_gqa_B16_Hq32_Hkv8_Lk32768_S64 split+merge, rmsnorm_gemm_4096^3",
                   "seeds": [I.SEED_BASE + i for i in range(5)]},
        "workloads": workloads,
        "further_cascades": further,
        # the kernel `value` describes; every other kernel under `rooflines`
        "roofline": {k: headline[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")} | {"kernel": headline["kernel"]} if headline else None,
        "rooflines": rooflines,
        "targets": {"hbm_frac": 0.70, "mfma_frac": 0.50,
                    "met": {r["kernel"]: bool(r["frac"] >= (0.70 if r["bound"] == "hbm" else 0.50)) for r in rooflines}},
        "traffic_record": {"file": "profiles/bench_all_workloads_hbm_traffic.txt", "measured_on_sources": traffic_sources,
                           "current_sources": kernel_sources, "used": bool(traffic_current)},
        "ceilings": ceilings,
        "graph_replay": graph_replay,
        "device": device,
        "cpu_baseline": cpu,
        "cpu_baselines": cpus,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()

"""Two sweeps that reproduce the paper's ablations on this GPU.

``--what splits`` (default): split-count sweep for multi-segment attention (the effect of the
number of segments on a long-sequence decode).  Times rf_cascade_attention_splitk +
rf_merge_states on the decode benchmark workload for several segment counts S and prints one
line per S; the fastest S is the value to pass as ``num_splits`` on this GPU.

``--what fusion``: the safe-softmax cascade fused at different levels (not fused / per lane /
per wavefront / per workgroup / across workgroups) for row lengths 1K..8K, 32768 rows of bf16, through
rf_diag_softmax_level.

``--what tables``: the fp32 attention workload and every shape of the paper's appendix tables for
the further cascades (MoE routing R1-R8, FP8 quant + GEMM Q1-Q10, variance V1-V8), one JSON line
each: the time of one call through the Python binding, and the time per call when 24 calls are
captured in a HIP graph and replayed (the host side of a launch is then out of the number).

``--what tilings``: the unmasked prefill cascade (head dimension 128) with 32 query rows per
wavefront and two wavefronts per SIMD (rf_cascade_attention) against 64 rows per wavefront and
one wavefront per SIMD (rf_diag_attention_wide), for several key lengths; the per-key-tile slope
and the fixed cost of a launch follow from the lines.

``--what eager``: the measure the paper's appendix uses for AMD hardware, speed-up over the plain
PyTorch operator chain on the same GPU, for the five benchmark workloads and the largest shapes of
the further cascades: the library's call and the PyTorch chain a user would write for the same
result (matmul -> softmax -> topk; var_mean; abs-max, scale, cast, scaled matmul; softmax;
scaled_dot_product_attention; rms_norm -> matmul), 24 calls captured in a HIP graph and replayed,
so that neither side pays the host for its launches.  Context only: PyTorch's kernels are a
library of their own, not part of this package, and nothing here calls them outside this sweep.

    python -m paper_2603_10026_amd.sweep [--what splits|fusion|tables|tilings|eager] [--splits 8,16,...] [--iters 20]
"""
import argparse
import json
import sys
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--splits", type=str, default="8,16,32,64,128,256,512")
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--what", type=str, default="splits", choices=["splits", "fusion", "tables", "tilings", "eager"])
    args = ap.parse_args()
    if args.what == "fusion":
        return fusion_sweep(args.iters)
    if args.what == "tables":
        return tables_sweep(args.iters)
    if args.what == "tilings":
        return tilings_sweep(args.iters)
    if args.what == "eager":
        return eager_sweep()
    import torch
    from . import binding as rf
    from . import inputs as I

    rf.load_library()
    dev = "cuda:0"
    c = I.WORKLOADS[3]
    n_rot = 3
    sets = [I.attention_inputs_device(I.SEED_BASE + 3 + 100 * r, c["B"], c["Hq"], c["Hkv"], c["Lq"], c["Lk"], c["d"], "bf16", dev)
            for r in range(n_rot)]
    scale = I.default_scale(c["d"])
    kv_bytes = 2.0 * c["B"] * c["Hkv"] * c["Lk"] * c["d"] * 2
    rows = []
    for S in [int(t) for t in args.splits.split(",")]:
        parts = [rf.alloc_partial_states(sets[r][0], S) for r in range(n_rot)]
        outs = [torch.empty_like(sets[r][0]) for r in range(n_rot)]

        def step(i):
            q, k, v = sets[i % n_rot]
            pm, pl, pacc = parts[i % n_rot]
            rf.rf_cascade_attention_splitk(q, k, v, S, pm, pl, pacc, scale, False)
            rf.rf_merge_states(pm, pl, pacc, outs[i % n_rot])

        for i in range(3):
            step(i)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.iters)]
        for i in range(args.iters):
            evs[i][0].record()
            step(i)
            evs[i][1].record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        med = ts[len(ts) // 2]
        part_bytes = 2.0 * c["B"] * c["Hq"] * S * (c["d"] + 2) * 4      # written, then read
        row = dict(num_splits=S, keys_per_segment=-(-c["Lk"] // S), workgroups=c["B"] * c["Hkv"] * S,
                   us_median=round(med, 1), us_min=round(ts[0], 1),
                   GBps_kv_only=round(kv_bytes / med / 1e3, 1), partial_state_MB=round(part_bytes / 1e6, 1))
        rows.append(row)
        print(json.dumps(row), flush=True)
        del parts, outs
    best = min(rows, key=lambda r: r["us_median"])
    print(json.dumps(dict(best_num_splits=best["num_splits"], us_median=best["us_median"])), flush=True)


def tilings_sweep(iters):
    import torch
    from . import binding as rf
    from . import inputs as I

    rf.load_library()
    dev = "cuda:0"
    c = I.WORKLOADS[2]
    scale = I.default_scale(c["d"])
    for Lk in (512, 1024, 2048, 4096, 8192):
        q, k, v = I.attention_inputs_device(I.SEED_BASE + 2, c["B"], c["Hq"], c["Hkv"], c["Lq"], Lk, c["d"], "bf16", dev)
        o = torch.empty_like(q)
        flops = 4.0 * c["B"] * c["Hq"] * c["Lq"] * Lk * c["d"]
        row = dict(workload=f"attn_prefill_bf16_B{c['B']}_H{c['Hq']}_Lq{c['Lq']}_Lk{Lk}_d{c['d']}_noncausal")
        for name, fn in (("rows32_two_wavefronts_per_simd", lambda: rf.rf_cascade_attention(q, k, v, scale, causal=False, o=o)),
                         ("rows64_one_wavefront_per_simd", lambda: rf.rf_diag_attention_wide(q, k, v, scale, o=o))):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
            for i in range(iters):
                evs[i][0].record()
                fn()
                evs[i][1].record()
            torch.cuda.synchronize()
            ts = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
            med = ts[len(ts) // 2]
            row[name] = dict(us_median=round(med, 1), TFLOPs=round(flops / med / 1e6, 1))
        print(json.dumps(row), flush=True)
        del q, k, v, o
    return 0


def fusion_sweep(iters):
    import torch
    from . import binding as rf
    from . import inputs as I

    rf.load_library()
    dev = "cuda:0"
    rows, n_rot = 32768, 3
    names = {0: "not fused (3 kernels)", 1: "fused per lane", 2: "fused per wavefront", 3: "fused per workgroup",
             4: "fused across workgroups (2 kernels)"}
    for n in (1024, 2048, 4096, 8192):
        xs = [I.softmax_inputs_device(I.SEED_BASE + 1 + 100 * r, rows, n, 2.0, "bf16", dev) for r in range(n_rot)]
        ys = [torch.empty_like(x) for x in xs]
        ml = torch.empty(8 * rows, dtype=torch.float32, device=dev)
        base = None
        for level in (0, 1, 2, 3, 4):
            for i in range(3):
                rf.rf_diag_softmax_level(xs[i % n_rot], ys[i % n_rot], level, ml)
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
            for i in range(iters):
                evs[i][0].record()
                rf.rf_diag_softmax_level(xs[i % n_rot], ys[i % n_rot], level, ml)
                evs[i][1].record()
            torch.cuda.synchronize()
            ts = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
            med = ts[len(ts) // 2]
            base = med if level == 0 else base
            print(json.dumps(dict(n=n, level=level, fusion=names[level], us_median=round(med, 1),
                                  GBps=round(4.0 * rows * n / med / 1e3, 1),
                                  speedup_over_unfused=round(base / med, 2))), flush=True)
        del xs, ys
    return 0


def tables_sweep(iters):
    import torch
    from . import binding as rf
    from . import inputs as I

    rf.load_library()
    dev = "cuda:0"
    n_rot = 3

    def timed(fn):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for i in range(iters):
            evs[i][0].record()
            fn(i)
            evs[i][1].record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        return ts[len(ts) // 2]

    def timed_graph(fn, launches=24, replays=7):
        """Per-call time with the host out of the picture: `launches` calls captured once in a
        HIP graph (inputs rotating as in `timed`) and replayed; median over the replays."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(launches):
                fn(i)
        graph.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(replays):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            graph.replay()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / launches)
        del graph
        return sorted(ts)[len(ts) // 2]

    c0 = I.WORKLOADS[0]
    q, k, v = I.attention_inputs_device(I.SEED_BASE, c0["B"], c0["Hq"], c0["Hkv"], c0["Lq"], c0["Lk"], c0["d"], "f32", dev)
    o = torch.empty_like(q)
    f0 = lambda i: rf.rf_cascade_attention(q, k, v, I.default_scale(c0["d"]), False, o=o)
    print(json.dumps(dict(config="C1", workload=c0["name"], us_median=round(timed(f0), 2),
                          us_graph_replay=round(timed_graph(f0), 2))), flush=True)

    for key in sorted(I.MOE_ROUTING_TABLE):
        c = I.table_workload(key)
        sets = []
        for r in range(n_rot):
            x, w = I.moe_routing_inputs_device(I.SEED_BASE + 5 + 100 * r, c["S"], c["hd"], c["E"], c["score_sigma"], "bf16", dev)
            sets.append((x, w, torch.empty((c["S"], c["topk"]), dtype=torch.float32, device=dev),
                         torch.empty((c["S"], c["topk"]), dtype=torch.int32, device=dev)))
        ws = torch.empty(rf.moe_routing_workspace_bytes(c["S"], c["hd"], c["E"]), dtype=torch.uint8, device=dev)
        fn = lambda i: rf.rf_moe_routing(sets[i % n_rot][0], sets[i % n_rot][1], c["topk"], prob=sets[i % n_rot][2],
                                         idx=sets[i % n_rot][3], workspace=ws)
        med, gr = timed(fn), timed_graph(fn)
        b = 2.0 * c["S"] * c["hd"] + 2.0 * c["hd"] * c["E"] + 8.0 * c["S"] * c["topk"]
        print(json.dumps(dict(config=key, workload=c["name"], us_median=round(med, 2), us_graph_replay=round(gr, 2),
                              algorithmic_MB=round(b / 1e6, 2), GBps=round(b / med / 1e3, 1),
                              GBps_graph_replay=round(b / gr / 1e3, 1))), flush=True)
        del sets, ws
    for key in sorted(I.FP8_QUANT_GEMM_TABLE, key=lambda k: int(k[1:])):
        c = I.table_workload(key)
        a, w = I.fp8_quant_gemm_inputs_device(I.SEED_BASE + 7, c["M"], c["K"], c["N"], dev)
        out = torch.empty((c["M"], c["N"]), dtype=torch.bfloat16, device=dev)
        fn = lambda i: rf.rf_fp8_quant_gemm(a, w, c=out)
        med, gr = timed(fn), timed_graph(fn, launches=12)
        fl = 2.0 * c["M"] * c["K"] * c["N"]
        print(json.dumps(dict(config=key, workload=c["name"], us_median=round(med, 2), us_graph_replay=round(gr, 2),
                              GFLOP=round(fl / 1e9, 1), TFLOPs=round(fl / med / 1e6, 1),
                              TFLOPs_graph_replay=round(fl / gr / 1e6, 1))), flush=True)
        del a, w, out
    for key in sorted(I.VARIANCE_TABLE, key=lambda k: int(k[1:])):
        c = I.table_workload(key)
        xs = [I.variance_inputs_device(I.SEED_BASE + 6 + 100 * r, c["bs"], c["l"], c["dtype"], c["mu"], c["sigma"], dev)
              for r in range(n_rot)]
        mv = [(torch.empty(c["bs"], dtype=torch.float32, device=dev), torch.empty(c["bs"], dtype=torch.float32, device=dev))
              for _ in range(n_rot)]
        fn = lambda i: rf.rf_variance(xs[i % n_rot], *mv[i % n_rot])
        med, gr = timed(fn), timed_graph(fn)
        b = 4.0 * c["bs"] * c["l"] + 8.0 * c["bs"]
        print(json.dumps(dict(config=key, workload=c["name"], us_median=round(med, 2), us_graph_replay=round(gr, 2),
                              algorithmic_MB=round(b / 1e6, 2), GBps=round(b / med / 1e3, 1),
                              GBps_graph_replay=round(b / gr / 1e3, 1))), flush=True)
        del xs, mv
    return 0


def eager_sweep():
    import torch
    import torch.nn.functional as F
    from . import binding as rf
    from . import inputs as I

    rf.load_library()
    dev = "cuda:0"
    n_rot = 3

    def timed_graph(fn, launches=24, replays=7):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(n_rot):
                fn(i)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(launches):
                fn(i)
        # (untimed replays for 150 ms: the first launches on an idle GPU do not run at the steady-state clock)
        t_end = time.perf_counter() + 0.15
        while time.perf_counter() < t_end:
            graph.replay()
            torch.cuda.synchronize()
        ts = []
        for _ in range(replays):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            graph.replay()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / launches)
        del graph
        return sorted(ts)[len(ts) // 2]

    def line(config, workload, ours, eager_fn, chain, launches=24):
        try:
            us_e = timed_graph(eager_fn, launches)
        except Exception as e:  # an operator this PyTorch build lacks for the shape: say so, go on
            print(json.dumps(dict(config=config, workload=workload, pytorch_chain=chain,
                                  error=str(e).splitlines()[0][:160])), flush=True)
            return
        us_o = timed_graph(ours, launches)
        print(json.dumps(dict(config=config, workload=workload, pytorch_chain=chain, us_pytorch=round(us_e, 2),
                              us_rf=round(us_o, 2), speedup=round(us_e / us_o, 2))), flush=True)

    W = I.WORKLOADS
    # softmax
    c = W[1]
    xs = [I.softmax_inputs_device(I.SEED_BASE + 1 + 100 * r, c["rows"], c["n"], c["sigma"], "bf16", dev) for r in range(n_rot)]
    ys = [torch.empty_like(x) for x in xs]
    line("W1", c["name"], lambda i: rf.rf_safe_softmax(xs[i % n_rot], ys[i % n_rot]),
         lambda i: torch.softmax(xs[i % n_rot], dim=-1, out=ys[i % n_rot]), "softmax")
    del xs, ys
    # prefill attention
    c = W[2]
    q, k, v = I.attention_inputs_device(I.SEED_BASE + 2, c["B"], c["Hq"], c["Hkv"], c["Lq"], c["Lk"], c["d"], "bf16", dev)
    o = torch.empty_like(q)
    sc = I.default_scale(c["d"])
    for causal in (False, True):
        line("W2" + ("c" if causal else ""), c["name"] + ("_causal" if causal else ""),
             lambda i: rf.rf_cascade_attention(q, k, v, sc, causal=causal, o=o),
             lambda i: F.scaled_dot_product_attention(q, k, v, is_causal=causal, scale=sc), "scaled_dot_product_attention",
             launches=12)
    del q, k, v, o
    # decode, grouped heads
    c = W[3]
    sets = [I.attention_inputs_device(I.SEED_BASE + 3 + 100 * r, c["B"], c["Hq"], c["Hkv"], c["Lq"], c["Lk"], c["d"], "bf16", dev)
            for r in range(n_rot)]
    parts = [rf.alloc_partial_states(sets[r][0], c["num_splits"]) for r in range(n_rot)]
    outs = [torch.empty_like(sets[r][0]) for r in range(n_rot)]

    def ours_decode(i):
        q, k, v = sets[i % n_rot]
        pm, pl, pacc = parts[i % n_rot]
        rf.rf_cascade_attention_splitk(q, k, v, c["num_splits"], pm, pl, pacc, sc, False)
        rf.rf_merge_states(pm, pl, pacc, outs[i % n_rot])

    def eager_decode(i):
        q, k, v = sets[i % n_rot]
        return F.scaled_dot_product_attention(q, k, v, scale=sc, enable_gqa=True)

    line("W3", c["name"], ours_decode, eager_decode, "scaled_dot_product_attention(enable_gqa=True)", launches=6)
    del sets, parts, outs
    # RMSNorm + linear
    c = W[4]
    x, g, w = I.rmsnorm_gemm_inputs_device(I.SEED_BASE + 4, c["M"], c["K"], c["N"], device=dev)
    y = torch.empty((c["M"], c["N"]), dtype=torch.bfloat16, device=dev)
    line("W4", c["name"], lambda i: rf.rf_rmsnorm_gemm(x, g, w, eps=1e-6, y=y),
         lambda i: torch.matmul(F.rms_norm(x, (c["K"],), g, 1e-6), w, out=y), "rms_norm -> matmul", launches=12)
    del x, g, w, y
    # MoE routing
    for key in ("R5", "R8"):
        c = I.table_workload(key)
        ms = []
        for r in range(n_rot):
            xx, ww = I.moe_routing_inputs_device(I.SEED_BASE + 5 + 100 * r, c["S"], c["hd"], c["E"], c["score_sigma"], "bf16", dev)
            ms.append((xx, ww, torch.empty((c["S"], c["topk"]), dtype=torch.float32, device=dev),
                       torch.empty((c["S"], c["topk"]), dtype=torch.int32, device=dev)))
        ws = torch.empty(rf.moe_routing_workspace_bytes(c["S"], c["hd"], c["E"]), dtype=torch.uint8, device=dev)
        line(key, c["name"],
             lambda i: rf.rf_moe_routing(ms[i % n_rot][0], ms[i % n_rot][1], c["topk"], prob=ms[i % n_rot][2],
                                         idx=ms[i % n_rot][3], workspace=ws),
             lambda i: torch.topk(torch.softmax(torch.matmul(ms[i % n_rot][0], ms[i % n_rot][1]).float(), dim=-1), c["topk"], dim=-1),
             "matmul -> softmax -> topk")
        del ms, ws
    # variance
    c = I.table_workload("V8")
    vs = [I.variance_inputs_device(I.SEED_BASE + 6 + 100 * r, c["bs"], c["l"], c["dtype"], c["mu"], c["sigma"], dev) for r in range(n_rot)]
    mv = [(torch.empty(c["bs"], dtype=torch.float32, device=dev), torch.empty(c["bs"], dtype=torch.float32, device=dev))
          for _ in range(n_rot)]
    line("V8", c["name"], lambda i: rf.rf_variance(vs[i % n_rot], *mv[i % n_rot]),
         lambda i: torch.var_mean(vs[i % n_rot], dim=-1, correction=0), "var_mean")
    del vs, mv
    # FP8 quantisation + GEMM
    for key in ("Q3", "Q4"):
        c = I.table_workload(key)
        a, w8 = I.fp8_quant_gemm_inputs_device(I.SEED_BASE + 7, c["M"], c["K"], c["N"], dev)
        out = torch.empty((c["M"], c["N"]), dtype=torch.bfloat16, device=dev)
        ones = torch.ones((1, c["N"]), dtype=torch.float32, device=dev)

        def eager_q(i):
            m = a.abs().amax(dim=1, keepdim=True).float()
            aq = (a.float() * (448.0 / m)).to(torch.float8_e4m3fn)
            return torch._scaled_mm(aq, w8.t(), scale_a=m / 448.0, scale_b=ones, out_dtype=torch.bfloat16)

        line(key, c["name"], lambda i: rf.rf_fp8_quant_gemm(a, w8, c=out), eager_q,
             "abs -> amax -> scale -> cast -> _scaled_mm (row-wise scales)", launches=12)
        del a, w8, out
    return 0


if __name__ == "__main__":
    sys.exit(main())

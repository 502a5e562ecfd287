#!/usr/bin/env python3
"""Benchmark of the Slide Attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One "step" = re-parameterise both kernels (one slide_reparam call over the key and value
kernels stacked along the channel axis, as a module would keep them) + slide_attn_fwd on the
stage-1 forward workload (B=64, 56x56, C=64, 2 heads, k=3, bf16), inputs already
resident in HBM.  Inputs rotate through a pool of buffer sets larger than the
256 MB last-level cache so the figure is HBM bandwidth, not cache bandwidth.
The timed steps are replayed from a HIP graph that holds one step per buffer set
(the two launches of a step take about as long to submit from Python as to run);
the per-launch time of the forward kernel for the roofline comes from HIP events
around a burst of launches queued back to back on the same stream (forward only).
Prints ONE JSON line: whole-job Gpixel*head/s, the HBM roofline of the forward
kernel (algorithmic bytes / measured kernel time), the training workload
(B=128 forward + backward) as extra context, and the CPU oracle timed on this
machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
POOL_SETS = 4                  # 4 x 103 MB > 256 MB cache


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-train", action="store_true")
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 4, 5],
                    help="which bf16 benchmark configuration's forward to time (default 2 = stage 1, "
                         "the configuration the metric is quoted on; the others are for profiling)")
    ap.add_argument("--heads", type=int, default=0,
                    help="profiling: run the configuration (and the training workload) with this many heads "
                         "over the same channels, e.g. 1 at stage 1 = one head of 64 channels")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (batch items, heads and tiles are "
              "independent, so the operator would shard without exchange; nothing here uses a "
              "second GPU); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2304_04237_amd as sa
    from paper_2304_04237_amd import synth

    sa.load_library()                       # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    wl, data = synth.make_config_inputs(args.config - 1)
    if args.heads:                              # same tensors' shapes, other head size
        if wl.C % args.heads != 0:
            print("bench.py: --heads must divide the %d channels" % wl.C, file=sys.stderr)
            sys.exit(2)
        wl = wl._replace(heads=args.heads, name="%s_heads%d" % (wl.name, args.heads))
        data = synth.make_inputs(wl.B, wl.H, wl.W, wl.C, wl.heads, wl.ksize, wl.dtype, seed=1000 + args.config - 1,
                                 with_dout=True)
    B, H, W, C, heads, ksize = wl.B, wl.H, wl.W, wl.C, wl.heads, wl.ksize
    px_heads = B * H * W * heads
    esz = 2
    alg_bytes = 4 * B * C * H * W * esz     # q, k, v read once + out written once

    # pool of input sets (set 0 holds the seeded tensors, the others are seeded copies
    # of the same distribution so every launch reads memory not touched recently)
    pool = []
    for s in range(POOL_SETS):
        d = data if s == 0 else synth.make_inputs(B, H, W, C, heads, ksize, wl.dtype, seed=5000 + s,
                                                  with_dout=False)
        pool.append({n: d[n].to(dev).to(torch.bfloat16) for n in ("q", "k", "v")})
        pool[-1]["out"] = torch.empty_like(pool[-1]["q"])
    wk_l = data["wk_learned"].to(dev)
    wv_l = data["wv_learned"].to(dev)
    bias = data["bias"].to(dev)
    # learned key and value kernels stacked [2C, k*k, k, k]: one re-parameterisation launch per step
    w_l = torch.cat([wk_l, wv_l]).contiguous()
    w_m = torch.empty_like(w_l)
    wk, wv = w_m[:C], w_m[C:]
    path = sa.slide_attn_fwd_path(B, H, W, C, heads, ksize, torch.bfloat16)

    ws_need = sa.slide_attn_workspace_bytes(B, H, W, C, heads, ksize, torch.bfloat16, False)
    ws = torch.empty(max(ws_need, 1), dtype=torch.uint8, device=dev)

    def step(i, ev=None):
        s = pool[i % POOL_SETS]
        sa.slide_reparam(w_l, w_m)
        if ev is not None:
            ev[0].record()
        sa.slide_attn_fwd(s["q"], s["k"], s["v"], wk, wv, bias, heads, ksize, out=s["out"], workspace=ws)
        if ev is not None:
            ev[1].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # forward kernel alone: HIP events around eager launches (on the launch stream)
    n_ev = max(20, min(args.steps, 200))
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(n_ev)]
    for i in range(n_ev):
        step(i, evs[i])
    torch.cuda.synchronize()
    fwd_ms = sorted(a.elapsed_time(b) for a, b in evs)
    fwd_avg_ms = sum(fwd_ms) / len(fwd_ms)
    fwd_med_ms = fwd_ms[len(fwd_ms) // 2]

    # the timed region: exactly args.steps steps, replayed from a graph of POOL_SETS steps
    launch = "hip graph of %d steps, replayed" % POOL_SETS
    graph = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(POOL_SETS):
                step(i)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(POOL_SETS):
                step(i)
        # a replay must reproduce the eager results bit for bit, on every buffer set, twice
        eager = [pool[i]["out"].clone() for i in range(POOL_SETS)]
        for _ in range(2):
            for i in range(POOL_SETS):
                pool[i]["out"].zero_()
            graph.replay()
            torch.cuda.synchronize()
            if not all(torch.equal(pool[i]["out"], eager[i]) for i in range(POOL_SETS)):
                raise RuntimeError("graph replay differs from eager launches")
        del eager
    except Exception as exc:                      # no graph support: plain launches
        graph = None
        launch = "eager (graph capture failed: %s)" % type(exc).__name__
        torch.cuda.synchronize()
    # forward kernel alone: one pair of HIP events around a burst of launches queued back to back
    # on the launch stream (the queue never runs dry, so the quotient is the kernel's duration as a
    # kernel trace reports it, plus at most the hardware's gap between two dispatches)
    n_burst = max(40, min(args.steps, 200))
    for i in range(POOL_SETS):
        s_ = pool[i]
        sa.slide_attn_fwd(s_["q"], s_["k"], s_["v"], wk, wv, bias, heads, ksize, out=s_["out"], workspace=ws)
    torch.cuda.synchronize()
    # (the clocks settle over the first few hundred launches: six bursts, the last three averaged)
    bursts = []
    for _ in range(6):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n_burst):
            s_ = pool[i % POOL_SETS]
            sa.slide_attn_fwd(s_["q"], s_["k"], s_["v"], wk, wv, bias, heads, ksize, out=s_["out"], workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        bursts.append(e0.elapsed_time(e1) / n_burst)
    fwd_burst_ms = sum(bursts[3:]) / 3
    # what the memory system gives for the forward's bytes without its arithmetic (context for
    # the roofline): a flat copy-like kernel and the streaming kernel's access pattern
    probes = {}
    variant = sa.slide_attn_fwd_variant(B, H, W, C, heads, ksize, torch.bfloat16, True)
    for mode, name in ((0, "flat_copy_us"), (1, "streaming_pattern_us")):
        if mode == 1 and variant != 24:
            continue
        try:
            for i in range(POOL_SETS):
                s_ = pool[i]
                sa.slide_attn_fwd_traffic_probe(s_["q"], s_["k"], s_["v"], s_["out"], heads, mode)
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            n_p = 40
            e0.record()
            for i in range(n_p):
                s_ = pool[i % POOL_SETS]
                sa.slide_attn_fwd_traffic_probe(s_["q"], s_["k"], s_["v"], s_["out"], heads, mode)
            e1.record()
            torch.cuda.synchronize()
            probes[name] = e0.elapsed_time(e1) / n_p * 1e3
        except Exception as exc:                  # noqa: BLE001
            probes[name] = "failed: %s" % exc
    # the plain-shift forward (no learned kernels, k*k instead of k^4 multiply-adds) on the same
    # buffers: the same data movement with the least arithmetic the operator can have
    try:
        for i in range(POOL_SETS):
            s_ = pool[i]
            sa.slide_attn_fwd_shift(s_["q"], s_["k"], s_["v"], bias, heads, ksize, out=s_["out"])
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(40):
            s_ = pool[i % POOL_SETS]
            sa.slide_attn_fwd_shift(s_["q"], s_["k"], s_["v"], bias, heads, ksize, out=s_["out"])
        e1.record()
        torch.cuda.synchronize()
        probes["plain_shift_forward_us"] = e0.elapsed_time(e1) / 40 * 1e3
    except Exception as exc:                      # noqa: BLE001
        probes["plain_shift_forward_us"] = "failed: %s" % exc
    # the same workload with channels-last activations ([B,H,W,C], slide_attn_fwd_nhwc)
    try:
        nh = [[torch.randn(B, H, W, C, device=dev).to(torch.bfloat16) for _ in range(3)] +
              [torch.empty(B, H, W, C, device=dev, dtype=torch.bfloat16)] for _ in range(POOL_SETS)]
        for s_ in nh:
            sa.slide_attn_fwd_nhwc(s_[0], s_[1], s_[2], wk, wv, bias, heads, ksize, out=s_[3])
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(40):
            s_ = nh[i % POOL_SETS]
            sa.slide_attn_fwd_nhwc(s_[0], s_[1], s_[2], wk, wv, bias, heads, ksize, out=s_[3])
        e1.record()
        torch.cuda.synchronize()
        probes["channels_last_forward_us"] = e0.elapsed_time(e1) / 40 * 1e3
        del nh
    except Exception as exc:                      # noqa: BLE001
        probes["channels_last_forward_us"] = "failed: %s" % exc
    n_replay, n_tail = (args.steps // POOL_SETS, args.steps % POOL_SETS) if graph is not None else (0, args.steps)
    t0 = time.perf_counter()
    start = torch.cuda.Event(enable_timing=True)
    end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(n_replay):
        graph.replay()
    for i in range(n_tail):
        step(i)
    end.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    total_ms = start.elapsed_time(end)
    ms_per_step = total_ms / args.steps

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_stage1_fwd.json" if args.config == 2 and not args.heads else "none")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("bytes_per_launch")
        except Exception:
            traffic = None
    launch_ms = fwd_burst_ms
    achieved = alg_bytes / (launch_ms * 1e-3) / 1e9
    result = {
        "metric": ("slide-attn fwd Gpixel*head/s at 56x56 stage-1 (reparam + forward per step)"
                   if args.config == 2 and not args.heads else
                   "slide-attn fwd Gpixel*head/s, configuration %d%s (reparam + forward per step)"
                   % (args.config, ", %d heads" % heads if args.heads else "")),
        "value": px_heads / (ms_per_step * 1e-3) / 1e9,
        "unit": "Gpixel*head/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 storage; f16 products and MFMA operands, f32 accumulation", "data": "synthetic",
        "config": {"workload": "%s: B=%d H=%d W=%d C=%d heads=%d head_dim=%d ksize=%d"
                               % (wl.name, B, H, W, C, heads, C // heads, ksize),
                   "inputs": "seeded N(0,1) q,k,v; N(0,0.02^2) learned kernels and bias",
                   "buffer_pool_sets": POOL_SETS, "fwd_kernel_path": path, "fwd_kernel_variant": variant,
                   "launch": launch,
                   "host_wall_ms_per_step": wall_ms / args.steps},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "slide_attn_fwd", "algorithmic_bytes": alg_bytes,
                     "avg_launch_ms": launch_ms,
                     "timing": "HIP events around a burst of %d launches queued back to back (six bursts, mean of the last three)" % n_burst,
                     "burst_avg_ms": bursts,
                     "eager_call_avg_ms": fwd_avg_ms, "eager_call_median_ms": fwd_med_ms,
                     "eager_call_min_ms": fwd_ms[0],
                     "same_bytes_no_arithmetic": probes},
    }

    # ---- training workload (B=128 forward + backward), extra context
    if not args.no_train:
        del pool
        torch.cuda.empty_cache()
        wl5, d5 = synth.make_config_inputs(4)
        if args.heads and wl5.C % args.heads == 0:
            wl5 = wl5._replace(heads=args.heads, name="%s_heads%d" % (wl5.name, args.heads))
            d5 = synth.make_inputs(wl5.B, wl5.H, wl5.W, wl5.C, wl5.heads, wl5.ksize, wl5.dtype, seed=1004, with_dout=True)
        sets = []
        for s in range(2):
            d = d5 if s == 0 else synth.make_inputs(wl5.B, wl5.H, wl5.W, wl5.C, wl5.heads, wl5.ksize,
                                                    wl5.dtype, seed=6000 + s)
            sets.append({n: d[n].to(dev).to(torch.bfloat16) for n in ("q", "k", "v", "dout")})
            sets[-1]["out"] = torch.empty_like(sets[-1]["q"])
        need = sa.slide_attn_workspace_bytes(wl5.B, wl5.H, wl5.W, wl5.C, wl5.heads, wl5.ksize,
                                             torch.bfloat16, True)
        ws = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
        outs = (torch.empty_like(sets[0]["q"]), torch.empty_like(sets[0]["q"]),
                torch.empty_like(sets[0]["q"]), torch.empty_like(wk), torch.empty_like(wv),
                torch.empty_like(bias))
        need_f = sa.slide_attn_workspace_bytes(wl5.B, wl5.H, wl5.W, wl5.C, wl5.heads, wl5.ksize,
                                               torch.bfloat16, False)
        ws_f = torch.empty(max(need_f, 1), dtype=torch.uint8, device=dev)
        n_train = max(4, min(20, args.steps // 10)) // 2 * 2

        def train_step(i):
            s = sets[i % 2]
            sa.slide_reparam(w_l, w_m)
            sa.slide_attn_fwd(s["q"], s["k"], s["v"], wk, wv, bias, wl5.heads, wl5.ksize, out=s["out"],
                              workspace=ws_f)
            sa.slide_attn_bwd(s["dout"], s["q"], s["k"], s["v"], wk, wv, bias, wl5.heads, wl5.ksize,
                              workspace=ws, outputs=outs)

        for i in range(2):
            train_step(i)
        torch.cuda.synchronize()
        want_dq = outs[0].clone()                       # eager result of set 1, the last one run
        # two steps (one per input set) captured in a HIP graph and replayed, like the forward;
        # eager launches if the capture fails or a replay does not reproduce the eager result
        train_graph = None
        try:
            g5 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g5):
                train_step(0)
                train_step(1)
            for _ in range(2):
                outs[0].zero_()
                g5.replay()
                torch.cuda.synchronize()
                if not torch.equal(outs[0], want_dq):
                    raise RuntimeError("graph replay differs from the eager step")
            train_graph = g5
        except Exception as exc:                        # noqa: BLE001
            print("bench.py: training steps launched eagerly (%s)" % exc, file=sys.stderr)
            torch.cuda.synchronize()
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        if train_graph is not None:
            for _ in range(n_train // 2):
                train_graph.replay()
        else:
            for i in range(n_train):
                train_step(i)
        b.record()
        torch.cuda.synchronize()
        tms = a.elapsed_time(b) / n_train
        pxh5 = wl5.B * wl5.H * wl5.W * wl5.heads
        # algorithmic bytes of one step: forward reads q, k, v and writes out; backward reads
        # q, k, v, dout and writes dq, dk, dv (11 tensor passes of B*C*H*W bf16 elements)
        alg5 = 11 * wl5.B * wl5.C * wl5.H * wl5.W * 2
        ach5 = alg5 / (tms * 1e-3) / 1e9
        result["training"] = {"workload": "%s: B=%d H=W=%d C=%d heads=%d ksize=%d, fwd+bwd"
                                          % (wl5.name, wl5.B, wl5.H, wl5.C, wl5.heads, wl5.ksize),
                              "ms_per_step": tms, "steps": n_train,
                              "value": pxh5 / (tms * 1e-3) / 1e9, "unit": "Gpixel*head/s",
                              "launch": ("hip graph of 2 steps, replayed" if train_graph is not None
                                         else "eager"),
                              "workspace_bytes": need,
                              "roofline": {"bound": "hbm", "achieved": ach5, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                           "frac": ach5 / HBM_PEAK_GBS, "algorithmic_bytes": alg5,
                                           "note": "whole step (reparam + forward + backward, 6 launches) "
                                                   "against the bytes of one forward and one backward"}}
        del sets, ws, outs
        torch.cuda.empty_cache()

    # ---- CPU oracle on this machine's host cores (a reported baseline, not a target)
    if not args.no_cpu_baseline:
        from oracle import slide_oracle as oracle
        nb, reps = min(64, B), 8                  # bounded sample: the whole stage-1 workload, eight times (about 17 core-seconds)
        n = {x: data[x][:nb].double().numpy() for x in ("q", "k", "v")}
        wkm = oracle.reparam(data["wk_learned"].double().numpy(), ksize)
        wvm = oracle.reparam(data["wv_learned"].double().numpy(), ksize)
        bn = data["bias"].double().numpy()
        oracle.fwd(n["q"][:1], n["k"][:1], n["v"][:1], wkm, wvm, bn, heads, ksize)      # warm up
        t1 = time.perf_counter()
        for _ in range(reps):
            oracle.fwd(n["q"], n["k"], n["v"], wkm, wvm, bn, heads, ksize)
        dt = (time.perf_counter() - t1) / reps
        cores = oracle.num_threads()
        # the same loops on one thread, on the first four batch items
        oracle.set_num_threads(1)
        t1 = time.perf_counter()
        n1 = min(4, nb)
        oracle.fwd(n["q"][:n1], n["k"][:n1], n["v"][:n1], wkm, wvm, bn, heads, ksize)
        dt1 = time.perf_counter() - t1
        oracle.set_num_threads(cores)
        result["cpu_baseline"] = {"value": nb * H * W * heads / dt / 1e9, "unit": "Gpixel*head/s",
                                  "cores": cores, "kind": "oracle",
                                  "sample": "forward of all %d batch items of the same workload, %d "
                                            "repetitions, fp64 C loops, OpenMP over (batch, head); "
                                            "%.2f s wall each" % (nb, reps, dt),
                                  "value_one_thread": n1 * H * W * heads / dt1 / 1e9,
                                  "sample_one_thread": "%d batch items, %.2f s" % (n1, dt1)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()

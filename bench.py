#!/usr/bin/env python3
"""Benchmark of the partitioned training step on one MI355X.

A "step" is one mini-batch pass of the whole hot path: every F_{z,j}, B_{z,j} of the planned
partitions plus one update per stage (lpm_schedule_run, overlapped schedule replayed as a HIP graph),
on synthetic inputs already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg16_cifar]

Only one GPU is used; --gpus N with N > 1 exits with a message.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"mfma_bf16": 2516.6e12, "fp32": 157.3e12, "hbm": 8.0e12}


def conv_ops(layers, m, first_needs_dgrad=False):
    """[(layer index, op, geometry dict, flops, ideal bytes)] for every contraction of one micro-batch."""
    ops = []
    for i, l in enumerate(layers):
        if l["kind"] not in ("conv", "fc"):
            continue
        kh, kw = (l["h_in"], l["w_in"]) if l["kind"] == "fc" else (l["kh"], l["kw"])
        s, p = (1, 0) if l["kind"] == "fc" else (l["stride"], l["pad"])
        g = dict(m=m, h=l["h_in"], w=l["w_in"], cin=l["cin"], cout=l["cout"], kh=kh, kw=kw, stride=s, pad=p)
        ho, wo = (g["h"] + 2 * p - kh) // s + 1, (g["w"] + 2 * p - kw) // s + 1
        flops = 2 * m * ho * wo * l["cout"] * l["cin"] * kh * kw
        in_el, out_el, w_el = m * g["h"] * g["w"] * l["cin"], m * ho * wo * l["cout"], l["cout"] * kh * kw * l["cin"]
        ops.append((i, "fwd", g, flops, 2 * (in_el + out_el + w_el)))
        if l["src"] >= 0 or first_needs_dgrad:
            ops.append((i, "dgrad", g, flops, 2 * (in_el + out_el + w_el)))
        ops.append((i, "wgrad", g, flops, 2 * (in_el + out_el) + 8 * w_el))
    return ops


def conv_buffers(torch, lpm, g, dtype):
    """Synthetic device operands of one contraction: x, dz-shaped y, w, transposed-shaped wt, dW, scratch."""
    ho = (g["h"] + 2 * g["pad"] - g["kh"]) // g["stride"] + 1
    wo = (g["w"] + 2 * g["pad"] - g["kw"]) // g["stride"] + 1
    tdt = torch.bfloat16 if dtype == lpm.BF16 else torch.float32
    K = g["kh"] * g["kw"] * g["cin"]
    xx = torch.randn(g["m"] * g["h"] * g["w"] * g["cin"], device="cuda").to(tdt)
    yy = torch.randn(g["m"] * ho * wo * g["cout"], device="cuda").to(tdt) * 1e-2
    ww = (torch.randn(g["cout"] * K, device="cuda") * (2.0 / K) ** 0.5).to(tdt)
    wt = ww.clone() if dtype == lpm.BF16 else None
    dw = torch.zeros(g["cout"] * K, device="cuda")
    ws = torch.zeros(max(max(lpm.lpm_conv_ws_bytes(g, dtype)), 256), dtype=torch.uint8, device="cuda")
    return xx, ww, wt, yy, dw, ws


OPI = {"fwd": 0, "dgrad": 1, "wgrad": 2}


def stored_traffic(workload, kernel):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (profiles/hbm_traffic_<workload>.md); None when that file is missing or describes another kernel."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.md" % workload)
    if not os.path.exists(path):
        return None
    kv = {}
    for line in open(path):
        if line.startswith("- ") and ": " in line:
            k, v = line[2:].split(": ", 1)
            kv[k.strip()] = v.strip()
    if kv.get("kernel") != kernel:
        return None
    try:
        return int(float(kv["traffic_bytes_per_launch"]))
    except (KeyError, ValueError):
        return None


def time_stream(torch, fn, iters, warm=3):
    """Average duration in seconds of fn() enqueued `iters` times on torch's current stream, by HIP events."""
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / iters


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vgg16_cifar")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-layer-table", action="store_true", help="skip the per-contraction timing table")
    ap.add_argument("--eager", action="store_true", help="enqueue the step kernel by kernel instead of replaying a graph")
    ap.add_argument("--pmc-probe", default=None, metavar="LAYER:OP",
                    help="counter-collection aid: launch one contraction (e.g. 1:wgrad) and a 256 MiB copy, nothing else")
    ap.add_argument("--only", choices=["locked", "overlapped", "pipelined"], default=None,
                    help="profiling aid: run just this schedule (eager enqueue) for --steps steps and print its time")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); got --gpus %d" % args.gpus,
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import workloads as wl
    import paper_2207_11019_amd as lpm

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)

    builder, batch, M, Z, dt, fixed = wl.CONFIGS[args.workload]
    layers = builder()
    m = batch // M
    dtype = lpm.BF16 if dt == "bf16" else lpm.F32
    cp = dict(lpm.MI355X_COST[dt], link_byte_per_us=0, microbatch=m, n_microbatch=M)
    fixed_starts = None
    if fixed is not None:
        fixed_starts = list(fixed)
    starts, stage_cost = lpm.lpm_partition(layers, Z, cp, fixed_starts)
    dx_wanted = layers[-1]["kind"] != "softmax_ce"
    net = lpm.Net(layers, starts, m, M, dtype, window=2, dx_wanted=dx_wanted, async_update=True)
    params, mom = wl.make_params(layers, bf16=(dt == "bf16"))
    net.load_params(params, mom)
    x, labels, g_up = wl.make_batch(layers, batch, bf16=(dt == "bf16"))
    xd = lpm.pack_act(x, dtype)
    ld = torch.from_numpy(labels).cuda() if labels is not None else None
    gd = lpm.pack_act(g_up, dtype) if g_up is not None else None
    lr, mu = 0.01, 0.9
    def run(mode, steps):
        for _ in range(steps):
            net.step(xd, ld, gd, lr, mu, mode)

    def timed(mode, steps):
        run(mode, args.warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(mode, steps)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    if args.pmc_probe:
        # counter-collection aid: 20 launches of one contraction, then 10 device copies of 256 MiB (the known-size
        # kernel the FETCH_SIZE / WRITE_SIZE readings are scaled by); run under rocprofv3 --pmc
        li, op = args.pmc_probe.split(":")
        g = [o for o in conv_ops(layers, m, dx_wanted) if o[0] == int(li) and o[1] == op][0][2]
        xx, ww, wt, yy, dw, ws = conv_buffers(torch, lpm, g, dtype)
        st = torch.cuda.Stream()
        us = lpm.lpm_conv_time(OPI[op], g, dtype, xx, ww, wt, yy, dw, ws, 0, 20, st)
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        for _ in range(10):
            a.copy_(b)
        torch.cuda.synchronize()
        print(json.dumps({"workload": args.workload, "probe": args.pmc_probe, "geometry": g, "avg_us": round(us, 2),
                          "copy_bytes": 256 << 20}))
        return 0

    if args.only:
        mode = {"locked": lpm.LOCKED, "overlapped": lpm.OVERLAPPED, "pipelined": lpm.PIPELINED}[args.only]
        t = timed(mode, args.steps)
        print(json.dumps({"workload": args.workload, "schedule": args.only, "ms_per_step": round(t / args.steps * 1e3, 4)}))
        return 0

    # the step is timed both enqueued kernel by kernel and replayed as a captured graph; the faster one is reported
    res = {}
    for name, gflag in (("eager", 0), ("graph", lpm.GRAPH)):
        if args.eager and name == "graph":
            continue
        res[name] = {"locked": timed(lpm.LOCKED | gflag, args.steps), "overlapped": timed(lpm.OVERLAPPED | gflag, args.steps)}
        if not gflag:      # the stage-parallel schedule and the per-micro-batch update are enqueue-only
            res[name]["pipelined"] = timed(lpm.PIPELINED, args.steps)
            res[name]["locked_async_update"] = timed(lpm.LOCKED | lpm.ASYNC_UPDATE, args.steps)
            res[name]["overlapped_async_update"] = timed(lpm.OVERLAPPED | lpm.ASYNC_UPDATE, args.steps)
    # headline: the fastest decoupled schedule; the locked time is taken in the same launch mode
    # (the per-micro-batch update computes something else -- M updates per step -- and is reported beside it)
    best, sched = min(((k, m) for k in res for m in res[k] if m in ("overlapped", "pipelined")), key=lambda km: res[km[0]][km[1]])
    t_locked, t_over = res[best]["locked"], res[best][sched]
    ms_step = t_over / args.steps * 1e3
    value = batch * args.steps / t_over

    # ---- per-partition throughput: F + B of every micro-batch + U of one stage alone, on one stream
    part = []
    cur = torch.cuda.Stream()          # not the null stream: its launches carry implicit synchronisation
    torch.cuda.synchronize()
    torch.cuda.set_stream(cur)
    for z, s in enumerate(net.stages):
        b = net.bufs[z]
        xin = xd if z == 0 else net.bufs[z - 1]["act_out"][0]
        loss_stage = layers[s.last - 1]["kind"] == "softmax_ce"
        dy = None if loss_stage else (gd if z == net.Z - 1 else net.bufs[z + 1]["grad_in"][0])
        dxp = b["grad_in"][0] if (z > 0 or dx_wanted) else None

        def one(s=s, b=b, xin=xin, dy=dy, dxp=dxp, loss_stage=loss_stage):
            for j in range(M):
                s.forward(xin, b["act_out"][0], ld if loss_stage else None, net.loss if loss_stage else None, b["params"],
                          b["lowp"], b["stash"][0], b["fwd_ws"], 1.0 / batch, cur)
                s.backward(xin, b["act_out"][0], dy, dxp, b["params"], b["lowp"], b["stash"][0], b["grads"], j > 0,
                           b["bwd_ws"], cur)
            s.update(b["params"], b["lowp"], b["grads"], b["momentum"], 0.0, mu, False, cur)   # lr 0: weights stay put

        t = time_stream(torch, one, max(3, args.steps // 3))
        part.append(dict(stage=z, layers=[starts[z], starts[z + 1]], images_per_s=round(batch / t, 1),
                         ms=round(t * 1e3, 4), model_cost_ps=int(stage_cost[z])))

    # ---- per-contraction table and the roofline of the dominant kernel
    roof, table = None, []
    if not args.no_layer_table:
        ops = conv_ops(layers, m, dx_wanted)
        cache = {}
        for (i, op, g, flops, byts) in ops:
            key = (op,) + tuple(sorted(g.items()))
            if key not in cache:
                xx, ww, wt, yy, dw, ws = conv_buffers(torch, lpm, g, dtype)
                us = lpm.lpm_conv_time(OPI[op], g, dtype, xx, ww, wt, yy, dw, ws, 10, 100, cur)
                cache[key] = us * 1e-6
            t = cache[key]
            ai = flops / byts
            peak_f = PEAK["mfma_bf16"] if dtype == lpm.BF16 else PEAK["fp32"]
            bound = "mfma" if ai >= peak_f / PEAK["hbm"] else "hbm"
            table.append(dict(layer=i, op=op, shape="m%d %dx%dx%d->%d k%d s%d" % (g["m"], g["h"], g["w"], g["cin"], g["cout"],
                                                                                    g["kh"], g["stride"]),
                              us=round(t * 1e6, 2), tflops=round(flops / t / 1e12, 2), gbps=round(byts / t / 1e9, 1),
                              bound=bound, flops=flops, bytes=byts, per_step_us=round(t * 1e6 * M, 1)))
        dom = max(table, key=lambda r: r["per_step_us"])
        t = dom["us"] * 1e-6
        if dom["bound"] == "mfma":
            peak_f = PEAK["mfma_bf16"] if dtype == lpm.BF16 else PEAK["fp32"]
            roof = dict(bound="mfma", achieved=round(dom["flops"] / t / 1e12, 3), peak=peak_f / 1e12, unit="TFLOP/s",
                        frac=round(dom["flops"] / t / peak_f, 5), traffic=None)
        else:
            roof = dict(bound="hbm", achieved=round(dom["bytes"] / t / 1e9, 2), peak=PEAK["hbm"] / 1e9, unit="GB/s",
                        frac=round(dom["bytes"] / t / PEAK["hbm"], 5), traffic=None)
        roof["kernel"] = "conv %s, layer %d (%s)" % (dom["op"], dom["layer"], dom["shape"])
        roof["traffic"] = stored_traffic(args.workload, roof["kernel"])
        roof["avg_us"] = dom["us"]
        tot_flops = sum(r["flops"] for r in table) * M
        roof["step_contraction_flops"] = tot_flops
        roof["step_frac_of_mfma_peak"] = round(tot_flops / (ms_step * 1e-3) / (PEAK["mfma_bf16"] if dtype == lpm.BF16 else PEAK["fp32"]), 5)

    # ---- layer-wise partitioning without merging ("Layer-wise Partitioning and Merging" section, fig. 1a): every layer
    # as n = Z sub-layers on n streams with concatenation / re-partition / summation, against the merged layer
    layerwise = None
    if table:
        n_sub = Z if 2 <= Z <= 8 else 4
        merged_us = lw_us = 0.0
        used = skipped = 0
        lcache = {}
        for i, l in enumerate(layers):
            mine = [r for r in table if r["layer"] == i]
            if not mine:
                continue
            if l["cout"] % (32 * n_sub):       # slices of fewer than 32 channels would fall to the generic data-gradient kernel
                skipped += 1
                continue
            g = next(g for (j, op, g, _, _) in ops if j == i)
            key = tuple(sorted(g.items()))
            if key not in lcache:
                xx, ww, wt, yy, dw, _ = conv_buffers(torch, lpm, g, dtype)
                lw = lpm.Layerwise(g, dtype, n_sub)
                ws = torch.zeros(max(lw.fwd_ws_bytes, lw.bwd_ws_bytes, 256), dtype=torch.uint8, device="cuda")
                want_dx = any(r["op"] == "dgrad" for r in mine)
                dxx = torch.empty_like(xx) if want_dx else None
                lcache[key] = lw.time(0, xx, ww, wt, yy, None, dw, ws, 5, 50, cur) + lw.time(1, xx, ww, wt, yy, dxx, dw, ws, 5, 50, cur)
                lw.close()
            used += 1
            merged_us += sum(r["us"] for r in mine)
            lw_us += lcache[key]
        if used:
            layerwise = dict(n=n_sub, layers=used, layers_skipped=skipped, merged_us_per_step=round(merged_us * M, 1),
                             layerwise_us_per_step=round(lw_us * M, 1), overhead=round(lw_us / merged_us, 3))

    # ---- cost-model feedback (eq. 10 with measured operation times): re-plan from the measured contraction
    # times (layers without a contraction keep their analytic cost) and time the step under that plan
    replan = None
    if table and fixed is None and Z > 1:
        meas = [0] * len(layers)
        for r in table:
            meas[r["layer"]] += int(round(r["us"] * 1e6))
        costs = [meas[i] if meas[i] > 0 else lpm.lpm_layer_cost(layers, i, cp) for i in range(len(layers))]
        starts2, cost2 = lpm.lpm_partition_costs(layers, Z, cp, costs)
        replan = {"plan": starts2, "stage_cost_ps": [int(c) for c in cost2],
                  "model_plan_stage_cost_ps": [int(c) for c in lpm.lpm_partition_costs(layers, Z, cp, costs, starts)[1]]}
        if starts2 != starts:
            del net
            torch.cuda.empty_cache()
            net = lpm.Net(layers, starts2, m, M, dtype, window=2, dx_wanted=dx_wanted)
            net.load_params(params, mom)
            mode = lpm.OVERLAPPED if sched == "overlapped" else lpm.PIPELINED
            replan["ms_per_step"] = round(timed(mode | (lpm.GRAPH if best == "graph" else 0), args.steps) / args.steps * 1e3, 4)
        else:
            replan["ms_per_step"] = round(ms_step, 4)

    # ---- the in-flight window: the headline keeps the method's figure (2: B_{0,j} ends before F_{0,j+2}); four
    # micro-batches in flight is the same computation with more overlap, reported beside it
    by_window = {"2": round(res["eager"]["overlapped"] / args.steps * 1e3, 4)}
    if M >= 4:
        del net
        torch.cuda.empty_cache()
        net = lpm.Net(layers, starts, m, M, dtype, window=4, dx_wanted=dx_wanted)
        net.load_params(params, mom)
        by_window["4"] = round(timed(lpm.OVERLAPPED, args.steps) / args.steps * 1e3, 4)

    # ---- the oracle on the host cores, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lpm_oracle as orc
        import copy
        n_mb = 2 if args.workload in ("vgg16_cifar", "lenet") else 1
        if args.workload == "lenet":
            n_mb = M
        xs = x[: n_mb * m]
        ls = labels[: n_mb * m] if labels is not None else None
        gs = g_up[: n_mb * m] if g_up is not None else None
        p2, m2 = copy.deepcopy(params), copy.deepcopy(mom)
        orc.run_schedule(layers, starts, p2, m2, xs[:m], ls[:m] if ls is not None else None,
                         gs[:m] if gs is not None else None, 1, lr, mu, orc.LOCKED, input_grad=dx_wanted)   # warm-up
        t0 = time.perf_counter()
        orc.run_schedule(layers, starts, p2, m2, xs, ls, gs, n_mb, lr, mu, orc.LOCKED, input_grad=dx_wanted)
        tc = time.perf_counter() - t0
        cpu = dict(value=round(n_mb * m / tc, 3), unit="images/s", cores=int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
                   kind="oracle", sample="%d of %d micro-batches (%d images), locked schedule, forward+backward+update, fp64"
                   % (n_mb, M, n_mb * m), seconds=round(tc, 2))

    out = {
        "metric": "partition train images/s (fwd+bwd+update) + % bf16 MFMA peak, 1 GPU",
        "value": round(value, 2), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dt, "data": "synthetic",
        "config": {"workload": args.workload, "global_batch": batch, "n_microbatch": M, "microbatch": m, "partitions": Z,
                   "plan": starts, "schedule": ("overlapped, forward / data-phase / weight-phase chains on HIP streams of their own" if sched == "overlapped" else "pipelined, HIP streams per partition")
                   + ", window 2, " + ("graph replay" if best == "graph" else "eager enqueue"),
                   "lr": lr, "momentum": mu},
        "locked_ms_per_step": round(t_locked / args.steps * 1e3, 4),
        "ms_per_step_by_launch_mode": {k: {m: round(t / args.steps * 1e3, 4) for m, t in v.items()} for k, v in res.items()},
        "overlap_speedup": round(t_locked / t_over, 4),
        "overlapped_ms_per_step_by_window": by_window,
        "partitions": part,
        "plan_from_measured_costs": replan,
        "layerwise_unmerged": layerwise,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    if table:
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "layer_table_%s.json" % args.workload), "w") as f:
            json.dump(table, f, indent=1)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

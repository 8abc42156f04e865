#!/usr/bin/env python3
"""Benchmark of the partitioned training step on one MI355X.

A "step" is one mini-batch pass of the whole hot path: every F_{z,j}, B_{z,j} of the planned partitions plus one
update per stage (lpm_schedule_run), on synthetic inputs already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload r50_conv4x]

The headline workload is the ResNet-50 conv4_x partition (the bf16 configuration the performance target names;
VGG-16 at 224x224, the largest one, and the other configurations are timed in the same run and reported under
"by_workload").  Weights are not reset between steps: every step applies its update (lr 0.01, momentum 0.9) to the
weights the previous step left, as training would.  Only one GPU is used; --gpus N with N > 1 exits with a message.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"mfma_bf16": 2516.6e12, "fp32": 157.3e12, "hbm": 8.0e12}
DESCRIBED_PLANS = {"vgg16_224": [0, 10, 18, 19, 22]}      # conv1-3 | conv4-5 | FC1 | FC2-3, as the configuration is described


def conv_ops(layers, m, first_needs_dgrad=False):
    """[(layer index, op, geometry dict, flops, ideal bytes)] for every contraction of one micro-batch."""
    ops = []
    for i, l in enumerate(layers):
        if l["kind"] not in ("conv", "fc"):
            continue
        kh, kw = (l["h_in"], l["w_in"]) if l["kind"] == "fc" else (l["kh"], l["kw"])
        s, p = (1, 0) if l["kind"] == "fc" else (l["stride"], l["pad"])
        g = dict(m=m, h=l["h_in"], w=l["w_in"], cin=l["cin"], cout=l["cout"], kh=kh, kw=kw, stride=s, pad=p)
        d = l.get("d_in", 1)                      # volumetric layers: depth, filter depth, depth padding
        kd, pd = (d, 0) if l["kind"] == "fc" else (l.get("kd", 1), l.get("pad_d", 0))
        if d > 1:
            g.update(d=d, kd=kd, pad_d=pd)
        do = (d + 2 * pd - kd) // s + 1
        ho, wo = (g["h"] + 2 * p - kh) // s + 1, (g["w"] + 2 * p - kw) // s + 1
        flops = 2 * m * do * ho * wo * l["cout"] * l["cin"] * kd * kh * kw
        in_el, out_el, w_el = m * d * g["h"] * g["w"] * l["cin"], m * do * ho * wo * l["cout"], l["cout"] * kd * kh * kw * l["cin"]
        ops.append((i, "fwd", g, flops, 2 * (in_el + out_el + w_el)))
        if l["src"] >= 0 or first_needs_dgrad:
            ops.append((i, "dgrad", g, flops, 2 * (in_el + out_el + w_el)))
        ops.append((i, "wgrad", g, flops, 2 * (in_el + out_el) + 8 * w_el))
    return ops


def conv_buffers(torch, lpm, g, dtype):
    """Synthetic device operands of one contraction: x, dz-shaped y, w, transposed-shaped wt, dW, scratch."""
    d, kd, pd = g.get("d", 1), g.get("kd", 1), g.get("pad_d", 0)
    do = (d + 2 * pd - kd) // g["stride"] + 1
    ho = (g["h"] + 2 * g["pad"] - g["kh"]) // g["stride"] + 1
    wo = (g["w"] + 2 * g["pad"] - g["kw"]) // g["stride"] + 1
    tdt = torch.bfloat16 if dtype == lpm.BF16 else torch.float32
    K = kd * g["kh"] * g["kw"] * g["cin"]
    xx = torch.randn(g["m"] * d * g["h"] * g["w"] * g["cin"], device="cuda").to(tdt)
    yy = torch.randn(g["m"] * do * ho * wo * g["cout"], device="cuda").to(tdt) * 1e-2
    ww = (torch.randn(g["cout"] * K, device="cuda") * (2.0 / K) ** 0.5).to(tdt)
    wt = ww.clone() if dtype == lpm.BF16 else None
    dw = torch.zeros(g["cout"] * K, device="cuda")
    ws = torch.zeros(max(max(lpm.lpm_conv_ws_bytes(g, dtype)), 256), dtype=torch.uint8, device="cuda")
    return xx, ww, wt, yy, dw, ws


OPI = {"fwd": 0, "dgrad": 1, "wgrad": 2}


def stored_traffic(workload, kernel):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (profiles/hbm_traffic_<workload>.md: pairs of "- kernel: ..." / "- traffic_bytes_per_launch: ..." lines, one pair per
    measured kernel); None when that file is missing or holds no entry for this kernel."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.md" % workload)
    if not os.path.exists(path):
        return None
    cur = None
    for line in open(path):
        if line.startswith("- kernel: "):
            cur = line[len("- kernel: "):].strip()
        elif line.startswith("- traffic_bytes_per_launch: ") and cur == kernel:
            try:
                return int(float(line.split(": ", 1)[1]))
            except ValueError:
                return None
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


class Workload:
    """One configuration resident on the GPU: layers, plan, network, inputs."""

    def __init__(self, torch, wl, lpm, name, plan=None, window=2, async_update=False):
        self.torch, self.lpm, self.name = torch, lpm, name
        builder, self.batch, self.M, self.Z, self.dt, fixed = {**wl.CONFIGS, **wl.EXTRA_CONFIGS}[name]
        self.layers = builder()
        self.m = self.batch // self.M
        self.dtype = lpm.BF16 if self.dt == "bf16" else lpm.F32
        self.cp = dict(lpm.MI355X_COST[self.dt], link_byte_per_us=0, microbatch=self.m, n_microbatch=self.M)
        self.fixed = fixed
        want = plan if plan is not None else (list(fixed) if fixed is not None else None)
        self.starts, self.stage_cost = lpm.lpm_partition(self.layers, self.Z, self.cp, want)
        self.dx_wanted = self.layers[-1]["kind"] != "softmax_ce"
        self.net = lpm.Net(self.layers, self.starts, self.m, self.M, self.dtype, window=window, dx_wanted=self.dx_wanted,
                           async_update=async_update)
        self.params, self.mom = wl.make_params(self.layers, bf16=(self.dt == "bf16"))
        self.net.load_params(self.params, self.mom)
        self.x, self.labels, self.g_up = wl.make_batch(self.layers, self.batch, bf16=(self.dt == "bf16"))
        self.xd = lpm.pack_act(self.x, self.dtype)
        self.ld = torch.from_numpy(self.labels).cuda() if self.labels is not None else None
        self.gd = lpm.pack_act(self.g_up, self.dtype) if self.g_up is not None else None
        self.lr, self.mu = 0.01, 0.9
        self.peak = PEAK["mfma_bf16"] if self.dtype == lpm.BF16 else PEAK["fp32"]
        self.step_flops = sum(o[3] for o in conv_ops(self.layers, self.m, self.dx_wanted)) * self.M

    def renet(self, starts=None, window=2):
        self.net = None
        self.torch.cuda.empty_cache()
        if starts is not None:
            self.starts = starts
        self.net = self.lpm.Net(self.layers, self.starts, self.m, self.M, self.dtype, window=window, dx_wanted=self.dx_wanted)
        self.net.load_params(self.params, self.mom)

    def timed(self, mode, steps, warmup):
        """Seconds for `steps` steps after `warmup` untimed ones, bracketed by device synchronisation."""
        for _ in range(warmup):
            self.net.step(self.xd, self.ld, self.gd, self.lr, self.mu, mode)
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.net.step(self.xd, self.ld, self.gd, self.lr, self.mu, mode)
        self.torch.cuda.synchronize()
        return time.perf_counter() - t0

    def summary(self, steps, warmup):
        """ms/step overlapped and locked (eager enqueue), images/s, contraction flops over step time as a share of the peak."""
        lpm = self.lpm
        t_o = self.timed(lpm.OVERLAPPED, steps, warmup) / steps
        t_l = self.timed(lpm.LOCKED, steps, warmup) / steps
        return dict(plan=self.starts, global_batch=self.batch, n_microbatch=self.M, ms_per_step=round(t_o * 1e3, 4),
                    locked_ms_per_step=round(t_l * 1e3, 4), images_per_s=round(self.batch / t_o, 1),
                    overlap_speedup=round(t_l / t_o, 4), step_contraction_gflop=round(self.step_flops / 1e9, 1),
                    step_frac_of_peak=round(self.step_flops / t_o / self.peak, 5), dtype=self.dt)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="r50_conv4x")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-layer-table", action="store_true", help="skip the per-contraction timing table")
    ap.add_argument("--layer-table", default=None, metavar="FILE", help="also write the per-contraction timing table (JSON) to FILE")
    ap.add_argument("--no-others", action="store_true", help="skip the other workloads (by_workload) and the memory-bound kernels")
    ap.add_argument("--eager", action="store_true", help="enqueue the step kernel by kernel only, no graph replay")
    ap.add_argument("--pmc-probe", default=None, metavar="WHAT",
                    help="counter-collection aid: launch one kernel a few times and a 256 MiB copy, nothing else.  "
                         "WHAT = LAYER:OP (a contraction, e.g. 1:wgrad), update:STAGE (the SGD update of a stage) or "
                         "pool:LAYER (the forward of a max-pooling layer as a stage of its own)")
    ap.add_argument("--only", choices=["locked", "overlapped", "pipelined"], default=None,
                    help="profiling aid: run just this schedule (eager enqueue) for --steps steps and print its time")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); got --gpus %d" % args.gpus,
              file=sys.stderr)
        return 2

    import numpy as np      # noqa: F401
    import torch
    import workloads as wl
    import paper_2207_11019_amd as lpm

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)

    if args.pmc_probe:
        return pmc_probe(args, torch, wl, lpm)

    W = Workload(torch, wl, lpm, args.workload, async_update=True)
    layers, starts, batch, M, m, dtype, net = W.layers, W.starts, W.batch, W.M, W.m, W.dtype, W.net
    dx_wanted, lr, mu, Z = W.dx_wanted, W.lr, W.mu, W.Z

    if args.only:
        mode = {"locked": lpm.LOCKED, "overlapped": lpm.OVERLAPPED, "pipelined": lpm.PIPELINED}[args.only]
        t = W.timed(mode, args.steps, args.warmup)
        print(json.dumps({"workload": args.workload, "schedule": args.only, "ms_per_step": round(t / args.steps * 1e3, 4)}))
        return 0

    # the step is timed both enqueued kernel by kernel and replayed as a captured graph; the faster one is reported
    res = {}
    for name, gflag in (("eager", 0), ("graph", lpm.GRAPH)):
        if args.eager and name == "graph":
            continue
        res[name] = {"locked": W.timed(lpm.LOCKED | gflag, args.steps, args.warmup),
                     "overlapped": W.timed(lpm.OVERLAPPED | gflag, args.steps, args.warmup)}
        if not gflag:      # the stage-parallel schedule and the per-micro-batch update are enqueue-only
            res[name]["pipelined"] = W.timed(lpm.PIPELINED, args.steps, args.warmup)
            res[name]["locked_async_update"] = W.timed(lpm.LOCKED | lpm.ASYNC_UPDATE, args.steps, args.warmup)
            res[name]["overlapped_async_update"] = W.timed(lpm.OVERLAPPED | lpm.ASYNC_UPDATE, args.steps, args.warmup)
    # headline: the fastest decoupled schedule; the locked time is taken in the same launch mode
    # (the per-micro-batch update computes something else -- M updates per step -- and is reported beside it)
    best, sched = min(((k, s) for k in res for s in res[k] if s in ("overlapped", "pipelined")), key=lambda ks: res[ks[0]][ks[1]])
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
        xin = W.xd if z == 0 else net.bufs[z - 1]["act_out"][0]
        loss_stage = layers[s.last - 1]["kind"] == "softmax_ce"
        dy = None if loss_stage else (W.gd if z == net.Z - 1 else net.bufs[z + 1]["grad_in"][0])
        dxp = b["grad_in"][0] if (z > 0 or dx_wanted) else None

        def one(s=s, b=b, xin=xin, dy=dy, dxp=dxp, loss_stage=loss_stage):
            for j in range(M):
                s.forward(xin, b["act_out"][0], W.ld if loss_stage else None, net.loss if loss_stage else None, b["params"],
                          b["lowp"], b["stash"][0], b["fwd_ws"], 1.0 / batch, cur)
                s.backward(xin, b["act_out"][0], dy, dxp, b["params"], b["lowp"], b["stash"][0], b["grads"], j > 0,
                           b["bwd_ws"], cur)
            s.update(b["params"], b["lowp"], b["grads"], b["momentum"], 0.0, mu, False, cur)   # lr 0: weights stay put

        t = time_stream(torch, one, max(3, args.steps // 3))
        part.append(dict(stage=z, layers=[starts[z], starts[z + 1]], images_per_s=round(batch / t, 1),
                         ms=round(t * 1e3, 4), model_cost_ps=int(W.stage_cost[z])))

    # ---- per-contraction table and the roofline of the dominant kernel
    roof, table, ops = None, [], []
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
            bound = "mfma" if ai >= W.peak / PEAK["hbm"] else "hbm"
            table.append(dict(layer=i, op=op, shape="m%d %s%dx%dx%d->%d k%d s%d" % (g["m"], "%dx" % g["d"] if "d" in g else "", g["h"], g["w"],
                                                                                      g["cin"], g["cout"], g["kh"], g["stride"]),
                              us=round(t * 1e6, 2), tflops=round(flops / t / 1e12, 2), gbps=round(byts / t / 1e9, 1),
                              frac_of_mfma_peak=round(flops / t / W.peak, 4),
                              bound=bound, flops=flops, bytes=byts, per_step_us=round(t * 1e6 * M, 1)))
        # the dominant kernel: the launch shape with the largest share of a step (identical layers add up)
        share = {}
        for r in table:
            share[(r["op"], r["shape"])] = share.get((r["op"], r["shape"]), 0.0) + r["per_step_us"]
        dkey = max(share, key=share.get)
        dom = next(r for r in table if (r["op"], r["shape"]) == dkey)
        t = dom["us"] * 1e-6
        if dom["bound"] == "mfma":
            roof = dict(bound="mfma", achieved=round(dom["flops"] / t / 1e12, 3), peak=W.peak / 1e12, unit="TFLOP/s",
                        frac=round(dom["flops"] / t / W.peak, 5), traffic=None)
        else:
            roof = dict(bound="hbm", achieved=round(dom["bytes"] / t / 1e9, 2), peak=PEAK["hbm"] / 1e9, unit="GB/s",
                        frac=round(dom["bytes"] / t / PEAK["hbm"], 5), traffic=None)
        roof["kernel"] = "conv %s, layer %d (%s)" % (dom["op"], dom["layer"], dom["shape"])
        roof["launches_per_step"] = int(round(share[dkey] / dom["per_step_us"])) * M
        roof["share_of_contraction_time"] = round(share[dkey] / sum(share.values()), 4)
        roof["traffic"] = stored_traffic(args.workload, roof["kernel"])
        roof["avg_us"] = dom["us"]
        roof["algorithmic_flops"] = dom["flops"]
        roof["algorithmic_bytes"] = dom["bytes"]
        roof["frac_of_mfma_peak"] = round(dom["flops"] / t / W.peak, 5)
        roof["step_contraction_flops"] = W.step_flops
        roof["step_frac_of_mfma_peak"] = round(W.step_flops / (ms_step * 1e-3) / W.peak, 5)
        fr = sorted(r["frac_of_mfma_peak"] for r in table if r["bound"] == "mfma")
        if fr:
            roof["mfma_bound_contractions_frac_of_peak"] = dict(min=fr[0], median=fr[len(fr) // 2], max=fr[-1], count=len(fr))

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
            if l["cout"] % (32 * n_sub) or l.get("d_in", 1) > 1:       # slices of fewer than 32 channels would fall to the generic
                skipped += 1                                            # data-gradient kernel; volumetric layers are not sliced
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
    if table and W.fixed is None and Z > 1:
        meas = [0] * len(layers)
        for r in table:
            meas[r["layer"]] += int(round(r["us"] * 1e6))
        costs = [meas[i] if meas[i] > 0 else lpm.lpm_layer_cost(layers, i, W.cp) for i in range(len(layers))]
        starts2, cost2 = lpm.lpm_partition_costs(layers, Z, W.cp, costs)
        replan = {"plan": starts2, "stage_cost_ps": [int(c) for c in cost2],
                  "model_plan_stage_cost_ps": [int(c) for c in lpm.lpm_partition_costs(layers, Z, W.cp, costs, starts)[1]]}
        if starts2 != starts:
            net = None
            W.renet(starts2)
            mode = lpm.OVERLAPPED if sched == "overlapped" else lpm.PIPELINED
            replan["ms_per_step"] = round(W.timed(mode | (lpm.GRAPH if best == "graph" else 0), args.steps, args.warmup) / args.steps * 1e3, 4)
            W.starts = starts
        else:
            replan["ms_per_step"] = round(ms_step, 4)

    # ---- the in-flight window: the headline keeps the method's figure (2: B_{0,j} ends before F_{0,j+2}); four
    # micro-batches in flight is the same computation with more overlap, reported beside it
    by_window = {"2": round(res["eager"]["overlapped"] / args.steps * 1e3, 4)}
    if M >= 4:
        net = None
        W.renet(starts, window=4)
        by_window["4"] = round(W.timed(lpm.OVERLAPPED, args.steps, args.warmup) / args.steps * 1e3, 4)
    net = None
    W.net = None
    torch.cuda.empty_cache()

    # ---- the other configurations, timed in the same run (eager enqueue, fewer steps), and the memory-bound kernels at
    # sizes beyond the 256 MB last-level cache (the 224x224 VGG-16: 103 M parameters in its first FC layer)
    by_workload, memory_bound = None, None
    if not args.no_others:
        by_workload, memory_bound = {}, {}
        n_other = max(5, args.steps // 3)
        for name in ("vgg16_cifar", "resnet18_cifar", "r50_conv4x", "vgg16_224", "lenet", "resattnet18_3d"):
            if name == args.workload:
                by_workload[name] = dict(plan=starts, global_batch=batch, n_microbatch=M, ms_per_step=round(res["eager"]["overlapped"] / args.steps * 1e3, 4),
                                         locked_ms_per_step=round(res["eager"]["locked"] / args.steps * 1e3, 4),
                                         images_per_s=round(batch * args.steps / res["eager"]["overlapped"], 1),
                                         overlap_speedup=round(res["eager"]["locked"] / res["eager"]["overlapped"], 4),
                                         step_contraction_gflop=round(W.step_flops / 1e9, 1),
                                         step_frac_of_peak=round(W.step_flops * args.steps / res["eager"]["overlapped"] / W.peak, 5), dtype=W.dt)
                continue
            V = Workload(torch, wl, lpm, name)
            by_workload[name] = V.summary(n_other, 3)
            if name in DESCRIBED_PLANS and V.starts != DESCRIBED_PLANS[name]:
                # the plan the configuration describes in words, beside the one the cost model picks
                by_workload[name]["plan_source"] = "cost model (lpm_partition)"
                if name == "vgg16_224":
                    memory_bound.update(memory_kernels(torch, lpm, V, cur))
                V.renet(DESCRIBED_PLANS[name])
                d = V.summary(n_other, 3)
                d["plan_source"] = "as the configuration is described (conv1-3 | conv4-5 | FC1 | FC2-3)"
                by_workload[name + "_described_plan"] = d
            V.net = None
            del V
            torch.cuda.empty_cache()

    # ---- the oracle on the host cores, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lpm_oracle as orc
        import copy
        # a sample of 10-30 s of host work: the whole step of the ResNet-50 stage (4 micro-batches, about 18 s on 16 cores)
        n_mb = {"vgg16_cifar": M, "lenet": M, "r50_conv4x": M, "resnet18_cifar": 2, "resattnet18_3d": M}.get(args.workload, 1)
        xs = W.x[: n_mb * m]
        ls = W.labels[: n_mb * m] if W.labels is not None else None
        gs = W.g_up[: n_mb * m] if W.g_up is not None else None
        p2, m2 = copy.deepcopy(W.params), copy.deepcopy(W.mom)
        # warm-up on two images (loads the library, starts the thread pool)
        orc.run_schedule(layers, starts, p2, m2, xs[:2], ls[:2] if ls is not None else None,
                         gs[:2] if gs is not None else None, 1, lr, mu, orc.LOCKED, input_grad=dx_wanted)
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
        "dtype": W.dt, "data": "synthetic",
        "config": {"workload": args.workload, "global_batch": batch, "n_microbatch": M, "microbatch": m, "partitions": Z,
                   "plan": starts, "schedule": ("overlapped, forward / data-phase / weight-phase chains on HIP streams of their own" if sched == "overlapped" else "pipelined, HIP streams per partition")
                   + ", window 2, " + ("graph replay" if best == "graph" else "eager enqueue"),
                   "lr": lr, "momentum": mu,
                   "weights": "drift: every step updates the weights the previous step left (no reset between steps)"},
        "locked_ms_per_step": round(t_locked / args.steps * 1e3, 4),
        "ms_per_step_by_launch_mode": {k: {s: round(t / args.steps * 1e3, 4) for s, t in v.items()} for k, v in res.items()},
        "overlap_speedup": round(t_locked / t_over, 4),
        "overlapped_ms_per_step_by_window": by_window,
        "partitions": part,
        "plan_from_measured_costs": replan,
        "layerwise_unmerged": layerwise,
        "by_workload": by_workload,
        "memory_bound_kernels": memory_bound,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    if table and args.layer_table:
        with open(args.layer_table, "w") as f:
            json.dump(table, f, indent=1)
    print(json.dumps(out))
    return 0


def pool_stage(lpm, V, layer):
    """A max-pooling layer of workload V as a stage of its own, with device buffers for one micro-batch."""
    torch = V.torch
    s = lpm.Stage(V.layers, layer, layer + 1, V.m, V.dtype)
    tdt = torch.bfloat16 if V.dtype == lpm.BF16 else torch.float32
    esz = 2 if V.dtype == lpm.BF16 else 4
    x = torch.randn(s.in_bytes // esz, device="cuda").to(tdt)
    y = torch.empty(s.out_bytes // esz, dtype=tdt, device="cuda")
    z = lambda n: torch.zeros(max(n, 256), dtype=torch.uint8, device="cuda")      # noqa: E731
    return s, x, y, z(s.param_bytes), z(s.stash_bytes), z(s.fwd_ws_bytes)


def memory_kernels(torch, lpm, V, cur):
    """HBM-bound kernels at the 224x224 VGG-16's sizes, timed with events on the launching stream: the SGD update of the
    stage that holds the first FC layer (22 bytes per parameter: g, p, v read; p, v and the bf16 copy written) and the
    first max-pooling forward (10 bytes per output element)."""
    out = {}
    z = max(range(V.net.Z), key=lambda k: V.net.stages[k].grad_bytes)
    s, b = V.net.stages[z], V.net.bufs[z]
    n = s.grad_bytes // 4
    t = time_stream(torch, lambda: s.update(b["params"], b["lowp"], b["grads"], b["momentum"], 0.0, V.mu, False, cur), 10)
    byts = 22 * n
    out["sgd_update"] = dict(kernel="sgd_kernel (+ transposed weight copies), stage %d of vgg16_224" % z, parameters=n, algorithmic_bytes=byts,
                             us=round(t * 1e6, 1), achieved_gbps=round(byts / t / 1e9, 1), peak_gbps=8000.0, frac=round(byts / t / PEAK["hbm"], 4))
    pl = next(i for i, l in enumerate(V.layers) if l["kind"] == "maxpool2")
    ps, x, y, par, stash, ws = pool_stage(lpm, V, pl)
    t = time_stream(torch, lambda: ps.forward(x, y, None, None, par, None if V.dtype != lpm.BF16 else par, stash, ws, 1.0, cur), 50)
    byts = ps.in_bytes + ps.out_bytes
    out["maxpool_forward"] = dict(kernel="maxpool_fwd_bf16x8, layer %d of vgg16_224 (micro-batch %d)" % (pl, V.m), algorithmic_bytes=byts,
                                  us=round(t * 1e6, 2), achieved_gbps=round(byts / t / 1e9, 1), peak_gbps=8000.0,
                                  frac=round(byts / t / PEAK["hbm"], 4), note="%d MB: resident in the 256 MB last-level cache" % (byts >> 20))
    ps.close()
    return out


def pmc_probe(args, torch, wl, lpm):
    """Counter-collection aid, run under `rocprofv3 --pmc ...`: a few launches of one kernel, then 10 device copies of
    256 MiB (the known-size kernel the FETCH_SIZE / WRITE_SIZE readings are scaled by).  Nothing else runs."""
    what, arg = args.pmc_probe.split(":")
    info = {"workload": args.workload, "probe": args.pmc_probe}
    builder, batch, M, Z, dt, fixed = wl.CONFIGS[args.workload]
    layers = builder()
    m = batch // M
    dtype = lpm.BF16 if dt == "bf16" else lpm.F32
    dx_wanted = layers[-1]["kind"] != "softmax_ce"
    st = torch.cuda.Stream()
    class V:          # what pool_stage needs of a workload, without its parameters (the kernels probed here do not read them)
        pass
    V.torch, V.layers, V.m, V.dtype = torch, layers, m, dtype
    if what == "update":
        cp = dict(lpm.MI355X_COST[dt], link_byte_per_us=0, microbatch=m, n_microbatch=M)
        starts, _ = lpm.lpm_partition(layers, Z, cp, list(fixed) if fixed is not None else None)
        z = int(arg)
        s = lpm.Stage(layers, starts[z], starts[z + 1], m, dtype)
        zb = lambda n: torch.zeros(max(n, 256), dtype=torch.uint8, device="cuda")      # noqa: E731
        b = dict(params=zb(s.param_bytes), lowp=zb(s.lowp_bytes), grads=zb(s.grad_bytes), momentum=zb(s.grad_bytes))
        torch.cuda.synchronize()
        for _ in range(5):
            s.update(b["params"], b["lowp"] if dtype == lpm.BF16 else None, b["grads"], b["momentum"], 0.0, 0.9, False, st)
        info.update(stage_layers=[starts[z], starts[z + 1]], parameters=s.grad_bytes // 4, algorithmic_bytes=22 * (s.grad_bytes // 4))
    elif what == "pool":
        ps, x, y, par, stash, ws = pool_stage(lpm, V, int(arg))
        torch.cuda.synchronize()
        for _ in range(20):
            ps.forward(x, y, None, None, par, par, stash, ws, 1.0, st)
        info.update(algorithmic_bytes=ps.in_bytes + ps.out_bytes)
    else:
        op = arg
        g, flops, byts = [(o[2], o[3], o[4]) for o in conv_ops(layers, m, dx_wanted) if o[0] == int(what) and o[1] == op][0]
        xx, ww, wt, yy, dw, ws = conv_buffers(torch, lpm, g, dtype)
        us = lpm.lpm_conv_time(OPI[op], g, dtype, xx, ww, wt, yy, dw, ws, 0, 20, st)
        info.update(geometry=g, avg_us=round(us, 2), algorithmic_flops=flops, algorithmic_bytes=byts)
    torch.cuda.synchronize()
    a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    b2 = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
    for _ in range(10):
        a.copy_(b2)
    torch.cuda.synchronize()
    info["copy_bytes"] = 256 << 20
    print(json.dumps(info))
    return 0


if __name__ == "__main__":
    sys.exit(main())

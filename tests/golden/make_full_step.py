#!/usr/bin/env python3
"""Writes tests/golden/full_step_<workload>.npz: expected values of ONE full mini-batch step (all M micro-batches,
gradient accumulation, update) of the full-size bf16 workloads, computed by the fp64 oracle alone.

The oracle needs minutes per workload (0.5 - 3 TFLOP of direct fp64 loops), more than a GPU test may spend, so its
result is stored -- as samples: per tensor, a seeded choice of element positions with the oracle's values there,
the tensor's largest magnitude (the denominator of the error measure) and its 2-norm.  Nothing here touches the
GPU library; the inputs are the seeded generators of workloads/ that the GPU tests call with the same arguments.

Two oracle runs per workload:
  A  store=None          the plain fp64 computation from bf16-representable inputs and weights: THE reference
  B  store=round_bf16    the same arithmetic with every stored activation rounded to bfloat16 once -- a second
                         valid result of a bf16 implementation
The distance B - A per tensor is stored beside A's samples as the workload's decision-flip noise floor
(tests/flipnoise.py explains the mechanism): a GPU result cannot be asked to be closer to A than another valid
bf16 result is.  Forward activations carry no decisions and are compared at the plain bar.

    python tests/golden/make_full_step.py [workload ...]
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import workloads as wl                      # noqa: E402
from oracle import lpm_oracle as orc        # noqa: E402
import flipnoise as fn                      # noqa: E402

# name -> (plan, mini-batch, micro-batches, upstream gradient wanted); seeds and hyper-parameters as the GPU test uses them
CASES = {
    "resnet18_cifar": ([0, 5, 10, 15, 23], 256, 8, False),
    "r50_conv4x": ([0, 19], 64, 4, True),
    "vgg16_224": ([0, 10, 18, 19, 22], 32, 8, False),      # the described plan: conv1-3 | conv4-5 | FC1 | FC2-3
    "resattnet18_3d": ([0, 3, 8, 18, 29], 6, 3, False),    # volumetric use case: 3x3x3 residual blocks and self-attention blocks
}
SEED, LR, MU, BIAS_STD, MOM_STD, NSAMPLE = 17, 0.01, 0.9, 0.05, 1e-3, 1024


def sample_positions(name, size):
    r = np.random.default_rng([SEED] + [ord(c) for c in name])      # (keyed by the tensor's name)
    if size <= NSAMPLE:
        return np.arange(size, dtype=np.int32)
    return np.sort(r.choice(size, NSAMPLE, replace=False)).astype(np.int32)


def run(layers, plan, batch, M, dx, store):
    params, mom = wl.make_params(layers, SEED, bf16=True, bias_std=BIAS_STD, momentum_std=MOM_STD)
    x, labels, g = wl.make_batch(layers, batch, SEED, bf16=True)
    ref = orc.run_schedule(layers, plan, params, mom, x, labels, g, M, LR, MU, orc.LOCKED, keep=True, input_grad=dx, store=store)
    return ref, params, mom


def tensors_of(layers, plan, M, dx, ref, params, mom):
    """{name: array} of everything a GPU step is compared on (logical layouts)."""
    out = {}
    for i in params:
        for k in ("W", "b"):
            if k in params[i]:
                out["grad.%d.%s" % (i, k)] = ref["grads"][i][k]
                out["param.%d.%s" % (i, k)] = params[i][k]
                out["mom.%d.%s" % (i, k)] = mom[i][k]
    j = M - 1
    for z in range(len(plan) - 1):
        st = ref["stash"][(z, j)]
        for t in range(plan[z], plan[z + 1]):
            if layers[t]["kind"] != "softmax_ce":
                out["act.%d" % t] = st[t]
        if z > 0 or dx:
            out["gin.%d" % z] = ref["gin"][(z, j)]
            if z > 0:        # sign of the stage input, for schedules that hand down the pre-activation gradient of the layer before the cut
                out["gin.%d.mask" % z] = (ref["stash"][(z - 1, j)][plan[z] - 1] > 0).astype(np.float64)
    return out


def main(names):
    for name in names:
        plan, batch, M, dx = CASES[name]
        layers = {**wl.CONFIGS, **wl.EXTRA_CONFIGS}[name][0]()
        t0 = time.time()
        A = run(layers, plan, batch, M, dx, None)
        print(name, "reference run %.0f s" % (time.time() - t0), flush=True)
        t0 = time.time()
        B = run(layers, plan, batch, M, dx, orc.round_bf16)
        print(name, "bf16-storage run %.0f s" % (time.time() - t0), flush=True)
        ta, tb = tensors_of(layers, plan, M, dx, *A), tensors_of(layers, plan, M, dx, *B)
        rec = {"loss": np.array([A[0]["loss"], B[0]["loss"]]), "plan": np.array(plan), "batch_M_seed": np.array([batch, M, SEED]),
               "hyper": np.array([LR, MU, BIAS_STD, MOM_STD])}
        for key, a in ta.items():
            a = np.asarray(a, dtype=np.float64)
            b = np.asarray(tb[key], dtype=np.float64)
            pos = sample_positions(key[:-5] if key.endswith(".mask") else key, a.size)      # (a mask is sampled where its gradient is)
            av, bv = a.reshape(-1)[pos], b.reshape(-1)[pos]
            maxabs, l2 = float(np.abs(a).max()), float(np.linalg.norm(a.ravel()))
            rec[key + ".idx"] = pos
            rec[key + ".val"] = av
            # [largest magnitude, 2-norm, floor (B - A) in the infinity measure on the whole tensor, in the 2-norm on the whole
            #  tensor, the same two on the sampled positions only, 2-norm of A's samples]
            rec[key + ".meta"] = np.array([maxabs, l2, fn.inf_err(b, a), fn.l2_err(b, a),
                                           float(np.abs(bv - av).max() / max(maxabs, 1e-30)),
                                           float(np.linalg.norm(bv - av) / max(np.linalg.norm(av), 1e-30)),
                                           float(np.linalg.norm(av))])
        flips = [fn.decision_disagreements(layers, plan[z], plan[z + 1], A[0]["stash"][(z, M - 1)], B[0]["stash"][(z, M - 1)])
                 for z in range(len(plan) - 1)]
        rec["flips_last_microbatch"] = np.array(flips).sum(axis=0)
        path = os.path.join(ROOT, "tests", "golden", "full_step_%s.npz" % name)
        np.savez_compressed(path, **rec)
        worst = sorted(((rec[k][3], k[:-5]) for k in rec if k.endswith(".meta") and k.startswith("grad.")), reverse=True)[:3]
        print(name, "written", path, "%.1f KB" % (os.path.getsize(path) / 1024), "flips (relu, of, pool, of)", rec["flips_last_microbatch"],
              "largest gradient floors (2-norm)", worst, flush=True)


if __name__ == "__main__":
    main(sys.argv[1:] or list(CASES))

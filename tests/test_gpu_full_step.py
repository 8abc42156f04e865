"""The timed path at full size: one OVERLAPPED mini-batch step (all M micro-batches, gradient accumulation, the staged
once-per-group weight gradients, the update) of each remaining bf16 workload against the fp64 oracle's step, and the
three schedules against each other bit for bit.

The oracle's step takes minutes per workload, so its result is read from tests/golden/full_step_<workload>.npz,
written by tests/golden/make_full_step.py from the oracle alone: per tensor a seeded sample of element positions
with the unrounded fp64 values there, the tensor's largest magnitude, and the workload's decision-flip noise floor
(how far a second valid bf16 result -- the same arithmetic with stored activations rounded to bfloat16 -- lies from
the unrounded one; tests/test_oracle_flip_noise.py pins the mechanism).  Bars:
  loss, every activation of the last micro-batch:   2e-2 (of the tensor's largest magnitude), against the unrounded oracle
  accumulated gradients, momentum, updated weights, boundary gradients:   2e-2 + 2 x floor, in the same measure taken over
  all but the worst 1 % of the sampled elements (one flipped decision moves single elements by up to the tensor's largest
  magnitude) and in the 2-norm (the weights move by lr x momentum, which for these workloads is several per cent of their size)
"""
import os

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module")
def lpm():
    import torch
    assert torch.cuda.is_available()
    import paper_2207_11019_amd as lpm
    return lpm


def _run(lpm, torch, layers, plan, batch, M, dx, params, mom, xd, ld, gd, lr, mu, mode):
    net = lpm.Net(layers, plan, batch // M, M, lpm.BF16, window=2, dx_wanted=dx)
    net.load_params(params, mom)
    net.step(xd, ld, gd, lr, mu, mode)
    torch.cuda.synchronize()
    return net


@pytest.mark.parametrize("name", ["r50_conv4x", "resnet18_cifar", "vgg16_224", "resattnet18_3d"])
def test_full_step_overlapped_bf16(lpm, name):
    import torch
    path = os.path.join(GOLDEN, "full_step_%s.npz" % name)
    assert os.path.exists(path), "run tests/golden/make_full_step.py %s" % name
    d = np.load(path)
    plan = [int(v) for v in d["plan"]]
    batch, M, seed = (int(v) for v in d["batch_M_seed"])
    lr, mu, bias_std, mom_std = (float(v) for v in d["hyper"])
    layers = {**wl.CONFIGS, **wl.EXTRA_CONFIGS}[name][0]()
    params, mom = wl.make_params(layers, seed, bf16=True, bias_std=bias_std, momentum_std=mom_std)
    x, labels, g = wl.make_batch(layers, batch, seed, bf16=True)
    dx = labels is None
    xd = lpm.pack_act(x, lpm.BF16)
    ld = torch.from_numpy(labels).to("cuda:0") if labels is not None else None
    gd = lpm.pack_act(g, lpm.BF16) if g is not None else None
    Z = len(plan) - 1
    print("workload", name, "plan", plan, "batch", batch, "M", M, flush=True)

    net = _run(lpm, torch, layers, plan, batch, M, dx, params, mom, xd, ld, gd, lr, mu, lpm.OVERLAPPED)
    got = {}
    gg, pp, vv = net.read_grads(), net.read_params(), net.read_momentum()
    for i in gg:
        for k in gg[i]:
            got["grad.%d.%s" % (i, k)], got["param.%d.%s" % (i, k)], got["mom.%d.%s" % (i, k)] = gg[i][k], pp[i][k], vv[i][k]
    slot = (M - 1) % 2
    for z in range(Z):
        for t in range(plan[z], plan[z + 1]):
            if layers[t]["kind"] != "softmax_ce":
                got["act.%d" % t] = net.read_act_out(z, slot) if t == net._out_tensor(z) else net.read_stash(t, slot)
        if z > 0 or dx:
            got["gin.%d" % z] = net.read_grad_in(z, slot)
    loss = net.loss_value() if labels is not None else None
    fused = {z: bool(z > 0 and net.schedule.cut_fused(z)) for z in range(Z)}
    ref_bits = {k: v.copy() for k, v in got.items() if k.startswith(("param.", "mom."))}
    del net

    keys = sorted(k[:-4] for k in d.files if k.endswith(".idx") and not k.endswith(".mask.idx"))
    assert set(keys) == set(got), (set(keys) ^ set(got))
    report, bad = [], []
    for key in keys:
        idx, val, meta = d[key + ".idx"], d[key + ".val"], d[key + ".meta"]
        kind = key.split(".")[0]
        if kind == "gin" and fused[int(key.split(".")[1])]:
            val = val * d[key + ".mask.val"]        # the cut hands down the gradient with the ReLU derivative of the stage input applied
        s = np.asarray(got[key], dtype=np.float64).reshape(-1)[idx]
        e_inf = float(np.abs(s - val).max() / max(meta[0], 1e-30))
        if kind != "act":
            # all but the worst 1 % of the sampled elements: a single flipped decision moves single elements of a boundary
            # gradient by up to the tensor's largest magnitude, whichever implementation flipped it
            e_inf = float(np.percentile(np.abs(s - val), 99.0) / max(meta[0], 1e-30))
        e_l2 = float(np.linalg.norm(s - val) / max(np.linalg.norm(val), 1e-30))
        if kind == "act":
            b_inf, b_l2 = 2e-2, None
        else:
            b_inf, b_l2 = 2e-2 + 2 * meta[2], 2e-2 + 2 * meta[3]
        report.append((key, e_inf, b_inf, e_l2, b_l2))
        if not (e_inf <= b_inf) or (b_l2 is not None and not (e_l2 <= b_l2)):
            bad.append(report[-1])
    for kind in ("act", "grad", "mom", "param", "gin"):
        rows = [r for r in report if r[0].startswith(kind + ".")]
        if rows:
            w = max(rows, key=lambda r: r[1] / r[2])
            print("%-5s %3d tensors; closest to its bound: %s  error %.4g (bound %.4g), 2-norm %.4g" % (kind, len(rows), w[0], w[1], w[2], w[3]),
                  flush=True)
    print("decisions on which the two oracle runs differ, last micro-batch (relu, of, pool, of):", d["flips_last_microbatch"], flush=True)
    if loss is not None:
        e = abs(loss - float(d["loss"][0])) / abs(float(d["loss"][0]))
        print("loss %.6f, oracle %.6f (bf16-storage oracle run %.6f)" % (loss, d["loss"][0], d["loss"][1]), flush=True)
        assert e <= 2e-2
    assert not bad, "over their bounds (tensor, error, bound, 2-norm error, bound): %s" % bad[:8]

    # the three schedules give the same bits at full size
    for mode, label in ((lpm.LOCKED, "locked"), (lpm.PIPELINED, "pipelined")):
        other = _run(lpm, torch, layers, plan, batch, M, dx, params, mom, xd, ld, gd, lr, mu, mode)
        pp, vv = other.read_params(), other.read_momentum()
        for i in pp:
            for k in ("W", "b"):
                if k in pp[i]:
                    np.testing.assert_array_equal(pp[i][k], ref_bits["param.%d.%s" % (i, k)], err_msg="%s param %d.%s" % (label, i, k))
                    np.testing.assert_array_equal(vv[i][k], ref_bits["mom.%d.%s" % (i, k)], err_msg="%s momentum %d.%s" % (label, i, k))
        if loss is not None:
            assert other.loss_value() == loss
        print(label, "== overlapped bitwise", flush=True)
        del other

"""Shared driver for the GPU parity tests: runs the oracle and the HIP library on the same seeded
inputs and compares tensor by tensor.

Error measure (both element types): max_i |gpu_i - ref_i| / max_i |ref_i| per tensor, i.e. the error
relative to the tensor's infinity norm; an element-wise relative error is meaningless at the zeros a
ReLU produces.  Bars: 1e-4 for the float path, 2e-2 for the bf16 path.
"""
import copy

import numpy as np

import workloads as wl
from oracle import lpm_oracle as orc
import flipnoise as fn

TOL = {0: 1e-4, 1: 2e-2}


def rel_err(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def read_tensor(net, z, t, slot):
    """Tensor t of stage z for the micro-batch in `slot`: the stage's output lives in the boundary ring, every other
    tensor of the stage in its stash slot."""
    if t == net._out_tensor(z):
        return net.read_act_out(z, slot)
    return net.read_stash(t, slot)


def oracle_step(layers, starts, batch, M, bf16, seed, lr, mu, dx_wanted=False, bias_std=0.05, momentum_std=1e-3, steps=1,
                mutate=None, plain=True):
    """One (or `steps`) mini-batch step(s) by the oracle.

    For the bf16 element type two results are returned: `ref` takes the backward pass's decisions (ReLU mask,
    pooling maximum) in the kernel's storage precision -- every stored activation rounded to bfloat16 once, all
    arithmetic fp64 -- and is what a bf16 implementation is held to element by element; `plain` (plain=True) is the
    unrounded fp64 computation from the same inputs, against which forward quantities are held to the same bar and
    backward quantities are reported (and asserted when the two oracle runs agree on every decision).
    mutate: optional function applied to the freshly made parameter dict (both sides then start from its result)."""
    def one(store):
        params, mom = wl.make_params(layers, seed, bf16=bf16, bias_std=bias_std, momentum_std=momentum_std)
        if mutate is not None:
            mutate(params)
        x, labels, g = wl.make_batch(layers, batch, seed, bf16=bf16)
        p0, m0 = copy.deepcopy(params), copy.deepcopy(mom)
        ref = None
        for _ in range(steps):
            ref = orc.run_schedule(layers, starts, params, mom, x, labels, g, M, lr, mu, orc.LOCKED, keep=True,
                                   input_grad=dx_wanted, store=store)
        return dict(p0=p0, m0=m0, x=x, labels=labels, g=g, ref=ref, params=params, mom=mom)

    o = one(orc.round_bf16 if bf16 else None)
    if bf16 and plain:
        o["plain"] = one(None)
    return o


def oracle_step_async(layers, starts, batch, M, bf16, seed, lr, mu, window, locked, bias_std=0.05, momentum_std=1e-3,
                      store="default", wstore="default"):
    """One pass with an update per micro-batch (oracle.run_schedule_async).  store / wstore: how stored activations and
    the weight copies the layers compute with are rounded (default: to bfloat16 for the bf16 element type)."""
    params, mom = wl.make_params(layers, seed, bf16=bf16, bias_std=bias_std, momentum_std=momentum_std)
    x, labels, g = wl.make_batch(layers, batch, seed, bf16=bf16)
    p0, m0 = copy.deepcopy(params), copy.deepcopy(mom)
    if store == "default":
        store = orc.round_bf16 if bf16 else None
    if wstore == "default":
        wstore = orc.round_bf16 if bf16 else None
    ref = orc.run_schedule_async(layers, starts, params, mom, x, labels, g, M, lr, mu, window=window, locked=locked,
                                 store=store, wstore=wstore)
    return dict(p0=p0, m0=m0, x=x, labels=labels, g=g, ref=ref, params=params, mom=mom)


def compare_async(net, dtype, o, tol=None, floors=None):
    """Loss, last micro-batch's gradient, final weights and momentum against the oracle.
    floors: optional {name: decision-flip noise floor}; a tensor's bound is then tol + 2 * floor."""
    tol = TOL[dtype] if tol is None else tol
    ref = o["ref"]
    errs = {"loss": abs(net.loss_value() - ref["loss"]) / max(abs(ref["loss"]), 1e-30)}
    g, p, v = net.read_grads(), net.read_params(), net.read_momentum()
    for i in o["params"]:
        for k in ("W", "b"):
            if k in o["params"][i]:
                errs["grad%d.%s" % (i, k)] = rel_err(g[i][k], ref["grads"][i][k])
                errs["param%d.%s" % (i, k)] = rel_err(p[i][k], o["params"][i][k])
                errs["mom%d.%s" % (i, k)] = rel_err(v[i][k], o["mom"][i][k])
    bad = {k: e for k, e in errs.items() if not (e <= tol + 2 * (floors or {}).get(k, 0.0))}
    assert not bad, "over the %g bar: %s" % (tol, sorted(bad.items(), key=lambda kv: -kv[1])[:8])
    return errs


def async_floors(layers, starts, batch, M, seed, lr, mu, window, locked, o, realisations=8):
    """Decision-flip noise floor of a bf16 asynchronous-update pass: the largest distance, over a few realisations, between
    the oracle's result and the same oracle arithmetic with accumulation-order noise (flipnoise.order_noise_store) on the
    stored activations and on the weight copies -- per compared tensor, in the harness's error measure."""
    fl = {}
    for r in range(realisations):
        q = oracle_step_async(layers, starts, batch, M, True, seed, lr, mu, window, locked,
                              store=fn.order_noise_store(100 + r), wstore=fn.order_noise_store(200 + r))
        cand = {"loss": abs(q["ref"]["loss"] - o["ref"]["loss"]) / max(abs(o["ref"]["loss"]), 1e-30)}
        for i in o["params"]:
            for k in ("W", "b"):
                if k in o["params"][i]:
                    cand["grad%d.%s" % (i, k)] = rel_err(q["ref"]["grads"][i][k], o["ref"]["grads"][i][k])
                    cand["param%d.%s" % (i, k)] = rel_err(q["params"][i][k], o["params"][i][k])
                    cand["mom%d.%s" % (i, k)] = rel_err(q["mom"][i][k], o["mom"][i][k])
        for k, e in cand.items():
            fl[k] = max(fl.get(k, 0.0), e)
    return fl


def gpu_step(lpm, layers, starts, batch, M, dtype, o, lr, mu, mode, window=2, dx_wanted=False, steps=1):
    import torch
    net = lpm.Net(layers, starts, batch // M, M, dtype, window=window, dx_wanted=dx_wanted,
                  async_update=bool(mode & lpm.ASYNC_UPDATE))
    net.load_params(o["p0"], o["m0"])
    xd = lpm.pack_act(o["x"], dtype)
    ld = torch.from_numpy(o["labels"]).to("cuda:0") if o["labels"] is not None else None
    gd = lpm.pack_act(o["g"], dtype) if o["g"] is not None else None
    for _ in range(steps):
        net.step(xd, ld, gd, lr, mu, mode)
    torch.cuda.synchronize()
    return net


def all_tensors(stash_by_stage, Z, j):
    """{tensor index: value} over all stages for micro-batch j, from the oracle's per-stage stashes."""
    out = {}
    for z in range(Z):
        out.update({t: v for t, v in stash_by_stage[(z, j)].items() if isinstance(t, int)})
    return out


def device_tensors(net, layers, starts, slot):
    out = {}
    for z in range(len(starts) - 1):
        for t in range(starts[z], starts[z + 1]):
            if layers[t]["kind"] != "softmax_ce":
                out[t] = read_tensor(net, z, t, slot)
    return out


def compare(net, layers, starts, M, dtype, o, dx_wanted=False, window=2, report=None, backward=True):
    """Compares loss, gradients, updated weights, momentum, and the last micro-batch's activations
    and boundary gradients.  Returns {name: error}; asserts every error is under the bar.
    backward=False restricts the comparison to the forward quantities (activations and loss).

    bf16: the element-wise bar is applied against the oracle run that decides in storage precision (o["ref"]); the
    count of decisions on which the device's stored activations differ from that run's is printed, and a failure
    names it.  Against the unrounded fp64 run (o["plain"]) the forward quantities must meet the same bar; the
    backward quantities are printed, and must meet it too whenever the two oracle runs agree on every decision."""
    tol = TOL[dtype]
    ref = o["ref"]
    errs = {}
    if o["labels"] is not None:
        errs["loss"] = abs(net.loss_value() - ref["loss"]) / max(abs(ref["loss"]), 1e-30)
    g, p, v = net.read_grads(), net.read_params(), net.read_momentum()
    for i in (o["params"] if backward else []):
        for k in ("W", "b"):
            if k in o["params"][i]:
                errs["grad%d.%s" % (i, k)] = rel_err(g[i][k], ref["grads"][i][k])
                errs["param%d.%s" % (i, k)] = rel_err(p[i][k], o["params"][i][k])
                errs["mom%d.%s" % (i, k)] = rel_err(v[i][k], o["mom"][i][k])
        if "s" in o["params"][i]:
            errs["scale%d" % i] = rel_err(p[i]["s"], o["params"][i]["s"])
    Z = len(starts) - 1
    j = M - 1
    slot = j % window
    dev = device_tensors(net, layers, starts, slot)
    want_t = all_tensors(ref["stash"], Z, j)
    for t, got in dev.items():
        errs["act%d" % t] = rel_err(got, want_t[t])
    gins = {}
    for z in range(Z):
        if backward and (z > 0 or dx_wanted):
            gins[z] = net.read_grad_in(z, slot)
            want = ref["gin"][(z, j)]
            if z > 0 and net.schedule.cut_fused(z):
                # the cut hands down the previous stage's pre-activation gradient: ReLU derivative of the stage input applied
                want = want * (ref["stash"][(z - 1, j)][starts[z] - 1] > 0)
            errs["gin%d" % z] = rel_err(gins[z], want)
    flips = None
    if dtype == 1:
        dev[-1] = want_t[-1] = o["x"][j * (len(o["x"]) // M):(j + 1) * (len(o["x"]) // M)]
        flips = fn.decision_disagreements(layers, 0, len(layers), dev, want_t)
        print("decisions differing from the storage-precision oracle run (relu, of, pool, of):", flips, flush=True)
    bad = {k: e for k, e in errs.items() if not (e <= tol)}
    if report is not None:
        report.update(errs)
    assert not bad, "over the %g bar (decision disagreements %s): %s" % (tol, flips, sorted(bad.items(), key=lambda kv: -kv[1])[:8])
    if dtype == 1 and "plain" in o:
        # against the unrounded fp64 computation
        pl = o["plain"]
        pr = pl["ref"]
        plain_t = all_tensors(pr["stash"], Z, j)
        plain_t[-1] = dev[-1]
        perr = {}
        if o["labels"] is not None:
            perr["loss"] = abs(net.loss_value() - pr["loss"]) / max(abs(pr["loss"]), 1e-30)
        for t, got in dev.items():
            if t >= 0:
                perr["act%d" % t] = rel_err(got, plain_t[t])
        # (a layer that exponentiates -- attention -- amplifies the storage rounding of its input: the forward bound is the bar
        #  plus twice the distance between the two oracle runs at that tensor, which is zero to a fraction of the bar elsewhere)
        ffloor = {"act%d" % t: rel_err(want_t[t], plain_t[t]) for t in dev if t >= 0}
        fwd_bad = {k: e for k, e in perr.items() if not (e <= tol + 2 * ffloor.get(k, 0.0))}
        berr = {}
        for i in (pl["params"] if backward else []):
            for k in ("W", "b"):
                if k in pl["params"][i]:
                    berr["grad%d.%s" % (i, k)] = rel_err(g[i][k], pr["grads"][i][k])
                    berr["param%d.%s" % (i, k)] = rel_err(p[i][k], pl["params"][i][k])
        for z, got in gins.items():
            want = pr["gin"][(z, j)]
            if z > 0 and net.schedule.cut_fused(z):
                want = want * (pr["stash"][(z - 1, j)][starts[z] - 1] > 0)
            berr["gin%d" % z] = rel_err(got, want)
        oracle_flips = fn.decision_disagreements(layers, 0, len(layers), plain_t, want_t)
        worst_f = max(perr.values()) if perr else 0.0
        worst_b = max(berr.values()) if berr else 0.0
        print("against the unrounded fp64 oracle: worst forward error %.4g, worst backward error %.4g; the two oracle runs "
              "differ on decisions (relu, of, pool, of) %s" % (worst_f, worst_b, oracle_flips), flush=True)
        if report is not None:
            report.update({"plain." + k: e for k, e in list(perr.items()) + list(berr.items())})
        assert not fwd_bad, "forward quantities over the %g bar against the unrounded oracle: %s" % (tol, sorted(fwd_bad.items(), key=lambda kv: -kv[1])[:8])
        if oracle_flips[0] == 0 and oracle_flips[2] == 0:
            bbad = {k: e for k, e in berr.items() if not (e <= tol)}
            assert not bbad, "backward quantities over the %g bar against the unrounded oracle (no decision depends on the storage precision here): %s" % (tol, sorted(bbad.items(), key=lambda kv: -kv[1])[:8])
    return errs


def l2_err(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm((got - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-30))


def stage_backward_isolated(lpm, layers, starts, m, batch_total, dtype, seed, dx_wanted=False, bias_std=0.05,
                            grad_std=1e-3, report=None, check_forward=False):
    """B_{z,j} of every stage on its own, at full micro-batch size, from a forward state prepared by the oracle.

    The backward pass takes two integer decisions on stored activations (ReLU mask, position of a pooling
    maximum).  In a deep bf16 network an end-to-end comparison lets last-bit differences of the forward
    pass flip a few of them, which moves gradients by far more than any arithmetic tolerance, on either
    side.  Here both sides take every decision on identical values: the oracle runs the forward pass
    (storing bf16-rounded activations for the bf16 element type), its stored tensors are written into
    the device buffers, and only lpm_stage_backward runs on the device.  Data flows oracle -> device only.
    check_forward=True first runs the device's own forward pass on the same micro-batch and compares every
    activation and the loss with the oracle's forward pass.
    """
    bf16 = dtype == 1
    q = orc.round_bf16 if bf16 else (lambda a: a)
    store = orc.round_bf16 if bf16 else None
    params, _ = wl.make_params(layers, seed, bf16=bf16, bias_std=bias_std)
    x, labels, g_up = wl.make_batch(layers, m, seed, bf16=bf16, grad_std=grad_std)
    Z = len(starts) - 1
    stashes, a, loss_ref = [], x, None
    for z in range(Z):
        last = z == Z - 1
        print("oracle forward stage", z, flush=True)
        a, stash, lz = orc.stage_forward(layers, starts[z], starts[z + 1], params, a,
                                         labels if (last and labels is not None) else None, batch_total, store)
        loss_ref = lz if lz is not None else loss_ref
        if "dlogits" in stash:
            stash["dlogits"] = q(stash["dlogits"])
        stashes.append(stash)
    net = lpm.Net(layers, starts, m, 1, dtype, dx_wanted=dx_wanted)
    net.load_params(params, None)
    xd = lpm.pack_act(x, dtype)
    tol = TOL[dtype]
    errs = {}
    if check_forward:
        # the device's own forward pass (one LOCKED step with learning rate 0) against the oracle's
        import torch
        ld = torch.from_numpy(labels).to("cuda:0") if labels is not None else None
        gd = lpm.pack_act(g_up, dtype) if g_up is not None else None
        print("device forward", flush=True)
        net.step(xd, ld, gd, 0.0, 0.0, 0)
        torch.cuda.synchronize()
        if labels is not None:
            errs["loss"] = abs(net.loss_value() * (m / batch_total) - loss_ref) / max(abs(loss_ref), 1e-30)
        for z in range(Z):
            for t in range(starts[z], starts[z + 1]):
                if layers[t]["kind"] == "softmax_ce":
                    continue
                errs["act%d" % t] = rel_err(read_tensor(net, z, t, 0), stashes[z][t])
    g_out = g_up
    for z in range(Z - 1, -1, -1):
        s0, s1 = starts[z], starts[z + 1]
        loss_stage = layers[s1 - 1]["kind"] == "softmax_ce"
        dy = None if loss_stage else q(g_out)
        grads = orc.zero_grads(layers, params)
        want = z > 0 or dx_wanted
        g_out = orc.stage_backward(layers, s0, s1, params, stashes[z], dy, grads, input_grad=want)
        # device: prepared forward state in slot 0
        for t in range(s0, s1 - 1):
            if layers[t]["kind"] == "softmax_ce" or (loss_stage and t == s1 - 2):
                continue
            net.write_stash(t, 0, stashes[z][t])
        t_out = s1 - 2 if loss_stage else s1 - 1
        net.write_act_out(z, 0, stashes[z][t_out])
        if loss_stage:
            net.write_stash("dlogits", 0, stashes[z]["dlogits"])
        if z > 0:
            net.write_act_out(z - 1, 0, stashes[z][s0 - 1])
        b = net.bufs[z]
        xin = xd if z == 0 else net.bufs[z - 1]["act_out"][0]
        dyd = None if loss_stage else lpm.pack_act(dy, dtype)
        print("isolated backward stage", z, "layers", s0, s1, flush=True)
        net.stages[z].backward(xin, b["act_out"][0], dyd, b["grad_in"][0] if want else None, b["params"], b["lowp"],
                               b["stash"][0], b["grads"], 0, b["bwd_ws"], None)
        net.torch.cuda.synchronize()
        gg = net.read_grads()
        for i in range(s0, s1):
            for k in ("W", "b"):
                if i in grads and k in grads[i]:
                    errs["z%d.grad%d.%s" % (z, i, k)] = rel_err(gg[i][k], grads[i][k])
        if want:
            errs["z%d.dx" % z] = rel_err(net.read_grad_in(z), g_out)
    if report is not None:
        report.update(errs)
    bad = {k: e for k, e in errs.items() if not (e <= tol)}
    assert not bad, "over the %g bar: %s" % (tol, sorted(bad.items(), key=lambda kv: -kv[1])[:8])
    return errs

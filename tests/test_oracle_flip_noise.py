"""The decision-flip noise floor of bf16 training steps, measured on the oracle alone (no GPU).

Two runs of the SAME fp64 arithmetic that differ only in how stored activations are rounded are two valid results
of a bf16 implementation.  These tests pin how far apart such results are: forward quantities and the gradients
behind which no decision lies agree to well under the 2e-2 bar; gradients of early layers of a deep ReLU / pooling
network do not, because a few decisions flip.  The GPU tests take their end-to-end bounds from this measurement
(tests/golden/make_full_step.py stores the floor of every full-size workload)."""
import numpy as np

import workloads as wl
from oracle import lpm_oracle as orc
import flipnoise as fn


def _run(layers, batch, M, seed, store):
    params, mom = wl.make_params(layers, seed, bf16=True, bias_std=0.05)
    x, labels, g = wl.make_batch(layers, batch, seed, bf16=True)
    ref = orc.run_schedule(layers, [0, len(layers)], params, mom, x, labels, g, M, 0.0, 0.0, orc.LOCKED, store=store, keep=True)
    ref["x"] = x
    return ref


def _tensors(ref, M):
    t = {k: v for k, v in ref["stash"][(0, M - 1)].items() if isinstance(k, int)}
    return t


def test_storage_rounding_flips_decisions_on_a_small_network():
    """tiny_vgg, 8 images: rounding the stored activations to bf16 (nothing else) changes a handful of the 6560
    decisions, and the first layers' weight gradients move by more than the 2e-2 bar, while every activation stays
    within it."""
    L = wl.tiny_vgg()
    A, B = _run(L, 8, 2, 11, None), _run(L, 8, 2, 11, orc.round_bf16)
    rf, rt, pf, pt = fn.decision_disagreements(L, 0, len(L), _tensors(A, 2), _tensors(B, 2))
    assert (rt, pt) == (5728, 832)
    assert 1 <= rf + pf <= 20
    acts = max(fn.inf_err(_tensors(B, 2)[t], _tensors(A, 2)[t]) for t in _tensors(A, 2) if t >= 0)
    assert acts <= 1e-2
    errs = {i: fn.inf_err(B["grads"][i]["W"], A["grads"][i]["W"]) for i in A["grads"]}
    first, head = min(errs), max(errs)
    assert errs[first] > 2e-2           # a flipped decision moved whole gradient elements of the first layer ...
    assert errs[head] < 5e-3            # ... but nothing behind the head, whose gradient sees only rounding
    assert abs(B["loss"] - A["loss"]) <= 2e-3 * abs(A["loss"])


def test_accumulation_order_noise_floor_vgg16_cifar():
    """One micro-batch (4 images) of the VGG-16/CIFAR workload: storing bf16(value * (1 + r)), |r| <= 4e-6 -- a float32
    sum taken in another order -- instead of bf16(value) flips a few decisions in ten thousand; the gradients of the
    convolutions then differ by several per cent of their largest element (first layer: over 5 %), in the 2-norm
    too.  Activations and the loss agree to a fraction of the bar.  No implementation can meet 2e-2 end to end on these
    gradients; they are compared stage by stage from a common forward state, and end to end against this floor."""
    L = wl.vgg16_cifar()
    B, C = _run(L, 4, 1, 11, orc.round_bf16), _run(L, 4, 1, 11, fn.order_noise_store(1))
    tb, tc = _tensors(B, 1), _tensors(C, 1)
    rf, rt, pf, pt = fn.decision_disagreements(L, 0, len(L), tb, tc)
    print("flips", rf, rt, pf, pt)
    assert 1e-5 < rf / rt < 2e-3 and 1e-5 < pf / pt < 1e-2
    assert max(fn.inf_err(tc[t], tb[t]) for t in tb if t >= 0) <= 1e-2
    assert abs(C["loss"] - B["loss"]) <= 2e-3 * abs(B["loss"])
    convs = [i for i in B["grads"] if L[i]["kind"] == "conv"]
    fcs = [i for i in B["grads"] if L[i]["kind"] == "fc"]
    inf = {i: fn.inf_err(C["grads"][i]["W"], B["grads"][i]["W"]) for i in B["grads"]}
    l2 = {i: fn.l2_err(C["grads"][i]["W"], B["grads"][i]["W"]) for i in B["grads"]}
    print("inf", {i: round(e, 4) for i, e in inf.items()})
    print("l2 ", {i: round(e, 4) for i, e in l2.items()})
    assert inf[convs[0]] > 5e-2 and l2[convs[0]] > 5e-2
    assert sum(inf[i] > 2e-2 for i in convs) >= len(convs) // 2
    assert inf[fcs[-1]] <= 2e-2          # the classifier's weight gradient: no decision behind it but its input's mask


def test_pooling_gradient_window_sums_do_not_depend_on_the_route():
    """Whichever element of a 2x2 window receives the pooling gradient, the window's sum is the output gradient: the
    quantity on which pooling-backward results can be compared when two sides disagree about a maximum."""
    r = np.random.default_rng(3)
    x = r.normal(size=(2, 3, 6, 8))
    dy = r.normal(size=(2, 3, 3, 4))
    y = x.copy()
    y[0, 0, 0, 0] = y[0, 0, 0, 1] = y[0, 0, 1, 1] = 7.0          # a tie: first maximum wins
    x2 = x.copy()
    x2[:, :, ::2, ::2] += 5.0                                      # every maximum moves to the window's first element
    for inp in (x, y, x2):
        dx = orc.maxpool2_bwd(inp, dy)
        np.testing.assert_allclose(fn.window_sums(dx), dy, rtol=0, atol=0)
        assert (np.count_nonzero(dx.reshape(2, 3, 3, 2, 4, 2), axis=(3, 5)) <= 1).all()
    assert (orc.maxpool2_bwd(y, dy)[0, 0, :2, :2] != 0).sum() == 1 and orc.maxpool2_bwd(y, dy)[0, 0, 0, 0] == dy[0, 0, 0, 0]

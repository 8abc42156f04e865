"""Pins for the oracle's micro-batching, schedules and update placement.

The overlapped schedule with gradient accumulation and one update per mini-batch reaches exactly the
plain mini-batch result, so every schedule is pinned to plain backpropagation on the whole batch."""
import copy

import numpy as np
import pytest

import workloads as wl
from oracle import lpm_oracle as orc


def _setup(net="tiny_lenet", batch=8, seed=3):
    layers = getattr(wl, net)()
    params, mom = wl.make_params(layers, seed=seed, bias_std=0.1, momentum_std=1e-2)
    x, labels, _ = wl.make_batch(layers, batch, seed=seed)
    return layers, params, mom, x, labels


def _plain_backprop(layers, params, mom, x, labels, lr, mu):
    """Whole network, whole batch, one forward, one backward, one update: no stages, no micro-batches."""
    L = len(layers)
    _, stash, loss = orc.stage_forward(layers, 0, L, params, x, labels, x.shape[0])
    grads = orc.zero_grads(layers, params)
    orc.stage_backward(layers, 0, L, params, stash, None, grads)
    orc.sgd_momentum(params, grads, mom, lr, mu)
    return loss, grads


def _starts(layers, Z):
    allowed = [i + 1 for i, l in enumerate(layers[:-1]) if l["cut_after"]]
    return [0] + allowed[:Z - 1] + [len(layers)]


def test_locked_single_microbatch_is_plain_backprop_exactly():
    layers, params, mom, x, labels = _setup()
    p2, m2 = copy.deepcopy(params), copy.deepcopy(mom)
    loss_ref, g_ref = _plain_backprop(layers, params, mom, x, labels, 0.01, 0.9)
    for Z in (1, 2, 3):
        p, m = copy.deepcopy(p2), copy.deepcopy(m2)
        out = orc.run_schedule(layers, _starts(layers, Z), p, m, x, labels, None, 1, 0.01, 0.9, orc.LOCKED)
        assert out["loss"] == loss_ref
        for i in params:
            for k in ("W", "b"):
                np.testing.assert_array_equal(out["grads"][i][k], g_ref[i][k])     # same op sequence: bit equal
                np.testing.assert_array_equal(p[i][k], params[i][k])
                np.testing.assert_array_equal(m[i][k], mom[i][k])


@pytest.mark.parametrize("net", ["tiny_lenet", "tiny_resnet"])
def test_microbatch_gradients_sum_to_full_batch(net):
    layers, params, mom, x, labels = _setup(net)
    p2, m2 = copy.deepcopy(params), copy.deepcopy(mom)
    loss_ref, g_ref = _plain_backprop(layers, params, mom, x, labels, 0.01, 0.9)
    for M in (2, 4, 8):
        p, m = copy.deepcopy(p2), copy.deepcopy(m2)
        out = orc.run_schedule(layers, _starts(layers, 2), p, m, x, labels, None, M, 0.01, 0.9, orc.LOCKED)
        assert abs(out["loss"] - loss_ref) < 1e-12
        for i in params:
            for k in ("W", "b"):
                np.testing.assert_allclose(out["grads"][i][k], g_ref[i][k], rtol=0, atol=1e-12)
                np.testing.assert_allclose(p[i][k], params[i][k], rtol=0, atol=1e-13)


@pytest.mark.parametrize("net,Z,M,window", [("tiny_lenet", 3, 4, 2), ("tiny_resnet", 2, 8, 2),
                                            ("tiny_lenet", 2, 4, 1), ("tiny_lenet", 3, 8, 3)])
def test_overlapped_equals_locked_for_random_legal_orders(net, Z, M, window):
    layers, params, mom, x, labels = _setup(net)
    starts = _starts(layers, Z)
    pl, ml = copy.deepcopy(params), copy.deepcopy(mom)
    ref = orc.run_schedule(layers, starts, pl, ml, x, labels, None, M, 0.02, 0.9, orc.LOCKED)
    r = np.random.default_rng(5)
    seen = set()
    for trial in range(6):
        p, m = copy.deepcopy(params), copy.deepcopy(mom)
        out = orc.run_schedule(layers, starts, p, m, x, labels, None, M, 0.02, 0.9, orc.OVERLAPPED,
                               window=window, order_rng=r if trial else None)
        seen.add(tuple(out["order"]))
        # accumulation order per stage is fixed by B_{z,j} after B_{z,j-1}: results are bit equal
        assert out["loss"] == ref["loss"]
        for i in params:
            for k in ("W", "b"):
                np.testing.assert_array_equal(out["grads"][i][k], ref["grads"][i][k])
                np.testing.assert_array_equal(p[i][k], pl[i][k])
    assert len(seen) > 1 or window == 1


def test_schedule_dependency_structure():
    Z, M = 4, 8
    d = orc.schedule_ops(Z, M, orc.OVERLAPPED, window=2)
    assert len(d) == 2 * Z * M + Z
    # the statement of the parallel schedule: B_{0,0} finishes before F_{0,2} in stage 0, likewise in stages 1..3
    for z in range(Z):
        for j in range(M - 2):
            assert ("B", z, j) in d[("F", z, j + 2)]
    # the backward of a micro-batch starts right after its own forward finishes
    assert d[("B", Z - 1, 0)] == {("F", Z - 1, 0)}
    # forward of micro-batch j+1 does not wait for backward of micro-batch j (update locking broken)
    assert all(op[0] != "B" for op in d[("F", 0, 1)])
    # every legal order keeps at most 2 micro-batches in flight per stage
    r = np.random.default_rng(0)
    for _ in range(20):
        order = orc.legal_order(d, r)
        live = [0] * Z
        for op in order:
            if op[0] == "F":
                live[op[1]] += 1
                assert live[op[1]] <= 2
            elif op[0] == "B":
                live[op[1]] -= 1
    # locked: a single chain in the order F_0..F_{Z-1}, B_{Z-1}..B_0 per micro-batch, then the updates
    dl = orc.schedule_ops(2, 2, orc.LOCKED)
    assert orc.legal_order(dl) != [] and len({len(v) for v in dl.values()}) == 2
    chain = orc.legal_order(dl, np.random.default_rng(1))
    assert chain == [("F", 0, 0), ("F", 1, 0), ("B", 1, 0), ("B", 0, 0),
                     ("F", 0, 1), ("F", 1, 1), ("B", 1, 1), ("B", 0, 1), ("U", 0), ("U", 1)]


def test_interpreter_rejects_broken_orders():
    """The interpreter's assertions fire when an order breaks the window or a dependency."""
    layers, params, mom, x, labels = _setup()
    starts = _starts(layers, 2)
    d = orc.schedule_ops(2, 4, orc.OVERLAPPED, 2)
    good = orc.legal_order(d)
    bad = [op for op in good if op != ("F", 0, 2)]
    bad.insert(2, ("F", 0, 2))          # third forward in stage 0 before B_{0,0}
    orig = orc.legal_order
    try:
        orc.legal_order = lambda deps, rng=None: bad
        with pytest.raises(AssertionError):
            orc.run_schedule(layers, starts, params, mom, x, labels, None, 4, 0.01, 0.9, orc.OVERLAPPED)
    finally:
        orc.legal_order = orig


def test_two_steps_with_momentum_match_plain():
    layers, params, mom, x, labels = _setup(batch=8)
    pr, mr = copy.deepcopy(params), copy.deepcopy(mom)
    for _ in range(2):
        _plain_backprop(layers, pr, mr, x, labels, 0.05, 0.9)
        orc.run_schedule(layers, _starts(layers, 3), params, mom, x, labels, None, 4, 0.05, 0.9, orc.OVERLAPPED)
    for i in params:
        for k in ("W", "b"):
            np.testing.assert_allclose(params[i][k], pr[i][k], rtol=0, atol=1e-12)


# ---------------------------------------------------------------- asynchronous (per-micro-batch) update

def _sequential_sgd(layers, starts, params, mom, x, labels, M, lr, mu):
    """Per-micro-batch SGD written with the synchronous interpreter: M one-micro-batch steps in a row."""
    m = x.shape[0] // M
    loss = 0.0
    for j in range(M):
        out = orc.run_schedule(layers, starts, params, mom, x[j * m:(j + 1) * m], labels[j * m:(j + 1) * m], None, 1,
                               lr, mu, orc.LOCKED)
        loss += out["loss"]
    return loss, out["grads"]


@pytest.mark.parametrize("net", ["tiny_lenet", "tiny_resnet"])
def test_async_update_without_overlap_is_sequential_sgd(net):
    """Locked, or overlapped with window 1: every forward pass sees all earlier updates."""
    layers, params, mom, x, labels = _setup(net)
    starts = _starts(layers, 2)
    p_ref, m_ref = copy.deepcopy(params), copy.deepcopy(mom)
    loss_ref, g_ref = _sequential_sgd(layers, starts, p_ref, m_ref, x, labels, 4, 0.05, 0.9)
    for kw in (dict(locked=True), dict(window=1), dict(window=1, order_rng=np.random.default_rng(2))):
        p, m = copy.deepcopy(params), copy.deepcopy(mom)
        out = orc.run_schedule_async(layers, starts, p, m, x, labels, None, 4, 0.05, 0.9, **kw)
        assert abs(out["loss"] - loss_ref) < 1e-12
        for i in p:
            for k in ("W", "b"):
                np.testing.assert_allclose(p[i][k], p_ref[i][k], rtol=0, atol=1e-13)
                np.testing.assert_allclose(m[i][k], m_ref[i][k], rtol=0, atol=1e-13)
                np.testing.assert_allclose(out["grads"][i][k], g_ref[i][k], rtol=0, atol=1e-13)


def test_async_update_single_microbatch_is_the_synchronous_step():
    layers, params, mom, x, labels = _setup()
    starts = _starts(layers, 3)
    p1, m1, p2, m2 = copy.deepcopy(params), copy.deepcopy(mom), copy.deepcopy(params), copy.deepcopy(mom)
    a = orc.run_schedule(layers, starts, p1, m1, x, labels, None, 1, 0.05, 0.9, orc.OVERLAPPED)
    b = orc.run_schedule_async(layers, starts, p2, m2, x, labels, None, 1, 0.05, 0.9, window=2)
    assert a["loss"] == b["loss"]
    for i in p1:
        for k in ("W", "b"):
            np.testing.assert_array_equal(p1[i][k], p2[i][k])


def test_async_update_result_is_order_independent_and_differs_from_sequential():
    layers, params, mom, x, labels = _setup("tiny_resnet")
    starts = _starts(layers, 2)
    ref = None
    for seed in (None, 0, 1, 2):
        p, m = copy.deepcopy(params), copy.deepcopy(mom)
        rng = None if seed is None else np.random.default_rng(seed)
        out = orc.run_schedule_async(layers, starts, p, m, x, labels, None, 4, 0.05, 0.9, window=2, order_rng=rng)
        if ref is None:
            ref = (p, m, out["loss"])
        else:
            assert out["loss"] == ref[2]
            for i in p:
                for k in ("W", "b"):
                    np.testing.assert_array_equal(p[i][k], ref[0][i][k])
    p_seq, m_seq = copy.deepcopy(params), copy.deepcopy(mom)
    _sequential_sgd(layers, starts, p_seq, m_seq, x, labels, 4, 0.05, 0.9)
    assert max(np.abs(ref[0][i]["W"] - p_seq[i]["W"]).max() for i in ref[0]) > 1e-6     # the delay is visible


def test_async_update_delay_by_hand():
    """Two FC layers, two micro-batches, window 2, no momentum, written out with matrix products:
    micro-batch 1's forward pass reads the initial weights (its update overlaps micro-batch 0's backward
    pass), its data gradient reads the weights after the first update."""
    b = wl.configs._Builder(6, 1, 1)
    b.fc(5); b.fc(4, relu=False); b.loss()
    layers = b.finish()
    params, mom = wl.make_params(layers, seed=9, bias_std=0.1, momentum_std=0.0)
    x, labels, _ = wl.make_batch(layers, 6, seed=9)
    lr, m = 0.1, 3
    W1, b1, W2, b2 = (params[0]["W"].reshape(5, 6).copy(), params[0]["b"].copy(), params[1]["W"].reshape(4, 5).copy(),
                      params[1]["b"].copy())

    def fwd(xb, W1, b1, W2, b2):
        h = np.maximum(xb @ W1.T + b1, 0.0)
        return h, h @ W2.T + b2

    def dlogits(z, lab):
        e = np.exp(z - z.max(axis=1, keepdims=True))
        p = e / e.sum(axis=1, keepdims=True)
        p[np.arange(len(lab)), lab] -= 1.0
        return p / len(lab)

    xb = [x[j * m:(j + 1) * m].reshape(m, 6) for j in range(2)]
    lb = [labels[j * m:(j + 1) * m] for j in range(2)]
    # micro-batch 0: everything at version 0
    h0, z0 = fwd(xb[0], W1, b1, W2, b2)
    d0 = dlogits(z0, lb[0])
    dh0 = (d0 @ W2) * (h0 > 0)
    V1 = dict(W1=W1 - lr * dh0.T @ xb[0], b1=b1 - lr * dh0.sum(0), W2=W2 - lr * d0.T @ h0, b2=b2 - lr * d0.sum(0))
    # micro-batch 1: forward at version 0, data gradient through W2 of version 1, update applied to version 1
    h1, z1 = fwd(xb[1], W1, b1, W2, b2)
    d1 = dlogits(z1, lb[1])
    dh1 = (d1 @ V1["W2"]) * (h1 > 0)
    V2 = dict(W1=V1["W1"] - lr * dh1.T @ xb[1], b1=V1["b1"] - lr * dh1.sum(0), W2=V1["W2"] - lr * d1.T @ h1,
              b2=V1["b2"] - lr * d1.sum(0))
    orc.run_schedule_async(layers, [0, 1, 3], params, mom, x, labels, None, 2, lr, 0.0, window=2)
    np.testing.assert_allclose(params[0]["W"].reshape(5, 6), V2["W1"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(params[0]["b"], V2["b1"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(params[1]["W"].reshape(4, 5), V2["W2"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(params[1]["b"], V2["b2"], rtol=0, atol=1e-14)

"""Pins for the oracle's layer arithmetic: hand-worked values, library routines on special cases,
adjoint identities and finite differences.  None of these re-types the oracle's own loops."""
import os

import numpy as np
import pytest
import scipy.signal
import scipy.special

import workloads as wl
from oracle import lpm_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _conv_layer(cin, cout, k, s, p, h, w):
    return dict(kind="conv", cin=cin, cout=cout, kh=k[0], kw=k[1], stride=s, pad=p, h_in=h, w_in=w,
                relu=False, bias=False, scale=False, src=-1, add_src=None, cut_after=False)


def _read_golden():
    cases, cur = {}, None
    for line in open(os.path.join(GOLD, "conv_hand_case.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        t = line.split()
        if t[0] in ("case", "points"):
            cur = (t[0], t[1])
            cases[cur] = []
        else:
            cases[cur].append([float(v) for v in t])
    return cases


def test_conv_hand_worked_case():
    g = _read_golden()
    x = (np.arange(25, dtype=np.float64) + 1).reshape(1, 1, 5, 5)
    W = np.array([[1, 0, -1], [2, 0, -2], [1, 0, -1]], dtype=np.float64).reshape(1, 1, 3, 3)
    z = orc.conv_fwd(x, W, _conv_layer(1, 1, (3, 3), 1, 0, 5, 5))
    np.testing.assert_array_equal(z[0, 0], np.array(g[("case", "s1p0")]))
    z = orc.conv_fwd(x, W, _conv_layer(1, 1, (3, 3), 1, 1, 5, 5))
    assert z.shape == (1, 1, 5, 5)
    for h, w, v in g[("points", "s1p1")]:
        assert z[0, 0, int(h), int(w)] == v
    z = orc.conv_fwd(x, W, _conv_layer(1, 1, (3, 3), 2, 1, 5, 5))
    assert z.shape == (1, 1, 3, 3)
    for h, w, v in g[("points", "s2p1")]:
        assert z[0, 0, int(h), int(w)] == v


@pytest.mark.parametrize("cin,cout,k,s,p,h,w", [(3, 4, (3, 3), 1, 1, 7, 6), (2, 3, (5, 5), 1, 0, 9, 9),
                                                (3, 2, (3, 3), 2, 1, 8, 8), (2, 2, (1, 1), 2, 0, 6, 6),
                                                (2, 3, (2, 2), 1, 1, 5, 4), (3, 2, (3, 3), 2, 1, 7, 5)])
def test_conv_matches_scipy_correlate(cin, cout, k, s, p, h, w):
    """Cross-correlation of the zero-padded image (scipy.signal.correlate2d, 'valid'), summed over
    input channels, sampled at the stride."""
    r = np.random.default_rng(1)
    x = r.standard_normal((2, cin, h, w))
    W = r.standard_normal((cout, cin) + k)
    z = orc.conv_fwd(x, W, _conv_layer(cin, cout, k, s, p, h, w))
    xp = np.pad(x, ((0, 0), (0, 0), (p, p), (p, p)))
    for n in range(2):
        for co in range(cout):
            ref = sum(scipy.signal.correlate2d(xp[n, ci], W[co, ci], mode="valid") for ci in range(cin))
            np.testing.assert_allclose(z[n, co], ref[::s, ::s], rtol=1e-12, atol=1e-12)


def test_conv_special_cases_reduce_to_matmul():
    r = np.random.default_rng(2)
    x = r.standard_normal((3, 5, 4, 6))
    # 1x1 conv == the same matrix applied at every pixel
    W = r.standard_normal((7, 5, 1, 1))
    z = orc.conv_fwd(x, W, _conv_layer(5, 7, (1, 1), 1, 0, 4, 6))
    np.testing.assert_allclose(z, np.einsum("oc,nchw->nohw", W[:, :, 0, 0], x), rtol=1e-12, atol=1e-12)
    # kernel covering the whole input == fully connected on the (C,H,W)-flattened input
    W = r.standard_normal((7, 5, 4, 6))
    fc = dict(_conv_layer(5, 7, (4, 6), 1, 0, 4, 6), kind="fc")
    z = orc.conv_fwd(x, W, fc)
    np.testing.assert_allclose(z.reshape(3, 7), x.reshape(3, -1) @ W.reshape(7, -1).T, rtol=1e-12, atol=1e-12)
    # identity kernel returns the input
    W = np.zeros((5, 5, 3, 3))
    W[np.arange(5), np.arange(5), 1, 1] = 1.0
    np.testing.assert_array_equal(orc.conv_fwd(x, W, _conv_layer(5, 5, (3, 3), 1, 1, 4, 6)), x)
    # a one-hot kernel tap shifts the image: z[h,w] = x[h+kh-1, w+kw-1]
    W = np.zeros((1, 1, 3, 3)); W[0, 0, 0, 2] = 1.0
    z = orc.conv_fwd(x[:, :1], W, _conv_layer(1, 1, (3, 3), 1, 1, 4, 6))
    np.testing.assert_array_equal(z[:, :, 1:, :-1], x[:, :1, :-1, 1:])
    assert np.all(z[:, :, 0, :] == 0) and np.all(z[:, :, :, -1] == 0)


@pytest.mark.parametrize("cin,cout,k,s,p,h,w", [(3, 4, (3, 3), 1, 1, 6, 5), (2, 3, (3, 3), 2, 1, 8, 8),
                                                (2, 3, (1, 1), 2, 0, 6, 6), (3, 2, (5, 5), 1, 0, 7, 7),
                                                (3, 2, (3, 3), 2, 1, 7, 5)])
def test_conv_backward_are_adjoints(cin, cout, k, s, p, h, w):
    """conv is bilinear: <conv(x,W),dz> = <x, bwd_data(dz,W)> = <W, bwd_weight(x,dz)> exactly (up to rounding).
    A wrong index, sign or transposition in either backward routine breaks one of the equalities."""
    r = np.random.default_rng(3)
    l = _conv_layer(cin, cout, k, s, p, h, w)
    x = r.standard_normal((2, cin, h, w)); W = r.standard_normal((cout, cin) + k)
    z = orc.conv_fwd(x, W, l)
    dz = r.standard_normal(z.shape)
    lhs = float((z * dz).sum())
    assert abs(lhs - float((x * orc.conv_bwd_data(dz, W, l)).sum())) < 1e-10 * max(1, abs(lhs))
    assert abs(lhs - float((W * orc.conv_bwd_weight(x, dz, l)).sum())) < 1e-10 * max(1, abs(lhs))


def test_conv_backward_data_one_hot():
    """dx for a one-hot dz is the kernel stamped at the strided position (written out by hand)."""
    l = _conv_layer(1, 1, (3, 3), 2, 1, 6, 6)
    W = np.arange(1, 10, dtype=np.float64).reshape(1, 1, 3, 3)
    dz = np.zeros((1, 1, 3, 3)); dz[0, 0, 1, 2] = 2.0          # output (1,2) <- input rows 1..3, cols 3..5
    dx = orc.conv_bwd_data(dz, W, l)
    ref = np.zeros((6, 6)); ref[1:4, 3:6] = 2.0 * W[0, 0]
    np.testing.assert_array_equal(dx[0, 0], ref)
    dz[:] = 0; dz[0, 0, 0, 0] = 1.0                              # corner: rows -1..1 -> only kernel rows 1..2 land
    dx = orc.conv_bwd_data(dz, W, l)
    ref = np.zeros((6, 6)); ref[0:2, 0:2] = W[0, 0, 1:, 1:]
    np.testing.assert_array_equal(dx[0, 0], ref)


def test_maxpool_hand_case_and_tie():
    x = np.array([[1, 5, 2, 2],
                  [3, 4, 2, 2],
                  [0, 0, 9, 7],
                  [0, -1, 8, 9]], dtype=np.float64).reshape(1, 1, 4, 4)
    y = orc.maxpool2_fwd(x)
    np.testing.assert_array_equal(y[0, 0], [[5, 2], [0, 9]])
    dy = np.array([[10, 20], [30, 40]], dtype=np.float64).reshape(1, 1, 2, 2)
    dx = orc.maxpool2_bwd(x, dy)
    ref = np.zeros((4, 4))
    ref[0, 1] = 10      # unique max
    ref[0, 2] = 20      # four-way tie -> first in row-major window order
    ref[2, 0] = 30      # tie of zeros -> first
    ref[2, 2] = 40      # 9 appears at (2,2) and (3,3): first wins
    np.testing.assert_array_equal(dx[0, 0], ref)
    r = np.random.default_rng(4)
    x = r.standard_normal((3, 4, 6, 8)); dy = r.standard_normal((3, 4, 3, 4))
    dx = orc.maxpool2_bwd(x, dy)
    np.testing.assert_allclose(dx.reshape(3, 4, 3, 2, 4, 2).sum(axis=(3, 5)), dy, rtol=0, atol=0)
    np.testing.assert_array_equal(orc.maxpool2_fwd(x), x.reshape(3, 4, 3, 2, 4, 2).max(axis=(3, 5)))
    assert np.all((dx != 0) <= (x == np.repeat(np.repeat(orc.maxpool2_fwd(x), 2, 2), 2, 3)))


def test_softmax_ce_pins():
    for C in (10, 1000):
        labels = np.arange(8) % C
        loss, d = orc.softmax_ce(np.full((8, C, 1, 1), 3.25), labels, 8)
        assert abs(loss - np.log(C)) < 1e-12                    # uniform prediction: loss = ln C
        np.testing.assert_allclose(d.reshape(8, C).sum(axis=1), 0, atol=1e-15)
    z = np.full((4, 10), -50.0); lab = np.array([1, 3, 5, 7]); z[np.arange(4), lab] = 50.0
    loss, d = orc.softmax_ce(z, lab, 4)
    assert 0 <= loss < 1e-40 or loss < 1e-30                    # confident and right: loss -> 0
    assert np.abs(d).max() < 1e-30
    r = np.random.default_rng(5)
    z = 5 * r.standard_normal((6, 10)); lab = r.integers(0, 10, 6)
    loss, d = orc.softmax_ce(z, lab, 12)                         # batch_total 12: a micro-batch of a larger batch
    ls = scipy.special.log_softmax(z, axis=1)
    assert abs(loss - (-ls[np.arange(6), lab].sum() / 12)) < 1e-13
    oh = np.zeros((6, 10)); oh[np.arange(6), lab] = 1
    np.testing.assert_allclose(d, (scipy.special.softmax(z, axis=1) - oh) / 12, atol=1e-15)
    # large logits do not overflow
    loss, d = orc.softmax_ce(np.array([[1000.0, 0.0]]), np.array([0]), 1)
    assert np.isfinite(loss) and np.all(np.isfinite(d))


def _loss_of(layers, params, x, labels):
    _, _, loss = orc.stage_forward(layers, 0, len(layers), params, x, labels, x.shape[0])
    return loss


@pytest.mark.parametrize("net", ["tiny_lenet", "tiny_resnet"])
def test_backward_matches_finite_differences(net):
    """Central differences in fp64 on whole tiny networks for dW, db and dx (eqs. 8-9).
    tiny_resnet has an identity-shortcut block, a strided projection block, frozen scales, GAP."""
    layers = getattr(wl, net)()
    params, _ = wl.make_params(layers, seed=7, bias_std=0.3)
    x, labels, _ = wl.make_batch(layers, 3, seed=7)
    a, stash, loss = orc.stage_forward(layers, 0, len(layers), params, x, labels, 3)
    grads = orc.zero_grads(layers, params)
    dx = orc.stage_backward(layers, 0, len(layers), params, stash, None, grads, input_grad=True)
    h = 1e-6
    r = np.random.default_rng(11)
    worst = 0.0
    for i, p in params.items():
        for k in ("W", "b"):
            if k not in p:
                continue
            flat = p[k].reshape(-1)
            for idx in r.choice(flat.size, size=min(flat.size, 12), replace=False):
                old = flat[idx]
                flat[idx] = old + h; lp = _loss_of(layers, params, x, labels)
                flat[idx] = old - h; lm = _loss_of(layers, params, x, labels)
                flat[idx] = old
                fd = (lp - lm) / (2 * h)
                an = grads[i][k].reshape(-1)[idx]
                worst = max(worst, abs(fd - an) / max(abs(an), 1e-2 * np.abs(grads[i][k]).max()))
    xf = x.reshape(-1)
    for idx in r.choice(xf.size, size=20, replace=False):
        old = xf[idx]
        xf[idx] = old + h; lp = _loss_of(layers, params, x, labels)
        xf[idx] = old - h; lm = _loss_of(layers, params, x, labels)
        xf[idx] = old
        worst = max(worst, abs((lp - lm) / (2 * h) - dx.reshape(-1)[idx]) / max(abs(dx.reshape(-1)[idx]), 1e-2 * np.abs(dx).max()))
    assert worst < 1e-6, worst


def test_partition_with_upstream_gradient_finite_differences():
    """A partition fed by an upstream activation and an upstream gradient g: d<g,y>/d(param) by central differences."""
    layers = wl.r50_conv4x(cin=4, hw=6, mid=3, cout=5, blocks=2)
    params, _ = wl.make_params(layers, seed=9, bias_std=0.2)
    x, _, g = wl.make_batch(layers, 2, seed=9, grad_std=1.0)
    y, stash, _ = orc.stage_forward(layers, 0, len(layers), params, x)
    grads = orc.zero_grads(layers, params)
    dx = orc.stage_backward(layers, 0, len(layers), params, stash, g, grads, input_grad=True)
    f = lambda: float((orc.stage_forward(layers, 0, len(layers), params, x)[0] * g).sum())
    h, r, worst = 1e-6, np.random.default_rng(12), 0.0
    for i, p in params.items():
        for k in ("W", "b"):
            flat = p[k].reshape(-1)
            for idx in r.choice(flat.size, size=min(flat.size, 6), replace=False):
                old = flat[idx]
                flat[idx] = old + h; lp = f()
                flat[idx] = old - h; lm = f()
                flat[idx] = old
                an = grads[i][k].reshape(-1)[idx]
                worst = max(worst, abs((lp - lm) / (2 * h) - an) / max(abs(an), 1e-2 * np.abs(grads[i][k]).max()))
    xf = x.reshape(-1)
    for idx in r.choice(xf.size, size=20, replace=False):
        old = xf[idx]
        xf[idx] = old + h; lp = f()
        xf[idx] = old - h; lm = f()
        xf[idx] = old
        worst = max(worst, abs((lp - lm) / (2 * h) - dx.reshape(-1)[idx]) / max(abs(dx.reshape(-1)[idx]), 1e-2 * np.abs(dx).max()))
    assert worst < 1e-6, worst


def test_sgd_momentum_pins():
    p0 = np.array([1.0, -2.0, 0.5]); g = np.array([0.3, -0.1, 2.0])
    # mu = 0 is eq. 6 exactly
    params = {0: {"W": p0.copy()}}; mom = {0: {"W": np.array([9.0, 9.0, 9.0])}}
    orc.sgd_momentum(params, {0: {"W": g}}, mom, 0.1, 0.0)
    np.testing.assert_array_equal(params[0]["W"], p0 - 0.1 * g)
    # constant gradient, v0 = 0: p_k = p_0 - lr*g*sum_{i=1..k} (1-mu^i)/(1-mu)
    params = {0: {"W": p0.copy()}}; mom = {0: {"W": np.zeros(3)}}
    lr, mu = 0.05, 0.9
    for k in range(1, 6):
        orc.sgd_momentum(params, {0: {"W": g}}, mom, lr, mu)
        closed = p0 - lr * g * sum((1 - mu ** i) / (1 - mu) for i in range(1, k + 1))
        np.testing.assert_allclose(params[0]["W"], closed, rtol=1e-14)
        if k == 1:
            np.testing.assert_array_equal(params[0]["W"], p0 - lr * g)     # first step == plain SGD
    # frozen scale untouched; stage range respected
    params = {0: {"W": p0.copy(), "s": np.ones(3)}, 1: {"W": p0.copy()}}
    mom = {0: {"W": np.zeros(3)}, 1: {"W": np.zeros(3)}}
    orc.sgd_momentum(params, {0: {"W": g}, 1: {"W": g}}, mom, 0.1, 0.9, first=1, last=2)
    np.testing.assert_array_equal(params[0]["W"], p0)
    np.testing.assert_array_equal(params[0]["s"], np.ones(3))
    np.testing.assert_array_equal(params[1]["W"], p0 - 0.1 * g)


def test_round_bf16_pins():
    """bfloat16 = top 16 bits of float32, round to nearest, ties to even (hand-picked bit patterns)."""
    cases = {1.0: 1.0, 1.00390625: 1.0,            # 1 + 2^-8: exactly half way between 1 and 1+2^-7 -> even (1.0)
             1.01171875: 1.015625,                 # 1 + 3*2^-8: half way, rounds to even mantissa (1+2^-6)
             1.005: 1.0078125, -2.7: -2.703125, 0.0: 0.0}
    got = orc.round_bf16(np.array(list(cases.keys())))
    np.testing.assert_allclose(got, np.array(list(cases.values())), rtol=1e-7)
    r = np.random.default_rng(0)
    a = r.standard_normal(10000) * 10.0 ** r.integers(-3, 4, 10000)
    b = orc.round_bf16(a)
    assert np.all(np.abs(b - a) <= np.abs(a) * 2.0 ** -8)                       # half an ulp of an 8-bit mantissa
    assert np.all((b.astype(np.float32).view(np.uint32) & 0xFFFF) == 0)          # representable
    np.testing.assert_array_equal(orc.round_bf16(b), b)                          # idempotent
    import torch                                                                 # library conversion, CPU
    np.testing.assert_array_equal(b, torch.tensor(a, dtype=torch.float32).bfloat16().double().numpy())
    # with store=round_bf16 every stored activation is representable, the rest of the step is unchanged
    layers = wl.tiny_vgg()
    params, _ = wl.make_params(layers, seed=2, bf16=True)
    x, labels, _ = wl.make_batch(layers, 2, seed=2, bf16=True)
    _, stash, _ = orc.stage_forward(layers, 0, len(layers), params, x, labels, 2, store=orc.round_bf16)
    for t, v in stash.items():
        if t != "dlogits":
            assert np.all((np.asarray(v).astype(np.float32).view(np.uint32) & 0xFFFF) == 0), t


def test_adam_pins():
    """Adam against what its definition fixes: the first step from a zero state moves every element by
    lr * g / (|g| + eps) whatever its size; under a constant gradient the bias-corrected moments are exactly g
    and g*g at every step, so T steps move by T times that; a zero gradient moves nothing; and a hand-computed
    second step with a different gradient."""
    rng_ = np.random.default_rng(3)
    g = rng_.standard_normal((4, 3, 2, 2)) * np.array([1e-3, 1.0, 50.0])[None, :, None, None]
    p0 = rng_.standard_normal(g.shape)
    lr, b1, b2, eps = 0.01, 0.9, 0.999, 1e-8
    params, m1, m2 = {0: {"W": p0.copy()}}, {0: {"W": np.zeros_like(g)}}, {0: {"W": np.zeros_like(g)}}
    orc.adam(params, {0: {"W": g}}, m1, m2, lr, b1, b2, eps, 1)
    step = lr * g / (np.abs(g) + eps)
    np.testing.assert_allclose(params[0]["W"], p0 - step, rtol=0, atol=1e-15)
    for t in range(2, 8):                      # constant gradient
        orc.adam(params, {0: {"W": g}}, m1, m2, lr, b1, b2, eps, t)
        np.testing.assert_allclose(params[0]["W"], p0 - t * step, rtol=0, atol=1e-12)
        np.testing.assert_allclose(m1[0]["W"] / (1 - b1 ** t), g, rtol=1e-12)
        np.testing.assert_allclose(m2[0]["W"] / (1 - b2 ** t), g * g, rtol=1e-12)
    # a second step with another gradient, written out element by element
    params, m1, m2 = {0: {"W": np.array([1.0])}}, {0: {"W": np.zeros(1)}}, {0: {"W": np.zeros(1)}}
    orc.adam(params, {0: {"W": np.array([2.0])}}, m1, m2, 0.1, 0.5, 0.75, 0.0, 1)      # m1 = 1, m2 = 1: p = 1 - 0.1
    orc.adam(params, {0: {"W": np.array([-4.0])}}, m1, m2, 0.1, 0.5, 0.75, 0.0, 2)
    # m1 = 0.5*1 + 0.5*(-4) = -1.5 -> /0.75 = -2 ; m2 = 0.75*1 + 0.25*16 = 4.75 -> /0.4375 ; p = 0.9 + 0.1*2/sqrt(4.75/0.4375)
    np.testing.assert_allclose(params[0]["W"], [0.9 + 0.2 / np.sqrt(4.75 / 0.4375)], rtol=1e-14)
    # zero gradient from a zero state: nothing moves (0 / (0 + eps)); the frozen scale and other layers are left alone
    params = {0: {"W": p0.copy(), "s": np.ones(3)}, 1: {"W": p0.copy()}}
    z = {i: {"W": np.zeros_like(g)} for i in (0, 1)}
    m1, m2 = {i: {"W": np.zeros_like(g)} for i in (0, 1)}, {i: {"W": np.zeros_like(g)} for i in (0, 1)}
    orc.adam(params, z, m1, m2, lr, b1, b2, eps, 1)
    np.testing.assert_array_equal(params[0]["W"], p0)
    orc.adam(params, {0: {"W": g}, 1: {"W": g}}, m1, m2, lr, b1, b2, eps, 1, first=1, last=2)
    np.testing.assert_array_equal(params[0]["W"], p0)
    np.testing.assert_array_equal(params[0]["s"], np.ones(3))
    assert not np.array_equal(params[1]["W"], p0)

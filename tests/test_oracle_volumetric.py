"""Pins for the oracle's volumetric (3-D) convolution and self-attention routines -- the layer kinds of the method's
first use case (3x3x3 convolution blocks, residual self-attention blocks).  No GPU."""
import copy

import numpy as np

import workloads as wl
from workloads import configs
from oracle import lpm_oracle as orc


def _l3(cin, cout, d, h, w, kd, kh, kw, stride=1, pad=0, pad_d=0):
    return dict(kind="conv", cin=cin, cout=cout, kh=kh, kw=kw, stride=stride, pad=pad, h_in=h, w_in=w, d_in=d, kd=kd, pad_d=pad_d,
                relu=False, bias=False, scale=False, src=-1, add_src=None, cut_after=False)


def test_conv3d_hand_case():
    """A 1-channel 3x3x3 volume holding 0..26, an all-ones 3x3x3 filter, pad 1: the centre output is the sum of all
    voxels (351), the corner output the sum of the 2x2x2 sub-volume at that corner; a filter that is 1 at one tap only
    shifts the volume.  Values written out by hand."""
    x = np.arange(27, dtype=np.float64).reshape(1, 1, 3, 3, 3)
    l = _l3(1, 1, 3, 3, 3, 3, 3, 3, pad=1, pad_d=1)
    z = orc.conv_fwd(x.reshape(1, 1, 9, 3), np.ones((1, 1, 9, 3)), l).reshape(3, 3, 3)
    assert z[1, 1, 1] == 351.0
    assert z[0, 0, 0] == 0 + 1 + 3 + 4 + 9 + 10 + 12 + 13 == 52.0
    assert z[2, 2, 2] == 26 + 25 + 23 + 22 + 17 + 16 + 14 + 13 == 156.0
    assert z[0, 1, 1] == sum(range(18)) == 153.0               # slices 0 and 1 in full
    W = np.zeros((1, 1, 3, 3, 3))
    W[0, 0, 2, 1, 0] = 1.0                                     # tap (kd, kh, kw) = (2, 1, 0): reads voxel (d+1, h, w-1)
    z = orc.conv_fwd(x.reshape(1, 1, 9, 3), W.reshape(1, 1, 9, 3), l).reshape(3, 3, 3)
    assert z[0, 1, 1] == x[0, 0, 1, 1, 0] == 12.0 and z[2, 1, 1] == 0.0 and z[1, 2, 0] == 0.0 and z[1, 2, 2] == 25.0


def test_conv3d_reduces_to_known_routines():
    r = np.random.default_rng(1)
    # one slice, filter depth 1: the two-dimensional routine
    x, W = r.normal(size=(2, 3, 7, 6)), r.normal(size=(4, 3, 3, 3))
    l2 = dict(_l3(3, 4, 1, 7, 6, 1, 3, 3, stride=2, pad=1))
    z2 = orc.conv_fwd(x, W, l2)
    z3 = np.empty_like(z2)
    orc._c().orc_conv3d_fwd(orc._p(x), orc._p(W), orc._p(z3), 2, 3, 1, 7, 6, 4, 1, 3, 3, 2, 0, 1)
    np.testing.assert_array_equal(z2, z3)
    # filter depth 1 over a volume: every slice is convolved on its own
    xv = r.normal(size=(2, 3, 5, 7, 6))
    l = _l3(3, 4, 5, 7, 6, 1, 3, 3, stride=1, pad=1)
    zv = orc.conv_fwd(xv.reshape(2, 3, 35, 6), W, l).reshape(2, 4, 5, 7, 6)
    for d in range(5):
        np.testing.assert_allclose(zv[:, :, d], orc.conv_fwd(xv[:, :, d], W, dict(l, d_in=1)), rtol=1e-13, atol=1e-13)
    # a 3x1x1 filter on one channel: a 1-D correlation along the depth (numpy's convolve with the filter reversed)
    xv = r.normal(size=(1, 1, 8, 2, 2))
    k = r.normal(size=3)
    l = _l3(1, 1, 8, 2, 2, 3, 1, 1, pad_d=1)
    zv = orc.conv_fwd(xv.reshape(1, 1, 16, 2), k.reshape(1, 1, 3, 1), l).reshape(8, 2, 2)
    for h in range(2):
        for w in range(2):
            np.testing.assert_allclose(zv[:, h, w], np.convolve(xv[0, 0, :, h, w], k[::-1], mode="same"), rtol=1e-13, atol=1e-13)


def test_conv3d_adjoints():
    """<conv(x; W), y> = <x, conv_bwd_data(y; W)> = <W, conv_bwd_weight(x, y)> for strided, padded volumetric layers."""
    r = np.random.default_rng(2)
    for (d, h, w, kd, k, s, p, pd) in ((5, 6, 4, 3, 3, 1, 1, 1), (7, 6, 5, 3, 3, 2, 1, 1), (4, 4, 4, 1, 1, 2, 0, 0), (6, 5, 5, 3, 2, 2, 0, 1)):
        l = _l3(3, 4, d, h, w, kd, k, k, stride=s, pad=p, pad_d=pd)
        x = r.normal(size=(2, 3, d * h, w))
        W = r.normal(size=(4, 3, kd * k, k))
        z = orc.conv_fwd(x, W, l)
        y = r.normal(size=z.shape)
        lhs = (z * y).sum()
        np.testing.assert_allclose(lhs, (x * orc.conv_bwd_data(y, W, l)).sum(), rtol=1e-12)
        np.testing.assert_allclose(lhs, (W * orc.conv_bwd_weight(x, y, l)).sum(), rtol=1e-12)


def test_attention_closed_forms():
    r = np.random.default_rng(3)
    N, C, H, W = 2, 4, 3, 2
    x = r.normal(size=(N, 3 * C, H, W))
    # zero queries: every score is 0, the softmax is uniform, the output is the mean of the values
    x0 = x.copy(); x0[:, :C] = 0.0
    y = orc.attn_fwd(x0)
    np.testing.assert_allclose(y, np.broadcast_to(x0[:, 2 * C:].mean(axis=(2, 3), keepdims=True), y.shape), rtol=1e-13, atol=1e-13)
    # values equal at every position: any row-stochastic mixing returns them
    xc = x.copy(); xc[:, 2 * C:] = r.normal(size=(N, C, 1, 1))
    np.testing.assert_allclose(orc.attn_fwd(xc), np.broadcast_to(xc[:, 2 * C:, :1, :1], (N, C, H, W)), rtol=1e-13, atol=1e-13)
    # a permutation of the positions permutes the output the same way
    perm = r.permutation(H * W)
    xp = x.reshape(N, 3 * C, H * W)[:, :, perm].reshape(N, 3 * C, H, W)
    np.testing.assert_allclose(orc.attn_fwd(xp).reshape(N, C, H * W), orc.attn_fwd(x).reshape(N, C, H * W)[:, :, perm], rtol=1e-12, atol=1e-13)
    # one key that matches its query overwhelmingly: the output at that query is that key's value
    xs = np.zeros((1, 3, 1, 3)); xs[0, 0, 0, 0] = 50.0; xs[0, 1, 0, 1] = 50.0; xs[0, 2, 0] = [1.0, 2.0, 3.0]
    assert abs(orc.attn_fwd(xs)[0, 0, 0, 0] - 2.0) < 1e-12


def test_attention_gradient_by_finite_differences():
    r = np.random.default_rng(4)
    x, dy = r.normal(size=(2, 6, 3, 2)), r.normal(size=(2, 2, 3, 2))
    g = orc.attn_bwd(x, dy)
    num = np.zeros_like(x)
    for idx in np.ndindex(x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += 1e-6; xm[idx] -= 1e-6
        num[idx] = ((orc.attn_fwd(xp) - orc.attn_fwd(xm)) * dy).sum() / 2e-6
    assert np.abs(num - g).max() <= 1e-7 * max(1.0, np.abs(g).max())


def test_volumetric_network_gradients_by_finite_differences():
    """tiny_conv3d (3x3x3 stem, residual block, strided block with 1x1x1 projection, attention block, head): parameter
    gradients of the whole network against central differences of the loss."""
    L = configs.tiny_conv3d()
    params, _ = wl.make_params(L, 3, bias_std=0.05)
    x, labels, _ = wl.make_batch(L, 2, 3)

    def loss_of(p):
        return orc.stage_forward(L, 0, len(L), p, x, labels, 2)[2]

    grads = orc.zero_grads(L, params)
    _, stash, _ = orc.stage_forward(L, 0, len(L), params, x, labels, 2)
    orc.stage_backward(L, 0, len(L), params, stash, None, grads)
    r = np.random.default_rng(5)
    checked = 0
    for i in params:
        for k in ("W", "b"):
            if k not in params[i]:
                continue
            for _ in range(3):
                idx = tuple(int(r.integers(n)) for n in params[i][k].shape)
                p2 = copy.deepcopy(params); p2[i][k][idx] += 1e-6
                p3 = copy.deepcopy(params); p3[i][k][idx] -= 1e-6
                num = (loss_of(p2) - loss_of(p3)) / 2e-6
                assert abs(num - grads[i][k][idx]) <= 1e-6 * max(1e-2, abs(num)), (i, k, idx, num, grads[i][k][idx])
                checked += 1
    assert checked >= 40


def test_micro_batches_and_schedules_on_the_volumetric_network():
    """Gradient accumulation over micro-batches equals the full-batch gradient, and the overlapped schedule equals the locked
    one, with the new layer kinds in the stages."""
    L = configs.tiny_conv3d()
    starts = [0, 3, 6, len(L)]
    out = []
    for M, mode in ((1, orc.LOCKED), (2, orc.LOCKED), (2, orc.OVERLAPPED)):
        params, mom = wl.make_params(L, 5, bias_std=0.05, momentum_std=1e-3)
        x, labels, _ = wl.make_batch(L, 4, 5)
        ref = orc.run_schedule(L, starts, params, mom, x, labels, None, M, 0.05, 0.9, mode, order_rng=np.random.default_rng(M))
        out.append((ref, params))
    for ref, params in out[1:]:
        assert abs(ref["loss"] - out[0][0]["loss"]) <= 1e-12
        for i in params:
            for k in ("W", "b"):
                if k in params[i]:
                    np.testing.assert_allclose(params[i][k], out[0][1][i][k], rtol=1e-10, atol=1e-12)

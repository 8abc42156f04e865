"""Layer-level GPU parity: the three contractions of a convolution / FC layer, through the C ABI,
against the oracle's direct loops.  Shapes span several tiles, ragged tails, strides, split reductions."""
import numpy as np
import pytest

import workloads as wl
from workloads import rng
from oracle import lpm_oracle as orc
from harness import rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lpm():
    import torch
    assert torch.cuda.is_available()
    import paper_2207_11019_amd as lpm
    return lpm


def _layer(g):
    return dict(kind="conv", cin=g["cin"], cout=g["cout"], kh=g["kh"], kw=g["kw"], stride=g["stride"], pad=g["pad"],
                h_in=g["h"], w_in=g["w"], d_in=g.get("d", 1), kd=g.get("kd", 1), pad_d=g.get("pad_d", 0),
                relu=False, bias=False, scale=False, src=-1, add_src=None, cut_after=False)


def G(m, h, w, cin, cout, k, s=1, p=0, kw=None):
    return dict(m=m, h=h, w=w, cin=cin, cout=cout, kh=k, kw=k if kw is None else kw, stride=s, pad=p)


def G3(m, d, h, w, cin, cout, k, s=1, p=0):
    """A volumetric layer: k x k x k filter over [m][d][h][w][cin]."""
    return dict(m=m, h=h, w=w, cin=cin, cout=cout, kh=k, kw=k, stride=s, pad=p, d=d, kd=k, pad_d=p)


SHAPES = [
    G(2, 8, 8, 32, 64, 3, 1, 1),          # one tile
    G(3, 9, 7, 64, 96, 3, 1, 1),          # ragged M and N
    G(2, 12, 12, 64, 40, 3, 2, 1),        # stride 2, N below a tile
    G(2, 11, 11, 32, 64, 3, 2, 1),        # stride 2, odd extent
    G(4, 28, 28, 64, 64, 3, 2, 1),        # stride 2, several row tiles per residue class
    G(2, 13, 13, 32, 32, 5, 2, 2),        # stride 2, 5x5: classes with 9, 6, 6 and 4 taps
    G(2, 13, 11, 32, 64, 3, 3, 1),        # stride 3: one tap per class
    G(1, 17, 17, 32, 32, 7, 4, 3),        # stride 4, 7x7
    G(2, 9, 9, 256, 64, 3, 2, 1),         # stride 2, long K: split reduction over the taps of a class
    G(4, 6, 6, 128, 256, 1, 1, 0),        # 1x1
    G(2, 8, 8, 64, 128, 1, 2, 0),         # 1x1 stride 2 (projection shortcut)
    G(2, 10, 10, 32, 32, 5, 1, 0),        # 5x5 valid
    G(16, 2, 2, 512, 512, 3, 1, 1),       # deep, few pixels: split reduction
    G(5, 4, 4, 64, 72, 4, 1, 0),          # kernel covers the input: a fully connected layer
    G(16, 1, 1, 512, 10, 1, 1, 0),        # classifier head (Cout = 10)
    G(4, 7, 7, 64, 520, 7, 1, 0),         # FC over a 7x7 map, 4 samples: weight-streaming kernels, ragged channel split
    G(13, 1, 1, 1032, 200, 1, 1, 0),      # FC, 13 samples, K not a multiple of the column block
    G(7, 2, 2, 24, 48, 2, 1, 0),          # FC, 7 samples, one partial column block
    G(4, 16, 16, 3, 64, 3, 1, 1),         # 3-channel first layer (generic kernels)
    G(3, 9, 11, 3, 40, 3, 2, 1),          # 3-channel first layer, stride 2, ragged
    G(2, 12, 12, 1, 16, 5, 1, 0),         # 1 channel, 5x5 (25 terms)
    G(16, 32, 32, 64, 160, 3, 1, 1),      # large: 128x128 tiles
    G(2, 14, 14, 256, 256, 3, 1, 1),      # both >= 128 channels: large weight-gradient tiles
    G(2, 15, 15, 512, 512, 3, 1, 1),      # 512 channels, images just below two patches
    G(3, 24, 15, 64, 128, 3, 1, 1),       # ragged in x only
    # large images: the weight gradient by 8x8 pixel patches (LDS transpose reads)
    G(1, 56, 56, 64, 64, 3, 1, 1),        # one tap per block, few patches per block
    G(2, 64, 64, 64, 128, 3, 1, 1),       # one tap per block, more blocks than CUs
    G(1, 57, 59, 128, 128, 3, 1, 1),      # a filter row per block, patches over the edge in both directions
    G(4, 64, 64, 128, 128, 3, 1, 0),      # a filter row per block, no padding
    G(1, 60, 60, 72, 136, 3, 1, 1),       # channel counts that are not multiples of the 64-channel tile
    # volumetric layers (3x3x3 and 1x1x1 filters, the first use case's shapes)
    G3(2, 6, 6, 6, 32, 64, 3, 1, 1),      # matrix-core kernels for all three contractions
    G3(1, 5, 7, 6, 64, 40, 3, 1, 1),      # ragged extents and channel tile
    G3(2, 8, 8, 8, 32, 64, 3, 2, 1),      # stride 2: the data gradient by residue classes of (d, h, w)
    dict(G3(2, 7, 9, 6, 32, 64, 3, 2, 1), h=9, w=6),      # stride 2, odd extents: eight classes of different sizes
    G3(1, 12, 12, 12, 64, 64, 3, 2, 1),   # stride 2, several row tiles per class
    G3(2, 5, 5, 5, 64, 256, 3, 2, 1),     # stride 2, long K: split reduction over the taps of a class
    G3(2, 8, 8, 8, 32, 64, 1, 2, 0),      # 1x1x1 stride-2 projection
    G3(2, 4, 4, 4, 128, 128, 3, 1, 1),    # long reduction: split over blocks
    G3(1, 4, 9, 8, 32, 64, 3, 1, 1),      # 8x8 patches of the output slices: the patch-based weight gradient, one tap per block
    G3(2, 6, 16, 16, 128, 128, 3, 1, 1),  # ... a filter row per block (27 taps in 9 groups)
    G3(1, 7, 15, 15, 32, 64, 3, 2, 1),    # ... stride 2, odd extents
    G3(2, 3, 8, 8, 64, 64, 1, 1, 0),      # ... 1x1x1: the voxels regrouped as one image of full patches
    G3(3, 4, 4, 4, 64, 192, 1, 1, 0),     # 1x1x1 (queries | keys | values of an attention block)
    G3(2, 8, 8, 8, 1, 16, 3, 1, 1),       # one-channel input volume: flattened (tap, channel) weight gradient
    dict(G3(1, 9, 7, 10, 2, 24, 3, 1, 1), h=7, w=10),     # two channels x 27 taps, ragged extents
    G3(2, 9, 9, 9, 1, 32, 3, 2, 1),       # one-channel volume, stride 2
    dict(G3(2, 3, 4, 4, 32, 48, 3, 1, 0), kd=3, pad_d=0, kh=4, kw=4),   # filter covers the whole volume: a fully connected layer
]


def _pack(lpm, torch, a):
    return lpm.pack_act(a, lpm.BF16)


@pytest.mark.parametrize("g", SHAPES, ids=lambda g: "m%d_%s%dx%dx%d_%d_k%dx%d_s%d_p%d" % (g["m"], ("d%dk%d_" % (g["d"], g["kd"])) if "d" in g else "", g["h"], g["w"], g["cin"], g["cout"], g["kh"], g["kw"], g["stride"], g["pad"]))
def test_conv_ops_bf16(lpm, g):
    import torch
    print("geometry", g, flush=True)
    l = _layer(g)
    seed = 3
    D, KD = g.get("d", 1), g.get("kd", 1)          # a volume's depth is folded into the height axis of the logical tensors
    x = rng.round_to_bf16(rng.normal(seed, 1, (g["m"], g["cin"], D * g["h"], g["w"])))
    W = rng.round_to_bf16(rng.normal(seed, 2, (g["cout"], g["cin"], KD * g["kh"], g["kw"]), 0.0, (2.0 / (g["cin"] * KD * g["kh"] * g["kw"])) ** 0.5))
    z = orc.conv_fwd(x, W, l)
    dz = rng.round_to_bf16(rng.normal(seed, 3, z.shape))
    sc = rng.uniform(seed, 4, (g["cout"],), 0.5, 1.5).astype(np.float32)
    bi = rng.normal(seed, 5, (g["cout"],)).astype(np.float32)
    add = rng.round_to_bf16(rng.normal(seed, 6, z.shape))
    dx0 = rng.round_to_bf16(rng.normal(seed, 7, x.shape))
    dw0 = rng.normal(seed, 8, W.shape).astype(np.float32).astype(np.float64)

    xd, dzd, addd = _pack(lpm, torch, x), _pack(lpm, torch, dz), _pack(lpm, torch, add)
    wd = torch.from_numpy(lpm.pack_weight(W)).cuda().to(torch.bfloat16)
    wtd = torch.from_numpy(np.ascontiguousarray(np.transpose(W, (1, 2, 3, 0)).astype(np.float32)).reshape(-1)).cuda().to(torch.bfloat16)
    scd, bid = torch.from_numpy(sc).cuda(), torch.from_numpy(bi).cuda()
    wsb = lpm.lpm_conv_ws_bytes(g, lpm.BF16)
    ws = torch.zeros(max(max(wsb), 256), dtype=torch.uint8, device="cuda")

    # forward, plain and with the full epilogue
    yd = torch.empty(z.size, dtype=torch.bfloat16, device="cuda")
    lpm.lpm_conv_forward(g, lpm.BF16, xd, wd, None, None, None, False, yd, ws)
    torch.cuda.synchronize()
    assert rel_err(lpm.unpack_act(yd, z.shape), z) <= 2e-2
    lpm.lpm_conv_forward(g, lpm.BF16, xd, wd, scd, bid, addd, True, yd, ws)
    torch.cuda.synchronize()
    ref = np.maximum(z * sc[None, :, None, None] + bi[None, :, None, None] + add, 0.0)
    assert rel_err(lpm.unpack_act(yd, z.shape), ref) <= 2e-2

    # data gradient, overwrite and accumulate, with and without the transposed weights
    dx_ref = orc.conv_bwd_data(dz, W, l)
    for wt in (wtd, None):
        dxd = _pack(lpm, torch, dx0).clone()
        lpm.lpm_conv_dgrad(g, lpm.BF16, dzd, wd, wt, dxd, False, ws)
        torch.cuda.synchronize()
        assert rel_err(lpm.unpack_act(dxd, x.shape), dx_ref) <= 2e-2
        dxd = _pack(lpm, torch, dx0).clone()
        lpm.lpm_conv_dgrad(g, lpm.BF16, dzd, wd, wt, dxd, True, ws)
        torch.cuda.synchronize()
        assert rel_err(lpm.unpack_act(dxd, x.shape), dx_ref + dx0) <= 2e-2

    # weight gradient (float output), overwrite and accumulate
    dw_ref = orc.conv_bwd_weight(x, dz, l)
    dwd = torch.from_numpy(lpm.pack_weight(dw0)).cuda()
    lpm.lpm_conv_wgrad(g, lpm.BF16, xd, dzd, dwd, False, ws)
    torch.cuda.synchronize()
    assert rel_err(lpm.unpack_weight(dwd.cpu().numpy(), W.shape), dw_ref) <= 1e-3
    dwd = torch.from_numpy(lpm.pack_weight(dw0)).cuda()
    lpm.lpm_conv_wgrad(g, lpm.BF16, xd, dzd, dwd, True, ws)
    torch.cuda.synchronize()
    assert rel_err(lpm.unpack_weight(dwd.cpu().numpy(), W.shape), dw_ref + dw0) <= 1e-3


@pytest.mark.parametrize("g", [G(2, 9, 7, 5, 7, 3, 2, 1), G(3, 6, 6, 4, 6, 5, 1, 0), G(4, 4, 4, 16, 10, 4, 1, 0)],
                         ids=["s2", "k5", "fc"])
def test_conv_ops_f32(lpm, g):
    import torch
    l = _layer(g)
    x = rng.normal(5, 1, (g["m"], g["cin"], g["h"], g["w"]))
    W = rng.normal(5, 2, (g["cout"], g["cin"], g["kh"], g["kw"]))
    z = orc.conv_fwd(x, W, l)
    dz = rng.normal(5, 3, z.shape)
    xd, dzd = lpm.pack_act(x, lpm.F32), lpm.pack_act(dz, lpm.F32)
    wd = torch.from_numpy(lpm.pack_weight(W)).cuda()
    ws = torch.zeros(max(max(lpm.lpm_conv_ws_bytes(g, lpm.F32)), 256), dtype=torch.uint8, device="cuda")
    yd = torch.empty(z.size, device="cuda")
    lpm.lpm_conv_forward(g, lpm.F32, xd, wd, None, None, None, False, yd, ws)
    dxd = torch.empty(x.size, device="cuda")
    lpm.lpm_conv_dgrad(g, lpm.F32, dzd, wd, None, dxd, False, ws)
    dwd = torch.empty(W.size, device="cuda")
    lpm.lpm_conv_wgrad(g, lpm.F32, xd, dzd, dwd, False, ws)
    torch.cuda.synchronize()
    assert rel_err(lpm.unpack_act(yd, z.shape), z) <= 1e-4
    assert rel_err(lpm.unpack_act(dxd, x.shape), orc.conv_bwd_data(dz, W, l)) <= 1e-4
    assert rel_err(lpm.unpack_weight(dwd.cpu().numpy(), W.shape), orc.conv_bwd_weight(x, dz, l)) <= 1e-4

"""Layer-wise partitioning of one layer (the paper's "Layer-wise Partitioning and Merging" section, fig. 1a) through
the C ABI: n sub-layers plus concatenation / re-partition / summation must give the merged layer's results, so the
reference is the oracle's plain convolution."""
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


def G(m, h, w, cin, cout, k, s=1, p=0):
    return dict(m=m, h=h, w=w, cin=cin, cout=cout, kh=k, kw=k, stride=s, pad=p)


def _layer(g):
    return dict(kind="conv", cin=g["cin"], cout=g["cout"], kh=g["kh"], kw=g["kw"], stride=g["stride"], pad=g["pad"],
                h_in=g["h"], w_in=g["w"], relu=False, bias=False, scale=False, src=-1, add_src=None, cut_after=False)


CASES = [
    (G(2, 8, 8, 32, 64, 3, 1, 1), 2),         # one tile per sub-layer
    (G(3, 9, 7, 64, 96, 3, 1, 1), 4),         # ragged rows, 24 channels per sub-layer
    (G(16, 32, 32, 64, 64, 3, 1, 1), 4),      # a VGG-16/CIFAR layer at its micro-batch: several row tiles, 16 channels each
    (G(4, 28, 28, 64, 128, 3, 2, 1), 4),      # stride 2
    (G(4, 6, 6, 128, 256, 1, 1, 0), 8),       # 1x1, eight sub-layers
    (G(16, 2, 2, 512, 512, 3, 1, 1), 4),      # deep, few pixels: split reductions inside every sub-layer
    (G(4, 7, 7, 64, 512, 7, 1, 0), 4),        # fully connected layer over a 7x7 map (weight-streaming kernels)
    (G(4, 16, 16, 3, 64, 3, 1, 1), 4),        # 3-channel first layer: weight slices that are not 256-byte multiples
    (G(1, 56, 56, 64, 128, 3, 1, 1), 2),      # large image: patch-based weight gradient inside the sub-layers
]


@pytest.mark.parametrize("g,n", CASES, ids=lambda v: str(v) if isinstance(v, int) else "m%d_%dx%dx%d_%d_k%d_s%d" % (v["m"], v["h"], v["w"], v["cin"], v["cout"], v["kh"], v["stride"]))
def test_layerwise_bf16(lpm, g, n):
    import torch
    print("geometry", g, "n", n, flush=True)
    l = _layer(g)
    seed = 11
    cn = g["cout"] // n
    x = rng.round_to_bf16(rng.normal(seed, 1, (g["m"], g["cin"], g["h"], g["w"])))
    W = rng.round_to_bf16(rng.normal(seed, 2, (g["cout"], g["cin"], g["kh"], g["kw"]), 0.0, (2.0 / (g["cin"] * g["kh"] * g["kw"])) ** 0.5))
    z = orc.conv_fwd(x, W, l)
    dz = rng.round_to_bf16(rng.normal(seed, 3, z.shape))
    sc = rng.uniform(seed, 4, (g["cout"],), 0.5, 1.5).astype(np.float32)
    bi = rng.normal(seed, 5, (g["cout"],)).astype(np.float32)
    dw0 = rng.normal(seed, 8, W.shape).astype(np.float32).astype(np.float64)

    xd, dzd = lpm.pack_act(x, lpm.BF16), lpm.pack_act(dz, lpm.BF16)
    wd = torch.from_numpy(lpm.pack_weight(W)).cuda().to(torch.bfloat16)
    # each sub-layer's weights transposed to [cin][kh][kw][cout/n], one after the other
    wt = np.concatenate([np.transpose(W[i * cn:(i + 1) * cn], (1, 2, 3, 0)).reshape(-1) for i in range(n)])
    wtd = torch.from_numpy(np.ascontiguousarray(wt.astype(np.float32))).cuda().to(torch.bfloat16)
    scd, bid = torch.from_numpy(sc).cuda(), torch.from_numpy(bi).cuda()

    lw = lpm.Layerwise(g, lpm.BF16, n)
    ws = torch.zeros(max(lw.fwd_ws_bytes, lw.bwd_ws_bytes, 256), dtype=torch.uint8, device="cuda")

    yd = torch.empty(z.size, dtype=torch.bfloat16, device="cuda")
    lw.forward(xd, wd, None, None, False, yd, ws)
    torch.cuda.synchronize()
    assert rel_err(lpm.unpack_act(yd, z.shape), z) <= 2e-2
    lw.forward(xd, wd, scd, bid, True, yd, ws)
    torch.cuda.synchronize()
    ref = np.maximum(z * sc[None, :, None, None] + bi[None, :, None, None], 0.0)
    assert rel_err(lpm.unpack_act(yd, z.shape), ref) <= 2e-2

    dx_ref = orc.conv_bwd_data(dz, W, l)
    dw_ref = orc.conv_bwd_weight(x, dz, l)
    for wt_arg in (wtd, None):
        dxd = torch.full((x.size,), 7.0, dtype=torch.bfloat16, device="cuda")
        dwd = torch.from_numpy(lpm.pack_weight(dw0)).cuda()
        lw.backward(xd, dzd, wd, wt_arg, dxd, dwd, False, ws)
        torch.cuda.synchronize()
        assert rel_err(lpm.unpack_act(dxd, x.shape), dx_ref) <= 2e-2
        assert rel_err(lpm.unpack_weight(dwd.cpu().numpy(), W.shape), dw_ref) <= 1e-3
    # accumulation into dw; no input gradient asked for
    dwd = torch.from_numpy(lpm.pack_weight(dw0)).cuda()
    lw.backward(xd, dzd, wd, wtd, None, dwd, True, ws)
    torch.cuda.synchronize()
    assert rel_err(lpm.unpack_weight(dwd.cpu().numpy(), W.shape), dw_ref + dw0) <= 1e-3
    lw.close()


def test_layerwise_f32(lpm):
    import torch
    g, n = G(3, 10, 10, 16, 32, 3, 1, 1), 2
    l = _layer(g)
    seed = 12
    x = rng.normal(seed, 1, (g["m"], g["cin"], g["h"], g["w"])).astype(np.float32).astype(np.float64)
    W = rng.normal(seed, 2, (g["cout"], g["cin"], 3, 3), 0.0, 0.1).astype(np.float32).astype(np.float64)
    z = orc.conv_fwd(x, W, l)
    dz = rng.normal(seed, 3, z.shape).astype(np.float32).astype(np.float64)
    xd, dzd = lpm.pack_act(x, lpm.F32), lpm.pack_act(dz, lpm.F32)
    wd = torch.from_numpy(lpm.pack_weight(W)).cuda()
    lw = lpm.Layerwise(g, lpm.F32, n)
    ws = torch.zeros(max(lw.fwd_ws_bytes, lw.bwd_ws_bytes, 256), dtype=torch.uint8, device="cuda")
    yd = torch.empty(z.size, dtype=torch.float32, device="cuda")
    lw.forward(xd, wd, None, None, False, yd, ws)
    dxd = torch.empty(x.size, dtype=torch.float32, device="cuda")
    dwd = torch.zeros(W.size, dtype=torch.float32, device="cuda")
    lw.backward(xd, dzd, wd, None, dxd, dwd, False, ws)
    torch.cuda.synchronize()
    assert rel_err(lpm.unpack_act(yd, z.shape), z) <= 1e-4
    assert rel_err(lpm.unpack_act(dxd, x.shape), orc.conv_bwd_data(dz, W, l)) <= 1e-4
    assert rel_err(lpm.unpack_weight(dwd.cpu().numpy(), W.shape), orc.conv_bwd_weight(x, dz, l)) <= 1e-4
    lw.close()


def test_layerwise_rejects(lpm):
    with pytest.raises(lpm.LpmError):
        lpm.Layerwise(G(2, 8, 8, 32, 64, 3, 1, 1), lpm.BF16, 1)      # fewer than two sub-layers
    with pytest.raises(lpm.LpmError):
        lpm.Layerwise(G(2, 8, 8, 32, 60, 3, 1, 1), lpm.BF16, 4)      # 15 channels per sub-layer
    with pytest.raises(lpm.LpmError):
        lpm.Layerwise(G(2, 8, 8, 32, 64, 3, 1, 1), lpm.BF16, 3)      # not divisible

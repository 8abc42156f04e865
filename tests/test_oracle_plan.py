"""Pins for the oracle's cost model and plan search."""
import itertools

import numpy as np
import pytest

import workloads as wl
from oracle import lpm_oracle as orc

CP = dict(flop_per_us=2_516_582_400, hbm_byte_per_us=8_000_000, link_byte_per_us=0,
          elem_bytes=2, microbatch=16, n_microbatch=8)
CP32 = dict(flop_per_us=157_286_400, hbm_byte_per_us=8_000_000, link_byte_per_us=0,
            elem_bytes=4, microbatch=8, n_microbatch=4)


def test_layer_cost_hand_computed_lenet():
    """Two LeNet layers worked by hand from the cost definition (fp32, m=8, M=4)."""
    L = wl.lenet()
    # conv1: 1x28x28 -> 6x24x24, 5x5, first layer (no data gradient)
    mac = 6 * 24 * 24 * 25
    flop = 2 * mac * 8 * 2
    in_el, out_el, w_el, p_el = 784, 3456, 150, 156
    fwd = (in_el + out_el) * 8 * 4 + w_el * 4
    bwd = (out_el + in_el) * 8 * 4 + w_el * 4 + 8 * w_el
    upd = p_el * 20
    expect = max(flop * 10**6 // 157_286_400, ((fwd + bwd) * 4 + upd) * 10**6 // (4 * 8_000_000))
    assert orc.layer_cost(L, 0, 8, 4, 4, 157_286_400, 8_000_000) == expect == 34317   # (273760*4+3120)*1e6 // 32e6; flop term 17578
    # fc1: 256 -> 120 (kernel covers the 16x4x4 input), not first
    mac = 120 * 256
    flop = 2 * mac * 8 * 3
    in_el, out_el, w_el, p_el = 256, 120, 30720, 30840
    fwd = (in_el + out_el) * 8 * 4 + w_el * 4
    bwd = (out_el + 2 * in_el) * 8 * 4 + w_el * 4 + 8 * w_el
    upd = p_el * 20
    expect = max(flop * 10**6 // 157_286_400, ((fwd + bwd) * 4 + upd) * 10**6 // (4 * 8_000_000))
    assert orc.layer_cost(L, 4, 8, 4, 4, 157_286_400, 8_000_000) == expect


def test_layer_cost_hand_computed_residual_bf16():
    """A ResNet-18 layer with a shortcut in the bf16 element type (m = 32, M = 8), worked by hand: the second 3x3
    convolution of the first basic block, 64 -> 64 channels over 32x32 pixels, which adds the stem's output.  The
    shortcut is one more tensor read forward and one more written backward, and the update moves 22 bytes per
    parameter (20 in float plus the 2-byte weight copy).  Every number below is written out, not computed."""
    L = wl.resnet18_cifar()
    assert L[2]["add_src"] == 0 and L[2]["cin"] == L[2]["cout"] == 64 and L[2]["h_in"] == 32
    # multiply-adds 64*32*32 * 64*9 = 37 748 736;  flop = 2 * mac * 32 images * 3 passes = 7 247 757 312
    # arithmetic time = 7 247 757 312 * 1e6 // 2 516 582 400 = 2 880 000 ps
    # elements per image: in = out = shortcut = 65 536;  weights 36 864, parameters 36 864 + 64 = 36 928
    # forward bytes  = (in + out + shortcut) * 32 * 2 + weights * 2            = 12 582 912 + 73 728      = 12 656 640
    # backward bytes = (dout + in + din + dshortcut) * 32 * 2 + weights*2 + 8*weights = 16 777 216 + 73 728 + 294 912 = 17 145 856
    # update bytes   = 36 928 * 22                                                                         =    812 416
    # traffic time = ((12 656 640 + 17 145 856) * 8 + 812 416) * 1e6 // (8 * 8 000 000) = 239 232 384 // 64 = 3 738 006 ps
    assert orc.layer_cost(L, 2, 32, 8, 2, 2_516_582_400, 8_000_000) == 3_738_006
    # without the shortcut terms the layer would be arithmetic-bound (2 689 430 < 2 880 000); with 20-byte updates 3 736 852
    assert 3_738_006 not in (2_880_000, 3_736_852)


def test_stage_cost_is_additive():
    L = wl.vgg16_cifar()
    c = [orc.layer_cost(L, i, 16, 8, 2, CP["flop_per_us"], CP["hbm_byte_per_us"]) for i in range(len(L))]
    starts = [0, 6, 10, 18, len(L)]
    costs, bb = orc.plan_cost(L, starts, CP)
    assert costs == [sum(c[a:b]) for a, b in zip(starts[:-1], starts[1:])]
    assert sum(costs) == sum(c)                                         # eq. 10: total is cut-invariant
    assert bb == sum(int(np.prod(wl.out_shape(L[s - 1]))) * 16 * 2 for s in starts[1:-1])
    # with a link the two stages adjacent to a cut each pay activation + gradient transfer
    cpl = dict(CP, link_byte_per_us=153_000)
    costs_l, _ = orc.plan_cost(L, starts, cpl)
    t = [2 * int(np.prod(wl.out_shape(L[s - 1]))) * 16 * 2 * 10**6 // 153_000 for s in starts[1:-1]]
    assert costs_l == [costs[0] + t[0], costs[1] + t[0] + t[1], costs[2] + t[1] + t[2], costs[3] + t[2]]


@pytest.mark.parametrize("name", ["lenet", "vgg16_cifar", "resnet18_cifar", "vgg16_224"])
def test_plan_properties(name):
    builder, batch, M, Z, dtype, _ = wl.CONFIGS[name]
    L = builder()
    cp = dict(CP32 if dtype == "f32" else CP, microbatch=batch // M, n_microbatch=M)
    c = [orc.layer_cost(L, i, cp["microbatch"], M, cp["elem_bytes"], cp["flop_per_us"], cp["hbm_byte_per_us"])
         for i in range(len(L))]
    n_allowed = sum(l["cut_after"] for l in L[:-1])
    prev = None
    for z in range(1, min(n_allowed + 1, 5) + 1):
        starts, costs = orc.plan_bruteforce(L, z, cp)
        # every layer exactly once, in order
        assert starts[0] == 0 and starts[-1] == len(L) and len(starts) == z + 1
        assert all(a < b for a, b in zip(starts[:-1], starts[1:]))
        assert all(L[s - 1]["cut_after"] for s in starts[1:-1])
        assert sum(costs) == sum(c)
        bott = max(costs)
        assert bott >= max(c) and bott >= -(-sum(c) // z)
        if prev is not None:
            assert bott <= prev                                          # non-increasing in Z
        prev = bott
    starts, _ = orc.plan_bruteforce(L, 1, cp)
    assert starts == [0, len(L)]
    starts, _ = orc.plan_bruteforce(L, n_allowed + 1, cp)
    assert starts == [0] + [i + 1 for i, l in enumerate(L[:-1]) if l["cut_after"]] + [len(L)]
    with pytest.raises(ValueError):
        orc.plan_bruteforce(L, n_allowed + 2, cp)


def test_lenet_plan_is_conv_block_then_fc_block():
    L = wl.lenet()
    starts, _ = orc.plan_bruteforce(L, 2, CP32)
    assert starts == [0, 4, 8]


def test_tie_breaks_on_synthetic_costs(monkeypatch):
    """Equal-cost layers: ties on the bottleneck are broken by boundary bytes, then by smallest starts."""
    L = [dict(kind="maxpool2", cin=c, cout=c, kh=2, kw=2, stride=2, pad=0, h_in=2, w_in=2, relu=False, bias=False,
              scale=False, src=i - 1, add_src=None, cut_after=True) for i, c in enumerate([8, 8, 2, 8, 8, 8])]
    monkeypatch.setattr(orc, "layer_cost", lambda *a, **k: 10)
    # Z=2, six layers of cost 10: bottleneck 30 only with the cut after layer 2 -> unique
    starts, costs = orc.plan_bruteforce(L, 2, CP)
    assert starts == [0, 3, 6] and costs == [30, 30]
    # Z=4: bottleneck 20 for several plans; boundary bytes prefer cutting after the narrow layer 2
    starts, costs = orc.plan_bruteforce(L, 4, CP)
    assert max(costs) == 20 and 3 in starts
    cands = []
    for cuts in itertools.combinations(range(1, 6), 3):
        s = [0] + list(cuts) + [6]
        cs, bb = orc.plan_cost(L, s, CP)
        if max(cs) == 20:
            cands.append((bb, s))
    assert starts == min(cands)[1]
    # all boundaries equal: the lexicographically smallest starts wins
    for l in L:
        l["cin"] = l["cout"] = 8
    starts, _ = orc.plan_bruteforce(L, 4, CP)
    assert starts == [0, 1, 2, 4, 6]

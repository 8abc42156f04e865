"""Host-side tests of the C ABI (no GPU): exported symbols, validation and error codes, the planner
against the oracle's exhaustive enumeration, stage buffer layout."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl
from oracle import lpm_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lpm():
    import paper_2207_11019_amd as lpm
    return lpm


def test_library_exports_every_declared_symbol(lpm):
    hdr = open(os.path.join(ROOT, "include", "lpm.h")).read()
    names = set(re.findall(r"\b(lpm_[a-z_0-9]+)\s*\(", hdr))
    assert {"lpm_partition", "lpm_stage_forward", "lpm_stage_backward", "lpm_stage_update", "lpm_schedule_run"} <= names
    for n in sorted(names):
        assert hasattr(lpm.lib, n), n
    assert lpm.lib.lpm_last_error() is not None


def _cp(dt, m, M, link=0):
    base = dict(flop_per_us=2_516_582_400, hbm_byte_per_us=8_000_000, elem_bytes=2) if dt == "bf16" else \
        dict(flop_per_us=157_286_400, hbm_byte_per_us=8_000_000, elem_bytes=4)
    return dict(base, link_byte_per_us=link, microbatch=m, n_microbatch=M)


@pytest.mark.parametrize("name", list(wl.CONFIGS) + list(wl.EXTRA_CONFIGS))
def test_plans_bit_exact_against_oracle(lpm, name):
    builder, batch, M, Z, dt, _ = dict(wl.CONFIGS, **wl.EXTRA_CONFIGS)[name]
    L = builder()
    for link in (0, 153_000):
        cp = _cp(dt, batch // M, M, link)
        for i in range(len(L)):
            assert lpm.lpm_layer_cost(L, i, cp) == orc.layer_cost(L, i, cp["microbatch"], M, cp["elem_bytes"],
                                                                  cp["flop_per_us"], cp["hbm_byte_per_us"])
        n_allowed = sum(l["cut_after"] for l in L[:-1])
        for z in range(1, min(5, n_allowed + 1) + 1):
            starts, costs = lpm.lpm_partition(L, z, cp)
            so, co = orc.plan_bruteforce(L, z, cp)
            assert starts == so and costs == co, (name, z, link)
            # fixed_starts only validates and costs
            s2, c2 = lpm.lpm_partition(L, z, cp, fixed_starts=so)
            assert s2 == so and c2 == co


def test_plans_on_random_chains(lpm):
    """Random conv/pool chains with random cut permissions: DP == exhaustive enumeration, ties included."""
    r = np.random.default_rng(0)
    for trial in range(40):
        n = int(r.integers(3, 11))
        c, h = int(r.choice([4, 8, 16])), 16
        L = []
        for i in range(n):
            if h >= 4 and r.random() < 0.3:
                l = dict(kind="maxpool2", cin=c, cout=c, kh=2, kw=2, stride=2, pad=0, h_in=h, w_in=h, relu=False, bias=False,
                         scale=False, src=i - 1, add_src=None, cut_after=bool(r.random() < 0.7))
                h //= 2
            else:
                co = int(r.choice([4, 8, 8, 16]))     # repeated widths make cost ties likely
                l = dict(kind="conv", cin=c, cout=co, kh=3, kw=3, stride=1, pad=1, h_in=h, w_in=h, relu=True, bias=True,
                         scale=False, src=i - 1, add_src=None, cut_after=bool(r.random() < 0.7))
                c = co
            L.append(l)
        cp = _cp("bf16", int(r.choice([1, 4])), int(r.choice([1, 4])), int(r.choice([0, 1000])))
        allowed = sum(l["cut_after"] for l in L[:-1])
        for Z in range(1, allowed + 2):
            starts, costs = lpm.lpm_partition(L, Z, cp)
            so, co_ = orc.plan_bruteforce(L, Z, cp)
            assert starts == so and costs == co_, (trial, Z)
        with pytest.raises(lpm.LpmError) as e:
            lpm.lpm_partition(L, allowed + 2, cp)
        assert e.value.code in (-6, -1)


def test_plans_from_supplied_costs(lpm):
    """The cost model with caller-supplied (measured) per-layer costs: the library's DP equals the oracle's
    enumeration with the same costs; a hand case pins the oracle itself (costs 5,1,1,1,5,1 into 3 stages:
    the two heavy layers must be separated, bottleneck 6; ties go to the smallest starts)."""
    L = [dict(kind="conv", cin=8, cout=8, kh=1, kw=1, stride=1, pad=0, h_in=2, w_in=2, relu=False, bias=False,
              scale=False, src=i - 1, add_src=None, cut_after=True) for i in range(6)]
    cp = _cp("bf16", 1, 1, 0)
    costs = [5, 1, 1, 1, 5, 1]
    so, co_ = orc.plan_bruteforce(L, 3, cp, layer_costs=costs)
    assert so == [0, 1, 4, 6] and co_ == [5, 3, 6]
    starts, sc = lpm.lpm_partition_costs(L, 3, cp, costs)
    assert starts == so and sc == co_
    # given costs equal to the analytic ones reproduce lpm_partition
    an = [lpm.lpm_layer_cost(L, i, cp) for i in range(6)]
    assert lpm.lpm_partition_costs(L, 3, cp, an) == lpm.lpm_partition(L, 3, cp)
    r = np.random.default_rng(1)
    for name in ("lenet", "vgg16_cifar", "resnet18_cifar"):
        builder, batch, M, Z, dt, _ = wl.CONFIGS[name]
        layers = builder()
        cpn = _cp(dt, batch // M, M, 0)
        for trial in range(3):
            costs = [int(v) for v in r.integers(1, 1000, len(layers))]
            starts, sc = lpm.lpm_partition_costs(layers, Z, cpn, costs)
            so, co_ = orc.plan_bruteforce(layers, Z, cpn, layer_costs=costs)
            assert starts == so and sc == co_, (name, trial)
    with pytest.raises(lpm.LpmError):
        lpm.lpm_partition_costs(L, 3, cp, [1, 2, 3])


def test_layer_cost_residual_bf16_hand_value(lpm):
    """The library's cost of a bf16 ResNet-18 layer with a shortcut equals the value worked by hand in
    tests/test_oracle_plan.py::test_layer_cost_hand_computed_residual_bf16 (shortcut bytes, 22-byte update)."""
    L = wl.resnet18_cifar()
    assert lpm.lpm_layer_cost(L, 2, _cp("bf16", 32, 8)) == 3_738_006


def test_fixed_plan_out_of_range_is_rejected(lpm):
    """A fixed plan whose entries point past the layer list is refused before any entry is used as an index."""
    L = wl.lenet()
    cp = _cp("f32", 8, 4)
    for plan in ([0, 1000, 8], [0, 8, 8], [0, 9, 8], [0, 4, 2000]):
        with pytest.raises(lpm.LpmError) as e:
            lpm.lpm_partition(L, 2, cp, fixed_starts=plan)
        assert e.value.code == -6, plan
    with pytest.raises(lpm.LpmError) as e:
        lpm.lpm_partition(L, 3, cp, fixed_starts=[0, 4, 100000, 8])
    assert e.value.code == -6


def test_error_codes(lpm):
    L = wl.lenet()
    cp = _cp("f32", 8, 4)
    with pytest.raises(lpm.LpmError) as e:
        lpm.lpm_partition(L, 0, cp)
    assert e.value.code == -1
    with pytest.raises(lpm.LpmError) as e:
        lpm.lpm_partition(L, 2, dict(cp, elem_bytes=3))
    assert e.value.code == -1
    with pytest.raises(lpm.LpmError) as e:                      # cut after conv1 (before its pool) is not allowed
        lpm.lpm_partition(L, 2, cp, fixed_starts=[0, 1, 8])
    assert e.value.code == -6
    bad = [dict(l) for l in L]
    bad[2]["cin"] = 7                                            # does not match the pool output
    with pytest.raises(lpm.LpmError) as e:
        lpm.lpm_partition(bad, 2, cp)
    assert e.value.code == -2
    bad = [dict(l) for l in L]
    bad[1]["h_in"] = bad[1]["w_in"] = 23
    bad[0]["kh"] = bad[0]["kw"] = 6                              # 28-6+1 = 23: odd extent into a 2x2 pool
    with pytest.raises(lpm.LpmError) as e:
        lpm.lpm_partition(bad, 2, cp)
    assert e.value.code == -2
    with pytest.raises(lpm.LpmError) as e:                      # a loss layer cannot be a stage by itself
        lpm.Stage(L, 7, 8, 8, lpm.F32)
    assert e.value.code == -2
    with pytest.raises(lpm.LpmError) as e:
        lpm.Stage(L, 0, 4, 0, lpm.F32)
    assert e.value.code == -1
    R = wl.tiny_resnet()
    with pytest.raises(lpm.LpmError) as e:                      # cutting inside a residual block
        lpm.Stage(R, 0, 2, 4, lpm.F32)
    assert e.value.code == -2
    # NULL and misaligned pointers are rejected before anything is enqueued (no device needed)
    s = lpm.Stage(L, 0, 4, 8, lpm.F32)
    with pytest.raises(lpm.LpmError) as e:
        s.forward(None, 256, None, None, 256, None, 256, 256, 1.0)
    assert e.value.code == -1
    with pytest.raises(lpm.LpmError) as e:
        s.forward(256, 256 + 64, None, None, 256, None, 256, 256, 1.0)
    assert e.value.code == -3
    with pytest.raises(lpm.LpmError) as e:
        s.update(256, None, 512, 130, 0.1, 0.9)
    assert e.value.code == -3
    with pytest.raises(lpm.LpmError) as e:
        lpm.lpm_conv_ws_bytes(dict(m=1, h=4, w=4, cin=8, cout=8, kh=5, kw=5, stride=1, pad=0), lpm.BF16)
    assert e.value.code == -2
    # layer-wise partitioning: the shape checks come before any device object is made
    g = dict(m=2, h=8, w=8, cin=32, cout=64, kh=3, kw=3, stride=1, pad=1)
    for n, code in ((1, -1), (9, -1), (3, -2)):
        with pytest.raises(lpm.LpmError) as e:
            lpm.Layerwise(g, lpm.BF16, n)
        assert e.value.code == code
    with pytest.raises(lpm.LpmError) as e:                      # 15 channels per sub-layer
        lpm.Layerwise(dict(g, cout=60), lpm.BF16, 4)
    assert e.value.code == -2
    with pytest.raises(lpm.LpmError) as e:
        lpm.Layerwise(dict(g, kh=11, kw=11), lpm.BF16, 2)
    assert e.value.code == -2


def test_stage_layout(lpm):
    L = wl.vgg16_cifar()
    s = lpm.Stage(L, 8, 12, 16, lpm.BF16)        # conv 256, pool, conv 512 x2
    assert s.in_bytes == 16 * 256 * 8 * 8 * 2 and s.out_bytes == 16 * 512 * 4 * 4 * 2
    seen = []
    for i in (8, 10, 11):
        ow, nw = s.param_offset(i, 0)
        ob, nb = s.param_offset(i, 1)
        assert nw == L[i]["cout"] * L[i]["cin"] * 9 and nb == L[i]["cout"]
        assert ow % 64 == 0 and ob % 64 == 0
        seen += [(ow, nw), (ob, nb)]
        assert not s.has_param(i, 2)
    assert not s.has_param(9, 0)
    seen.sort()
    assert all(a + n <= b for (a, n), (b, _) in zip(seen[:-1], seen[1:]))
    assert s.grad_bytes == 4 * (seen[-1][0] + 512) and s.param_bytes == s.grad_bytes
    assert s.lowp_bytes >= s.grad_bytes // 2 + 2 * sum(n for (_, n) in seen if n > 512)   # mirror + transposed copies
    # internal tensors 8, 9, 10 are stashed; the stage output (11) and input (7) are the caller's
    offs = [s.stash_offset(t) for t in (8, 9, 10)]
    assert offs[0][1] == 16 * 256 * 8 * 8 * 2 and offs[1][1] == 16 * 256 * 4 * 4 * 2 and offs[2][1] == 16 * 512 * 4 * 4 * 2
    with pytest.raises(lpm.LpmError):
        s.stash_offset(11)
    R = wl.resnet18_cifar()
    s = lpm.Stage(R, 0, 5, 32, lpm.BF16)
    assert s.has_param(0, 2) and s.param_bytes > s.grad_bytes          # frozen scales sit after the trainable part
    o_s, _ = s.param_offset(0, 2)
    assert o_s * 4 >= s.grad_bytes


def test_binding_rejects_undersized_operands(lpm):
    """The C ABI takes plain pointers, so the binding checks a tensor's size against the geometry before the library's
    kernels would read or write past its end (CPU tensors: the check comes before any GPU work)."""
    import torch
    g3 = dict(m=2, h=8, w=8, cin=32, cout=64, kh=3, kw=3, stride=1, pad=1, d=8, kd=3, pad_d=1)
    gg = lpm.binding._geom(g3)
    xb, yb, wb, db = lpm.binding._conv_sizes(gg, lpm.BF16)
    assert (xb, yb, wb, db) == (2 * 8 * 8 * 8 * 32 * 2, 2 * 8 * 8 * 8 * 64 * 2, 64 * 27 * 32 * 2, 64 * 27 * 32 * 4)
    flat = dict(g3); del flat["d"], flat["kd"], flat["pad_d"]
    x2 = torch.zeros(2 * 8 * 8 * 32, dtype=torch.bfloat16)                # sized for one slice: too small for the volume
    w3 = torch.zeros(64 * 27 * 32, dtype=torch.bfloat16)
    y3 = torch.zeros(2 * 8 * 8 * 8 * 64, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="x holds"):
        lpm.lpm_conv_forward(g3, lpm.BF16, x2, w3, None, None, None, False, y3)
    with pytest.raises(ValueError, match="dw holds"):
        lpm.lpm_conv_wgrad(g3, lpm.BF16, torch.zeros(xb // 2, dtype=torch.bfloat16), y3, torch.zeros(10))
    with pytest.raises(ValueError, match="holds"):
        lpm.lpm_conv_time(0, g3, lpm.BF16, x2, w3, w3, y3, torch.zeros(db // 4), torch.zeros(256, dtype=torch.uint8))
    assert lpm.binding._conv_sizes(lpm.binding._geom(flat), lpm.F32)[0] == 2 * 8 * 8 * 32 * 4

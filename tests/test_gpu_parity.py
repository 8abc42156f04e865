"""GPU parity: the HIP library against the fp64 oracle, element by element, through the C ABI."""
import numpy as np
import pytest

import workloads as wl
from workloads import rng
from oracle import lpm_oracle as orc
from harness import oracle_step, gpu_step, compare, rel_err, l2_err, stage_backward_isolated
import flipnoise as fn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lpm():
    import torch
    assert torch.cuda.is_available()
    import paper_2207_11019_amd as lpm
    return lpm


def _starts(layers, Z):
    allowed = [i + 1 for i, l in enumerate(layers[:-1]) if l["cut_after"]]
    pick = [allowed[(k + 1) * len(allowed) // Z - 1] for k in range(Z - 1)] if Z > 1 else []
    return [0] + sorted(set(pick)) + [len(layers)]


CASES = [
    # name, builder, batch, M, Z, dtype, modes
    ("tiny_lenet_f32", wl.tiny_lenet, 8, 4, 3, 0),
    ("tiny_resnet_f32", wl.tiny_resnet, 6, 3, 2, 0),
    ("tiny_vgg_f32", wl.tiny_vgg, 8, 2, 3, 0),
    ("tiny_lenet_bf16", wl.tiny_lenet, 8, 4, 3, 1),
    ("tiny_resnet_bf16", wl.tiny_resnet, 6, 3, 2, 1),
    ("tiny_vgg_bf16", wl.tiny_vgg, 8, 2, 3, 1),
    # a 512 x 64 fully connected layer at 2 samples per micro-batch: its weight gradient is contracted once per mini-batch
    ("tiny_fc_bf16", wl.tiny_fc, 8, 4, 2, 1),
    ("tiny_fc_bf16_one_stage", wl.tiny_fc, 6, 3, 1, 1),
    # 64-channel convolutions over 4x4 and 2x2 images: the same for convolutions
    ("tiny_wide_bf16", wl.tiny_wide, 8, 4, 2, 1),
    # a split forward reduction into 72 channels whose second kernel also pools
    ("tiny_deep_pool_bf16", wl.tiny_deep_pool, 16, 2, 1, 1),
    # the volumetric use case: 3x3x3 residual blocks, a strided block with a 1x1x1 projection, a residual self-attention block
    ("tiny_conv3d_f32", wl.tiny_conv3d, 4, 2, 3, 0),
    ("tiny_conv3d_bf16", wl.tiny_conv3d, 4, 2, 3, 1),
    ("tiny_conv3d_mfma_bf16", wl.tiny_conv3d_mfma, 4, 2, 2, 1),       # 32 / 64 channels: the matrix-core kernels
]


@pytest.mark.parametrize("name,builder,batch,M,Z,dtype", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("mode", [0, 1, 17, 2], ids=["locked", "overlapped", "overlapped_graph", "pipelined"])
def test_small_networks(lpm, name, builder, batch, M, Z, dtype, mode):
    layers = builder()
    starts = _starts(layers, Z)
    print("case", name, "starts", starts, "mode", mode, flush=True)
    o = oracle_step(layers, starts, batch, M, dtype == 1, seed=101, lr=0.05, mu=0.9)
    net = gpu_step(lpm, layers, starts, batch, M, dtype, o, 0.05, 0.9, mode)
    compare(net, layers, starts, M, dtype, o)


@pytest.mark.parametrize("window", [1, 3, 4])
@pytest.mark.parametrize("mode", [1, 2, 17], ids=["overlapped", "pipelined", "overlapped_graph"])
def test_other_windows(lpm, window, mode):
    """Window 1 (no overlap), and windows wider than the two copies of the backward scratch (the explicit
    wait on micro-batch j-2), with more micro-batches than slots and fewer."""
    layers = wl.tiny_vgg()
    starts = _starts(layers, 3)
    for batch, M in ((12, 6), (4, 2)):
        print("window", window, "mode", mode, "M", M, flush=True)
        o = oracle_step(layers, starts, batch, M, False, seed=31, lr=0.05, mu=0.9)
        net = gpu_step(lpm, layers, starts, batch, M, 0, o, 0.05, 0.9, mode, window=window)
        compare(net, layers, starts, M, 0, o, window=window)


@pytest.mark.parametrize("mode", [0, 1, 2, 17], ids=["locked", "overlapped", "pipelined", "overlapped_graph"])
def test_single_microbatch(lpm, mode):
    """M = 1: nothing to overlap and nothing to accumulate; every schedule is plain backpropagation on the batch."""
    layers = wl.tiny_vgg()
    for Z in (1, 3):
        starts = _starts(layers, Z)
        o = oracle_step(layers, starts, 4, 1, True, seed=41, lr=0.05, mu=0.9)
        net = gpu_step(lpm, layers, starts, 4, 1, 1, o, 0.05, 0.9, mode)
        compare(net, layers, starts, 1, 1, o)


def test_stage_without_parameters(lpm):
    """A partition made of a pooling layer alone: nothing to update, no weight gradient, gradients pass through."""
    layers = wl.tiny_vgg()
    pool = [i for i, l in enumerate(layers) if l["kind"] == "maxpool2"][0]
    starts = [0, pool, pool + 1, len(layers)]
    for dtype in (0, 1):
        o = oracle_step(layers, starts, 8, 2, dtype == 1, seed=37, lr=0.05, mu=0.9)
        for mode in (lpm.LOCKED, lpm.OVERLAPPED, lpm.PIPELINED):
            net = gpu_step(lpm, layers, starts, 8, 2, dtype, o, 0.05, 0.9, mode)
            compare(net, layers, starts, 2, dtype, o)


def test_maxpool_backward_full_size_with_ties(lpm):
    """Pooling backward at the 224x224 VGG-16's first pooling size (4 x 64 x 224 x 224) as a stage of its own, on an input
    quantised to multiples of 1/4 so that many windows hold their maximum twice or more: the gradient must land on the
    first maximum in row-major window order, bit for bit; the 2x2 window sums of the result equal the incoming gradient
    whichever element received it.  The count of tie windows is printed."""
    import torch
    import flipnoise as fn
    layers = [dict(kind="maxpool2", cin=64, cout=64, kh=2, kw=2, stride=2, pad=0, h_in=224, w_in=224, relu=False, bias=False,
                   scale=False, src=-1, add_src=None, cut_after=False)]
    m = 4
    x = np.round(rng.normal(3, 1, (m, 64, 224, 224)) * 4.0) / 4.0
    dy = rng.round_to_bf16(rng.normal(3, 2, (m, 64, 112, 112)))
    win = x.reshape(m, 64, 112, 2, 112, 2).transpose(0, 1, 2, 4, 3, 5).reshape(m, 64, 112, 112, 4)
    ties = int(((win == win.max(axis=-1, keepdims=True)).sum(axis=-1) > 1).sum())
    print("windows whose maximum occurs more than once: %d of %d" % (ties, win.shape[0] * 64 * 112 * 112), flush=True)
    assert ties > 100000
    want = orc.maxpool2_bwd(x, dy)
    net = lpm.Net(layers, [0, 1], m, 1, lpm.BF16, dx_wanted=True)
    for mode in (lpm.LOCKED, lpm.OVERLAPPED):
        net.step(lpm.pack_act(x, lpm.BF16), None, lpm.pack_act(dy, lpm.BF16), 0.0, 0.0, mode)
        torch.cuda.synchronize()
        got = net.read_grad_in(0, 0)
        np.testing.assert_array_equal(fn.window_sums(got), dy)
        np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(net.read_act_out(0, 0), orc.maxpool2_fwd(x))


def test_pipelined_graph_is_refused(lpm):
    """Stage-parallel streams are not captured into a graph: the call fails before anything is enqueued."""
    layers = wl.tiny_lenet()
    starts = _starts(layers, 2)
    import torch
    net = lpm.Net(layers, starts, 2, 2, 0)
    x = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(Exception, match="LPM_GRAPH"):
        net.step(x, None, None, 0.1, 0.0, lpm.PIPELINED | lpm.GRAPH)


ASYNC = [
    # name, builder, batch, M, Z, dtype
    ("tiny_lenet_f32", wl.tiny_lenet, 8, 4, 3, 0),
    ("tiny_resnet_f32_odd", wl.tiny_resnet, 6, 3, 2, 0),
    # bf16: a network without ReLU / max-pooling.  After an update the bf16 weight copies of the two sides differ
    # in a few last bits, and with a handful of samples per micro-batch the sign / maximum decisions of a ReLU
    # network turn that into 10-50 % changes of the next gradient (measured on the oracle against itself).
    ("tiny_linear_bf16", wl.tiny_linear, 8, 4, 2, 1),
]


@pytest.mark.parametrize("name,builder,batch,M,Z,dtype", ASYNC, ids=[c[0] for c in ASYNC])
@pytest.mark.parametrize("sched", ["locked", "overlapped_w1", "overlapped_w2"])
def test_async_update(lpm, name, builder, batch, M, Z, dtype, sched):
    """One update per micro-batch: plain per-micro-batch SGD when nothing overlaps, forward passes one update
    behind with two micro-batches in flight."""
    from harness import oracle_step_async, compare_async
    layers = builder()
    starts = _starts(layers, Z)
    window = 1 if sched == "overlapped_w1" else 2
    mode = (lpm.LOCKED if sched == "locked" else lpm.OVERLAPPED) | lpm.ASYNC_UPDATE
    print("async case", name, sched, "starts", starts, flush=True)
    o = oracle_step_async(layers, starts, batch, M, dtype == 1, seed=23, lr=0.05, mu=0.9, window=window, locked=sched == "locked")
    net = gpu_step(lpm, layers, starts, batch, M, dtype, o, 0.05, 0.9, mode, window=window)
    compare_async(net, dtype, o)


@pytest.mark.parametrize("sched", ["locked", "overlapped_w2"])
def test_async_update_bf16_relu_network(lpm, sched):
    """The per-micro-batch update in bf16 on a network WITH ReLU and max-pooling (tiny_vgg, 4 micro-batches of 2).
    After the first update the two sides' bf16 weight copies differ in a few last bits, which can flip decisions of
    later micro-batches; each tensor is therefore held to the bar plus twice the decision-flip noise floor of this
    very case, measured on the oracle (eight realisations of accumulation-order noise, harness.async_floors)."""
    from harness import oracle_step_async, compare_async, async_floors
    layers = wl.tiny_vgg()
    starts = _starts(layers, 2)
    window, locked = (2, False) if sched == "overlapped_w2" else (2, True)
    mode = (lpm.LOCKED if locked else lpm.OVERLAPPED) | lpm.ASYNC_UPDATE
    o = oracle_step_async(layers, starts, 8, 4, True, seed=23, lr=0.05, mu=0.9, window=window, locked=locked)
    floors = async_floors(layers, starts, 8, 4, 23, 0.05, 0.9, window, locked, o, realisations=16)
    print("largest floors", sorted(floors.items(), key=lambda kv: -kv[1])[:5], flush=True)
    net = gpu_step(lpm, layers, starts, 8, 4, 1, o, 0.05, 0.9, mode, window=window)
    # With two samples per micro-batch one flipped decision moves the last micro-batch's gradient (and the momentum, which
    # adds it with weight 1) by tens of per cent, and sixteen realisations sample that floor only coarsely: those tensors are
    # printed with their floors; the loss and the final weights -- four updates deep -- are held to the bar plus twice
    # their floor.  The exact check of the version rule is the device-side identity below (locked) and the ReLU-free
    # network of test_async_update (overlapped).
    held = {k: v for k, v in floors.items() if k == "loss" or k.startswith("param")}
    errs = compare_async(net, 1, o, floors=dict(held, **{k: 1e9 for k in floors if k not in held}))
    print("largest errors (error, floor)", [(k, round(e, 4), round(floors.get(k, 0.0), 4)) for k, e in sorted(errs.items(), key=lambda kv: -kv[1])[:6]],
          flush=True)
    if locked:
        # nothing overlaps: the pass is M synchronous steps on mini-batches of m samples, one after the other -- on the device
        # too (the same kernels except where a schedule contracts a weight gradient over a group of micro-batches: compared to 1e-5)
        ref = lpm.Net(layers, starts, 2, 1, 1)
        ref.load_params(o["p0"], o["m0"])
        import torch
        for j in range(4):
            xj = lpm.pack_act(o["x"][2 * j:2 * j + 2], 1)
            lj = torch.from_numpy(o["labels"][2 * j:2 * j + 2]).to("cuda:0")
            ref.step(xj, lj, None, 0.05, 0.9, lpm.LOCKED)
        torch.cuda.synchronize()
        a, b = net.read_params(), ref.read_params()
        for i in a:
            for k in a[i]:
                assert rel_err(a[i][k], b[i][k]) <= 1e-5, (i, k)


def test_lenet_config_f32(lpm):
    """The LeNet workload at its full size: batch 32, 4 micro-batches of 8, 2 partitions, lr 0.01, momentum 0.9."""
    layers = wl.lenet()
    cp = dict(lpm.MI355X_COST["f32"], link_byte_per_us=0, microbatch=8, n_microbatch=4)
    starts, _ = lpm.lpm_partition(layers, 2, cp)
    assert starts == [0, 4, 8]
    o = oracle_step(layers, starts, 32, 4, False, seed=7, lr=0.01, mu=0.9)
    nets = {}
    for mode in (lpm.LOCKED, lpm.OVERLAPPED, lpm.PIPELINED):
        print("lenet mode", mode, flush=True)
        nets[mode] = gpu_step(lpm, layers, starts, 32, 4, 0, o, 0.01, 0.9, mode)
        compare(nets[mode], layers, starts, 4, 0, o)
    # the schedules are bitwise identical
    a = nets[lpm.LOCKED].read_params()
    for mode in (lpm.OVERLAPPED, lpm.PIPELINED):
        b = nets[mode].read_params()
        for i in a:
            for k in a[i]:
                np.testing.assert_array_equal(a[i][k], b[i][k])
        assert nets[lpm.LOCKED].loss_value() == nets[mode].loss_value()


def test_overlapped_on_changing_streams(lpm):
    """OVERLAPPED picks the weight phases' streams for the caller's pair of streams at the first run on that pair:
    steps on a second pair, on the first pair again and with the two streams swapped must all give LOCKED's bits."""
    import torch
    layers = wl.tiny_vgg()
    starts = _starts(layers, 2)
    o = oracle_step(layers, starts, 8, 4, True, seed=9, lr=0.05, mu=0.9)
    ref = gpu_step(lpm, layers, starts, 8, 4, 1, o, 0.05, 0.9, lpm.LOCKED)
    compare(ref, layers, starts, 4, 1, o)
    a = ref.read_params()
    net = lpm.Net(layers, starts, 2, 4, 1)
    xd = lpm.pack_act(o["x"], 1)
    ld = torch.from_numpy(o["labels"]).to("cuda:0")
    first = (net.stream_fwd, net.stream_bwd)
    second = (torch.cuda.Stream(), torch.cuda.Stream())
    for k, (sf, sb) in enumerate((first, second, first, (second[1], second[0]))):
        print("stream pair", k, flush=True)
        net.stream_fwd, net.stream_bwd = sf, sb
        net.load_params(o["p0"], o["m0"])
        net.step(xd, ld, None, 0.05, 0.9, lpm.OVERLAPPED)
        torch.cuda.synchronize()
        b = net.read_params()
        for i in a:
            for key in a[i]:
                np.testing.assert_array_equal(a[i][key], b[i][key])
        assert ref.loss_value() == net.loss_value()


@pytest.mark.parametrize("dtype", [0, 1], ids=["f32", "bf16"])
def test_adam_update(lpm, dtype):
    """lpm_stage_update_adam against the oracle's Adam: three steps with a new gradient each, every stage of a
    small network; for bf16 the low-precision copy must be the rounded new weights."""
    import copy
    import torch
    layers = wl.tiny_vgg()
    starts = _starts(layers, 2)
    params, _ = wl.make_params(layers, 21, bf16=bool(dtype), bias_std=0.05, momentum_std=0.0)
    net = lpm.Net(layers, starts, 2, 4, dtype)
    zeros = {i: {k: np.zeros_like(v) for k, v in p.items() if k != "s"} for i, p in params.items()}
    net.load_params(params, zeros)                      # the momentum buffer serves as the first moment
    second = [torch.zeros_like(b["momentum"]) for b in net.bufs]
    ref_p, ref_m1, ref_m2 = copy.deepcopy(params), copy.deepcopy(zeros), copy.deepcopy(zeros)
    # the C ABI takes the hyper-parameters as floats: both sides get the float values (1 - 0.999 differs from
    # 1 - float(0.999) by 1.3e-5 of itself, which would show in the second moment)
    lr, b1, b2, eps = (float(np.float32(v)) for v in (0.01, 0.9, 0.999, 1e-8))
    for t in (1, 2, 3):
        grads = {i: {k: rng.normal(100 + t, 10 * i + j, v.shape, 0.0, 10.0 ** (t - 3)).astype(np.float32).astype(np.float64)
                     for j, (k, v) in enumerate(p.items()) if k != "s"} for i, p in params.items()}
        net._write("grads", grads, ("W", "b"))
        for z, st in enumerate(net.stages):
            b = net.bufs[z]
            st.update_adam(b["params"], b["lowp"], b["grads"], b["momentum"], second[z], lr, b1, b2, eps, t)
        torch.cuda.synchronize()
        orc.adam(ref_p, grads, ref_m1, ref_m2, lr, b1, b2, eps, t)
        got_p, got_m1 = net.read_params(), net.read_momentum()
        for i in ref_p:
            for k in ("W", "b"):
                if k in ref_p[i]:
                    assert rel_err(got_p[i][k], ref_p[i][k]) <= 1e-5, (t, i, k)
                    assert rel_err(got_m1[i][k], ref_m1[i][k]) <= 1e-5, (t, i, k)
    # second moments: read them through the same unpacking by lending the buffers to the net
    for z, b in enumerate(net.bufs):
        b["momentum"], second[z] = second[z], b["momentum"]
    got_m2 = net.read_momentum()
    for i in ref_m2:
        for k in ref_m2[i]:
            assert rel_err(got_m2[i][k], ref_m2[i][k]) <= 1e-5, (i, k)
    if dtype == 1:
        for z, st in enumerate(net.stages):
            n = st.param_bytes // 4
            p32 = net.bufs[z]["params"].view(torch.float32)[:n]
            low = net.bufs[z]["lowp"].view(torch.bfloat16)[:n]
            # the mirrored region covers the trainable parameters, which come first
            off, cnt = st.param_offset(st.first, 0)
            assert torch.equal(low[off:off + cnt], p32[off:off + cnt].to(torch.bfloat16))
    with pytest.raises(lpm.LpmError):
        net.stages[0].update_adam(net.bufs[0]["params"], net.bufs[0]["lowp"], net.bufs[0]["grads"], net.bufs[0]["momentum"],
                                  second[0], lr, b1, b2, eps, 0)


def test_two_steps_with_momentum(lpm):
    layers = wl.tiny_vgg()
    starts = _starts(layers, 2)
    o = oracle_step(layers, starts, 8, 4, False, seed=5, lr=0.05, mu=0.9, steps=2)
    net = gpu_step(lpm, layers, starts, 8, 4, 0, o, 0.05, 0.9, lpm.OVERLAPPED, steps=2)
    compare(net, layers, starts, 4, 0, o)


@pytest.mark.parametrize("dtype", [0, 1], ids=["f32", "bf16"])
def test_partition_with_upstream_gradient(lpm, dtype):
    """A bottleneck-block partition fed by an activation and an upstream gradient (all data gradients needed)."""
    layers = wl.r50_conv4x(cin=16, hw=12, mid=8, cout=32, blocks=2)
    starts = [0, len(layers)]
    o = oracle_step(layers, starts, 4, 1, dtype == 1, seed=13, lr=0.05, mu=0.9, dx_wanted=True)
    net = gpu_step(lpm, layers, starts, 4, 1, dtype, o, 0.05, 0.9, lpm.LOCKED, dx_wanted=True)
    compare(net, layers, starts, 1, dtype, o, dx_wanted=True)


# (tiny_resnet in bf16 is left out: with two thirds of its 4 - 6 channels silenced its bias gradients are sums that cancel to a
#  few per cent of their terms, and storing activation gradients in bf16 -- which the oracle does not -- then shows as 3 - 5 %
#  of the result; the same rounding applied inside the oracle reproduces those figures)
@pytest.mark.parametrize("net,dtype", [("bottleneck32", 0), ("bottleneck32", 1), ("tiny_resnet", 0)],
                         ids=["bottleneck32-f32", "bottleneck32-bf16", "tiny_resnet-f32"])
def test_zero_and_tiny_scales(lpm, net, dtype):
    """Frozen per-channel scales of exactly 0 and of 1e-20 (a zero-initialised folded normalisation is a legal value):
    the bias gradient is the sum of the masked output gradient whatever the scale (eq. 8 for the bias), the weight
    gradient of a zero-scale channel is 0, and nothing is divided by a scale.  bottleneck32: 32- and 64-channel
    bottleneck blocks (matrix-core kernels, fused epilogue backward); tiny_resnet: 4 and 6 channels (generic kernels)."""
    if net == "bottleneck32":
        layers = wl.r50_conv4x(cin=64, hw=8, mid=32, cout=64, blocks=2)
        batch, M, dx = 8, 2, True
    else:
        layers = wl.tiny_resnet()
        batch, M, dx = 6, 3, False
    starts = [0, len(layers)]

    def mutate(params):
        for i, p in params.items():
            if "s" in p:
                p["s"][0::3] = 0.0
                p["s"][1::3] = 1e-20

    o = oracle_step(layers, starts, batch, M, dtype == 1, seed=29, lr=0.05, mu=0.9, dx_wanted=dx, mutate=mutate)
    for mode in (lpm.LOCKED, lpm.OVERLAPPED):
        net_ = gpu_step(lpm, layers, starts, batch, M, dtype, o, 0.05, 0.9, mode, dx_wanted=dx)
        errs = compare(net_, layers, starts, M, dtype, o, dx_wanted=dx)
        g = net_.read_grads()
        for i in g:
            for k in g[i]:
                assert np.isfinite(g[i][k]).all(), (i, k)
        # the bias gradient of zero-scale channels is generally not zero, and must match the oracle's
        i0 = [i for i in o["params"] if "s" in o["params"][i]][0]
        assert np.abs(o["ref"]["grads"][i0]["b"][0::3]).max() > 0
        print(net, dtype, mode, "worst", sorted(errs.items(), key=lambda kv: -kv[1])[:3], flush=True)


def test_vgg16_cifar_config_bf16(lpm):
    """The VGG-16/CIFAR workload at full size (batch 128, 8 micro-batches of 16, 4 planned partitions).

    Forward quantities are compared end to end, against the storage-precision oracle run and against the unrounded
    one.  Backward: (a) end to end against the unrounded fp64 step, each gradient tensor held to the bar plus twice the
    decision-flip noise floor of this workload (the distance between the two oracle runs; mechanism pinned by
    tests/test_oracle_flip_noise.py: over 13 bf16 layers ReLU / pooling decisions are not stable against last-bit
    differences, on either side); (b) element-wise at the bar, stage by stage from a forward state prepared by the
    oracle (harness.stage_backward_isolated), where both sides decide on identical stored values."""
    layers = wl.vgg16_cifar()
    cp = dict(lpm.MI355X_COST["bf16"], link_byte_per_us=0, microbatch=16, n_microbatch=8)
    starts, _ = lpm.lpm_partition(layers, 4, cp)
    print("vgg16_cifar plan", starts, flush=True)
    o = oracle_step(layers, starts, 128, 8, True, seed=11, lr=0.01, mu=0.9, bias_std=0.0, momentum_std=0.0)
    print("oracle done", flush=True)
    rep = {}
    nets = {}
    for mode in (lpm.LOCKED, lpm.OVERLAPPED | lpm.GRAPH, lpm.PIPELINED):
        nets[mode] = gpu_step(lpm, layers, starts, 128, 8, 1, o, 0.01, 0.9, mode)
        compare(nets[mode], layers, starts, 8, 1, o, report=rep, backward=False)
        print("mode", mode, "worst", sorted(rep.items(), key=lambda kv: -kv[1])[:5], flush=True)
    a = nets[lpm.LOCKED].read_params()
    for mode in nets:
        b = nets[mode].read_params()
        for i in a:
            for k in a[i]:
                np.testing.assert_array_equal(a[i][k], b[i][k])
    # End-to-end gradients against the unrounded fp64 step.  The bound per tensor is the bar plus twice the distance between
    # the two oracle runs (stored activations rounded to bf16, or not): a second valid bf16 result is that far from the
    # unrounded one (tests/test_oracle_flip_noise.py); the element-wise bar itself is applied per stage below.
    g = nets[lpm.LOCKED].read_grads()
    A, B = o["plain"]["ref"]["grads"], o["ref"]["grads"]
    over = []
    for i in g:
        for k in g[i]:
            f_inf, f_l2 = fn.inf_err(B[i][k], A[i][k]), fn.l2_err(B[i][k], A[i][k])
            e_inf, e_l2 = fn.inf_err(g[i][k], A[i][k]), fn.l2_err(g[i][k], A[i][k])
            print("end-to-end grad%d.%s: error %.4f (floor %.4f), 2-norm %.4f (floor %.4f)" % (i, k, e_inf, f_inf, e_l2, f_l2), flush=True)
            if not (e_inf <= 2e-2 + 2 * f_inf and e_l2 <= 2e-2 + 2 * f_l2):
                over.append((i, k, e_inf, f_inf, e_l2, f_l2))
    assert not over, over
    del nets
    rep = {}
    stage_backward_isolated(lpm, layers, starts, 16, 128, 1, seed=11, report=rep)
    print("isolated backward worst", sorted(rep.items(), key=lambda kv: -kv[1])[:5], flush=True)


FULL = [
    # name, builder, plan, micro-batch, mini-batch, upstream gradient wanted
    ("resnet18_cifar", wl.resnet18_cifar, [0, 5, 10, 15, 23], 32, 256, False),
    ("resnet34_cifar", wl.resnet34_cifar, [0, 7, 16, 29, 39], 32, 256, False),
    ("r50_conv4x", wl.r50_conv4x, [0, 19], 16, 64, True),
    ("vgg16_224", wl.vgg16_224, [0, 10, 18, 19, 22], 4, 32, False),
    # a 3D-ResAttNet18-shaped network on 32^3 one-channel volumes, two volumes per micro-batch (plan: the cost model's, 4 partitions)
    ("resattnet18_3d", wl.resattnet18_3d, None, 2, 6, False),
]


@pytest.mark.parametrize("name,builder,plan,m,batch,dx", FULL, ids=[f[0] for f in FULL])
def test_full_size_microbatch_bf16(lpm, name, builder, plan, m, batch, dx):
    """One micro-batch of each remaining workload at its real shape: the device's forward pass against the
    oracle's, then B of every stage from the oracle's forward state (element-wise, 2e-2 of each tensor's
    infinity norm).  VGG-16/224 uses the described plan (conv1-3 | conv4-5 | FC1 | FC2-3)."""
    layers = builder()
    rep = {}
    if plan is None:
        plan, _ = lpm.lpm_partition(layers, 4, dict(lpm.MI355X_COST["bf16"], link_byte_per_us=0, microbatch=m, n_microbatch=batch // m))
    print("workload", name, "plan", plan, flush=True)
    stage_backward_isolated(lpm, layers, plan, m, batch, 1, seed=17, dx_wanted=dx, report=rep, check_forward=True)
    print(name, "worst", sorted(rep.items(), key=lambda kv: -kv[1])[:6], flush=True)

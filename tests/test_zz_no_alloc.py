"""lpm_conv_wgrad_static (the weight gradient with the library's built-in scratch area, for callers that cannot
allocate) against lpm_conv_wgrad with a caller workspace: same kernels, so the same bits, and both against the
oracle's direct loops.  Two calls in a row share the area; the second is smaller than the first."""
import numpy as np
import pytest

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


def _case(lpm, torch, g, dtype, seed):
    l = dict(kind="conv", cin=g["cin"], cout=g["cout"], kh=g["kh"], kw=g["kw"], stride=g["stride"], pad=g["pad"],
             h_in=g["h"], w_in=g["w"], relu=False, bias=False, scale=False, src=-1, add_src=None, cut_after=False)
    q = rng.round_to_bf16 if dtype == lpm.BF16 else (lambda a: a)
    x = q(rng.normal(seed, 1, (g["m"], g["cin"], g["h"], g["w"])))
    ho = (g["h"] + 2 * g["pad"] - g["kh"]) // g["stride"] + 1
    wo = (g["w"] + 2 * g["pad"] - g["kw"]) // g["stride"] + 1
    dz = q(rng.normal(seed, 3, (g["m"], g["cout"], ho, wo)))
    wshape = (g["cout"], g["cin"], g["kh"], g["kw"])
    dw0 = rng.normal(seed, 8, wshape).astype(np.float32).astype(np.float64)
    return dict(g=g, xd=lpm.pack_act(x, dtype), dzd=lpm.pack_act(dz, dtype), dw0=dw0, wshape=wshape,
                ref=orc.conv_bwd_weight(x, dz, l))


def test_static_scratch_weight_gradient(lpm):
    import torch
    big = dict(m=4, h=28, w=28, cin=64, cout=96, kh=3, kw=3, stride=1, pad=1)      # split partials, patch-based kernel
    small = dict(m=32, h=4, w=4, cin=64, cout=64, kh=3, kw=3, stride=1, pad=1)     # smaller partials, the pixel-tiled kernel
    f32 = dict(m=4, h=9, w=7, cin=5, cout=7, kh=3, kw=3, stride=2, pad=1)          # float path (generic kernels)
    cases = [(big, lpm.BF16), (small, lpm.BF16), (f32, lpm.F32), (big, lpm.BF16)]
    assert lpm.lpm_conv_ws_bytes(big, lpm.BF16)[2] > lpm.lpm_conv_ws_bytes(small, lpm.BF16)[2] > 0
    st = torch.cuda.Stream()
    data = [_case(lpm, torch, g, dt, 11 + k) for k, (g, dt) in enumerate(cases)]
    for accumulate in (False, True):
        outs = []
        # the calls follow each other on one stream with no synchronisation in between: they share the area in stream order
        for d, (g, dt) in zip(data, cases):
            dw = torch.from_numpy(lpm.pack_weight(d["dw0"])).cuda()
            torch.cuda.synchronize()
            outs.append(dw)
        for d, (g, dt), dw in zip(data, cases, outs):
            print("static weight gradient", g, "dtype", dt, "accumulate", accumulate, flush=True)
            lpm.lpm_conv_wgrad_static(g, dt, d["xd"], d["dzd"], dw, accumulate, st)
        st.synchronize()
        for d, (g, dt), dw in zip(data, cases, outs):
            ws = torch.zeros(max(lpm.lpm_conv_ws_bytes(g, dt)[2], 256), dtype=torch.uint8, device="cuda")
            ref_dw = torch.from_numpy(lpm.pack_weight(d["dw0"])).cuda()
            lpm.lpm_conv_wgrad(g, dt, d["xd"], d["dzd"], ref_dw, accumulate, ws, st)
            st.synchronize()
            assert torch.equal(dw, ref_dw), g                      # same kernels, same summation order: same bits
            want = d["ref"] + (d["dw0"] if accumulate else 0.0)
            tol = 1e-3 if dt == lpm.BF16 else 1e-4
            assert rel_err(lpm.unpack_weight(dw.cpu().numpy(), d["wshape"]), want) <= tol, g


def test_static_scratch_rejects_oversize(lpm):
    import torch
    # a 256 -> 256 channel 3x3 layer over 16 images of 14x14: five pixel ranges x 2.36 MB of partial sums
    g = dict(m=16, h=14, w=14, cin=256, cout=256, kh=3, kw=3, stride=1, pad=1)
    need = lpm.lpm_conv_ws_bytes(g, lpm.BF16)[2]
    assert need > lpm.STATIC_SCRATCH_BYTES
    x = torch.zeros(16 * 14 * 14 * 256, dtype=torch.bfloat16, device="cuda")          # operands of the right size: the call is
    dw = torch.zeros(256 * 9 * 256, dtype=torch.float32, device="cuda")              # refused for its scratch need alone
    with pytest.raises(lpm.LpmError) as e:
        lpm.lpm_conv_wgrad_static(g, lpm.BF16, x, x, dw, False, None)
    assert e.value.code == -1 and "scratch" in str(e.value)

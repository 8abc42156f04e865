"""ctypes binding of liblpm.so: same names as the C ABI, argument marshalling only.

PyTorch is used for device memory and streams; no torch operator takes part in the training step.
The library is required: importing this module fails if liblpm.so has not been built
(python paper_2207_11019_amd/build.py or __graft_entry__.build()).
"""
import ctypes as C
import os

import numpy as np

__all__ = ["LpmError", "lib", "lpm_conv_geom", "lpm_conv_ws_bytes", "lpm_conv_forward", "lpm_conv_dgrad", "lpm_conv_wgrad", "lpm_conv_wgrad_static", "STATIC_SCRATCH_BYTES", "lpm_conv_time", "Layerwise", "lpm_layer", "lpm_cost_params", "lpm_stage_buffers", "layers_from_dicts",
           "lpm_layer_cost", "lpm_partition", "lpm_partition_costs", "Stage", "Schedule", "Net", "F32", "BF16", "LOCKED", "OVERLAPPED", "PIPELINED", "ASYNC_UPDATE",
           "GRAPH", "pack_act", "unpack_act", "pack_weight", "unpack_weight", "MI355X_COST"]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = os.path.join(_HERE, "liblpm.so")
if not os.path.exists(_LIB):
    raise ImportError("liblpm.so is missing: build it with `python paper_2207_11019_amd/build.py`")
lib = C.CDLL(_LIB)

F32, BF16 = 0, 1
LOCKED, OVERLAPPED, PIPELINED, GRAPH, ASYNC_UPDATE = 0, 1, 2, 16, 32
KINDS = {"conv": 0, "fc": 1, "maxpool2": 2, "gap": 3, "softmax_ce": 4, "attn": 5}
RELU, BIAS, SCALE = 1, 2, 4
NONE = -2
MAX_WINDOW = 4


class LpmError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("lpm error %d: %s" % (code, text))
        self.code = code


class lpm_layer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "cin", "cout", "kh", "kw", "stride", "pad", "h_in", "w_in", "flags",
                                         "src", "add_src", "cut_allowed_after", "d_in", "kd", "pad_d")]


class lpm_cost_params(C.Structure):
    _fields_ = [("flop_per_us", C.c_uint64), ("hbm_byte_per_us", C.c_uint64), ("link_byte_per_us", C.c_uint64),
                ("elem_bytes", C.c_int32), ("microbatch", C.c_int32), ("n_microbatch", C.c_int32)]


class lpm_stage_buffers(C.Structure):
    _fields_ = [("params", C.c_void_p), ("lowp", C.c_void_p), ("grads", C.c_void_p), ("momentum", C.c_void_p),
                ("stash", C.c_void_p * MAX_WINDOW), ("act_out", C.c_void_p * MAX_WINDOW), ("grad_in", C.c_void_p * MAX_WINDOW),
                ("fwd_ws", C.c_void_p), ("bwd_ws", C.c_void_p), ("params_alt", C.c_void_p), ("lowp_alt", C.c_void_p)]


class lpm_conv_geom(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("m", "h", "w", "cin", "cout", "kh", "kw", "stride", "pad", "d", "kd", "pad_d")]


lib.lpm_last_error.restype = C.c_char_p
_vp, _i32, _sz = C.c_void_p, C.c_int32, C.c_size_t
_psz = C.POINTER(C.c_size_t)
lib.lpm_layer_cost.argtypes = [C.POINTER(lpm_layer), _i32, _i32, C.POINTER(lpm_cost_params), C.POINTER(C.c_uint64)]
lib.lpm_partition.argtypes = [C.POINTER(lpm_layer), _i32, _i32, C.POINTER(lpm_cost_params), C.POINTER(_i32),
                              C.POINTER(_i32), C.POINTER(C.c_uint64)]
lib.lpm_partition_costs.argtypes = [C.POINTER(lpm_layer), _i32, _i32, C.POINTER(lpm_cost_params), C.POINTER(C.c_uint64),
                                    C.POINTER(_i32), C.POINTER(_i32), C.POINTER(C.c_uint64)]
lib.lpm_stage_create.argtypes = [C.POINTER(lpm_layer), _i32, _i32, _i32, _i32, _i32, C.POINTER(_vp)]
lib.lpm_stage_destroy.argtypes = [_vp]
lib.lpm_stage_sizes.argtypes = [_vp] + [_psz] * 8
lib.lpm_stage_param_offset.argtypes = [_vp, _i32, _i32, _psz, _psz]
lib.lpm_stage_stash_offset.argtypes = [_vp, _i32, _psz, _psz]
lib.lpm_stage_grad_offset.argtypes = [_vp, _i32, _psz, _psz]
lib.lpm_stage_sync_lowp.argtypes = [_vp, _vp, _vp, _vp]
lib.lpm_stage_forward.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, C.c_float, _vp]
lib.lpm_stage_backward.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]
lib.lpm_stage_update.argtypes = [_vp, _vp, _vp, _vp, _vp, C.c_float, C.c_float, _i32, _vp]
lib.lpm_stage_update_adam.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, C.c_float, C.c_float, C.c_float, C.c_float, _i32, _i32, _vp]
lib.lpm_stage_update_adam.restype = C.c_int32
lib.lpm_schedule_create.argtypes = [C.POINTER(_vp), _i32, _i32, _i32, C.POINTER(_vp)]
lib.lpm_schedule_destroy.argtypes = [_vp]
lib.lpm_schedule_cut_fused.argtypes = [_vp, _i32]
lib.lpm_schedule_run.argtypes = [_vp, _i32, _vp, _vp, _vp, C.POINTER(lpm_stage_buffers), _i32, C.c_float, C.c_float,
                                 _vp, _vp, _vp]
lib.lpm_conv_ws_bytes.argtypes = [C.POINTER(lpm_conv_geom), _i32, _psz, _psz, _psz]
lib.lpm_conv_forward.argtypes = [C.POINTER(lpm_conv_geom), _i32, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp]
lib.lpm_conv_dgrad.argtypes = [C.POINTER(lpm_conv_geom), _i32, _vp, _vp, _vp, _vp, _i32, _vp, _vp]
lib.lpm_conv_wgrad.argtypes = [C.POINTER(lpm_conv_geom), _i32, _vp, _vp, _vp, _i32, _vp, _vp]
lib.lpm_conv_wgrad_static.argtypes = [C.POINTER(lpm_conv_geom), _i32, _vp, _vp, _vp, _i32, _vp]
lib.lpm_conv_time.argtypes = [_i32, C.POINTER(lpm_conv_geom), _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp,
                              C.POINTER(C.c_float)]
lib.lpm_layerwise_create.argtypes = [C.POINTER(lpm_conv_geom), _i32, _i32, C.POINTER(_vp)]
lib.lpm_layerwise_destroy.argtypes = [_vp]
lib.lpm_layerwise_ws_bytes.argtypes = [_vp, _psz, _psz]
lib.lpm_layerwise_forward.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp]
lib.lpm_layerwise_backward.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]
lib.lpm_layerwise_time.argtypes = [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, C.POINTER(C.c_float)]
for _f in ("lpm_layerwise_create", "lpm_layerwise_destroy", "lpm_layerwise_ws_bytes", "lpm_layerwise_forward",
           "lpm_layerwise_backward", "lpm_layerwise_time", "lpm_conv_time", "lpm_conv_ws_bytes", "lpm_conv_forward", "lpm_conv_dgrad", "lpm_conv_wgrad", "lpm_conv_wgrad_static", "lpm_layer_cost", "lpm_partition", "lpm_partition_costs", "lpm_stage_create", "lpm_stage_destroy", "lpm_stage_sizes",
           "lpm_stage_param_offset", "lpm_stage_stash_offset", "lpm_stage_grad_offset", "lpm_stage_sync_lowp",
           "lpm_stage_forward", "lpm_stage_backward", "lpm_stage_update", "lpm_schedule_create",
           "lpm_schedule_destroy", "lpm_schedule_cut_fused", "lpm_schedule_run"):
    getattr(lib, _f).restype = C.c_int32

# public MI355X figures used as cost-model parameters: 2.5166 PFLOP/s bf16 MFMA, 157.3 TFLOP/s fp32, 8 TB/s HBM
MI355X_COST = {"bf16": dict(flop_per_us=2_516_582_400, hbm_byte_per_us=8_000_000, elem_bytes=2),
               "f32": dict(flop_per_us=157_286_400, hbm_byte_per_us=8_000_000, elem_bytes=4)}


def _check(rc):
    if rc != 0:
        raise LpmError(rc, lib.lpm_last_error().decode())


def layers_from_dicts(layers):
    """list of layer dicts (see workloads.configs) -> ctypes array of lpm_layer."""
    arr = (lpm_layer * len(layers))()
    for i, l in enumerate(layers):
        flags = (RELU if l.get("relu") else 0) | (BIAS if l.get("bias") else 0) | (SCALE if l.get("scale") else 0)
        add = l.get("add_src")
        arr[i] = lpm_layer(KINDS[l["kind"]], l["cin"], l["cout"], l["kh"], l["kw"], l["stride"], l["pad"], l["h_in"],
                           l["w_in"], flags, l["src"], NONE if add is None else add, 1 if l.get("cut_after") else 0,
                           l.get("d_in", 1), l.get("kd", 1), l.get("pad_d", 0))
    return arr


def _as_layers(layers):
    return layers if isinstance(layers, C.Array) else layers_from_dicts(layers)


def _cp(cp):
    return lpm_cost_params(cp["flop_per_us"], cp["hbm_byte_per_us"], cp.get("link_byte_per_us", 0), cp["elem_bytes"],
                           cp["microbatch"], cp["n_microbatch"])


def lpm_layer_cost(layers, i, cp):
    arr = _as_layers(layers)
    out = C.c_uint64()
    c = _cp(cp)
    _check(lib.lpm_layer_cost(arr, len(arr), i, C.byref(c), C.byref(out)))
    return out.value


def lpm_partition(layers, Z, cp, fixed_starts=None):
    """-> (starts[Z+1], stage_cost[Z])"""
    arr = _as_layers(layers)
    c = _cp(cp)
    starts = (C.c_int32 * (Z + 1))()
    cost = (C.c_uint64 * Z)()
    fixed = None
    if fixed_starts is not None:
        if len(fixed_starts) != Z + 1:
            raise LpmError(-1, "fixed_starts needs Z+1 entries")
        fixed = (C.c_int32 * (Z + 1))(*fixed_starts)
    _check(lib.lpm_partition(arr, len(arr), Z, C.byref(c), fixed, starts, cost))
    return list(starts), list(cost)


def lpm_partition_costs(layers, Z, cp, layer_cost_ps, fixed_starts=None):
    """The plan from caller-supplied per-layer costs (integer picoseconds) -> (starts[Z+1], stage_cost[Z])"""
    arr = _as_layers(layers)
    c = _cp(cp)
    if len(layer_cost_ps) != len(arr):
        raise LpmError(-1, "layer_cost_ps needs one entry per layer")
    costs = (C.c_uint64 * len(arr))(*[int(v) for v in layer_cost_ps])
    starts = (C.c_int32 * (Z + 1))()
    cost = (C.c_uint64 * Z)()
    fixed = None
    if fixed_starts is not None:
        if len(fixed_starts) != Z + 1:
            raise LpmError(-1, "fixed_starts needs Z+1 entries")
        fixed = (C.c_int32 * (Z + 1))(*fixed_starts)
    _check(lib.lpm_partition_costs(arr, len(arr), Z, C.byref(c), costs, fixed, starts, cost))
    return list(starts), list(cost)


def _geom(g):
    if isinstance(g, lpm_conv_geom):
        return g
    return lpm_conv_geom(*([g[k] for k in ("m", "h", "w", "cin", "cout", "kh", "kw", "stride", "pad")] +
                           [g.get("d", 1), g.get("kd", 1), g.get("pad_d", 0)]))


def _conv_sizes(gg, dtype):
    """Bytes of the operands of one contraction: (x, y or dz, w, dw)."""
    e = 2 if dtype == BF16 else 4
    d, kd, pd = max(gg.d, 1), max(gg.kd, 1), gg.pad_d
    do = (d + 2 * pd - kd) // gg.stride + 1
    ho = (gg.h + 2 * gg.pad - gg.kh) // gg.stride + 1
    wo = (gg.w + 2 * gg.pad - gg.kw) // gg.stride + 1
    wn = gg.cout * kd * gg.kh * gg.kw * gg.cin
    return gg.m * d * gg.h * gg.w * gg.cin * e, gg.m * do * ho * wo * gg.cout * e, wn * e, wn * 4


def _holds(name, t, nbytes):
    """The library sees plain pointers; a tensor handed over here is checked against the geometry before its kernels run
    (a buffer that is too small would be read or written past its end on the GPU)."""
    if t is None or isinstance(t, int):
        return
    have = t.numel() * t.element_size()
    if have < nbytes:
        raise ValueError("%s holds %d bytes, the geometry needs %d" % (name, have, nbytes))


def lpm_conv_ws_bytes(g, dtype):
    """-> (fwd, dgrad, wgrad) scratch bytes"""
    v = [C.c_size_t() for _ in range(3)]
    gg = _geom(g)
    _check(lib.lpm_conv_ws_bytes(C.byref(gg), dtype, *[C.byref(x) for x in v]))
    return tuple(x.value for x in v)


def lpm_conv_forward(g, dtype, x, w, scale, bias, add, relu, y, ws=None, stream=None):
    gg = _geom(g)
    xb, yb, wb, _ = _conv_sizes(gg, dtype)
    _holds("x", x, xb), _holds("w", w, wb), _holds("add", add, yb), _holds("y", y, yb), _holds("ws", ws, lpm_conv_ws_bytes(gg, dtype)[0])
    _check(lib.lpm_conv_forward(C.byref(gg), dtype, _ptr(x), _ptr(w), _ptr(scale), _ptr(bias), _ptr(add), int(relu), _ptr(y),
                                _ptr(ws), _stream(stream)))


def lpm_conv_dgrad(g, dtype, dz, w, wt, dx, accumulate=False, ws=None, stream=None):
    gg = _geom(g)
    xb, yb, wb, _ = _conv_sizes(gg, dtype)
    _holds("dz", dz, yb), _holds("w", w, wb), _holds("wt", wt, wb), _holds("dx", dx, xb), _holds("ws", ws, lpm_conv_ws_bytes(gg, dtype)[1])
    _check(lib.lpm_conv_dgrad(C.byref(gg), dtype, _ptr(dz), _ptr(w), _ptr(wt), _ptr(dx), int(accumulate), _ptr(ws),
                              _stream(stream)))


def lpm_conv_wgrad(g, dtype, x, dz, dw, accumulate=False, ws=None, stream=None):
    gg = _geom(g)
    xb, yb, _, db = _conv_sizes(gg, dtype)
    _holds("x", x, xb), _holds("dz", dz, yb), _holds("dw", dw, db), _holds("ws", ws, lpm_conv_ws_bytes(gg, dtype)[2])
    _check(lib.lpm_conv_wgrad(C.byref(gg), dtype, _ptr(x), _ptr(dz), _ptr(dw), int(accumulate), _ptr(ws), _stream(stream)))


STATIC_SCRATCH_BYTES = 8 << 20


def lpm_conv_wgrad_static(g, dtype, x, dz, dw, accumulate=False, stream=None):
    """lpm_conv_wgrad with the library's built-in scratch area: no workspace argument, nothing allocated."""
    gg = _geom(g)
    xb, yb, _, db = _conv_sizes(gg, dtype)
    _holds("x", x, xb), _holds("dz", dz, yb), _holds("dw", dw, db)
    _check(lib.lpm_conv_wgrad_static(C.byref(gg), dtype, _ptr(x), _ptr(dz), _ptr(dw), int(accumulate), _stream(stream)))


def lpm_conv_time(op, g, dtype, x, w, wt, y, dw, ws, warmup=3, iters=20, stream=None):
    """Average microseconds of one launch of contraction op (0 forward, 1 data gradient, 2 weight gradient)."""
    gg = _geom(g)
    xb, yb, wb, db = _conv_sizes(gg, dtype)
    _holds("x", x, xb), _holds("w", w, wb), _holds("wt", wt, wb), _holds("y", y, yb), _holds("dw", dw, db)
    _holds("ws", ws, max(lpm_conv_ws_bytes(gg, dtype)))
    out = C.c_float()
    _check(lib.lpm_conv_time(op, C.byref(gg), dtype, _ptr(x), _ptr(w), _ptr(wt), _ptr(y), _ptr(dw), _ptr(ws), warmup, iters,
                             _stream(stream), C.byref(out)))
    return out.value


class Layerwise:
    """lpm_layerwise handle (one layer computed as n sub-layers); methods are the lpm_layerwise_* calls."""

    def __init__(self, g, dtype, n):
        self.h = None
        gg = _geom(g)
        h = C.c_void_p()
        _check(lib.lpm_layerwise_create(C.byref(gg), dtype, n, C.byref(h)))
        self.h, self.n, self.dtype = h, n, dtype
        f, b = C.c_size_t(), C.c_size_t()
        _check(lib.lpm_layerwise_ws_bytes(self.h, C.byref(f), C.byref(b)))
        self.fwd_ws_bytes, self.bwd_ws_bytes = f.value, b.value

    def forward(self, x, w, scale, bias, relu, y, ws, stream=None):
        _check(lib.lpm_layerwise_forward(self.h, _ptr(x), _ptr(w), _ptr(scale), _ptr(bias), int(relu), _ptr(y), _ptr(ws),
                                         _stream(stream)))

    def backward(self, x, dz, w, wt, dx, dw, accumulate, ws, stream=None):
        _check(lib.lpm_layerwise_backward(self.h, _ptr(x), _ptr(dz), _ptr(w), _ptr(wt), _ptr(dx), _ptr(dw), int(accumulate),
                                          _ptr(ws), _stream(stream)))

    def time(self, op, x, w, wt, y, dx, dw, ws, warmup=3, iters=20, stream=None):
        """Average microseconds of one forward (op 0) or backward (op 1) call."""
        out = C.c_float()
        _check(lib.lpm_layerwise_time(self.h, op, _ptr(x), _ptr(w), _ptr(wt), _ptr(y), _ptr(dx), _ptr(dw), _ptr(ws), warmup,
                                      iters, _stream(stream), C.byref(out)))
        return out.value

    def close(self):
        if self.h:
            lib.lpm_layerwise_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s):
    if s is None:
        return None
    return s if isinstance(s, int) else s.cuda_stream


class Stage:
    """lpm_stage handle; methods are the lpm_stage_* calls."""

    def __init__(self, layers, first, last, microbatch, dtype):
        self._arr = _as_layers(layers)
        self.first, self.last, self.m, self.dtype = first, last, microbatch, dtype
        h = C.c_void_p()
        _check(lib.lpm_stage_create(self._arr, len(self._arr), first, last, microbatch, dtype, C.byref(h)))
        self.h = h
        v = [C.c_size_t() for _ in range(8)]
        _check(lib.lpm_stage_sizes(self.h, *[C.byref(x) for x in v]))
        (self.param_bytes, self.lowp_bytes, self.grad_bytes, self.stash_bytes, self.fwd_ws_bytes, self.bwd_ws_bytes,
         self.in_bytes, self.out_bytes) = [x.value for x in v]

    def close(self):
        if getattr(self, "h", None):
            lib.lpm_stage_destroy(self.h)
            self.h = None

    __del__ = close

    def param_offset(self, layer, which):
        o, n = C.c_size_t(), C.c_size_t()
        _check(lib.lpm_stage_param_offset(self.h, layer, which, C.byref(o), C.byref(n)))
        return o.value, n.value

    def has_param(self, layer, which):
        o, n = C.c_size_t(), C.c_size_t()
        return lib.lpm_stage_param_offset(self.h, layer, which, C.byref(o), C.byref(n)) == 0

    def stash_offset(self, t):
        o, n = C.c_size_t(), C.c_size_t()
        _check(lib.lpm_stage_stash_offset(self.h, t, C.byref(o), C.byref(n)))
        return o.value, n.value

    def grad_offset(self, t):
        o, n = C.c_size_t(), C.c_size_t()
        _check(lib.lpm_stage_grad_offset(self.h, t, C.byref(o), C.byref(n)))
        return o.value, n.value

    def sync_lowp(self, params, lowp, stream=None):
        _check(lib.lpm_stage_sync_lowp(self.h, _ptr(params), _ptr(lowp), _stream(stream)))

    def forward(self, x, y, labels, loss_accum, params, lowp, stash, fwd_ws, loss_scale, stream=None):
        _check(lib.lpm_stage_forward(self.h, _ptr(x), _ptr(y), _ptr(labels), _ptr(loss_accum), _ptr(params), _ptr(lowp),
                                     _ptr(stash), _ptr(fwd_ws), loss_scale, _stream(stream)))

    def backward(self, x, y, dy, dx, params, lowp, stash, grads, accumulate, bwd_ws, stream=None):
        _check(lib.lpm_stage_backward(self.h, _ptr(x), _ptr(y), _ptr(dy), _ptr(dx), _ptr(params), _ptr(lowp), _ptr(stash),
                                      _ptr(grads), int(accumulate), _ptr(bwd_ws), _stream(stream)))

    def update(self, params, lowp, grads, momentum, lr, mu, zero_grads=False, stream=None):
        _check(lib.lpm_stage_update(self.h, _ptr(params), _ptr(lowp), _ptr(grads), _ptr(momentum), lr, mu,
                                    int(zero_grads), _stream(stream)))


    def update_adam(self, params, lowp, grads, m1, m2, lr, beta1, beta2, eps, step, zero_grads=False, stream=None):
        _check(lib.lpm_stage_update_adam(self.h, _ptr(params), _ptr(lowp), _ptr(grads), _ptr(m1), _ptr(m2), lr, beta1, beta2,
                                         eps, int(step), int(zero_grads), _stream(stream)))


class Schedule:
    """lpm_schedule handle."""

    def __init__(self, stages, n_microbatch, window=2):
        self.stages = stages
        arr = (C.c_void_p * len(stages))(*[s.h for s in stages])
        h = C.c_void_p()
        _check(lib.lpm_schedule_create(arr, len(stages), n_microbatch, window, C.byref(h)))
        self.h = h

    def cut_fused(self, z):
        """True when grad_in of stage z holds the gradient with the previous stage's ReLU mask applied."""
        r = lib.lpm_schedule_cut_fused(self.h, z)
        if r < 0:
            _check(r)
        return bool(r)

    def close(self):
        if getattr(self, "h", None):
            lib.lpm_schedule_destroy(self.h)
            self.h = None

    __del__ = close

    def run(self, mode, x_batch, labels, dy_batch, per_stage, dx_wanted, lr, mu, loss_out, stream_fwd, stream_bwd):
        _check(lib.lpm_schedule_run(self.h, mode, _ptr(x_batch), _ptr(labels), _ptr(dy_batch), per_stage, int(dx_wanted),
                                    lr, mu, _ptr(loss_out), _stream(stream_fwd), _stream(stream_bwd)))


# ------------------------------------------------------------------------------------------ layouts
# Logical tensors (numpy, [N][C][H][W] and [Cout][Cin][Kh][Kw]) <-> device layouts ([m][H][W][C],
# [Cout][Kh][Kw][Cin]).  Pure data movement.

def _torch():
    import torch
    return torch


def pack_act(a, dtype, device="cuda:0"):
    torch = _torch()
    t = torch.from_numpy(np.ascontiguousarray(np.transpose(np.asarray(a, dtype=np.float32), (0, 2, 3, 1))))
    return t.to(device=device, dtype=torch.bfloat16 if dtype == BF16 else torch.float32).contiguous()


def unpack_act(t, shape_nchw):
    n, c, h, w = shape_nchw
    return np.transpose(t.float().cpu().numpy().reshape(n, h, w, c), (0, 3, 1, 2)).astype(np.float64)


def pack_weight(w):
    return np.ascontiguousarray(np.transpose(np.asarray(w, dtype=np.float32), (0, 2, 3, 1))).reshape(-1)


def unpack_weight(flat, shape_oihw):
    o, i, kh, kw = shape_oihw
    return np.transpose(np.asarray(flat).reshape(o, kh, kw, i), (0, 3, 1, 2)).astype(np.float64)


def _oshape(l):
    """(C, H, W) of a layer's output for one sample; a volumetric layer's depth is folded into H."""
    k = l["kind"]
    if k == "conv":
        d, kd, pd = l.get("d_in", 1), l.get("kd", 1), l.get("pad_d", 0)
        return (l["cout"], ((d + 2 * pd - kd) // l["stride"] + 1) * ((l["h_in"] + 2 * l["pad"] - l["kh"]) // l["stride"] + 1),
                (l["w_in"] + 2 * l["pad"] - l["kw"]) // l["stride"] + 1)
    if k == "fc":
        return (l["cout"], 1, 1)
    if k == "maxpool2":
        return (l["cin"], l["h_in"] // 2, l["w_in"] // 2)
    if k == "attn":
        return (l["cout"], l["h_in"], l["w_in"])
    return (l["cin"], 1, 1)


def _wshape(l):
    """Logical weight shape [Cout][Cin][Kd*Kh][Kw] (the filter depth folded into its height, like the activations)."""
    if l["kind"] == "fc":
        return (l["cout"], l["cin"], l.get("d_in", 1) * l["h_in"], l["w_in"])
    return (l["cout"], l["cin"], l.get("kd", 1) * l["kh"], l["kw"])


_NET_STREAMS = {}


def _net_streams(torch, device):
    """One pair of streams per device, shared by every Net of the process."""
    key = str(device)
    if key not in _NET_STREAMS:
        _NET_STREAMS[key] = (torch.cuda.Stream(device=device), torch.cuda.Stream(device=device))
    return _NET_STREAMS[key]


class Net:
    """A partitioned network resident on one GPU: stages, their device buffers and a schedule.

    layers: list of layer dicts; starts: plan (Z+1 entries); dtype F32/BF16.
    """

    def __init__(self, layers, starts, microbatch, n_microbatch, dtype, window=2, device="cuda:0", dx_wanted=False,
                 async_update=False):
        """async_update: also allocate the second weight version the ASYNC_UPDATE schedules need."""
        torch = _torch()
        self.torch = torch
        self.layers, self.starts, self.m, self.M, self.dtype, self.window = layers, list(starts), microbatch, n_microbatch, dtype, window
        self.device = torch.device(device)
        self.Z = len(starts) - 1
        self.dx_wanted = dx_wanted
        arr = layers_from_dicts(layers)
        self.stages = [Stage(arr, starts[z], starts[z + 1], microbatch, dtype) for z in range(self.Z)]
        self.schedule = Schedule(self.stages, n_microbatch, window)
        self.tdtype = torch.bfloat16 if dtype == BF16 else torch.float32

        def buf(nbytes, zero=True):
            n = max(int(nbytes), 256)
            t = torch.zeros(n, dtype=torch.uint8, device=self.device) if zero else torch.empty(n, dtype=torch.uint8, device=self.device)
            assert t.data_ptr() % 256 == 0
            return t

        self.bufs = []
        self.cbufs = (lpm_stage_buffers * self.Z)()
        for z, s in enumerate(self.stages):
            b = dict(params=buf(s.param_bytes), lowp=buf(s.lowp_bytes) if dtype == BF16 else None, grads=buf(s.grad_bytes),
                     momentum=buf(s.grad_bytes), stash=[buf(s.stash_bytes) for _ in range(window)],
                     act_out=[buf(s.out_bytes) for _ in range(window)],
                     grad_in=[buf(s.in_bytes) if (z > 0 or dx_wanted) else None for _ in range(window)],
                     fwd_ws=buf(s.fwd_ws_bytes), bwd_ws=buf(s.bwd_ws_bytes))
            self.bufs.append(b)
            cb = self.cbufs[z]
            cb.params, cb.lowp, cb.grads, cb.momentum = _ptr(b["params"]), _ptr(b["lowp"]), _ptr(b["grads"]), _ptr(b["momentum"])
            for w in range(window):
                cb.stash[w] = _ptr(b["stash"][w])
                cb.act_out[w] = _ptr(b["act_out"][w])
                cb.grad_in[w] = _ptr(b["grad_in"][w])
            cb.fwd_ws, cb.bwd_ws = _ptr(b["fwd_ws"]), _ptr(b["bwd_ws"])
            b["params_alt"] = buf(s.param_bytes) if async_update else None
            b["lowp_alt"] = buf(s.lowp_bytes) if (async_update and dtype == BF16) else None
            cb.params_alt, cb.lowp_alt = _ptr(b["params_alt"]), _ptr(b["lowp_alt"])
        self.loss = torch.zeros(64, dtype=torch.float32, device=self.device)
        self.stream_fwd, self.stream_bwd = _net_streams(torch, self.device)

    def stage_of(self, layer):
        for z in range(self.Z):
            if self.starts[z] <= layer < self.starts[z + 1]:
                return z
        raise IndexError(layer)

    # ---- parameters: logical numpy dicts {layer: {'W','b','s'}} <-> packed device buffers
    def _write(self, name, values, keys):
        torch = self.torch
        for z, s in enumerate(self.stages):
            host = self.bufs[z][name].view(torch.float32).cpu().numpy().copy()
            for i in range(s.first, s.last):
                if i not in values:
                    continue
                for which, k in enumerate(("W", "b", "s")):
                    if k in keys and k in values[i]:
                        off, n = s.param_offset(i, which)
                        v = pack_weight(values[i][k]) if k == "W" else np.asarray(values[i][k], dtype=np.float32)
                        host[off:off + n] = v
            self.bufs[z][name].view(torch.float32).copy_(torch.from_numpy(host))

    def _read(self, name, keys):
        torch = self.torch
        out = {}
        for z, s in enumerate(self.stages):
            host = self.bufs[z][name].view(torch.float32).cpu().numpy()
            for i in range(s.first, s.last):
                l = self.layers[i]
                if l["kind"] not in ("conv", "fc"):
                    continue
                d = {}
                for which, k in enumerate(("W", "b", "s")):
                    if k in keys and s.has_param(i, which):
                        off, n = s.param_offset(i, which)
                        d[k] = unpack_weight(host[off:off + n], _wshape(l)) if k == "W" else host[off:off + n].astype(np.float64)
                out[i] = d
        return out

    def load_params(self, params, momentum=None):
        self._write("params", params, ("W", "b", "s"))
        if momentum is not None:
            self._write("momentum", momentum, ("W", "b"))
        if self.dtype == BF16:
            for z, s in enumerate(self.stages):
                s.sync_lowp(self.bufs[z]["params"], self.bufs[z]["lowp"], None)
        for b in self.bufs:                       # the second weight version starts as a copy (frozen scales included)
            if b["params_alt"] is not None:
                b["params_alt"].copy_(b["params"])
            if b["lowp_alt"] is not None:
                b["lowp_alt"].copy_(b["lowp"])
        self.torch.cuda.synchronize(self.device)

    def read_params(self):
        return self._read("params", ("W", "b", "s"))

    def read_grads(self):
        return self._read("grads", ("W", "b"))

    def read_momentum(self):
        return self._read("momentum", ("W", "b"))

    # ---- tensors
    def tensor_shape(self, t):
        l0 = self.layers[0]
        return _oshape(self.layers[t]) if t >= 0 else (l0["cin"], l0.get("d_in", 1) * l0["h_in"], l0["w_in"])

    def read_stash(self, t, slot):
        """Logical [m][C][H][W] value of internal tensor t from a stash slot."""
        z = self.stage_of(t)
        off, n = self.stages[z].stash_offset(t)
        raw = self.bufs[z]["stash"][slot][off:off + n].view(self.tdtype)
        return unpack_act(raw, (self.m,) + self.tensor_shape(t))

    def read_act_out(self, z, slot):
        s = self.stages[z]
        t = s.last - 1 if self.layers[s.last - 1]["kind"] != "softmax_ce" else s.last - 2
        n = s.out_bytes
        return unpack_act(self.bufs[z]["act_out"][slot][:n].view(self.tdtype), (self.m,) + self.tensor_shape(t))

    def _out_tensor(self, z):
        s = self.stages[z]
        return s.last - 1 if self.layers[s.last - 1]["kind"] != "softmax_ce" else s.last - 2

    def write_stash(self, t, slot, value):
        """Store a logical [m][C][H][W] array as internal tensor t of a stash slot (t = 'dlogits' for the
        loss gradient).  For tests that hand a stage a prepared forward state."""
        if t == "dlogits":
            z = self.Z - 1
            off, n = self.stages[z].stash_offset(-100)
        else:
            z = self.stage_of(t)
            off, n = self.stages[z].stash_offset(t)
        src = pack_act(value, self.dtype, self.device).reshape(-1).view(self.torch.uint8)
        assert src.numel() == n, (src.numel(), n)
        self.bufs[z]["stash"][slot][off:off + n].copy_(src)

    def write_act_out(self, z, slot, value):
        src = pack_act(value, self.dtype, self.device).reshape(-1).view(self.torch.uint8)
        assert src.numel() == self.stages[z].out_bytes
        self.bufs[z]["act_out"][slot][:src.numel()].copy_(src)

    def read_grad_in(self, z, slot=0):
        s = self.stages[z]
        return unpack_act(self.bufs[z]["grad_in"][slot][:s.in_bytes].view(self.tdtype), (self.m,) + self.tensor_shape(s.first - 1))

    # ---- one mini-batch step
    def step(self, x_batch, labels, dy_batch, lr, mu, mode=OVERLAPPED):
        """x_batch, labels, dy_batch: device tensors already in device layout (see pack_act)."""
        torch = self.torch
        cur = torch.cuda.current_stream(self.device)
        self.stream_fwd.wait_stream(cur)
        self.schedule.run(mode, x_batch, labels, dy_batch, self.cbufs, self.dx_wanted, lr, mu, self.loss,
                          self.stream_fwd, self.stream_bwd)
        cur.wait_stream(self.stream_fwd)

    def loss_value(self):
        self.torch.cuda.synchronize(self.device)
        return float(self.loss[0].item())

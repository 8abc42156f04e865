"""fp64 CPU oracle for the partitioned training step (layers, loss, backward, update, plan, schedules).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The product path never calls it, and it imports nothing from the GPU
package.  It shares no code with the HIP sources.

What it computes is plain mini-batch backpropagation plus SGD, re-organised in time:
  * layers            a^{l+1} = g_l(a^l, p^l)                       (Problem Statement, eq. 1)
  * loss              f(a^L, e), softmax cross-entropy              (Problem Statement, eq. 3; Results section)
  * backward          chain rule for parameter/activation gradients (Problem Statement, eqs. 8-9)
  * update            p <- p - alpha * omega                        (Problem Statement, eq. 6)
                      (and Adam, which the same passage names as the alternative)
  * partitions        stacks of consecutive layers (sub-modules)    (Layer-wise Partitioning and Merging)
  * cost              additive over the F_{i,j}, B_{i,j} operations (Cost Model, eq. 10)
  * schedules         locked F_1..F_n then B_n..B_1; overlapped F/B of different micro-batches,
                      gradient accumulation and one update per mini-batch
                      (Forward Pass and Backward Pass Parallelisation and Optimisation)

Convolution and pooling loops are the C routines of lpm_oracle.c (direct fp64 loops);
everything else is numpy in float64.  Layouts are logical: activations [N][C][H][W],
weights [Cout][Cin][Kh][Kw].  Layers are the plain dicts of workloads.configs.
A volumetric (3-D) convolution keeps its tensors as [N][C][D*H][W] and its weights as [Cout][Cin][Kd*Kh][Kw]:
only the convolution routines unfold the depth (keys d_in, kd, pad_d of the layer dict).

Readings taken where the paper is silent are listed next to each function.
"""
import ctypes
import itertools
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liblpm_oracle.so")
_SRC = os.path.join(_HERE, "lpm_oracle.c")


def build(force=False):
    """Compile lpm_oracle.c (gcc -O2 -fopenmp) into liblpm_oracle.so next to it."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _SO, _SRC])
    return _SO


_lib = None


def _c():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# --------------------------------------------------------------------------- layers

def _depth(l):
    """(D, Kd, pad_d) of a convolution: 1, 1, 0 for a two-dimensional layer.  A volumetric layer reads its input
    [N][C][D][H][W] stored as [N][C][D*H][W] (depth folded into the height axis), so that every other routine of this
    file -- epilogue, pooling-free residual sums, global average pooling -- sees an ordinary 4-index tensor."""
    D = l.get("d_in", 1)
    if l["kind"] == "fc":
        return D, D, 0
    return D, l.get("kd", 1), l.get("pad_d", 0)


def _oshape(l):
    k = l["kind"]
    if k == "conv":
        D, Kd, pd = _depth(l)
        Do = (D + 2 * pd - Kd) // l["stride"] + 1
        return (l["cout"], Do * ((l["h_in"] + 2 * l["pad"] - l["kh"]) // l["stride"] + 1),
                (l["w_in"] + 2 * l["pad"] - l["kw"]) // l["stride"] + 1)
    if k in ("fc",):
        return (l["cout"], 1, 1)
    if k == "maxpool2":
        return (l["cin"], l["h_in"] // 2, l["w_in"] // 2)
    if k == "attn":
        return (l["cout"], l["h_in"], l["w_in"])
    return (l["cin"], 1, 1)          # gap, softmax_ce


def _geom(l):
    """(Cin,H,W,Cout,Kh,Kw,stride,pad); an fc layer is a conv whose kernel covers its whole input."""
    if l["kind"] == "fc":
        return l["cin"], l["h_in"], l["w_in"], l["cout"], l["h_in"], l["w_in"], 1, 0
    return l["cin"], l["h_in"], l["w_in"], l["cout"], l["kh"], l["kw"], l["stride"], l["pad"]


def _is3d(l):
    D, Kd, _ = _depth(l)
    return D > 1 or Kd > 1


def conv_fwd(x, W, l):
    Cin, H, Wd, Cout, Kh, Kw, s, p = _geom(l)
    if _is3d(l):
        D, Kd, pd = _depth(l)
        x = _f64(x).reshape(-1, Cin, D, H, Wd)
        N = x.shape[0]
        z = np.empty((N,) + _oshape(l))
        _c().orc_conv3d_fwd(_p(x), _p(_f64(W)), _p(z), N, Cin, D, H, Wd, Cout, Kd, Kh, Kw, s, pd, p)
        return z
    x = _f64(x).reshape(-1, Cin, H, Wd)
    N = x.shape[0]
    z = np.empty((N,) + _oshape(l))
    _c().orc_conv_fwd(_p(x), _p(_f64(W)), _p(z), N, Cin, H, Wd, Cout, Kh, Kw, s, p)
    return z


def conv_bwd_data(dz, W, l):
    Cin, H, Wd, Cout, Kh, Kw, s, p = _geom(l)
    dz = _f64(dz)
    N = dz.shape[0]
    if _is3d(l):
        D, Kd, pd = _depth(l)
        dx = np.empty((N, Cin, D * H, Wd))
        _c().orc_conv3d_bwd_data(_p(dz), _p(_f64(W)), _p(dx), N, Cin, D, H, Wd, Cout, Kd, Kh, Kw, s, pd, p)
        return dx
    dx = np.empty((N, Cin, H, Wd))
    _c().orc_conv_bwd_data(_p(dz), _p(_f64(W)), _p(dx), N, Cin, H, Wd, Cout, Kh, Kw, s, p)
    return dx


def conv_bwd_weight(x, dz, l):
    Cin, H, Wd, Cout, Kh, Kw, s, p = _geom(l)
    dz = _f64(dz)
    if _is3d(l):
        D, Kd, pd = _depth(l)
        x = _f64(x).reshape(-1, Cin, D, H, Wd)
        dW = np.empty((Cout, Cin, Kd * Kh, Kw))          # [Cout][Cin][Kd][Kh][Kw] with (Kd, Kh) folded, like the activations
        _c().orc_conv3d_bwd_weight(_p(x), _p(dz), _p(dW), x.shape[0], Cin, D, H, Wd, Cout, Kd, Kh, Kw, s, pd, p)
        return dW
    x = _f64(x).reshape(-1, Cin, H, Wd)
    dW = np.empty((Cout, Cin, Kh, Kw))
    _c().orc_conv_bwd_weight(_p(x), _p(dz), _p(dW), x.shape[0], Cin, H, Wd, Cout, Kh, Kw, s, p)
    return dW


def attn_fwd(x):
    """Self-attention over the positions of one sample (reading of the use case's "self-attention layer": scaled
    dot-product attention, one head).  x [N][3C][H][W] holds queries, keys and values as three groups of C channels
    (made by the 1x1 convolution in front of this layer); with P = H*W positions
        S[i][j] = sum_c q[c][i] k[c][j] / sqrt(C),   A = softmax over j of S,   y[c][i] = sum_j A[i][j] v[c][j].
    Returns y [N][C][H][W]."""
    x = _f64(x)
    N, C3, H, W = x.shape
    C = C3 // 3
    q, k, v = (x[:, g * C:(g + 1) * C].reshape(N, C, H * W) for g in range(3))
    S = np.einsum("nci,ncj->nij", q, k) / np.sqrt(C)
    S = S - S.max(axis=2, keepdims=True)
    A = np.exp(S)
    A /= A.sum(axis=2, keepdims=True)
    return np.einsum("nij,ncj->nci", A, v).reshape(N, C, H, W)


def attn_bwd(x, dy):
    """Gradient of attn_fwd w.r.t. x, by the chain rule through y = A v, A = softmax(S), S = q^T k / sqrt(C):
        dv[c][j] = sum_i A[i][j] dy[c][i];   dA[i][j] = sum_c dy[c][i] v[c][j];
        dS[i][j] = A[i][j] (dA[i][j] - sum_j' A[i][j'] dA[i][j']);
        dq[c][i] = sum_j dS[i][j] k[c][j] / sqrt(C);   dk[c][j] = sum_i dS[i][j] q[c][i] / sqrt(C)."""
    x, dy = _f64(x), _f64(dy)
    N, C3, H, W = x.shape
    C = C3 // 3
    q, k, v = (x[:, g * C:(g + 1) * C].reshape(N, C, H * W) for g in range(3))
    g = dy.reshape(N, C, H * W)
    S = np.einsum("nci,ncj->nij", q, k) / np.sqrt(C)
    S = S - S.max(axis=2, keepdims=True)
    A = np.exp(S)
    A /= A.sum(axis=2, keepdims=True)
    dv = np.einsum("nij,nci->ncj", A, g)
    dA = np.einsum("nci,ncj->nij", g, v)
    dS = A * (dA - (A * dA).sum(axis=2, keepdims=True))
    dq = np.einsum("nij,ncj->nci", dS, k) / np.sqrt(C)
    dk = np.einsum("nij,nci->ncj", dS, q) / np.sqrt(C)
    return np.concatenate([dq, dk, dv], axis=1).reshape(N, C3, H, W)


def maxpool2_fwd(x):
    x = _f64(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, H // 2, W // 2))
    _c().orc_maxpool2_fwd(_p(x), _p(y), N, C, H, W)
    return y


def maxpool2_bwd(x, dy):
    """Gradient goes to the first maximum of each window (row-major inside the window)."""
    x, dy = _f64(x), _f64(dy)
    N, C, H, W = x.shape
    dx = np.empty_like(x)
    _c().orc_maxpool2_bwd(_p(x), _p(dy), _p(dx), N, C, H, W)
    return dx


def softmax_ce(logits, labels, batch_total):
    """Per-call partial of the mini-batch mean loss and its gradient.

    loss_partial = (1/b) * sum_n -log softmax(logits_n)[e_n];  dlogits = (softmax - onehot)/b,
    with b = batch_total, the size of the WHOLE mini-batch (reading: the loss is the mean over
    the mini-batch b_t of eq. 7, so gradients of micro-batches add up to the mini-batch gradient).
    """
    z = _f64(logits).reshape(len(labels), -1)
    zs = z - z.max(axis=1, keepdims=True)
    lse = np.log(np.exp(zs).sum(axis=1))
    rows = np.arange(z.shape[0])
    loss = float((lse - zs[rows, labels]).sum() / batch_total)
    d = np.exp(zs - lse[:, None])
    d[rows, labels] -= 1.0
    return loss, (d / batch_total).reshape(np.shape(logits))


# --------------------------------------------------------------------------- a stage (sub-module)

def round_bf16(a):
    """Nearest bfloat16 (ties to even) of every element, returned as float64.  Models the STORAGE
    precision of the bf16 workloads; arithmetic stays fp64."""
    f = np.ascontiguousarray(a, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(a))


def stage_forward(layers, first, last, params, a_in, labels=None, batch_total=None, store=None):
    """F_{z,j}: evaluate layers [first,last) on one micro-batch.

    store: optional function applied to every layer output as it is stored (e.g. round_bf16).  The
    bf16 workloads keep activations in bfloat16, and two decisions of the backward pass are taken on
    stored values: the ReLU mask (y > 0) and the position of a pooling window's maximum.  Both sides
    of a comparison must take them in the same precision, so for those workloads the oracle rounds
    each stored activation once, exactly where the device stores it, and computes everything else in
    fp64.  With store=None the oracle is the unrounded textbook computation.

    a_in is tensor first-1 (the activation handed over by the previous sub-module, or the
    network input).  Returns (a_out, stash, loss_partial): the stash maps tensor index ->
    value for every tensor backward needs (first-1 .. last-1); if the stage ends in the loss
    layer, a_out is the logits and stash['dlogits'] holds the loss gradient.
    """
    T = {first - 1: _f64(a_in)}
    loss = None
    for i in range(first, last):
        l = layers[i]
        x = T[l["src"]]
        k = l["kind"]
        if k in ("conv", "fc"):
            p = params[i]
            z = conv_fwd(x, p["W"], l)
            if l["scale"]:
                z = z * p["s"][None, :, None, None]
            if l["bias"]:
                z = z + p["b"][None, :, None, None]
            if l["add_src"] is not None:
                z = z + T[l["add_src"]]
            T[i] = np.maximum(z, 0.0) if l["relu"] else z
        elif k == "maxpool2":
            T[i] = maxpool2_fwd(x)
        elif k == "gap":
            T[i] = x.mean(axis=(2, 3), keepdims=True)
        elif k == "attn":
            T[i] = attn_fwd(x)
        elif k == "softmax_ce":
            loss, T["dlogits"] = softmax_ce(x, labels, batch_total)
            T[i] = x
        else:
            raise ValueError(k)
        if store is not None and k != "softmax_ce":
            T[i] = store(T[i])
    return T[last - 1], T, loss


def stage_backward(layers, first, last, params, stash, g_out, grads, input_grad=None):
    """B_{z,j}: reverse pass over layers [first,last) for one micro-batch.

    g_out is the gradient w.r.t. the stage output (None for a stage ending in the loss layer).
    Parameter gradients are ADDED into grads[i]['W'|'b'] (gradient accumulation over
    micro-batches).  Returns the gradient w.r.t. tensor first-1; by default None when first == 0
    (the network input needs no gradient); input_grad=True forces it, for a partition whose input
    is an upstream activation.  ReLU'(0) = 0 (mask is y > 0).
    """
    G = {}
    if input_grad is None:
        input_grad = first > 0

    def acc(t, g):
        G[t] = g if t not in G else G[t] + g

    if layers[last - 1]["kind"] == "softmax_ce":
        acc(last - 1, stash["dlogits"])
    else:
        acc(last - 1, _f64(g_out))
    for i in range(last - 1, first - 1, -1):
        l = layers[i]
        g = G.pop(i)
        k = l["kind"]
        src = l["src"]
        if k in ("conv", "fc"):
            p = params[i]
            gm = g * (stash[i] > 0.0) if l["relu"] else g
            if l["add_src"] is not None:
                acc(l["add_src"], gm)
            if l["bias"]:
                grads[i]["b"] += gm.sum(axis=(0, 2, 3))
            dz = gm * p["s"][None, :, None, None] if l["scale"] else gm
            grads[i]["W"] += conv_bwd_weight(stash[src], dz, l)
            if src >= first or input_grad:
                acc(src, conv_bwd_data(dz, p["W"], l).reshape(stash[src].shape))
        elif k == "maxpool2":
            acc(src, maxpool2_bwd(stash[src], g))
        elif k == "gap":
            x = stash[src]
            acc(src, np.broadcast_to(g / (x.shape[2] * x.shape[3]), x.shape).copy())
        elif k == "attn":
            acc(src, attn_bwd(stash[src], g))
        elif k == "softmax_ce":
            acc(src, g)
    return G.get(first - 1) if input_grad else None


def zero_grads(layers, params):
    return {i: {k: np.zeros_like(v) for k, v in p.items() if k != "s"} for i, p in params.items()}


def sgd_momentum(params, grads, momentum, lr, mu, first=0, last=None):
    """v <- mu*v + g ; p <- p - lr*v  for the trainable tensors of layers [first,last), in place.

    With mu = 0 this is eq. 6, p <- p - alpha*omega.  The momentum form (no dampening, no
    Nesterov, no weight decay) is this build's reading: the paper's update has no momentum term.
    The frozen per-channel scale 's' is never updated.
    """
    for i, p in params.items():
        if i < first or (last is not None and i >= last):
            continue
        for k in ("W", "b"):
            if k in p:
                momentum[i][k] = mu * momentum[i][k] + grads[i][k]
                p[k] = p[k] - lr * momentum[i][k]


def adam(params, grads, m1, m2, lr, beta1, beta2, eps, t, first=0, last=None):
    """The other update rule the Problem Statement names beside SGD (it prints only SGD's formula, eq. 6): Adam as
    published by Kingma and Ba, step t = 1, 2, ... for the trainable tensors of layers [first,last), in place.

        m1 <- beta1*m1 + (1-beta1)*g          m2 <- beta2*m2 + (1-beta2)*g*g
        p  <- p - lr * (m1 / (1-beta1^t)) / (sqrt(m2 / (1-beta2^t)) + eps)

    No weight decay, no AMSGrad.  The frozen per-channel scale 's' is never updated.
    """
    c1, c2 = 1.0 - beta1 ** t, 1.0 - beta2 ** t
    for i, p in params.items():
        if i < first or (last is not None and i >= last):
            continue
        for k in ("W", "b"):
            if k in p:
                g = grads[i][k]
                m1[i][k] = beta1 * m1[i][k] + (1.0 - beta1) * g
                m2[i][k] = beta2 * m2[i][k] + (1.0 - beta2) * g * g
                p[k] = p[k] - lr * (m1[i][k] / c1) / (np.sqrt(m2[i][k] / c2) + eps)


# --------------------------------------------------------------------------- schedules

LOCKED, OVERLAPPED = 0, 1


def schedule_ops(Z, M, mode, window=2):
    """Operation set and dependency map of one mini-batch step.

    Ops are ('F',z,j), ('B',z,j), ('U',z).  Returns {op: set(prerequisite ops)}.
    LOCKED: a single chain  F_{0,j}..F_{Z-1,j}, B_{Z-1,j}..B_{0,j}  for j = 0..M-1, then U_0..U_{Z-1}
    (the non-parallel schedule).  OVERLAPPED (reading of the parallel schedule):
      F_{z,j} after F_{z-1,j} and F_{z,j-1};  B_{z,j} after B_{z+1,j} (or F_{Z-1,j} for the last
      stage) and B_{z,j-1} (fixed accumulation order);  window: F_{z,j+window} after B_{z,j}
      (with window 2 this is "B_{0,0} finishes before F_{0,2}");  U_z after B_{z,M-1}.
    """
    deps = {}
    if mode == LOCKED:
        chain = []
        for j in range(M):
            chain += [("F", z, j) for z in range(Z)] + [("B", z, j) for z in range(Z - 1, -1, -1)]
        chain += [("U", z) for z in range(Z)]
        for a, b in zip([None] + chain[:-1], chain):
            deps[b] = set() if a is None else {a}
        return deps
    for j in range(M):
        for z in range(Z):
            d = set()
            if z > 0:
                d.add(("F", z - 1, j))
            if j > 0:
                d.add(("F", z, j - 1))
            if j >= window:
                d.add(("B", z, j - window))
            deps[("F", z, j)] = d
            d = {("B", z + 1, j)} if z < Z - 1 else {("F", Z - 1, j)}
            if j > 0:
                d.add(("B", z, j - 1))
            deps[("B", z, j)] = d
    for z in range(Z):
        deps[("U", z)] = {("B", z, M - 1)}
    return deps


def legal_order(deps, rng=None):
    """One topological order of deps; random among the ready ops when rng (numpy Generator) is given,
    else the first ready op in sorted order."""
    done, order = set(), []
    remaining = dict(deps)
    while remaining:
        ready = sorted(op for op, d in remaining.items() if d <= done)
        assert ready, "dependency cycle"
        op = ready[int(rng.integers(len(ready)))] if rng is not None else ready[0]
        order.append(op)
        done.add(op)
        del remaining[op]
    return order


def run_schedule(layers, starts, params, momentum, x, labels, g_up, M, lr, mu, mode=LOCKED, window=2,
                 order_rng=None, keep=False, input_grad=False, store=None):
    """Execute one mini-batch step under a schedule; returns dict(loss, grads, [acts, gins]).

    The batch is split in order into M contiguous micro-batches; per-micro-batch gradients are
    summed; every stage is updated once, after its last backward.  Ops run in a legal topological
    order of schedule_ops (randomised when order_rng is given) and every dependency, the
    in-flight window and the stash-slot discipline (slot j mod window is never overwritten while
    its micro-batch is still awaiting backward) are asserted as they run.
    params and momentum are updated in place.
    """
    Z = len(starts) - 1
    b = x.shape[0]
    assert b % M == 0
    m = b // M
    deps = schedule_ops(Z, M, mode, window)
    order = legal_order(deps, order_rng)
    grads = zero_grads(layers, params)
    slots = [[None] * window for _ in range(Z)]          # slot -> (j, stash)
    act = {}                                             # (z,j) -> activation handed to stage z+1
    gin = {}                                             # (z,j) -> gradient handed to stage z-1
    done = set()
    loss = 0.0
    acts_keep, gins_keep = {}, {}
    for op in order:
        assert deps[op] <= done, ("dependency violated", op)
        if op[0] == "F":
            _, z, j = op
            a_in = x[j * m:(j + 1) * m] if z == 0 else act[(z - 1, j)]
            lab = labels[j * m:(j + 1) * m] if (labels is not None and z == Z - 1) else None
            a_out, stash, lp = stage_forward(layers, starts[z], starts[z + 1], params, a_in, lab, b, store)
            s = j % window
            assert slots[z][s] is None, ("stash slot overwritten while live", op)
            assert sum(e is not None for e in slots[z]) < window
            slots[z][s] = (j, stash)
            act[(z, j)] = a_out
            if lp is not None:
                loss += lp
            if keep:
                acts_keep[(z, j)] = stash
        elif op[0] == "B":
            _, z, j = op
            s = j % window
            assert slots[z][s] is not None and slots[z][s][0] == j, ("stash missing", op)
            if z == Z - 1:
                g_out = None if labels is not None else g_up[j * m:(j + 1) * m]
            else:
                g_out = gin[(z + 1, j)]
            g = stage_backward(layers, starts[z], starts[z + 1], params, slots[z][s][1], g_out, grads,
                               input_grad=(z > 0 or input_grad))
            slots[z][s] = None
            gin[(z, j)] = g
            if keep:
                gins_keep[(z, j)] = g
        else:
            _, z = op
            sgd_momentum(params, grads, momentum, lr, mu, starts[z], starts[z + 1])
        done.add(op)
    out = dict(loss=loss, grads=grads, order=order)
    if keep:
        out["stash"], out["gin"] = acts_keep, gins_keep
    return out


# --------------------------------------------------------------------------- asynchronous update

def weight_version_read_by_forward(j, window):
    """Index of the weight version F_{z,j} reads under the asynchronous update.

    Reading of "asynchronous parameter update" (Forward Pass and Backward Pass Parallelisation and
    Optimisation): every micro-batch updates the weights, U_{z,j} right after B_{z,j}; version 0 is the
    state at the start of the step and U_{z,j} turns version j into version j+1.  A forward pass that
    overlaps the backward pass of the previous micro-batch cannot see that micro-batch's update, so
    with `window` micro-batches in flight F_{z,j} reads version max(0, j - (window - 1)): no delay
    for window 1 (plain per-micro-batch SGD), one update behind for window 2.  B_{z,j} runs after
    U_{z,j-1} and reads version j for its data gradients (no weight stashing), its activations are
    the ones F_{z,j} stored."""
    return max(0, j - (window - 1))


def schedule_ops_async(Z, M, window=2, locked=False):
    """Operation set and dependencies with one update per micro-batch: ('F',z,j), ('B',z,j), ('U',z,j).
    locked: the single chain F_{0,j}..F_{Z-1,j}, then B_{z,j}, U_{z,j} for z = Z-1..0, for j = 0..M-1.
    Otherwise F_{z,j} after F_{z-1,j}, F_{z,j-1} and U_{z,j-window}; B_{z,j} after B_{z+1,j} (F_{Z-1,j} for
    the last stage) and U_{z,j-1}; U_{z,j} after B_{z,j}."""
    deps = {}
    if locked:
        chain = []
        for j in range(M):
            chain += [("F", z, j) for z in range(Z)]
            for z in range(Z - 1, -1, -1):
                chain += [("B", z, j), ("U", z, j)]
        for a, b in zip([None] + chain[:-1], chain):
            deps[b] = set() if a is None else {a}
        return deps
    for j in range(M):
        for z in range(Z):
            d = set()
            if z > 0:
                d.add(("F", z - 1, j))
            if j > 0:
                d.add(("F", z, j - 1))
            if j >= window:
                d.add(("U", z, j - window))
            deps[("F", z, j)] = d
            d = {("B", z + 1, j)} if z < Z - 1 else {("F", Z - 1, j)}
            if j > 0:
                d.add(("U", z, j - 1))
            deps[("B", z, j)] = d
            deps[("U", z, j)] = {("B", z, j)}
    return deps


def run_schedule_async(layers, starts, params, momentum, x, labels, g_up, M, lr, mu, window=2, locked=False,
                       order_rng=None, input_grad=False, store=None, wstore=None):
    """One pass over the mini-batch with an update after every micro-batch (see
    weight_version_read_by_forward).  Each micro-batch is a mini-batch of its own: its loss is the mean
    over its m samples.  At most two weight versions of a stage are alive at any time (asserted: an
    older one is dropped when a new one is made, and reading a dropped version fails).  Ops run in a
    legal order of schedule_ops_async (randomised when order_rng is given); the result does not
    depend on it.  params and momentum are updated in place to the final version; returns
    dict(loss = sum of the micro-batches' mean losses, grads = gradient of the last micro-batch).
    wstore: optional function applied to the weight tensors 'W' the layers compute with (e.g. round_bf16:
    the bf16 workloads compute from a bfloat16 copy of the full-precision master weights, which the update
    refreshes; within the synchronous step that copy never changes, here it does after every update)."""
    import copy
    Z = len(starts) - 1
    b = x.shape[0]
    assert b % M == 0
    m = b // M
    w_eff = 1 if locked else window
    deps = schedule_ops_async(Z, M, window, locked)
    order = legal_order(deps, order_rng)
    ver = [{0: {i: copy.deepcopy(params[i]) for i in range(starts[z], starts[z + 1]) if i in params}} for z in range(Z)]
    slots = [[None] * max(window, 1) for _ in range(Z)]
    act, gin, gr = {}, {}, {}
    done = set()
    loss = 0.0
    for op in order:
        assert deps[op] <= done, ("dependency violated", op)
        _, z, j = op
        first, last = starts[z], starts[z + 1]
        if op[0] == "F":
            P = _compute_copy(ver[z][weight_version_read_by_forward(j, w_eff)], wstore)
            a_in = x[j * m:(j + 1) * m] if z == 0 else act[(z - 1, j)]
            lab = labels[j * m:(j + 1) * m] if (labels is not None and z == Z - 1) else None
            a_out, stash, lp = stage_forward(layers, first, last, P, a_in, lab, m, store)
            s = j % len(slots[z])
            assert slots[z][s] is None, ("stash slot overwritten while live", op)
            slots[z][s] = (j, stash)
            act[(z, j)] = a_out
            if lp is not None:
                loss += lp
        elif op[0] == "B":
            P = _compute_copy(ver[z][j], wstore)
            s = j % len(slots[z])
            assert slots[z][s] is not None and slots[z][s][0] == j, ("stash missing", op)
            if z == Z - 1:
                g_out = None if labels is not None else g_up[j * m:(j + 1) * m]
            else:
                g_out = gin[(z + 1, j)]
            g = zero_grads(layers, P)
            gin[(z, j)] = stage_backward(layers, first, last, P, slots[z][s][1], g_out, g, input_grad=(z > 0 or input_grad))
            slots[z][s] = None
            gr[(z, j)] = g
        else:
            new = copy.deepcopy(ver[z][j])
            sgd_momentum(new, gr[(z, j)], momentum, lr, mu, first, last)
            ver[z][j + 1] = new
            ver[z].pop(j - 1, None)          # two versions alive: j and j+1
            assert len(ver[z]) <= 2
        done.add(op)
    grads = {}
    for z in range(Z):
        for i, p in ver[z][M].items():
            params[i] = p
        grads.update(gr[(z, M - 1)])
    return dict(loss=loss, grads=grads, order=order)


def _compute_copy(P, wstore):
    """The weights the layers compute with: the master version, or its stored (rounded) copy."""
    if wstore is None:
        return P
    return {i: {k: (wstore(v) if k == "W" else v) for k, v in p.items()} for i, p in P.items()}


# --------------------------------------------------------------------------- cost model and plan

def layer_cost(layers, i, m, M, elem_bytes, flop_per_us, hbm_byte_per_us):
    """Integer cost (picoseconds) of F+B of layer i on one micro-batch of m images plus 1/M of its update.

    Reading of the cost functions T(F_{i,j}), T(B_{i,j}) of eq. 10, which the paper leaves opaque:
    the larger of arithmetic time and ideal memory-traffic time,
        c = max( flop*1e6 // flop_per_us ,  (M*byte_fb + byte_upd)*1e6 // (M*hbm_byte_per_us) )
    flop      = 2*MAC*m*(3 passes, or 2 if the layer reads the network input: no data gradient)
    byte_fb   = forward (in + out [+ shortcut] + W) + backward (dout + stashed in + din [+ dshortcut]
                + W + fp32 dW read and write)
    byte_upd  = P*(20 [+2 for the low-precision weight copy])   (P = trainable parameters)
    All quantities are integers derived from the descriptor, so plans are reproducible bit for bit.
    """
    l = layers[i]
    e = elem_bytes
    cin, h, w = l["cin"], l["h_in"], l["w_in"]
    co, ho, wo = _oshape(l)
    in_el, out_el = cin * h * w, co * ho * wo
    has_w = l["kind"] in ("conv", "fc")
    kh, kw = (l["h_in"], l["w_in"]) if l["kind"] == "fc" else (l["kh"], l["kw"])
    D, Kd, _ = _depth(l) if has_w else (1, 1, 0)
    in_el *= D                                     # a volumetric layer's input has D slices of h x w
    w_el = co * cin * Kd * kh * kw if has_w else 0
    p_el = w_el + (co if (has_w and l["bias"]) else 0)
    mac = out_el * cin * Kd * kh * kw if has_w else 0
    if l["kind"] == "attn":                        # the two products S = q^T k and y = A v: 2 * P * P * C multiply-adds
        mac = 2 * (h * w) * (h * w) * co
    first = l["src"] < 0
    flop = 2 * mac * m * (2 if first else 3)
    sc = out_el if l.get("add_src") is not None else 0
    fwd = (in_el + out_el + sc) * m * e + w_el * e
    bwd = (out_el + in_el + (0 if first else in_el) + sc) * m * e + w_el * e + 8 * w_el
    upd = p_el * (20 + (2 if e == 2 else 0))
    t_flop = flop * 1000000 // flop_per_us
    t_byte = ((fwd + bwd) * M + upd) * 1000000 // (M * hbm_byte_per_us)
    return max(t_flop, t_byte)


def boundary_bytes(layers, i, m, elem_bytes):
    """Bytes of the activation crossing a cut placed after layer i, for one micro-batch."""
    co, ho, wo = _oshape(layers[i])
    return co * ho * wo * m * elem_bytes


def plan_cost(layers, starts, cp, layer_costs=None):
    """(per-stage costs, total boundary bytes) of a plan.  cp: dict with flop_per_us, hbm_byte_per_us,
    link_byte_per_us (0 = ignore transfers), elem_bytes, microbatch, n_microbatch.
    A stage's cost is the sum of its layers' costs (eq. 10 is additive) plus, when link_byte_per_us > 0,
    2*bytes*1e6 // link for each of its boundaries (activation forward and gradient backward).
    layer_costs: per-layer costs given by the caller (eq. 10's T(F), T(B) as measured times, integer
    picoseconds) in place of the analytic per-layer model."""
    m, M, e = cp["microbatch"], cp["n_microbatch"], cp["elem_bytes"]
    if layer_costs is not None:
        c = [int(v) for v in layer_costs]
        assert len(c) == len(layers)
    else:
        c = [layer_cost(layers, i, m, M, e, cp["flop_per_us"], cp["hbm_byte_per_us"]) for i in range(len(layers))]
    Z = len(starts) - 1
    costs, tot = [], 0
    for z in range(Z):
        sc = sum(c[starts[z]:starts[z + 1]])
        for cut in ([starts[z] - 1] if z > 0 else []) + ([starts[z + 1] - 1] if z < Z - 1 else []):
            bb = boundary_bytes(layers, cut, m, e)
            if cp.get("link_byte_per_us", 0) > 0:
                sc += 2 * bb * 1000000 // cp["link_byte_per_us"]
        costs.append(sc)
    for z in range(1, Z):
        tot += boundary_bytes(layers, starts[z] - 1, m, e)
    return costs, tot


def plan_bruteforce(layers, Z, cp, layer_costs=None):
    """The plan by exhaustive enumeration: among all ways of cutting the layer list into Z non-empty
    contiguous stages at allowed cut points, the one minimising, lexicographically,
    (largest stage cost, total boundary bytes, starts).  Reading of the partition-and-merge objective:
    eq. 10's plain sum does not depend on the cuts, so the bottleneck stage (which bounds a pipelined
    step) is minimised first, then the communication volume merging is meant to reduce."""
    L = len(layers)
    allowed = [i + 1 for i in range(L - 1) if layers[i]["cut_after"]]
    best = None
    for cuts in itertools.combinations(allowed, Z - 1):
        starts = [0] + list(cuts) + [L]
        costs, bb = plan_cost(layers, starts, cp, layer_costs)
        key = (max(costs), bb, starts)
        if best is None or key < best[0]:
            best = (key, starts, costs)
    if best is None:
        raise ValueError("no plan with %d stages" % Z)
    return best[1], best[2]

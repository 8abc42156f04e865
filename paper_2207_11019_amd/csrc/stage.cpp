// A stage = one sub-module (a stack of consecutive layers) and its three operations
// F_{z,j}, B_{z,j}, U_z.  Host code only: validates, lays out buffers, enqueues kernels.
//
// Layer-wise Partitioning and Merging: sub-module z takes the activation of z-1 in the forward
// pass and the gradient of z+1 in the backward pass.  Problem Statement eqs. 1, 8, 9 define what
// each layer computes in the two passes; eq. 6 the update.
#include "lpm_internal.h"

#include <algorithm>
#include <new>

#include "stage.h"
#include <cmath>

using namespace lpm;

static bool misaligned(const void* p) { return ((uintptr_t)p & 255u) != 0; }

extern "C" int32_t lpm_stage_create(const lpm_layer* layers, int32_t L, int32_t first, int32_t last,
                                    int32_t microbatch, int32_t dtype, lpm_stage** out) {
    if (!out) return fail(LPM_EINVAL, "out is NULL");
    *out = nullptr;
    if (dtype != LPM_F32 && dtype != LPM_BF16) return fail(LPM_EINVAL, "dtype must be LPM_F32 or LPM_BF16");
    if (microbatch <= 0) return fail(LPM_EINVAL, "microbatch must be positive");
    lpm_stage* s = new (std::nothrow) lpm_stage();
    if (!s) return fail(LPM_ENOMEM, "out of host memory");
    int32_t rc = validate_network(layers, L, s->net, s->shapes);
    if (rc) { delete s; return rc; }
    if (first < 0 || last > L || first >= last) { delete s; return fail(LPM_EINVAL, "stage range [%d,%d) is not inside the network", first, last); }
    s->first = first; s->last = last; s->m = microbatch; s->dtype = dtype; s->L = L;
    s->esz = dtype == LPM_BF16 ? 2 : 4;
    s->loss = s->net[last - 1].kind == LPM_SOFTMAX_CE;
    if (s->loss && last - first < 2) { delete s; return fail(LPM_ESHAPE, "the loss layer cannot form a stage on its own"); }
    // every tensor read from outside must be the stage input
    for (int32_t i = first; i < last; ++i) {
        const lpm_layer& l = s->net[i];
        if (l.src < first - 1 || (l.add_src != LPM_NONE && l.add_src < first - 1)) {
            delete s;
            return fail(LPM_ESHAPE, "layer %d reads a tensor produced before the stage input (%d)", i, first - 1);
        }
    }
    // no tensor of this stage other than its output may be read by a later layer
    for (int32_t i = last; i < L; ++i) {
        const lpm_layer& l = s->net[i];
        for (int32_t ref : {l.src, l.add_src}) {
            if (ref != LPM_NONE && ref >= first && ref < last - 1) {
                delete s;
                return fail(LPM_ESHAPE, "layer %d reads tensor %d across the stage boundary", i, ref);
            }
        }
    }

    // tensors first-1 .. last-1
    s->ten.resize((size_t)(last - first + 1));
    s->t_out = s->loss ? last - 2 : last - 1;
    size_t stash = 0, gws = 0;
    for (int32_t t = first - 1; t < last; ++t) {
        TensorRt& tr = s->T(t);
        tr.shape = s->shapes[(size_t)t + 1];
        tr.bytes = tr.shape.elems() * (size_t)microbatch * s->esz;
        if (t == first - 1) tr.loc = LOC_X;
        else if (t == s->t_out || (s->loss && t == last - 1)) tr.loc = LOC_Y;
        else {
            tr.loc = LOC_STASH;
            tr.stash_off = stash;
            stash += align_up(tr.bytes, 256);
            tr.g_off = gws;
            gws += align_up(tr.bytes, 256);
        }
    }
    if (s->loss) {
        s->dlogits_off = stash;
        stash += align_up(s->T(last - 2).bytes, 256);
    }
    s->stash_bytes = stash;

    // parameters: trainable (W, bias per layer) first, frozen scales after
    s->lay.resize((size_t)(last - first));
    size_t off = 0, lowp = 0, kws = 0, wws = 0, fws = 0, fcs = 0;
    for (int32_t i = first; i < last; ++i) {
        LayerRt& lr = s->Ly(i);
        lr.d = s->net[i];
        const lpm_layer& l = lr.d;
        const Shape o = s->shapes[(size_t)i + 1];
        lr.g = ConvGeom{microbatch, l.h_in, l.w_in, l.cin, o.h, o.w, o.c, l.kh, l.kw, l.stride, l.pad};
        if (!has_weights(l)) {
            if (l.kind == LPM_ATTN) {
                if (!attn_ok(l.h_in * l.w_in, l.cout)) { delete s; return fail(LPM_ESHAPE, "layer %d: attention over %d positions of %d channels is outside the kernel's limits", i, l.h_in * l.w_in, l.cout); }
                kws = std::max(kws, align_up(attn_bwd_ws_bytes(microbatch, l.h_in * l.w_in), 256));
            }
            continue;
        }
        if (l.d_in > 1 || l.kd > 1) {          // a volumetric layer: the tensor heights are slices x rows
            lr.g.D = l.d_in; lr.g.Kd = l.kd; lr.g.pad_d = l.pad_d;
            lr.g.Do = (l.d_in + 2 * l.pad_d - l.kd) / l.stride + 1;
            lr.g.Ho = o.h / lr.g.Do;
        }
        lr.w_count = (size_t)l.cout * taps_of(l) * l.cin;
        lr.w_off = off;
        off += align_up(lr.w_count, 64);
        if (l.flags & LPM_BIAS) { lr.b_off = off; off += align_up((size_t)l.cout, 64); }
        if (dtype == LPM_BF16) {
            lr.lowp_w_off = lr.w_off * 2;      // the bf16 copies mirror the float layout element for element
            if (dgrad_uses_wt(dtype, lr.g)) { lr.lowp_wt_off = lowp; lowp += align_up(lr.w_count * 2, 256); }   // rebased below
        }
        // A scaled layer whose weight-gradient kernel also sums the bias gradient keeps dz free of the scale: the bias
        // gradient is then the plain column sum of dz (eq. 8 for the bias), whatever the scale's value -- zero included.
        lr.dz_unscaled = dtype == LPM_BF16 && (l.flags & LPM_SCALE) && wgrad_fuses_bias(dtype, lr.g);
        if (l.flags & (LPM_RELU | LPM_SCALE)) {          // needs its own dz buffer (it outlives the layer's turn)
            lr.dz_off = gws;
            gws += align_up(o.elems() * (size_t)microbatch * s->esz, 256);
        }
        lr.wws_off = wws;                        // every layer its own area: the reductions of a pass run in one launch
        wws += align_up(std::max({wgrad_ws_bytes(dtype, lr.g), wgrad_staged_ws_bytes(dtype, lr.g),
                                  epi_bwd_ws_bytes(lr.g.rows_out(), l.cout)}), 256);   // (a bias-only reduction runs here too)
        if (wgrad_staged_ok(dtype, lr.g)) {
            lr.fcs_x_off = fcs;  fcs += align_up((size_t)LPM_FC_STAGE_SLOTS * lr.g.rows_in() * lr.g.Cin * 2, 256);
            lr.fcs_dz_off = fcs; fcs += align_up((size_t)LPM_FC_STAGE_SLOTS * lr.g.rows_out() * lr.g.Cout * 2, 256);
        }
        kws = std::max(kws, align_up(dgrad_ws_bytes(dtype, lr.g), 256));
        kws = std::max(kws, align_up(epi_bwd_ws_bytes(lr.g.rows_out(), l.cout), 256));
        fws = std::max(fws, align_up(fwd_ws_bytes(dtype, lr.g), 256));
    }
    // Epilogue-backward fusion: when a layer's output feeds exactly one later layer through its `src` edge, that
    // layer's backward kernel (data gradient / pooling backward) applies the ReLU mask and the scale itself and
    // writes dz directly; the bias gradient then comes out of the weight-gradient kernel.
    for (int32_t i = first; i < last; ++i) {
        LayerRt& lr = s->Ly(i);
        const lpm_layer& l = lr.d;
        if (dtype != LPM_BF16 || !has_weights(l) || !(l.flags & (LPM_RELU | LPM_SCALE))) continue;
        if (i == s->t_out) continue;           // its gradient arrives from outside the stage
        int n_src = 0, n_other = 0, n_add = 0;
        int32_t consumer = -1, first_add = last;
        for (int32_t j = i + 1; j < last; ++j) {
            const lpm_layer& c = s->net[j];
            if (c.src == i) { ((c.kind == LPM_SOFTMAX_CE || c.kind == LPM_ATTN) ? n_other : n_src)++; consumer = j; }
            if (c.add_src == i) { ++n_add; first_add = std::min(first_add, j); }
        }
        if (n_src != 1 || n_other != 0) continue;
        if ((l.flags & LPM_BIAS) && !wgrad_fuses_bias(dtype, lr.g)) continue;
        if (l.add_src != LPM_NONE || n_add > 0) {
            // Residual blocks.  The layer adds a shortcut, and / or later layers use its output as their shortcut: the
            // single layer that reads it as its input comes first in layer order, so its data gradient is the last
            // contribution in the backward pass, and an MFMA data gradient can add the earlier ones, mask, and write
            // both this layer's dz and the shortcut's gradient.
            const lpm_layer& c = s->net[(size_t)consumer];
            if (!has_weights(c) || first_add < consumer || !dgrad_has_side(dtype, s->Ly(consumer).g)) continue;
            lr.fused_side = true;
        }
        lr.fused_in = true;
    }
    // ... and a projection shortcut: a scale-only layer (no ReLU, no shortcut of its own) whose output is read by
    // exactly one layer, as its shortcut, when that layer is fused_side: the shortcut gradient that layer's fused
    // epilogue writes is this layer's output gradient, and times this layer's scale it is this layer's dz.
    for (int32_t i = first; i < last; ++i) {
        LayerRt& lr = s->Ly(i);
        const lpm_layer& l = lr.d;
        if (dtype != LPM_BF16 || !has_weights(l) || (l.flags & LPM_RELU) || !(l.flags & LPM_SCALE) || l.add_src != LPM_NONE) continue;
        if (i == s->t_out) continue;
        if ((l.flags & LPM_BIAS) && !wgrad_fuses_bias(dtype, lr.g)) continue;
        int n_src = 0, n_add = 0;
        int32_t user = -1;
        for (int32_t j = i + 1; j < last; ++j) {
            if (s->net[(size_t)j].src == i) ++n_src;
            if (s->net[(size_t)j].add_src == i) { ++n_add; user = j; }
        }
        if (n_src != 0 || n_add != 1 || !s->Ly(user).fused_side) continue;
        lr.fused_in = true;
        lr.via_shortcut = true;
    }
    // Pooling-backward fusion: a 2x2 max-pooling (even input extent) whose output feeds exactly one layer, a
    // convolution whose data gradient runs on the stride-1 MFMA kernel: that kernel routes its result to the
    // window maxima itself and the gradient of the pooling output is never stored.
    for (int32_t i = first; i < last; ++i) {
        LayerRt& lr = s->Ly(i);
        const lpm_layer& l = lr.d;
        if (!has_weights(l) || l.src < first || s->net[(size_t)l.src].kind != LPM_MAXPOOL2) continue;
        const int32_t p = l.src;
        const lpm_layer& pl = s->net[(size_t)p];
        if (p == s->t_out || (pl.h_in & 1) || (pl.w_in & 1) || !dgrad_can_unpool(dtype, lr.g) || !dgrad_uses_wt(dtype, lr.g)) continue;
        int n_cons = 0;
        for (int32_t j = p + 1; j < last; ++j) n_cons += (s->net[(size_t)j].src == p) + (s->net[(size_t)j].add_src == p);
        if (n_cons != 1) continue;
        lr.unpool_of = p;
        s->Ly(p).unpooled = true;
    }
    // Pooling-forward fusion: a convolution whose output feeds a 2x2 max-pooling inside the stage and whose forward
    // contraction ends in a split reduction: that reduction stores the pooled tensor as well (one kernel less per pool
    // on the forward chain; the pooling layer's own input stays stored, the backward pass needs it).
    for (int32_t i = first; i + 1 < last; ++i) {
        LayerRt& lr = s->Ly(i);
        const lpm_layer& l = lr.d;
        const lpm_layer& pl = s->net[(size_t)i + 1];
        if (!has_weights(l) || l.add_src != LPM_NONE || pl.kind != LPM_MAXPOOL2 || pl.src != i) continue;
        if ((pl.h_in & 1) || (pl.w_in & 1) || !fwd_can_pool(dtype, lr.g)) continue;
        lr.pool_fwd = i + 1;
        s->Ly(i + 1).pooled_fwd = true;
    }
    s->n_trainable = off;
    if (dtype == LPM_BF16) {                   // transposed copies follow the mirrored region
        const size_t base = align_up(off * 2, 256);
        for (int32_t i = first; i < last; ++i)
            if (s->Ly(i).lowp_wt_off != NO) s->Ly(i).lowp_wt_off += base;
        lowp += base;
    }
    for (int32_t i = first; i < last; ++i) {
        LayerRt& lr = s->Ly(i);
        if (has_weights(lr.d) && (lr.d.flags & LPM_SCALE)) { lr.s_off = off; off += align_up((size_t)lr.d.cout, 64); }
    }
    s->n_params = off;
    s->lowp_bytes = lowp;
    // backward scratch: two copies of the gradient / dz area (a schedule alternates between them so the weight
    // phase of one micro-batch may still read its dz while the next data phase writes), then kernel scratch
    s->gws_bytes = gws;
    s->kws_off = 2 * gws;
    s->wws_off = 2 * gws + kws;
    for (int32_t i = first; i < last; ++i) {     // the staging areas follow the kernel scratch
        LayerRt& lr = s->Ly(i);
        if (lr.fcs_x_off != NO) { lr.fcs_x_off += 2 * gws + kws + wws; lr.fcs_dz_off += 2 * gws + kws + wws; }
    }
    s->bwd_ws = std::max<size_t>(2 * gws + kws + wws + fcs, 256);
    s->fwd_ws = std::max<size_t>(fws, 256);
    *out = s;
    return LPM_OK;
}

lpm_stage::~lpm_stage() {
    if (ev_fork) (void)hipEventDestroy(ev_fork);
    if (ev_join) (void)hipEventDestroy(ev_join);
    if (ev_w2_fork) (void)hipEventDestroy(ev_w2_fork);
    if (ev_w2_join) (void)hipEventDestroy(ev_w2_join);
    for (hipEvent_t v : ev_layer) if (v) (void)hipEventDestroy(v);
}

// Borrows the side stream and creates the events on first use (needs a device; stage creation does not).
int32_t lpm_stage_prepare(lpm_stage* s) {
    if (s->side) return LPM_OK;
    hipStream_t st = nullptr;
    LPM_HIP(pooled_stream(next_side_stream_index(), &st));
    hipEvent_t ej = nullptr, ef = nullptr, e2f = nullptr, e2j = nullptr;
    hipError_t e = hipEventCreateWithFlags(&ej, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ef, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&e2f, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&e2j, hipEventDisableTiming);
    if (e != hipSuccess) {
        if (ej) (void)hipEventDestroy(ej);
        if (ef) (void)hipEventDestroy(ef);
        if (e2f) (void)hipEventDestroy(e2f);
        return hip_fail(e, "hipEventCreateWithFlags");
    }
    std::vector<hipEvent_t> evl((size_t)(s->last - s->first) * LPM_MAX_WINDOW, nullptr);
    for (int32_t i = s->first; i < s->last && e == hipSuccess; ++i) {
        if (!has_weights(s->Ly(i).d)) continue;
        for (int k = 0; k < LPM_MAX_WINDOW && e == hipSuccess; ++k)
            e = hipEventCreateWithFlags(&evl[(size_t)(i - s->first) * LPM_MAX_WINDOW + k], hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        for (hipEvent_t v : evl) if (v) (void)hipEventDestroy(v);
        (void)hipEventDestroy(ej); (void)hipEventDestroy(ef); (void)hipEventDestroy(e2f); (void)hipEventDestroy(e2j);
        return hip_fail(e, "hipEventCreateWithFlags");
    }
    s->ev_layer = std::move(evl);
    s->ev_join = ej;
    s->ev_fork = ef;
    s->ev_w2_fork = e2f;
    s->ev_w2_join = e2j;
    s->side = st;
    return LPM_OK;
}

extern "C" int32_t lpm_stage_destroy(lpm_stage* s) {
    delete s;
    return LPM_OK;
}

extern "C" int32_t lpm_stage_sizes(const lpm_stage* s, size_t* param_bytes, size_t* lowp_bytes, size_t* grad_bytes,
                                   size_t* stash_bytes, size_t* fwd_ws_bytes_, size_t* bwd_ws_bytes,
                                   size_t* in_bytes, size_t* out_bytes) {
    if (!s) return fail(LPM_EINVAL, "stage is NULL");
    if (param_bytes) *param_bytes = std::max<size_t>(s->n_params * 4, 256);
    if (lowp_bytes) *lowp_bytes = s->lowp_bytes;
    if (grad_bytes) *grad_bytes = std::max<size_t>(s->n_trainable * 4, 256);
    if (stash_bytes) *stash_bytes = std::max<size_t>(s->stash_bytes, 256);
    if (fwd_ws_bytes_) *fwd_ws_bytes_ = s->fwd_ws;
    if (bwd_ws_bytes) *bwd_ws_bytes = s->bwd_ws;
    if (in_bytes) *in_bytes = s->T(s->first - 1).bytes;
    if (out_bytes) *out_bytes = s->T(s->t_out).bytes;
    return LPM_OK;
}

extern "C" int32_t lpm_stage_param_offset(const lpm_stage* s, int32_t layer, int32_t which, size_t* offset, size_t* count) {
    if (!s || !offset || !count) return fail(LPM_EINVAL, "NULL argument");
    if (layer < s->first || layer >= s->last) return fail(LPM_EINVAL, "layer %d is not in the stage", layer);
    const LayerRt& lr = s->Ly(layer);
    size_t o = NO, c = 0;
    if (which == 0) { o = lr.w_off; c = lr.w_count; }
    else if (which == 1) { o = lr.b_off; c = (size_t)lr.d.cout; }
    else if (which == 2) { o = lr.s_off; c = (size_t)lr.d.cout; }
    if (o == NO) return fail(LPM_EINVAL, "layer %d has no parameter tensor %d", layer, which);
    *offset = o; *count = c;
    return LPM_OK;
}

extern "C" int32_t lpm_stage_stash_offset(const lpm_stage* s, int32_t t, size_t* offset, size_t* bytes) {
    if (!s || !offset || !bytes) return fail(LPM_EINVAL, "NULL argument");
    if (t == -100) {
        if (!s->loss) return fail(LPM_EINVAL, "not a loss stage");
        *offset = s->dlogits_off; *bytes = s->T(s->last - 2).bytes;
        return LPM_OK;
    }
    if (t < s->first - 1 || t >= s->last || s->T(t).loc != LOC_STASH) return fail(LPM_EINVAL, "tensor %d is not in the stash", t);
    *offset = s->T(t).stash_off; *bytes = s->T(t).bytes;
    return LPM_OK;
}

extern "C" int32_t lpm_stage_grad_offset(const lpm_stage* s, int32_t t, size_t* offset, size_t* bytes) {
    if (!s || !offset || !bytes) return fail(LPM_EINVAL, "NULL argument");
    if (t < s->first - 1 || t >= s->last || s->T(t).loc != LOC_STASH) return fail(LPM_EINVAL, "tensor %d has no gradient in the scratch", t);
    *offset = s->T(t).g_off; *bytes = s->T(t).bytes;
    return LPM_OK;
}

// the [Cin][Kh][Kw][Cout] copies of every layer whose data gradient reads one, all in one launch
static hipError_t transpose_copies(const lpm_stage* s, const float* params, void* lowp, hipStream_t st) {
    std::vector<TransposeDesc> d;
    for (int32_t i = s->first; i < s->last; ++i) {
        const LayerRt& lr = s->Ly(i);
        if (lr.lowp_wt_off != NO)
            d.push_back(TransposeDesc{params + lr.w_off, (uint16_t*)((char*)lowp + lr.lowp_wt_off), lr.d.cout, taps_of(lr.d), lr.d.cin,
                                      lr.dz_unscaled ? params + lr.s_off : nullptr});
    }
    return d.empty() ? hipSuccess : launch_weight_transpose_batch(d.data(), (int)d.size(), st);
}

extern "C" int32_t lpm_stage_sync_lowp(lpm_stage* s, const float* params, void* lowp, void* stream) {
    if (!s || !params) return fail(LPM_EINVAL, "NULL argument");
    if (s->dtype != LPM_BF16) return LPM_OK;
    if (!lowp) return fail(LPM_EINVAL, "lowp is NULL");
    if (misaligned(params) || misaligned(lowp)) return fail(LPM_EALIGN, "buffers must be 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    LPM_HIP(launch_f32_to_bf16(params, (uint16_t*)lowp, s->n_trainable, st));
    LPM_HIP(transpose_copies(s, params, lowp, st));
    return LPM_OK;
}

namespace {
// Where tensor t lives for this call.
inline const void* tptr(const lpm_stage* s, int32_t t, const void* x, const void* y, const void* stash) {
    const TensorRt& tr = s->T(t);
    if (tr.loc == LOC_X) return x;
    if (tr.loc == LOC_Y) return y;
    return (const char*)stash + tr.stash_off;
}
}  // namespace

extern "C" int32_t lpm_stage_forward(lpm_stage* s, const void* x, void* y, const int32_t* labels, float* loss_accum,
                                     const float* params, const void* lowp, void* stash, void* fwd_ws,
                                     float loss_scale, void* stream) {
    if (!s || !x || !y || !params || !stash || !fwd_ws) return fail(LPM_EINVAL, "NULL argument");
    if (s->dtype == LPM_BF16 && !lowp) return fail(LPM_EINVAL, "lowp is NULL for a bf16 stage");
    if (s->loss && (!labels || !loss_accum)) return fail(LPM_EINVAL, "a loss stage needs labels and loss_accum");
    if (misaligned(x) || misaligned(y) || misaligned(params) || misaligned(stash) || misaligned(fwd_ws) ||
        (lowp && misaligned(lowp)))
        return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    if (s->loss && (((uintptr_t)labels & 3u) || ((uintptr_t)loss_accum & 3u))) return fail(LPM_EALIGN, "labels / loss_accum must be 4-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    for (int32_t i = s->first; i < s->last; ++i) {
        const LayerRt& lr = s->Ly(i);
        const lpm_layer& l = lr.d;
        const void* in = tptr(s, l.src, x, y, stash);
        void* outp = const_cast<void*>(tptr(s, i, x, y, stash));
        switch (l.kind) {
            case LPM_CONV:
            case LPM_FC: {
                const void* w = s->dtype == LPM_BF16 ? (const void*)((const char*)lowp + lr.lowp_w_off)
                                                     : (const void*)(params + lr.w_off);
                const float* sc = lr.s_off != NO ? params + lr.s_off : nullptr;
                const float* bi = lr.b_off != NO ? params + lr.b_off : nullptr;
                const void* add = l.add_src != LPM_NONE ? tptr(s, l.add_src, x, y, stash) : nullptr;
                void* pooled = lr.pool_fwd >= 0 ? const_cast<void*>(tptr(s, lr.pool_fwd, x, y, stash)) : nullptr;
                LPM_HIP(launch_conv_fwd(s->dtype, lr.g, in, w, sc, bi, add, (l.flags & LPM_RELU) != 0, outp, fwd_ws, st, pooled));
                break;
            }
            case LPM_MAXPOOL2:
                if (lr.pooled_fwd) break;        // stored by the producer's forward kernel
                LPM_HIP(launch_maxpool_fwd(s->dtype, s->m, l.h_in, l.w_in, l.cin, in, outp, st));
                break;
            case LPM_GAP:
                LPM_HIP(launch_gap_fwd(s->dtype, s->m, l.h_in * l.w_in, l.cin, in, outp, st));
                break;
            case LPM_ATTN:
                LPM_HIP(launch_attn_fwd(s->dtype, s->m, l.h_in * l.w_in, l.cout, in, outp, st));
                break;
            case LPM_SOFTMAX_CE:
                LPM_HIP(launch_softmax_ce(s->dtype, s->m, l.cin, in, labels, loss_scale, (char*)stash + s->dlogits_off,
                                          loss_accum, st));
                break;
        }
    }
    return LPM_OK;
}

extern "C" int32_t lpm_stage_backward(lpm_stage* s, const void* x, const void* y, const void* dy, void* dx,
                                      const float* params, const void* lowp, const void* stash, float* grads,
                                      int32_t accumulate, void* bwd_ws, void* stream) {
    return lpm_stage_backward_on(s, x, y, dy, dx, params, lowp, stash, grads, accumulate, bwd_ws, stream, nullptr, 0, LPM_PHASE_DATA | LPM_PHASE_WEIGHTS);
}

// B_{z,j} in two phases.  Data phase (on `stream`): everything the next stage down waits for -- epilogue
// backward, pooling backward, data gradients -- leaving every layer's dz in the backward scratch.  Weight
// phase: the weight (and fused bias) gradients, which nothing in the same pass reads, enqueued after the
// data phase on `wstream` behind a single event.  wstream == stream: no event at all (fully serial);
// wstream == NULL: the stage's own side stream, joined back into `stream` before returning (the
// contract of lpm_stage_backward); any other stream: the caller orders later work after it.
// phases: LPM_PHASE_DATA | LPM_PHASE_WEIGHTS as described; LPM_PHASE_DATA alone enqueues only the data
// phase; LPM_PHASE_WEIGHTS alone only the weight phase on wstream, with no event -- the caller has ordered
// wstream after the data phase (separate enqueue threads for the two).
// parity (0 / 1) selects the copy of the gradient / dz area in bwd_ws this pass uses.
// While `stream` is being captured the weight gradients stay on it and are taken out of its dependency
// frontier instead.
// wstream2 (with wstream, eager only): every other weight gradient of the phase runs on this second stream, forked from
// wstream at the start of the phase and joined back into it before the reduction of the partial sums -- a weight
// gradient is some 250 blocks and half fixed cost, so two of them side by side fill what one leaves idle.
int32_t lpm_stage_backward_on(lpm_stage* s, const void* x, const void* y, const void* dy, void* dx,
                              const float* params, const void* lowp, const void* stash, float* grads,
                              int32_t accumulate, void* bwd_ws, void* stream, void* wstream, int32_t parity,
                              int32_t phases, int32_t fc_slot, int32_t fc_flush, int32_t layer_slot, int32_t boundary, void* wstream2) {
    if ((boundary & LPM_MASK_DX) && !lpm_stage_can_mask_dx(s)) return fail(LPM_EINVAL, "internal: this stage cannot mask its input gradient");
    if ((boundary & LPM_DY_IS_DZ) && !lpm_stage_takes_dz(s)) return fail(LPM_EINVAL, "internal: this stage needs the gradient of its output");
    if (layer_slot >= LPM_MAX_WINDOW) return fail(LPM_EINVAL, "internal: layer event slot out of range");
    if (fc_slot >= LPM_FC_STAGE_SLOTS || fc_flush > LPM_FC_STAGE_SLOTS) return fail(LPM_EINVAL, "internal: staging slot out of range");
    if (!s || !x || !y || !params || !stash || !grads || !bwd_ws) return fail(LPM_EINVAL, "NULL argument");
    if (!s->loss && !dy) return fail(LPM_EINVAL, "dy is NULL for a stage that is not a loss stage");
    if (s->dtype == LPM_BF16 && !lowp) return fail(LPM_EINVAL, "lowp is NULL for a bf16 stage");
    if (misaligned(x) || misaligned(y) || misaligned(params) || misaligned(stash) || misaligned(grads) ||
        misaligned(bwd_ws) || (dy && misaligned(dy)) || (dx && misaligned(dx)) || (lowp && misaligned(lowp)))
        return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    const int32_t first = s->first, last = s->last;
    const bool acc = accumulate != 0;
    char* ws = (char*)bwd_ws;
    void* kws = ws + s->kws_off;
    void* wws = ws + s->wws_off;
    char* gw = ws + (parity ? s->gws_bytes : 0);
    int32_t prc = lpm_stage_prepare(s);
    if (prc) return prc;
    // While the caller's stream is being captured into a graph no second stream is involved: the weight
    // gradient nodes are taken out of the stream's dependency frontier instead (they depend on what came
    // before them and on the previous weight gradient, nothing later depends on them until the join).
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    LPM_HIP(hipStreamIsCapturing(st, &cap));
    const bool deferred = cap == hipStreamCaptureStatusNone;
    const bool do_data = (phases & LPM_PHASE_DATA) != 0, do_weights = (phases & LPM_PHASE_WEIGHTS) != 0;
    if (!deferred && !(do_data && do_weights)) return fail(LPM_EINVAL, "a captured backward pass cannot be split into phases");
    if (!do_data && (!do_weights || !wstream)) return fail(LPM_EINVAL, "internal: bad phase selection");
    // layer_slot >= 0 (the two phases come as separate calls with the same slot): the data phase records, per weight
    // layer, the point in its stream where that layer's output gradient is final, and the weight phase waits for
    // that point before the layer's weight gradient instead of for the end of the data phase
    const bool by_layer = layer_slot >= 0 && deferred && (do_data != do_weights);
    // bias_g != NULL: the layer's bias gradient is a plain column sum of bias_g that nothing in the data phase needs;
    // it runs in the weight phase, ahead of the layer's weight gradient (scratch: the layer's own area)
    struct WgradJob { const LayerRt* lr; const void* xin; const void* dz; float* wdb; const float* sc; const void* bias_g; float* bias_db; };
    // One weight gradient on stream q.  fc_slot = j >= 0 (of fc_flush = M micro-batches): a layer with staging areas
    // files its operands under slot j and contracts a group of slots at a time; the first group overwrites the accumulator.
    auto one_wgrad = [&](const WgradJob& j, hipStream_t q, ReduceDesc* d) -> hipError_t {
        const LayerRt& lr = *j.lr;
        if (fc_slot >= 0 && lr.fcs_x_off != NO) {
            if (d) d->splits = 0;
            hipError_t e = stage_operands(lr.g, j.xin, j.dz, ws + lr.fcs_x_off, ws + lr.fcs_dz_off, fc_slot, q);
            if (e != hipSuccess) return e;
            // Contract in groups of G micro-batches.  One group (G = M) touches dW once, but all of that work then sits
            // behind the last micro-batch, where nothing overlaps it; two groups leave half of it there.  Gradient
            // matrices of 64 MiB and more are bound by their own traffic and keep the single pass.
            const int32_t M = fc_flush;
            const int32_t G = ((size_t)lr.w_count * 4 >= ((size_t)64 << 20)) ? M : std::max(1, (M + 1) / 2);
            if ((fc_slot + 1) % G != 0 && fc_slot != M - 1) return hipSuccess;
            const int32_t j0 = (fc_slot / G) * G;
            const size_t xb = (size_t)lr.g.rows_in() * lr.g.Cin * 2, db = (size_t)lr.g.rows_out() * lr.g.Cout * 2;
            return launch_wgrad_staged(s->dtype, lr.g, ws + lr.fcs_x_off + (size_t)j0 * xb, ws + lr.fcs_dz_off + (size_t)j0 * db,
                                       fc_slot - j0 + 1, grads + lr.w_off, j.wdb, j.sc, j0 > 0, (char*)wws + lr.wws_off, q, d);
        }
        return launch_conv_wgrad(s->dtype, lr.g, j.xin, j.dz, grads + lr.w_off, j.wdb, j.sc, acc, (char*)wws + lr.wws_off, q, d);
    };
    std::vector<WgradJob> jobs;            // eager: the weight phase, in layer order (last layer first)
    std::vector<hipGraphNode_t> wtail;     // capture: frontier left by the last weight gradient
    auto frontier = [&](std::vector<hipGraphNode_t>& out) -> hipError_t {
        hipStreamCaptureStatus stt;
        const hipGraphNode_t* deps = nullptr;
        size_t nd = 0;
        hipError_t e = hipStreamGetCaptureInfo_v2(st, &stt, nullptr, nullptr, &deps, &nd);
        if (e == hipSuccess) out.assign(deps, deps + nd);
        return e;
    };

    // gradient buffer of every tensor, and whether it already holds a contribution
    std::vector<void*> G((size_t)(last - first + 1), nullptr);
    std::vector<char> have((size_t)(last - first + 1), 0);
    auto gi = [&](int32_t t) { return (size_t)(t - (first - 1)); };
    for (int32_t t = first; t < last; ++t)
        if (s->T(t).loc == LOC_STASH) G[gi(t)] = gw + s->T(t).g_off;
    G[gi(first - 1)] = dx;
    int32_t top = last - 1;
    if (s->loss) {
        top = last - 2;
        G[gi(top)] = const_cast<char*>((const char*)stash) + s->dlogits_off;
    } else {
        G[gi(top)] = const_cast<void*>(dy);
    }
    have[gi(top)] = 1;

    for (int32_t i = top; i >= first; --i) {
        const LayerRt& lr = s->Ly(i);
        const lpm_layer& l = lr.d;
        const void* g = G[gi(i)];
        if (!have[gi(i)]) return fail(LPM_ESHAPE, "internal: tensor %d has no consumer", i);
        const bool want_src = (l.src >= first) || (dx != nullptr);
        switch (l.kind) {
            case LPM_CONV:
            case LPM_FC: {
                const void* yout = tptr(s, i, x, y, stash);
                const float* sc = lr.s_off != NO ? params + lr.s_off : nullptr;
                const bool relu = (l.flags & LPM_RELU) != 0;
                float* dbias = lr.b_off != NO ? grads + lr.b_off : nullptr;
                const bool bias_in_wgrad = dbias && wgrad_fuses_bias(s->dtype, lr.g);
                const void* dz = g;
                const void* bias_g = nullptr;
                if (lr.fused_in) {
                    dz = gw + lr.dz_off;           // written by the consumer's backward kernel
                } else if (i == s->t_out && (boundary & LPM_DY_IS_DZ)) {
                    dz = g;                        // the next stage applied this layer's ReLU mask to what it handed down
                } else {
                    void* gadd = nullptr;
                    int gadd_acc = 0;
                    if (l.add_src != LPM_NONE && ((l.add_src >= first) || dx != nullptr)) {
                        gadd = G[gi(l.add_src)];
                        gadd_acc = have[gi(l.add_src)];
                        have[gi(l.add_src)] = 1;
                    }
                    const bool need_dz = relu || sc;
                    if (!need_dz && !gadd && dbias && !bias_in_wgrad && deferred) {
                        bias_g = g;
                    } else if (need_dz || gadd || (dbias && !bias_in_wgrad)) {
                        if (do_data) LPM_HIP(launch_epilogue_bwd(s->dtype, lr.g.rows_out(), l.cout, g, relu ? yout : nullptr, lr.dz_unscaled ? nullptr : sc,
                                                    need_dz ? (void*)(gw + lr.dz_off) : nullptr, gadd, gadd_acc,
                                                    bias_in_wgrad ? nullptr : dbias, acc, kws, st));
                        if (need_dz) dz = gw + lr.dz_off;
                    }
                }
                if (by_layer && do_data) LPM_HIP(hipEventRecord(s->ev_layer[(size_t)(i - first) * LPM_MAX_WINDOW + layer_slot], st));
                float* wdb = bias_in_wgrad ? dbias : nullptr;
                // where the gradient w.r.t. this layer's input goes: the producer's dz (fused) or the tensor's gradient
                void* gsrc = nullptr;
                int gsrc_acc = 0;
                const void* gmask = nullptr;
                const float* gmscale = nullptr;
                const bool want = (l.src >= first) || (dx != nullptr);
                UnpoolDesc unpool{};
                if (lr.unpool_of >= 0) {
                    // this layer's input is a max-pooling output nobody else reads: route the data gradient through the
                    // pooling to where the pooling backward would have written (the same choices as in the pooling case below)
                    const int32_t p = lr.unpool_of, q = s->Ly(p).d.src;
                    have[gi(p)] = 1;
                    if (q >= first || dx != nullptr) {
                        unpool.pool_x = tptr(s, q, x, y, stash);
                        unpool.dst = G[gi(q)];
                        unpool.accumulate = have[gi(q)];
                        if (q >= first && s->Ly(q).fused_in) {
                            const LayerRt& pr = s->Ly(q);
                            unpool.dst = gw + pr.dz_off;
                            unpool.accumulate = 0;
                            unpool.mask = (pr.d.flags & LPM_RELU) != 0;
                            unpool.mscale = (pr.s_off != NO && !pr.dz_unscaled) ? params + pr.s_off : nullptr;
                        } else if (q == first - 1 && (boundary & LPM_MASK_DX)) {
                            unpool.mask = 1;
                        }
                        have[gi(q)] = 1;
                    }
                }
                DgradSide side{};
                bool use_side = false;
                if (want && lr.unpool_of < 0) {
                    if (l.src >= first && s->Ly(l.src).fused_in) {
                        const LayerRt& pr = s->Ly(l.src);
                        gsrc = gw + pr.dz_off;
                        gmask = (pr.d.flags & LPM_RELU) ? tptr(s, l.src, x, y, stash) : nullptr;
                        gmscale = (pr.s_off != NO && !pr.dz_unscaled) ? params + pr.s_off : nullptr;
                        if (pr.fused_side) {
                            // the producer sits in a residual block: what its shortcut users have already put into its output
                            // gradient is added, and the masked sum is also the gradient of the producer's own shortcut
                            use_side = true;
                            side.earlier = have[gi(l.src)] ? G[gi(l.src)] : nullptr;
                            const int32_t a = pr.d.add_src;
                            if (a != LPM_NONE && a >= first && s->Ly(a).via_shortcut) {
                                side.shortcut = gw + s->Ly(a).dz_off;           // the projection's dz
                                side.shortcut_scale = s->Ly(a).dz_unscaled ? nullptr : params + s->Ly(a).s_off;
                                have[gi(a)] = 1;
                            } else if (a != LPM_NONE && (a >= first || dx != nullptr)) {
                                side.shortcut = G[gi(a)];
                                side.shortcut_acc = have[gi(a)];
                                have[gi(a)] = 1;
                            }
                        }
                    } else {
                        gsrc = G[gi(l.src)];
                        gsrc_acc = have[gi(l.src)];
                        if (l.src == first - 1 && (boundary & LPM_MASK_DX)) gmask = x;      // ReLU backward of the previous stage's last layer
                    }
                    have[gi(l.src)] = 1;
                }
                const void* xin = tptr(s, l.src, x, y, stash);
                if (deferred) {
                    jobs.push_back(WgradJob{&lr, xin, dz, wdb, lr.dz_unscaled ? sc : nullptr, bias_g, bias_g ? dbias : nullptr});
                } else {
                    std::vector<hipGraphNode_t> before;
                    LPM_HIP(frontier(before));
                    if (!wtail.empty())       // weight gradients share one scratch area: keep them in a chain
                        LPM_HIP(hipStreamUpdateCaptureDependencies(st, wtail.data(), wtail.size(), hipStreamAddCaptureDependencies));
                    LPM_HIP(one_wgrad(WgradJob{&lr, xin, dz, wdb, lr.dz_unscaled ? sc : nullptr, nullptr, nullptr}, st, nullptr));
                    LPM_HIP(frontier(wtail));
                    LPM_HIP(hipStreamUpdateCaptureDependencies(st, before.data(), before.size(), hipStreamSetCaptureDependencies));
                }
                if (want) {
                    const void* w = s->dtype == LPM_BF16 ? (const void*)((const char*)lowp + lr.lowp_w_off)
                                                         : (const void*)(params + lr.w_off);
                    const void* wt = (s->dtype == LPM_BF16 && lr.lowp_wt_off != NO)
                                         ? (const void*)((const char*)lowp + lr.lowp_wt_off) : nullptr;
                    if (lr.unpool_of >= 0) {
                        if (do_data && unpool.dst) LPM_HIP(launch_conv_dgrad(s->dtype, lr.g, dz, w, wt, nullptr, 0, nullptr, nullptr, kws, st, &unpool,
                                                                             nullptr, lr.dz_unscaled ? sc : nullptr));
                    } else if (do_data) {
                        LPM_HIP(launch_conv_dgrad(s->dtype, lr.g, dz, w, wt, gsrc, gsrc_acc, gmask, gmscale, kws, st, nullptr,
                                                  use_side ? &side : nullptr, lr.dz_unscaled ? sc : nullptr));
                    }
                }
                break;
            }
            case LPM_MAXPOOL2:
            case LPM_GAP:
                if (lr.unpooled) break;          // done by the consumer's data gradient
                if (want_src) {
                    void* gsrc = G[gi(l.src)];
                    int gsrc_acc = have[gi(l.src)];
                    const void* gmask = nullptr;
                    const float* gmscale = nullptr;
                    if (l.src >= first && s->Ly(l.src).fused_in) {
                        const LayerRt& pr = s->Ly(l.src);
                        gsrc = gw + pr.dz_off;
                        gsrc_acc = 0;
                        gmask = (pr.d.flags & LPM_RELU) ? tptr(s, l.src, x, y, stash) : nullptr;
                        gmscale = (pr.s_off != NO && !pr.dz_unscaled) ? params + pr.s_off : nullptr;
                    } else if (l.src == first - 1 && (boundary & LPM_MASK_DX)) {
                        gmask = x;
                    }
                    if (do_data && l.kind == LPM_MAXPOOL2)
                        LPM_HIP(launch_maxpool_bwd(s->dtype, s->m, l.h_in, l.w_in, l.cin, tptr(s, l.src, x, y, stash),
                                                   tptr(s, i, x, y, stash), g, gsrc, gsrc_acc, gmask != nullptr, gmscale, st));
                    else if (do_data)
                        LPM_HIP(launch_gap_bwd(s->dtype, s->m, l.h_in * l.w_in, l.cin, g, gsrc, gsrc_acc, gmask, gmscale, st));
                    have[gi(l.src)] = 1;
                }
                break;
            case LPM_ATTN:
                if (want_src) {
                    if (do_data)
                        LPM_HIP(launch_attn_bwd(s->dtype, s->m, l.h_in * l.w_in, l.cout, tptr(s, l.src, x, y, stash), g, G[gi(l.src)],
                                                have[gi(l.src)], kws, st));
                    have[gi(l.src)] = 1;
                }
                break;
            default:
                return fail(LPM_ESHAPE, "internal: unexpected layer kind in backward");
        }
    }
    if (!wtail.empty())
        LPM_HIP(hipStreamUpdateCaptureDependencies(st, wtail.data(), wtail.size(), hipStreamAddCaptureDependencies));
    if (do_weights && (!jobs.empty() || (wstream && wstream != stream && deferred))) {
        hipStream_t wst = wstream ? (hipStream_t)wstream : s->side;
        if (wst != st && do_data) {
            LPM_HIP(hipEventRecord(s->ev_fork, st));
            LPM_HIP(hipStreamWaitEvent(wst, s->ev_fork, 0));
        }
        std::vector<ReduceDesc> red;
        red.reserve(jobs.size());
        hipStream_t wst2 = (wstream && wstream2 && deferred && jobs.size() > 1) ? (hipStream_t)wstream2 : nullptr;
        if (wst2 == wst) wst2 = nullptr;
        if (wst2) {        // ordered after everything the phase's stream holds (the previous micro-batch's reduction reads the areas written now)
            LPM_HIP(hipEventRecord(s->ev_w2_fork, wst));
            LPM_HIP(hipStreamWaitEvent(wst2, s->ev_w2_fork, 0));
        }
        size_t k = 0;
        for (const WgradJob& j : jobs) {
            ReduceDesc d{};
            hipStream_t q = (wst2 && (k++ & 1)) ? wst2 : wst;
            if (by_layer)
                LPM_HIP(hipStreamWaitEvent(q, s->ev_layer[(size_t)(j.lr - &s->lay[0]) * LPM_MAX_WINDOW + layer_slot], 0));
            if (j.bias_g)
                LPM_HIP(launch_epilogue_bwd(s->dtype, j.lr->g.rows_out(), j.lr->d.cout, j.bias_g, nullptr, nullptr, nullptr, nullptr, 0,
                                            j.bias_db, acc, (char*)wws + j.lr->wws_off, q));
            LPM_HIP(one_wgrad(j, q, &d));
            if (d.splits > 0) red.push_back(d);
        }
        if (wst2) {
            LPM_HIP(hipEventRecord(s->ev_w2_join, wst2));
            LPM_HIP(hipStreamWaitEvent(wst, s->ev_w2_join, 0));
        }
        if (!red.empty()) LPM_HIP(launch_reduce_batch(red.data(), (int)red.size(), wst));
        if (!wstream) {      // join: the caller's stream is ordered after every weight gradient
            LPM_HIP(hipEventRecord(s->ev_join, s->side));
            LPM_HIP(hipStreamWaitEvent(st, s->ev_join, 0));
        }
    }
    return LPM_OK;
}

bool lpm_stage_can_mask_dx(const lpm_stage* s) {
    if (!s || s->dtype != LPM_BF16 || s->first == 0) return false;
    int n = 0;
    for (int32_t i = s->first; i < s->last; ++i) {
        const lpm_layer& l = s->net[(size_t)i];
        if (l.add_src == s->first - 1) return false;
        if (l.src != s->first - 1) continue;
        if (l.kind != LPM_CONV && l.kind != LPM_FC && l.kind != LPM_MAXPOOL2 && l.kind != LPM_GAP) return false;
        ++n;
    }
    return n == 1;
}

bool lpm_stage_takes_dz(const lpm_stage* s) {
    if (!s || s->dtype != LPM_BF16 || s->loss) return false;
    const int32_t i = s->t_out;
    if (i != s->last - 1) return false;
    const LayerRt& lr = s->Ly(i);
    const lpm_layer& l = lr.d;
    if (!has_weights(l) || !(l.flags & LPM_RELU) || (l.flags & LPM_SCALE) || l.add_src != LPM_NONE) return false;
    return !(l.flags & LPM_BIAS) || wgrad_fuses_bias(s->dtype, lr.g);
}

extern "C" int32_t lpm_stage_update(lpm_stage* s, float* params, void* lowp, float* grads, float* momentum,
                                    float lr_, float mu, int32_t zero_grads, void* stream) {
    return lpm_stage_update_to(s, params, params, lowp, grads, momentum, lr_, mu, zero_grads, stream);
}

// U with the new weights written to another buffer than the one they are read from (params_out may equal
// params_in): the asynchronous update keeps two versions of a stage's weights.  Frozen scales are not touched.
int32_t lpm_stage_update_to(lpm_stage* s, const float* params_in, float* params, void* lowp, float* grads, float* momentum,
                            float lr_, float mu, int32_t zero_grads, void* stream) {
    if (!s || !params_in || !params || !grads || !momentum) return fail(LPM_EINVAL, "NULL argument");
    if (s->dtype == LPM_BF16 && !lowp) return fail(LPM_EINVAL, "lowp is NULL for a bf16 stage");
    if (misaligned(params_in) || misaligned(params) || misaligned(grads) || misaligned(momentum) || (lowp && misaligned(lowp)))
        return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    if (s->n_trainable == 0) return LPM_OK;
    if (s->dtype != LPM_BF16) {
        LPM_HIP(launch_sgd(params_in, params, nullptr, grads, momentum, s->n_trainable, lr_, mu, zero_grads, st));
        return LPM_OK;
    }
    LPM_HIP(launch_sgd(params_in, params, (uint16_t*)lowp, grads, momentum, s->n_trainable, lr_, mu, zero_grads, st));
    LPM_HIP(transpose_copies(s, params, lowp, st));
    return LPM_OK;
}

extern "C" int32_t lpm_stage_update_adam(lpm_stage* s, float* params, void* lowp, float* grads, float* m1, float* m2,
                                         float lr_, float beta1, float beta2, float eps, int32_t step, int32_t zero_grads,
                                         void* stream) {
    if (!s || !params || !grads || !m1 || !m2) return fail(LPM_EINVAL, "NULL argument");
    if (s->dtype == LPM_BF16 && !lowp) return fail(LPM_EINVAL, "lowp is NULL for a bf16 stage");
    if (step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
        return fail(LPM_EINVAL, "Adam needs step >= 1, 0 <= beta < 1 and eps >= 0");
    if (misaligned(params) || misaligned(grads) || misaligned(m1) || misaligned(m2) || (lowp && misaligned(lowp)))
        return fail(LPM_EALIGN, "device buffers must be 256-byte aligned");
    if (s->n_trainable == 0) return LPM_OK;
    // bias corrections in double on the host: 1 - beta^t loses digits in float for beta close to 1
    const float inv_c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
    const float inv_c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
    hipStream_t st = (hipStream_t)stream;
    LPM_HIP(launch_adam(params, s->dtype == LPM_BF16 ? (uint16_t*)lowp : nullptr, grads, m1, m2, s->n_trainable, lr_, beta1, beta2,
                        eps, inv_c1, inv_c2, zero_grads, st));
    if (s->dtype == LPM_BF16) LPM_HIP(transpose_copies(s, params, lowp, st));
    return LPM_OK;
}

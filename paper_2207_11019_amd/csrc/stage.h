// Host-side layout of a stage (shared by the stage and schedule sources).
#pragma once
#include "lpm_internal.h"

namespace lpm {

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static const size_t NO = (size_t)-1;

enum Loc { LOC_X = 0, LOC_Y = 1, LOC_STASH = 2 };

struct TensorRt {
    Shape shape{};
    size_t bytes = 0;
    int loc = LOC_STASH;
    size_t stash_off = NO;   // byte offset in a stash slot
    size_t g_off = NO;       // byte offset of its gradient in the backward scratch
};

struct LayerRt {
    lpm_layer d{};
    ConvGeom g{};
    size_t w_off = NO, b_off = NO, s_off = NO;   // float offsets into params
    size_t w_count = 0;
    size_t lowp_w_off = NO, lowp_wt_off = NO;    // byte offsets into lowp
    size_t dz_off = NO;                          // byte offset of its pre-activation gradient in the backward scratch
    size_t wws_off = 0;                          // this layer's weight-gradient partials inside the backward scratch
    size_t fcs_x_off = NO, fcs_dz_off = NO;      // staging areas of a layer whose weight gradient a schedule contracts
                                                 // once per mini-batch (byte offsets in the backward scratch)
    int32_t unpool_of = -1;                      // conv/FC: index of the max-pooling layer whose backward its data gradient performs
    bool fused_side = false;                     // fused_in, and the consumer's data gradient also adds the earlier contributions to this
                                                 // layer's output gradient and writes the gradient of this layer's shortcut (DgradSide)
    bool via_shortcut = false;                   // fused_in: a scale-only layer read as a shortcut by one fused_side layer; the kernel that
                                                 // writes that layer's shortcut gradient writes this layer's dz instead
    int32_t pool_fwd = -1;                       // conv/FC: index of the max-pooling layer whose forward its own forward kernel performs
    bool pooled_fwd = false;                     // max-pooling: its forward runs inside its producer's forward kernel
    bool unpooled = false;                       // max-pooling: its backward runs inside its consumer's data gradient
    bool fused_in = false;                       // its consumer's backward kernel writes dz directly (mask and scale fused)
    bool dz_unscaled = false;                    // its dz buffer holds the gradient BEFORE the layer's per-channel scale: the weight-gradient
                                                 // kernel multiplies row co of dW by scale[co] and sums dz for the bias gradient as it is, the
                                                 // data gradient reads transposed weights that carry the scale (or scales dz as it loads it)
};

}  // namespace lpm

struct lpm_stage {
    // (fields use the lpm:: types declared above)
    int32_t first = 0, last = 0, m = 0, dtype = 0, L = 0;
    bool loss = false;
    size_t esz = 4;
    std::vector<lpm_layer> net;
    std::vector<lpm::Shape> shapes;
    std::vector<lpm::LayerRt> lay;         // indexed by network layer index - first
    std::vector<lpm::TensorRt> ten;        // indexed by tensor index - (first-1)
    int32_t t_out = 0;                // tensor written to y
    size_t n_trainable = 0, n_params = 0;   // floats
    size_t lowp_bytes = 0, stash_bytes = 0, fwd_ws = 0, bwd_ws = 0;
    size_t dlogits_off = lpm::NO, kws_off = lpm::NO, wws_off = lpm::NO;   // stash / bwd-scratch offsets
    size_t gws_bytes = 0;             // size of one copy of the gradient / dz area at the head of the backward scratch
    // Weight gradients are off the critical path of B (nothing in the same pass reads them), so they run on
    // a side stream (borrowed from the library's pool), forked from and joined back into the caller's stream.
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    hipEvent_t ev_w2_fork = nullptr, ev_w2_join = nullptr;      // a weight phase spread over two streams (lpm_stage_backward_on)
    // per weight layer and micro-batch slot: "this layer's output gradient is final" in the data phase's stream
    // order, for schedules that let the weight phase follow the data phase layer by layer
    std::vector<hipEvent_t> ev_layer;      // [(layer - first) * LPM_MAX_WINDOW + slot]
    ~lpm_stage();

    lpm::TensorRt& T(int32_t t) { return ten[(size_t)(t - (first - 1))]; }
    const lpm::TensorRt& T(int32_t t) const { return ten[(size_t)(t - (first - 1))]; }
    lpm::LayerRt& Ly(int32_t i) { return lay[(size_t)(i - first)]; }
    const lpm::LayerRt& Ly(int32_t i) const { return lay[(size_t)(i - first)]; }
};

// B_{z,j} with the weight phase on a stream of the caller's choice (see stage.cpp).
int32_t lpm_stage_backward_on(lpm_stage* s, const void* x, const void* y, const void* dy, void* dx,
                              const float* params, const void* lowp, const void* stash, float* grads,
                              int32_t accumulate, void* bwd_ws, void* stream, void* wstream, int32_t parity,
                              int32_t phases, int32_t fc_slot = -1, int32_t fc_flush = 0, int32_t layer_slot = -1,
                              int32_t boundary = 0, void* wstream2 = nullptr);
// boundary: a schedule may move the ReLU backward of a stage's last layer into the next stage, whose kernel that
// writes the gradient w.r.t. its input then masks it with that input (the producer's output) -- one kernel less
// per cut and micro-batch.  LPM_MASK_DX: this stage masks its dx; LPM_DY_IS_DZ: the gradient this stage receives
// already is the pre-activation gradient of its last layer.  Both sides must agree (see the two predicates).
enum { LPM_MASK_DX = 1, LPM_DY_IS_DZ = 2 };
bool lpm_stage_can_mask_dx(const lpm_stage* s);        // its input tensor has exactly one consumer, a layer whose backward kernel can mask
bool lpm_stage_takes_dz(const lpm_stage* s);           // its last layer is conv/FC + ReLU (no scale, no shortcut), bias gradient from the weight-gradient kernel
enum { LPM_PHASE_DATA = 1, LPM_PHASE_WEIGHTS = 2 };

// U_z reading one weight version and writing another (see stage.cpp).
int32_t lpm_stage_update_to(lpm_stage* s, const float* params_in, float* params_out, void* lowp_out, float* grads,
                            float* momentum, float lr, float mu, int32_t zero_grads, void* stream);

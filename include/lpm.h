/*
 * lpm -- layer-wise partition-and-merge training step for one AMD MI355X (gfx950).
 *
 * C ABI of the library.  The calls follow the method's problem statement:
 *   - a network is a list of L consecutive layers            (Problem Statement, eq. 1)
 *   - the list is cut into Z sub-modules ("partitions", "stages") of consecutive
 *     layers                                                  (Layer-wise Partitioning and Merging)
 *   - a cost T(F_{i,j}), T(B_{i,j}) is attached to every forward / backward
 *     operation of stage i on micro-batch j                   (Cost Model, eq. 10)
 *   - a mini-batch of b samples is split into micro-batches; F_{i,j} and B_{i,j}
 *     of different micro-batches overlap; gradients are accumulated and every
 *     stage is updated once per mini-batch                    (Forward Pass and Backward Pass
 *                                                              Parallelisation and Optimisation)
 *   - the update is p <- p - alpha * omega                    (Problem Statement, eq. 6),
 *     here with an optional momentum term.
 *
 * General rules
 *   * Every function returns an int32 status: LPM_OK (0) or a negative LPM_E* code.
 *     No exception crosses the ABI.  lpm_last_error() returns a thread-local text
 *     for the last failing call.
 *   * Pointers named "host" are host memory; all others are DEVICE memory owned by
 *     the caller (allocated by any means; this library never allocates or frees
 *     device memory) and must be 256-byte aligned unless stated otherwise.
 *   * Streams are caller-owned hipStream_t handles passed as void* (NULL = the
 *     default stream).  Stage calls only enqueue work and return; they never
 *     synchronise the device.  Arguments are validated before anything is
 *     enqueued, so a failing call has no device side effects.
 *   * Device layouts: activations [m][H][W][C] (channels innermost), convolution
 *     weights [Cout][Kh][Kw][Cin]; a fully connected layer is a convolution whose
 *     kernel covers its whole input, so its weights are [Cout][H][W][Cin] too.
 *     Element type of activations and activation gradients: float (LPM_F32) or
 *     bfloat16 (LPM_BF16).  Master weights, momentum, weight gradients, bias and
 *     scale: always float.  Labels: int32.
 *   * Handles (lpm_stage, lpm_schedule) are host objects created and destroyed in
 *     pairs.  A handle may be used from one host thread at a time.
 */
#ifndef LPM_H
#define LPM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ---- */
#define LPM_OK        0
#define LPM_EINVAL   (-1)   /* bad argument value / NULL where a pointer is required          */
#define LPM_ESHAPE   (-2)   /* layer descriptors inconsistent with each other                  */
#define LPM_EALIGN   (-3)   /* device pointer not 256-byte aligned                             */
#define LPM_ENOMEM   (-4)   /* host allocation failed                                          */
#define LPM_EHIP     (-5)   /* a HIP runtime call failed; see lpm_last_error()                 */
#define LPM_ENOPLAN  (-6)   /* no plan with the requested number of stages exists              */

/* ---- layer kinds ---- */
#define LPM_CONV        0   /* 2-D cross-correlation, zero padding, then the epilogue below    */
#define LPM_FC          1   /* fully connected on the flattened input (= conv, kernel = input) */
#define LPM_MAXPOOL2    2   /* 2x2 window, stride 2 (H, W even); gradient to the first maximum */
#define LPM_GAP         3   /* global average pool over H x W                                  */
#define LPM_SOFTMAX_CE  4   /* softmax cross-entropy on the logits; must be the last layer     */
#define LPM_ATTN        5   /* one-head self-attention over the positions of a sample (the "self-attention layer" of
                               the volumetric use case): the input's 3*cout channels are queries | keys | values,
                               y_i = sum_j softmax_j(q_i.k_j / sqrt(cout)) v_j; no parameters                  */

/* ---- layer flags (CONV / FC): y = relu( scale_c * z + bias_c + T[add_src] ) ---- */
#define LPM_RELU   1
#define LPM_BIAS   2        /* trainable per-channel bias                                       */
#define LPM_SCALE  4        /* frozen per-channel multiplier (a folded normalisation layer)     */

#define LPM_NONE  (-2)      /* value of add_src when there is no shortcut                       */

/* ---- element types ---- */
#define LPM_F32   0
#define LPM_BF16  1

/* ---- schedule modes ---- */
#define LPM_LOCKED      0   /* F_{0,j}..F_{Z-1,j}, B_{Z-1,j}..B_{0,j} for j=0..M-1 on one stream, then U_z */
#define LPM_OVERLAPPED  1   /* forward chain of micro-batch j+1 runs beside the backward chain of j        */
#define LPM_PIPELINED   2   /* as OVERLAPPED, and every stage runs on its own pair of streams (owned by the
                               schedule): stages work on different micro-batches at the same time         */
#define LPM_ASYNC_UPDATE 32  /* OR-ed into LOCKED or OVERLAPPED: one update per micro-batch (see lpm_schedule_run) */
#define LPM_GRAPH       16  /* OR-ed into mode: replay the step as a captured HIP graph                    */

/* One layer a^{l+1} = g_l(a^l, p^l).  Tensor index t means "output of layer t"; t = -1 is the
 * network input.  All fields are in the logical (layout-free) sense. */
typedef struct lpm_layer {
    int32_t kind;               /* LPM_CONV ...                                                     */
    int32_t cin, cout;          /* channels in / out (pool, gap, loss: cout = cin)                  */
    int32_t kh, kw, stride, pad;/* CONV only; FC uses kh=h_in, kw=w_in, stride 1, pad 0 implicitly  */
    int32_t h_in, w_in;         /* spatial extent of the input tensor                               */
    int32_t flags;              /* LPM_RELU | LPM_BIAS | LPM_SCALE                                  */
    int32_t src;                /* tensor read as input (normally l-1)                              */
    int32_t add_src;            /* tensor added before the ReLU, or LPM_NONE                        */
    int32_t cut_allowed_after;  /* non-zero: a partition boundary may follow this layer             */
    /* Volumetric (3-D) convolutions, the 3x3x3 layers of the method's first use case.  A tensor [C][D][H][W] is handled
     * as [C][D*H][W] by every other layer kind (depth folded into the height); a CONV / FC layer with d_in > 1 unfolds
     * it: its input tensor must have height d_in * h_in, its kernel is kd x kh x kw (weights [Cout][Kd][Kh][Kw][Cin]),
     * the one stride applies to all three axes, pad_d pads the depth.  0 in d_in / kd means 1 (a 2-D layer). */
    int32_t d_in, kd, pad_d;
} lpm_layer;

/* Machine and workload parameters of the cost model (all integers: plans are reproducible). */
typedef struct lpm_cost_params {
    uint64_t flop_per_us;       /* matrix throughput                                                */
    uint64_t hbm_byte_per_us;   /* memory bandwidth                                                 */
    uint64_t link_byte_per_us;  /* device-to-device link; 0 = ignore transfers                      */
    int32_t  elem_bytes;        /* 4 (LPM_F32) or 2 (LPM_BF16)                                      */
    int32_t  microbatch;        /* m: samples per micro-batch                                       */
    int32_t  n_microbatch;      /* M: micro-batches per mini-batch                                  */
} lpm_cost_params;

typedef struct lpm_stage lpm_stage;
typedef struct lpm_schedule lpm_schedule;

/* Text describing the last error raised on the calling thread (host memory owned by the library,
 * valid until the next failing call on this thread).  Never NULL. */
const char* lpm_last_error(void);

/* Cost of layer i (Cost Model, eq. 10: the T(F_{i,j}) + T(B_{i,j}) of one micro-batch plus 1/M of the
 * update), in integer picoseconds:
 *   max( flop*1e6 / flop_per_us , (M*bytes_fwd_bwd + bytes_update)*1e6 / (M*hbm_byte_per_us) )
 * flop = 2*MAC*m*(3, or 2 when the layer reads the network input); bytes = ideal tensor traffic.
 * layers: host, L entries.  out_cost: host, one value.  Errors: LPM_EINVAL, LPM_ESHAPE. */
int32_t lpm_layer_cost(const lpm_layer* layers, int32_t L, int32_t i, const lpm_cost_params* cp,
                       uint64_t* out_cost);

/* Partition-and-merge plan (Layer-wise Partitioning and Merging; Cost Model): cut the L layers into Z
 * non-empty stages of consecutive layers, cutting only after layers with cut_allowed_after != 0,
 * minimising lexicographically (largest stage cost, total bytes crossing the cuts, starts).
 * A stage's cost is the sum of its layers' costs plus, when link_byte_per_us > 0, the transfer time of
 * the activation and gradient at each of its boundaries.
 *   layers        host, L entries, validated as a whole network
 *   fixed_starts  host, NULL or Z+1 entries: only validate and cost this plan
 *   out_starts    host, Z+1 entries: out_starts[0]=0 .. out_starts[Z]=L
 *   out_stage_cost host, Z entries (may be NULL)
 * Pure host code, deterministic, integer arithmetic only.
 * Errors: LPM_EINVAL, LPM_ESHAPE, LPM_ENOPLAN (fewer than Z-1 allowed cuts, or fixed_starts illegal). */
int32_t lpm_partition(const lpm_layer* layers, int32_t L, int32_t Z, const lpm_cost_params* cp,
                      const int32_t* fixed_starts, int32_t* out_starts, uint64_t* out_stage_cost);

/* The same plan from per-layer costs the caller supplies -- the cost model (eq. 10) asks for the times
 * T(F_ij), T(B_ij) of the operations; here they can be measured ones.  layer_cost_ps: host array of L
 * costs in picoseconds (forward + backward of one micro-batch, plus the layer's share of the update),
 * used in place of the analytic per-layer cost; cp still supplies the micro-batch size, element size and
 * link rate for the boundary terms.  Everything else as lpm_partition.  Errors: as lpm_partition. */
int32_t lpm_partition_costs(const lpm_layer* layers, int32_t L, int32_t Z, const lpm_cost_params* cp,
                            const uint64_t* layer_cost_ps, const int32_t* fixed_starts, int32_t* out_starts,
                            uint64_t* out_stage_cost);

/* Create the stage that owns layers [first, last) of the network for micro-batches of `microbatch`
 * samples (a sub-module z of Layer-wise Partitioning and Merging).
 *   layers  host, the WHOLE network (L entries); copied.
 *   dtype   LPM_F32 or LPM_BF16
 * Every tensor the stage reads from outside must be tensor first-1.  A stage whose last layer is
 * LPM_SOFTMAX_CE is a loss stage: its output buffer receives the logits.
 * Errors: LPM_EINVAL, LPM_ESHAPE, LPM_ENOMEM. */
int32_t lpm_stage_create(const lpm_layer* layers, int32_t L, int32_t first, int32_t last,
                         int32_t microbatch, int32_t dtype, lpm_stage** out);
int32_t lpm_stage_destroy(lpm_stage* s);

/* Buffer sizes in bytes (all host out-pointers, any may be NULL).
 *   param_bytes     float master parameters: trainable tensors first (W, bias per layer, each starting
 *                   on a 256-byte boundary), then the frozen scales
 *   lowp_bytes      bf16 copies of the weights used by the contractions (0 for LPM_F32)
 *   grad_bytes      float gradient accumulator = momentum size = trainable part of params
 *   stash_bytes     one stash slot: what F keeps for B of the same micro-batch
 *   fwd_ws_bytes    scratch used by lpm_stage_forward   (F and B of one stage may run concurrently,
 *   bwd_ws_bytes    scratch used by lpm_stage_backward   so the two scratch areas are distinct)
 *   in_bytes, out_bytes  stage input / output activation for one micro-batch */
int32_t lpm_stage_sizes(const lpm_stage* s, size_t* param_bytes, size_t* lowp_bytes, size_t* grad_bytes,
                        size_t* stash_bytes, size_t* fwd_ws_bytes, size_t* bwd_ws_bytes,
                        size_t* in_bytes, size_t* out_bytes);

/* Element offset (in floats, from the start of params / grads / momentum) and element count of one
 * parameter tensor.  layer is the network-wide index; which: 0 = W, 1 = bias, 2 = scale.
 * Errors: LPM_EINVAL when the layer has no such tensor. */
int32_t lpm_stage_param_offset(const lpm_stage* s, int32_t layer, int32_t which, size_t* offset, size_t* count);

/* Byte offset inside a stash slot of tensor t (first <= t < last-1; stage input and output live in the
 * caller's x / y buffers), or of the loss gradient when t == -100.  Errors: LPM_EINVAL. */
int32_t lpm_stage_stash_offset(const lpm_stage* s, int32_t t, size_t* offset, size_t* bytes);

/* Byte offset inside the backward scratch of the gradient w.r.t. internal tensor t (first <= t < last-1),
 * valid after lpm_stage_backward has run.  For tests.  The gradient of a max-pooling output that feeds a single
 * convolution may not be stored at all (that layer's data-gradient kernel routes it to the pooling input
 * directly); the offset then names memory the pass leaves untouched.  Likewise for LPM_BF16 the output of a
 * conv/FC layer with ReLU or scale whose epilogue backward runs inside its reader's data-gradient kernel: the
 * area then holds only the contributions that arrived before that kernel's own (those of the layers that use the
 * tensor as a shortcut), or nothing.  Gradients of pooling inputs and of tensors with several readers are
 * complete.  Errors: LPM_EINVAL. */
int32_t lpm_stage_grad_offset(const lpm_stage* s, int32_t t, size_t* offset, size_t* bytes);

/* (Re)build the low-precision weight copies from the float master parameters (LPM_BF16 stages; a
 * no-op for LPM_F32).  Call once after filling params; lpm_stage_update keeps them current. */
int32_t lpm_stage_sync_lowp(lpm_stage* s, const float* params, void* lowp, void* stream);

/* F_{z,j}: forward pass of the stage on one micro-batch (eq. 1 applied layer by layer).
 *   x        stage input  [m][H][W][C]            (read)
 *   y        stage output [m][Ho][Wo][Co], or the logits [m][classes] for a loss stage   (written)
 *   labels   loss stage only: int32 [m], every value in [0, classes); 4-byte aligned is enough.  A value outside
 *            that range reads nothing out of bounds: the row gets no one-hot term and the loss becomes NaN
 *   loss_accum loss stage only: one float, += loss_scale * sum_n -log softmax(logits_n)[label_n]
 *   params, lowp   as sized by lpm_stage_sizes (lowp may be NULL for LPM_F32)
 *   stash    one stash slot (written)
 *   fwd_ws   forward scratch
 *   loss_scale  1/b with b the size of the whole mini-batch; also scales the loss gradient
 * Errors: LPM_EINVAL, LPM_EALIGN, LPM_EHIP. */
int32_t lpm_stage_forward(lpm_stage* s, const void* x, void* y, const int32_t* labels, float* loss_accum,
                          const float* params, const void* lowp, void* stash, void* fwd_ws,
                          float loss_scale, void* stream);

/* B_{z,j}: backward pass of the stage on the micro-batch whose forward filled `stash` (eqs. 8, 9).
 *   x, y     the same buffers F read and wrote (read)
 *   dy       gradient w.r.t. y (read); ignored (may be NULL) for a loss stage
 *   dx       gradient w.r.t. x (written); NULL = not wanted (first stage of a network)
 *   grads    float accumulator, trainable layout of params; accumulate = 0 overwrites, 1 adds
 *            (gradient accumulation over the micro-batches of a mini-batch)
 *   bwd_ws   backward scratch
 * Errors: LPM_EINVAL, LPM_EALIGN, LPM_EHIP. */
int32_t lpm_stage_backward(lpm_stage* s, const void* x, const void* y, const void* dy, void* dx,
                           const float* params, const void* lowp, const void* stash, float* grads,
                           int32_t accumulate, void* bwd_ws, void* stream);

/* U_z: v <- mu*v + g ; p <- p - lr*v over the trainable parameters (eq. 6 when mu = 0); refreshes the
 * low-precision copies; zero_grads != 0 also clears g.  Errors: LPM_EINVAL, LPM_EALIGN, LPM_EHIP. */
int32_t lpm_stage_update(lpm_stage* s, float* params, void* lowp, float* grads, float* momentum,
                         float lr, float mu, int32_t zero_grads, void* stream);

/* U_z with Adam (Kingma and Ba), the update rule the problem statement names beside SGD (it prints only SGD's,
 * eq. 6):  m1 <- beta1*m1 + (1-beta1)*g;  m2 <- beta2*m2 + (1-beta2)*g*g;
 *          p <- p - lr * (m1 / (1-beta1^step)) / (sqrt(m2 / (1-beta2^step)) + eps),   step = 1, 2, ...
 * m1, m2: two device buffers laid out like momentum (momentum_bytes each), zero before the first step.
 * Refreshes the low-precision copies like lpm_stage_update; the schedules keep calling that one.
 * Errors: LPM_EINVAL (also step < 1, beta outside [0, 1), eps < 0), LPM_EALIGN, LPM_EHIP. */
int32_t lpm_stage_update_adam(lpm_stage* s, float* params, void* lowp, float* grads, float* m1, float* m2,
                              float lr, float beta1, float beta2, float eps, int32_t step, int32_t zero_grads,
                              void* stream);

/* Device buffers of one stage as used by a schedule. */
#define LPM_MAX_WINDOW 4
typedef struct lpm_stage_buffers {
    float* params;  void* lowp;  float* grads;  float* momentum;
    void*  stash[LPM_MAX_WINDOW];   /* one slot per in-flight micro-batch                            */
    void*  act_out[LPM_MAX_WINDOW]; /* stage output ring (logits for the loss stage), out_bytes each */
    void*  grad_in[LPM_MAX_WINDOW]; /* gradient w.r.t. the stage input, in_bytes each; may be NULL for stage 0 */
    void*  fwd_ws;  void* bwd_ws;
    float* params_alt;  void* lowp_alt;   /* second weight version (same sizes as params / lowp) for
                                             LPM_ASYNC_UPDATE, frozen scales filled in like params; else NULL */
} lpm_stage_buffers;

/* A schedule over Z stages that form one network, M micro-batches per mini-batch, at most `window`
 * micro-batches in flight per stage (1 <= window <= LPM_MAX_WINDOW; the method's figure uses 2:
 * B_{0,0} finishes before F_{0,2}).  stages: host array of Z handles, which must outlive the schedule.
 * Errors: LPM_EINVAL, LPM_ESHAPE, LPM_ENOMEM, LPM_EHIP. */
int32_t lpm_schedule_create(lpm_stage* const* stages, int32_t Z, int32_t n_microbatch, int32_t window,
                            lpm_schedule** out);
int32_t lpm_schedule_destroy(lpm_schedule* s);

/* What per_stage[z].grad_in holds after a run (F/B parallelisation section: the gradient a sub-module hands to
 * its neighbour).  0: the gradient w.r.t. the input of stage z (eq. 9).  1: that gradient with the ReLU
 * derivative of the previous stage's last layer already applied (zero where the stage input is <= 0), i.e. the
 * pre-activation gradient of that layer: when stage z-1 ends in conv/FC + ReLU without scale or shortcut and
 * stage z's input has a single consumer, the schedule lets stage z's backward kernel apply the mask instead of
 * running a separate kernel in stage z-1.  Always 0 for z = 0 and for the float path.  Negative: LPM_EINVAL. */
int32_t lpm_schedule_cut_fused(const lpm_schedule* s, int32_t z);

/* One mini-batch step: all F_{z,j}, B_{z,j}, then U_z for every stage (one update per mini-batch with
 * the accumulated gradient).
 *   mode       LPM_LOCKED or LPM_OVERLAPPED, optionally | LPM_GRAPH; or LPM_PIPELINED (LPM_PIPELINED | LPM_GRAPH
 *              is refused with LPM_EINVAL)
 *   x_batch    [M*m][H][W][C] network input (micro-batch j is the j-th contiguous block of m samples)
 *   labels     int32 [M*m] when the last stage is a loss stage, else NULL
 *   dy_batch   upstream gradient [M*m][..] of the last stage's output when it is not a loss stage
 *   per_stage  host array of Z buffer sets
 *   dx_wanted  non-zero: stage 0 also produces the gradient w.r.t. x (micro-batch j into
 *              per_stage[0].grad_in[j % window]; for partitions fed by an upstream activation)
 *   loss_out   device float; set to the mini-batch mean loss (loss stage only; may be NULL otherwise)
 *   stream_fwd, stream_bwd  two distinct streams for LPM_OVERLAPPED (forward chains and the data phases of the
 *              backward chains; the weight phases run on streams of the library, forked from and joined back
 *              into these.  The first such run on a pair of streams launches a few short probe kernels on them
 *              and synchronises them, to find library streams that do not share a hardware queue with them);
 *              LPM_LOCKED and LPM_PIPELINED use stream_fwd only (PIPELINED forks its own streams from it and
 *              joins them back).
 * Micro-batch j uses slot j % window of stash, act_out and grad_in in every mode.
 * mode | LPM_ASYNC_UPDATE (with LPM_LOCKED or LPM_OVERLAPPED, window <= 2, not with LPM_GRAPH): the
 *   asynchronous parameter update.  Every micro-batch is a mini-batch of its own (loss = mean over its m
 *   samples) and U_{z,j} follows B_{z,j}; version 0 of a stage's weights is the state at the start of the call
 *   and U_{z,j} turns version j into version j+1.  B_{z,j} reads version j.  F_{z,j} reads version j when
 *   nothing overlaps (LPM_LOCKED, or window 1) and version max(0, j-1) with window 2, where it runs beside
 *   B_{z,j-1}: one update behind.  Even versions live in params / lowp, odd ones in params_alt / lowp_alt;
 *   on return the final version (n_microbatch) is in params / lowp (copied there if n_microbatch is odd),
 *   grads holds the gradient of the last micro-batch and loss_out the sum of the micro-batches' mean losses.
 * On return all work is enqueued and stream_fwd is ordered after everything the call enqueued.
 * Results are bitwise identical between the modes (fixed accumulation order, no float atomics).
 * Errors: LPM_EINVAL, LPM_EALIGN, LPM_EHIP. */
int32_t lpm_schedule_run(lpm_schedule* s, int32_t mode, const void* x_batch, const int32_t* labels,
                         const void* dy_batch, const lpm_stage_buffers* per_stage, int32_t dx_wanted,
                         float lr, float mu, float* loss_out, void* stream_fwd, void* stream_bwd);

/* ---- single-layer contractions (the kernels inside F and B), for tests and measurement ---------- */

/* Geometry of one convolution on a micro-batch of m samples: input [m][h][w][cin], weights
 * [cout][kh][kw][cin], output [m][ho][wo][cout] with ho = (h + 2*pad - kh)/stride + 1 (same for wo).
 * A fully connected layer is kh = h, kw = w, stride 1, pad 0. */
typedef struct lpm_conv_geom {
    int32_t m, h, w, cin, cout, kh, kw, stride, pad;
    int32_t d, kd, pad_d;      /* volumetric form: input [m][d][h][w][cin], weights [cout][kd][kh][kw][cin]; 0 = 1 (2-D) */
} lpm_conv_geom;

/* Scratch bytes the three contractions need for this geometry (host out-pointers, any may be NULL). */
int32_t lpm_conv_ws_bytes(const lpm_conv_geom* g, int32_t dtype, size_t* fwd, size_t* dgrad, size_t* wgrad);

/* y = relu?( scale_c * (w (*) x) + bias_c + add )  -- eq. 1 for a convolution / FC layer.
 *   w: float weights for LPM_F32, bf16 weights for LPM_BF16; scale, bias, add may be NULL. */
int32_t lpm_conv_forward(const lpm_conv_geom* g, int32_t dtype, const void* x, const void* w, const float* scale,
                         const float* bias, const void* add, int32_t relu, void* y, void* ws, void* stream);

/* dx (+)= gradient w.r.t. the layer input given dz, the gradient w.r.t. its pre-activation -- eq. 9.
 *   wt: the same weights laid out [cin][kh][kw][cout] (bf16), or NULL when the caller has none. */
int32_t lpm_conv_dgrad(const lpm_conv_geom* g, int32_t dtype, const void* dz, const void* w, const void* wt, void* dx,
                       int32_t accumulate, void* ws, void* stream);

/* dw (+)= gradient w.r.t. the weights, float [cout][kh][kw][cin] -- eq. 8. */
int32_t lpm_conv_wgrad(const lpm_conv_geom* g, int32_t dtype, const void* x, const void* dz, float* dw,
                       int32_t accumulate, void* ws, void* stream);

/* lpm_conv_wgrad for callers that cannot allocate device memory and have none to lend: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels and the same bits as
 * lpm_conv_wgrad, but the split partials go to a fixed area of LPM_STATIC_SCRATCH_BYTES inside the library's device
 * image instead of a caller buffer; the call allocates and frees nothing, on the host side of the runtime or on the
 * device.  x, dz, dw as for lpm_conv_wgrad (caller-owned device memory, 256-byte aligned).
 * All calls on one GPU share that GPU's area: calls that may overlap on one GPU (two streams, two threads) race and
 * must be serialised by the caller; consecutive calls on one stream are ordered by the stream.
 * Errors: as lpm_conv_wgrad; LPM_EINVAL when the geometry needs more scratch than the area holds (lpm_conv_ws_bytes
 * tells how much), before anything is enqueued. */
#define LPM_STATIC_SCRATCH_BYTES (8u << 20)
int32_t lpm_conv_wgrad_static(const lpm_conv_geom* g, int32_t dtype, const void* x, const void* dz, float* dw,
                              int32_t accumulate, void* stream);

/* Measurement helper: enqueues one of the three contractions `iters` times back to back on `stream`
 * between two HIP events (after `warmup` untimed launches), waits for them, and returns the average
 * duration of one launch in microseconds.  op: 0 = forward (x, w -> y, ReLU epilogue), 1 = data gradient
 * (y as dz, w, wt -> x as dx), 2 = weight gradient (x, y as dz -> dw, accumulating).  Buffers as in the
 * calls above; synchronises the stream.  Errors: as the calls above, LPM_EHIP. */
int32_t lpm_conv_time(int32_t op, const lpm_conv_geom* g, int32_t dtype, void* x, const void* w, const void* wt,
                      void* y, float* dw, void* ws, int32_t warmup, int32_t iters, void* stream, float* avg_us);

/* ---- layer-wise partitioning of one layer ("Layer-wise Partitioning and Merging" section, fig. 1a) ---- */

/* The un-merged form of the method: a layer's output channels are split into n equal sub-layers (n = the paper's
 * number of devices), each sub-layer is computed by its own launch with its slice of the weights -- on the caller's
 * stream and up to three streams of the library's pool that were measured to feed other hardware queues (the
 * stand-ins for devices; further sub-layers share them in turn) -- and the outputs are concatenated for the next layer.
 * Backward, the incoming gradient is re-partitioned by channel, each sub-layer produces its slice of the weight
 * gradient and a full-size partial input gradient, and the partials are added in sub-layer order.  The results are
 * those of the merged layer (lpm_conv_*); the difference in time is the overhead that merging removes.
 * Geometry as lpm_conv_geom; cout must be divisible by n with cout / n a multiple of 8; 2 <= n <= 8.
 * The handle owns host objects only (events).  Errors: LPM_EINVAL, LPM_ESHAPE, LPM_ENOMEM, LPM_EHIP. */
typedef struct lpm_layerwise lpm_layerwise;
int32_t lpm_layerwise_create(const lpm_conv_geom* g, int32_t dtype, int32_t n, lpm_layerwise** out);
int32_t lpm_layerwise_destroy(lpm_layerwise* lw);

/* Device scratch (caller-owned, 256-byte aligned) the two calls below need: the sub-layer outputs / the
 * re-partitioned gradient and partial input gradients, plus each sub-layer's own contraction scratch. */
int32_t lpm_layerwise_ws_bytes(const lpm_layerwise* lw, size_t* forward, size_t* backward);

/* y = relu?( scale_c * (w (*) x) + bias_c ), computed as n sub-layers and one concatenation (eq. 1 per sub-layer).
 *   x [m][h][w][cin], w [cout][kh][kw][cin] (sub-layer i owns rows i*cout/n ...), y [m][ho][wo][cout]; scale, bias
 *   (float [cout]) may be NULL.  Enqueues on `stream` and on pooled streams that fork from and join back into it
 *   (the first call on a stream runs a few short probe kernels on it and synchronises it);
 *   calls on one handle must not overlap (they share its events and the scratch). */
int32_t lpm_layerwise_forward(lpm_layerwise* lw, const void* x, const void* w, const float* scale, const float* bias,
                              int32_t relu, void* y, void* ws, void* stream);

/* dw (+)= weight gradient (float [cout][kh][kw][cin], eq. 8), dx = input gradient (eq. 9; NULL: not computed) from dz,
 * the gradient w.r.t. the pre-activation [m][ho][wo][cout].
 *   wt: for LPM_BF16, the n sub-layers' weights transposed one after the other, each [cin][kh][kw][cout/n] (what
 *   each device would keep beside its slice of w), or NULL (slower kernels). */
int32_t lpm_layerwise_backward(lpm_layerwise* lw, const void* x, const void* dz, const void* w, const void* wt, void* dx,
                               float* dw, int32_t accumulate, void* ws, void* stream);

/* Measurement helper, as lpm_conv_time: op 0 = lpm_layerwise_forward (ReLU epilogue), op 1 = lpm_layerwise_backward
 * (y as dz, accumulating into dw; dx may be NULL).  Returns the average microseconds of one call; synchronises. */
int32_t lpm_layerwise_time(lpm_layerwise* lw, int32_t op, const void* x, const void* w, const void* wt, void* y, void* dx,
                           float* dw, void* ws, int32_t warmup, int32_t iters, void* stream, float* avg_us);

#ifdef __cplusplus
}
#endif
#endif /* LPM_H */

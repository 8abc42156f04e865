// Internal declarations shared by the host-side sources and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <vector>
#include "../../include/lpm.h"

namespace lpm {

// ---- error text (thread local) -------------------------------------------------------------------
int32_t fail(int32_t code, const char* fmt, ...);
int32_t hip_fail(hipError_t e, const char* what);
#define LPM_HIP(call)                                            \
    do {                                                         \
        hipError_t e__ = (call);                                 \
        if (e__ != hipSuccess) return lpm::hip_fail(e__, #call); \
    } while (0)

// ---- pooled worker streams (per device, created on first use, alive until the process ends) --------
constexpr int LPM_POOL_SCHEDULE_STREAMS = 8;    // indices 0..7: forward / backward stream of stage z at 2z, 2z+1 (mod 8)
constexpr int LPM_POOL_STREAMS = 12;            // indices 8..11: weight-gradient side streams, handed out round-robin
hipError_t pooled_stream(int index, hipStream_t* out);
int next_side_stream_index();
// The runtime spreads a process's streams over a few hardware queues (four by default), and a hardware queue runs
// its kernels strictly one after the other -- two streams on one queue never overlap, and a wait at the head of one
// holds up the other.  Which queue a stream gets is not exposed, so it is measured: a short spin kernel on each of the
// two streams, started together; *shared = they ran back to back.  Synchronises both streams.
hipError_t streams_share_queue(hipStream_t a, hipStream_t b, bool* shared);
// Up to `want` pooled streams that share a hardware queue neither with one of taken[0..n_taken) nor with each other.
hipError_t pick_concurrent_streams(const hipStream_t* taken, int n_taken, hipStream_t* out, int want, int* found);
hipError_t launch_spin(long long ticks, hipStream_t st);

// ---- validated network description ---------------------------------------------------------------
struct Shape { int32_t c, h, w; size_t elems() const { return (size_t)c * h * w; } };      // (a volume's depth is folded into h)

// Checks the whole list (kinds, extents, references, shapes) and returns per-tensor shapes:
// shapes[0] is tensor -1 (the network input), shapes[t+1] the output of layer t.
// FC layers are rewritten to their convolution form (kh=h_in, kw=w_in, stride 1, pad 0).
int32_t validate_network(const lpm_layer* layers, int32_t L, std::vector<lpm_layer>& norm,
                         std::vector<Shape>& shapes);

inline bool has_weights(const lpm_layer& l) { return l.kind == LPM_CONV || l.kind == LPM_FC; }
inline int32_t taps_of(const lpm_layer& l) { return (l.kd > 0 ? l.kd : 1) * l.kh * l.kw; }      // after validate_network: kd >= 1

// ---- geometry handed to the kernel launchers -----------------------------------------------------
// Volumetric layers: D input slices of H x W, kernel Kd x Kh x Kw, Do output slices (2-D layers: D = Do = Kd = 1,
// pad_d = 0).  Only the kernels that say so handle is3d() geometries; the others are not offered them.
struct ConvGeom {
    int32_t m, H, W, Cin, Ho, Wo, Cout, Kh, Kw, stride, pad;
    int32_t D = 1, Do = 1, Kd = 1, pad_d = 0;
    __host__ __device__ int64_t rows_out() const { return (int64_t)m * Do * Ho * Wo; }
    __host__ __device__ int64_t rows_in() const { return (int64_t)m * D * H * W; }
    __host__ __device__ int32_t K() const { return Kd * Kh * Kw * Cin; }
    __host__ __device__ int32_t taps() const { return Kd * Kh * Kw; }
    __host__ __device__ bool is3d() const { return D > 1 || Kd > 1; }
};

// All launchers enqueue on `st` and return the launch status.  `dtype` selects the element type of
// activations / activation gradients / low-precision weights (LPM_F32: float everywhere).

// y = relu?( scale_c * conv(x, w) + bias_c + add )      (scale, bias, add may be NULL)
// pool_y (may be NULL; only when fwd_can_pool and add == NULL): also stores the 2x2 max-pooling of y, [m][Ho/2][Wo/2][Cout]
hipError_t launch_conv_fwd(int dtype, const ConvGeom& g, const void* x, const void* w, const float* scale,
                           const float* bias, const void* add, int relu, void* y, void* ws, hipStream_t st,
                           void* pool_y = nullptr);
bool fwd_can_pool(int dtype, const ConvGeom& g);
// dx (+)= conv_transpose(dz, w);  then, when given, dx = dx * [mask > 0] * mscale_c -- the epilogue backward of
// the layer that produced the tensor dx belongs to (mask = that tensor, mscale = that layer's scale)
// unpool (may be NULL; only when dgrad_can_unpool): dx is the gradient of a 2x2 max-pooling output that nothing else
// reads -- it is not stored; the kernel routes each element straight to the first maximum of its pooling window
// (found in pool_x, the pooling input [m][2H][2W][Cin]) and writes the four window positions of dst (same shape):
// dst (+)= route(dx) * [max > 0 if mask] * mscale_c.  dx, accumulate, mask, mscale of the plain form are then unused.
struct UnpoolDesc { const void* pool_x; void* dst; int accumulate; int mask; const float* mscale; };
// side (may be NULL; only when dgrad_has_side): this data gradient is the last contribution to the gradient of a tensor
// y = relu(scale*z + bias + shortcut) and performs that layer's epilogue backward on the way:
//   v = conv_transpose(dz, w) + earlier (the contributions already there, may be NULL);  m = v * [mask > 0];
//   dx = m * mscale_c (the producer's dz);   shortcut (+)= m * shortcut_scale_c (the gradient of the producer's shortcut
//   tensor, may be NULL; with a scale: the dz of the scale-only layer -- a projection -- that made the shortcut)
struct DgradSide { const void* earlier; void* shortcut; int shortcut_acc; const float* shortcut_scale; };
// dzscale (may be NULL): dz is the gradient before the layer's own per-channel scale.  The kernels that read w multiply
// channel co of dz by dzscale[co]; wt, when given, must then already carry the factor (wt[ci][kh][kw][co] = w[co][kh][kw][ci] * dzscale[co]).
hipError_t launch_conv_dgrad(int dtype, const ConvGeom& g, const void* dz, const void* w, const void* wt,
                             void* dx, int accumulate, const void* mask, const float* mscale, void* ws, hipStream_t st,
                             const UnpoolDesc* unpool = nullptr, const DgradSide* side = nullptr, const float* dzscale = nullptr);
bool dgrad_has_side(int dtype, const ConvGeom& g);
bool dgrad_can_unpool(int dtype, const ConvGeom& g);
// dw (+)= sum over pixels of dz (x) x         ws: split-reduction partials (wgrad_ws_bytes)
// dbias (may be NULL, only when wgrad_fuses_bias): dbias (+)= sum over pixels of dz
// rscale (may be NULL): dz is the gradient before the layer's per-channel scale; row co of dw is multiplied by rscale[co]
// deferred (may be NULL): when the kernel leaves split partials, describe their reduction there instead of launching
// it (deferred->splits stays 0 when nothing is left to do); the caller runs launch_reduce_batch later on the stream.
struct ReduceDesc {
    const float* part; size_t stride; int splits;      // partial s of output i at part[s*stride + i]
    float* dst; int64_t n;                              // dst[i] (+)= sum_s part, i < n
    float* db; int nb;                                  // db[c] (+)= sum_s part[s*stride + n + c], c < nb
    const float* rscale; int row_len;                   // (may be NULL) the sum of output i is multiplied by rscale[i / row_len]
    int accumulate;
};
hipError_t launch_conv_wgrad(int dtype, const ConvGeom& g, const void* x, const void* dz, float* dw, float* dbias,
                             const float* rscale, int accumulate, void* ws, hipStream_t st, ReduceDesc* deferred = nullptr);
constexpr int LPM_REDUCE_BATCH = 24;
// the reductions of up to LPM_REDUCE_BATCH weight gradients in one launch (each in its fixed split order)
hipError_t launch_reduce_batch(const ReduceDesc* d, int count, hipStream_t st);
// Layers whose fp32 gradient matrix is much larger than their activations (fully connected layers at a few samples
// per micro-batch, 512-channel convolutions over 2x2 or 4x4 images): accumulating dW micro-batch by micro-batch
// reads and writes the whole matrix M times.  A schedule may instead file the layer's input and output gradient of
// every micro-batch under slot j and contract over the whole mini-batch once, at the last one.
constexpr int LPM_FC_STAGE_SLOTS = 32;
bool wgrad_staged_ok(int dtype, const ConvGeom& g);
size_t wgrad_staged_ws_bytes(int dtype, const ConvGeom& g);      // split partials of the contraction, any slot count
hipError_t stage_operands(const ConvGeom& g, const void* x, const void* dz, void* xs, void* dzs, int slot, hipStream_t st);
// dw (+)= the gradient over `slots` staged micro-batches starting at xs / dzs; `deferred` as for launch_conv_wgrad
hipError_t launch_wgrad_staged(int dtype, const ConvGeom& g, const void* xs, const void* dzs, int slots, float* dw, float* dbias,
                               const float* rscale, int accumulate, void* ws, hipStream_t st, ReduceDesc* deferred);
bool wgrad_fuses_bias(int dtype, const ConvGeom& g);
bool dgrad_uses_wt(int dtype, const ConvGeom& g);
size_t wgrad_ws_bytes(int dtype, const ConvGeom& g);
size_t fwd_ws_bytes(int dtype, const ConvGeom& g);
size_t dgrad_ws_bytes(int dtype, const ConvGeom& g);

// gm = dy * [y>0] (y NULL: gm = dy);  dz = gm * scale_c;  gadd (+)= gm;  dbias (+)= sum_rows gm
// ws: per-block bias partials (epi_bwd_ws_bytes)
hipError_t launch_epilogue_bwd(int dtype, int64_t rows, int32_t C, const void* dy, const void* y,
                               const float* scale, void* dz, void* gadd, int gadd_acc, float* dbias,
                               int db_acc, void* ws, hipStream_t st);
size_t epi_bwd_ws_bytes(int64_t rows, int32_t C);

hipError_t launch_maxpool_fwd(int dtype, int32_t m, int32_t H, int32_t W, int32_t C, const void* x, void* y,
                              hipStream_t st);
// dx (+)= dy routed to the first maximum of each window (recomputed from x and y)
hipError_t launch_maxpool_bwd(int dtype, int32_t m, int32_t H, int32_t W, int32_t C, const void* x,
                              const void* y, const void* dy, void* dx, int accumulate, int mask, const float* mscale,
                              hipStream_t st);
hipError_t launch_gap_fwd(int dtype, int32_t m, int32_t HW, int32_t C, const void* x, void* y, hipStream_t st);
hipError_t launch_gap_bwd(int dtype, int32_t m, int32_t HW, int32_t C, const void* dy, void* dx, int accumulate,
                          const void* mask, const float* mscale, hipStream_t st);
// dlogits = (softmax(logits) - onehot) * loss_scale;  *loss_accum += loss_scale * sum_n -log p_n[label_n]
// one-head self-attention over P positions per sample: x [m][P][3C] (queries | keys | values), y [m][P][C]
hipError_t launch_attn_fwd(int dtype, int32_t m, int32_t P, int32_t C, const void* x, void* y, hipStream_t st);
// dx (+)= gradient w.r.t. x given dy [m][P][C]; ws: attn_bwd_ws_bytes (row statistics of the recomputed softmax)
hipError_t launch_attn_bwd(int dtype, int32_t m, int32_t P, int32_t C, const void* x, const void* dy, void* dx, int accumulate,
                           void* ws, hipStream_t st);
size_t attn_bwd_ws_bytes(int32_t m, int32_t P);
bool attn_ok(int32_t P, int32_t C);
hipError_t launch_softmax_ce(int dtype, int32_t m, int32_t C, const void* logits, const int32_t* labels,
                             float loss_scale, void* dlogits, float* loss_accum, hipStream_t st);
// v = mu*v + g; p = p_in - lr*v (p_in may be p); lowp[i] = bf16(p[i]) (lowp may be NULL); optionally g = 0.   n % 4 == 0
hipError_t launch_sgd(const float* p_in, float* p, uint16_t* lowp, float* g, float* v, size_t n, float lr, float mu, int zero_g,
                      hipStream_t st);
hipError_t launch_adam(float* p, uint16_t* lowp, float* g, float* m1, float* m2, size_t n, float lr, float beta1, float beta2,
                       float eps, float inv_c1, float inv_c2, int zero_g, hipStream_t st);
hipError_t launch_f32_to_bf16(const float* src, uint16_t* dst, size_t n, hipStream_t st);
// dst[ci][kh][kw][co] = bf16(src[co][kh][kw][ci] * scale[co]) for a list of weight tensors (scale may be NULL), one launch per
// LPM_TRANSPOSE_BATCH of them
struct TransposeDesc { const float* src; uint16_t* dst; int32_t Cout, KK, Cin; const float* scale; };
constexpr int LPM_TRANSPOSE_BATCH = 24;
hipError_t launch_weight_transpose_batch(const TransposeDesc* d, int count, hipStream_t st);
hipError_t launch_fill_f32(float* p, size_t n, float v, hipStream_t st);

}  // namespace lpm

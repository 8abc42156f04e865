// Host-side network validation, layer cost model and partition-and-merge planner.
// Plain C++, integer arithmetic only: a plan is reproducible bit for bit.
//
// Layer-wise Partitioning and Merging: the layer list is cut into Z stacks of consecutive layers.
// Cost Model, eq. 10: the cost of a step is the sum of the costs of the forward and backward
// operations, so a stage's cost is the sum of its layers' costs.
#include "lpm_internal.h"

#include <cstdio>
#include <cstring>
#include <limits>
#include <string>

namespace lpm {

static thread_local std::string g_err = "";

int32_t fail(int32_t code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

int32_t hip_fail(hipError_t e, const char* what) {
    return fail(LPM_EHIP, "%s failed: %s", what, hipGetErrorString(e));
}

int32_t validate_network(const lpm_layer* layers, int32_t L, std::vector<lpm_layer>& norm,
                         std::vector<Shape>& shapes) {
    if (!layers || L <= 0) return fail(LPM_EINVAL, "layer list is empty");
    norm.assign(layers, layers + L);
    shapes.assign((size_t)L + 1, Shape{0, 0, 0});
    if (layers[0].src != -1) return fail(LPM_ESHAPE, "layer 0 must read tensor -1 (the network input)");
    const int32_t d0 = (has_weights(layers[0]) && layers[0].d_in > 1) ? layers[0].d_in : 1;
    shapes[0] = Shape{layers[0].cin, d0 * layers[0].h_in, layers[0].w_in};
    for (int32_t i = 0; i < L; ++i) {
        lpm_layer& l = norm[i];
        if (l.kind < LPM_CONV || l.kind > LPM_ATTN) return fail(LPM_EINVAL, "layer %d: unknown kind %d", i, l.kind);
        if (l.d_in < 0 || l.kd < 0 || l.pad_d < 0) return fail(LPM_ESHAPE, "layer %d: negative depth field", i);
        if (!has_weights(l) && (l.d_in > 1 || l.kd > 1 || l.pad_d > 0))
            return fail(LPM_ESHAPE, "layer %d: only CONV / FC layers take a depth (other kinds see it folded into the height)", i);
        if (l.d_in == 0) l.d_in = 1;
        if (l.kd == 0) l.kd = 1;
        if (l.cin <= 0 || l.h_in <= 0 || l.w_in <= 0) return fail(LPM_ESHAPE, "layer %d: non-positive input extent", i);
        if (l.src < -1 || l.src >= i) return fail(LPM_ESHAPE, "layer %d: src %d is not an earlier tensor", i, l.src);
        const Shape in = shapes[(size_t)l.src + 1];
        if (in.c != l.cin || in.h != l.d_in * l.h_in || in.w != l.w_in)
            return fail(LPM_ESHAPE, "layer %d: input extent %dx%dx%d does not match tensor %d (%dx%dx%d)", i, l.cin,
                        l.h_in, l.w_in, l.src, in.c, in.h, in.w);
        Shape out{};
        switch (l.kind) {
            case LPM_FC:
                l.kh = l.h_in; l.kw = l.w_in; l.stride = 1; l.pad = 0; l.kd = l.d_in; l.pad_d = 0;
                [[fallthrough]];
            case LPM_CONV: {
                if (l.cout <= 0 || l.kh <= 0 || l.kw <= 0 || l.stride <= 0 || l.pad < 0)
                    return fail(LPM_ESHAPE, "layer %d: bad convolution geometry", i);
                if (l.pad >= l.kh || l.pad >= l.kw || l.pad_d >= l.kd) return fail(LPM_ESHAPE, "layer %d: pad must be smaller than the kernel", i);
                const int32_t ho = (l.h_in + 2 * l.pad - l.kh), wo = (l.w_in + 2 * l.pad - l.kw), dpo = (l.d_in + 2 * l.pad_d - l.kd);
                if (ho < 0 || wo < 0 || dpo < 0) return fail(LPM_ESHAPE, "layer %d: kernel larger than padded input", i);
                out = Shape{l.cout, (dpo / l.stride + 1) * (ho / l.stride + 1), wo / l.stride + 1};
                if (l.flags & ~(LPM_RELU | LPM_BIAS | LPM_SCALE)) return fail(LPM_EINVAL, "layer %d: unknown flags", i);
                if (l.add_src != LPM_NONE) {
                    if (l.add_src < -1 || l.add_src >= i) return fail(LPM_ESHAPE, "layer %d: add_src %d is not an earlier tensor", i, l.add_src);
                    const Shape a = shapes[(size_t)l.add_src + 1];
                    if (a.c != out.c || a.h != out.h || a.w != out.w)
                        return fail(LPM_ESHAPE, "layer %d: shortcut tensor %d has a different extent", i, l.add_src);
                }
                break;
            }
            case LPM_MAXPOOL2:
                if ((l.h_in & 1) || (l.w_in & 1)) return fail(LPM_ESHAPE, "layer %d: 2x2 pooling needs even H and W", i);
                out = Shape{l.cin, l.h_in / 2, l.w_in / 2};
                break;
            case LPM_GAP:
                out = Shape{l.cin, 1, 1};
                break;
            case LPM_ATTN:
                if (l.cin % 3) return fail(LPM_ESHAPE, "layer %d: attention needs 3*C input channels (queries | keys | values)", i);
                out = Shape{l.cin / 3, l.h_in, l.w_in};
                break;
            case LPM_SOFTMAX_CE:
                if (i != L - 1) return fail(LPM_ESHAPE, "layer %d: the loss must be the last layer", i);
                if (l.h_in != 1 || l.w_in != 1) return fail(LPM_ESHAPE, "layer %d: the loss needs a 1x1 input", i);
                if (l.src != i - 1 || i == 0) return fail(LPM_ESHAPE, "layer %d: the loss must read the previous layer", i);
                out = Shape{l.cin, 1, 1};
                break;
        }
        if (!has_weights(l)) {
            if (l.add_src != LPM_NONE) return fail(LPM_ESHAPE, "layer %d: only CONV/FC layers take a shortcut", i);
            l.cout = out.c; l.flags = 0;
        }
        shapes[(size_t)i + 1] = out;
    }
    return LPM_OK;
}

typedef unsigned __int128 u128;

static int32_t check_cp(const lpm_cost_params* cp) {
    if (!cp) return fail(LPM_EINVAL, "cost parameters are NULL");
    if (cp->flop_per_us == 0 || cp->hbm_byte_per_us == 0) return fail(LPM_EINVAL, "flop_per_us and hbm_byte_per_us must be positive");
    if (cp->elem_bytes != 2 && cp->elem_bytes != 4) return fail(LPM_EINVAL, "elem_bytes must be 2 or 4");
    if (cp->microbatch <= 0 || cp->n_microbatch <= 0) return fail(LPM_EINVAL, "microbatch and n_microbatch must be positive");
    return LPM_OK;
}

// Cost of one layer: larger of arithmetic time and ideal-traffic time, in picoseconds.
static uint64_t layer_cost(const std::vector<lpm_layer>& net, const std::vector<Shape>& shapes, int32_t i,
                           const lpm_cost_params& cp) {
    const lpm_layer& l = net[i];
    const u128 e = (u128)cp.elem_bytes, m = (u128)cp.microbatch, M = (u128)cp.n_microbatch;
    const u128 in_el = shapes[(size_t)l.src + 1].elems(), out_el = shapes[(size_t)i + 1].elems();
    const bool hw = has_weights(l);
    const u128 w_el = hw ? (u128)l.cout * l.cin * taps_of(l) : 0;
    const u128 p_el = w_el + ((hw && (l.flags & LPM_BIAS)) ? (u128)l.cout : 0);
    u128 mac = hw ? out_el * (u128)l.cin * taps_of(l) : 0;
    if (l.kind == LPM_ATTN) mac = 2 * (u128)l.h_in * l.w_in * l.h_in * l.w_in * (u128)(l.cin / 3);      // S = q^T k and y = A v
    const bool first = l.src < 0;
    const u128 flop = 2 * mac * m * (first ? 2 : 3);
    const u128 sc = (l.add_src != LPM_NONE) ? out_el : 0;
    const u128 fwd = (in_el + out_el + sc) * m * e + w_el * e;
    const u128 bwd = (out_el + in_el + (first ? 0 : in_el) + sc) * m * e + w_el * e + 8 * w_el;
    const u128 upd = p_el * (u128)(20 + (cp.elem_bytes == 2 ? 2 : 0));
    const u128 t_flop = flop * 1000000u / cp.flop_per_us;
    const u128 t_byte = ((fwd + bwd) * M + upd) * 1000000u / (M * cp.hbm_byte_per_us);
    const u128 t = t_flop > t_byte ? t_flop : t_byte;
    return (uint64_t)t;
}

struct Planner {
    int32_t L, Z;
    std::vector<uint64_t> prefix;      // prefix[i] = sum of layer costs [0,i)
    std::vector<uint64_t> cut_bytes;   // bytes crossing a cut placed after layer i
    std::vector<uint64_t> cut_time;    // transfer time of that cut (0 when no link)
    std::vector<char> allowed;         // cut allowed after layer i

    uint64_t stage_cost(int32_t i, int32_t j) const {   // layers [i,j); boundaries exist unless at the ends
        uint64_t c = prefix[j] - prefix[i];
        if (i > 0) c += cut_time[i - 1];
        if (j < L) c += cut_time[j - 1];
        return c;
    }
};

}  // namespace lpm

using namespace lpm;

extern "C" const char* lpm_last_error(void) { return g_err.c_str(); }

extern "C" int32_t lpm_layer_cost(const lpm_layer* layers, int32_t L, int32_t i, const lpm_cost_params* cp,
                                  uint64_t* out_cost) {
    std::vector<lpm_layer> net;
    std::vector<Shape> shapes;
    int32_t rc = validate_network(layers, L, net, shapes);
    if (rc) return rc;
    if ((rc = check_cp(cp))) return rc;
    if (i < 0 || i >= L || !out_cost) return fail(LPM_EINVAL, "layer index out of range or NULL output");
    *out_cost = layer_cost(net, shapes, i, *cp);
    return LPM_OK;
}

static int32_t plan(const lpm_layer* layers, int32_t L, int32_t Z, const lpm_cost_params* cp, const uint64_t* given_cost,
                    const int32_t* fixed_starts, int32_t* out_starts, uint64_t* out_stage_cost) {
    std::vector<lpm_layer> net;
    std::vector<Shape> shapes;
    int32_t rc = validate_network(layers, L, net, shapes);
    if (rc) return rc;
    if ((rc = check_cp(cp))) return rc;
    if (Z <= 0 || Z > L) return fail(LPM_EINVAL, "Z must be in 1..L");
    if (!out_starts) return fail(LPM_EINVAL, "out_starts is NULL");

    Planner P;
    P.L = L; P.Z = Z;
    P.prefix.assign((size_t)L + 1, 0);
    P.cut_bytes.assign(L, 0); P.cut_time.assign(L, 0); P.allowed.assign(L, 0);
    for (int32_t i = 0; i < L; ++i) {
        const uint64_t c = given_cost ? given_cost[i] : layer_cost(net, shapes, i, *cp);
        if (P.prefix[i] + c < P.prefix[i]) return fail(LPM_EINVAL, "layer costs overflow 64 bits");
        P.prefix[i + 1] = P.prefix[i] + c;
        P.cut_bytes[i] = (uint64_t)shapes[(size_t)i + 1].elems() * (uint64_t)cp->microbatch * (uint64_t)cp->elem_bytes;
        if (cp->link_byte_per_us > 0)
            P.cut_time[i] = (uint64_t)((u128)2 * P.cut_bytes[i] * 1000000u / cp->link_byte_per_us);
        P.allowed[i] = (i < L - 1) && net[i].cut_allowed_after != 0;
    }

    std::vector<int32_t> starts((size_t)Z + 1, 0);
    if (fixed_starts) {
        if (fixed_starts[0] != 0 || fixed_starts[Z] != L) return fail(LPM_ENOPLAN, "fixed plan must start at 0 and end at L");
        for (int32_t z = 1; z <= Z; ++z) {
            if (fixed_starts[z] <= fixed_starts[z - 1]) return fail(LPM_ENOPLAN, "fixed plan has an empty or reversed stage");
            if (fixed_starts[z] > L || (z < Z && fixed_starts[z] >= L))          // (before the value indexes anything)
                return fail(LPM_ENOPLAN, "fixed plan: stage %d would start at layer %d of %d", z, fixed_starts[z], L);
            if (z < Z && !P.allowed[fixed_starts[z] - 1])
                return fail(LPM_ENOPLAN, "fixed plan cuts after layer %d, where no cut is allowed", fixed_starts[z] - 1);
        }
        starts.assign(fixed_starts, fixed_starts + Z + 1);
    } else {
        const uint64_t INF = std::numeric_limits<uint64_t>::max();
        // f[k][i]: smallest achievable bottleneck when layers [i,L) form stages k..Z-1
        std::vector<std::vector<uint64_t>> f((size_t)Z + 1, std::vector<uint64_t>((size_t)L + 1, INF));
        auto can_start = [&](int32_t k, int32_t i) { return k == 0 ? i == 0 : (i > 0 && P.allowed[i - 1]); };
        for (int32_t i = 0; i < L; ++i)
            if (can_start(Z - 1, i)) f[Z - 1][i] = P.stage_cost(i, L);
        for (int32_t k = Z - 2; k >= 0; --k)
            for (int32_t i = 0; i < L; ++i) {
                if (!can_start(k, i)) continue;
                for (int32_t j = i + 1; j < L; ++j) {
                    if (!P.allowed[j - 1] || f[k + 1][j] == INF) continue;
                    const uint64_t c = P.stage_cost(i, j);
                    const uint64_t b = c > f[k + 1][j] ? c : f[k + 1][j];
                    if (b < f[k][i]) f[k][i] = b;
                }
            }
        const uint64_t best = f[0][0];
        if (best == INF) return fail(LPM_ENOPLAN, "the network has fewer than %d allowed cut points", Z - 1);
        // g[k][i]: smallest total boundary bytes for [i,L) as stages k..Z-1 with every stage cost <= best
        std::vector<std::vector<uint64_t>> g((size_t)Z + 1, std::vector<uint64_t>((size_t)L + 1, INF));
        for (int32_t i = 0; i < L; ++i)
            if (can_start(Z - 1, i) && P.stage_cost(i, L) <= best) g[Z - 1][i] = 0;
        for (int32_t k = Z - 2; k >= 0; --k)
            for (int32_t i = 0; i < L; ++i) {
                if (!can_start(k, i)) continue;
                for (int32_t j = i + 1; j < L; ++j) {
                    if (!P.allowed[j - 1] || g[k + 1][j] == INF || P.stage_cost(i, j) > best) continue;
                    const uint64_t b = P.cut_bytes[j - 1] + g[k + 1][j];
                    if (b < g[k][i]) g[k][i] = b;
                }
            }
        // smallest starts among the plans reaching (best, g[0][0])
        int32_t i = 0;
        for (int32_t k = 0; k < Z - 1; ++k) {
            int32_t pick = -1;
            for (int32_t j = i + 1; j < L && pick < 0; ++j) {
                if (!P.allowed[j - 1] || g[k + 1][j] == INF || P.stage_cost(i, j) > best) continue;
                if (P.cut_bytes[j - 1] + g[k + 1][j] == g[k][i]) pick = j;
            }
            if (pick < 0) return fail(LPM_ENOPLAN, "internal: plan reconstruction failed");
            starts[k + 1] = pick;
            i = pick;
        }
        starts[Z] = L;
    }
    for (int32_t z = 0; z <= Z; ++z) out_starts[z] = starts[z];
    if (out_stage_cost)
        for (int32_t z = 0; z < Z; ++z) out_stage_cost[z] = P.stage_cost(starts[z], starts[z + 1]);
    return LPM_OK;
}

extern "C" int32_t lpm_partition(const lpm_layer* layers, int32_t L, int32_t Z, const lpm_cost_params* cp,
                                 const int32_t* fixed_starts, int32_t* out_starts, uint64_t* out_stage_cost) {
    return plan(layers, L, Z, cp, nullptr, fixed_starts, out_starts, out_stage_cost);
}

extern "C" int32_t lpm_partition_costs(const lpm_layer* layers, int32_t L, int32_t Z, const lpm_cost_params* cp,
                                       const uint64_t* layer_cost_ps, const int32_t* fixed_starts, int32_t* out_starts,
                                       uint64_t* out_stage_cost) {
    if (!layer_cost_ps) return fail(LPM_EINVAL, "layer_cost_ps is NULL");
    return plan(layers, L, Z, cp, layer_cost_ps, fixed_starts, out_starts, out_stage_cost);
}

// extern "C" boundary: plan handling, the step executor (Algorithm 1 then Algorithm 2, as
// lowered by plan.cpp into a launch list) and the per-kernel entry points.
#include <cmath>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/monet.h"
#include "../../include/monet_kernels.h"
#include "kernels.hpp"
#include "plan.hpp"

using namespace monet;

static thread_local std::string g_err;

struct monet_plan;
namespace {
void build_programs(monet_plan *p);
}

// One entry of the step program: a single operator launch, or two neighbours run as one fused kernel.
enum { FUSE_NONE = 0, FUSE_BN_RELU_FWD, FUSE_ADD_RELU_FWD, FUSE_RELU_BN_BWD, FUSE_RELU_ADD_BWD,
       FUSE_CONV_BN_APPLY,                             // a recomputed convolution applies its in-place BatchNorm in the epilogue
       FUSE_BN_ADD_RELU_FWD, FUSE_RELU_ADD_BN_BWD,     // these two join three launches (tail of a residual block)
       FUSE_CONV_BN_RELU };                            // FUSE_CONV_BN_APPLY plus the in-place ReLU behind the BatchNorm (three launches)
struct ProgStep {
    int fuse;
    size_t a, b, c;   // indices into Plan::launches (b when fused, c when three are fused)
    bool three() const { return fuse == FUSE_BN_ADD_RELU_FWD || fuse == FUSE_RELU_ADD_BN_BWD || fuse == FUSE_CONV_BN_RELU; }
    size_t last() const { return fuse == FUSE_NONE ? a : (three() ? c : b); }
};

struct monet_plan {
    Plan plan;
    std::vector<ProgStep> prog_plain, prog_fused;
    // per launch: a forward convolution whose epilogue also leaves the partial statistics of the BatchNorm that
    // runs next (feeds_stats), and that BatchNorm launch (stats_fed), which then only merges them
    std::vector<char> feeds_stats, stats_fed;
    bool fusion = true;
    bool timed_fused = false;
    char *base = nullptr;      // device memory bound by the caller
    size_t bound_bytes = 0;
    bool poison = false;
    int64_t stop_after = -1;
    bool timing = false;
    std::vector<hipEvent_t> ev;   // 2 per launch, created on first use
    bool timed_step_done = false;
    ~monet_plan() {
        for (auto e : ev) (void)hipEventDestroy(e);
    }
};

template <class F>
static int guarded(F &&f) {
    try {
        f();
        return MONET_OK;
    } catch (const PlanError &e) {
        g_err = e.what();
        return e.code;
    } catch (const KernelError &e) {
        g_err = e.what();
        return MONET_HIP_ERROR;
    } catch (const std::exception &e) {
        g_err = e.what();
        return MONET_BAD_ARGUMENT;
    }
}

extern "C" const char *monet_last_error(void) { return g_err.c_str(); }

extern "C" int monet_plan_load(const char *graph, size_t graph_len, const char *schedule, size_t schedule_len, monet_plan **out) {
    if (!graph || !schedule || !out) { g_err = "monet_plan_load: null argument"; return MONET_BAD_ARGUMENT; }
    *out = nullptr;
    monet_plan *p = nullptr;
    int rc = guarded([&] {
        p = new monet_plan();
        p->plan.build(std::string(graph, graph_len), std::string(schedule, schedule_len));
        build_programs(p);
    });
    if (rc != MONET_OK) { delete p; return rc; }
    *out = p;
    return MONET_OK;
}

extern "C" void monet_free(monet_plan *p) { delete p; }
extern "C" int64_t monet_plan_exact_peak(const monet_plan *p) { return p ? p->plan.exact_peak : MONET_BAD_ARGUMENT; }
extern "C" int64_t monet_plan_predicted_peak(const monet_plan *p) { return p ? p->plan.predicted_peak : MONET_BAD_ARGUMENT; }
extern "C" int64_t monet_plan_predicted_peak_tight(const monet_plan *p) { return p ? p->plan.predicted_peak_tight : MONET_BAD_ARGUMENT; }
extern "C" int64_t monet_plan_arena_bytes(const monet_plan *p) { return p ? p->plan.persistent_bytes + p->plan.dynamic_bytes : MONET_BAD_ARGUMENT; }
extern "C" int64_t monet_plan_persistent_bytes(const monet_plan *p) { return p ? p->plan.persistent_bytes : MONET_BAD_ARGUMENT; }
extern "C" int monet_plan_num_params(const monet_plan *p) { return p ? (int)p->plan.g.params.size() : MONET_BAD_ARGUMENT; }
extern "C" int monet_plan_num_inputs(const monet_plan *p) { return p ? (int)p->plan.g.exts.size() : MONET_BAD_ARGUMENT; }

extern "C" int monet_plan_bind_arena(monet_plan *p, void *dev_base, size_t bytes) {
    if (!p || !dev_base) { g_err = "monet_plan_bind_arena: null argument"; return MONET_BAD_ARGUMENT; }
    if (((uintptr_t)dev_base) % kAlign) { g_err = "monet_plan_bind_arena: base must be 256-byte aligned"; return MONET_BAD_ARGUMENT; }
    if ((int64_t)bytes < p->plan.persistent_bytes + p->plan.dynamic_bytes) {
        g_err = "monet_plan_bind_arena: " + std::to_string(bytes) + " bytes bound, " +
                std::to_string(p->plan.persistent_bytes + p->plan.dynamic_bytes) + " needed";
        return MONET_ARENA_TOO_SMALL;
    }
    p->base = (char *)dev_base;
    p->bound_bytes = bytes;
    return MONET_OK;
}

extern "C" int monet_plan_trace(const monet_plan *p, const monet_event **events, size_t *count) {
    if (!p || !events || !count) { g_err = "monet_plan_trace: null argument"; return MONET_BAD_ARGUMENT; }
    *events = p->plan.events.data();
    *count = p->plan.events.size();
    return MONET_OK;
}

extern "C" int monet_plan_set_poison(monet_plan *p, int on) {
    if (!p) return MONET_BAD_ARGUMENT;
    p->poison = on != 0;
    return MONET_OK;
}

extern "C" int monet_plan_set_stop_after(monet_plan *p, int64_t event_index) {
    if (!p) return MONET_BAD_ARGUMENT;
    p->stop_after = event_index;
    return MONET_OK;
}

extern "C" int64_t monet_plan_tensor_offset(const monet_plan *p, size_t event_index, int node, int is_grad) {
    if (!p) return MONET_BAD_ARGUMENT;
    const Plan &pl = p->plan;
    for (size_t i = 0; i < pl.launches.size(); ++i)
        if (pl.launches[i].event == event_index) {
            auto it = pl.where[i].find({node, is_grad ? 1 : 0});
            return it == pl.where[i].end() ? -1 : pl.persistent_bytes + it->second;
        }
    return -1;
}

extern "C" int64_t monet_plan_bn_stats_offset(const monet_plan *p, int node) {
    if (!p) return MONET_BAD_ARGUMENT;
    auto it = p->plan.bn_stats_off.find(node);
    return it == p->plan.bn_stats_off.end() ? -1 : it->second;
}

// ------------------------------------------------------------------ the step
namespace {

struct StepCtx {
    monet_plan *mp;
    hipStream_t st;
    const void *const *inputs;
    const float *const *weights;
    float *const *grads;
    char *arena() const { return mp->base + mp->plan.persistent_bytes; }
    void *ptr(const Ref &r) const {
        switch (r.region) {
            case R_ARENA: return arena() + r.off;
            case R_EXT: return const_cast<void *>(inputs[r.off]);
            case R_PERSIST: return mp->base + r.off;
            default: return nullptr;
        }
    }
    float *scratch() const { return (float *)(mp->base + mp->plan.scratch_off); }
    size_t scratch_bytes() const { return (size_t)mp->plan.scratch_bytes; }
    float *bn_stats(int node) const { return (float *)(mp->base + mp->plan.bn_stats_off.at(node)); }
    size_t index_of(const Launch &L) const { return (size_t)(&L - mp->plan.launches.data()); }
    bool feeds_stats(const Launch &L) const { return mp->feeds_stats[index_of(L)] != 0; }
    bool stats_fed(const Launch &L) const { return mp->stats_fed[index_of(L)] != 0; }
};

ConvShape conv_shape(const Graph &g, const Node &n) {
    const auto &is = g.shape_of(n.ins[0]);
    ConvShape cs;
    cs.N = (int)is[0]; cs.H = (int)is[1]; cs.W = (int)is[2]; cs.C = (int)is[3];
    cs.K = (int)n.shape[3]; cs.R = n.attr_int("R"); cs.S = n.attr_int("S");
    cs.stride = n.attr_int("stride", 1); cs.pad = n.attr_int("pad", 0);
    cs.P = (int)n.shape[1]; cs.Q = (int)n.shape[2];
    return cs;
}
// A transposed convolution x[N,H,W,C] -> y[N,P,Q,K] with filter C,R,S,K is the adjoint of the convolution
// y-shaped -> x-shaped with that same array read as its K',R,S,C' filter (K' = C, C' = K): forward = that
// convolution's input gradient, input gradient = its forward, filter gradient = its filter gradient with
// input and output-gradient exchanged.  This returns the shape of that convolution.
ConvShape tconv_adjoint_shape(const Graph &g, const Node &n) {
    const auto &is = g.shape_of(n.ins[0]);
    ConvShape cs;
    cs.N = (int)is[0]; cs.H = (int)n.shape[1]; cs.W = (int)n.shape[2]; cs.C = (int)n.shape[3];
    cs.K = (int)is[3]; cs.R = n.attr_int("R"); cs.S = n.attr_int("S");
    cs.stride = n.attr_int("stride", 1); cs.pad = 0;
    cs.P = (int)is[1]; cs.Q = (int)is[2];
    if ((cs.H - cs.R) / cs.stride + 1 != cs.P || (cs.W - cs.S) / cs.stride + 1 != cs.Q || (cs.H - cs.R) % cs.stride || (cs.W - cs.S) % cs.stride)
        throw KernelError("transposed convolution: output extent does not match (H-1)*stride+R");
    return cs;
}
int64_t numel_of(const std::vector<int64_t> &s);
ConvShape linear_shape(const Graph &g, const Node &n) {   // a linear layer is a 1x1 convolution on a 1x1 image
    const auto &is = g.shape_of(n.ins[0]);
    ConvShape cs;
    cs.N = (int)is[0]; cs.H = 1; cs.W = 1; cs.C = (int)(numel_of(is) / is[0]);
    cs.K = (int)n.shape[1]; cs.R = 1; cs.S = 1; cs.stride = 1; cs.pad = 0; cs.P = 1; cs.Q = 1;
    return cs;
}
PoolShape pool_shape(const Graph &g, const Node &n) {
    const auto &is = g.shape_of(n.ins[0]);
    PoolShape ps;
    ps.N = (int)is[0]; ps.H = (int)is[1]; ps.W = (int)is[2]; ps.C = (int)is[3];
    ps.k = n.attr_int("k"); ps.stride = n.attr_int("stride", 1); ps.pad = n.attr_int("pad", 0);
    ps.P = (int)n.shape[1]; ps.Q = (int)n.shape[2];
    return ps;
}
int64_t numel_of(const std::vector<int64_t> &s) {
    int64_t n = 1;
    for (auto d : s) n *= d;
    return n;
}

// number of reduction splits an implementation record asks for ("splitk" / "igemm_splitk" carry splits=S)
// output tile edge of a Winograd implementation name, 0 for any other
int winograd_tile(const std::string &algo) { return algo == "winograd" ? 2 : (algo == "winograd4" || algo == "winograd4f") ? 4 : 0; }
// the one-kernel F(4x4) form (workspace: transformed filters only)
bool winograd_is_fused(const std::string &algo) { return algo == "winograd4f"; }

int splits_of(const std::string &algo, const Attrs &extra) {
    if (algo.find("splitk") == std::string::npos) return 1;
    auto it = extra.find("splits");
    if (it == extra.end()) throw KernelError("split implementation without a 'splits' field");
    return std::stoi(it->second);
}

void run_forward(const StepCtx &c, const Launch &L, const BnAffine *affine = nullptr) {
    const Graph &g = c.mp->plan.g;
    const Node &n = g.nodes[L.id];
    const float *in0 = (const float *)c.ptr(L.a[0]);
    float *out = (float *)c.ptr(L.a[2]);
    const std::string &op = n.op;
    if (op == "conv") {
        const FwdImpl &im = n.fimpls[L.impl];
        if (im.algo == "im2col")
            conv_im2col_fwd(c.st, in0, c.weights[n.pars[0]], out, conv_shape(g, n), (float *)c.ptr(L.a[4]), (size_t)align_up(im.ws), false);
        else if (winograd_is_fused(im.algo))
            conv_winograd_fused(c.st, in0, c.weights[n.pars[0]], out, conv_shape(g, n), false, false, (float *)c.ptr(L.a[4]),
                                (size_t)align_up(im.ws), affine);
        else if (const int m = winograd_tile(im.algo))
            conv_winograd(c.st, in0, c.weights[n.pars[0]], out, conv_shape(g, n), m, false, false, (float *)c.ptr(L.a[4]),
                          (size_t)align_up(im.ws), affine);
        else
            conv_fwd(c.st, in0, c.weights[n.pars[0]], out, conv_shape(g, n), splits_of(im.algo, im.extra), (float *)c.ptr(L.a[4]),
                     (size_t)(im.ws > 0 ? align_up(im.ws) : 0), false, c.feeds_stats(L) ? c.scratch() : nullptr, affine);
    } else if (op == "tconv") {
        conv_dgrad(c.st, in0, c.weights[n.pars[0]], out, tconv_adjoint_shape(g, n), false);
    } else if (op == "dwconv") {
        dwconv_fwd(c.st, in0, c.weights[n.pars[0]], out, conv_shape(g, n), affine);
    } else if (op == "concat") {
        const int Ca = (int)g.shape_of(n.ins[0]).back(), Cb = (int)g.shape_of(n.ins[1]).back();
        const int64_t rows = numel_of(n.shape) / (Ca + Cb);
        column_copy(c.st, in0, Ca, out, Ca + Cb, Ca, rows, false);
        column_copy(c.st, (const float *)c.ptr(L.a[1]), Cb, out + Ca, Ca + Cb, Cb, rows, false);
    } else if (op == "bn") {
        int C = (int)n.shape.back();
        int64_t rows = numel_of(n.shape) / C;
        float *stats = c.bn_stats(L.id);
        // statistics are computed by the forward pass and reused when the node is recomputed
        if (L.kind == EV_RUN_FWD)
            bn_stats(c.st, in0, stats, rows, C, (float)n.attr_f("eps", 1e-5), c.scratch(), c.scratch_bytes(), c.stats_fed(L));
        bn_apply(c.st, in0, out, c.weights[n.pars[0]], c.weights[n.pars[1]], stats, rows, C);
    } else if (op == "relu" || op == "relu6") {
        relu_fwd(c.st, in0, out, (L.flags & 2) ? (uint64_t *)c.ptr(L.a[3]) : nullptr, numel_of(n.shape), op == "relu6");
    } else if (op == "maxpool") {
        maxpool_fwd(c.st, in0, out, (L.flags & 2) ? (uint8_t *)c.ptr(L.a[3]) : nullptr, pool_shape(g, n));
    } else if (op == "add") {
        add_fwd(c.st, in0, (const float *)c.ptr(L.a[1]), out, numel_of(n.shape));
    } else if (op == "avgpool") {
        const auto &is = g.shape_of(n.ins[0]);
        avgpool_fwd(c.st, in0, out, (int)is[0], (int)(is[1] * is[2]), (int)is[3]);
    } else if (op == "linear") {
        const auto &is = g.shape_of(n.ins[0]);
        linear_fwd(c.st, in0, c.weights[n.pars[0]], c.weights[n.pars[1]], out, (int)is[0], (int)(numel_of(is) / is[0]), (int)n.shape[1],
                   c.scratch(), c.scratch_bytes());
    } else if (op == "softmaxce") {
        const auto &is = g.shape_of(n.ins[0]);
        const int classes = (int)is.back();
        const int64_t rows = numel_of(is) / classes;
        // few classes (per-pixel scores): one thread per row; many classes: one workgroup per row
        if (classes <= 32) softmaxce_rows_fwd(c.st, in0, (const int32_t *)c.ptr(L.a[1]), out, rows, classes, c.scratch(), c.scratch_bytes());
        else {
            if ((size_t)rows * 4 > c.scratch_bytes()) throw KernelError("softmaxce: scratch too small for the row losses");
            softmaxce_fwd(c.st, in0, (const int32_t *)c.ptr(L.a[1]), out, (int)rows, classes, c.scratch());
        }
    } else if (op == "sumloss") {
        sumloss_fwd(c.st, in0, out, numel_of(g.shape_of(n.ins[0])), c.scratch(), c.scratch_bytes());
    } else {
        throw KernelError("no kernel for forward operator " + op);
    }
}

void run_backward(const StepCtx &c, const Launch &L) {
    const Graph &g = c.mp->plan.g;
    const Bop &b = g.bops[L.id];
    const Node &n = g.nodes[b.node];
    const BwdImpl &im = b.impls[L.impl];
    const float *gy = (const float *)c.ptr(L.a[0]);
    const void *dep = c.ptr(L.a[1]);
    float *d0 = (float *)c.ptr(L.a[2]);
    const bool acc0 = L.flags & 1;
    const std::string &kd = b.kind;
    if (kd == "conv_wgrad") {
        if (im.algo == "im2col")
            conv_im2col_wgrad(c.st, (const float *)dep, gy, c.grads[n.pars[0]], conv_shape(g, n), (float *)c.ptr(L.a[4]), (size_t)align_up(im.ws));
        else if (const int m = winograd_tile(im.algo))
            conv_winograd_wgrad(c.st, (const float *)dep, gy, c.grads[n.pars[0]], conv_shape(g, n), m, (float *)c.ptr(L.a[4]),
                                (size_t)align_up(im.ws));
        else
            conv_wgrad(c.st, (const float *)dep, gy, c.grads[n.pars[0]], conv_shape(g, n), splits_of(im.algo, im.extra),
                       (float *)c.ptr(L.a[4]), (size_t)(im.ws > 0 ? align_up(im.ws) : 0));
    } else if (kd == "conv_dgrad") {
        if (winograd_is_fused(im.algo))
            conv_winograd_fused(c.st, gy, c.weights[n.pars[0]], d0, conv_shape(g, n), true, acc0, (float *)c.ptr(L.a[4]), (size_t)align_up(im.ws));
        else if (const int m = winograd_tile(im.algo))
            conv_winograd(c.st, gy, c.weights[n.pars[0]], d0, conv_shape(g, n), m, true, acc0, (float *)c.ptr(L.a[4]), (size_t)align_up(im.ws));
        else
            conv_dgrad(c.st, gy, c.weights[n.pars[0]], d0, conv_shape(g, n), acc0, splits_of(im.algo, im.extra), (float *)c.ptr(L.a[4]),
                       (size_t)(im.ws > 0 ? align_up(im.ws) : 0));
    } else if (kd == "tconv_wgrad") {
        // filter gradient of the adjoint convolution: its input is this operator's output gradient, its
        // output gradient this operator's input
        conv_wgrad(c.st, gy, (const float *)dep, c.grads[n.pars[0]], tconv_adjoint_shape(g, n), splits_of(im.algo, im.extra),
                   (float *)c.ptr(L.a[4]), (size_t)(im.ws > 0 ? align_up(im.ws) : 0));
    } else if (kd == "tconv_dgrad") {
        conv_fwd(c.st, gy, c.weights[n.pars[0]], d0, tconv_adjoint_shape(g, n), 1, nullptr, 0, acc0);
    } else if (kd == "dwconv_wgrad") {
        dwconv_wgrad(c.st, (const float *)dep, gy, c.grads[n.pars[0]], conv_shape(g, n), c.scratch(), c.scratch_bytes());
    } else if (kd == "dwconv_dgrad") {
        dwconv_dgrad(c.st, gy, c.weights[n.pars[0]], d0, conv_shape(g, n), acc0);
    } else if (kd == "concat_bwd") {
        const int Ca = (int)g.shape_of(n.ins[0]).back(), Cb = (int)g.shape_of(n.ins[1]).back();
        const int64_t rows = numel_of(n.shape) / (Ca + Cb);
        if (n.ins[0] > 0) column_copy(c.st, gy, Ca + Cb, d0, Ca, Ca, rows, acc0);
        if (n.ins[1] > 0) column_copy(c.st, gy + Ca, Ca + Cb, (float *)c.ptr(L.a[3]), Cb, Cb, rows, (L.flags & 2) != 0);
    } else if (kd == "bn_bwd") {
        int C = (int)n.shape.back();
        int64_t rows = numel_of(n.shape) / C;
        bn_bwd(c.st, gy, (const float *)dep, im.algo == "from_output", c.weights[n.pars[0]], c.weights[n.pars[1]], c.bn_stats(b.node), d0,
               c.grads[n.pars[0]], c.grads[n.pars[1]], rows, C, acc0, c.scratch(), c.scratch_bytes());
    } else if (kd == "relu_bwd" || kd == "relu6_bwd") {
        int mode = im.algo == "from_input" ? RELU_FROM_INPUT : (im.algo == "from_output" ? RELU_FROM_OUTPUT : RELU_FROM_MASK);
        relu_bwd(c.st, gy, dep, mode, d0, numel_of(n.shape), kd == "relu6_bwd", acc0);
    } else if (kd == "maxpool_bwd") {
        bool from_idx = im.algo == "from_index";
        maxpool_bwd(c.st, gy, from_idx ? nullptr : (const float *)dep, from_idx ? (const uint8_t *)dep : nullptr, d0, pool_shape(g, n), acc0);
    } else if (kd == "add_bwd") {
        int64_t cnt = numel_of(n.shape);
        if (n.ins[0] > 0) copy_or_accumulate(c.st, gy, d0, cnt, acc0);
        if (n.ins.size() > 1 && n.ins[1] > 0) copy_or_accumulate(c.st, gy, (float *)c.ptr(L.a[3]), cnt, (L.flags & 2) != 0);
    } else if (kd == "avgpool_bwd") {
        const auto &is = g.shape_of(n.ins[0]);
        avgpool_bwd(c.st, gy, d0, (int)is[0], (int)(is[1] * is[2]), (int)is[3], acc0);
    } else if (kd == "linear_wgrad") {
        const auto &is = g.shape_of(n.ins[0]);
        linear_wgrad(c.st, (const float *)dep, gy, c.grads[n.pars[0]], c.grads[n.pars[1]], (int)is[0], (int)(numel_of(is) / is[0]), (int)n.shape[1]);
    } else if (kd == "linear_dgrad") {
        const auto &is = g.shape_of(n.ins[0]);
        linear_dgrad(c.st, gy, c.weights[n.pars[0]], d0, (int)is[0], (int)(numel_of(is) / is[0]), (int)n.shape[1], acc0, c.scratch(),
                     c.scratch_bytes());
    } else if (kd == "softmaxce_bwd") {
        const auto &is = g.shape_of(n.ins[0]);
        Ref lab; lab.region = R_EXT; lab.off = -n.ins[1];
        const int classes = (int)is.back();
        const int64_t rows = numel_of(is) / classes;
        if (classes <= 32) softmaxce_rows_bwd(c.st, (const float *)dep, (const int32_t *)c.ptr(lab), d0, rows, classes, acc0);
        else softmaxce_bwd(c.st, (const float *)dep, (const int32_t *)c.ptr(lab), d0, (int)rows, classes, acc0);
    } else if (kd == "sumloss_bwd") {
        int64_t cnt = numel_of(g.shape_of(n.ins[0]));
        if (acc0) throw KernelError("sumloss_bwd cannot accumulate");
        fill_f32(c.st, d0, cnt, 1.0f);
    } else {
        throw KernelError("no kernel for backward operator " + kd);
    }
}

}  // namespace

namespace {

// neighbouring operators whose kinds and data flow allow one kernel
int fusable_pattern(const Plan &pl, const Launch &L1, const Launch &L2) {
    const Graph &g = pl.g;
    const bool f1 = L1.kind != EV_RUN_BWD, f2 = L2.kind != EV_RUN_BWD;
    if (f1 && f2) {
        const Node &n1 = g.nodes[L1.id], &n2 = g.nodes[L2.id];
        if ((n2.op != "relu" && n2.op != "relu6") || n2.ins[0] != n1.id) return FUSE_NONE;
        if (numel_of(n2.shape) % 4) return FUSE_NONE;
        if (n1.op == "bn" && n1.shape.back() % 4 == 0) return FUSE_BN_RELU_FWD;
        if (n1.op == "add") return FUSE_ADD_RELU_FWD;
        return FUSE_NONE;
    }
    if (!f1 && !f2) {
        const Bop &b1 = g.bops[L1.id], &b2 = g.bops[L2.id];
        if (b1.kind != "relu_bwd" && b1.kind != "relu6_bwd") return FUSE_NONE;
        const Node &r = g.nodes[b1.node];
        if (b2.node != r.ins[0] || (L1.flags & 1) || numel_of(r.shape) % 4) return FUSE_NONE;
        if (b2.kind == "bn_bwd" && b1.impls[L1.impl].algo == "from_mask") return FUSE_RELU_BN_BWD;
        if (b2.kind == "add_bwd") return FUSE_RELU_ADD_BWD;
    }
    return FUSE_NONE;
}

// A fused kernel reads the first operator's inputs while it writes the second operator's outputs.
// In the one-by-one order those inputs may already be freed when the outputs are allocated, so the
// arena may have placed an output on top of them.  Same offset and same size is harmless for a
// tensor that every thread reads and writes at its own index; any other overlap forbids fusion.
struct Span { Ref r; int64_t bytes; bool same_index_ok; };
bool spans_conflict(const std::vector<Span> &ins, const std::vector<Span> &outs) {
    for (const Span &o : outs) {
        if (o.r.region != R_ARENA) continue;
        for (const Span &i : ins) {
            if (i.r.region != R_ARENA) continue;
            const bool disjoint = o.r.off + o.bytes <= i.r.off || i.r.off + i.bytes <= o.r.off;
            if (disjoint) continue;
            if (i.same_index_ok && i.r.off == o.r.off && i.bytes == o.bytes) continue;
            return true;
        }
    }
    return false;
}

// which neighbours can share a kernel
int fusable(const Plan &pl, const Launch &L1, const Launch &L2) {
    const Graph &g = pl.g;
    int f = fusable_pattern(pl, L1, L2);
    if (!f) return FUSE_NONE;
    std::vector<Span> ins, outs;
    if (f == FUSE_BN_RELU_FWD || f == FUSE_ADD_RELU_FWD) {
        const Node &n1 = g.nodes[L1.id], &n2 = g.nodes[L2.id];
        ins.push_back({L1.a[0], n1.bytes, true});
        if (f == FUSE_ADD_RELU_FWD) ins.push_back({L1.a[1], n1.bytes, true});
        if (!(L2.flags & 1)) outs.push_back({L1.a[2], n1.bytes, false});
        outs.push_back({L2.a[2], n2.bytes, false});
        if (L2.flags & 2) outs.push_back({L2.a[3], g.nodes[n2.aux_children[0]].bytes, false});
    } else {
        const Bop &b1 = g.bops[L1.id], &b2 = g.bops[L2.id];
        const Node &r = g.nodes[b1.node];
        const bool from_mask = b1.impls[L1.impl].algo == "from_mask";
        ins.push_back({L1.a[0], r.bytes, true});
        ins.push_back({L1.a[1], from_mask ? g.nodes[r.aux_children[0]].bytes : r.bytes, !from_mask});
        if (f == FUSE_RELU_BN_BWD) ins.push_back({L2.a[1], r.bytes, true});
        outs.push_back({L2.a[2], r.bytes, false});
        if (f == FUSE_RELU_ADD_BWD) outs.push_back({L2.a[3], r.bytes, false});
    }
    // an output may sit exactly on one input, but then on no other, and two outputs never share memory
    return spans_conflict(ins, outs) ? FUSE_NONE : f;
}

// true if the forward tensor of `node` is released between two events of the trace (exclusive)
bool freed_between(const Plan &pl, int node, size_t ev_from, size_t ev_to) {
    for (size_t e = ev_from + 1; e < ev_to && e < pl.events.size(); ++e)
        if (pl.events[e].kind == EV_FREE && pl.events[e].node == node && pl.events[e].aux == T_FWD) return true;
    return false;
}

// BatchNorm -> add -> ReLU in the forward direction.  Returns the input position of the BatchNorm in the add, or -1.
int triple_fwd(const Plan &pl, const Launch &L1, const Launch &L2, const Launch &L3) {
    const Graph &g = pl.g;
    if (L1.kind == EV_RUN_BWD || L2.kind == EV_RUN_BWD || L3.kind == EV_RUN_BWD) return -1;
    const Node &bn = g.nodes[L1.id], &ad = g.nodes[L2.id], &re = g.nodes[L3.id];
    if (bn.op != "bn" || ad.op != "add" || (re.op != "relu" && re.op != "relu6")) return -1;
    if (re.ins[0] != ad.id || ad.ins.size() != 2 || ad.ins[0] == ad.ins[1]) return -1;
    const int pos = ad.ins[0] == bn.id ? 0 : (ad.ins[1] == bn.id ? 1 : -1);
    if (pos < 0 || bn.shape.back() % 4 || numel_of(re.shape) % 4) return -1;
    std::vector<Span> ins, outs;
    ins.push_back({L1.a[0], bn.bytes, true});
    ins.push_back({L2.a[1 - pos], ad.bytes, true});
    if (!freed_between(pl, bn.id, L2.event, L3.event)) outs.push_back({L1.a[2], bn.bytes, false});
    if (!(L3.flags & 1)) outs.push_back({L2.a[2], ad.bytes, false});
    outs.push_back({L3.a[2], re.bytes, false});
    if (L3.flags & 2) outs.push_back({L3.a[3], g.nodes[re.aux_children[0]].bytes, false});
    return spans_conflict(ins, outs) ? -1 : pos;
}

// ReLU backward -> add backward -> BatchNorm backward of one of the add's inputs.  Returns that input's position, or -1.
int triple_bwd(const Plan &pl, const Launch &L1, const Launch &L2, const Launch &L3) {
    const Graph &g = pl.g;
    if (L1.kind != EV_RUN_BWD || L2.kind != EV_RUN_BWD || L3.kind != EV_RUN_BWD) return -1;
    const Bop &b1 = g.bops[L1.id], &b2 = g.bops[L2.id], &b3 = g.bops[L3.id];
    if ((b1.kind != "relu_bwd" && b1.kind != "relu6_bwd") || b2.kind != "add_bwd" || b3.kind != "bn_bwd") return -1;
    const Node &re = g.nodes[b1.node], &ad = g.nodes[b2.node], &bn = g.nodes[b3.node];
    if (re.ins[0] != ad.id || ad.ins.size() != 2 || ad.ins[0] == ad.ins[1]) return -1;
    const int pos = ad.ins[0] == bn.id ? 0 : (ad.ins[1] == bn.id ? 1 : -1);
    if (pos < 0 || (L1.flags & 1) || ((L2.flags >> pos) & 1)) return -1;    // both gradients in between are written fresh
    if (bn.shape.back() % 4 || numel_of(re.shape) % 4) return -1;
    const bool from_mask = b1.impls[L1.impl].algo == "from_mask";
    std::vector<Span> ins, outs;
    ins.push_back({L1.a[0], re.bytes, true});
    ins.push_back({L1.a[1], from_mask ? g.nodes[re.aux_children[0]].bytes : re.bytes, !from_mask});
    ins.push_back({L3.a[1], bn.bytes, true});
    outs.push_back({L3.a[2], bn.bytes, false});
    if (ad.ins[1 - pos] > 0) outs.push_back({L2.a[2 + (1 - pos)], ad.bytes, false});
    return spans_conflict(ins, outs) ? -1 : pos;
}

// Forward convolution directly followed by the first run of the BatchNorm of its output: the statistics' partial
// results come out of the convolution's epilogue, bit-identical to the stand-alone kernel's (tile_stats.hpp), so
// this is independent of launch fusion and of the schedule.
bool conv_feeds_bn_stats(const Plan &pl, const Launch &L1, const Launch &L2) {
    const Graph &g = pl.g;
    if (L1.kind != EV_RUN_FWD || L2.kind != EV_RUN_FWD) return false;
    const Node &cv = g.nodes[L1.id], &bn = g.nodes[L2.id];
    if (cv.op != "conv" || bn.op != "bn" || bn.ins[0] != cv.id) return false;
    const ConvShape cs = conv_shape(g, cv);
    if (winograd_tile(cv.fimpls[L1.impl].algo) || cv.fimpls[L1.impl].algo == "im2col") return false;
    if (!conv_fwd_aligned(cs) || cs.K % 4 || splits_of(cv.fimpls[L1.impl].algo, cv.fimpls[L1.impl].extra) != 1) return false;
    return bn_stats_in_row_groups(cs.M(), cs.K, (size_t)pl.scratch_bytes);
}

// A recomputed convolution followed by the recomputation of its BatchNorm, in place: the statistics are the forward
// pass's, so the apply step is one multiply-add per element in the convolution's epilogue (bn_affine.hpp: the bits
// bn_apply would write), and the convolution's raw output, which the in-place BatchNorm overwrites anyway, never
// reaches memory.
bool conv_applies_bn(const Plan &pl, const Launch &L1, const Launch &L2) {
    const Graph &g = pl.g;
    if (L1.kind != EV_RUN_RECOMPUTE || L2.kind != EV_RUN_RECOMPUTE) return false;
    const Node &cv = g.nodes[L1.id], &bn = g.nodes[L2.id];
    if ((cv.op != "conv" && cv.op != "dwconv") || bn.op != "bn" || bn.ins[0] != cv.id) return false;
    if (!(L2.flags & 1) || L2.a[2].region != L1.a[2].region || L2.a[2].off != L1.a[2].off) return false;
    const ConvShape cs = conv_shape(g, cv);
    if (cv.op == "dwconv") return dwconv_fwd_takes_affine(cs);
    const FwdImpl &im = cv.fimpls[L1.impl];
    if (im.algo == "im2col") return false;
    if (winograd_is_fused(im.algo)) return winograd_fused_applies(cs, false);
    if (winograd_tile(im.algo)) return winograd_applies(cs, false);
    return conv_fwd_aligned(cs) && cs.K % 4 == 0 && splits_of(im.algo, im.extra) == 1;
}

// ... and the ReLU (ReLU6) behind that BatchNorm: the clamp is one more operation on the value the epilogue holds.  In
// place it replaces the BatchNorm's output; out of place (the BatchNorm's output is kept for its own backward operator) it
// is written to the ReLU's buffer beside it, which saves reading the tensor again and a launch.  A recomputed ReLU that
// writes its sign mask again (the mask was not kept from the forward pass) rides along where the kernel can assemble the
// mask words; elsewhere it stays a launch of its own behind the fused pair.
bool conv_applies_bn_relu(const Plan &pl, const Launch &L1, const Launch &L2, const Launch &L3) {
    if (!conv_applies_bn(pl, L1, L2) || L3.kind != EV_RUN_RECOMPUTE) return false;
    const Graph &g = pl.g;
    const Node &bn = g.nodes[L2.id], &re = g.nodes[L3.id];
    if ((re.op != "relu" && re.op != "relu6") || re.ins[0] != bn.id) return false;
    const Node &cv = g.nodes[L1.id];
    const FwdImpl &im = cv.fimpls[L1.impl];
    // What the fused launch writes beside the BatchNorm's output must not lie on anything it still reads (the convolution's
    // input and workspace are read until the last tile is done, and the arena may have handed out a block freed before it)
    auto clear_of = [&](const Ref &w, int64_t wbytes) {
        if (w.region != R_ARENA) return false;
        const int64_t lo = w.off, hi = lo + wbytes;
        auto clear = [&](const Ref &r, int64_t bytes) { return r.region != R_ARENA || r.off + bytes <= lo || r.off >= hi; };
        return clear(L1.a[0], 4 * numel_of(g.shape_of(cv.ins[0]))) && clear(L1.a[2], 4 * numel_of(cv.shape)) &&
               clear(L1.a[4], im.ws > 0 ? align_up(im.ws) : 0);
    };
    if (L3.flags & 2) {
        // the sign code comes from the epilogue too where the kernel can write it: the implicit GEMM and the one-kernel
        // Winograd form, 64 | K (a word of the code is 64 channels of one position)
        if (cv.op != "conv" || (winograd_tile(im.algo) && !winograd_is_fused(im.algo))) return false;
        if (!conv_epilogue_writes_mask(conv_shape(g, cv), winograd_is_fused(im.algo))) return false;
        if (!clear_of(L3.a[3], (numel_of(re.shape) + 63) / 64 * 8)) return false;
    }
    const bool same = L3.a[2].region == L2.a[2].region && L3.a[2].off == L2.a[2].off;
    if (L3.flags & 1) return same;                                                         // in place: over the BatchNorm's output
    if (same) return false;
    return clear_of(L3.a[2], 4 * numel_of(re.shape));
}

void build_programs(monet_plan *p) {
    const Plan &pl = p->plan;
    const size_t n = pl.launches.size();
    p->feeds_stats.assign(n, 0);
    p->stats_fed.assign(n, 0);
    for (size_t i = 0; i + 1 < n; ++i)
        if (conv_feeds_bn_stats(pl, pl.launches[i], pl.launches[i + 1])) p->feeds_stats[i] = p->stats_fed[i + 1] = 1;
    for (size_t i = 0; i < n; ++i) p->prog_plain.push_back(ProgStep{FUSE_NONE, i, i, i});
    for (size_t i = 0; i < n; ++i) {
        if (i + 2 < n) {
            if (triple_fwd(pl, pl.launches[i], pl.launches[i + 1], pl.launches[i + 2]) >= 0) {
                p->prog_fused.push_back(ProgStep{FUSE_BN_ADD_RELU_FWD, i, i + 1, i + 2});
                i += 2;
                continue;
            }
            if (triple_bwd(pl, pl.launches[i], pl.launches[i + 1], pl.launches[i + 2]) >= 0) {
                p->prog_fused.push_back(ProgStep{FUSE_RELU_ADD_BN_BWD, i, i + 1, i + 2});
                i += 2;
                continue;
            }
        }
        if (i + 2 < n && conv_applies_bn_relu(pl, pl.launches[i], pl.launches[i + 1], pl.launches[i + 2])) {
            p->prog_fused.push_back(ProgStep{FUSE_CONV_BN_RELU, i, i + 1, i + 2});
            i += 2;
            continue;
        }
        if (i + 1 < n && conv_applies_bn(pl, pl.launches[i], pl.launches[i + 1])) {
            p->prog_fused.push_back(ProgStep{FUSE_CONV_BN_APPLY, i, i + 1, i + 1});
            ++i;
            continue;
        }
        int f = i + 1 < n ? fusable(pl, pl.launches[i], pl.launches[i + 1]) : FUSE_NONE;
        if (f) { p->prog_fused.push_back(ProgStep{f, i, i + 1, i + 1}); ++i; }
        else p->prog_fused.push_back(ProgStep{FUSE_NONE, i, i, i});
    }
}

void run_fused(const StepCtx &c, const ProgStep &ps) {
    const Graph &g = c.mp->plan.g;
    const Plan &pl = c.mp->plan;
    const Launch &L1 = c.mp->plan.launches[ps.a], &L2 = c.mp->plan.launches[ps.b];
    if (ps.fuse == FUSE_CONV_BN_APPLY || ps.fuse == FUSE_CONV_BN_RELU) {
        const Node &bn = g.nodes[L2.id];
        BnAffine affine{c.weights[bn.pars[0]], c.weights[bn.pars[1]], c.bn_stats(L2.id)};
        if (ps.fuse == FUSE_CONV_BN_RELU) {
            const Launch &L3 = pl.launches[ps.c];
            affine.relu = g.nodes[L3.id].op == "relu6" ? 2 : 1;
            affine.relu_out = (L3.flags & 1) ? nullptr : (float *)c.ptr(L3.a[2]);
            affine.mask = (L3.flags & 2) ? (unsigned long long *)c.ptr(L3.a[3]) : nullptr;
        }
        run_forward(c, L1, &affine);
        return;
    }
    if (ps.fuse == FUSE_BN_ADD_RELU_FWD) {
        const Launch &L3 = pl.launches[ps.c];
        const Node &bn = g.nodes[L1.id], &ad = g.nodes[L2.id], &re = g.nodes[L3.id];
        const int pos = ad.ins[0] == bn.id ? 0 : 1;
        const float *x = (const float *)c.ptr(L1.a[0]);
        const float *other = (const float *)c.ptr(L2.a[1 - pos]);
        // tensors between the operators are written only if something later still reads them
        float *out_bn = freed_between(pl, bn.id, L2.event, L3.event) ? nullptr : (float *)c.ptr(L1.a[2]);
        float *out_pre = (L3.flags & 1) ? nullptr : (float *)c.ptr(L2.a[2]);
        float *out = (float *)c.ptr(L3.a[2]);
        uint64_t *mask = (L3.flags & 2) ? (uint64_t *)c.ptr(L3.a[3]) : nullptr;
        const int64_t n = numel_of(re.shape);
        const int C = (int)bn.shape.back();
        float *stats = c.bn_stats(L1.id);
        if (L1.kind == EV_RUN_FWD)
            bn_stats(c.st, x, stats, n / C, C, (float)bn.attr_f("eps", 1e-5), c.scratch(), c.scratch_bytes(), c.stats_fed(L1));
        fwd_chain(c.st, x, other, c.weights[bn.pars[0]], c.weights[bn.pars[1]], stats, C, out_bn, out_pre, out, mask, n, re.op == "relu6");
        return;
    }
    if (ps.fuse == FUSE_RELU_ADD_BN_BWD) {
        const Launch &L3 = pl.launches[ps.c];
        const Bop &b1 = g.bops[L1.id], &b2 = g.bops[L2.id], &b3 = g.bops[L3.id];
        const Node &re = g.nodes[b1.node], &ad = g.nodes[b2.node], &bn = g.nodes[b3.node];
        const int pos = ad.ins[0] == bn.id ? 0 : 1, oth = 1 - pos;
        const std::string &algo = b1.impls[L1.impl].algo;
        const int mode = algo == "from_input" ? RELU_FROM_INPUT : (algo == "from_output" ? RELU_FROM_OUTPUT : RELU_FROM_MASK);
        float *side = ad.ins[oth] > 0 ? (float *)c.ptr(L2.a[2 + oth]) : nullptr;
        const int C = (int)bn.shape.back();
        bn_bwd(c.st, (const float *)c.ptr(L1.a[0]), (const float *)c.ptr(L3.a[1]), b3.impls[L3.impl].algo == "from_output",
               c.weights[bn.pars[0]], c.weights[bn.pars[1]], c.bn_stats(b3.node), (float *)c.ptr(L3.a[2]), c.grads[bn.pars[0]],
               c.grads[bn.pars[1]], numel_of(re.shape) / C, C, (L3.flags & 1) != 0, c.scratch(), c.scratch_bytes(), c.ptr(L1.a[1]), mode,
               b1.kind == "relu6_bwd", side, ((L2.flags >> oth) & 1) != 0);
        return;
    }
    if (ps.fuse == FUSE_BN_RELU_FWD || ps.fuse == FUSE_ADD_RELU_FWD) {
        const Node &n1 = g.nodes[L1.id], &n2 = g.nodes[L2.id];
        const float *x = (const float *)c.ptr(L1.a[0]);
        const bool relu_inplace = L2.flags & 1;
        float *pre = relu_inplace ? nullptr : (float *)c.ptr(L1.a[2]);   // the tensor between the two is only written if it survives
        float *out = (float *)c.ptr(L2.a[2]);
        uint64_t *mask = (L2.flags & 2) ? (uint64_t *)c.ptr(L2.a[3]) : nullptr;
        const int64_t n = numel_of(n2.shape);
        const bool six = n2.op == "relu6";
        if (ps.fuse == FUSE_BN_RELU_FWD) {
            const int C = (int)n1.shape.back();
            float *stats = c.bn_stats(L1.id);
            if (L1.kind == EV_RUN_FWD)
                bn_stats(c.st, x, stats, n / C, C, (float)n1.attr_f("eps", 1e-5), c.scratch(), c.scratch_bytes(), c.stats_fed(L1));
            fwd_chain(c.st, x, nullptr, c.weights[n1.pars[0]], c.weights[n1.pars[1]], stats, C, nullptr, pre, out, mask, n, six);
        } else {
            fwd_chain(c.st, x, (const float *)c.ptr(L1.a[1]), nullptr, nullptr, nullptr, 0, nullptr, pre, out, mask, n, six);
        }
        return;
    }
    const Bop &b1 = g.bops[L1.id], &b2 = g.bops[L2.id];
    const Node &r = g.nodes[b1.node];
    const std::string &algo = b1.impls[L1.impl].algo;
    const float *dz = (const float *)c.ptr(L1.a[0]);
    const void *t = c.ptr(L1.a[1]);
    const int64_t n = numel_of(r.shape);
    const bool six = b1.kind == "relu6_bwd";
    if (ps.fuse == FUSE_RELU_BN_BWD) {
        const Node &bn = g.nodes[b2.node];
        const int C = (int)bn.shape.back();
        bn_bwd(c.st, dz, (const float *)c.ptr(L2.a[1]), b2.impls[L2.impl].algo == "from_output", c.weights[bn.pars[0]], c.weights[bn.pars[1]],
               c.bn_stats(b2.node), (float *)c.ptr(L2.a[2]), c.grads[bn.pars[0]], c.grads[bn.pars[1]], n / C, C, (L2.flags & 1) != 0, c.scratch(),
               c.scratch_bytes(), t, RELU_FROM_MASK, six);
    } else {
        const Node &ad = g.nodes[b2.node];
        int mode = algo == "from_input" ? RELU_FROM_INPUT : (algo == "from_output" ? RELU_FROM_OUTPUT : RELU_FROM_MASK);
        float *d0 = ad.ins[0] > 0 ? (float *)c.ptr(L2.a[2]) : nullptr;
        float *d1 = ad.ins.size() > 1 && ad.ins[1] > 0 ? (float *)c.ptr(L2.a[3]) : nullptr;
        relu_bwd_fanout(c.st, dz, t, mode, d0, (L2.flags & 1) != 0, d1, (L2.flags & 2) != 0, n, six);
    }
}

}  // namespace

extern "C" int monet_plan_set_fusion(monet_plan *p, int on) {
    if (!p) return MONET_BAD_ARGUMENT;
    p->fusion = on != 0;
    return MONET_OK;
}

extern "C" int64_t monet_step(monet_plan *p, void *hip_stream, const void *const *inputs, const float *const *weights,
                              float *const *grads, float *dev_loss) {
    if (!p || !inputs || !weights || !grads) { g_err = "monet_step: null argument"; return MONET_BAD_ARGUMENT; }
    if (!p->base) { g_err = "monet_step: no arena bound"; return MONET_ARENA_TOO_SMALL; }
    int64_t peak = 0;
    int rc = guarded([&] {
        const Plan &pl = p->plan;
        StepCtx c{p, (hipStream_t)hip_stream, inputs, weights, grads};
        // arrival counts of cut convolution tiles start at zero whatever an earlier, failed step left behind
        conv_reset_arrivals(c.st);
        // arena accounting: replay the trace's alloc/free records against the launches
        int64_t live = 0;
        size_t next_event = 0, next_poison = 0;
        if (p->timing && p->ev.size() != 2 * pl.launches.size()) {     // enough for either program
            p->ev.resize(2 * pl.launches.size());
            for (auto &e : p->ev) hip_check(hipEventCreate(&e), "event create");
        }
        // Debug modes (poison fill, early stop) run the operators one by one; otherwise adjacent
        // bandwidth-bound operators go out as one fused kernel (same arithmetic, same trace).
        const bool fuse = p->fusion && !p->poison && p->stop_after < 0;
        const std::vector<ProgStep> &prog = fuse ? p->prog_fused : p->prog_plain;
        for (size_t si = 0; si < prog.size(); ++si) {
            const ProgStep &ps = prog[si];
            const Launch &Llast = pl.launches[ps.last()];
            if (p->stop_after >= 0 && (int64_t)Llast.event > p->stop_after) break;
            for (; next_event <= Llast.event; ++next_event) {
                const monet_event &e = pl.events[next_event];
                if (e.kind == EV_ALLOC) live += e.bytes;
                else if (e.kind == EV_FREE) live -= e.bytes;
                if (live != e.live_after) throw KernelError("arena accounting diverged from the plan");
                peak = std::max(peak, live);
            }
            if (p->poison)
                for (; next_poison < pl.poison.size() && pl.poison[next_poison].before_launch <= ps.a; ++next_poison)
                    fill_u32(c.st, (uint32_t *)(c.arena() + pl.poison[next_poison].off), pl.poison[next_poison].bytes / 4, 0x7fc00000u);
            if (p->timing) hip_check(hipEventRecord(p->ev[2 * si], c.st), "event record");
            const Launch &L = pl.launches[ps.a];
            if (ps.fuse) run_fused(c, ps);
            else if (L.kind == EV_RUN_BWD) run_backward(c, L);
            else run_forward(c, L);
            if (p->timing) hip_check(hipEventRecord(p->ev[2 * si + 1], c.st), "event record");
        }
        p->timed_fused = fuse;
        p->timed_step_done = p->timing;
        if (p->stop_after < 0) {
            for (; next_event < pl.events.size(); ++next_event) {
                const monet_event &e = pl.events[next_event];
                if (e.kind == EV_ALLOC) live += e.bytes;
                else if (e.kind == EV_FREE) live -= e.bytes;
                peak = std::max(peak, live);
            }
            if (live != 0) throw KernelError("arena not empty at the end of the step");
        }
        if (dev_loss)
            hip_check(hipMemcpyAsync(dev_loss, p->base + pl.loss_off, 4, hipMemcpyDeviceToDevice, c.st), "loss copy");
    });
    return rc == MONET_OK ? peak : rc;
}

// ------------------------------------------------------------------ measurement aids
static const std::vector<ProgStep> &current_program(const monet_plan *p) {
    return (p->fusion && !p->poison && p->stop_after < 0) ? p->prog_fused : p->prog_plain;
}

extern "C" int monet_plan_num_launches(const monet_plan *p) { return p ? (int)current_program(p).size() : MONET_BAD_ARGUMENT; }

// flop a convolution implementation issues: the algorithmic count, or for Winograd F(m x m, 3x3) the (m+2)^2 GEMMs over the tiles
static double issued_conv_flops(const ConvShape &cs, const std::string &algo) {
    const int m = winograd_tile(algo);
    if (!m) return 2.0 * (double)cs.M() * cs.K * (double)cs.RSC();
    const double tiles = (double)cs.N * ((cs.H + m - 1) / m) * ((cs.W + m - 1) / m);
    return 2.0 * (m + 2) * (m + 2) * tiles * cs.K * cs.C;
}

extern "C" int monet_plan_launch_info(const monet_plan *p, size_t index, monet_launch_info *out) {
    if (!p || !out || index >= current_program(p).size()) { g_err = "monet_plan_launch_info: bad argument"; return MONET_BAD_ARGUMENT; }
    const Graph &g = p->plan.g;
    const ProgStep &ps = current_program(p)[index];
    const Launch &L = p->plan.launches[ps.a];
    std::memset(out, 0, sizeof(*out));
    if (ps.fuse) {
        const Launch &L2 = p->plan.launches[ps.b];
        out->kind = L.kind; out->id = L.id; out->impl = L.impl; out->flags = L.flags;
        double e, bytes;
        const char *label;
        if (ps.fuse == FUSE_CONV_BN_APPLY || ps.fuse == FUSE_CONV_BN_RELU) {
            const ConvShape cs = conv_shape(g, g.nodes[L.id]);
            if (g.nodes[L.id].op == "dwconv") {
                bytes = 4.0 * cs.N * cs.H * cs.W * cs.C + 4.0 * (double)cs.M() * cs.K;
                label = "dwconv_fwd";
            } else {
                out->flops = 2.0 * (double)cs.M() * cs.K * (double)cs.RSC();
                out->issued_flops = issued_conv_flops(cs, g.nodes[L.id].fimpls[L.impl].algo);
                bytes = 4.0 * cs.N * cs.H * cs.W * cs.C + 4.0 * cs.K * (double)cs.RSC() + 4.0 * (double)cs.M() * cs.K;
                label = winograd_tile(g.nodes[L.id].fimpls[L.impl].algo) ? "conv_fwd_winograd" : "conv_fwd";
            }
            if (ps.fuse == FUSE_CONV_BN_RELU) {      // the ReLU's result beside the BatchNorm's, its sign mask
                const Launch &L3 = p->plan.launches[ps.c];
                if (!(L3.flags & 1)) bytes += 4.0 * (double)cs.M() * cs.K;
                if (L3.flags & 2) bytes += (double)cs.M() * cs.K / 8.0;
            }
        } else if (ps.fuse == FUSE_BN_ADD_RELU_FWD) {
            const Launch &L3 = p->plan.launches[ps.c];
            e = 4.0 * (double)numel_of(g.nodes[L3.id].shape);
            const bool keep_bn = !freed_between(p->plan, L.id, L2.event, L3.event), pre = !(L3.flags & 1), mk = L3.flags & 2;
            // + the statistics pass, unless the convolution before it already left the partial results
            bytes = 2 * e + (keep_bn ? e : 0) + (pre ? e : 0) + e + (mk ? e / 32 : 0) + (L.kind == EV_RUN_FWD && !p->stats_fed[ps.a] ? e : 0);
            label = L.kind == EV_RUN_FWD ? "bn_add_relu_fwd" : "bn_add_relu_apply";
        } else if (ps.fuse == FUSE_RELU_ADD_BN_BWD) {
            const Launch &L3 = p->plan.launches[ps.c];
            const Bop &b1 = g.bops[L.id];
            const Node &ad = g.nodes[g.bops[L2.id].node];
            const int pos = ad.ins[0] == g.bops[L3.id].node ? 0 : 1, oth = 1 - pos;
            e = 4.0 * (double)numel_of(g.nodes[b1.node].shape);
            const double t = b1.impls[L.impl].algo == "from_mask" ? e / 32 : e;
            bytes = 2 * (e + t + e) + e + ((L3.flags & 1) ? e : 0);                 // two passes over dz, gate, bn tensor; dx
            if (ad.ins[oth] > 0) bytes += e + (((L2.flags >> oth) & 1) ? e : 0);    // the other branch's gradient
            label = "relu_add_bn_bwd";
        } else if (ps.fuse == FUSE_BN_RELU_FWD || ps.fuse == FUSE_ADD_RELU_FWD) {
            e = 4.0 * (double)numel_of(g.nodes[L2.id].shape);
            const bool pre = !(L2.flags & 1), mk = L2.flags & 2;
            bytes = (ps.fuse == FUSE_ADD_RELU_FWD ? 2 : 1) * e + (pre ? e : 0) + e + (mk ? e / 32 : 0);
            if (ps.fuse == FUSE_BN_RELU_FWD && L.kind == EV_RUN_FWD && !p->stats_fed[ps.a]) bytes += e;        // statistics pass
            label = ps.fuse == FUSE_ADD_RELU_FWD ? "add_relu_fwd" : (L.kind == EV_RUN_FWD ? "bn_relu_fwd" : "bn_relu_apply");
        } else {
            const Bop &b1 = g.bops[L.id];
            e = 4.0 * (double)numel_of(g.nodes[b1.node].shape);
            const double t = b1.impls[L.impl].algo == "from_mask" ? e / 32 : e;
            if (ps.fuse == FUSE_RELU_BN_BWD) { bytes = 2 * (e + t + e) + e + ((L2.flags & 1) ? e : 0); label = "relu_bn_bwd"; }
            else {
                const Node &ad = g.nodes[g.bops[L2.id].node];
                bytes = e + t;
                for (size_t q = 0; q < ad.ins.size() && q < 2; ++q)
                    if (ad.ins[q] > 0) bytes += e + (((L2.flags >> q) & 1) ? e : 0);
                label = "relu_add_bwd";
            }
        }
        out->bytes = bytes;
        std::strncpy(out->label, label, sizeof(out->label) - 1);
        return MONET_OK;
    }
    out->kind = L.kind; out->id = L.id; out->impl = L.impl; out->flags = L.flags;
    std::string label;
    double flops = 0, bytes = 0, issued = -1;
    auto conv_cost = [&](const ConvShape &cs, const char *which) {
        flops = 2.0 * (double)cs.M() * cs.K * (double)cs.RSC();
        double x = 4.0 * cs.N * cs.H * cs.W * cs.C, w = 4.0 * cs.K * (double)cs.RSC(), y = 4.0 * (double)cs.M() * cs.K;
        bytes = x + w + y;
        label = which;
    };
    if (L.kind == EV_RUN_BWD) {
        const Bop &b = g.bops[L.id];
        const Node &n = g.nodes[b.node];
        double e = 4.0 * (double)numel_of(n.shape);
        label = b.kind;
        if (b.kind == "conv_wgrad" || b.kind == "conv_dgrad") {
            // the Winograd forms (transform kernels + batched GEMMs) are classes of their own
            conv_cost(conv_shape(g, n), (b.kind + (winograd_tile(b.impls[L.impl].algo) ? "_winograd" : "")).c_str());
            issued = issued_conv_flops(conv_shape(g, n), b.impls[L.impl].algo);
        }
        else if (b.kind == "tconv_wgrad") conv_cost(tconv_adjoint_shape(g, n), "tconv_wgrad");
        else if (b.kind == "tconv_dgrad") conv_cost(tconv_adjoint_shape(g, n), "tconv_dgrad");
        else if (b.kind == "linear_wgrad") conv_cost(linear_shape(g, n), "linear_wgrad");
        else if (b.kind == "linear_dgrad") conv_cost(linear_shape(g, n), "linear_dgrad");
        else if (b.kind == "bn_bwd") bytes = 5 * e;                      // reduce pass reads dy,t; apply pass reads dy,t, writes dx
        else if (b.kind == "relu_bwd" || b.kind == "relu6_bwd")
            bytes = (b.impls[L.impl].algo == "from_mask" ? 2.0 + 1.0 / 32 : 3.0) * e;
        else if (b.kind == "maxpool_bwd") {
            double in = 4.0 * (double)numel_of(g.shape_of(n.ins[0]));
            bytes = in + (b.impls[L.impl].algo == "from_index" ? 1.25 * e : e + in);
        } else if (b.kind == "add_bwd") bytes = 4 * e;
        else if (b.kind == "concat_bwd") bytes = 2 * e;
        else if (b.kind == "dwconv_dgrad" || b.kind == "dwconv_wgrad") bytes = 4.0 * (double)numel_of(g.shape_of(n.ins[0])) + e;
        else if (b.kind == "avgpool_bwd") bytes = 4.0 * (double)numel_of(g.shape_of(n.ins[0])) + e;
        else bytes = 2.0 * 4.0 * (double)numel_of(g.shape_of(n.ins[0]));
        if ((b.kind == "relu_bwd" || b.kind == "relu6_bwd" || b.kind == "bn_bwd" || b.kind == "conv_dgrad") && (L.flags & 1)) bytes += e;
    } else {
        const Node &n = g.nodes[L.id];
        double e = 4.0 * (double)numel_of(n.shape);
        label = n.op + "_fwd";
        if (n.op == "conv") {
            conv_cost(conv_shape(g, n), winograd_tile(n.fimpls[L.impl].algo) ? "conv_fwd_winograd" : "conv_fwd");
            issued = issued_conv_flops(conv_shape(g, n), n.fimpls[L.impl].algo);
        } else if (n.op == "tconv") conv_cost(tconv_adjoint_shape(g, n), "tconv_fwd");
        else if (n.op == "concat") bytes = 2 * e;
        else if (n.op == "linear") conv_cost(linear_shape(g, n), "linear_fwd");
        else if (n.op == "bn") {
            if (L.kind == EV_RUN_FWD) bytes = (p->stats_fed[ps.a] ? 2 : 3) * e;   // statistics pass (unless fed by the convolution) + apply pass
            else { bytes = 2 * e; label = "bn_apply"; }                  // recomputation reuses the statistics
        } else if (n.op == "relu" || n.op == "relu6") bytes = (2.0 + ((L.flags & 2) ? 1.0 / 32 : 0.0)) * e;
        else if (n.op == "maxpool") bytes = 4.0 * (double)numel_of(g.shape_of(n.ins[0])) + e * ((L.flags & 2) ? 1.25 : 1.0);
        else if (n.op == "add") bytes = 3 * e;
        else bytes = 4.0 * (double)numel_of(g.shape_of(n.ins[0])) + e;
    }
    out->flops = flops;
    out->issued_flops = issued < 0 ? flops : issued;
    out->bytes = bytes;
    std::strncpy(out->label, label.c_str(), sizeof(out->label) - 1);
    return MONET_OK;
}

extern "C" int monet_plan_set_timing(monet_plan *p, int on) {
    if (!p) return MONET_BAD_ARGUMENT;
    p->timing = on != 0;
    p->timed_step_done = false;
    return MONET_OK;
}

extern "C" int monet_plan_read_timing(monet_plan *p, float *ms, size_t n) {
    if (!p || !ms) { g_err = "monet_plan_read_timing: null argument"; return MONET_BAD_ARGUMENT; }
    if (!p->timed_step_done || n != (p->timed_fused ? p->prog_fused : p->prog_plain).size() || p->ev.size() < 2 * n || n == 0) {
        g_err = "monet_plan_read_timing: no timed step to read";
        return MONET_BAD_ARGUMENT;
    }
    return guarded([&] {
        hip_check(hipEventSynchronize(p->ev[2 * n - 1]), "event synchronize");
        for (size_t i = 0; i < n; ++i) hip_check(hipEventElapsedTime(&ms[i], p->ev[2 * i], p->ev[2 * i + 1]), "event elapsed");
    });
}

// ------------------------------------------------------------------ linear layer = 1x1 convolution + bias
namespace monet {

void linear_bias_add(hipStream_t st, float *y, const float *b, int N, int out);
void linear_bias_grad(hipStream_t st, const float *dy, float *db, int N, int out);

// A batch of a few hundred rows gives a handful of output tiles: the reduction is cut into ranges (partial
// results in the caller's scratch, added in range order) until about a thousand workgroups exist.
static int linear_splits(int64_t rows, int64_t cols, int64_t reduction, int64_t out_elems, size_t scratch_bytes) {
    int64_t tiles = ((rows + 127) / 128) * ((cols + 127) / 128);
    int64_t sp = std::min<int64_t>({1024 / tiles, reduction / 128, (int64_t)(scratch_bytes / (4 * out_elems)), (int64_t)64});
    return (int)std::max<int64_t>(1, sp);
}

void linear_fwd(hipStream_t st, const float *x, const float *w, const float *b, float *y, int N, int in, int out, float *scratch,
                size_t scratch_bytes) {
    ConvShape cs{N, 1, 1, in, out, 1, 1, 1, 0, 1, 1};
    const int sp = scratch ? linear_splits(N, out, in, (int64_t)N * out, scratch_bytes) : 1;
    conv_fwd(st, x, w, y, cs, sp, sp > 1 ? scratch : nullptr, sp > 1 ? scratch_bytes : 0);
    linear_bias_add(st, y, b, N, out);
}
void linear_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, float *db, int N, int in, int out) {
    ConvShape cs{N, 1, 1, in, out, 1, 1, 1, 0, 1, 1};
    conv_wgrad(st, x, dy, dw, cs, 1, nullptr, 0);
    linear_bias_grad(st, dy, db, N, out);
}
void linear_dgrad(hipStream_t st, const float *dy, const float *w, float *dx, int N, int in, int out, bool accumulate, float *scratch,
                  size_t scratch_bytes) {
    ConvShape cs{N, 1, 1, in, out, 1, 1, 1, 0, 1, 1};
    const int sp = scratch ? linear_splits(N, in, out, (int64_t)N * in, scratch_bytes) : 1;
    conv_dgrad(st, dy, w, dx, cs, accumulate, sp, sp > 1 ? scratch : nullptr, sp > 1 ? scratch_bytes : 0);
}

}  // namespace monet

// ------------------------------------------------------------------ per-kernel entry points
static ConvShape mk_conv(int N, int H, int W, int C, int K, int R, int S, int stride, int pad) {
    ConvShape cs{N, H, W, C, K, R, S, stride, pad, 0, 0};
    if (stride > 0) {
        cs.P = (H + 2 * pad - R) / stride + 1;
        cs.Q = (W + 2 * pad - S) / stride + 1;
    }
    return cs;
}
static PoolShape mk_pool(int N, int H, int W, int C, int k, int stride, int pad) {
    PoolShape ps{N, H, W, C, k, stride, pad, 0, 0};
    if (stride > 0) {
        ps.P = (H + 2 * pad - k) / stride + 1;
        ps.Q = (W + 2 * pad - k) / stride + 1;
    }
    return ps;
}

extern "C" int monet_conv_fwd(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int C, int K, int R, int S,
                              int stride, int pad, int splits, float *ws, size_t ws_bytes) {
    return guarded([&] { conv_fwd((hipStream_t)stream, x, w, y, mk_conv(N, H, W, C, K, R, S, stride, pad), splits, ws, ws_bytes); });
}
extern "C" int monet_conv_reset_arrivals(void *stream) {
    return guarded([&] { conv_reset_arrivals((hipStream_t)stream); });
}
extern "C" int monet_conv_fwd_bn_stats(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int C, int K, int R, int S,
                                       int stride, int pad, float *ws, size_t ws_bytes, float *stats, float eps, float *scratch,
                                       size_t scratch_bytes) {
    return guarded([&] {
        const ConvShape cs = mk_conv(N, H, W, C, K, R, S, stride, pad);
        if (!bn_stats_in_row_groups(cs.M(), cs.K, scratch_bytes))
            throw KernelError("monet_conv_fwd_bn_stats: scratch too small for 2 floats per 64 output rows and channel");
        conv_fwd((hipStream_t)stream, x, w, y, cs, 1, ws, ws_bytes, false, scratch);
        bn_stats((hipStream_t)stream, y, stats, cs.M(), cs.K, eps, scratch, scratch_bytes, true);
    });
}
extern "C" int monet_conv_fwd_bn_apply(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int C, int K, int R, int S,
                                       int stride, int pad, int winograd_m, float *ws, size_t ws_bytes, const float *gamma, const float *beta,
                                       const float *stats) {
    return guarded([&] {
        const ConvShape cs = mk_conv(N, H, W, C, K, R, S, stride, pad);
        const BnAffine affine{gamma, beta, stats};
        if (winograd_m == 5) conv_winograd_fused((hipStream_t)stream, x, w, y, cs, false, false, ws, ws_bytes, &affine);
        else if (winograd_m) conv_winograd((hipStream_t)stream, x, w, y, cs, winograd_m, false, false, ws, ws_bytes, &affine);
        else conv_fwd((hipStream_t)stream, x, w, y, cs, 1, ws, ws_bytes, false, nullptr, &affine);
    });
}
extern "C" int monet_conv_fwd_bn_relu(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int C, int K, int R, int S,
                                      int stride, int pad, int winograd_m, float *ws, size_t ws_bytes, const float *gamma, const float *beta,
                                      const float *stats, int six, float *relu_out, uint64_t *mask) {
    return guarded([&] {
        const ConvShape cs = mk_conv(N, H, W, C, K, R, S, stride, pad);
        BnAffine affine{gamma, beta, stats};
        affine.relu = six ? 2 : 1;
        affine.relu_out = relu_out;
        affine.mask = (unsigned long long *)mask;
        if (winograd_m == 5) conv_winograd_fused((hipStream_t)stream, x, w, y, cs, false, false, ws, ws_bytes, &affine);
        else if (winograd_m) conv_winograd((hipStream_t)stream, x, w, y, cs, winograd_m, false, false, ws, ws_bytes, &affine);
        else conv_fwd((hipStream_t)stream, x, w, y, cs, 1, ws, ws_bytes, false, nullptr, &affine);
    });
}
extern "C" int monet_conv_winograd(void *stream, const float *in, const float *w, float *out, int N, int H, int W, int C, int K,
                                   int m, int adjoint, int accumulate, float *ws, size_t ws_bytes) {
    return guarded([&] {
        conv_winograd((hipStream_t)stream, in, w, out, mk_conv(N, H, W, C, K, 3, 3, 1, 1), m, adjoint != 0, accumulate != 0, ws, ws_bytes);
    });
}
extern "C" int monet_conv_winograd_fused(void *stream, const float *in, const float *w, float *out, int N, int H, int W, int C, int K,
                                         int adjoint, int accumulate, float *ws, size_t ws_bytes) {
    return guarded([&] {
        conv_winograd_fused((hipStream_t)stream, in, w, out, mk_conv(N, H, W, C, K, 3, 3, 1, 1), adjoint != 0, accumulate != 0, ws, ws_bytes);
    });
}
extern "C" int64_t monet_conv_winograd_fused_workspace_bytes(int N, int H, int W, int C, int K, int adjoint) {
    int64_t bytes = -1;
    int rc = guarded([&] { bytes = (int64_t)winograd_fused_workspace_bytes(mk_conv(N, H, W, C, K, 3, 3, 1, 1), adjoint != 0); });
    return rc == MONET_OK ? bytes : (int64_t)rc;
}
extern "C" int monet_conv_winograd_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int C, int K,
                                         int m, float *ws, size_t ws_bytes) {
    return guarded([&] { conv_winograd_wgrad((hipStream_t)stream, x, dy, dw, mk_conv(N, H, W, C, K, 3, 3, 1, 1), m, ws, ws_bytes); });
}
extern "C" int64_t monet_conv_winograd_wgrad_workspace_bytes(int N, int H, int W, int C, int K, int m) {
    int64_t bytes = -1;
    int rc = guarded([&] { bytes = (int64_t)winograd_wgrad_workspace_bytes(mk_conv(N, H, W, C, K, 3, 3, 1, 1), m); });
    return rc == MONET_OK ? bytes : (int64_t)rc;
}
extern "C" int64_t monet_conv_winograd_workspace_bytes(int N, int H, int W, int C, int K, int m) {
    int64_t bytes = -1;
    int rc = guarded([&] { bytes = (int64_t)winograd_workspace_bytes(mk_conv(N, H, W, C, K, 3, 3, 1, 1), m); });
    return rc == MONET_OK ? bytes : (int64_t)rc;
}
extern "C" int64_t monet_conv_workspace_bytes(int which, int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int splits) {
    int64_t bytes = -1;
    int rc = guarded([&] {
        if (which != 0 && which != 1) throw KernelError("monet_conv_workspace_bytes: which must be 0 (forward) or 1 (input gradient)");
        if (splits < 1) throw KernelError("monet_conv_workspace_bytes: splits must be >= 1");
        bytes = (int64_t)conv_workspace_bytes(which, mk_conv(N, H, W, C, K, R, S, stride, pad), splits);
    });
    return rc == MONET_OK ? bytes : (int64_t)rc;
}
extern "C" int monet_conv_dgrad(void *stream, const float *dy, const float *w, float *dx, int N, int H, int W, int C, int K, int R, int S,
                                int stride, int pad, int accumulate, int splits, float *ws, size_t ws_bytes) {
    return guarded([&] {
        conv_dgrad((hipStream_t)stream, dy, w, dx, mk_conv(N, H, W, C, K, R, S, stride, pad), accumulate != 0, splits, ws, ws_bytes);
    });
}
extern "C" int monet_conv_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int C, int K, int R, int S,
                                int stride, int pad, int splits, float *ws, size_t ws_bytes) {
    return guarded([&] { conv_wgrad((hipStream_t)stream, x, dy, dw, mk_conv(N, H, W, C, K, R, S, stride, pad), splits, ws, ws_bytes); });
}
extern "C" int monet_bn_stats(void *stream, const float *x, float *stats, int64_t rows, int C, float eps, float *scratch, size_t scratch_bytes) {
    return guarded([&] { bn_stats((hipStream_t)stream, x, stats, rows, C, eps, scratch, scratch_bytes); });
}
extern "C" int monet_bn_stats_static(void *stream, const float *x, float *stats, int64_t rows, int C, float eps) {
    return guarded([&] { bn_stats_static((hipStream_t)stream, x, stats, rows, C, eps); });
}
extern "C" int monet_bn_apply(void *stream, const float *x, float *y, const float *gamma, const float *beta, const float *stats,
                              int64_t rows, int C) {
    return guarded([&] { bn_apply((hipStream_t)stream, x, y, gamma, beta, stats, rows, C); });
}
extern "C" int monet_bn_bwd(void *stream, const float *dy, const float *t, int from_output, const float *gamma, const float *beta,
                            const float *stats, float *dx, float *dgamma, float *dbeta, int64_t rows, int C, int accumulate,
                            float *scratch, size_t scratch_bytes) {
    return guarded([&] {
        bn_bwd((hipStream_t)stream, dy, t, from_output != 0, gamma, beta, stats, dx, dgamma, dbeta, rows, C, accumulate != 0, scratch, scratch_bytes);
    });
}
extern "C" int monet_relu_fwd(void *stream, const float *x, float *y, uint64_t *mask, int64_t n, int six) {
    return guarded([&] { relu_fwd((hipStream_t)stream, x, y, mask, n, six != 0); });
}
extern "C" int monet_relu_bwd(void *stream, const float *dz, const void *t, int mode, float *dx, int64_t n, int six, int accumulate) {
    return guarded([&] { relu_bwd((hipStream_t)stream, dz, t, mode, dx, n, six != 0, accumulate != 0); });
}
extern "C" int monet_maxpool_fwd(void *stream, const float *x, float *y, uint8_t *idx, int N, int H, int W, int C, int k, int stride, int pad) {
    return guarded([&] { maxpool_fwd((hipStream_t)stream, x, y, idx, mk_pool(N, H, W, C, k, stride, pad)); });
}
extern "C" int monet_maxpool_bwd(void *stream, const float *dy, const float *x, const uint8_t *idx, float *dx, int N, int H, int W, int C,
                                 int k, int stride, int pad, int accumulate) {
    return guarded([&] { maxpool_bwd((hipStream_t)stream, dy, x, idx, dx, mk_pool(N, H, W, C, k, stride, pad), accumulate != 0); });
}
extern "C" int monet_conv_im2col_fwd(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int C, int K, int R, int S,
                                     int stride, int pad, int accumulate, float *ws, size_t ws_bytes) {
    return guarded([&] { conv_im2col_fwd((hipStream_t)stream, x, w, y, mk_conv(N, H, W, C, K, R, S, stride, pad), ws, ws_bytes, accumulate != 0); });
}
extern "C" int monet_conv_im2col_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int C, int K, int R,
                                       int S, int stride, int pad, float *ws, size_t ws_bytes) {
    return guarded([&] { conv_im2col_wgrad((hipStream_t)stream, x, dy, dw, mk_conv(N, H, W, C, K, R, S, stride, pad), ws, ws_bytes); });
}
extern "C" int64_t monet_conv_im2col_workspace_bytes(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int wgrad) {
    int64_t bytes = 0;
    int rc = guarded([&] { bytes = (int64_t)conv_im2col_workspace_bytes(mk_conv(N, H, W, C, K, R, S, stride, pad), wgrad != 0); });
    return rc == MONET_OK ? bytes : rc;
}
extern "C" int monet_conv_pointwise_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int C, int K, int splits,
                                         float *ws, size_t ws_bytes) {
    return guarded([&] { pointwise_wgrad((hipStream_t)stream, x, dy, dw, mk_conv(N, H, W, C, K, 1, 1, 1, 0), splits, ws, ws_bytes); });
}
extern "C" int monet_conv_stem_fwd(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int K, int R, int S, int stride,
                                   int pad) {
    return guarded([&] { stem_fwd((hipStream_t)stream, x, w, y, mk_conv(N, H, W, 3, K, R, S, stride, pad)); });
}
extern "C" int monet_conv_stem_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int K, int R, int S,
                                     int stride, int pad, int splits, float *ws, size_t ws_bytes) {
    return guarded([&] { stem_wgrad((hipStream_t)stream, x, dy, dw, mk_conv(N, H, W, 3, K, R, S, stride, pad), splits, ws, ws_bytes); });
}
extern "C" int monet_conv_force_tile(int cfg) {
    if (cfg < -1 || cfg > 5) { g_err = "monet_conv_force_tile: cfg must be -1..5"; return MONET_BAD_ARGUMENT; }
    conv_force_tile(cfg);
    return MONET_OK;
}
extern "C" int monet_copy(void *stream, const float *src, float *dst, int64_t n) {
    return guarded([&] { copy_or_accumulate((hipStream_t)stream, src, dst, n, false); });
}

// transposed convolution through the convolution it is the adjoint of (see tconv_adjoint_shape)
static ConvShape mk_tconv_adjoint(int N, int H, int W, int C, int K, int R, int S, int stride) {
    ConvShape cs{N, 0, 0, K, C, R, S, stride, 0, H, W};
    if (stride > 0) {
        cs.H = (H - 1) * stride + R;
        cs.W = (W - 1) * stride + S;
    }
    return cs;
}
extern "C" int monet_tconv_fwd(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int C, int K, int R, int S, int stride) {
    return guarded([&] { conv_dgrad((hipStream_t)stream, x, w, y, mk_tconv_adjoint(N, H, W, C, K, R, S, stride), false); });
}
extern "C" int monet_tconv_dgrad(void *stream, const float *dy, const float *w, float *dx, int N, int H, int W, int C, int K, int R, int S,
                                 int stride, int accumulate) {
    return guarded([&] { conv_fwd((hipStream_t)stream, dy, w, dx, mk_tconv_adjoint(N, H, W, C, K, R, S, stride), 1, nullptr, 0, accumulate != 0); });
}
extern "C" int monet_tconv_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int C, int K, int R, int S,
                                 int stride, int splits, float *ws, size_t ws_bytes) {
    return guarded([&] { conv_wgrad((hipStream_t)stream, dy, x, dw, mk_tconv_adjoint(N, H, W, C, K, R, S, stride), splits, ws, ws_bytes); });
}
extern "C" int monet_dwconv_fwd(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int C, int R, int S, int stride, int pad) {
    return guarded([&] { dwconv_fwd((hipStream_t)stream, x, w, y, mk_conv(N, H, W, C, C, R, S, stride, pad)); });
}
extern "C" int monet_dwconv_dgrad(void *stream, const float *dy, const float *w, float *dx, int N, int H, int W, int C, int R, int S, int stride,
                                  int pad, int accumulate) {
    return guarded([&] { dwconv_dgrad((hipStream_t)stream, dy, w, dx, mk_conv(N, H, W, C, C, R, S, stride, pad), accumulate != 0); });
}
extern "C" int monet_dwconv_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int C, int R, int S, int stride,
                                  int pad, float *scratch, size_t scratch_bytes) {
    return guarded([&] { dwconv_wgrad((hipStream_t)stream, x, dy, dw, mk_conv(N, H, W, C, C, R, S, stride, pad), scratch, scratch_bytes); });
}
extern "C" int monet_column_copy(void *stream, const float *src, int64_t src_ld, float *dst, int64_t dst_ld, int cols, int64_t rows, int accumulate) {
    return guarded([&] { column_copy((hipStream_t)stream, src, src_ld, dst, dst_ld, cols, rows, accumulate != 0); });
}
extern "C" int monet_softmaxce_rows_fwd(void *stream, const float *logits, const int32_t *labels, float *loss, int64_t rows, int classes,
                                        float *scratch, size_t scratch_bytes) {
    return guarded([&] { softmaxce_rows_fwd((hipStream_t)stream, logits, labels, loss, rows, classes, scratch, scratch_bytes); });
}
extern "C" int monet_softmaxce_rows_bwd(void *stream, const float *logits, const int32_t *labels, float *dlogits, int64_t rows, int classes,
                                        int accumulate) {
    return guarded([&] { softmaxce_rows_bwd((hipStream_t)stream, logits, labels, dlogits, rows, classes, accumulate != 0); });
}

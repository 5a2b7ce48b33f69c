// Host side of the gpupoly C ABI: network description, dependence-window planning, and the
// back-substitution driver that enqueues the kernels of cross.hip, scan.hip and layers.hip.
//
// Driver (paper Section 2 "Bottleneck Backsubstitution", Section 4.2 for the order of layers):
// layers are visited in id order; every layer that needs intervals is the start layer of a batch
// of rows which are back-substituted, chunk by chunk, through all earlier layers down to the
// input; candidates are taken wherever the expression ranges over a single layer.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "../../include/gpupoly.h"
#include "kernels.hpp"

static __device__ __align__(256) unsigned char scratch[32u << 20];

namespace {

enum LType { T_INPUT = 0, T_DENSE = 1, T_CONV = 2, T_RELU = 3, T_ADD = 4, T_POOL = 5 };   // T_POOL: average pooling

// Dependence window of a row in some layer, before clipping to the layer (Section 4.3):
// origin = S*pos - P (accumulated stride S, eq. 9; P accumulates padding), size W (eq. 4).
struct Geom {
    int Sy = 0, Sx = 0, Py = 0, Px = 0, Wy = 1, Wx = 1;
};

struct Layer {
    int type = T_INPUT, a = -1, b = -1;
    int C = 0, H = 0, W = 0;
    long long n = 0;
    int kh = 1, kw = 1, sh = 1, sw = 1, ph = 0, pw = 0;
    std::vector<float> wt_host;    // crossing layout [tap][C_in][C] (own channels innermost), kept until uploaded
    std::vector<float> wti_host;   // initial-expression layout [tap][C][C_in] (dense: [C][n_in])
    std::vector<float> bias_host;  // [C]
    double rowabs = 0.0;           // max_i sum_j |F_ij|
    bool need_bounds = false;      // intervals are computed for this layer (derived from the topology)
    bool req_bounds = false;       // asked for through gp_request_bounds
    bool feeds_relu = false;       // some ReLU layer reads this layer (the termination criterion applies to it)
    // topology-derived
    std::vector<int> land;         // affine layers a block over this layer is crossed through next
    std::vector<double> beff_host; // [C] summed bias of those layers (float64: the sum of two float32 is kept exact)
    // device
    float* d_wt = nullptr;
    double* d_wt64 = nullptr;      // the same in float64: the filter operand of the float64 MFMAs, read without conversion
    float* d_wti = nullptr;
    float* d_bias = nullptr;
    double* d_beff = nullptr;
    double *d_lo = nullptr, *d_hi = nullptr, *d_xmax = nullptr;
    double *d_rho = nullptr, *d_kap = nullptr;   // ReLU layers: candidate and intercept multipliers after substitution
    float* d_grl = nullptr;        // packed ReLU relaxation (see relax_factor in device_common.hpp)
    int* d_term = nullptr;         // early termination: per task the layer at which it met the criterion
    // inference rounding (Section 4.1): per neuron, how far a float32 evaluation can be from the exact expression over
    // the predecessors.  d_eta: affine layers their own error; sum layers their own rounding plus what their summands
    // pass on (a coefficient over the sum crosses all of them at once).  d_eta_thru: sum layers, the summands' part alone.
    double* d_eta = nullptr;
    double* d_eta_thru = nullptr;
};

struct PlanOp {
    enum Kind { INIT = 0, SCAN = 1, CROSS = 2, FINALIZE = 3 } kind = INIT;
    int slot_in = -1, slot_out = -1, slot_add = -1;
    Geom g_in, g_out, g_add;
    Geom t_in;             // CROSS: the rows' exact dependence window over layer_in (never clipped or widened)
    int layer_in = -1, layer_out = -1;
    bool relaxed = false;  // CROSS/INIT: apply the ReLU substitution of layer_out to the new block; SCAN: block holds such coefficients
    bool consts_only = false;
    bool do_consts = false, update_best = false, rounded = false;
    int init_mode = 0;     // INIT: 0 one-hot over the start layer, 1 certification rows, 2 the start layer's own matrix rows
};

struct Plan {
    bool valid = false;
    std::vector<PlanOp> ops;
    int n_slots = 0;
    long long slot_elems = 0;         // largest block, elements per row
    std::vector<int32_t> steps;       // gp_debug_plan records, 8 ints each
    std::vector<double> rem_flop;     // per op: arithmetic, per row, of the crossings from this op on (size ops + 1)
};

const double kRoundCoef = 0x1p-24 * (1.0 + 0x1p-20);   // float32 rounding of a float64 value
const double kRoundCoef64 = 0x1p-53 * (1.0 + 0x1p-20); // rounding of a product or sum of two float64 values (float64 storage)
const int kMaxSlots = 6;
const long long kMaxLayerWeights = 1LL << 28;
const int kGenMinRows = 16384;        // launches with more rows let the scan make a start layer's own rows (run_plan)

}  // namespace

struct gp_net {
    std::vector<Layer> L;
    std::string err;
    hipStream_t stream = nullptr;
    void* ws_user = nullptr;
    long long ws_user_bytes = 0;
    void* ws_own = nullptr;
    long long ws_own_bytes = 0;
    bool topo_ready = false;
    std::vector<Plan> plans;     // per layer
    Plan cert_plan;
    int batch = 0;               // boxes of the last analysis (what gp_get_bounds* and gp_certify* index)
    int batch_cap = 0;           // boxes the per-layer device arrays are sized for (0: none allocated); arrays are
                                 // [box][neuron], so an analysis of fewer boxes uses a prefix of each
    bool analyzed = false;
    bool weights_uploaded = false;
    int* d_flag = nullptr;
    double* d_xmax_all = nullptr;  // [layers][batch] running max of |bounds| per layer and box (one array: one clear per pass)
    int* d_labels = nullptr;
    float* d_margins = nullptr;
    // arbitrary linear forms of the outputs (gp_bound_outputs)
    float *d_forms = nullptr, *d_form_off = nullptr, *d_form_out = nullptr;
    long long d_forms_cap = 0, d_form_out_cap = 0;
    int n_forms = 0;               // > 0 while run_plan works on caller-given forms instead of certification rows
    bool forms_have_offset = false;
    float* d_centers = nullptr;
    long long d_centers_cap = 0;
    int device = -1;
    // early termination (Sections 3.2, 4.2)
    bool early = false;
    // Graph replay (gp_set_graph_replay): the launches of one box analysis, captured once and replayed.  A pass over a
    // small batch is a chain of ~150 dependent launches of a few microseconds each; replayed as one graph the
    // per-launch dispatch cost goes away.  Valid for one (batch, centres pointer, eps, clip, workspace, stream).
    bool graph_on = false;
    hipGraphExec_t graph_exec = nullptr;
    hipStream_t cap_stream = nullptr;      // launches are captured on a stream of the library's own (the legacy default
                                           // stream cannot be captured), the graph then runs on the caller's stream
    struct GraphKey { int batch; const float* centers; float eps, clo, chi; void* ws; long long ws_bytes; hipStream_t stream; };
    GraphKey graph_key = {};
    bool float_inference = false;  // bounds also hold for every float32 evaluation order of the network (Section 4.1)
    bool coef64 = false;           // coefficient blocks are stored in float64 (the paper's double precision build, Section 5)
    // set for the duration of gp_analyze_batch_dev_static: nothing may be allocated or freed; the rows' coefficient
    // blocks live in the library's static device array
    bool static_call = false;
    void* static_ws = nullptr;
    double acc_unit = 0x1p-50;     // unit roundoff the accumulation-error term is priced at (gp_debug_set_accumulation_roundoff)
    bool interval = false;         // the paper's literal scheme: interval coefficients, directed rounding (Section 4.1)
    bool chain_on = true;          // chains of narrow dense layers go through the fused kernel (gp_set_chain_fusion)
    int relu_reader = -1;          // during run_plan: the ReLU layer whose constants the launch that stores the bounds writes too (-1: none)
    int* d_count = nullptr;
    int* h_count = nullptr;        // pinned: task counts read back while the GPU keeps working
    hipEvent_t count_ev = nullptr;
    double early_flop_done = 0.0, early_flop_full = 0.0;   // crossing work carried out / work without any removal
    // optional per-kernel timing (gp_profile_*): index 0 = affine crossing, 1 = row scan
    bool prof_on = false;
    std::vector<hipEvent_t> prof_ev[2];     // start/stop pairs
    size_t prof_used[2] = {0, 0};
    double prof_flop[2] = {0, 0}, prof_bytes[2] = {0, 0};
    struct ProfRec { int kind, start, layer, nrows, in_el, out_el, n, k; double flop; };
    std::vector<ProfRec> prof_recs[2];
};

namespace {

gp_status fail(const gp_net* net, gp_status st, const char* fmt, ...) {
    if (net) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof(buf), fmt, ap);
        va_end(ap);
        const_cast<gp_net*>(net)->err = buf;
    }
    return st;
}

#define HIP_TRY(net, call)                                                                          \
    do {                                                                                            \
        hipError_t e__ = (call);                                                                    \
        if (e__ != hipSuccess)                                                                      \
            return fail(net, e__ == hipErrorOutOfMemory ? GP_ERR_NOMEM : GP_ERR_DEVICE, "%s: %s", #call, \
                        hipGetErrorString(e__));                                                    \
    } while (0)

void dfree(void* p) {
    if (p) (void)hipFree(p);
}

// ---- the static workspace of gp_analyze_batch_dev_static -------------------------------------------------------------------
// Device memory that exists from the moment the library's code object is loaded on a GPU until the process ends, one
// copy per GPU.  In host code the array's name is only a handle for hipGetSymbolAddress: the address kernels are given
// is looked up once per device, with that device current, and kept in g_scratch_ptr.
constexpr long long kStaticScratchBytes = 32LL << 20;
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

// a captured graph holds device addresses: whatever frees or moves device memory drops it
void drop_graph(gp_net* net) {
    if (net->graph_exec) { (void)hipGraphExecDestroy(net->graph_exec); net->graph_exec = nullptr; }
}

bool all_finite(const float* p, size_t n) {
    for (size_t i = 0; i < n; ++i)
        if (!std::isfinite(p[i])) return false;
    return true;
}

bool is_affine(const Layer& l) { return l.type == T_DENSE || l.type == T_CONV || l.type == T_POOL; }
// an average-pooling layer is a convolution whose filter is the constant 1/(kh*kw) on the channel diagonal: same window
// geometry, no stored filter, no contraction over channels
double pool_scale(const Layer& l) { return l.type == T_POOL ? 1.0 / ((double)l.kh * l.kw) : 0.0; }

// ---- window geometry -------------------------------------------------------------------------
void normalise(Geom& g, const Layer& l) {
    if (g.Wy >= l.H) { g.Sy = 0; g.Py = 0; g.Wy = l.H; }
    if (g.Wx >= l.W) { g.Sx = 0; g.Px = 0; g.Wx = l.W; }
}

// window in the input layer of affine layer `a` from the window g in its output (eqs. 4, 6-9)
Geom cross_geom(const Geom& g, const Layer& a, const Layer& pred) {
    Geom o;
    if (a.type == T_DENSE) {
        o.Sy = o.Sx = o.Py = o.Px = 0;
        o.Wy = pred.H;
        o.Wx = pred.W;
    } else {
        o.Sy = g.Sy * a.sh; o.Py = g.Py * a.sh + a.ph; o.Wy = (g.Wy - 1) * a.sh + a.kh;
        o.Sx = g.Sx * a.sw; o.Px = g.Px * a.sw + a.pw; o.Wx = (g.Wx - 1) * a.sw + a.kw;
    }
    normalise(o, pred);
    return o;
}

bool hull_dim(int S1, int P1, int W1, int S2, int P2, int W2, int H, int& S, int& P, int& W) {
    bool full1 = (W1 >= H), full2 = (W2 >= H);
    if (full1 || full2) { S = 0; P = 0; W = H; return true; }
    if (S1 != S2) return false;
    S = S1;
    P = std::max(P1, P2);
    W = std::max(W1 - P1, W2 - P2) + P;
    return true;
}

bool hull(const Geom& a, const Geom& b, const Layer& l, Geom& o) {
    if (!hull_dim(a.Sy, a.Py, a.Wy, b.Sy, b.Py, b.Wy, l.H, o.Sy, o.Py, o.Wy)) return false;
    if (!hull_dim(a.Sx, a.Px, a.Wx, b.Sx, b.Px, b.Wx, l.W, o.Sx, o.Px, o.Wx)) return false;
    normalise(o, l);
    return true;
}

// The exact dependence window of a row (Section 4.3), carried beside the stored one.  The stored window is clipped
// to the layer and shifted inside it at the borders, and it is widened to the whole layer once it is as large; the
// entries it holds outside the exact window are structural zeros, which the crossing kernel skips.
const int kEverywhere = 1 << 20;
Geom everywhere() {
    Geom g;
    g.Sy = g.Sx = 0; g.Py = g.Px = kEverywhere; g.Wy = g.Wx = 2 * kEverywhere;
    return g;
}
bool is_everywhere(const Geom& g) { return g.Wy >= 2 * kEverywhere || g.Wx >= 2 * kEverywhere; }

Geom cross_exact(const Geom& t, const Layer& a) {
    if (a.type == T_DENSE || is_everywhere(t)) return everywhere();
    Geom o;
    o.Sy = t.Sy * a.sh; o.Py = t.Py * a.sh + a.ph; o.Wy = (t.Wy - 1) * a.sh + a.kh;
    o.Sx = t.Sx * a.sw; o.Px = t.Px * a.sw + a.pw; o.Wx = (t.Wx - 1) * a.sw + a.kw;
    if (o.Wy >= kEverywhere / 4 || o.Wx >= kEverywhere / 4 || o.Py >= kEverywhere / 4 || o.Px >= kEverywhere / 4) return everywhere();
    return o;
}

Geom hull_exact(const Geom& a, const Geom& b) {
    if (is_everywhere(a) || is_everywhere(b) || a.Sy != b.Sy || a.Sx != b.Sx) return everywhere();
    Geom o;
    o.Sy = a.Sy; o.Py = std::max(a.Py, b.Py); o.Wy = std::max(a.Wy - a.Py, b.Wy - b.Py) + o.Py;
    o.Sx = a.Sx; o.Px = std::max(a.Px, b.Px); o.Wx = std::max(a.Wx - a.Px, b.Wx - b.Px) + o.Px;
    return o;
}

long long block_elems(const Geom& g, const Layer& l) {
    return (long long)std::min(g.Wy, l.H) * std::min(g.Wx, l.W) * l.C;
}

// Average, over the positions of the start layer, of the share of a stored window that lies inside the exact
// dependence window: the stored block of a border row is a full-size window shifted inside the layer (or the whole
// layer), and what it holds outside the exact window are structural zeros that no step multiplies.  The algorithmic
// work of a step counts the exact part only.
double exact_share(const Geom& g, const Geom& t, const Layer& l, int Hs, int Ws) {
    if (is_everywhere(t)) return 1.0;
    auto axis = [](int S, int P, int W, int tS, int tP, int tW, int H, int n_pos) {
        const int w = std::min(W, H);
        double sum = 0.0;
        for (int pos = 0; pos < n_pos; ++pos) {
            const int o = std::min(std::max(S * pos - P, 0), H - w);
            const int lo = std::max(std::max(tS * pos - tP, o), 0), hi = std::min(std::min(tS * pos - tP + tW, o + w), H);
            sum += std::max(hi - lo, 0);
        }
        return sum / ((double)n_pos * w);
    };
    return axis(g.Sy, g.Py, g.Wy, t.Sy, t.Py, t.Wy, l.H, Hs) * axis(g.Sx, g.Px, g.Wx, t.Sx, t.Px, t.Wx, l.W, Ws);
}

// ---- topology-derived data ---------------------------------------------------------------------
void land_of(const gp_net* net, int q, std::vector<int>& out) {   // where a coefficient over layer q goes next
    const Layer& l = net->L[q];
    if (is_affine(l)) out.push_back(q);
    else if (l.type == T_ADD) { land_of(net, l.a, out); land_of(net, l.b, out); }
}

gp_status prepare_topology(gp_net* net) {
    if (net->topo_ready) return GP_OK;
    int nl = (int)net->L.size();
    for (int i = 0; i < nl; ++i) { net->L[i].need_bounds = net->L[i].req_bounds; net->L[i].feeds_relu = false; }
    for (int i = 1; i < nl; ++i) {
        Layer& l = net->L[i];
        // every crossing must land on a layer with intervals (they bound the rounding slack)
        if (is_affine(l)) net->L[l.a].need_bounds = true;
        if (l.type == T_RELU) { net->L[l.a].need_bounds = true; net->L[l.a].feeds_relu = true; }
        // the rounding error of a float32 addition is relative to the sum: a sum layer needs its own interval
        if (l.type == T_ADD && net->float_inference) l.need_bounds = true;
    }
    net->L[nl - 1].need_bounds = true;
    for (int i = 0; i < nl; ++i) {
        Layer& l = net->L[i];
        l.land.clear();
        if (is_affine(l)) l.land.push_back(i);
        else if (l.type == T_RELU) land_of(net, l.a, l.land);
        else if (l.type == T_ADD) { land_of(net, l.a, l.land); land_of(net, l.b, l.land); }
        if (l.land.size() > 2) return fail(net, GP_ERR_UNSUPPORTED, "layer %d: more than two affine branches meet", i);
        l.beff_host.assign(l.C, 0.0);
        for (int q : l.land)
            for (int c = 0; c < l.C; ++c) l.beff_host[c] += (double)net->L[q].bias_host[c];
    }
    net->plans.assign(nl, Plan());
    net->cert_plan = Plan();
    net->topo_ready = true;
    return GP_OK;
}

// ---- planning ------------------------------------------------------------------------------------
struct Desc {
    int slot = -1;
    Geom g;
    Geom t;                  // exact dependence window (see cross_exact)
    bool consumed = false;   // the constants of the next step have been added to the rows' constant
};

void push_step(Plan& pl, int kind, int layer, const Geom& g, const Layer& l, int merged) {
    int32_t rec[8] = {kind, layer, std::min(g.Wy, l.H), std::min(g.Wx, l.W), l.C, g.Sy, g.Py, merged};
    pl.steps.insert(pl.steps.end(), rec, rec + 8);
}

gp_status build_plan(gp_net* net, int start, bool certify, Plan& pl) {
    pl = Plan();
    const std::vector<Layer>& L = net->L;
    std::vector<int> ref(kMaxSlots, 0);
    auto alloc_slot = [&]() {
        for (int i = 0; i < kMaxSlots; ++i)
            if (ref[i] == 0) { ref[i] = 1; pl.n_slots = std::max(pl.n_slots, i + 1); return i; }
        return -1;
    };
    std::map<int, Desc> expr;
    Geom g0;
    if (certify) { g0.Sy = g0.Sx = g0.Py = g0.Px = 0; g0.Wy = L[start].H; g0.Wx = L[start].W; }
    else { g0.Sy = g0.Sx = 1; g0.Py = g0.Px = 0; g0.Wy = g0.Wx = 1; }
    const Geom t0 = certify ? everywhere() : g0;
    normalise(g0, L[start]);
    if (!certify && is_affine(L[start]) && L[start].type != T_POOL) {
        // the neuron's own affine expression (Section 2): the filter placed in the window over the predecessor
        const int pr = L[start].a;
        Geom g1 = cross_geom(g0, L[start], L[pr]);
        const bool relu_pred = L[pr].type == T_RELU;
        PlanOp op;
        op.kind = PlanOp::INIT;
        op.init_mode = 2;
        op.slot_out = alloc_slot();
        op.g_out = g1;
        op.layer_in = start;
        op.layer_out = pr;
        op.relaxed = relu_pred;
        pl.ops.push_back(op);
        pl.slot_elems = std::max(pl.slot_elems, block_elems(g1, L[pr]));
        PlanOp sc;
        sc.kind = PlanOp::SCAN;
        sc.slot_in = op.slot_out; sc.g_in = g1; sc.layer_in = pr;
        sc.do_consts = true; sc.update_best = true; sc.rounded = relu_pred; sc.relaxed = relu_pred;
        pl.ops.push_back(sc);
        Desc d; d.slot = op.slot_out; d.g = g1; d.t = cross_exact(t0, L[start]); d.consumed = true;
        expr[relu_pred ? L[pr].a : pr] = d;
        push_step(pl, 0, start, g0, L[start], 0);
        push_step(pl, 1, start, g1, L[pr], 0);
        if (relu_pred) push_step(pl, 2, pr, g1, L[pr], 0);
    } else {
        PlanOp op;
        op.kind = PlanOp::INIT;
        op.init_mode = certify ? 1 : 0;
        op.slot_out = alloc_slot();
        op.g_out = g0;
        op.layer_out = start;
        pl.ops.push_back(op);
        pl.slot_elems = std::max(pl.slot_elems, block_elems(g0, L[start]));
        PlanOp sc;
        sc.kind = PlanOp::SCAN;
        sc.slot_in = op.slot_out; sc.g_in = g0; sc.layer_in = start;
        sc.do_consts = true; sc.update_best = false; sc.rounded = false;
        pl.ops.push_back(sc);
        Desc d; d.slot = op.slot_out; d.g = g0; d.t = t0; d.consumed = true;
        expr[start] = d;
        push_step(pl, 0, start, g0, L[start], 0);
    }
    auto insert = [&](int t, const Desc& d) -> bool {
        if (expr.count(t)) return false;
        expr[t] = d;
        return true;
    };
    while (true) {
        int k = expr.rbegin()->first;
        if (k == 0) break;
        Desc d = expr[k];
        expr.erase(k);
        const Layer& l = L[k];
        if (!d.consumed) {
            if (l.type == T_RELU)
                return fail(net, GP_ERR_UNSUPPORTED, "layer %d: a partial expression over a ReLU layer is never joined", k);
            PlanOp sc;
            sc.kind = PlanOp::SCAN;
            sc.slot_in = d.slot; sc.g_in = d.g; sc.layer_in = k;
            sc.do_consts = true; sc.update_best = false; sc.rounded = false;
            sc.consts_only = true;
            pl.ops.push_back(sc);
            d.consumed = true;
        }
        if (l.type == T_RELU) {
            return fail(net, GP_ERR_UNSUPPORTED, "layer %d: ReLU of a layer that is not crossed by an affine layer", k);
        } else if (l.type == T_ADD) {
            if (l.a == l.b) return fail(net, GP_ERR_UNSUPPORTED, "layer %d: sum of a layer with itself", k);
            if (!insert(l.a, d) || !insert(l.b, d))
                return fail(net, GP_ERR_UNSUPPORTED, "layer %d: two expressions meet before an affine layer", k);
            ref[d.slot] += 1;
            push_step(pl, 3, k, d.g, l, 0);
        } else if (is_affine(l)) {
            const int p = l.a;
            Geom g = cross_geom(d.g, l, L[p]);
            Geom t = cross_exact(d.t, l);
            PlanOp op;
            op.kind = PlanOp::CROSS;
            op.slot_in = d.slot; op.g_in = d.g; op.t_in = d.t; op.layer_in = k; op.layer_out = p;
            Desc ad;
            bool has_add = expr.count(p) > 0;
            if (has_add) {
                ad = expr[p];
                expr.erase(p);
                Geom h;
                if (!hull(g, ad.g, L[p], h))
                    return fail(net, GP_ERR_UNSUPPORTED, "layer %d: branches with different accumulated strides", p);
                g = h;
                t = hull_exact(t, ad.t);
                if (l.type == T_DENSE && block_elems(ad.g, L[p]) != L[p].n)
                    return fail(net, GP_ERR_UNSUPPORTED, "layer %d: windowed block joins a dense branch", p);
                op.slot_add = ad.slot; op.g_add = ad.g;
            }
            op.slot_out = alloc_slot();
            if (op.slot_out < 0) return fail(net, GP_ERR_UNSUPPORTED, "too many live coefficient blocks");
            op.g_out = g;
            bool complete = true;
            for (auto& kv : expr)
                if (kv.first > p) complete = false;
            // a complete block over a ReLU layer takes the ReLU substitution at once (sign-split, Section 2)
            // and then ranges over the ReLU's input layer
            const bool relaxed = complete && L[p].type == T_RELU;
            const int key = relaxed ? L[p].a : p;
            if (relaxed && expr.count(key))
                return fail(net, GP_ERR_UNSUPPORTED, "layer %d: two expressions meet before an affine layer", key);
            op.relaxed = relaxed;
            pl.ops.push_back(op);
            pl.slot_elems = std::max(pl.slot_elems, block_elems(g, L[p]));
            ref[d.slot] -= 1;
            if (has_add) ref[ad.slot] -= 1;
            PlanOp sc;
            sc.kind = PlanOp::SCAN;
            sc.slot_in = op.slot_out; sc.g_in = g; sc.layer_in = p;
            sc.do_consts = complete; sc.update_best = expr.empty(); sc.rounded = true; sc.relaxed = relaxed;
            pl.ops.push_back(sc);
            Desc nd; nd.slot = op.slot_out; nd.g = g; nd.t = t; nd.consumed = complete;
            expr[key] = nd;
            push_step(pl, 1, k, g, L[p], has_add ? 1 : 0);
            if (relaxed) push_step(pl, 2, p, g, L[p], 0);
        } else {
            return fail(net, GP_ERR_UNSUPPORTED, "layer %d: unexpected type", k);
        }
    }
    if (expr.size() != 1) return fail(net, GP_ERR_UNSUPPORTED, "expression did not reach the input layer alone");
    PlanOp fin;
    fin.kind = PlanOp::FINALIZE;
    pl.ops.push_back(fin);
    // per row: arithmetic of the crossings that follow each op of the plan (what removing a row saves)
    pl.rem_flop.assign(pl.ops.size() + 1, 0.0);
    for (size_t i = pl.ops.size(); i-- > 0;) {
        pl.rem_flop[i] = pl.rem_flop[i + 1];
        const PlanOp& op = pl.ops[i];
        if (op.kind == PlanOp::CROSS) {
            const Layer& a = L[op.layer_in];
            const Layer& p = L[op.layer_out];
            const double taps = (a.type == T_DENSE) ? 1.0 : (double)a.kh * a.kw;
            const double cin = (a.type == T_DENSE) ? (double)p.n : (a.type == T_POOL) ? 1.0 : (double)p.C;
            pl.rem_flop[i] += 2.0 * (double)block_elems(op.g_in, a) * taps * cin *
                              (certify ? 1.0 : exact_share(op.g_in, op.t_in, a, L[start].H, L[start].W));
        }
    }
    pl.valid = true;
    return GP_OK;
}

gp_status get_plan(gp_net* net, int lid, Plan** out) {
    gp_status st = prepare_topology(net);
    if (st != GP_OK) return st;
    Plan& pl = net->plans[lid];
    if (!pl.valid) {
        st = build_plan(net, lid, false, pl);
        if (st != GP_OK) return st;
    }
    *out = &pl;
    return GP_OK;
}

// ---- device state ------------------------------------------------------------------------------
void free_layer_bounds(Layer& l) {   // callers drop the captured graph
    dfree(l.d_lo); dfree(l.d_hi); dfree(l.d_rho); dfree(l.d_kap); dfree(l.d_grl); dfree(l.d_term);   // d_xmax: part of d_xmax_all
    dfree(l.d_eta); dfree(l.d_eta_thru);
    l.d_lo = l.d_hi = l.d_rho = l.d_kap = l.d_xmax = l.d_eta = l.d_eta_thru = nullptr;
    l.d_grl = nullptr;
    l.d_term = nullptr;
}

// what a coefficient over layer lid picks up per unit of magnitude when it is substituted (inference rounding), or null
const double* eta_of(const gp_net* net, int lid) {
    const Layer& l = net->L[lid];
    if (!net->float_inference) return nullptr;
    if (is_affine(l) || l.type == T_ADD) return l.d_eta;
    if (l.type == T_RELU) return eta_of(net, l.a);
    return nullptr;
}
// a coefficient over a sum layer is handed to both summands unchanged: it crosses a summand that is an affine or a sum
// layer in the same step (like land_of), while a ReLU summand is substituted later, as a block of its own
bool summand_passes_eta(const gp_net* net, int lid) {
    return is_affine(net->L[lid]) || net->L[lid].type == T_ADD;
}

bool has_bounds(const gp_net* net, int lid) {
    const Layer& l = net->L[lid];
    return lid == 0 || l.type == T_RELU || l.need_bounds;
}

// everything whose size depends on the batch
void release_batch_state(gp_net* net) {
    for (auto& l : net->L) free_layer_bounds(l);
    dfree(net->d_labels); net->d_labels = nullptr;
    dfree(net->d_margins); net->d_margins = nullptr;
    dfree(net->d_xmax_all); net->d_xmax_all = nullptr;
}

gp_status allocate_batch_state(gp_net* net, int batch) {
    HIP_TRY(net, hipMalloc((void**)&net->d_xmax_all, sizeof(double) * batch * net->L.size()));
    for (size_t i = 0; i < net->L.size(); ++i) {
        Layer& l = net->L[i];
        size_t cnt = (size_t)l.n * batch;
        // with early termination every layer carries intervals (its interval image at least)
        if (has_bounds(net, (int)i) || net->early) {
            HIP_TRY(net, hipMalloc((void**)&l.d_lo, cnt * sizeof(double)));
            HIP_TRY(net, hipMalloc((void**)&l.d_hi, cnt * sizeof(double)));
            l.d_xmax = net->d_xmax_all + i * (size_t)batch;
        }
        if (net->early && l.need_bounds && l.type != T_RELU && i > 0)
            HIP_TRY(net, hipMalloc((void**)&l.d_term, cnt * sizeof(int)));
        if (net->float_inference && (is_affine(l) || l.type == T_ADD))
            HIP_TRY(net, hipMalloc((void**)&l.d_eta, cnt * sizeof(double)));
        if (net->float_inference && l.type == T_ADD && (summand_passes_eta(net, l.a) || summand_passes_eta(net, l.b)))
            HIP_TRY(net, hipMalloc((void**)&l.d_eta_thru, cnt * sizeof(double)));
        if (l.type == T_RELU) {
            HIP_TRY(net, hipMalloc((void**)&l.d_grl, cnt * sizeof(float)));
            HIP_TRY(net, hipMalloc((void**)&l.d_rho, cnt * sizeof(double)));
            HIP_TRY(net, hipMalloc((void**)&l.d_kap, cnt * sizeof(double)));
        }
    }
    long long nout = net->L.back().n;
    HIP_TRY(net, hipMalloc((void**)&net->d_labels, sizeof(int) * batch));
    HIP_TRY(net, hipMalloc((void**)&net->d_margins, sizeof(float) * batch * std::max<long long>(nout - 1, 1)));
    return GP_OK;
}

gp_status ensure_device(gp_net* net, int batch) {
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return fail(net, GP_ERR_DEVICE, "no HIP device");
    if (net->static_call) {      // nothing may be allocated: everything must be there from an earlier analysis
        if (!net->d_flag || !net->d_count || !net->h_count || !net->count_ev || !net->weights_uploaded || batch > net->batch_cap)
            return fail(net, GP_ERR_STATE, "no analysis of at least %d boxes has run on this net since its topology or modes last changed: "
                                           "the allocation-free call has no per-layer arrays to work in", batch);
        net->batch = batch;
        return GP_OK;
    }
    if (net->device < 0) HIP_TRY(net, hipGetDevice(&net->device));
    // Address of the static workspace on this device, for gp_analyze_batch_dev_static: looked up here, once per device
    // and with that device current (every GPU holds its own copy at its own address), because the runtime may
    // materialise the array at the first lookup and that call must not allocate.
    if (net->device >= 0 && net->device < kMaxDevices && !g_scratch_ptr[net->device]) {
        void* ptr = nullptr;
        HIP_TRY(net, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(net, GP_ERR_DEVICE, "the static workspace has no device address");
        g_scratch_ptr[net->device] = ptr;
    }
    if (!net->d_flag) HIP_TRY(net, hipMalloc((void**)&net->d_flag, sizeof(int)));
    if (!net->d_count) HIP_TRY(net, hipMalloc((void**)&net->d_count, sizeof(int)));
    if (!net->h_count) HIP_TRY(net, hipHostMalloc((void**)&net->h_count, 2 * sizeof(int), hipHostMallocDefault));
    if (!net->count_ev) HIP_TRY(net, hipEventCreateWithFlags(&net->count_ev, hipEventDisableTiming));
    if (!net->weights_uploaded) {
        for (auto& l : net->L) {
            if (!l.wt_host.empty() && !l.d_wt) {
                HIP_TRY(net, hipMalloc((void**)&l.d_wt, l.wt_host.size() * sizeof(float)));
                HIP_TRY(net, hipMemcpy(l.d_wt, l.wt_host.data(), l.wt_host.size() * sizeof(float), hipMemcpyHostToDevice));
                {   // (twice the bytes of the float32 weights again; ResNet-34: 170 MB)
                    std::vector<double> w64(l.wt_host.begin(), l.wt_host.end());
                    HIP_TRY(net, hipMalloc((void**)&l.d_wt64, w64.size() * sizeof(double)));
                    HIP_TRY(net, hipMemcpy(l.d_wt64, w64.data(), w64.size() * sizeof(double), hipMemcpyHostToDevice));
                }
            }
            if (!l.wti_host.empty() && !l.d_wti) {
                HIP_TRY(net, hipMalloc((void**)&l.d_wti, l.wti_host.size() * sizeof(float)));
                HIP_TRY(net, hipMemcpy(l.d_wti, l.wti_host.data(), l.wti_host.size() * sizeof(float), hipMemcpyHostToDevice));
                HIP_TRY(net, hipMalloc((void**)&l.d_bias, l.C * sizeof(float)));
                HIP_TRY(net, hipMemcpy(l.d_bias, l.bias_host.data(), l.C * sizeof(float), hipMemcpyHostToDevice));
            }
            if (!l.d_beff && l.C > 0) {
                HIP_TRY(net, hipMalloc((void**)&l.d_beff, l.C * sizeof(double)));
                HIP_TRY(net, hipMemcpy(l.d_beff, l.beff_host.data(), l.C * sizeof(double), hipMemcpyHostToDevice));
            }
        }
        net->weights_uploaded = true;
    }
    if (batch > net->batch_cap) {
        // Nothing is sized for any batch while this block runs: the capacity is 0 until the last allocation has
        // succeeded, and a failure on the way frees what was allocated, so that the next call (at whatever batch)
        // starts from scratch instead of launching kernels on buffers that are gone or sized for the batch that failed.
        drop_graph(net);
        net->batch_cap = 0;
        net->batch = 0;
        net->analyzed = false;
        release_batch_state(net);
        const gp_status st = allocate_batch_state(net, batch);
        if (st != GP_OK) { release_batch_state(net); (void)hipGetLastError(); return st; }   // (the sticky error is reported here, once)
        net->batch_cap = batch;
    }
    net->batch = batch;
    return GP_OK;
}

long long align_up(long long v, long long a) { return (v + a - 1) / a * a; }

// bytes of one stored coefficient: float32, float64, or an interval of two float64
int coef_bytes(const gp_net* net) { return net->interval ? 16 : net->coef64 ? 8 : 4; }

// bytes one task (both signs) needs for this plan
long long task_bytes(const Plan& pl, int nsign, int csize) {
    // blocks; constant, slack (twice: rows are moved when tasks are removed), best; row lists and flags; chunk sums of
    // the scan of long rows (5 doubles per 512 coefficients)
    const long long chunks = pl.slot_elems > 1024 ? (pl.slot_elems + 511) / 512 : 0;
    return (long long)nsign * (pl.n_slots * align_up(pl.slot_elems * csize, 16) + 5 * 8 + chunks * 40) + 16;
}

gp_status get_workspace(gp_net* net, long long want, char** ws, long long* bytes) {
    if (net->static_call) { *ws = (char*)net->static_ws; *bytes = kStaticScratchBytes; return GP_OK; }
    if (net->ws_user) { *ws = (char*)net->ws_user; *bytes = net->ws_user_bytes; return GP_OK; }
    const long long cap = 32LL << 30;
    long long need = std::min(want, cap);
    need = align_up(std::max(need, 1LL << 20), 1 << 20);
    if (net->ws_own_bytes < need) {
        drop_graph(net);
        dfree(net->ws_own);
        net->ws_own = nullptr; net->ws_own_bytes = 0;
        HIP_TRY(net, hipMalloc(&net->ws_own, need));
        net->ws_own_bytes = need;
    }
    *ws = (char*)net->ws_own; *bytes = net->ws_own_bytes;
    return GP_OK;
}

gp::BlockDesc make_desc(const gp_net* net, const float* data, const Geom& g, int layer, const Geom* exact = nullptr) {
    const Layer& l = net->L[layer];
    gp::BlockDesc b;
    b.data = data;
    b.H = l.H; b.W = l.W; b.C = l.C;
    b.wy = std::min(g.Wy, l.H); b.wx = std::min(g.Wx, l.W);
    b.Sy = g.Sy; b.Sx = g.Sx; b.Py = g.Py; b.Px = g.Px;
    const Geom t = (exact && l.H < 32768 && l.W < 32768) ? *exact : everywhere();
    b.tSy = t.Sy; b.tSx = t.Sx; b.tPy = t.Py; b.tPx = t.Px; b.tWy = t.Wy; b.tWx = t.Wx;
    return b;
}

void prof_mark(gp_net* net, int kind, bool stop) {
    if (!net->prof_on) return;
    std::vector<hipEvent_t>& ev = net->prof_ev[kind];
    size_t& used = net->prof_used[kind];
    if (used == ev.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        ev.push_back(e);
    }
    (void)stop;
    (void)hipEventRecord(ev[used++], net->stream);
}

// the per-neuron constants and slack parameters of the candidate taken over op.layer_in (everything of ScanParams that
// does not depend on the rows); returns whether the candidate has interval terms
bool scan_setup(const gp_net* net, const PlanOp& op, int start, bool certify, gp::ScanParams& sp) {
    const Layer& l = net->L[op.layer_in];
    const bool interval_terms = !op.consts_only && has_bounds(net, op.layer_in) && op.layer_in != start;
    sp.cpos = sp.cneg = sp.xlo = sp.xhi = sp.kap = nullptr;
    sp.xmax_self = nullptr;
    if (interval_terms) {
        if (op.relaxed) {      // coefficients already multiplied by the ReLU slopes: they range over the ReLU's input
            const Layer& q = net->L[l.a];
            sp.cpos = l.d_rho; sp.cneg = l.d_lo; sp.xlo = q.d_lo; sp.xhi = q.d_hi; sp.xmax_self = q.d_xmax;
        } else {
            sp.cpos = l.d_hi; sp.cneg = l.d_lo; sp.xlo = l.d_lo; sp.xhi = l.d_hi; sp.xmax_self = l.d_xmax;
        }
    }
    if (op.relaxed) sp.kap = l.d_kap;
    sp.beff = l.land.empty() ? nullptr : l.d_beff;
    // a sum layer's own rows bound the exact sum of its summands; its one rounding is added when they are stored
    sp.eta = (!certify && op.layer_in == start && l.type == T_ADD) ? l.d_eta_thru : eta_of(net, op.layer_in);
    sp.e1_a = sp.e1_b = 0.0;
    sp.xmax_a = sp.xmax_b = nullptr;
    for (size_t i = 0; i < l.land.size(); ++i) {
        const Layer& q = net->L[l.land[i]];
        double K = (double)q.kh * q.kw * (q.type == T_POOL ? 1.0 : (double)q.C);   // terms of one new coefficient
        double e1 = (K + 8.0) * net->acc_unit * q.rowabs;
        if (i == 0) { sp.e1_a = e1; sp.xmax_a = net->L[q.a].d_xmax; }
        else { sp.e1_b = e1; sp.xmax_b = net->L[q.a].d_xmax; }
    }
    sp.round_coef = op.rounded ? (net->coef64 ? kRoundCoef64 : kRoundCoef) : 0.0;
    sp.coef64 = net->coef64 ? 1 : 0;
    // what vanishes when a coefficient is stored: below the subnormal step of the storage type, times the
    // 2^20 by which a substituted ReLU slope (kept >= 2^-20) may have shrunk it
    sp.coef_floor = net->coef64 ? 0x1p-1050 : 0x1p-128;
    sp.do_consts = op.do_consts ? 1 : 0;
    sp.update_best = op.update_best ? 1 : 0;
    return interval_terms;
}

// Chains of narrow dense layers: the whole plan of a start layer in ONE launch (chain.hip), the rows' blocks in LDS.
// Decided by the network alone (layer types and widths), never by the number of rows, so that a box gets the same
// bits alone and in a batch.  Returns false when the plan is not such a chain (then p is undefined).
const int kChainMaxHidden = 256, kChainMaxLast = 1024;
bool build_chain(const gp_net* net, const Plan& pl, int start, gp::ChainParams& p, double* flop_per_row) {
    const Layer& ls = net->L[start];
    if (!net->chain_on || net->early || net->float_inference || net->coef64 || net->interval || ls.type != T_DENSE) return false;
    // a wide start layer has many rows per box; its rows go through the general kernels like those of a wide hidden layer
    // (measured on the 500 own rows per box of FC 9x500's first layer, 784 wide: 0.37 against 0.09 ms at 100 boxes)
    if (ls.n > kChainMaxHidden) return false;
    const size_t nops = pl.ops.size();
    if (nops < 3 || nops % 2 == 0) return false;                         // INIT SCAN (CROSS SCAN)* FINALIZE
    if (pl.ops[0].kind != PlanOp::INIT || pl.ops[0].init_mode != 2 || pl.ops[nops - 1].kind != PlanOp::FINALIZE) return false;
    const int nsteps = (int)(nops - 1) / 2;
    if (nsteps > gp::kMaxChainSteps) return false;
    std::memset(&p, 0, sizeof(p));
    *flop_per_row = 0.0;
    int hid = 0;
    for (int st = 0; st < nsteps; ++st) {
        const PlanOp& op = pl.ops[2 * st];
        const PlanOp& sc = pl.ops[2 * st + 1];
        if (sc.kind != PlanOp::SCAN || sc.consts_only || !sc.update_best || sc.slot_in != op.slot_out) return false;
        if (st > 0 && (op.kind != PlanOp::CROSS || net->L[op.layer_in].type != T_DENSE || op.slot_add >= 0)) return false;
        const Layer& lb = net->L[sc.layer_in];                         // the layer the block ranges over
        if (block_elems(sc.g_in, lb) != lb.n) return false;
        const bool last = st == nsteps - 1;
        if (lb.n > (last ? kChainMaxLast : kChainMaxHidden)) return false;
        gp::ScanParams sp;
        std::memset(&sp, 0, sizeof(sp));
        if (!scan_setup(net, sc, start, false, sp) || sp.xmax_b || sp.eta) return false;
        gp::ChainStep& cs = p.steps[st];
        cs.n = (int)lb.n;
        cs.grl = op.relaxed ? lb.d_grl : nullptr;
        if (st > 0) {
            const Layer& a = net->L[op.layer_in];
            if (!a.d_wt) return false;
            cs.K = (int)a.n;
            cs.w = a.d_wt;
            *flop_per_row += 2.0 * (double)a.n * (double)lb.n;
        }
        cs.cpos = sp.cpos; cs.cneg = sp.cneg; cs.xlo = sp.xlo; cs.xhi = sp.xhi; cs.kap = sp.kap; cs.beff = sp.beff;
        cs.xmax_self = sp.xmax_self; cs.xmax_a = sp.xmax_a; cs.e1_a = sp.e1_a; cs.round_coef = sp.round_coef;
        cs.do_consts = sp.do_consts;
        p.coef_floor = sp.coef_floor;
        if (!last) hid = std::max(hid, (int)lb.n);
    }
    p.nsteps = nsteps;
    p.w0 = ls.d_wti; p.bias0 = ls.d_bias;
    p.n_start = (int)ls.n;
    p.div_n = gp::make_fastdiv((uint32_t)ls.n);
    // row strides of 4*(odd) floats: the 16 rows of a 16-byte LDS access fall into distinct banks
    p.hid_stride = ((std::max(hid, 1) + 15) & ~15) + 4;
    p.last_stride = ((p.steps[nsteps - 1].n + 15) & ~15) + 4;
    p.lo = ls.d_lo; p.hi = ls.d_hi; p.xmax = ls.d_xmax; p.flag = net->d_flag;
    return gp::chain_lds_bytes(p) <= 150 * 1024;
}

// the ReLU layer lid: where its intervals and relaxation go
gp::ReluParams relu_params(gp_net* net, int lid, int batch) {
    Layer& l = net->L[lid];
    gp::ReluParams rp;
    rp.plo = net->L[l.a].d_lo; rp.phi = net->L[l.a].d_hi;
    rp.lo = l.d_lo; rp.hi = l.d_hi; rp.grl = l.d_grl; rp.rho = l.d_rho; rp.kap = l.d_kap;
    rp.xmax = l.d_xmax; rp.flag = net->d_flag;
    rp.total = l.n * batch;
    rp.n = l.n;
    rp.margin = net->coef64 ? 0x1p-50 : 0x1p-22;
    return rp;
}

// run one plan over all its tasks, chunk by chunk (Section 4.2 "Memory management").
// With early termination (Sections 3.2, 4.2) the rows' best bounds start from the layer's interval image, tasks
// whose interval does not strictly contain 0 never start, and after every candidate the tasks that have come to
// meet the criterion are flagged; flagged tasks keep their bounds, and once enough of them have gathered their
// rows are removed from the block (prefix sum over the flags, rows copied to a free block).
gp_status run_plan(gp_net* net, const Plan& pl, int start, bool certify, int batch) {
    const Layer& ls = net->L[start];
    const int nsign = certify ? 1 : 2;
    const bool forms = certify && net->n_forms > 0;
    const long long n_start = forms ? net->n_forms : certify ? (ls.n - 1) : ls.n;
    const long long total = n_start * batch;
    if (total <= 0) return GP_OK;
    if (!certify && total < (1LL << 31)) {
        gp::ChainParams chp;
        double flop_per_row = 0.0;
        if (build_chain(net, pl, start, chp, &flop_per_row)) {
            chp.row0 = 0; chp.Rc = (int)total;
            chp.has_relu = net->relu_reader >= 0 ? 1 : 0;
            if (chp.has_relu) chp.relu = relu_params(net, net->relu_reader, batch);
            // (timed as a crossing launch when it contains products; a plan without any is bookkeeping only)
            const bool timed = flop_per_row > 0.0;
            if (timed) prof_mark(net, 0, false);
            const bool ok = gp::launch_chain(chp, net->stream);
            if (timed) prof_mark(net, 0, true);
            if (!ok) return fail(net, GP_ERR_DEVICE, "the fused chain kernel could not get %zu bytes of LDS", gp::chain_lds_bytes(chp));
            if (net->prof_on && timed) {
                net->prof_flop[0] += flop_per_row * 2.0 * (double)total;
                net->prof_bytes[0] += 16.0 * (double)total;
                net->prof_recs[0].push_back({2, start, start, (int)(2 * total), 0, 0, 0, 0, flop_per_row * 2.0 * (double)total});
            }
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return fail(net, GP_ERR_DEVICE, "kernel launch: %s", hipGetErrorString(e));
            return GP_OK;
        }
    }
    const bool early = net->early && !certify;
    const bool may_stop = early && ls.feeds_relu && !ls.req_bounds && start != (int)net->L.size() - 1;
    const int csize = coef_bytes(net);                  // bytes per stored coefficient
    const long long tb = task_bytes(pl, nsign, csize);
    char* ws; long long ws_bytes;
    gp_status st = get_workspace(net, tb * total + 16384, &ws, &ws_bytes);
    if (st != GP_OK) return st;
    long long Rc_max = (ws_bytes - 16384) / tb;
    if (total >= (1LL << 31)) return fail(net, GP_ERR_SHAPE, "batch * layer size must stay below 2^31");
    // rows * window pixels of any step must stay below 2^31 (32-bit indexing in the kernels)
    long long max_pix = 1;
    for (const PlanOp& op : pl.ops)
        if (op.kind == PlanOp::CROSS) {
            const Layer& pp = net->L[op.layer_out];
            max_pix = std::max(max_pix, (long long)std::min(op.g_out.Wy, pp.H) * std::min(op.g_out.Wx, pp.W));
        }
    Rc_max = std::min(Rc_max, ((1LL << 31) - 256) / (nsign * max_pix));
    if (Rc_max <= 0) return fail(net, GP_ERR_WORKSPACE, "workspace of %lld bytes cannot hold one row (%lld bytes)", ws_bytes, tb);
    // a tile of up to 128 rows of a block is addressed through 32-bit byte offsets of one buffer resource
    if (128LL * pl.slot_elems * csize >= (1LL << 31))
        return fail(net, GP_ERR_SHAPE, "a row's coefficient block of %lld elements is too long for the kernels' 32-bit offsets", pl.slot_elems);
    // when the rows do not fit at once, chunks start at multiples of 64 tasks (kernels that want rows grouped by position)
    if (Rc_max < total && Rc_max > 64) Rc_max -= Rc_max % 64;
    Rc_max = std::min(Rc_max, total);
    const long long nrows_max = Rc_max * nsign;
    // header: per-row scalars (two copies of constant and slack), then the task lists of early termination
    double* d_cbuf[2] = {(double*)ws, (double*)ws + nrows_max};
    double* d_ebuf[2] = {(double*)ws + 2 * nrows_max, (double*)ws + 3 * nrows_max};
    double* d_best = (double*)ws + 4 * nrows_max;
    int* d_rowid[2] = {(int*)(d_best + nrows_max), (int*)(d_best + nrows_max) + Rc_max};
    int* d_sel = d_rowid[1] + Rc_max;
    int* d_wg = d_sel + Rc_max;
    const long long nwg_max = (Rc_max + 255) / 256 + 1;
    unsigned char* d_done[2] = {(unsigned char*)(d_wg + nwg_max), (unsigned char*)(d_wg + nwg_max) + Rc_max};
    const long long chunks_max = pl.slot_elems > 1024 ? (pl.slot_elems + 511) / 512 : 0;
    double* d_partial = (double*)(ws + align_up((d_done[1] + Rc_max) - (unsigned char*)ws, 256));
    char* slots0 = (char*)d_partial + align_up(nrows_max * chunks_max * 40, 256);
    const long long slot_bytes = align_up(nrows_max * pl.slot_elems * csize, 256);
    if (slots0 + slot_bytes * pl.n_slots > ws + ws_bytes) return fail(net, GP_ERR_WORKSPACE, "workspace layout overflow");

    const std::vector<double>& rem_flop = pl.rem_flop;   // per row: arithmetic of the crossings that follow each op

    for (long long row0 = 0; row0 < total; row0 += Rc_max) {
        gp::RowMap rm;
        rm.row0 = (int)row0;
        rm.Rc = (int)std::min(Rc_max, total - row0);
        rm.nsign = nsign;
        rm.n_start = (int)n_start;
        if (certify) { rm.Hs = 1; rm.Ws = 1; rm.Cs = (int)n_start; }
        else { rm.Hs = ls.H; rm.Ws = ls.W; rm.Cs = ls.C; }
        rm.div_n = gp::make_fastdiv((uint32_t)rm.n_start);
        rm.div_c = gp::make_fastdiv((uint32_t)rm.Cs);
        rm.div_w = gp::make_fastdiv((uint32_t)rm.Ws);
        rm.rowid = nullptr;
        rm.Rc0 = rm.Rc;
        const gp::RowMap rm0 = rm;            // the chunk before any removal (layout of `best`)
        int phys[kMaxSlots];
        for (int i = 0; i < kMaxSlots; ++i) phys[i] = i;
        auto slot_ptr = [&](int s) { return (float*)(slots0 + slot_bytes * phys[s]); };
        int cur = 0;                          // which copy of constant / slack / task list / flags is current
        double *d_c = d_cbuf[0], *d_err = d_ebuf[0];
        bool have_rows = false;               // constants and slack exist (an INIT has run)
        bool stop_all = false;                // every task met the criterion: skip to FINALIZE

        // Flag the tasks that meet the criterion and count the ones kept.  The count of one check is read at the
        // next one (the GPU works on the step in between, so the host does not make it wait); only when that
        // count says that removing rows pays is the stream drained for the exact count, and the rows removed.
        bool pending = false;
        auto check_termination = [&](int key, bool first, int slot, long long nelem, double rem_flop) -> gp_status {
            gp::TermParams tp;
            tp.best = d_best; tp.Rc0 = rm.Rc0; tp.rowid = rm.rowid; tp.Ra = rm.Rc;
            tp.done = d_done[cur]; tp.term_layer = ls.d_term;
            tp.row0 = rm.row0; tp.key = key; tp.first = first ? 1 : 0; tp.may_stop = may_stop ? 1 : 0;
            tp.wgcount = d_wg;
            gp::launch_term(tp, net->d_count, net->stream);
            // When all crossings still to come for this chunk take less than a few host round trips, removing rows
            // cannot pay: the flags are kept up to date (they decide what a task keeps), nothing is read back.
            if ((double)rm.Rc * nsign * rem_flop / 30e12 < 200e-6) return GP_OK;
            // removing rows costs a copy of the rows kept (and an idle moment of the GPU); the rows removed would
            // have cost their share of the crossings still to come
            auto pays = [&](int kept) {
                if (first) return kept < rm.Rc;                  // nothing to copy yet
                const double gone = (double)(rm.Rc - kept) * nsign, stay = (double)kept * nsign;
                return gone * rem_flop / 30e12 > 1.5 * (stay * (double)nelem * 8.0 / 2.5e12 + 30e-6);
            };
            bool exact = first;
            if (!first && pending) {
                HIP_TRY(net, hipEventSynchronize(net->count_ev));
                pending = false;
                const int before = net->h_count[0];
                if (before == 0) { stop_all = true; return GP_OK; }   // flags only ever grow
                exact = before > 0 && before <= rm.Rc && pays(before);
            }
            if (!exact) {
                HIP_TRY(net, hipMemcpyAsync(net->h_count, net->d_count, sizeof(int), hipMemcpyDeviceToHost, net->stream));
                HIP_TRY(net, hipEventRecord(net->count_ev, net->stream));
                pending = true;
                return GP_OK;
            }
            HIP_TRY(net, hipMemcpyAsync(net->h_count + 1, net->d_count, sizeof(int), hipMemcpyDeviceToHost, net->stream));
            HIP_TRY(net, hipStreamSynchronize(net->stream));
            const int kept = net->h_count[1];
            if (kept < 0 || kept > rm.Rc) return fail(net, GP_ERR_DEVICE, "task count out of range");
            if (kept == 0) { stop_all = true; return GP_OK; }
            if (!pays(kept)) return GP_OK;
            gp::CompactParams cp;
            cp.done = d_done[cur]; cp.wgoffset = d_wg; cp.Ra = rm.Rc;
            cp.rowid_old = rm.rowid; cp.rowid_new = d_rowid[cur ^ 1]; cp.sel = d_sel;
            cp.c_old = have_rows ? d_c : nullptr; cp.err_old = have_rows ? d_err : nullptr;
            cp.c_new = d_cbuf[cur ^ 1]; cp.err_new = d_ebuf[cur ^ 1];
            cp.count = net->d_count; cp.nsign = nsign; cp.done_new = d_done[cur ^ 1];
            gp::launch_compact(cp, net->stream);
            if (slot >= 0) {
                const int other = (slot + 1) % pl.n_slots;      // every other block is dead at a candidate
                gp::CopyRowsParams cr;
                cr.src = slot_ptr(slot); cr.dst = slot_ptr(other); cr.sel = d_sel;
                cr.Ra_old = rm.Rc; cr.Ra_new = kept; cr.nsign = nsign;
                cr.nelem = (int)nelem * (csize / 4);        // rows are copied as 4-byte words
                gp::launch_copy_rows(cr, net->stream);
                std::swap(phys[slot], phys[other]);
            }
            cur ^= 1;
            d_c = d_cbuf[cur]; d_err = d_ebuf[cur];
            rm.rowid = d_rowid[cur];
            rm.Rc = kept;
            return GP_OK;
        };

        if (early) {
            gp::SeedParams sd;
            sd.lo = ls.d_lo; sd.hi = ls.d_hi; sd.best = d_best; sd.row0 = rm.row0; sd.Rc0 = rm.Rc0;
            gp::launch_seed(sd, net->stream);
            if (may_stop) {
                st = check_termination(start, true, -1, 0, rem_flop[0]);
                if (st != GP_OK) return st;
            } else if (ls.d_term) {
                gp::launch_fill_i32(ls.d_term + row0, 0, rm.Rc, net->stream);
            }
        }
        bool gen_pending = false, gen_write = false;      // an INIT left to the scan that follows it
        gp::GenParams gen = {};
        for (size_t oi = 0; oi < pl.ops.size(); ++oi) {
            const PlanOp& op = pl.ops[oi];
            const int nrows = rm.Rc * nsign;
            if (stop_all && op.kind != PlanOp::FINALIZE) continue;
            if (op.kind == PlanOp::INIT) {
                const Layer& lo = net->L[op.layer_out];
                gp::InitParams ip;
                std::memset(&ip, 0, sizeof(ip));
                ip.out = slot_ptr(op.slot_out);
                ip.rm = rm; ip.nrows = nrows;
                ip.nelem = (int)block_elems(op.g_out, lo);
                ip.mode = (forms && op.init_mode == 1) ? 3 : op.init_mode;
                ip.labels = net->d_labels;
                ip.forms = net->d_forms;
                ip.offsets = net->forms_have_offset ? net->d_form_off : nullptr;
                ip.H = lo.H; ip.W = lo.W; ip.C = lo.C;
                if (op.init_mode == 2) {
                    ip.wy = std::min(op.g_out.Wy, lo.H); ip.wx = std::min(op.g_out.Wx, lo.W);
                    ip.Sy = op.g_out.Sy; ip.Sx = op.g_out.Sx; ip.Py = op.g_out.Py; ip.Px = op.g_out.Px;
                    ip.kh = ls.kh; ip.kw = ls.kw; ip.sh = ls.sh; ip.sw = ls.sw; ip.ph = ls.ph; ip.pw = ls.pw;
                    ip.dense = ls.type == T_DENSE ? 1 : 0;
                    ip.Cs = ls.C;
                    ip.wt = ls.d_wti; ip.bias = ls.d_bias;
                    ip.out_grl = op.relaxed ? lo.d_grl : nullptr;
                    ip.eta = net->float_inference ? ls.d_eta : nullptr;
                }
                ip.c = d_c; ip.err = d_err; ip.best = d_best;
                ip.seeded = early ? 1 : 0;
                ip.coef64 = net->coef64 ? 1 : 0;
                // The start layer's own matrix rows followed by their scan: the scan makes the rows itself (same values,
                // same roundings), so the block is not read back, and not even written when no later step reads it
                // (the first layer's rows over the input).  The bits are those of the two-kernel form, so the choice may
                // depend on the launch: with few rows the two kernels, which spread over more work-groups, are faster
                // (one box of FC 9x500: 1.40 against 1.46 ms per pass).
                gen_pending = false;
                if (op.init_mode == 2 && nrows > kGenMinRows && !net->interval && !net->coef64 && !early && !ip.eta && oi + 1 < pl.ops.size() &&
                    pl.ops[oi + 1].kind == PlanOp::SCAN && pl.ops[oi + 1].slot_in == op.slot_out && !pl.ops[oi + 1].consts_only) {
                    gen_pending = true;
                    gen.wt = ip.wt; gen.bias = ip.bias; gen.out_grl = ip.out_grl;
                    gen.H = ip.H; gen.W = ip.W; gen.C = ip.C;
                    gen.wy = ip.wy; gen.wx = ip.wx; gen.Sy = ip.Sy; gen.Sx = ip.Sx; gen.Py = ip.Py; gen.Px = ip.Px;
                    gen.kh = ip.kh; gen.kw = ip.kw; gen.sh = ip.sh; gen.sw = ip.sw; gen.ph = ip.ph; gen.pw = ip.pw;
                    gen.dense = ip.dense; gen.Cs = ip.Cs;
                    gen_write = false;
                    for (size_t k = oi + 2; k < pl.ops.size(); ++k) {
                        if (pl.ops[k].slot_in == op.slot_out || pl.ops[k].slot_add == op.slot_out) { gen_write = true; break; }
                        if (pl.ops[k].slot_out == op.slot_out) break;          // the slot is written again before anyone reads it
                    }
                } else if (net->interval) gp::launch_iv_init(ip, net->stream);
                else gp::launch_init(ip, net->stream);
                have_rows = true;
            } else if (op.kind == PlanOp::SCAN && net->interval) {
                // literal interval coefficients (Section 4.1): the candidate over the block's layer, then the ReLU
                // substitution as a step of its own (nothing is fused into the product here), then the bias constants
                const Layer& l = net->L[op.layer_in];
                gp::IvRowParams rp;
                std::memset(&rp, 0, sizeof(rp));
                rp.blk = make_desc(net, slot_ptr(op.slot_in), op.g_in, op.layer_in);
                rp.rm = rm; rp.nrows = nrows; rp.batch_stride = (int)l.n;
                rp.c = d_c; rp.best = d_best;
                if (!op.consts_only && op.update_best && has_bounds(net, op.layer_in) && op.layer_in != start) {
                    rp.xlo = l.d_lo; rp.xhi = l.d_hi;
                    gp::launch_iv_cand(rp, net->stream);
                }
                if (op.relaxed) {
                    const Layer& q = net->L[l.a];
                    rp.xlo = q.d_lo; rp.xhi = q.d_hi; rp.grl = l.d_grl;
                    gp::launch_iv_relu(rp, net->stream);
                }
                if (op.do_consts && !l.land.empty()) {
                    rp.beff = l.d_beff;
                    gp::launch_iv_bias(rp, net->stream);
                }
            } else if (op.kind == PlanOp::SCAN) {
                const Layer& l = net->L[op.layer_in];
                gp::ScanParams sp;
                sp.blk = make_desc(net, slot_ptr(op.slot_in), op.g_in, op.layer_in);
                sp.rm = rm; sp.nrows = nrows;
                sp.batch_stride = (int)l.n;
                const bool interval_terms = scan_setup(net, op, start, certify, sp);
                sp.c = d_c; sp.err = d_err; sp.best = d_best;
                sp.done = may_stop ? d_done[cur] : nullptr;
                sp.partial = chunks_max ? d_partial : nullptr;
                if (gen_pending) { sp.gen = 1; sp.gen_write = gen_write ? 1 : 0; sp.g = gen; gen_pending = false; }
                prof_mark(net, 1, false);
                gp::launch_scan(sp, net->stream);
                prof_mark(net, 1, true);
                if (net->prof_on) {
                    net->prof_bytes[1] += (double)csize * nrows * (double)block_elems(op.g_in, l);
                    net->prof_recs[1].push_back({1, start, op.layer_in, nrows, (int)block_elems(op.g_in, l), 0, l.C, 0, 0.0});
                }
                // a candidate over a hidden layer has just been folded into best: re-evaluate the criterion
                if (may_stop && op.update_best && interval_terms && op.layer_in != 0) {
                    st = check_termination(op.layer_in, false, op.slot_in, block_elems(op.g_in, l), rem_flop[oi]);
                    if (st != GP_OK) return st;
                }
            } else if (op.kind == PlanOp::CROSS) {
                const Layer& a = net->L[op.layer_in];
                const Layer& p = net->L[op.layer_out];
                gp::CrossParams cp;
                cp.in = make_desc(net, slot_ptr(op.slot_in), op.g_in, op.layer_in, &op.t_in);
                cp.out_grl = (op.relaxed && !net->interval) ? p.d_grl : nullptr;
                cp.wt = a.d_wt;
                cp.wt64 = a.d_wt64;
                cp.pool_scale = pool_scale(a);
                cp.coef64 = net->coef64 ? 1 : 0;
                cp.kh = a.kh; cp.kw = a.kw; cp.sh = a.sh; cp.sw = a.sw; cp.ph = a.ph; cp.pw = a.pw;
                cp.out = slot_ptr(op.slot_out);
                if (a.type == T_DENSE) {   // a dense layer is a 1x1 convolution over the flattened predecessor
                    cp.Ho = 1; cp.Wo = 1; cp.Co = (int)p.n;
                    cp.owy = cp.owx = 1; cp.oSy = cp.oSx = cp.oPy = cp.oPx = 0;
                    cp.add.data = nullptr;
                    if (op.slot_add >= 0) {
                        cp.add = make_desc(net, slot_ptr(op.slot_add), op.g_add, op.layer_out);
                        // full-layer addend seen as one pixel with n channels
                        cp.add.H = cp.add.W = 1; cp.add.C = (int)p.n; cp.add.wy = cp.add.wx = 1;
                        cp.add.Sy = cp.add.Sx = cp.add.Py = cp.add.Px = 0;
                    }
                } else {
                    cp.Ho = p.H; cp.Wo = p.W; cp.Co = p.C;
                    cp.owy = std::min(op.g_out.Wy, p.H); cp.owx = std::min(op.g_out.Wx, p.W);
                    cp.oSy = op.g_out.Sy; cp.oSx = op.g_out.Sx; cp.oPy = op.g_out.Py; cp.oPx = op.g_out.Px;
                    cp.add.data = nullptr;
                    if (op.slot_add >= 0) cp.add = make_desc(net, slot_ptr(op.slot_add), op.g_add, op.layer_out);
                }
                cp.rm = rm; cp.nrows = nrows;
                cp.div_owx = gp::make_fastdiv((uint32_t)cp.owx);
                cp.div_sh = gp::make_fastdiv((uint32_t)cp.sh);
                cp.div_sw = gp::make_fastdiv((uint32_t)cp.sw);
                cp.div_kw = gp::make_fastdiv((uint32_t)cp.kw);
                prof_mark(net, 0, false);
                if (net->interval) gp::launch_iv_cross(cp, net->stream);
                else gp::launch_cross(cp, net->stream);
                prof_mark(net, 0, true);
                // algorithmic work of the step (Section 2: one product M^k * F^k): every coefficient of the
                // row's block meets every filter tap and every input channel once; the one-hot start block
                // of a row is bookkeeping, not part of the method, and counts as zero
                const double in_el = (double)block_elems(op.g_in, a), out_el = (double)block_elems(op.g_out, p);
                const double taps = (a.type == T_DENSE) ? 1.0 : (double)a.kh * a.kw;
                const double cin = (a.type == T_DENSE) ? (double)p.n : (a.type == T_POOL) ? 1.0 : (double)p.C;
                const bool first = (op.layer_in == start);
                // (averaged over the start layer's positions, the part of the stored block inside the exact window)
                const double share = certify ? 1.0 : exact_share(op.g_in, op.t_in, a, ls.H, ls.W);
                const double per_row = first ? 0.0 : 2.0 * in_el * taps * cin * share;
                if (early) {
                    net->early_flop_done += per_row * nrows;
                    net->early_flop_full += per_row * rm0.Rc * nsign;
                }
                if (net->prof_on) {
                    net->prof_flop[0] += per_row * nrows;
                    net->prof_recs[0].push_back({0, start, op.layer_in, nrows, (int)in_el, (int)out_el, (int)cin, (int)(taps * a.C),
                                                 per_row * nrows});
                    net->prof_bytes[0] += (double)csize * nrows * (in_el + out_el) + 4.0 * (double)a.wt_host.size();
                }
            } else if (op.kind == PlanOp::FINALIZE) {
                if (certify) {
                    gp::launch_margins(d_best, (forms ? net->d_form_out : net->d_margins) + row0, rm0.Rc, net->d_flag, net->stream);
                } else {
                    gp::FinalizeParams fp;
                    fp.rm = rm0; fp.best = d_best;
                    fp.lo = net->L[start].d_lo; fp.hi = net->L[start].d_hi;
                    fp.xmax = net->L[start].d_xmax; fp.flag = net->d_flag;
                    fp.widen = (net->float_inference && net->L[start].type == T_ADD) ? 0x1p-24 * (1.0 + 0x1p-20) : 0.0;
                    fp.has_relu = net->relu_reader >= 0 ? 1 : 0;
                    if (fp.has_relu) fp.relu = relu_params(net, net->relu_reader, batch);
                    else std::memset(&fp.relu, 0, sizeof(fp.relu));
                    gp::launch_finalize(fp, net->stream);
                }
            }
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(net, GP_ERR_DEVICE, "kernel launch: %s", hipGetErrorString(e));
    return GP_OK;
}

gp_status check_flag(gp_net* net) {
    int flag = 0;
    HIP_TRY(net, hipMemcpyAsync(&flag, net->d_flag, sizeof(int), hipMemcpyDeviceToHost, net->stream));
    HIP_TRY(net, hipStreamSynchronize(net->stream));
    if (flag) return fail(net, GP_ERR_NONFINITE, "NaN or Inf in the inputs or in computed bounds");
    return GP_OK;
}

// all layers after the input box is on the device
gp_status analyze_layers(gp_net* net, int batch) {
    int nl = (int)net->L.size();
    std::vector<char> relu_done(nl, 0);
    for (int i = 1; i < nl; ++i) {
        Layer& l = net->L[i];
        if (l.type == T_RELU) {
            if (relu_done[i]) continue;        // written by the launch that stored its predecessor's bounds
            gp::launch_relu(relu_params(net, i, batch), net->stream);
        } else {
            if (net->float_inference && l.type == T_ADD && l.d_eta_thru) {
                gp::SumEtaParams ep;
                ep.lo = ep.hi = nullptr; ep.u = 0.0;
                ep.ea = summand_passes_eta(net, l.a) ? net->L[l.a].d_eta : nullptr;
                ep.eb = summand_passes_eta(net, l.b) ? net->L[l.b].d_eta : nullptr;
                ep.out = l.d_eta_thru; ep.total = l.n * batch;
                gp::launch_sum_eta(ep, net->stream);
            }
            if (net->early || (net->float_inference && is_affine(l))) {
                // forward interval analysis of this layer from what is known of its predecessors (Section 4.2), and/or
                // the error of its float32 evaluation given those intervals (Section 4.1)
                if (l.type == T_ADD) {
                    gp::AddIvalParams ap;
                    ap.widen = net->float_inference ? 0x1p-24 * (1.0 + 0x1p-20) : 0.0;
                    ap.alo = net->L[l.a].d_lo; ap.ahi = net->L[l.a].d_hi;
                    ap.blo = net->L[l.b].d_lo; ap.bhi = net->L[l.b].d_hi;
                    ap.lo = l.d_lo; ap.hi = l.d_hi; ap.total = l.n * batch; ap.flag = net->d_flag;
                    gp::launch_add_ival(ap, net->stream);
                } else {
                    const Layer& p = net->L[l.a];
                    gp::IvalParams ip;
                    ip.plo = p.d_lo; ip.phi = p.d_hi; ip.wt = l.d_wti; ip.bias = l.d_bias;
                    ip.pool_scale = pool_scale(l);
                    ip.lo = net->early ? l.d_lo : nullptr; ip.hi = net->early ? l.d_hi : nullptr; ip.flag = net->d_flag;
                    ip.eta = net->float_inference ? l.d_eta : nullptr;
                    if (l.type == T_DENSE) { ip.Hi = ip.Wi = 1; ip.Ci = (int)p.n; }
                    else { ip.Hi = p.H; ip.Wi = p.W; ip.Ci = p.C; }
                    ip.H = l.H; ip.W = l.W; ip.C = l.C;
                    ip.kh = l.kh; ip.kw = l.kw; ip.sh = l.sh; ip.sw = l.sw; ip.ph = l.ph; ip.pw = l.pw;
                    ip.batch = batch;
                    gp::launch_ival(ip, net->stream);
                }
            }
            if (l.need_bounds) {
                Plan* pl;
                gp_status st = get_plan(net, i, &pl);
                if (st != GP_OK) return st;
                // A ReLU layer that reads this layer: the launch that stores the layer's bounds writes the ReLU's
                // intervals and relaxation as well (same arithmetic, one launch fewer).  Early termination keeps the
                // kernel of its own (it seeds the ReLU layer's state between the two).
                net->relu_reader = -1;
                if (!net->early)
                    for (int j = i + 1; j < nl; ++j)
                        if (net->L[j].type == T_RELU && net->L[j].a == i && !relu_done[j]) { net->relu_reader = j; break; }
                st = run_plan(net, *pl, i, false, batch);
                if (net->relu_reader >= 0 && st == GP_OK) relu_done[net->relu_reader] = 1;
                net->relu_reader = -1;
                if (st != GP_OK) return st;
            }
            if (net->float_inference && l.type == T_ADD) {
                gp::SumEtaParams ep;
                ep.lo = l.d_lo; ep.hi = l.d_hi; ep.u = 0x1p-24;
                ep.ea = l.d_eta_thru; ep.eb = nullptr;
                ep.out = l.d_eta; ep.total = l.n * batch;
                gp::launch_sum_eta(ep, net->stream);
            }
        }
    }
    return GP_OK;
}

gp_status finish_analysis(gp_net* net) {
    gp_status st = check_flag(net);
    if (st != GP_OK) return st;
    net->analyzed = true;
    return GP_OK;
}

gp_status begin_analysis(gp_net* net, int batch) {
    if (!net) return GP_ERR_ARG;
    if (batch <= 0) return fail(net, GP_ERR_ARG, "batch must be positive");
    if (net->L.size() < 2) return fail(net, GP_ERR_STATE, "network has no layers");
    net->analyzed = false;
    if (net->interval && (net->early || net->float_inference))
        return fail(net, GP_ERR_UNSUPPORTED, "interval coefficients cannot be combined with early termination or float32-inference mode");
    gp_status st = prepare_topology(net);
    if (st != GP_OK) return st;
    // plan everything first so that unsupported topologies fail before any GPU work
    for (size_t i = 1; i < net->L.size(); ++i)
        if (net->L[i].type != T_RELU && net->L[i].need_bounds) {
            Plan* pl;
            st = get_plan(net, (int)i, &pl);
            if (st != GP_OK) return st;
        }
    st = ensure_device(net, batch);
    if (st != GP_OK) return st;
    net->early_flop_done = net->early_flop_full = 0.0;
    return GP_OK;
}

void enqueue_reset(gp_net* net, int batch) {
    (void)batch;
    gp::launch_fill_i32(net->d_flag, 0, 1, net->stream);
    // [layer][box capacity]: the boxes of this analysis are a prefix of every layer's segment
    gp::launch_fill_f64(net->d_xmax_all, 0.0, (long long)net->batch_cap * (long long)net->L.size(), net->stream);
}

bool same_key(const gp_net::GraphKey& a, const gp_net::GraphKey& b) {
    return a.batch == b.batch && a.centers == b.centers && a.eps == b.eps && a.clo == b.clo && a.chi == b.chi &&
           a.ws == b.ws && a.ws_bytes == b.ws_bytes && a.stream == b.stream;
}

// the library's own workspace sized for the largest plan, so that nothing allocates while launches are captured
gp_status reserve_workspace(gp_net* net, int batch) {
    if (net->ws_user) return GP_OK;
    long long want = 0;
    for (size_t i = 1; i < net->L.size(); ++i) {
        const Layer& l = net->L[i];
        if (l.type == T_RELU || !l.need_bounds) continue;
        const Plan& pl = net->plans[i];
        if (pl.valid) want = std::max(want, task_bytes(pl, 2, coef_bytes(net)) * l.n * batch + 16384);
    }
    char* ws; long long bytes;
    return get_workspace(net, want, &ws, &bytes);
}

void hwc_from_chw(const Layer& l, const float* src, double* dst) {
    long long hw = (long long)l.H * l.W;
    for (long long pix = 0; pix < hw; ++pix)
        for (int c = 0; c < l.C; ++c) dst[pix * l.C + c] = (double)src[c * hw + pix];
}

}  // namespace

// ================================================================================================
extern "C" {

const char* gp_version(void) { return "gpupoly-hip 0.1 (gfx950)"; }

gp_status gp_net_create(int32_t c, int32_t h, int32_t w, gp_net** out) {
    if (!out) return GP_ERR_ARG;
    *out = nullptr;
    if (c <= 0 || h <= 0 || w <= 0) return GP_ERR_ARG;
    if ((long long)c * h * w > (1LL << 30)) return GP_ERR_SHAPE;
    gp_net* net = new (std::nothrow) gp_net();
    if (!net) return GP_ERR_NOMEM;
    Layer in;
    in.type = T_INPUT; in.C = c; in.H = h; in.W = w; in.n = (long long)c * h * w;
    net->L.push_back(in);
    *out = net;
    return GP_OK;
}

void gp_net_destroy(gp_net* net) {
    if (!net) return;
    for (auto& l : net->L) {
        free_layer_bounds(l);
        dfree(l.d_wt); dfree(l.d_wt64); dfree(l.d_wti); dfree(l.d_bias); dfree(l.d_beff);
    }
    dfree(net->d_count);
    if (net->h_count) (void)hipHostFree(net->h_count);
    if (net->count_ev) (void)hipEventDestroy(net->count_ev);
    if (net->graph_exec) (void)hipGraphExecDestroy(net->graph_exec);
    if (net->cap_stream) (void)hipStreamDestroy(net->cap_stream);
    dfree(net->d_forms); dfree(net->d_form_off); dfree(net->d_form_out);
    dfree(net->d_xmax_all);
    dfree(net->d_flag); dfree(net->d_labels); dfree(net->d_margins); dfree(net->d_centers);
    dfree(net->ws_own);
    for (int k = 0; k < 2; ++k)
        for (hipEvent_t e : net->prof_ev[k]) (void)hipEventDestroy(e);
    delete net;
}

static gp_status check_new_layer(gp_net* net, int32_t in_layer, int32_t* layer_id) {
    if (!net) return GP_ERR_ARG;
    if (!layer_id) return fail(net, GP_ERR_ARG, "layer_id is null");
    if (in_layer < 0 || in_layer >= (int)net->L.size()) return fail(net, GP_ERR_ARG, "layer %d does not exist", in_layer);
    return GP_OK;
}

static void topology_changed(gp_net* net) {
    drop_graph(net);
    net->topo_ready = false;
    net->analyzed = false;
    net->weights_uploaded = false;
    if (net->batch_cap) {
        for (auto& l : net->L) free_layer_bounds(l);
        for (auto& l : net->L) { dfree(l.d_beff); l.d_beff = nullptr; }
        net->batch = net->batch_cap = 0;
    }
}

gp_status gp_add_dense(gp_net* net, int32_t in_layer, int32_t out_dim, const float* W, const float* b,
                       int32_t* layer_id) {
    gp_status st = check_new_layer(net, in_layer, layer_id);
    if (st != GP_OK) return st;
    if (out_dim <= 0 || !W) return fail(net, GP_ERR_ARG, "dense: bad out_dim or null weights");
    const Layer& p = net->L[in_layer];
    const long long n_in = p.n;
    // the kernels address a layer's weights through 32-bit byte offsets of a buffer resource, also in their float64
    // copy: 2^28 weights (2 GiB as float64) is the limit
    if (n_in * (long long)out_dim >= kMaxLayerWeights) return fail(net, GP_ERR_SHAPE, "dense layer too large (2^28 weights or more)");
    if (!all_finite(W, (size_t)n_in * out_dim) || (b && !all_finite(b, out_dim)))
        return fail(net, GP_ERR_NONFINITE, "dense: NaN/Inf in weights");
    Layer l;
    l.type = T_DENSE; l.a = in_layer; l.C = out_dim; l.H = 1; l.W = 1; l.n = out_dim;
    l.wt_host.resize((size_t)n_in * out_dim);
    l.wti_host.resize((size_t)n_in * out_dim);
    const long long hw = (long long)p.H * p.W;
    double rowabs = 0;
    for (int o = 0; o < out_dim; ++o) {
        double s = 0;
        const float* src = W + (size_t)o * n_in;
        for (long long pix = 0; pix < hw; ++pix)
            for (int c = 0; c < p.C; ++c) {
                float v = src[c * hw + pix];
                l.wt_host[(size_t)(pix * p.C + c) * out_dim + o] = v;    // [n_in in H,W,C order][out]
                l.wti_host[(size_t)o * n_in + (pix * p.C + c)] = v;      // [out][n_in in H,W,C order]
                s += std::fabs((double)v);
            }
        rowabs = std::max(rowabs, s);
    }
    l.rowabs = rowabs * (1.0 + 1e-9);
    l.bias_host.assign(out_dim, 0.f);
    if (b) std::copy(b, b + out_dim, l.bias_host.begin());
    net->L.push_back(std::move(l));
    topology_changed(net);
    *layer_id = (int)net->L.size() - 1;
    return GP_OK;
}

gp_status gp_add_conv2d(gp_net* net, int32_t in_layer, int32_t c_out, int32_t kh, int32_t kw, int32_t stride_h,
                        int32_t stride_w, int32_t pad_h, int32_t pad_w, const float* W, const float* b,
                        int32_t* layer_id) {
    gp_status st = check_new_layer(net, in_layer, layer_id);
    if (st != GP_OK) return st;
    if (c_out <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0 || !W)
        return fail(net, GP_ERR_ARG, "conv2d: bad argument");
    const Layer& p = net->L[in_layer];
    if (p.H + 2 * pad_h < kh || p.W + 2 * pad_w < kw) return fail(net, GP_ERR_SHAPE, "conv2d: kernel larger than padded input");
    if (pad_h >= kh || pad_w >= kw) return fail(net, GP_ERR_SHAPE, "conv2d: padding must be smaller than the kernel");
    const int ho = (p.H + 2 * pad_h - kh) / stride_h + 1, wo = (p.W + 2 * pad_w - kw) / stride_w + 1;
    if ((long long)c_out * p.C * kh * kw >= kMaxLayerWeights) return fail(net, GP_ERR_SHAPE, "conv2d: filter too large (2^28 weights or more)");
    const size_t nw = (size_t)c_out * p.C * kh * kw;
    if (!all_finite(W, nw) || (b && !all_finite(b, c_out))) return fail(net, GP_ERR_NONFINITE, "conv2d: NaN/Inf in weights");
    if ((long long)c_out * ho * wo > (1LL << 30)) return fail(net, GP_ERR_SHAPE, "conv2d: layer too large");
    Layer l;
    l.type = T_CONV; l.a = in_layer; l.C = c_out; l.H = ho; l.W = wo; l.n = (long long)c_out * ho * wo;
    l.kh = kh; l.kw = kw; l.sh = stride_h; l.sw = stride_w; l.ph = pad_h; l.pw = pad_w;
    l.wt_host.resize(nw);
    l.wti_host.resize(nw);
    double rowabs = 0;
    for (int co = 0; co < c_out; ++co) {
        double s = 0;
        for (int ci = 0; ci < p.C; ++ci)
            for (int f = 0; f < kh; ++f)
                for (int g = 0; g < kw; ++g) {
                    float v = W[(((size_t)co * p.C + ci) * kh + f) * kw + g];
                    l.wt_host[((size_t)(f * kw + g) * p.C + ci) * c_out + co] = v;
                    l.wti_host[((size_t)(f * kw + g) * c_out + co) * p.C + ci] = v;
                    s += std::fabs((double)v);
                }
        rowabs = std::max(rowabs, s);
    }
    l.rowabs = rowabs * (1.0 + 1e-9);
    l.bias_host.assign(c_out, 0.f);
    if (b) std::copy(b, b + c_out, l.bias_host.begin());
    net->L.push_back(std::move(l));
    topology_changed(net);
    *layer_id = (int)net->L.size() - 1;
    return GP_OK;
}

gp_status gp_add_avgpool2d(gp_net* net, int32_t in_layer, int32_t kh, int32_t kw, int32_t stride_h, int32_t stride_w,
                           int32_t pad_h, int32_t pad_w, int32_t* layer_id) {
    gp_status st = check_new_layer(net, in_layer, layer_id);
    if (st != GP_OK) return st;
    if (kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0)
        return fail(net, GP_ERR_ARG, "avgpool2d: bad argument");
    const Layer& p = net->L[in_layer];
    if (p.H + 2 * pad_h < kh || p.W + 2 * pad_w < kw) return fail(net, GP_ERR_SHAPE, "avgpool2d: window larger than padded input");
    if (pad_h >= kh || pad_w >= kw) return fail(net, GP_ERR_SHAPE, "avgpool2d: padding must be smaller than the window");
    if ((long long)kh * kw > (1 << 20)) return fail(net, GP_ERR_SHAPE, "avgpool2d: window too large");
    const int ho = (p.H + 2 * pad_h - kh) / stride_h + 1, wo = (p.W + 2 * pad_w - kw) / stride_w + 1;
    Layer l;
    l.type = T_POOL; l.a = in_layer; l.C = p.C; l.H = ho; l.W = wo; l.n = (long long)p.C * ho * wo;
    l.kh = kh; l.kw = kw; l.sh = stride_h; l.sw = stride_w; l.ph = pad_h; l.pw = pad_w;
    l.rowabs = 1.0 + 1e-9;             // kh*kw weights of 1/(kh*kw) each
    l.bias_host.assign(l.C, 0.f);
    net->L.push_back(std::move(l));
    topology_changed(net);
    *layer_id = (int)net->L.size() - 1;
    return GP_OK;
}

gp_status gp_add_relu(gp_net* net, int32_t in_layer, int32_t* layer_id) {
    gp_status st = check_new_layer(net, in_layer, layer_id);
    if (st != GP_OK) return st;
    const Layer& p = net->L[in_layer];
    Layer l;
    l.type = T_RELU; l.a = in_layer; l.C = p.C; l.H = p.H; l.W = p.W; l.n = p.n;
    net->L.push_back(l);
    topology_changed(net);
    *layer_id = (int)net->L.size() - 1;
    return GP_OK;
}

gp_status gp_add_residual(gp_net* net, int32_t layer_a, int32_t layer_b, int32_t* layer_id) {
    gp_status st = check_new_layer(net, layer_a, layer_id);
    if (st != GP_OK) return st;
    if (layer_b < 0 || layer_b >= (int)net->L.size()) return fail(net, GP_ERR_ARG, "layer %d does not exist", layer_b);
    const Layer &pa = net->L[layer_a], &pb = net->L[layer_b];
    if (pa.C != pb.C || pa.H != pb.H || pa.W != pb.W) return fail(net, GP_ERR_SHAPE, "residual: shapes differ");
    Layer l;
    l.type = T_ADD; l.a = layer_a; l.b = layer_b; l.C = pa.C; l.H = pa.H; l.W = pa.W; l.n = pa.n;
    net->L.push_back(l);
    topology_changed(net);
    *layer_id = (int)net->L.size() - 1;
    return GP_OK;
}

gp_status gp_request_bounds(gp_net* net, int32_t layer_id) {
    if (!net) return GP_ERR_ARG;
    if (layer_id <= 0 || layer_id >= (int)net->L.size()) return fail(net, GP_ERR_ARG, "layer %d does not exist", layer_id);
    if (net->L[layer_id].type == T_RELU) return GP_OK;
    net->L[layer_id].req_bounds = true;
    topology_changed(net);
    return GP_OK;
}

gp_status gp_set_early_termination(gp_net* net, int32_t on) {
    if (!net) return GP_ERR_ARG;
    const bool want = on != 0;
    if (want != net->early) {
        net->early = want;
        net->analyzed = false;
        if (net->batch_cap) {       // the set of layers that carry intervals changes
            drop_graph(net);
            for (auto& l : net->L) free_layer_bounds(l);
            net->batch = net->batch_cap = 0;
        }
    }
    return GP_OK;
}

gp_status gp_set_graph_replay(gp_net* net, int32_t on) {
    if (!net) return GP_ERR_ARG;
    net->graph_on = on != 0;
    if (!net->graph_on) drop_graph(net);
    return GP_OK;
}

gp_status gp_debug_set_accumulation_roundoff(gp_net* net, double unit) {
    if (!net) return GP_ERR_ARG;
    if (!(unit >= 0x1p-50) || !(unit <= 0x1p-8)) return fail(net, GP_ERR_ARG, "unit roundoff must lie in [2^-50, 2^-8]");
    drop_graph(net);
    net->acc_unit = unit;
    net->analyzed = false;
    return GP_OK;
}

gp_status gp_set_interval_coefficients(gp_net* net, int32_t on) {
    if (!net) return GP_ERR_ARG;
    drop_graph(net);
    net->interval = on != 0;
    net->analyzed = false;
    return GP_OK;
}

gp_status gp_set_chain_fusion(gp_net* net, int32_t on) {
    if (!net) return GP_ERR_ARG;
    drop_graph(net);
    net->chain_on = on != 0;
    net->analyzed = false;
    return GP_OK;
}

gp_status gp_set_coefficient_storage(gp_net* net, int32_t bits) {
    if (!net) return GP_ERR_ARG;
    if (bits != 32 && bits != 64) return fail(net, GP_ERR_ARG, "coefficient storage: 32 or 64 bits");
    drop_graph(net);
    if ((bits == 64) != net->coef64) {
        net->coef64 = bits == 64;
        net->analyzed = false;
    }
    return GP_OK;
}

gp_status gp_set_float_inference(gp_net* net, int32_t on) {
    if (!net) return GP_ERR_ARG;
    drop_graph(net);
    const bool want = on != 0;
    if (want != net->float_inference) {
        net->float_inference = want;
        net->analyzed = false;
        net->topo_ready = false;    // sum layers carry intervals in this mode
        if (net->batch_cap) {
            for (auto& l : net->L) free_layer_bounds(l);
            net->batch = net->batch_cap = 0;
        }
    }
    return GP_OK;
}

gp_status gp_get_term_layer(const gp_net* net, int32_t layer_id, int32_t batch_index, int32_t* term) {
    if (!net) return GP_ERR_ARG;
    if (!term) return fail(net, GP_ERR_ARG, "output pointer is null");
    if (layer_id <= 0 || layer_id >= (int)net->L.size() || net->L[layer_id].type == T_RELU)
        return fail(net, GP_ERR_ARG, "layer %d starts no back-substitution", layer_id);
    if (!net->analyzed || !net->early) return fail(net, GP_ERR_STATE, "no successful analysis with early termination yet");
    if (batch_index < 0 || batch_index >= net->batch) return fail(net, GP_ERR_ARG, "batch index out of range");
    const Layer& l = net->L[layer_id];
    if (!l.d_term) return fail(net, GP_ERR_STATE, "layer %d has no bounds (see gp_request_bounds)", layer_id);
    std::vector<int> t(l.n);
    HIP_TRY(net, hipMemcpy(t.data(), l.d_term + (size_t)batch_index * l.n, l.n * sizeof(int), hipMemcpyDeviceToHost));
    const long long hw = (long long)l.H * l.W;
    for (long long pix = 0; pix < hw; ++pix)
        for (int c = 0; c < l.C; ++c) term[c * hw + pix] = t[pix * l.C + c];
    return GP_OK;
}

gp_status gp_get_early_termination_stats(const gp_net* net, double* flop_done, double* flop_full) {
    if (!net || !flop_done || !flop_full) return GP_ERR_ARG;
    if (!net->analyzed || !net->early) return fail(net, GP_ERR_STATE, "no successful analysis with early termination yet");
    *flop_done = net->early_flop_done;
    *flop_full = net->early_flop_full;
    return GP_OK;
}

gp_status gp_set_stream(gp_net* net, void* hip_stream) {
    if (!net) return GP_ERR_ARG;
    net->stream = (hipStream_t)hip_stream;
    return GP_OK;
}

gp_status gp_workspace_size(const gp_net* cnet, int32_t batch, int64_t* min_bytes, int64_t* full_bytes) {
    gp_net* net = const_cast<gp_net*>(cnet);
    if (!net || batch <= 0 || !min_bytes || !full_bytes) return GP_ERR_ARG;
    gp_status st = prepare_topology(net);
    if (st != GP_OK) return st;
    long long mn = 0, full = 0;
    for (size_t i = 1; i < net->L.size(); ++i) {
        if (net->L[i].type == T_RELU || !net->L[i].need_bounds) continue;
        Plan* pl;
        st = get_plan(net, (int)i, &pl);
        if (st != GP_OK) return st;
        long long tb = task_bytes(*pl, 2, coef_bytes(net));
        mn = std::max(mn, tb + 16384);
        full = std::max(full, tb * net->L[i].n * batch + 16384);
    }
    *min_bytes = mn;
    *full_bytes = full;
    return GP_OK;
}

gp_status gp_set_workspace(gp_net* net, void* ptr_dev, int64_t bytes) {
    if (!net) return GP_ERR_ARG;
    if (ptr_dev && (bytes <= 0 || ((uintptr_t)ptr_dev & 255))) return fail(net, GP_ERR_ARG, "workspace must be 256-byte aligned and non-empty");
    net->ws_user = ptr_dev;
    net->ws_user_bytes = ptr_dev ? bytes : 0;
    return GP_OK;
}

gp_status gp_analyze_batch_dev(gp_net* net, int32_t batch, const float* centers_dev, float eps, float clip_lo,
                               float clip_hi) {
    if (!net) return GP_ERR_ARG;
    if (!centers_dev) return fail(net, GP_ERR_ARG, "centers is null");
    if (!(eps >= 0.f) || !std::isfinite(eps)) return fail(net, GP_ERR_ARG, "eps must be finite and >= 0");
    if (!(clip_lo <= clip_hi)) return fail(net, GP_ERR_ARG, "clip_lo > clip_hi");
    gp_status st = begin_analysis(net, batch);
    if (st != GP_OK) return st;
    const Layer& in = net->L[0];
    gp::BoxParams bp;
    bp.centers = centers_dev; bp.eps = eps; bp.clip_lo = clip_lo; bp.clip_hi = clip_hi;
    bp.lo = in.d_lo; bp.hi = in.d_hi; bp.xmax = in.d_xmax; bp.flag = net->d_flag;
    bp.C = in.C; bp.H = in.H; bp.W = in.W; bp.batch = batch;
    auto enqueue = [&]() -> gp_status {
        enqueue_reset(net, batch);
        gp::launch_box(bp, net->stream);
        return analyze_layers(net, batch);
    };
    // early termination reads counts back between the steps and profiling records events: both stay eager
    if (!net->graph_on || net->early || net->prof_on) {
        st = enqueue();
        if (st != GP_OK) return st;
        return finish_analysis(net);
    }
    const gp_net::GraphKey key = {batch, centers_dev, eps, clip_lo, clip_hi, net->ws_user, net->ws_user_bytes, net->stream};
    if (!net->graph_exec || !same_key(key, net->graph_key)) {
        drop_graph(net);
        st = reserve_workspace(net, batch);
        if (st != GP_OK) return st;
        HIP_TRY(net, hipStreamSynchronize(net->stream));
        if (!net->cap_stream) HIP_TRY(net, hipStreamCreateWithFlags(&net->cap_stream, hipStreamNonBlocking));
        hipStream_t const user = net->stream;
        HIP_TRY(net, hipStreamBeginCapture(net->cap_stream, hipStreamCaptureModeThreadLocal));
        net->stream = net->cap_stream;
        st = enqueue();
        net->stream = user;
        hipGraph_t graph = nullptr;
        const hipError_t ec = hipStreamEndCapture(net->cap_stream, &graph);
        if (st != GP_OK) { if (graph) (void)hipGraphDestroy(graph); return st; }
        if (ec != hipSuccess || !graph) return fail(net, GP_ERR_DEVICE, "graph capture: %s", hipGetErrorString(ec));
        const hipError_t ei = hipGraphInstantiate(&net->graph_exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (ei != hipSuccess) { net->graph_exec = nullptr; return fail(net, GP_ERR_DEVICE, "graph instantiate: %s", hipGetErrorString(ei)); }
        net->graph_key = key;
    }
    HIP_TRY(net, hipGraphLaunch(net->graph_exec, net->stream));
    return finish_analysis(net);
}

// bounds of a layer from the library's [box][y][x][channel] arrays into the caller's [box][channel][y][x] arrays
__global__ void export_bounds_kernel(const double* lo, const double* hi, double* out_lo, double* out_hi, int C, int HW,
                                     long long total) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const long long n = (long long)C * HW, b = i / n, r = i - b * n;
    const long long pix = r / C, c = r - pix * C;
    const long long o = b * n + c * HW + pix;
    out_lo[o] = lo[i];
    out_hi[o] = hi[i];
}

gp_status gp_analyze_batch_dev_static(gp_net* net, int32_t batch, const float* centers_dev, float eps, float clip_lo,
                                      float clip_hi, double* lower_dev, double* upper_dev) {
    if (!net) return GP_ERR_ARG;
    if (!centers_dev || !lower_dev || !upper_dev) return fail(net, GP_ERR_ARG, "centers, lower or upper is null");
    if (batch <= 0) return fail(net, GP_ERR_ARG, "batch must be positive");
    if (!(eps >= 0.f) || !std::isfinite(eps)) return fail(net, GP_ERR_ARG, "eps must be finite and >= 0");
    if (!(clip_lo <= clip_hi)) return fail(net, GP_ERR_ARG, "clip_lo > clip_hi");
    if (net->L.size() < 2) return fail(net, GP_ERR_STATE, "network has no layers");
    if (net->prof_on) return fail(net, GP_ERR_STATE, "per-kernel profiling creates events: switch it off for the allocation-free call");
    // the static workspace must hold at least one row (both signs) of every plan; this needs the topology only
    gp_status st = prepare_topology(net);
    if (st != GP_OK) return st;
    for (size_t i = 1; i < net->L.size(); ++i) {
        if (net->L[i].type == T_RELU || !net->L[i].need_bounds) continue;
        Plan* pl;
        st = get_plan(net, (int)i, &pl);
        if (st != GP_OK) return st;
        const long long need = task_bytes(*pl, 2, coef_bytes(net)) + 16384;
        if (need > kStaticScratchBytes)
            return fail(net, GP_ERR_WORKSPACE, "one row of layer %d needs %lld bytes of workspace; the static workspace of the "
                                               "allocation-free call holds %lld", (int)i, need, kStaticScratchBytes);
    }
    int ndev = 0, dev = -1;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return fail(net, GP_ERR_DEVICE, "no HIP device");
    HIP_TRY(net, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(net, GP_ERR_DEVICE, "device index %d out of range", dev);
    if (net->device >= 0 && net->device != dev) return fail(net, GP_ERR_STATE, "the net lives on device %d, the current device is %d", net->device, dev);
    // (looked up by the analysis that sized the per-layer arrays: the runtime may materialise the array at the first lookup)
    if (!g_scratch_ptr[dev]) return fail(net, GP_ERR_STATE, "no analysis has run on device %d yet: the static workspace has no address", dev);
    net->static_call = true;
    net->static_ws = g_scratch_ptr[dev];
    auto run = [&]() -> gp_status {
        gp_status s2 = begin_analysis(net, batch);
        if (s2 != GP_OK) return s2;
        const Layer& in = net->L[0];
        gp::BoxParams bp;
        bp.centers = centers_dev; bp.eps = eps; bp.clip_lo = clip_lo; bp.clip_hi = clip_hi;
        bp.lo = in.d_lo; bp.hi = in.d_hi; bp.xmax = in.d_xmax; bp.flag = net->d_flag;
        bp.C = in.C; bp.H = in.H; bp.W = in.W; bp.batch = batch;
        enqueue_reset(net, batch);
        gp::launch_box(bp, net->stream);
        s2 = analyze_layers(net, batch);
        if (s2 != GP_OK) return s2;
        const Layer& out = net->L.back();
        const long long total = out.n * batch;
        export_bounds_kernel<<<(unsigned)((total + 255) / 256), 256, 0, net->stream>>>(out.d_lo, out.d_hi, lower_dev, upper_dev, out.C,
                                                                                        out.H * out.W, total);
        return finish_analysis(net);
    };
    st = run();
    net->static_call = false;
    net->static_ws = nullptr;
    return st;
}

gp_status gp_analyze_batch(gp_net* net, int32_t batch, const float* centers, float eps, float clip_lo, float clip_hi) {
    if (!net) return GP_ERR_ARG;
    if (!centers) return fail(net, GP_ERR_ARG, "centers is null");
    if (batch <= 0) return fail(net, GP_ERR_ARG, "batch must be positive");
    if (!(eps >= 0.f) || !std::isfinite(eps)) return fail(net, GP_ERR_ARG, "eps must be finite and >= 0");
    if (!(clip_lo <= clip_hi)) return fail(net, GP_ERR_ARG, "clip_lo > clip_hi");
    const long long cnt = net->L[0].n * batch;
    if (!all_finite(centers, (size_t)cnt)) return fail(net, GP_ERR_NONFINITE, "NaN/Inf in the centres");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return fail(net, GP_ERR_DEVICE, "no HIP device");
    if (net->d_centers_cap < cnt) {
        dfree(net->d_centers); net->d_centers = nullptr; net->d_centers_cap = 0;
        HIP_TRY(net, hipMalloc((void**)&net->d_centers, cnt * sizeof(float)));
        net->d_centers_cap = cnt;
    }
    HIP_TRY(net, hipMemcpyAsync(net->d_centers, centers, cnt * sizeof(float), hipMemcpyHostToDevice, net->stream));
    HIP_TRY(net, hipStreamSynchronize(net->stream));
    return gp_analyze_batch_dev(net, batch, net->d_centers, eps, clip_lo, clip_hi);
}

gp_status gp_analyze(gp_net* net, const float* center, float eps, float clip_lo, float clip_hi) {
    return gp_analyze_batch(net, 1, center, eps, clip_lo, clip_hi);
}

gp_status gp_analyze_box(gp_net* net, const float* lo, const float* hi) {
    if (!net) return GP_ERR_ARG;
    if (!lo || !hi) return fail(net, GP_ERR_ARG, "box is null");
    const Layer& in = net->L[0];
    for (long long i = 0; i < in.n; ++i) {
        if (!std::isfinite(lo[i]) || !std::isfinite(hi[i])) return fail(net, GP_ERR_NONFINITE, "NaN/Inf in the box");
        if (lo[i] > hi[i]) return fail(net, GP_ERR_ARG, "box: lo > hi at %lld", i);
    }
    gp_status st = begin_analysis(net, 1);
    if (st != GP_OK) return st;
    std::vector<double> l(in.n), h(in.n);
    hwc_from_chw(in, lo, l.data());
    hwc_from_chw(in, hi, h.data());
    double xmax = 0;
    for (long long i = 0; i < in.n; ++i) xmax = std::max(xmax, std::max(std::fabs(l[i]), std::fabs(h[i])));
    HIP_TRY(net, hipMemcpyAsync(in.d_lo, l.data(), in.n * sizeof(double), hipMemcpyHostToDevice, net->stream));
    HIP_TRY(net, hipMemcpyAsync(in.d_hi, h.data(), in.n * sizeof(double), hipMemcpyHostToDevice, net->stream));
    enqueue_reset(net, 1);
    HIP_TRY(net, hipMemcpyAsync(in.d_xmax, &xmax, sizeof(double), hipMemcpyHostToDevice, net->stream));
    HIP_TRY(net, hipStreamSynchronize(net->stream));
    st = analyze_layers(net, 1);
    if (st != GP_OK) return st;
    return finish_analysis(net);
}

gp_status gp_get_bounds_f64(const gp_net* net, int32_t layer_id, int32_t batch_index, double* lower, double* upper) {
    if (!net) return GP_ERR_ARG;
    if (!lower || !upper) return fail(net, GP_ERR_ARG, "output pointer is null");
    if (layer_id < 0 || layer_id >= (int)net->L.size()) return fail(net, GP_ERR_ARG, "layer %d does not exist", layer_id);
    if (!net->analyzed) return fail(net, GP_ERR_STATE, "no successful analysis yet");
    if (batch_index < 0 || batch_index >= net->batch) return fail(net, GP_ERR_ARG, "batch index out of range");
    const Layer& l = net->L[layer_id];
    if (!has_bounds(net, layer_id) || !l.d_lo) return fail(net, GP_ERR_STATE, "layer %d has no bounds (see gp_request_bounds)", layer_id);
    std::vector<double> lo(l.n), hi(l.n);
    HIP_TRY(net, hipMemcpy(lo.data(), l.d_lo + (size_t)batch_index * l.n, l.n * sizeof(double), hipMemcpyDeviceToHost));
    HIP_TRY(net, hipMemcpy(hi.data(), l.d_hi + (size_t)batch_index * l.n, l.n * sizeof(double), hipMemcpyDeviceToHost));
    const long long hw = (long long)l.H * l.W;
    for (long long pix = 0; pix < hw; ++pix)
        for (int c = 0; c < l.C; ++c) {
            lower[c * hw + pix] = lo[pix * l.C + c];
            upper[c * hw + pix] = hi[pix * l.C + c];
        }
    return GP_OK;
}

gp_status gp_get_bounds_batch(const gp_net* net, int32_t layer_id, int32_t batch_index, float* lower, float* upper) {
    if (!net) return GP_ERR_ARG;
    if (!lower || !upper) return fail(net, GP_ERR_ARG, "output pointer is null");
    if (layer_id < 0 || layer_id >= (int)net->L.size()) return fail(net, GP_ERR_ARG, "layer %d does not exist", layer_id);
    std::vector<double> lo(net->L[layer_id].n), hi(net->L[layer_id].n);
    gp_status st = gp_get_bounds_f64(net, layer_id, batch_index, lo.data(), hi.data());
    if (st != GP_OK) return st;
    for (size_t i = 0; i < lo.size(); ++i) {
        float f = (float)lo[i];
        if ((double)f > lo[i]) f = std::nextafterf(f, -INFINITY);
        lower[i] = f;
        f = (float)hi[i];
        if ((double)f < hi[i]) f = std::nextafterf(f, INFINITY);
        upper[i] = f;
    }
    return GP_OK;
}

gp_status gp_get_bounds(const gp_net* net, int32_t layer_id, float* lower, float* upper) {
    return gp_get_bounds_batch(net, layer_id, 0, lower, upper);
}

gp_status gp_get_relu_lambda(const gp_net* net, int32_t layer_id, int32_t batch_index, int8_t* lam) {
    if (!net) return GP_ERR_ARG;
    if (!lam) return fail(net, GP_ERR_ARG, "output pointer is null");
    if (layer_id <= 0 || layer_id >= (int)net->L.size() || net->L[layer_id].type != T_RELU)
        return fail(net, GP_ERR_ARG, "layer %d is not a ReLU layer", layer_id);
    if (!net->analyzed) return fail(net, GP_ERR_STATE, "no successful analysis yet");
    if (batch_index < 0 || batch_index >= net->batch) return fail(net, GP_ERR_ARG, "batch index out of range");
    const Layer& l = net->L[layer_id];
    std::vector<float> v(l.n);
    HIP_TRY(net, hipMemcpy(v.data(), l.d_grl + (size_t)batch_index * l.n, l.n * sizeof(float), hipMemcpyDeviceToHost));
    const long long hw = (long long)l.H * l.W;
    for (long long pix = 0; pix < hw; ++pix)
        for (int c = 0; c < l.C; ++c) lam[c * hw + pix] = std::signbit(v[pix * l.C + c]) ? 0 : 1;
    return GP_OK;
}

gp_status gp_get_relu_slopes(const gp_net* net, int32_t layer_id, int32_t batch_index, float* slope) {
    if (!net) return GP_ERR_ARG;
    if (!slope) return fail(net, GP_ERR_ARG, "output pointer is null");
    if (layer_id <= 0 || layer_id >= (int)net->L.size() || net->L[layer_id].type != T_RELU)
        return fail(net, GP_ERR_ARG, "layer %d is not a ReLU layer", layer_id);
    if (!net->analyzed) return fail(net, GP_ERR_STATE, "no successful analysis yet");
    if (batch_index < 0 || batch_index >= net->batch) return fail(net, GP_ERR_ARG, "batch index out of range");
    const Layer& l = net->L[layer_id];
    std::vector<float> v(l.n);
    HIP_TRY(net, hipMemcpy(v.data(), l.d_grl + (size_t)batch_index * l.n, l.n * sizeof(float), hipMemcpyDeviceToHost));
    const long long hw = (long long)l.H * l.W;
    for (long long pix = 0; pix < hw; ++pix)
        for (int c = 0; c < l.C; ++c) slope[c * hw + pix] = std::fabs(v[pix * l.C + c]);
    return GP_OK;
}

gp_status gp_certify_batch(gp_net* net, const int32_t* labels, int32_t* verified, float* margins) {
    if (!net) return GP_ERR_ARG;
    if (!labels || !margins) return fail(net, GP_ERR_ARG, "null pointer");
    if (!net->analyzed) return fail(net, GP_ERR_STATE, "no successful analysis yet");
    const int last = (int)net->L.size() - 1;
    const Layer& lo = net->L[last];
    if (lo.type == T_RELU) return fail(net, GP_ERR_UNSUPPORTED, "the last layer must be affine or a sum");
    if (lo.n < 2) return fail(net, GP_ERR_SHAPE, "need at least two outputs");
    for (int b = 0; b < net->batch; ++b)
        if (labels[b] < 0 || labels[b] >= lo.n) return fail(net, GP_ERR_ARG, "label out of range");
    if (!net->cert_plan.valid) {
        gp_status st = build_plan(net, last, true, net->cert_plan);
        if (st != GP_OK) return st;
    }
    HIP_TRY(net, hipMemcpyAsync(net->d_labels, labels, sizeof(int) * net->batch, hipMemcpyHostToDevice, net->stream));
    HIP_TRY(net, hipStreamSynchronize(net->stream));
    gp::launch_fill_i32(net->d_flag, 0, 1, net->stream);
    gp_status st = run_plan(net, net->cert_plan, last, true, net->batch);
    if (st != GP_OK) return st;
    st = check_flag(net);
    if (st != GP_OK) return st;
    const long long cnt = (lo.n - 1) * net->batch;
    HIP_TRY(net, hipMemcpy(margins, net->d_margins, cnt * sizeof(float), hipMemcpyDeviceToHost));
    if (verified)
        for (int b = 0; b < net->batch; ++b) {
            int ok = 1;
            for (long long j = 0; j < lo.n - 1; ++j)
                if (!(margins[b * (lo.n - 1) + j] > 0.f)) ok = 0;
            verified[b] = ok;
        }
    return GP_OK;
}

gp_status gp_bound_outputs(gp_net* net, int32_t n_forms, const float* coef, const float* offset, float* lower) {
    if (!net) return GP_ERR_ARG;
    if (n_forms <= 0 || !coef || !lower) return fail(net, GP_ERR_ARG, "n_forms must be positive, coef and lower non-null");
    if (!net->analyzed) return fail(net, GP_ERR_STATE, "no successful analysis yet");
    const int last = (int)net->L.size() - 1;
    const Layer& lo = net->L[last];
    if (lo.type == T_RELU) return fail(net, GP_ERR_UNSUPPORTED, "the last layer must be affine or a sum");
    if (!all_finite(coef, (size_t)n_forms * lo.n) || (offset && !all_finite(offset, n_forms)))
        return fail(net, GP_ERR_NONFINITE, "NaN/Inf in the forms");
    if (!net->cert_plan.valid) {
        gp_status st = build_plan(net, last, true, net->cert_plan);
        if (st != GP_OK) return st;
    }
    const long long ncoef = (long long)n_forms * lo.n, nout = (long long)n_forms * net->batch;
    if (net->d_forms_cap < ncoef) {
        dfree(net->d_forms); dfree(net->d_form_off);
        net->d_forms = net->d_form_off = nullptr; net->d_forms_cap = 0;
        HIP_TRY(net, hipMalloc((void**)&net->d_forms, ncoef * sizeof(float)));
        HIP_TRY(net, hipMalloc((void**)&net->d_form_off, (size_t)n_forms * sizeof(float)));
        net->d_forms_cap = ncoef;
    }
    if (net->d_form_out_cap < nout) {
        dfree(net->d_form_out); net->d_form_out = nullptr; net->d_form_out_cap = 0;
        HIP_TRY(net, hipMalloc((void**)&net->d_form_out, nout * sizeof(float)));
        net->d_form_out_cap = nout;
    }
    HIP_TRY(net, hipMemcpyAsync(net->d_forms, coef, ncoef * sizeof(float), hipMemcpyHostToDevice, net->stream));
    if (offset)
        HIP_TRY(net, hipMemcpyAsync(net->d_form_off, offset, (size_t)n_forms * sizeof(float), hipMemcpyHostToDevice, net->stream));
    HIP_TRY(net, hipStreamSynchronize(net->stream));
    gp::launch_fill_i32(net->d_flag, 0, 1, net->stream);
    net->n_forms = n_forms;
    net->forms_have_offset = offset != nullptr;
    gp_status st = run_plan(net, net->cert_plan, last, true, net->batch);
    net->n_forms = 0;
    if (st != GP_OK) return st;
    st = check_flag(net);
    if (st != GP_OK) return st;
    HIP_TRY(net, hipMemcpy(lower, net->d_form_out, nout * sizeof(float), hipMemcpyDeviceToHost));
    return GP_OK;
}

gp_status gp_certify(gp_net* net, int32_t label, int32_t* verified, float* margins) {
    if (!net) return GP_ERR_ARG;
    if (net->analyzed && net->batch != 1) return fail(net, GP_ERR_STATE, "the last analysis was a batch: use gp_certify_batch");
    return gp_certify_batch(net, &label, verified, margins);
}

gp_status gp_debug_plan(const gp_net* cnet, int32_t layer_id, int32_t* steps, int32_t max_steps, int32_t* n_steps) {
    gp_net* net = const_cast<gp_net*>(cnet);
    if (!net || !n_steps) return GP_ERR_ARG;
    if (layer_id <= 0 || layer_id >= (int)net->L.size() || net->L[layer_id].type == T_RELU)
        return fail(net, GP_ERR_ARG, "layer %d cannot start a back-substitution", layer_id);
    gp_status st = prepare_topology(net);
    if (st != GP_OK) return st;
    Plan pl;
    st = build_plan(net, layer_id, false, pl);
    if (st != GP_OK) return st;
    int n = (int)pl.steps.size() / 8;
    *n_steps = n;
    if (steps)
        for (int i = 0; i < std::min(n, (int)max_steps) * 8; ++i) steps[i] = pl.steps[i];
    return GP_OK;
}

int32_t gp_num_layers(const gp_net* net) { return net ? (int32_t)net->L.size() : -1; }
int32_t gp_layer_size(const gp_net* net, int32_t layer_id) {
    if (!net || layer_id < 0 || layer_id >= (int)net->L.size()) return -1;
    return (int32_t)net->L[layer_id].n;
}
const char* gp_last_error(const gp_net* net) { return net ? net->err.c_str() : "null net"; }

gp_status gp_profile_enable(gp_net* net, int32_t on) {
    if (!net) return GP_ERR_ARG;
    net->prof_on = on != 0;
    for (int k = 0; k < 2; ++k) { net->prof_used[k] = 0; net->prof_flop[k] = net->prof_bytes[k] = 0.0; net->prof_recs[k].clear(); }
    return GP_OK;
}

// Writes one CSV line per profiled launch since gp_profile_enable (kernel, start layer, layer, rows, block sizes,
// N, K, algorithmic flop, duration in us); synchronises.  Call before gp_profile_read, which resets the records.
gp_status gp_profile_dump(gp_net* net, const char* path) {
    if (!net || !path) return GP_ERR_ARG;
    HIP_TRY(net, hipStreamSynchronize(net->stream));
    FILE* f = fopen(path, "w");
    if (!f) return fail(net, GP_ERR_ARG, "cannot open %s", path);
    fprintf(f, "kernel,start_layer,layer,rows,in_elems,out_elems,N,K,alg_flop,us\n");
    for (int k = 0; k < 2; ++k)
        for (size_t i = 0; i < net->prof_recs[k].size() && 2 * i + 1 < net->prof_used[k]; ++i) {
            float t = 0.f;
            (void)hipEventElapsedTime(&t, net->prof_ev[k][2 * i], net->prof_ev[k][2 * i + 1]);
            const gp_net::ProfRec& r = net->prof_recs[k][i];
            fprintf(f, "%s,%d,%d,%d,%d,%d,%d,%d,%.6g,%.2f\n", r.kind == 2 ? "chain" : k == 0 ? "cross" : "scan", r.start, r.layer, r.nrows, r.in_el,
                    r.out_el, r.n, r.k, r.flop, t * 1e3);
        }
    fclose(f);
    return GP_OK;
}

gp_status gp_profile_read(gp_net* net, int64_t* launches, double* total_ms, double* alg_flop, double* alg_bytes) {
    if (!net || !launches || !total_ms || !alg_flop || !alg_bytes) return GP_ERR_ARG;
    HIP_TRY(net, hipStreamSynchronize(net->stream));
    for (int k = 0; k < 2; ++k) {
        double ms = 0.0;
        for (size_t i = 0; i + 1 < net->prof_used[k]; i += 2) {
            float t = 0.f;
            HIP_TRY(net, hipEventElapsedTime(&t, net->prof_ev[k][i], net->prof_ev[k][i + 1]));
            ms += t;
        }
        launches[k] = (int64_t)(net->prof_used[k] / 2);
        total_ms[k] = ms;
        alg_flop[k] = net->prof_flop[k];
        alg_bytes[k] = net->prof_bytes[k];
        net->prof_used[k] = 0;
        net->prof_flop[k] = net->prof_bytes[k] = 0.0;
        net->prof_recs[k].clear();
    }
    return GP_OK;
}

// test hook: D[16][16] = A[16][K] * B[K][16] with the float64 MFMA instruction (device pointers)
gp_status gp_debug_mfma_f64(const double* A_dev, const double* B_dev, double* D_dev, int32_t K, void* hip_stream) {
    if (!A_dev || !B_dev || !D_dev || K <= 0 || (K & 3)) return GP_ERR_ARG;
    gp::launch_mfma_check(A_dev, B_dev, D_dev, K, (hipStream_t)hip_stream);
    return hipGetLastError() == hipSuccess ? GP_OK : GP_ERR_DEVICE;
}

// test hook: D[16][4] = A[16][K] * B[K][4] with the 4-column float64 MFMA instruction (device pointers)
gp_status gp_debug_mfma_f64_4col(const double* A_dev, const double* B_dev, double* D_dev, int32_t K, void* hip_stream) {
    if (!A_dev || !B_dev || !D_dev || K <= 0 || (K & 3)) return GP_ERR_ARG;
    gp::launch_mfma4_check(A_dev, B_dev, D_dev, K, (hipStream_t)hip_stream);
    return hipGetLastError() == hipSuccess ? GP_OK : GP_ERR_DEVICE;
}

}  // extern "C"

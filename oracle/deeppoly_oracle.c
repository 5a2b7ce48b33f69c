/*
 * DeepPoly back-substitution — CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call this file.
 * It shares no code with the HIP library and must never be linked or imported by it.
 *
 * What it computes (paper, Section 2 "DeepPoly analysis" and "Bottleneck Backsubstitution";
 * Section 4.1 for floating point):
 *   - every neuron of an affine layer that feeds a ReLU, and of the last layer, gets an interval
 *     [l,u] by back-substitution: start from the neuron's own affine expression, replace every
 *     neuron of the latest layer in the expression by its upper or lower polyhedral bound
 *     according to the sign of its coefficient, repeat down to the input layer, and keep the best
 *     of the candidate bounds obtained by concretising the expression with the intervals of the
 *     layer it currently ranges over;
 *   - all coefficients are intervals; every operation rounds lower ends towards -inf and upper
 *     ends towards +inf (Section 4.1), in float64.
 *
 * Representation: dense.  No dependence windows, no blocking or fusion.  Early termination
 * (Section 3.2 "Early termination", Section 4.2 "Implementing early termination") is a separate
 * mode, off by default; see dp_set_early_termination.
 * A convolution is its defining loop nest with zero padding (the index map of Algorithm 1:
 * output (y,x), tap (f,g) reads input (y*s - p + f, x*s - p + g)).  A residual sum forwards an
 * expression's coefficients to both summands (Section 3.1, "Dependence set and residual
 * networks"); the two branches meet again automatically because an expression is kept as one
 * dense coefficient vector per layer.
 *
 * Readings where the paper is silent (all listed in the design notes of the repository):
 *   - ReLU relaxation constants (the paper only says they are fixed by l,u): for l<0<u the upper
 *     line has slope g = u/(u-l) and intercept d = max(-g*l, u-g*u) rounded up (sound for any
 *     g in [0,1]); the lower line is lam*x with lam=1 iff u > -l, else 0.  l>=0: identity.
 *     u<=0: zero.
 *   - an interval coefficient that straddles zero at an unstable ReLU is replaced by the interval
 *     image of coefficient*neuron over the neuron's interval.
 *   - a candidate is evaluated whenever the expression ranges over exactly one layer that has
 *     intervals.
 *   - a label is certified by lower bounds of y_label - y_j.
 *   - width of the interval coefficients.  Section 4.1 keeps every coefficient as an interval for the
 *     whole back-substitution.  Pushed through further layers the WIDTHS are multiplied by |F| while the
 *     coefficients are multiplied by F, so relative to the coefficients they grow by about
 *     0.4*sqrt(fan-in) per layer; after some 15 convolutional layers a float64 interval is as wide as
 *     the coefficient itself and the bounds are useless (measured on a 50-layer residual net).  The
 *     paper's networks are analysed with early termination, which hides this.  Reading taken here
 *     (option collapse = 1, the default): before a layer of the expression is substituted, every
 *     interval coefficient [lo,hi] over a neuron with known interval is replaced by a point m in it
 *     and max(hi-m, m-lo) * max|neuron| is added outward to the constant.  This is sound for the same
 *     reason concretisation is, keeps float64 and outward rounding, and stops the growth.  collapse = 0
 *     is the literal scheme.
 *
 *   - rounding of the inference itself (Section 4.1, last paragraph; the paper names the goal and defers the
 *     technique to a citation).  Reading taken here, a separate mode that is off by default
 *     (dp_set_float_inference): the network is evaluated in float32, every affine neuron as a sum of float32
 *     products and its bias in ANY order, fused or not, a residual sum as one rounded addition, ReLU exactly.
 *     The classical bound for such a sum of K products and a bias is
 *         |computed - exact| <= gamma(K+1) * (sum_j |w_j|*|x_j| + |b|) + (K+1)*2^-149,   gamma(k) = k*u/(1-k*u),
 *     u = 2^-24 (the last term covers products that underflow).  With |x_j| <= max(|l_j|,|u_j|) this is a constant
 *     eta_i per neuron, and the neuron's relation becomes x_i in sum_j w_ij x_j + b_i + [-eta_i, eta_i]: substituting
 *     a coefficient a over x_i adds |a|*eta_i to the constant, outward.  A rounded addition is monotone, so the
 *     interval of a residual sum is the interval of the exact sum moved outward by u*|end|, and a coefficient a
 *     over it adds |a|*u*max|end| when it is substituted.  The analysis then bounds every such float32 evaluation
 *     (and the real-valued one).
 *
 * Neuron order inside a layer: C,H,W flattened (channel outermost).
 *
 * Pins: see tests/test_oracle_*.py (closed forms, eps=0, all-stable composition, hand example,
 * conv==dense Toeplitz, residual==dense, brute-force containment, nested boxes).
 * Parity with DeepPoly numbers on the paper's own trained networks (Tables 2-4): parity unpinned
 * (datasets and weights unavailable).
 */
#include <fenv.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#pragma STDC FENV_ACCESS ON

enum { L_INPUT = 0, L_DENSE = 1, L_CONV = 2, L_RELU = 3, L_ADD = 4, L_POOL = 5 };
enum { DP_OK = 0, DP_ERR_ARG = 1, DP_ERR_STATE = 3, DP_ERR_NOMEM = 4 };

typedef struct {
    int type, a, b;          /* predecessors (b only for L_ADD)                    */
    int C, H, W, n;
    double *wt;              /* dense [n][n_in]; conv [C][Cin][kh][kw]             */
    double *bias;            /* [n] dense, [C] conv                                */
    int kh, kw, sh, sw, ph, pw;
    double w_dn, w_up;       /* average pooling: 1/(kh*kw) rounded down / up               */
    double *lo, *hi;         /* intervals of this layer's neurons                  */
    int has_bounds, need_bounds;
    double *gam, *del;       /* ReLU: upper line gam*x+del (unstable neurons)      */
    signed char *lam;        /* ReLU: lower line lam*x                             */
    signed char *lam_force;  /* optional per-neuron override: -1 none, 0, 1        */
    double *gam_force;       /* optional per-neuron slope of the upper line (NaN: none) */
    /* early-termination mode */
    int feeds_relu, requested;
    double *ilo, *ihi;       /* interval image of the layer from its predecessors' intervals */
    int has_ival;
    int *term;               /* per neuron: layer the expression ranged over when it was dropped; the layer's own
                                id = never started; 0 = substituted down to the input                 */
    int *term_force;         /* optional per-neuron override of the decision (-1: none)               */
    /* float32-inference mode */
    double *eta;             /* per neuron: bound on |float32 evaluation - exact value| given the predecessors     */
    int has_eta;
} layer_t;

typedef struct {
    int n_layers, cap;
    layer_t *L;
    int lambda_policy;       /* 0: lam=1 iff u>-l   1: always 0   2: always 1      */
    int candidates;          /* 0: every step       1: input layer only            */
    int collapse;            /* 1: re-centre interval coefficients before each substitution (default) */
    int early_term;          /* 1: forward interval pass + termination criterion (Sections 3.2, 4.2)  */
    int float_inference;     /* 1: bounds also hold for every float32 evaluation order (Section 4.1)  */
    int analyzed;
} dp_net;

/* ---- directed rounding, valid while the thread's mode is FE_UPWARD ---------------------- */
static inline double add_up(double x, double y) { return x + y; }
static inline double add_dn(double x, double y) { return -((-x) - y); }
static inline double mul_up(double x, double y) { return x * y; }
static inline double mul_dn(double x, double y) { return -((-x) * y); }
static inline double sub_up(double x, double y) { return x - y; }
static inline double dmin(double x, double y) { return x < y ? x : y; }
static inline double dmax(double x, double y) { return x > y ? x : y; }

/* ---- construction ------------------------------------------------------------------------ */
dp_net *dp_create(int c, int h, int w) {
    if (c <= 0 || h <= 0 || w <= 0) return NULL;
    dp_net *N = (dp_net *)calloc(1, sizeof(dp_net));
    N->cap = 16;
    N->collapse = 1;
    N->L = (layer_t *)calloc(N->cap, sizeof(layer_t));
    N->n_layers = 1;
    layer_t *I = &N->L[0];
    I->type = L_INPUT; I->a = I->b = -1; I->C = c; I->H = h; I->W = w; I->n = c * h * w;
    I->lo = (double *)calloc(I->n, sizeof(double));
    I->hi = (double *)calloc(I->n, sizeof(double));
    return N;
}

static layer_t *new_layer(dp_net *N) {
    if (N->n_layers == N->cap) {
        N->cap *= 2;
        N->L = (layer_t *)realloc(N->L, N->cap * sizeof(layer_t));
    }
    layer_t *l = &N->L[N->n_layers++];
    memset(l, 0, sizeof(*l));
    l->a = l->b = -1;
    N->analyzed = 0;
    return l;
}

static void alloc_bounds(layer_t *l) {
    l->lo = (double *)calloc(l->n, sizeof(double));
    l->hi = (double *)calloc(l->n, sizeof(double));
    if (l->type != L_RELU) {
        l->ilo = (double *)calloc(l->n, sizeof(double));
        l->ihi = (double *)calloc(l->n, sizeof(double));
        l->term = (int *)calloc(l->n, sizeof(int));
        l->eta = (double *)calloc(l->n, sizeof(double));
    }
}

int dp_add_dense(dp_net *N, int src, int n_out, const float *W, const float *b) {
    if (!N || src < 0 || src >= N->n_layers || n_out <= 0 || !W) return -1;
    int n_in = N->L[src].n;
    layer_t *l = new_layer(N);
    l->type = L_DENSE; l->a = src; l->C = n_out; l->H = 1; l->W = 1; l->n = n_out;
    l->wt = (double *)malloc(sizeof(double) * (size_t)n_out * n_in);
    l->bias = (double *)calloc(n_out, sizeof(double));
    for (size_t i = 0; i < (size_t)n_out * n_in; ++i) l->wt[i] = (double)W[i];
    if (b) for (int i = 0; i < n_out; ++i) l->bias[i] = (double)b[i];
    alloc_bounds(l);
    return N->n_layers - 1;
}

int dp_add_conv2d(dp_net *N, int src, int c_out, int kh, int kw, int sh, int sw, int ph, int pw,
                  const float *W, const float *b) {
    if (!N || src < 0 || src >= N->n_layers || c_out <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 ||
        ph < 0 || pw < 0 || !W) return -1;
    layer_t *p = &N->L[src];
    int ho = (p->H + 2 * ph - kh) / sh + 1, wo = (p->W + 2 * pw - kw) / sw + 1;
    if (p->H + 2 * ph < kh || p->W + 2 * pw < kw) return -1;
    int cin = p->C;
    layer_t *l = new_layer(N);
    l->type = L_CONV; l->a = src; l->C = c_out; l->H = ho; l->W = wo; l->n = c_out * ho * wo;
    l->kh = kh; l->kw = kw; l->sh = sh; l->sw = sw; l->ph = ph; l->pw = pw;
    size_t nw = (size_t)c_out * cin * kh * kw;
    l->wt = (double *)malloc(sizeof(double) * nw);
    l->bias = (double *)calloc(c_out, sizeof(double));
    for (size_t i = 0; i < nw; ++i) l->wt[i] = (double)W[i];
    if (b) for (int i = 0; i < c_out; ++i) l->bias[i] = (double)b[i];
    alloc_bounds(l);
    return N->n_layers - 1;
}

/* Average pooling: every channel on its own, out(c,y,x) = (1/(kh*kw)) * sum of the window of in(c,.,.) at
   (y*sh - ph + f, x*sw - pw + g); positions in the zero padding add nothing and the divisor stays kh*kw.  An affine
   layer like a convolution (Section 2: the affine transformer is exact), with no stored filter. */
int dp_add_avgpool2d(dp_net *N, int src, int kh, int kw, int sh, int sw, int ph, int pw) {
    if (!N || src < 0 || src >= N->n_layers || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0) return -1;
    layer_t *p = &N->L[src];
    if (p->H + 2 * ph < kh || p->W + 2 * pw < kw) return -1;
    int ho = (p->H + 2 * ph - kh) / sh + 1, wo = (p->W + 2 * pw - kw) / sw + 1;
    int C = p->C;
    layer_t *l = new_layer(N);
    l->type = L_POOL; l->a = src; l->C = C; l->H = ho; l->W = wo; l->n = C * ho * wo;
    l->kh = kh; l->kw = kw; l->sh = sh; l->sw = sw; l->ph = ph; l->pw = pw;
    int old = fegetround();
    fesetround(FE_UPWARD);
    volatile double k = (double)kh * kw, one = 1.0;
    l->w_up = one / k;
    l->w_dn = -((-one) / k);
    fesetround(old);
    alloc_bounds(l);
    return N->n_layers - 1;
}

int dp_add_relu(dp_net *N, int src) {
    if (!N || src < 0 || src >= N->n_layers) return -1;
    layer_t *p = &N->L[src];
    int C = p->C, H = p->H, W = p->W, n = p->n;
    N->L[src].need_bounds = 1;
    N->L[src].feeds_relu = 1;
    layer_t *l = new_layer(N);
    l->type = L_RELU; l->a = src; l->C = C; l->H = H; l->W = W; l->n = n;
    alloc_bounds(l);
    l->gam = (double *)calloc(n, sizeof(double));
    l->del = (double *)calloc(n, sizeof(double));
    l->lam = (signed char *)calloc(n, 1);
    return N->n_layers - 1;
}

int dp_add_residual(dp_net *N, int a, int b) {
    if (!N || a < 0 || b < 0 || a >= N->n_layers || b >= N->n_layers) return -1;
    layer_t *pa = &N->L[a], *pb = &N->L[b];
    if (pa->C != pb->C || pa->H != pb->H || pa->W != pb->W) return -1;
    int C = pa->C, H = pa->H, W = pa->W, n = pa->n;
    layer_t *l = new_layer(N);
    l->type = L_ADD; l->a = a; l->b = b; l->C = C; l->H = H; l->W = W; l->n = n;
    alloc_bounds(l);
    return N->n_layers - 1;
}

void dp_destroy(dp_net *N) {
    if (!N) return;
    for (int i = 0; i < N->n_layers; ++i) {
        layer_t *l = &N->L[i];
        free(l->wt); free(l->bias); free(l->lo); free(l->hi); free(l->gam); free(l->del);
        free(l->lam); free(l->lam_force); free(l->gam_force);
        free(l->ilo); free(l->ihi); free(l->term); free(l->term_force); free(l->eta);
    }
    free(N->L); free(N);
}

int dp_num_layers(const dp_net *N) { return N ? N->n_layers : -1; }
int dp_layer_size(const dp_net *N, int lid) { return (N && lid >= 0 && lid < N->n_layers) ? N->L[lid].n : -1; }
int dp_set_options(dp_net *N, int lambda_policy, int candidates) {
    if (!N || lambda_policy < 0 || lambda_policy > 2 || candidates < 0 || candidates > 1) return DP_ERR_ARG;
    N->lambda_policy = lambda_policy; N->candidates = candidates;
    return DP_OK;
}
int dp_set_collapse(dp_net *N, int on) {
    if (!N) return DP_ERR_ARG;
    N->collapse = on ? 1 : 0;
    return DP_OK;
}
int dp_request_bounds(dp_net *N, int lid) {
    if (!N || lid <= 0 || lid >= N->n_layers) return DP_ERR_ARG;
    N->L[lid].need_bounds = 1;
    N->L[lid].requested = 1;
    return DP_OK;
}
/* Early termination (Section 3.2: a neuron whose interval does not strictly contain 0 has an exact ReLU
   relaxation and gains nothing from further back-substitution; Section 4.2: a forward interval pass gives
   the first intervals, only the other neurons of a ReLU's input layer are back-substituted, and during the
   back-substitution the criterion is checked again whenever a candidate has been evaluated). */
int dp_set_early_termination(dp_net *N, int on) {
    if (!N) return DP_ERR_ARG;
    N->early_term = on ? 1 : 0;
    N->analyzed = 0;
    return DP_OK;
}
/* Bounds that also hold for every float32 evaluation of the network (any summation order, fused or unfused
   multiply-add; Section 4.1, last paragraph).  See the header for the error model. */
int dp_set_float_inference(dp_net *N, int on) {
    if (!N) return DP_ERR_ARG;
    N->float_inference = on ? 1 : 0;
    for (int i = 0; i < N->n_layers; ++i) N->L[i].has_eta = 0;
    N->analyzed = 0;
    return DP_OK;
}
int dp_get_inference_error(const dp_net *N, int lid, double *eta) {
    if (!N || lid <= 0 || lid >= N->n_layers || !N->L[lid].has_eta) return DP_ERR_STATE;
    memcpy(eta, N->L[lid].eta, sizeof(double) * N->L[lid].n);
    return DP_OK;
}
/* term[i] >= 0 fixes where neuron i of layer lid stops: lid = it is not back-substituted at all, k = right
   after the candidate over layer k, 0 = at the input; -1 leaves the decision to the criterion.  NULL removes
   the override.  Only used in early-termination mode. */
int dp_set_term_override(dp_net *N, int lid, const int *term) {
    if (!N || lid <= 0 || lid >= N->n_layers || N->L[lid].type == L_RELU) return DP_ERR_ARG;
    layer_t *l = &N->L[lid];
    free(l->term_force); l->term_force = NULL;
    if (term) { l->term_force = (int *)malloc(sizeof(int) * l->n); memcpy(l->term_force, term, sizeof(int) * l->n); }
    return DP_OK;
}
int dp_get_term_layer(const dp_net *N, int lid, int *term) {
    if (!N || lid <= 0 || lid >= N->n_layers || N->L[lid].type == L_RELU || !term) return DP_ERR_ARG;
    if (!N->L[lid].has_bounds || !N->early_term) return DP_ERR_STATE;
    memcpy(term, N->L[lid].term, sizeof(int) * N->L[lid].n);
    return DP_OK;
}
/* the interval image of a layer (early-termination mode; also for layers without back-substituted bounds) */
int dp_get_interval_image(const dp_net *N, int lid, double *lo, double *hi) {
    if (!N || lid <= 0 || lid >= N->n_layers || N->L[lid].type == L_RELU) return DP_ERR_ARG;
    if (!N->L[lid].has_ival) return DP_ERR_STATE;
    memcpy(lo, N->L[lid].ilo, sizeof(double) * N->L[lid].n);
    memcpy(hi, N->L[lid].ihi, sizeof(double) * N->L[lid].n);
    return DP_OK;
}
/* force[i] in {-1 (no override), 0, 1}; NULL removes the override.  lid is a ReLU layer. */
int dp_set_lambda_override(dp_net *N, int lid, const signed char *force) {
    if (!N || lid <= 0 || lid >= N->n_layers || N->L[lid].type != L_RELU) return DP_ERR_ARG;
    layer_t *l = &N->L[lid];
    free(l->lam_force); l->lam_force = NULL;
    if (force) { l->lam_force = (signed char *)malloc(l->n); memcpy(l->lam_force, force, l->n); }
    return DP_OK;
}

/* gam[i]: slope to use for the upper line of unstable neuron i (any value in [0,1] is sound, see relu_layer);
   NaN entries and NULL mean "the oracle's own choice".  lid is a ReLU layer. */
int dp_set_gamma_override(dp_net *N, int lid, const double *gam) {
    if (!N || lid <= 0 || lid >= N->n_layers || N->L[lid].type != L_RELU) return DP_ERR_ARG;
    layer_t *l = &N->L[lid];
    free(l->gam_force); l->gam_force = NULL;
    if (gam) { l->gam_force = (double *)malloc(sizeof(double) * l->n); memcpy(l->gam_force, gam, sizeof(double) * l->n); }
    return DP_OK;
}

/* ---- input box (paper, Section 2: the L-infinity ball around the image, here clipped) ------ */
int dp_set_box(dp_net *N, const double *lo, const double *hi) {
    if (!N || !lo || !hi) return DP_ERR_ARG;
    layer_t *I = &N->L[0];
    for (int i = 0; i < I->n; ++i) {
        if (!(lo[i] <= hi[i]) || !isfinite(lo[i]) || !isfinite(hi[i])) return DP_ERR_ARG;
    }
    memcpy(I->lo, lo, sizeof(double) * I->n);
    memcpy(I->hi, hi, sizeof(double) * I->n);
    I->has_bounds = 1;
    for (int i = 1; i < N->n_layers; ++i) { N->L[i].has_bounds = 0; N->L[i].has_ival = 0; }
    N->analyzed = 0;
    return DP_OK;
}

int dp_set_ball(dp_net *N, const float *center, float eps, float clip_lo, float clip_hi) {
    if (!N || !center || !(eps >= 0.0f) || !(clip_lo <= clip_hi)) return DP_ERR_ARG;
    layer_t *I = &N->L[0];
    double *lo = (double *)malloc(sizeof(double) * I->n), *hi = (double *)malloc(sizeof(double) * I->n);
    int old = fegetround();
    fesetround(FE_UPWARD);
    for (int i = 0; i < I->n; ++i) {
        double c = (double)center[i], e = (double)eps;
        lo[i] = dmax(add_dn(c, -e), (double)clip_lo);
        hi[i] = dmin(add_up(c, e), (double)clip_hi);
        if (lo[i] > hi[i]) { /* centre outside the clip range: degenerate to the nearest clip end */
            if (c < (double)clip_lo) lo[i] = hi[i] = (double)clip_lo; else lo[i] = hi[i] = (double)clip_hi;
        }
    }
    fesetround(old);
    int rc = dp_set_box(N, lo, hi);
    free(lo); free(hi);
    return rc;
}

/* teacher forcing: install intervals computed elsewhere as this layer's intervals */
int dp_set_bounds(dp_net *N, int lid, const double *lo, const double *hi) {
    if (!N || lid <= 0 || lid >= N->n_layers || !lo || !hi) return DP_ERR_ARG;
    layer_t *l = &N->L[lid];
    memcpy(l->lo, lo, sizeof(double) * l->n);
    memcpy(l->hi, hi, sizeof(double) * l->n);
    l->has_bounds = 1;
    return DP_OK;
}

int dp_get_bounds(const dp_net *N, int lid, double *lo, double *hi) {
    if (!N || lid < 0 || lid >= N->n_layers) return DP_ERR_ARG;
    const layer_t *l = &N->L[lid];
    if (!l->has_bounds) return DP_ERR_STATE;
    memcpy(lo, l->lo, sizeof(double) * l->n);
    memcpy(hi, l->hi, sizeof(double) * l->n);
    return DP_OK;
}

int dp_get_relaxation(const dp_net *N, int lid, double *gam, double *del, signed char *lam) {
    if (!N || lid <= 0 || lid >= N->n_layers || N->L[lid].type != L_RELU) return DP_ERR_ARG;
    const layer_t *l = &N->L[lid];
    if (!l->has_bounds) return DP_ERR_STATE;
    memcpy(gam, l->gam, sizeof(double) * l->n);
    memcpy(del, l->del, sizeof(double) * l->n);
    memcpy(lam, l->lam, l->n);
    return DP_OK;
}

/* ---- ReLU layer: intervals and relaxation constants from the predecessor's intervals -------- */
/* must run with FE_UPWARD */
static void relu_layer(dp_net *N, int lid) {
    layer_t *r = &N->L[lid];
    const layer_t *p = &N->L[r->a];
    for (int i = 0; i < r->n; ++i) {
        double l = p->lo[i], u = p->hi[i];
        r->lo[i] = dmax(l, 0.0);
        r->hi[i] = dmax(u, 0.0);
        if (l >= 0.0) { r->gam[i] = 1.0; r->del[i] = 0.0; r->lam[i] = 1; }
        else if (u <= 0.0) { r->gam[i] = 0.0; r->del[i] = 0.0; r->lam[i] = 0; }
        else {
            double g = u / sub_up(u, l);           /* any value in [0,1] is sound */
            if (r->gam_force && r->gam_force[i] == r->gam_force[i]) g = r->gam_force[i];
            if (g > 1.0) g = 1.0;
            if (g < 0.0) g = 0.0;
            double d1 = mul_up(-l, g);             /* -g*l, rounded up            */
            double d2 = sub_up(u, mul_dn(g, u));   /* u - g*u, rounded up         */
            r->gam[i] = g;
            r->del[i] = dmax(d1, d2);
            int lam;
            if (N->lambda_policy == 1) lam = 0;
            else if (N->lambda_policy == 2) lam = 1;
            else lam = (u > -l) ? 1 : 0;
            if (r->lam_force && r->lam_force[i] >= 0) lam = r->lam_force[i] ? 1 : 0;
            r->lam[i] = (signed char)lam;
        }
    }
    r->has_bounds = 1;
}

/* ---- one expression: per layer a dense vector of interval coefficients + interval constant -- */
typedef struct {
    int n_layers;
    double **lo, **hi;       /* [layer][neuron]                                           */
    int *active;             /* layer has (possibly) non-zero coefficients                */
    double clo, chi;
} expr_t;

static expr_t *expr_new(const dp_net *N) {
    expr_t *e = (expr_t *)calloc(1, sizeof(expr_t));
    e->n_layers = N->n_layers;
    e->lo = (double **)calloc(N->n_layers, sizeof(double *));
    e->hi = (double **)calloc(N->n_layers, sizeof(double *));
    e->active = (int *)calloc(N->n_layers, sizeof(int));
    for (int i = 0; i < N->n_layers; ++i) {
        e->lo[i] = (double *)calloc(N->L[i].n, sizeof(double));
        e->hi[i] = (double *)calloc(N->L[i].n, sizeof(double));
    }
    return e;
}
static void expr_free(expr_t *e) {
    for (int i = 0; i < e->n_layers; ++i) { free(e->lo[i]); free(e->hi[i]); }
    free(e->lo); free(e->hi); free(e->active); free(e);
}
static void expr_clear(expr_t *e, const dp_net *N) {
    for (int i = 0; i < e->n_layers; ++i)
        if (e->active[i]) {
            memset(e->lo[i], 0, sizeof(double) * N->L[i].n);
            memset(e->hi[i], 0, sizeof(double) * N->L[i].n);
            e->active[i] = 0;
        }
    e->clo = e->chi = 0.0;
}

/* coefficient interval [alo,ahi] times scalar w, accumulated outward into (*lo,*hi) */
static inline void acc_scaled(double *lo, double *hi, double alo, double ahi, double w) {
    if (w >= 0.0) { *lo = add_dn(*lo, mul_dn(alo, w)); *hi = add_up(*hi, mul_up(ahi, w)); }
    else          { *lo = add_dn(*lo, mul_dn(ahi, w)); *hi = add_up(*hi, mul_up(alo, w)); }
}

/* float32-inference mode: the neuron the coefficient [a,b] stood over is its exact expression plus an error in
   [-eta, eta] */
static inline void acc_error(expr_t *e, double a, double b, double eta) {
    double s = mul_up(dmax(fabs(a), fabs(b)), eta);
    e->chi = add_up(e->chi, s);
    e->clo = add_dn(e->clo, -s);
}

/* candidate bound of the expression part that ranges over layer k (sense +1: upper, -1: lower) */
static double concretise(const dp_net *N, const expr_t *e, int k, int sense) {
    const layer_t *l = &N->L[k];
    const double *alo = e->lo[k], *ahi = e->hi[k];
    double acc = (sense > 0) ? e->chi : e->clo;
    for (int j = 0; j < l->n; ++j) {
        double a = alo[j], b = ahi[j];
        if (a == 0.0 && b == 0.0) continue;
        double L = l->lo[j], U = l->hi[j];
        if (sense > 0) {
            double m = dmax(dmax(mul_up(a, L), mul_up(a, U)), dmax(mul_up(b, L), mul_up(b, U)));
            acc = add_up(acc, m);
        } else {
            double m = dmin(dmin(mul_dn(a, L), mul_dn(a, U)), dmin(mul_dn(b, L), mul_dn(b, U)));
            acc = add_dn(acc, m);
        }
    }
    return acc;
}

/* Replace every interval coefficient over layer k by a point inside it; the part given up,
   |coefficient - point| <= w, can change the expression by at most w * max|x_j|, which goes into the
   constant on the side that keeps the bound valid. */
static void collapse_width(const dp_net *N, expr_t *e, int k, int sense) {
    const layer_t *l = &N->L[k];
    double *alo = e->lo[k], *ahi = e->hi[k];
    for (int j = 0; j < l->n; ++j) {
        double a = alo[j], b = ahi[j];
        if (a == b) continue;
        double m = a + (b - a) * 0.5;
        if (!(m >= a && m <= b)) m = a;
        double w = dmax(sub_up(b, m), sub_up(m, a));
        double X = dmax(fabs(l->lo[j]), fabs(l->hi[j]));
        double slack = mul_up(w, X);
        if (sense > 0) e->chi = add_up(e->chi, slack);
        else e->clo = add_dn(e->clo, -slack);
        alo[j] = ahi[j] = m;
    }
}

/* substitute the ReLU layer k: its neurons are replaced by their relaxation over layer a */
static void step_relu(const dp_net *N, expr_t *e, int k, int sense) {
    const layer_t *r = &N->L[k];
    const layer_t *p = &N->L[r->a];
    double *slo = e->lo[k], *shi = e->hi[k];
    double *dlo = e->lo[r->a], *dhi = e->hi[r->a];
    for (int j = 0; j < r->n; ++j) {
        double a = slo[j], b = shi[j];
        if (a == 0.0 && b == 0.0) continue;
        double l = p->lo[j], u = p->hi[j];
        if (l >= 0.0) {                       /* y = x exactly */
            dlo[j] = add_dn(dlo[j], a); dhi[j] = add_up(dhi[j], b);
        } else if (u <= 0.0) {                /* y = 0 exactly */
        } else {
            /* which line bounds coefficient*y from the side we need? */
            int use_upper_line, straddle = 0;
            if (a >= 0.0) use_upper_line = (sense > 0);
            else if (b <= 0.0) use_upper_line = (sense < 0);
            else { straddle = 1; use_upper_line = 0; }
            if (straddle) {
                double L = r->lo[j], U = r->hi[j];
                if (sense > 0) {
                    double m = dmax(dmax(mul_up(a, L), mul_up(a, U)), dmax(mul_up(b, L), mul_up(b, U)));
                    e->chi = add_up(e->chi, m); e->clo = add_dn(e->clo, m);
                } else {
                    double m = dmin(dmin(mul_dn(a, L), mul_dn(a, U)), dmin(mul_dn(b, L), mul_dn(b, U)));
                    e->chi = add_up(e->chi, m); e->clo = add_dn(e->clo, m);
                }
            } else if (use_upper_line) {
                double g = r->gam[j], d = r->del[j];
                acc_scaled(&dlo[j], &dhi[j], a, b, g);
                acc_scaled(&e->clo, &e->chi, a, b, d);
            } else {
                if (r->lam[j]) { dlo[j] = add_dn(dlo[j], a); dhi[j] = add_up(dhi[j], b); }
            }
        }
        slo[j] = shi[j] = 0.0;
    }
    e->active[k] = 0;
    e->active[r->a] = 1;
}

static void step_dense(const dp_net *N, expr_t *e, int k) {
    const layer_t *d = &N->L[k];
    int n_in = N->L[d->a].n;
    double *slo = e->lo[k], *shi = e->hi[k];
    double *dlo = e->lo[d->a], *dhi = e->hi[d->a];
    for (int i = 0; i < d->n; ++i) {
        double a = slo[i], b = shi[i];
        if (a == 0.0 && b == 0.0) continue;
        const double *w = d->wt + (size_t)i * n_in;
        for (int j = 0; j < n_in; ++j) acc_scaled(&dlo[j], &dhi[j], a, b, w[j]);
        acc_scaled(&e->clo, &e->chi, a, b, d->bias[i]);
        if (d->has_eta) acc_error(e, a, b, d->eta[i]);
        slo[i] = shi[i] = 0.0;
    }
    e->active[k] = 0;
    e->active[d->a] = 1;
}

static void step_conv(const dp_net *N, expr_t *e, int k) {
    const layer_t *c = &N->L[k];
    const layer_t *p = &N->L[c->a];
    double *slo = e->lo[k], *shi = e->hi[k];
    double *dlo = e->lo[c->a], *dhi = e->hi[c->a];
    for (int d = 0; d < c->C; ++d)
        for (int y = 0; y < c->H; ++y)
            for (int x = 0; x < c->W; ++x) {
                int i = (d * c->H + y) * c->W + x;
                double a = slo[i], b = shi[i];
                if (a == 0.0 && b == 0.0) continue;
                for (int ci = 0; ci < p->C; ++ci)
                    for (int f = 0; f < c->kh; ++f) {
                        int iy = y * c->sh - c->ph + f;
                        if (iy < 0 || iy >= p->H) continue;
                        for (int g = 0; g < c->kw; ++g) {
                            int ix = x * c->sw - c->pw + g;
                            if (ix < 0 || ix >= p->W) continue;
                            double w = c->wt[(((size_t)d * p->C + ci) * c->kh + f) * c->kw + g];
                            int j = (ci * p->H + iy) * p->W + ix;
                            acc_scaled(&dlo[j], &dhi[j], a, b, w);
                        }
                    }
                acc_scaled(&e->clo, &e->chi, a, b, c->bias[d]);
                if (c->has_eta) acc_error(e, a, b, c->eta[i]);
                slo[i] = shi[i] = 0.0;
            }
    e->active[k] = 0;
    e->active[c->a] = 1;
}

/* coefficient interval [alo,ahi] times the pooling weight, known only as w_dn <= 1/(kh*kw) <= w_up (both > 0) */
static inline void acc_pooled(double *lo, double *hi, double alo, double ahi, double w_dn, double w_up) {
    *lo = add_dn(*lo, alo >= 0.0 ? mul_dn(alo, w_dn) : mul_dn(alo, w_up));
    *hi = add_up(*hi, ahi >= 0.0 ? mul_up(ahi, w_up) : mul_up(ahi, w_dn));
}

static void step_pool(const dp_net *N, expr_t *e, int k) {
    const layer_t *c = &N->L[k];
    const layer_t *p = &N->L[c->a];
    double *slo = e->lo[k], *shi = e->hi[k];
    double *dlo = e->lo[c->a], *dhi = e->hi[c->a];
    for (int d = 0; d < c->C; ++d)
        for (int y = 0; y < c->H; ++y)
            for (int x = 0; x < c->W; ++x) {
                int i = (d * c->H + y) * c->W + x;
                double a = slo[i], b = shi[i];
                if (a == 0.0 && b == 0.0) continue;
                for (int f = 0; f < c->kh; ++f) {
                    int iy = y * c->sh - c->ph + f;
                    if (iy < 0 || iy >= p->H) continue;
                    for (int g = 0; g < c->kw; ++g) {
                        int ix = x * c->sw - c->pw + g;
                        if (ix < 0 || ix >= p->W) continue;
                        int j = (d * p->H + iy) * p->W + ix;
                        acc_pooled(&dlo[j], &dhi[j], a, b, c->w_dn, c->w_up);
                    }
                }
                if (c->has_eta) acc_error(e, a, b, c->eta[i]);
                slo[i] = shi[i] = 0.0;
            }
    e->active[k] = 0;
    e->active[c->a] = 1;
}

static void step_add(const dp_net *N, expr_t *e, int k) {
    const layer_t *s = &N->L[k];
    double *slo = e->lo[k], *shi = e->hi[k];
    for (int j = 0; j < s->n; ++j) {
        double a = slo[j], b = shi[j];
        if (a == 0.0 && b == 0.0) continue;
        e->lo[s->a][j] = add_dn(e->lo[s->a][j], a); e->hi[s->a][j] = add_up(e->hi[s->a][j], b);
        e->lo[s->b][j] = add_dn(e->lo[s->b][j], a); e->hi[s->b][j] = add_up(e->hi[s->b][j], b);
        if (s->has_eta) acc_error(e, a, b, s->eta[j]);
        slo[j] = shi[j] = 0.0;
    }
    e->active[k] = 0;
    e->active[s->a] = 1;
    e->active[s->b] = 1;
}

/* Back-substitute the expression down to the input layer; return the best candidate. */
static double backsubstitute(const dp_net *N, expr_t *e, int sense) {
    double best = (sense > 0) ? INFINITY : -INFINITY;
    for (;;) {
        int k = -1, count = 0;
        for (int i = N->n_layers - 1; i >= 0; --i)
            if (e->active[i]) { if (k < 0) k = i; ++count; }
        if (k < 0) {           /* constant expression */
            double v = (sense > 0) ? e->chi : e->clo;
            return (sense > 0) ? dmin(best, v) : dmax(best, v);
        }
        if (N->collapse && N->L[k].has_bounds) collapse_width(N, e, k, sense);
        if (count == 1 && N->L[k].has_bounds && (k == 0 || N->candidates == 0)) {
            double v = concretise(N, e, k, sense);
            best = (sense > 0) ? dmin(best, v) : dmax(best, v);
        }
        if (k == 0) return best;
        switch (N->L[k].type) {
            case L_RELU:  step_relu(N, e, k, sense); break;
            case L_DENSE: step_dense(N, e, k); break;
            case L_CONV:  step_conv(N, e, k); break;
            case L_POOL:  step_pool(N, e, k); break;
            case L_ADD:   step_add(N, e, k); break;
            default: return NAN;
        }
    }
}

/* ---- float32-inference mode (Section 4.1, last paragraph) ------------------------------------------- */
static const double kU32 = 0x1p-24;           /* unit roundoff of float32 */

/* eta of an affine layer from the intervals of its predecessor (pl, pu); FE_UPWARD */
static void affine_inference_error(layer_t *l, const layer_t *p, const double *pl, const double *pu) {
    /* summands of one neuron; an average is the float32 sum of its kh*kw window values in any order followed by one
       rounded multiplication by a rounded 1/(kh*kw) or one rounded division: K + 1 roundings at most, like a sum of K
       products and a bias */
    const double K = (l->type == L_DENSE) ? (double)p->n : (l->type == L_POOL) ? (double)l->kh * l->kw : (double)l->kh * l->kw * p->C;
    const double ku = (K + 1.0) * kU32;
    const double gamma = ku / (-(ku - 1.0));                     /* k*u/(1-k*u): the denominator rounds down */
    const double floor_ = (K + 1.0) * 0x1p-149;
    if (l->type == L_DENSE) {
        for (int i = 0; i < l->n; ++i) {
            const double *w = l->wt + (size_t)i * p->n;
            double s = fabs(l->bias[i]);
            for (int j = 0; j < p->n; ++j) s = add_up(s, mul_up(fabs(w[j]), dmax(fabs(pl[j]), fabs(pu[j]))));
            l->eta[i] = add_up(mul_up(s, gamma), floor_);
        }
    } else if (l->type == L_POOL) {
        for (int d = 0; d < l->C; ++d)
            for (int y = 0; y < l->H; ++y)
                for (int x = 0; x < l->W; ++x) {
                    double s = 0.0;
                    for (int f = 0; f < l->kh; ++f) {
                        int iy = y * l->sh - l->ph + f;
                        if (iy < 0 || iy >= p->H) continue;
                        for (int g = 0; g < l->kw; ++g) {
                            int ix = x * l->sw - l->pw + g;
                            if (ix < 0 || ix >= p->W) continue;
                            int j = (d * p->H + iy) * p->W + ix;
                            s = add_up(s, dmax(fabs(pl[j]), fabs(pu[j])));
                        }
                    }
                    l->eta[(d * l->H + y) * l->W + x] = add_up(mul_up(mul_up(s, l->w_up), gamma), floor_);
                }
    } else {
        for (int d = 0; d < l->C; ++d)
            for (int y = 0; y < l->H; ++y)
                for (int x = 0; x < l->W; ++x) {
                    double s = fabs(l->bias[d]);
                    for (int ci = 0; ci < p->C; ++ci)
                        for (int f = 0; f < l->kh; ++f) {
                            int iy = y * l->sh - l->ph + f;
                            if (iy < 0 || iy >= p->H) continue;
                            for (int g = 0; g < l->kw; ++g) {
                                int ix = x * l->sw - l->pw + g;
                                if (ix < 0 || ix >= p->W) continue;
                                double w = l->wt[(((size_t)d * p->C + ci) * l->kh + f) * l->kw + g];
                                int j = (ci * p->H + iy) * p->W + ix;
                                s = add_up(s, mul_up(fabs(w), dmax(fabs(pl[j]), fabs(pu[j]))));
                            }
                        }
                    l->eta[(d * l->H + y) * l->W + x] = add_up(mul_up(s, gamma), floor_);
                }
    }
    l->has_eta = 1;
}

/* a rounded float32 addition is monotone: the interval of the exact sum moves outward by u*|end|; FE_UPWARD */
static inline void widen_rounded_sum(double *lo, double *hi) {
    *lo = add_dn(*lo, -mul_up(fabs(*lo), kU32));
    *hi = add_up(*hi, mul_up(fabs(*hi), kU32));
}

/* eta of a residual sum from its own (already widened) interval */
static void sum_inference_error(layer_t *l) {
    int old = fegetround();
    fesetround(FE_UPWARD);
    for (int i = 0; i < l->n; ++i) l->eta[i] = mul_up(dmax(fabs(l->lo[i]), fabs(l->hi[i])), kU32);
    fesetround(old);
    l->has_eta = 1;
}

/* before the rows of layer lid are bounded: the layer's own eta (affine) or none yet (sum) */
static int prepare_inference_error(dp_net *N, int lid, int early) {
    layer_t *l = &N->L[lid];
    l->has_eta = 0;
    if (!N->float_inference || (l->type != L_DENSE && l->type != L_CONV && l->type != L_POOL)) return DP_OK;
    const layer_t *p = &N->L[l->a];
    if (!p->has_bounds && !(early && p->has_ival)) return DP_ERR_STATE;
    int old = fegetround();
    fesetround(FE_UPWARD);
    affine_inference_error(l, p, p->has_bounds ? p->lo : p->ilo, p->has_bounds ? p->hi : p->ihi);
    fesetround(old);
    return DP_OK;
}

/* bounds of rows[0..n_rows) of layer lid, from the intervals already stored for earlier layers */
int dp_bound_rows(dp_net *N, int lid, const int *rows, int n_rows, double *out_lo, double *out_hi) {
    if (!N || lid <= 0 || lid >= N->n_layers || !rows || n_rows < 0) return DP_ERR_ARG;
    layer_t *l = &N->L[lid];
    if (l->type == L_RELU) return DP_ERR_ARG;
    for (int i = 0; i < n_rows; ++i) if (rows[i] < 0 || rows[i] >= l->n) return DP_ERR_ARG;
#pragma omp parallel
    {
        int old = fegetround();
        fesetround(FE_UPWARD);
        expr_t *e = expr_new(N);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_rows; ++r) {
            for (int sense = 1; sense >= -1; sense -= 2) {
                expr_clear(e, N);
                e->lo[lid][rows[r]] = 1.0; e->hi[lid][rows[r]] = 1.0;   /* x_i = 1 * x_i */
                e->active[lid] = 1;
                /* the neuron's own layer has no interval yet: the first candidate is taken after
                   the first substitution, i.e. over its predecessor(s) */
                int saved = l->has_bounds; (void)saved;
                double v;
                {
                    /* first step by hand so that a stale has_bounds flag of this layer is ignored */
                    switch (l->type) {
                        case L_DENSE: step_dense(N, e, lid); break;
                        case L_CONV:  step_conv(N, e, lid); break;
                        case L_POOL:  step_pool(N, e, lid); break;
                        case L_ADD:   step_add(N, e, lid); break;
                        default: break;
                    }
                    v = backsubstitute(N, e, sense);
                }
                if (sense > 0) out_hi[r] = v; else out_lo[r] = v;
            }
            if (N->float_inference && l->type == L_ADD) widen_rounded_sum(&out_lo[r], &out_hi[r]);
        }
        expr_free(e);
        fesetround(old);
    }
    return DP_OK;
}

/* ---- early termination (Sections 3.2 and 4.2) ------------------------------------------------------- */
/* intervals of layer q as known so far: back-substituted ones if the layer has them, else its interval image */
static const double *cur_lo(const layer_t *q) { return q->has_bounds ? q->lo : q->ilo; }
static const double *cur_hi(const layer_t *q) { return q->has_bounds ? q->hi : q->ihi; }

/* forward interval analysis of one layer (Section 4.2, the preliminary / updating step); FE_UPWARD */
static void interval_image(dp_net *N, int lid) {
    layer_t *l = &N->L[lid];
    const layer_t *p = &N->L[l->a];
    const double *pl = cur_lo(p), *pu = cur_hi(p);
    if (l->type == L_DENSE) {
        for (int i = 0; i < l->n; ++i) {
            const double *w = l->wt + (size_t)i * p->n;
            double lo = l->bias[i], hi = l->bias[i];
            for (int j = 0; j < p->n; ++j) {
                if (w[j] >= 0.0) { lo = add_dn(lo, mul_dn(w[j], pl[j])); hi = add_up(hi, mul_up(w[j], pu[j])); }
                else             { lo = add_dn(lo, mul_dn(w[j], pu[j])); hi = add_up(hi, mul_up(w[j], pl[j])); }
            }
            if (l->has_eta) { lo = add_dn(lo, -l->eta[i]); hi = add_up(hi, l->eta[i]); }
            l->ilo[i] = lo; l->ihi[i] = hi;
        }
    } else if (l->type == L_CONV) {
        for (int d = 0; d < l->C; ++d)
            for (int y = 0; y < l->H; ++y)
                for (int x = 0; x < l->W; ++x) {
                    double lo = l->bias[d], hi = l->bias[d];
                    for (int ci = 0; ci < p->C; ++ci)
                        for (int f = 0; f < l->kh; ++f) {
                            int iy = y * l->sh - l->ph + f;
                            if (iy < 0 || iy >= p->H) continue;
                            for (int g = 0; g < l->kw; ++g) {
                                int ix = x * l->sw - l->pw + g;
                                if (ix < 0 || ix >= p->W) continue;
                                double w = l->wt[(((size_t)d * p->C + ci) * l->kh + f) * l->kw + g];
                                int j = (ci * p->H + iy) * p->W + ix;
                                if (w >= 0.0) { lo = add_dn(lo, mul_dn(w, pl[j])); hi = add_up(hi, mul_up(w, pu[j])); }
                                else          { lo = add_dn(lo, mul_dn(w, pu[j])); hi = add_up(hi, mul_up(w, pl[j])); }
                            }
                        }
                    int i = (d * l->H + y) * l->W + x;
                    if (l->has_eta) { lo = add_dn(lo, -l->eta[i]); hi = add_up(hi, l->eta[i]); }
                    l->ilo[i] = lo; l->ihi[i] = hi;
                }
    } else if (l->type == L_POOL) {
        for (int d = 0; d < l->C; ++d)
            for (int y = 0; y < l->H; ++y)
                for (int x = 0; x < l->W; ++x) {
                    double lo = 0.0, hi = 0.0;
                    for (int f = 0; f < l->kh; ++f) {
                        int iy = y * l->sh - l->ph + f;
                        if (iy < 0 || iy >= p->H) continue;
                        for (int g = 0; g < l->kw; ++g) {
                            int ix = x * l->sw - l->pw + g;
                            if (ix < 0 || ix >= p->W) continue;
                            int j = (d * p->H + iy) * p->W + ix;
                            lo = add_dn(lo, pl[j]); hi = add_up(hi, pu[j]);
                        }
                    }
                    lo = lo >= 0.0 ? mul_dn(lo, l->w_dn) : mul_dn(lo, l->w_up);
                    hi = hi >= 0.0 ? mul_up(hi, l->w_up) : mul_up(hi, l->w_dn);
                    int i = (d * l->H + y) * l->W + x;
                    if (l->has_eta) { lo = add_dn(lo, -l->eta[i]); hi = add_up(hi, l->eta[i]); }
                    l->ilo[i] = lo; l->ihi[i] = hi;
                }
    } else if (l->type == L_ADD) {
        const layer_t *q = &N->L[l->b];
        const double *ql = cur_lo(q), *qu = cur_hi(q);
        for (int i = 0; i < l->n; ++i) {
            l->ilo[i] = add_dn(pl[i], ql[i]); l->ihi[i] = add_up(pu[i], qu[i]);
            if (N->float_inference) widen_rounded_sum(&l->ilo[i], &l->ihi[i]);
        }
    }
    l->has_ival = 1;
}

static void step_any(const dp_net *N, expr_t *e, int k, int sense) {
    switch (N->L[k].type) {
        case L_RELU:  step_relu(N, e, k, sense); break;
        case L_DENSE: step_dense(N, e, k); break;
        case L_CONV:  step_conv(N, e, k); break;
        case L_POOL:  step_pool(N, e, k); break;
        case L_ADD:   step_add(N, e, k); break;
        default: break;
    }
}

/* Upper and lower expression of one neuron substituted in lock step.  *lo,*hi hold the neuron's interval so
   far and are tightened by every candidate.  After a candidate over a layer k > 0 the termination criterion is
   checked (may_stop), or the given decision is followed (forced >= 0).  Returns the layer the pair stopped at. */
static int backsubstitute_pair(const dp_net *N, expr_t *eu, expr_t *el, double *lo, double *hi, int may_stop,
                               int forced) {
    for (;;) {
        int k = -1, count = 0;
        for (int i = N->n_layers - 1; i >= 0; --i)
            if (eu->active[i]) { if (k < 0) k = i; ++count; }
        if (k < 0) {
            *hi = dmin(*hi, eu->chi); *lo = dmax(*lo, el->clo);
            return 0;
        }
        if (N->collapse && N->L[k].has_bounds) { collapse_width(N, eu, k, +1); collapse_width(N, el, k, -1); }
        if (count == 1 && N->L[k].has_bounds && (k == 0 || N->candidates == 0)) {
            *hi = dmin(*hi, concretise(N, eu, k, +1));
            *lo = dmax(*lo, concretise(N, el, k, -1));
            if (k > 0) {
                int stop = (forced >= 0) ? (forced == k) : (may_stop && (*lo >= 0.0 || *hi <= 0.0));
                if (stop) return k;
            }
        }
        if (k == 0) return 0;
        step_any(N, eu, k, +1);
        step_any(N, el, k, -1);
    }
}

/* one layer in early-termination mode */
static int analyze_layer_early(dp_net *N, int lid) {
    layer_t *l = &N->L[lid];
    {
        int rc = prepare_inference_error(N, lid, 1);
        if (rc != DP_OK) return rc;
        int old = fegetround();
        fesetround(FE_UPWARD);
        interval_image(N, lid);
        fesetround(old);
    }
    const int wants = l->need_bounds || lid == N->n_layers - 1;
    if (!wants) return DP_OK;
    /* the criterion speaks about inputs of ReLU layers; rows asked for otherwise are always substituted fully */
    const int may_stop = l->feeds_relu && !l->requested && lid != N->n_layers - 1;
    l->has_bounds = 0;
#pragma omp parallel
    {
        int old = fegetround();
        fesetround(FE_UPWARD);
        expr_t *eu = expr_new(N), *el = expr_new(N);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < l->n; ++r) {
            double lo = l->ilo[r], hi = l->ihi[r];
            const int forced = l->term_force ? l->term_force[r] : -1;
            int skip = (forced >= 0) ? (forced == lid) : (may_stop && !(lo < 0.0 && hi > 0.0));
            if (skip) { l->lo[r] = lo; l->hi[r] = hi; l->term[r] = lid; continue; }
            expr_clear(eu, N); expr_clear(el, N);
            eu->lo[lid][r] = eu->hi[lid][r] = 1.0; eu->active[lid] = 1;
            el->lo[lid][r] = el->hi[lid][r] = 1.0; el->active[lid] = 1;
            step_any(N, eu, lid, +1);
            step_any(N, el, lid, -1);
            l->term[r] = backsubstitute_pair(N, eu, el, &lo, &hi, may_stop, forced);
            if (N->float_inference && l->type == L_ADD) {
                /* candidates bound the exact sum, the interval image already the rounded one */
                widen_rounded_sum(&lo, &hi);
                lo = dmax(lo, l->ilo[r]); hi = dmin(hi, l->ihi[r]);
            }
            l->lo[r] = lo; l->hi[r] = hi;
        }
        expr_free(eu); expr_free(el);
        fesetround(old);
    }
    l->has_bounds = 1;
    if (N->float_inference && l->type == L_ADD) sum_inference_error(l);
    return DP_OK;
}

int dp_analyze_layer(dp_net *N, int lid) {
    if (!N || lid <= 0 || lid >= N->n_layers) return DP_ERR_ARG;
    layer_t *l = &N->L[lid];
    if (l->type == L_RELU) {
        if (!N->L[l->a].has_bounds) return DP_ERR_STATE;
        int old = fegetround();
        fesetround(FE_UPWARD);
        relu_layer(N, lid);
        fesetround(old);
        return DP_OK;
    }
    if (N->early_term) return analyze_layer_early(N, lid);
    int rc = prepare_inference_error(N, lid, 0);
    if (rc != DP_OK) return rc;
    int *rows = (int *)malloc(sizeof(int) * l->n);
    for (int i = 0; i < l->n; ++i) rows[i] = i;
    l->has_bounds = 0;
    rc = dp_bound_rows(N, lid, rows, l->n, l->lo, l->hi);
    free(rows);
    if (rc == DP_OK) {
        l->has_bounds = 1;
        if (N->float_inference && l->type == L_ADD) sum_inference_error(l);
    }
    return rc;
}

int dp_analyze(dp_net *N) {
    if (!N || !N->L[0].has_bounds) return DP_ERR_STATE;
    for (int i = 1; i < N->n_layers; ++i) {
        layer_t *l = &N->L[i];
        /* in float32-inference mode a residual sum needs its own interval (its rounding error is relative to it) */
        if (l->type == L_RELU || l->need_bounds || i == N->n_layers - 1 || N->early_term ||
            (N->float_inference && l->type == L_ADD)) {
            int rc = dp_analyze_layer(N, i);
            if (rc != DP_OK) return rc;
        } else {
            int rc = prepare_inference_error(N, i, 0);      /* crossed by later expressions all the same */
            if (rc != DP_OK) return rc;
        }
    }
    N->analyzed = 1;
    return DP_OK;
}

/* lower bounds of y_label - y_j over the last layer, j != label, in increasing j */
int dp_certify(dp_net *N, int label, int *verified, double *margins) {
    if (!N) return DP_ERR_STATE;
    int lid = N->n_layers - 1;
    layer_t *l = &N->L[lid];
    if (!l->has_bounds) return DP_ERR_STATE;   /* the analysis (whole or layer by layer) must have reached the end */
    if (label < 0 || label >= l->n || l->type == L_RELU) return DP_ERR_ARG;
    int ok = 1;
#pragma omp parallel
    {
        int old = fegetround();
        fesetround(FE_UPWARD);
        expr_t *e = expr_new(N);
#pragma omp for schedule(dynamic, 1)
        for (int j = 0; j < l->n; ++j) {
            if (j == label) continue;
            expr_clear(e, N);
            e->lo[lid][label] = e->hi[lid][label] = 1.0;
            e->lo[lid][j] = e->hi[lid][j] = -1.0;
            e->active[lid] = 1;
            switch (l->type) {
                case L_DENSE: step_dense(N, e, lid); break;
                case L_CONV:  step_conv(N, e, lid); break;
                case L_POOL:  step_pool(N, e, lid); break;
                case L_ADD:   step_add(N, e, lid); break;
                default: break;
            }
            double v = backsubstitute(N, e, -1);
            margins[j - (j > label)] = v;
        }
        expr_free(e);
        fesetround(old);
    }
    for (int j = 0; j < l->n - 1; ++j) if (!(margins[j] > 0.0)) ok = 0;
    if (verified) *verified = ok;
    return DP_OK;
}

/* Lower bounds of arbitrary linear forms of the last layer, sum_j coef[r][j]*y_j + offset[r] (the certification
   rows y_label - y_j are the special case dp_certify computes): other output specifications than robustness. */
int dp_bound_forms(dp_net *N, int n_forms, const double *coef, const double *offset, double *lower) {
    if (!N || n_forms < 0 || !coef || !lower) return DP_ERR_ARG;
    int lid = N->n_layers - 1;
    layer_t *l = &N->L[lid];
    if (!l->has_bounds) return DP_ERR_STATE;
    if (l->type == L_RELU) return DP_ERR_ARG;
#pragma omp parallel
    {
        int old = fegetround();
        fesetround(FE_UPWARD);
        expr_t *e = expr_new(N);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_forms; ++r) {
            expr_clear(e, N);
            for (int j = 0; j < l->n; ++j) e->lo[lid][j] = e->hi[lid][j] = coef[(size_t)r * l->n + j];
            e->active[lid] = 1;
            e->clo = e->chi = offset ? offset[r] : 0.0;
            switch (l->type) {
                case L_DENSE: step_dense(N, e, lid); break;
                case L_CONV:  step_conv(N, e, lid); break;
                case L_POOL:  step_pool(N, e, lid); break;
                case L_ADD:   step_add(N, e, lid); break;
                default: break;
            }
            lower[r] = backsubstitute(N, e, -1);
        }
        expr_free(e);
        fesetround(old);
    }
    return DP_OK;
}

/* Self-check that the compiler kept the directed-rounding idioms intact (returns 0 when fine).
   The inputs come from the caller so that nothing can be folded at compile time. */
int dp_selftest_rounding(double one, double tiny, double third) {
    int old = fegetround(), bad = 0;
    fesetround(FE_UPWARD);
    if (!(add_up(one, tiny) > one)) bad |= 1;
    if (!(add_dn(one, tiny) == one)) bad |= 2;
    if (!(add_dn(one, -tiny) < one)) bad |= 4;
    if (!(add_up(one, -tiny) == one)) bad |= 8;
    if (!(mul_dn(third, third) < mul_up(third, third))) bad |= 16;
    if (!(mul_dn(-third, third) < mul_up(-third, third))) bad |= 32;
    double lo = 0.0, hi = 0.0;
    acc_scaled(&lo, &hi, third, third, third);
    if (!(lo < hi)) bad |= 64;
    lo = hi = 0.0;
    acc_scaled(&lo, &hi, third, third, -third);
    if (!(lo < hi)) bad |= 128;
    if (!(sub_up(one, mul_dn(third, third)) >= sub_up(one, mul_up(third, third)))) bad |= 256;
    fesetround(old);
    return bad;
}

int dp_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

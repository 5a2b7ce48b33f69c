/*
 * gpupoly — DeepPoly back-substitution on one AMD MI355X (gfx950).  C ABI.
 *
 * The library bounds every neuron of a ReLU network over an L-infinity box by the DeepPoly
 * relaxation with back-substitution (paper Section 2, "DeepPoly analysis" and "Bottleneck
 * Backsubstitution"), using dependence windows for convolutional and residual layers
 * (Sections 3.1, 4.3, Algorithm 1) and floating-point-sound arithmetic (Section 4.1).
 *
 * Conventions
 *   - All pointers are HOST pointers unless the name ends in _dev (then: device memory on the
 *     current HIP device).  Host arrays are read or written during the call and never retained.
 *   - Layer id 0 is the input; every gp_add_* call creates the next id and returns it.
 *     A layer may only reference earlier ids, so ids are a topological order of the network DAG
 *     (Section 3.1 "Network DAG").
 *   - Neurons of a layer are numbered C,H,W-flattened (channel outermost) at this boundary.
 *   - Every call returns a gp_status; nothing throws or aborts across the boundary; a failed call
 *     leaves the net usable.  gp_last_error() gives a message for the last failure on that net.
 *   - Bounds are reported for: the input, every layer that feeds a ReLU, every ReLU layer, every layer
 *     that an affine layer reads directly, the last layer, and layers marked with gp_request_bounds()
 *     (with gp_set_float_inference also every residual sum layer).  Other layers: GP_ERR_STATE.
 *   - Soundness: reported bounds contain the exact real-arithmetic output range of the network
 *     with the given float32 weights over the box (rounding of the analysis itself is accounted
 *     for); with gp_set_float_inference they also contain what a float32 evaluation of the network
 *     computes, in any summation order.
 *   - Calls on one net must not overlap in time.  Different nets may be used from different threads.
 */
#ifndef GPUPOLY_H
#define GPUPOLY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gp_net gp_net; /* opaque; owns device copies of weights and of all bounds */

typedef enum {
    GP_OK = 0,
    GP_ERR_ARG = 1,         /* null pointer, id out of range, negative size or eps             */
    GP_ERR_SHAPE = 2,       /* shapes of layers do not fit                                      */
    GP_ERR_STATE = 3,       /* call order: no analysis yet, layer has no bounds, ...            */
    GP_ERR_NOMEM = 4,       /* host or device allocation failed                                 */
    GP_ERR_DEVICE = 5,      /* no usable GPU, or a HIP call failed                              */
    GP_ERR_NONFINITE = 6,   /* NaN/Inf in weights, inputs or computed bounds                    */
    GP_ERR_WORKSPACE = 7,   /* workspace too small even for one row                             */
    GP_ERR_UNSUPPORTED = 8  /* topology the back-substitution engine cannot handle              */
} gp_status;

/* Input layer of shape (c,h,w); a flat input of n values is (n,1,1).  Paper Section 2. */
gp_status gp_net_create(int32_t c, int32_t h, int32_t w, gp_net** out);
void gp_net_destroy(gp_net* net);

/* Affine layers (paper Section 2 "Classification network": x' = A x + b).
 * W: [out_dim][n_in] row-major, n_in = C*H*W of in_layer, flattened C,H,W.  b: [out_dim] or NULL. */
gp_status gp_add_dense(gp_net* net, int32_t in_layer, int32_t out_dim, const float* W, const float* b,
                       int32_t* layer_id);
/* W: [c_out][c_in][kh][kw]; b: [c_out] or NULL; zero padding; output (y,x), tap (f,g) reads input
 * (y*stride_h - pad_h + f, x*stride_w - pad_w + g)  (index map of Algorithm 1). */
gp_status gp_add_conv2d(gp_net* net, int32_t in_layer, int32_t c_out, int32_t kh, int32_t kw,
                        int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                        const float* W, const float* b, int32_t* layer_id);
/* Average pooling, every channel on its own: output (c,y,x) = (1/(kh*kw)) * sum over the window taps (f,g) of input
 * (c, y*stride_h - pad_h + f, x*stride_w - pad_w + g); taps in the zero padding add nothing and the divisor stays kh*kw.
 * An affine layer (Section 2, affine transformer; Section 3.1: its dependence sets are those of a convolution with the
 * same window) without a stored filter: crossing it costs window-size operations per coefficient instead of a
 * contraction over channels.  pad < window in both dimensions. */
gp_status gp_add_avgpool2d(gp_net* net, int32_t in_layer, int32_t kh, int32_t kw, int32_t stride_h, int32_t stride_w,
                           int32_t pad_h, int32_t pad_w, int32_t* layer_id);
/* Element-wise max(x,0) of in_layer. */
gp_status gp_add_relu(gp_net* net, int32_t in_layer, int32_t* layer_id);
/* Element-wise sum of two layers of equal shape: the exit of a residual block (Section 3.1,
 * "Dependence set and residual networks"). */
gp_status gp_add_residual(gp_net* net, int32_t layer_a, int32_t layer_b, int32_t* layer_id);
/* Also compute bounds for this (affine or sum) layer although no ReLU reads it. */
gp_status gp_request_bounds(gp_net* net, int32_t layer_id);

/* Early termination (paper Section 3.2 "Early termination", Section 4.2 "Implementing early termination"); off by
 * default.  When on, every layer first gets its interval image from its predecessors' intervals (forward interval
 * analysis); of a layer that feeds a ReLU only the neurons whose interval strictly contains 0 are back-substituted,
 * and a neuron stops as soon as a candidate shows lower >= 0 or upper <= 0 (checked after every candidate over a
 * hidden layer); it keeps the bounds it has then.  Rows of stopped neurons are removed from the coefficient blocks.
 * Reported bounds are the intersection of the interval image and the candidates.  The last layer, layers marked with
 * gp_request_bounds and certification rows are always substituted down to the input.  Takes effect at the next
 * analysis; bounds of stopped neurons are sound but in general looser than without early termination. */
gp_status gp_set_early_termination(gp_net* net, int32_t on);
/* Plumbing; off by default.  When on, gp_analyze, gp_analyze_batch and gp_analyze_batch_dev capture their kernel launches
 * into a HIP graph the first time and replay it afterwards: one pass over a small batch is a chain of some 150 dependent
 * launches of a few microseconds each, and the replay removes their per-launch dispatch cost.  The graph is rebuilt
 * whenever batch, centres pointer (the library's own staging buffer for host centres), eps, clip range, workspace or
 * stream differ from the captured ones or the network or a mode changes; with early termination (the host reads
 * counts between steps) and while profiling the calls run as usual.  Results are bit-identical either way.  The
 * capture itself runs with the stream idle (the call synchronises it first). */
gp_status gp_set_graph_replay(gp_net* net, int32_t on);
/* Rounding of the inference itself (paper Section 4.1, last paragraph: the analysis should also cover the error a
 * floating-point evaluation of the network makes, whatever the order of its sums); off by default.  When on, every
 * bound holds for the real-valued network AND for every float32 evaluation of it in which an affine neuron is a sum
 * of float32 products and its bias taken in any order, with or without fused multiply-add, an average is the float32
 * sum of its window in any order followed by one rounded division or one multiplication by the rounded reciprocal
 * (the affine formula below with K = window size, |w_j| = 1/K, b = 0), a residual sum is one rounded addition and
 * ReLU is exact (round to nearest, gradual underflow, no overflow).  Mechanism: an affine neuron
 * of K inputs is its exact expression plus an error of at most gamma(K+1)*(sum|w_j||x_j| + |b|) + (K+1)*2^-149,
 * gamma(k) = k*2^-24/(1 - k*2^-24), evaluated with the predecessors' bounds; that constant is added, times the
 * magnitude of the coefficient, whenever an expression is substituted through the neuron.  A residual sum layer's
 * interval is moved outward by 2^-24*|end| (so sum layers always get bounds in this mode).  Takes effect at the
 * next analysis.  The bounds of gp_certify and gp_bound_outputs then speak about the float32 outputs. */
gp_status gp_set_float_inference(gp_net* net, int32_t on);
/* The paper's literal floating-point scheme (Section 4.1), for tightness studies on small networks; off by default.
 * When on, every coefficient of an expression is an interval of two float64 values, every operation rounds lower ends
 * towards -inf and upper ends towards +inf (the vector unit's rounding mode; the matrix instructions have none, so
 * this mode runs on plain vector arithmetic, one thread per new coefficient), weights stay scalars, and the intervals
 * are kept to the end of the back-substitution.  Same plans, dependence windows and residual joins as the default
 * mode; no rounding-slack terms (the intervals carry the rounding).  16 bytes per coefficient; on deep networks the
 * widths grow with depth and the bounds become looser than the default mode's.  Cannot be combined with early
 * termination or float32-inference mode (GP_ERR_UNSUPPORTED at the next analysis); float64 storage and chain fusion
 * are ignored while it is on.  Takes effect at the next analysis. */
gp_status gp_set_interval_coefficients(gp_net* net, int32_t on);
/* Plumbing; on by default.  The rows of a dense layer of at most 256 neurons whose back-substitution runs through dense
 * layers only, all of at most 256 neurons (the last block, usually over the input, at most 1024), are carried through ALL their steps by one
 * kernel launch per start layer, with the coefficient block in LDS (Section 2, "Bottleneck Backsubstitution": the rows
 * are independent, so a work-group can follow its rows to the input on its own).  Whether a layer takes this path
 * depends on the network alone, not on the batch.  The arithmetic per step is that of the general kernels (float32
 * coefficients, float64 accumulation, the same slack terms), but sums are formed in another order, so bounds differ
 * from the general path in the last bits; both are sound.  Off: every layer takes the general kernels.  Not used with
 * early termination, float32-inference mode or float64 storage.  The fused path serves latency (a few boxes per call);
 * with more than about 6000 rows per start layer (2 * neurons * boxes) the general kernels are faster, and a caller
 * that passes hundreds of boxes per call should switch it off. */
gp_status gp_set_chain_fusion(gp_net* net, int32_t on);
/* Precision of the stored coefficients (the paper evaluates a single and a double precision build, Section 5); 32
 * (default) or 64.  With 32 every new coefficient of a row's block is rounded once to float32 and the rounding is
 * paid into the row's slack; with 64 the blocks hold float64 values: twice the memory and traffic, only the general
 * crossing kernel, and bounds whose distance to exact arithmetic is of the order 1e-12 relative instead of 1e-6 (the
 * weights stay the float32 values handed over; the relaxation slopes stay float32 values, any slope is sound).
 * Takes effect at the next analysis. */
gp_status gp_set_coefficient_storage(gp_net* net, int32_t bits);
/* After an analysis with early termination: for each neuron of a layer that has bounds, the id of the layer its
 * expression ranged over when it stopped; layer_id itself = never back-substituted, 0 = substituted down to the
 * input.  term: [n_layer]. */
gp_status gp_get_term_layer(const gp_net* net, int32_t layer_id, int32_t batch_index, int32_t* term);
/* Work of the affine crossings in the last analysis with early termination: floating-point operations carried out,
 * and what the same analysis costs when no row is ever removed. */
gp_status gp_get_early_termination_stats(const gp_net* net, double* flop_done, double* flop_full);

/* HIP stream (hipStream_t) all work of this net is enqueued on; NULL = the default stream. */
gp_status gp_set_stream(gp_net* net, void* hip_stream);
/* Scratch memory for the coefficient blocks of the rows in flight (Section 4.2 "Memory
 * management": rows are processed in chunks that fit).  min_bytes: smallest workable size for this
 * net and batch; full_bytes: size at which no layer needs chunking. */
gp_status gp_workspace_size(const gp_net* net, int32_t batch, int64_t* min_bytes, int64_t* full_bytes);
/* Device memory owned by the caller (e.g. a torch tensor), 256-byte aligned, kept alive until
 * replaced or the net is destroyed.  Without it the library allocates its own on first use. */
gp_status gp_set_workspace(gp_net* net, void* ptr_dev, int64_t bytes);

/* Analyse the box  [max(center-eps, clip_lo), min(center+eps, clip_hi)]  (Section 2, L-infinity
 * robustness).  center: [n_in].  Blocks until the bounds are on the device. */
gp_status gp_analyze(gp_net* net, const float* center, float eps, float clip_lo, float clip_hi);
/* Analyse an explicit box lo <= x <= hi, both [n_in]. */
gp_status gp_analyze_box(gp_net* net, const float* lo, const float* hi);
/* `batch` independent boxes at once; rows of all boxes share the kernel launches.
 * centers: [batch][n_in]. */
gp_status gp_analyze_batch(gp_net* net, int32_t batch, const float* centers, float eps, float clip_lo,
                           float clip_hi);
/* Same with the centres already in device memory ([batch][n_in] float). */
gp_status gp_analyze_batch_dev(gp_net* net, int32_t batch, const float* centers_dev, float eps,
                               float clip_lo, float clip_hi);

/* For callers that cannot allocate device memory at the time of the call: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same analysis as gp_analyze_batch_dev, with the coefficient blocks of the
 * rows in flight kept in a static device array of the library (32 MiB per GPU, held from the moment the library is
 * loaded until the process ends) instead of a workspace, and with the bounds of the last layer also written to arrays
 * of the caller: lower_dev, upper_dev, device memory, [batch][n_out] float64, outputs numbered C,H,W.  The call makes no
 * device or pinned-memory allocation and frees none (no hipMalloc, hipFree, event or stream creation); rows are
 * processed in chunks that fit the array (Section 4.2 "Memory management"), which changes no bit of the result.
 * Preconditions, reported and never worked around by allocating:
 *   - an analysis of at least `batch` boxes has completed on this net since its topology or modes last changed (that
 *     call sized the per-layer arrays, which this one reuses): otherwise GP_ERR_STATE;
 *   - one row (both signs) of every layer's plan fits the static array: otherwise GP_ERR_WORKSPACE, the message gives
 *     the bytes needed and the size of the array;
 *   - per-kernel profiling is off (it creates events): otherwise GP_ERR_STATE.
 * A workspace set with gp_set_workspace and graph replay are ignored by this call.  All calls on one GPU share that
 * GPU's array (whatever the net): calls that overlap in time on one GPU race on it.  The array keeps the previous
 * call's contents; nothing in it is expected to be zero.  gp_get_bounds* and gp_certify* work afterwards as after any
 * analysis. */
gp_status gp_analyze_batch_dev_static(gp_net* net, int32_t batch, const float* centers_dev, float eps, float clip_lo,
                                      float clip_hi, double* lower_dev, double* upper_dev);

/* Bounds of one layer for box `batch_index` of the last analysis: lower/upper [n_layer] float32,
 * rounded outward from the internal float64 values. */
gp_status gp_get_bounds(const gp_net* net, int32_t layer_id, float* lower, float* upper);
gp_status gp_get_bounds_batch(const gp_net* net, int32_t layer_id, int32_t batch_index, float* lower,
                              float* upper);
/* The same as float64 (the values the analysis itself uses for later layers). */
gp_status gp_get_bounds_f64(const gp_net* net, int32_t layer_id, int32_t batch_index, double* lower,
                            double* upper);
/* Lower relaxation slope (0 or 1) chosen for each neuron of a ReLU layer; [n_layer] bytes. */
gp_status gp_get_relu_lambda(const gp_net* net, int32_t relu_layer_id, int32_t batch_index, int8_t* lam);
/* Slope of the upper relaxation line used for each neuron of a ReLU layer (1 for stably active, 0 for
 * stably inactive neurons; any slope in [0,1] is sound with the matching intercept); [n_layer] floats. */
gp_status gp_get_relu_slopes(const gp_net* net, int32_t relu_layer_id, int32_t batch_index, float* slope);

/* Robustness of `label` over the analysed box: margins[r] = sound lower bound of
 * y_label - y_j over the last layer for the r-th j != label (increasing j), obtained by
 * back-substituting the difference; verified = all margins > 0.  margins: [n_out-1]. */
gp_status gp_certify(gp_net* net, int32_t label, int32_t* verified, float* margins);
/* labels: [batch]; verified: [batch]; margins: [batch][n_out-1]. */
gp_status gp_certify_batch(gp_net* net, const int32_t* labels, int32_t* verified, float* margins);

/* Sound lower bounds of arbitrary linear forms of the last layer over the analysed box(es):
 *   lower[b][r] <= sum_j coef[r][j] * y_j + offset[r]   for every input of box b
 * by back-substituting the form (the certification rows y_label - y_j of gp_certify are the special case; the paper's
 * introduction names properties other than robustness that reduce to such forms).  coef: [n_forms][n_out] with the
 * outputs numbered C,H,W; offset: [n_forms] or NULL; lower: [batch][n_forms], rounded down to float32. */
gp_status gp_bound_outputs(gp_net* net, int32_t n_forms, const float* coef, const float* offset, float* lower);

/* Introspection (host only, no GPU needed): the sequence of back-substitution steps planned for
 * the rows of `layer_id`.  Each step is 8 int32: {kind, layer, window_h, window_w, channels,
 * acc_stride_h, acc_pad_h, merged}; kind 0 = initial block, 1 = affine crossing, 2 = ReLU,
 * 3 = residual fork.  Window sizes are those of eqs. (4),(5) of Section 4.3 clipped to the layer.
 * Returns the number of steps in *n_steps (at most max_steps are written). */
gp_status gp_debug_plan(const gp_net* net, int32_t layer_id, int32_t* steps, int32_t max_steps,
                        int32_t* n_steps);

/* Per-kernel timing with HIP events on the net's stream.  While enabled, every launch of the two
 * back-substitution kernels is bracketed by events: index 0 = affine crossing (the product
 * M^{k-1} = M^k F^k of Section 2 / Algorithm 1), index 1 = per-row scan (candidate bound,
 * relaxation constants).  gp_profile_read synchronises, returns for each of the two kernels the
 * number of launches, their summed duration in ms, and the algorithmic flops and bytes of the
 * steps they carried out, then resets the counters.  All four arrays have 2 entries. */
gp_status gp_profile_enable(gp_net* net, int32_t on);
gp_status gp_profile_read(gp_net* net, int64_t* launches, double* total_ms, double* alg_flop, double* alg_bytes);
/* One CSV line per launch recorded since gp_profile_enable (kernel, start layer, layer, rows, block sizes, N, K,
 * algorithmic flop, duration in us), written to `path`; call it before gp_profile_read. */
gp_status gp_profile_dump(gp_net* net, const char* path);

/* Study hook: the unit roundoff at which the accumulation-error term of a crossing is priced.  A crossing adds
 * (K+8) * unit * (largest absolute row sum of the layer's matrix) * max|x| * sum|m| to a row's slack for the sum of K
 * products it forms per new coefficient; the default 2^-50 covers the float64 matrix instruction.  A larger value
 * makes the analysis report the bounds it would report if the products were accumulated in a narrower format with that
 * unit roundoff and the same a-priori error term (2^-24: float32; Section 4.1 discusses the cost of sound floating
 * point) - the arithmetic itself stays float64, so the bounds stay sound - which is how the slack of such a kernel is
 * measured against the oracle before anyone builds it.  unit in [2^-50, 2^-8]. */
gp_status gp_debug_set_accumulation_roundoff(gp_net* net, double unit);

/* Self-check of the matrix instruction the crossing kernel relies on: D[16][16] = A[16][K] * B[K][16]
 * in float64 MFMA (K a multiple of 4; A, B, D row-major in device memory), enqueued on hip_stream.
 * The rounding slack of a crossing assumes |D - exact| <= (K+8) * 2^-50 * sum|terms|; tests check it. */
gp_status gp_debug_mfma_f64(const double* A_dev, const double* B_dev, double* D_dev, int32_t K, void* hip_stream);
/* The same check for the 4-column instruction that crosses layers with at most 4 input channels (the image):
 * D[16][4] = A[16][K] * B[K][4]. */
gp_status gp_debug_mfma_f64_4col(const double* A_dev, const double* B_dev, double* D_dev, int32_t K, void* hip_stream);

int32_t gp_num_layers(const gp_net* net);
int32_t gp_layer_size(const gp_net* net, int32_t layer_id);
const char* gp_last_error(const gp_net* net);
const char* gp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GPUPOLY_H */

// Plain-data kernel parameter blocks and launchers of the back-substitution kernels (gfx950).
//
// Vocabulary (paper Sections 2, 3.1, 4.3):
//   row     one back-substitution task: the upper-bound expression of +x_i or of -x_i for a neuron
//           x_i of the start layer (a lower bound of x_i is minus an upper bound of -x_i, so every
//           row is an upper-bound expression and all kernels have a single sign convention);
//   block   a row's dense coefficient cuboid M^k(x_i) over its dependence window in layer k,
//           stored [window_y][window_x][channel] in float32, channel innermost;
//   window  the dependence set D^{l-k}(x_i) of Section 4.3, clipped to the layer: every row of a
//           step has the same window size, and an origin that depends on the row's position.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gp {

// Unsigned division by a run-time constant without a divide instruction: q = (mulhi(m, x) + x) >> s.
// Exact for 1 <= d < 2^31 and x < 2^31 (the round-up method with a 33-bit multiplier whose top bit is the "+ x").
struct FastDiv {
    uint32_t d, m, s;
};
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    f.s = s;
    f.m = (uint32_t)((((1ull << 32) * ((1ull << s) - d)) / d) + 1);
    return f;
}
__host__ __device__ inline uint32_t fast_div(uint32_t x, const FastDiv& f) {
#if defined(__HIP_DEVICE_COMPILE__)
    return (__umulhi(f.m, x) + x) >> f.s;
#else
    return (uint32_t)(((((uint64_t)f.m * x) >> 32) + x) >> f.s);
#endif
}

// which neurons the rows of a launch stand for
struct RowMap {
    int row0;        // first task of this chunk, counted over batch * n_start (< 2^31)
    int Rc;          // tasks in the chunk
    int nsign;       // 2: rows [0,Rc) are +x, rows [Rc,2Rc) are -x;  1: one row per task
    int n_start;     // tasks per box of the batch
    int Hs, Ws, Cs;  // start layer dims; task i sits at position ((i/Cs)/Ws, (i/Cs)%Ws), channel i%Cs
    FastDiv div_n, div_c, div_w;   // n_start, Cs, Ws
    // early termination (Section 4.2): after rows have been removed, row rr of a half stands for task
    // row0 + rowid[rr] (null: rr itself); Rc0 = tasks of the chunk before any removal (`best` keeps that layout)
    const int* rowid;
    int Rc0;
};

struct BlockDesc {
    const float* data;   // [nrows][wy][wx][C]; float64 values instead when the parameter block's coef64 is set
    int H, W, C;         // dims of the layer the block ranges over
    int wy, wx;          // window size (already clipped to the layer)
    int Sy, Sx, Py, Px;  // window origin of a row at (ys,xs): clamp(S*ys - P, 0, H - wy)  (eqs. 6-9 with padding)
    // the row's exact dependence window: origin tS*pos - tP (may be negative), size tW (may exceed the layer); the
    // stored window contains its part inside the layer, and every stored entry outside it is a structural zero
    // (read by the crossing kernel only; H, W < 32768 there)
    int tSy, tSx, tPy, tPx, tWy, tWx;
};

struct CrossParams {       // one back-substitution step through an affine layer (Algorithm 1 per row)
    BlockDesc in;          // block over the layer's OUTPUT neurons
    const float* wt;       // [kh*kw][Co][in.C]  (the layer's own output channels innermost)
    const double* wt64;    // the same values in float64 (every layer with weights has the copy)
    double pool_scale;     // 0: a layer with a filter; else the layer is average pooling (channels pass through,
                           //   Co == in.C, wt unused) and this is 1/(kh*kw)
    int kh, kw, sh, sw, ph, pw;
    float* out;            // new block over the layer's INPUT neurons
    const float* out_grl;  // when the input layer is a ReLU layer and the block is complete: its packed relaxation
                           //   [batch][Ho*Wo*Co] (|g| = upper slope; sign bit set = lower slope 0, clear = 1), applied to
                           //   the new coefficients before they are rounded and stored; null: store as is
    int Ho, Wo, Co;        // dims of the input layer
    int owy, owx, oSy, oSx, oPy, oPx;
    FastDiv div_owx, div_sh, div_sw, div_kw;     // owx, sh, sw, kw
    int ntiles_m, ntiles_n;                      // filled by the launcher: tiles of rows / of input channels
    FastDiv div_ntiles_n, div_opix;
    int lds_wt;                                  // filled by the launcher (cross_direct_kernel, image layers): filter staged in LDS
    int cls_ny, cls_nx;                          // filled by the launcher (cross_image_kernel): pixels per parity class (it also sets div_ntiles_n to a divider by in.C)
    FastDiv div_cls, div_cls_nx;
    BlockDesc add;         // optional block over the same input layer to be summed in (residual join)
    RowMap rm;
    int nrows;
    int coef64;            // coefficient blocks (in, out, add) hold float64 instead of float32 values
};

struct GenParams {         // a start layer's own matrix rows (InitParams mode 2), for the scan that makes them itself
    const float* wt;       // [tap][Cs][C] (predecessor channels innermost); dense: [Cs][nelem]
    const float* bias;     // [Cs]
    const float* out_grl;  // packed relaxation of the predecessor when it is a ReLU layer (applied), else null
    int H, W, C;           // dims of the predecessor
    int wy, wx, Sy, Sx, Py, Px;
    int kh, kw, sh, sw, ph, pw, dense;
    int Cs;                // channels of the start layer
};

struct ScanParams {        // per-row reductions over a block
    BlockDesc blk;
    RowMap rm;
    int nrows;
    int batch_stride;      // H*W*C
    const double* cpos;    // candidate multiplier of a positive / negative coefficient, [batch][n]; null: no candidate
    const double* cneg;    //   (a layer's own upper / lower interval ends, or rho / lower end after a ReLU substitution)
    const double* xlo;     // intervals of the neurons the STORED coefficients multiply (rounding slack); null with cpos
    const double* xhi;
    const double* kap;     // constant per unit of positive coefficient (ReLU upper intercept / slope); null if none
    const double* beff;    // [C] bias of the affine layer(s) crossed next; null if none
    const double* eta;     // [batch][n] constant per unit of |coefficient|: how far a float32 evaluation of the neuron
                           //   can be from its exact affine expression (Section 4.1, inference rounding); null: none
    double e1_a, e1_b;     // accumulation-error constants of the next crossing(s), times xmax_a[box] / xmax_b[box]
    const double* xmax_a;
    const double* xmax_b;
    const double* xmax_self; // [batch] largest |bound| of the block's own layer (subnormal floor of the rounding slack)
    double round_coef;     // relative rounding error of the stored coefficients (0 for exact blocks)
    int do_consts;         // add the constants of the next step (relaxation intercepts, bias) to c
    int update_best;       // the expression ranges over this layer only: fold the candidate into best
    double* c;             // per-row constant
    double* err;           // per-row accumulated slack (>= 0)
    double* best;          // per-row best candidate so far (indexed by the row's place before any removal)
    const unsigned char* done;   // per task of the chunk (compact): 1 = termination criterion met, best is final; null: none
    double* partial;       // scratch for rows longer than 1024 coefficients: [nrows][ceil(nelem/512)][5]; null: not available
    int coef64;            // the block holds float64 values
    FastDiv div_C, div_wx; // filled by the launcher: blk.C, blk.wx
    double coef_floor;     // smallest magnitude a stored coefficient resolves, times 2^20 (see scan_finish)
    // gen: the block does not exist yet.  It holds the rows that init_kernel would write in mode 2 (float32 storage, no
    // seeded bounds, no inference-rounding term): the scan computes a row's coefficients where it would have loaded
    // them, takes the row's constant from the bias (err = 0, best = +inf), and writes the coefficients to blk.data only
    // if gen_write is set (a block that no later step reads is never stored).
    int gen = 0, gen_write = 0;
    GenParams g = {};
};

struct InitParams {
    float* out;            // [nrows][nelem]
    RowMap rm;
    int nrows;
    int nelem;             // elements per row
    int mode;              // 0: one-hot over the start layer; 1: certification rows; 2: the start layer's own matrix row;
                           // 3: minus a caller-given linear form of the last layer (rows of `forms`, C,H,W order)
    const float* out_grl;  // mode 2: packed relaxation of the predecessor when it is a ReLU layer (applied), else null
    const int* labels;     // mode 1: [batch]
    const float* forms;    // mode 3: [n_forms][nelem]
    const float* offsets;  // mode 3: [n_forms] or null
    int H, W, C;           // dims of the layer the block ranges over (mode 1: last layer; mode 2: predecessor)
    // mode 2: window geometry over the predecessor and the start layer's filter
    int wy, wx, Sy, Sx, Py, Px;
    int kh, kw, sh, sw, ph, pw, dense;
    int Cs;                // channels of the start layer
    const float* wt;       // [tap][Cs][C] (predecessor channels innermost); dense: [Cs][nelem]
    const float* bias;     // [Cs]
    const double* eta;     // mode 2: [batch][n_start] float32 evaluation error of the start neurons (added to c); null: none
    double* c; double* err; double* best;
    int seeded;            // best already holds the rows' interval image: leave it
    int coef64;            // out holds float64 values
    FastDiv div_C, div_wx; // filled by the launcher
};

struct ReluParams {
    const double* plo; const double* phi;   // predecessor intervals [total]
    double* lo; double* hi;                 // this layer's intervals
    float* grl;                             // packed relaxation (slope, lower choice)
    double* rho; double* kap;               // u/slope and intercept/slope, rounded up (see scan kernel)
    double* xmax; int* flag;
    long long total;                        // batch * n
    long long n;                            // neurons per box
    double margin;                          // relative margin of rho and kap: 2^-22 for float32 storage, 2^-50 for float64
};

struct FinalizeParams {
    RowMap rm;
    const double* best;
    double* lo; double* hi;   // [batch][n_start] of the start layer
    double* xmax;             // [batch] running max of |bounds| of that layer, per box
    int* flag;                // set to 1 on NaN/Inf
    double widen;             // each end moves outward by widen*|end| (a sum layer's one float32 rounding); 0: none
    int has_relu;             // a ReLU layer reads this layer: its intervals and relaxation (relu, plo/phi unused) are
    ReluParams relu;          //   written by the same launch, neuron by neuron, as relu_kernel would write them
};


struct BoxParams {
    const float* centers;   // [batch][n] in C,H,W order (device)
    float eps, clip_lo, clip_hi;
    double* lo; double* hi;  // [batch][n] in H,W,C order
    double* xmax; int* flag;
    int C, H, W, batch;
};

// ---- early termination (Sections 3.2 and 4.2) ---------------------------------------------------------
struct IvalParams {          // forward interval analysis of an affine layer
    const double* plo; const double* phi;   // predecessor intervals [batch][Hi*Wi*Ci], H,W,C order
    const float* wt;         // [tap][C][Ci] (dense: [C][n_in], seen as one tap over a 1x1 layer with n_in channels)
    const float* bias;       // [C]
    double pool_scale;       // 0: a layer with weights; else average pooling (C == Ci, wt and bias unused): 1/(kh*kw)
    double* lo; double* hi;  // [batch][H*W*C]; null: intervals not wanted
    double* eta;             // [batch][H*W*C] out: float32 evaluation error of each neuron (also widens lo, hi); null: none
    int* flag;
    int Hi, Wi, Ci, H, W, C, kh, kw, sh, sw, ph, pw, batch;
};
struct SumEtaParams {        // out = u*max(|lo|,|hi|) + ea + eb (each part optional), rounded up
    const double *lo, *hi; double u;
    const double *ea, *eb;
    double* out;
    long long total;
};
struct AddIvalParams {       // sum layer: interval sum, rounded outward
    const double *alo, *ahi, *blo, *bhi;
    double *lo, *hi;
    long long total;
    int* flag;
    double widen;            // relative outward widening of each end (one float32 rounding); 0: none
};
struct SeedParams {          // best[r] = upper end, best[Rc0 + r] = -(lower end) of task row0 + r
    const double* lo; const double* hi;
    double* best;
    int row0, Rc0;
};
struct TermParams {          // termination criterion per task of the chunk, and the number of tasks kept per 256
    const double* best; int Rc0;
    const int* rowid; int Ra;            // current compact list (null: identity) and its length
    unsigned char* done;                 // [Ra] in/out
    int* term_layer;                     // [batch * n_start]: layer at which a task met the criterion
    int row0, key, first, may_stop;      // first: before any step (done has no previous value; tasks kept get 0)
    int* wgcount;                        // [ceil(Ra/256)] tasks kept per work-group
};
struct CompactParams {       // order-preserving removal of the tasks that are done
    const unsigned char* done; const int* wgoffset; int Ra;
    const int* rowid_old; int* rowid_new; int* sel;      // sel[new] = old compact position
    const double *c_old, *err_old; double *c_new, *err_new;   // both halves ([2*Ra] -> [2*Ra_new]); null before the first step
    const int* count;        // device: Ra_new
    int nsign;
    unsigned char* done_new; // [Ra_new] cleared
};
struct CopyRowsParams {      // dst row (h*Ra_new + i) = src row (h*Ra_old + sel[i])
    const float* src; float* dst; const int* sel;
    int Ra_old, Ra_new, nsign, nelem;
};

// ---- fused chain of narrow dense layers (chain.hip): one launch carries the rows of a start layer through every step
constexpr int kMaxChainSteps = 16;
struct ChainStep {           // the block after this step and the constants of its candidate (cf. ScanParams)
    int n;                   // coefficients per row: neurons of the layer the block ranges over
    int K;                   // contraction length of the product that makes the block (n of the step before); step 0: unused
    const float* w;          // [n][K] matrix of the dense layer crossed (the crossing layout of its weights); step 0: null
    const float* grl;        // [batch][n] packed ReLU relaxation substituted into the new coefficients; null: none
    const double *cpos, *cneg, *xlo, *xhi;   // [batch][n]
    const double* kap;       // [batch][n] or null
    const double* beff;      // [n] or null
    const double* xmax_self; // [batch] or null
    const double* xmax_a;    // [batch] or null
    double e1_a;
    double round_coef;
    int do_consts;
};
struct ChainParams {
    ChainStep steps[kMaxChainSteps];
    int nsteps;
    const float* w0;         // the start layer's matrix [n_start][steps[0].n] (float32) and bias [n_start]
    const float* bias0;
    int row0, Rc, n_start;   // tasks row0 .. row0+Rc of batch * n_start
    FastDiv div_n;
    int hid_stride, last_stride;   // LDS row strides (floats): every block but the last one / the last one
    double coef_floor;
    double* lo; double* hi;  // [batch][n_start] bounds of the start layer
    double* xmax; int* flag;
    int has_relu;            // as in FinalizeParams
    ReluParams relu;
};
bool launch_chain(const ChainParams& p, hipStream_t s);
size_t chain_lds_bytes(const ChainParams& p);

// ---- literal interval-coefficient mode (interval.hip): blocks hold [lo, hi] pairs of float64
struct IvRowParams {         // per-row passes over a block of interval coefficients
    BlockDesc blk;           // data: [nrows][wy][wx][C] pairs of doubles
    RowMap rm;
    int nrows;
    int batch_stride;        // neurons per box of the layer the block ranges over
    const double* xlo;       // [batch][n] intervals: of the block's layer (candidate) / of the ReLU's input layer (substitution)
    const double* xhi;
    const float* grl;        // [batch][n] packed relaxation of the ReLU layer (substitution)
    const double* beff;      // [C] bias of the affine layer(s) crossed next (constants)
    double* c;               // per-row constant (upper end)
    double* best;            // per-row best candidate
};
void launch_iv_init(const InitParams& p, hipStream_t s);
void launch_iv_cand(const IvRowParams& p, hipStream_t s);
void launch_iv_relu(const IvRowParams& p, hipStream_t s);
void launch_iv_bias(const IvRowParams& p, hipStream_t s);
void launch_iv_cross(const CrossParams& p, hipStream_t s);    // in/out/add hold interval pairs; out_grl, wt64 unused

void launch_cross(const CrossParams& p, hipStream_t s);
void launch_scan(const ScanParams& p, hipStream_t s);
void launch_init(const InitParams& p, hipStream_t s);
void launch_finalize(const FinalizeParams& p, hipStream_t s);
void launch_relu(const ReluParams& p, hipStream_t s);
void launch_box(const BoxParams& p, hipStream_t s);
void launch_fill_f64(double* p, double v, long long n, hipStream_t s);
void launch_fill_i32(int* p, int v, long long n, hipStream_t s);
void launch_ival(const IvalParams& p, hipStream_t s);
void launch_add_ival(const AddIvalParams& p, hipStream_t s);
void launch_sum_eta(const SumEtaParams& p, hipStream_t s);
void launch_seed(const SeedParams& p, hipStream_t s);
void launch_term(const TermParams& p, int* count, hipStream_t s);      // flags, counts, scan; *count (device) = tasks kept
void launch_compact(const CompactParams& p, hipStream_t s);
void launch_copy_rows(const CopyRowsParams& p, hipStream_t s);
void launch_margins(const double* best, float* margins, long long n, int* flag, hipStream_t s);
// float64 MFMA self-check: D[16][16] = A[16][K] * B[K][16], same instruction and layout as the crossing kernel
void launch_mfma_check(const double* A, const double* B, double* D, int K, hipStream_t s);
// the same for the 4-column instruction (4x4x4, four blocks): D[16][4] = A[16][K] * B[K][4]
void launch_mfma4_check(const double* A, const double* B, double* D, int K, hipStream_t s);

}  // namespace gp

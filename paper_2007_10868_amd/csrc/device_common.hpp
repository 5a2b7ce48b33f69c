// Device-side helpers shared by the kernel files: how a row of a launch maps to its neuron, range-checked buffer
// loads, the packed ReLU relaxation.
#pragma once
#include "kernels.hpp"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <type_traits>

namespace gp {

typedef double double4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return min(max(v, lo), hi); }

struct RowInfo {
    int b, ys, xs, cs;
    float sign;
};

__device__ __forceinline__ RowInfo row_info(const RowMap& rm, int r) {
    RowInfo ri;
    int rr = r;
    ri.sign = 1.f;
    if (r >= rm.Rc) {
        rr = r - rm.Rc;
        ri.sign = -1.f;
    }
    if (rm.rowid) rr = rm.rowid[rr];
    const uint32_t g = (uint32_t)(rm.row0 + rr);
    const uint32_t b = fast_div(g, rm.div_n);
    const uint32_t i = g - b * (uint32_t)rm.n_start;
    const uint32_t pos = fast_div(i, rm.div_c);
    const uint32_t ys = fast_div(pos, rm.div_w);
    ri.b = (int)b;
    ri.cs = (int)(i - pos * (uint32_t)rm.Cs);
    ri.ys = (int)ys;
    ri.xs = (int)(pos - ys * (uint32_t)rm.Ws);
    return ri;
}

// where row r keeps its best candidate: the layout of the chunk before any row was removed
__device__ __forceinline__ int best_index(const RowMap& rm, int r) {
    const int half = r >= rm.Rc ? 1 : 0;
    int rr = r - half * rm.Rc;
    if (rm.rowid) rr = rm.rowid[rr];
    return half * rm.Rc0 + rr;
}

typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));

struct F4 {
    float v[4];
};

// a value every lane of the wave holds alike, moved to scalar registers: what is derived from it (loop bounds, tap
// numbers, scalar offsets and resource descriptors of buffer loads) then stays scalar; left in vector registers the
// compiler would wrap every such load into a loop over the distinct values
__device__ __forceinline__ unsigned long long wave_uniform(unsigned long long v) {
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}

constexpr uint32_t kOOB = 0x80000000u;   // byte offset beyond every buffer range: the load returns 0

// 4 consecutive floats at byte offset `off` of a buffer resource; offsets beyond the resource's range
// read as 0 (hardware range check), so invalid taps / rows / channels need no masking instructions.
template <bool VEC>
__device__ __forceinline__ F4 buf_ld4(__amdgpu_buffer_rsrc_t rsrc, uint32_t off, int nvalid) {
    F4 r;
    if (VEC) {
        uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
        r.v[0] = __uint_as_float(v.x); r.v[1] = __uint_as_float(v.y);
        r.v[2] = __uint_as_float(v.z); r.v[3] = __uint_as_float(v.w);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t o = (j < nvalid) ? off + 4u * j : kOOB;
            r.v[j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)o, 0, 0));
        }
    }
    return r;
}

// the same for float64 storage (32 bytes): r receives the 4 values
typedef unsigned int uint2_t __attribute__((ext_vector_type(2)));
template <bool VEC>
__device__ __forceinline__ void buf_ld4_f64(__amdgpu_buffer_rsrc_t rsrc, uint32_t off, int nvalid, double (&r)[4]) {
    if (VEC) {
        const uint4_t v0 = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
        const uint4_t v1 = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(off == kOOB ? kOOB : off + 16u), 0, 0);
        r[0] = __hiloint2double((int)v0.y, (int)v0.x); r[1] = __hiloint2double((int)v0.w, (int)v0.z);
        r[2] = __hiloint2double((int)v1.y, (int)v1.x); r[3] = __hiloint2double((int)v1.w, (int)v1.z);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t o = (j < nvalid && off != kOOB) ? off + 8u * j : kOOB;
            const uint2_t v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)o, 0, 0);
            r[j] = __hiloint2double((int)v.y, (int)v.x);
        }
    }
}

// ReLU relaxation of one neuron packed in one float: |g| is the slope of the upper line, the sign bit
// is set when the lower line is 0 (lam = 0) and clear when it is x (lam = 1).
// A coefficient a over relu(x) becomes a * relax_factor(a, g) over x (Section 2: positive coefficients
// take the upper line, negative ones the lower line, for an upper bound).
__device__ __forceinline__ float relax_factor(double a, float g) {
    return a >= 0.0 ? fabsf(g) : (signbit(g) ? 0.f : 1.f);
}

// ---- arithmetic of the per-row reductions over a block, shared by the scan kernels and the fused chain kernel ---------------
// One coefficient's contribution to the five per-row sums.  Written with explicit fused multiply-adds only, so that
// every scan kernel performs exactly the same operations in the same order per lane and a row's result does not
// depend on which kernel (i.e. on how many rows share the launch) handled it.
template <typename CT>
__device__ __forceinline__ void scan_term(bool has_cand, bool do_consts, CT mf, double cp, double cn, double X, double kp,
                                          double be, double& cand, double& absx, double& cst, double& cstabs, double& s1) {
    const double m = (double)mf;
    const double am = fabs(m);
    if (has_cand) {
        cand = fma(m, mf >= (CT)0 ? cp : cn, cand);
        absx = fma(am, X, absx);
    }
    if (do_consts) {
        const double mp = fmax(m, 0.0);
        cst = fma(m, be, fma(mp, kp, cst));
        cstabs = fma(am, fabs(be), fma(mp, kp, cstabs));
        s1 += am;
    }
}


// Per-row bookkeeping after the reductions (Section 2: candidate bounds; Section 4.1: the rounding slack): slack of the
// stored coefficients, candidate folded into best, constants of the next step added to c, slack of the next accumulation.
//   floor_x: coef_floor * xmax of the block's own layer (0: exact block); e1: accumulation-error constant of the next
//   crossing(s) times the largest magnitude of their input layer.
__device__ __forceinline__ void scan_finish_math(int nelem, double round_coef, double floor_x, bool has_cand, bool do_consts,
                                                 double e1, double t_cand, double t_absx, double t_cst, double t_cstabs,
                                                 double t_s1, double& c, double& err, double& best) {
    // a sum of n float64 terms in any order is off by at most (n-1)*2^-53*sum|terms|*(1+tiny)
    const double esum = (double)(nelem + 16) * 0x1p-52;
    // slack of the stored coefficients: |true - stored| <= round_coef*|stored| (+ subnormal floor)
    err += t_absx * round_coef * (1.0 + esum);
    // values below the float32 subnormal step vanish; with a substituted ReLU the lost coefficient is
    // up to 2^20 times larger (slopes are kept >= 2^-20)
    err += floor_x * (double)nelem;
    if (has_cand) {
        double v = c + t_cand + err;
        // (the candidate's terms are at most 3*|m|*X in magnitude when the multiplier comes as a difference, see
        // scan_term_staged)
        v += (fabs(c) + fabs(t_cand) + err) * 0x1p-50 + 3.0 * t_absx * esum;
        best = fmin(best, v);
    }
    if (do_consts) {
        const double cn = c + t_cst;
        err += t_cstabs * esum + (fabs(c) + fabs(t_cst)) * 0x1p-51 + t_s1 * e1 * (1.0 + esum);
        c = cn;
    }
    err *= (1.0 + 0x1p-48);   // the few float64 operations above
}

// ReLU layer, one neuron: intervals [max(l,0), max(u,0)] and the relaxation  lam*x <= relu(x) <= gam*x + del  (Section 2,
// ReLU transformer).  Any gam in [0,1] is sound when del >= max(-gam*l, u - gam*u); gam is the float32 nearest to
// u/(u-l).  Returns the neuron's largest magnitude (0 when not finite).  Shared by relu_kernel and by the kernels that
// store a layer's bounds and know that a ReLU layer reads them.
__device__ __forceinline__ double relu_neuron(const ReluParams& p, long long i, double l, double u) {
    if (!isfinite(l) || !isfinite(u)) *p.flag = 1;
    p.lo[i] = fmax(l, 0.0);
    p.hi[i] = fmax(u, 0.0);
    float g, lam;
    double rho = 0.0, kap = 0.0;
    if (l >= 0.0) { g = 1.f; lam = 1.f; rho = u; }
    else if (u <= 0.0) { g = 0.f; lam = 0.f; }
    else {
        g = (float)(u / (u - l));
        g = fminf(fmaxf(g, 0x1p-20f), 1.f);       // a positive coefficient must stay recoverable from its product with g
        const double gd = (double)g;
        const double d1 = -gd * l, d2 = u - gd * u;     // each off by a few ulps at most
        double d = fmax(d1, d2);
        d = d + (fabs(d) + fabs(u)) * 0x1p-50 + 0x1p-1000;
        lam = (u > -l) ? 1.f : 0.f;
        // rounded up, including the rounding of the stored product coefficient*g (p.margin: four roundings of the
        // storage type)
        rho = (u / gd) * (1.0 + p.margin);
        kap = (d / gd) * (1.0 + p.margin);
    }
    p.grl[i] = lam != 0.f ? g : -g;      // -0.0f encodes slope 0 with lam = 0
    p.rho[i] = rho;
    p.kap[i] = kap;
    double x = fmax(u, 0.0);
    if (!isfinite(x)) x = 0.0;
    return x;
}

}  // namespace gp

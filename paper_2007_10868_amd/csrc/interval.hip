// The paper's literal floating-point scheme (Section 4.1): every coefficient of an expression is an INTERVAL, lower
// ends are rounded towards -inf and upper ends towards +inf in every operation, weights stay scalars, and the intervals
// are kept until the end of the back-substitution (nothing is re-centred on the way).  A mode for tightness studies on
// small networks (gp_set_interval_coefficients), not a fast path: plain float64 vector arithmetic, one thread per new
// coefficient, the same plans, windows and residual joins as the default path (Sections 3.1, 4.3, Algorithm 1).
//
// Directed rounding.  The matrix instructions have no rounding control, the vector unit has: the wave's MODE register
// holds the rounding mode of float64 operations.  Every kernel here switches it to round-towards-+inf at its start
// (the mode is per wave and ends with it) and does ALL its interval arithmetic through up_add / up_mul below, written
// as single instructions the compiler can neither contract, reorder across the switch, nor fold; a lower end is
// obtained as -up(-x), which is exact negation around an upward-rounded operation.
#include "device_common.hpp"

namespace gp {

namespace {

struct Iv {            // one interval coefficient
    double lo, hi;
};

__device__ __forceinline__ void round_up_mode() {
    // hwreg(MODE, offset 2, size 2): rounding of float64 (and float16) operations; 1 = towards +inf
    __builtin_amdgcn_s_setreg((1 << 11) | (2 << 6) | 1, 1);
}
__device__ __forceinline__ double up_add(double a, double b) {
    double r;
    asm volatile("v_add_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ double up_mul(double a, double b) {
    double r;
    asm volatile("v_mul_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ double dn_add(double a, double b) { return -up_add(-a, -b); }
__device__ __forceinline__ double dn_mul(double a, double b) { return -up_mul(-a, b); }

// acc += [a.lo, a.hi] * w for a scalar w of either sign, outward
__device__ __forceinline__ void acc_scaled(Iv& acc, const Iv a, double w) {
    if (w >= 0.0) { acc.lo = dn_add(acc.lo, dn_mul(a.lo, w)); acc.hi = up_add(acc.hi, up_mul(a.hi, w)); }
    else          { acc.lo = dn_add(acc.lo, dn_mul(a.hi, w)); acc.hi = up_add(acc.hi, up_mul(a.lo, w)); }
}
// upper end of [a.lo, a.hi] * [L, U]
__device__ __forceinline__ double up_image(const Iv a, double L, double U) {
    return fmax(fmax(up_mul(a.lo, L), up_mul(a.lo, U)), fmax(up_mul(a.hi, L), up_mul(a.hi, U)));
}
// sum over the lanes of a wave, rounded up at every addition
__device__ __forceinline__ double wave_sum_up(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = up_add(v, __shfl_xor(v, off, 64));
    return v;
}

// neuron (index inside its box) that element e of a row's block stands over
__device__ __forceinline__ long long block_neuron(const BlockDesc& B, const RowInfo& ri, int e) {
    const int pix = e / B.C, c = e - pix * B.C;
    const int a = pix / B.wx, b = pix - a * B.wx;
    const int oy = clampi(B.Sy * ri.ys - B.Py, 0, B.H - B.wy), ox = clampi(B.Sx * ri.xs - B.Px, 0, B.W - B.wx);
    return ((long long)(oy + a) * B.W + (ox + b)) * B.C + c;
}

}  // namespace

// ---- initial block (Section 2: the neuron's own affine expression; modes as in InitParams): exact point intervals
__global__ __launch_bounds__(256) void iv_init_kernel(const InitParams p) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= p.nrows) return;
    const RowInfo ri = row_info(p.rm, r);
    Iv* out = reinterpret_cast<Iv*>(p.out) + (size_t)r * p.nelem;
    for (int e = threadIdx.x & 63; e < p.nelem; e += 64) {
        double v = 0.0;
        if (p.mode == 0) {
            v = (e == ri.cs) ? (double)ri.sign : 0.0;
        } else if (p.mode == 1) {
            const int label = p.labels[ri.b];
            const int j = ri.cs + (ri.cs >= label ? 1 : 0);
            const int pix = e / p.C, c = e - pix * p.C;
            const int chw = c * (p.H * p.W) + pix;
            if (chw == j) v = 1.0;
            else if (chw == label) v = -1.0;
        } else if (p.mode == 3) {
            const int pix = e / p.C, c = e - pix * p.C;
            v = -(double)p.forms[(size_t)ri.cs * p.nelem + (size_t)c * (p.H * p.W) + pix];
        } else if (p.dense) {
            v = (double)(ri.sign * p.wt[(size_t)ri.cs * p.nelem + e]);
        } else {
            const int pix = e / p.C, c = e - pix * p.C;
            const int a = pix / p.wx, bb = pix - a * p.wx;
            const int A = clampi(p.Sy * ri.ys - p.Py, 0, p.H - p.wy) + a;
            const int B = clampi(p.Sx * ri.xs - p.Px, 0, p.W - p.wx) + bb;
            const int f = A - (ri.ys * p.sh - p.ph), g = B - (ri.xs * p.sw - p.pw);
            if (f >= 0 && f < p.kh && g >= 0 && g < p.kw)
                v = (double)(ri.sign * p.wt[((size_t)(f * p.kw + g) * p.Cs + ri.cs) * p.C + c]);
        }
        out[e] = Iv{v, v};
    }
    if ((threadIdx.x & 63) == 0) {
        p.c[r] = (p.mode == 2) ? (double)(ri.sign * p.bias[ri.cs]) : (p.mode == 3 && p.offsets) ? -(double)p.offsets[ri.cs] : 0.0;
        p.best[r] = INFINITY;
    }
}

// ---- candidate bound (Section 2): upper end of c + sum_j [a_j, b_j] * [L_j, U_j]; one wave per row
__global__ __launch_bounds__(256) void iv_cand_kernel(const IvRowParams p) {
    round_up_mode();
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= p.nrows) return;
    const RowInfo ri = row_info(p.rm, r);
    const int nelem = p.blk.wy * p.blk.wx * p.blk.C;
    const Iv* src = reinterpret_cast<const Iv*>(p.blk.data) + (size_t)r * nelem;
    const long long base = (long long)ri.b * p.batch_stride;
    double acc = 0.0;
    for (int e = threadIdx.x & 63; e < nelem; e += 64) {
        const Iv a = src[e];
        if (a.lo == 0.0 && a.hi == 0.0) continue;
        const long long j = base + block_neuron(p.blk, ri, e);
        acc = up_add(acc, up_image(a, p.xlo[j], p.xhi[j]));
    }
    acc = wave_sum_up(acc);
    if ((threadIdx.x & 63) == 0) {
        const double v = up_add(p.c[r], acc);
        p.best[r] = fmin(p.best[r], v);
    }
}

// ---- ReLU substitution (Section 2: positive coefficients take the upper line, negative ones the lower line), in place.
// The block over the ReLU layer becomes a block over its input layer; intercepts and the images of coefficients whose
// interval straddles 0 go into the row's constant.  xlo/xhi: intervals of the ReLU's INPUT layer; grl: packed relaxation.
__global__ __launch_bounds__(256) void iv_relu_kernel(const IvRowParams p) {
    round_up_mode();
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= p.nrows) return;
    const RowInfo ri = row_info(p.rm, r);
    const int nelem = p.blk.wy * p.blk.wx * p.blk.C;
    Iv* blk = reinterpret_cast<Iv*>(const_cast<float*>(p.blk.data)) + (size_t)r * nelem;
    const long long base = (long long)ri.b * p.batch_stride;
    double acc = 0.0;
    for (int e = threadIdx.x & 63; e < nelem; e += 64) {
        Iv a = blk[e];
        if (a.lo == 0.0 && a.hi == 0.0) continue;
        const long long j = base + block_neuron(p.blk, ri, e);
        const double l = p.xlo[j], u = p.xhi[j];
        if (l >= 0.0) continue;                                  // y = x exactly
        if (u <= 0.0) { blk[e] = Iv{0.0, 0.0}; continue; }        // y = 0 exactly
        const float gp_ = p.grl[j];
        const double g = (double)fabsf(gp_);                     // slope of the upper line; any value in [0,1] is sound with
        const bool lam = !signbit(gp_);                           // the intercept below.  lam: the lower line is x (else 0)
        if (a.lo >= 0.0) {
            const double d = fmax(up_mul(-l, g), up_add(u, -dn_mul(g, u)));     // max(-g*l, u - g*u), rounded up
            acc = up_add(acc, up_mul(a.hi, d));
            blk[e] = Iv{dn_mul(a.lo, g), up_mul(a.hi, g)};
        } else if (a.hi <= 0.0) {
            if (!lam) blk[e] = Iv{0.0, 0.0};
        } else {                                                 // sign unknown: the term's image over y in [0, u]
            acc = up_add(acc, up_image(a, 0.0, u));
            blk[e] = Iv{0.0, 0.0};
        }
    }
    acc = wave_sum_up(acc);
    if ((threadIdx.x & 63) == 0) p.c[r] = up_add(p.c[r], acc);
}

// ---- constants of the next product(s): c += sum_j [a_j, b_j] * bias_{channel(j)} (upper end)
__global__ __launch_bounds__(256) void iv_bias_kernel(const IvRowParams p) {
    round_up_mode();
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= p.nrows) return;
    const int nelem = p.blk.wy * p.blk.wx * p.blk.C;
    const Iv* src = reinterpret_cast<const Iv*>(p.blk.data) + (size_t)r * nelem;
    double acc = 0.0;
    for (int e = threadIdx.x & 63; e < nelem; e += 64) {
        const Iv a = src[e];
        const double be = p.beff[e % p.blk.C];
        acc = up_add(acc, be >= 0.0 ? up_mul(a.hi, be) : up_mul(a.lo, be));
    }
    acc = wave_sum_up(acc);
    if ((threadIdx.x & 63) == 0) p.c[r] = up_add(p.c[r], acc);
}

// ---- one back-substitution step through an affine layer (Section 2: M^{k-1} = M^k F^k; Algorithm 1 for the index map of
// a convolution), gather form: one thread per new coefficient (row, window pixel, input channel) adds, for every filter
// tap that reaches its pixel from inside the row's window and every output channel d, [M] * F outward; then the other
// branch's block where a residual block is joined.
__global__ __launch_bounds__(256) void iv_cross_kernel(const CrossParams p) {
    round_up_mode();
    const int opix = p.owy * p.owx;
    const long long total = (long long)p.nrows * opix * p.Co;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx % p.Co);
    const long long t = idx / p.Co;
    const int pix = (int)(t % opix);
    const int r = (int)(t / opix);
    const RowInfo ri = row_info(p.rm, r);
    const int pa = pix / p.owx, pb = pix - pa * p.owx;
    const int A = clampi(p.oSy * ri.ys - p.oPy, 0, p.Ho - p.owy) + pa;       // absolute position in the layer's input
    const int B = clampi(p.oSx * ri.xs - p.oPx, 0, p.Wo - p.owx) + pb;
    const int oiy = clampi(p.in.Sy * ri.ys - p.in.Py, 0, p.in.H - p.in.wy), oix = clampi(p.in.Sx * ri.xs - p.in.Px, 0, p.in.W - p.in.wx);
    const int Ck = p.in.C;
    const Iv* in = reinterpret_cast<const Iv*>(p.in.data) + (size_t)r * p.in.wy * p.in.wx * Ck;
    Iv acc = {0.0, 0.0};
    for (int f = 0; f < p.kh; ++f) {
        const int yy = A + p.ph - f;
        if (yy < 0 || yy % p.sh) continue;
        const int y = yy / p.sh - oiy;
        if (y < 0 || y >= p.in.wy) continue;
        for (int g = 0; g < p.kw; ++g) {
            const int xx = B + p.pw - g;
            if (xx < 0 || xx % p.sw) continue;
            const int x = xx / p.sw - oix;
            if (x < 0 || x >= p.in.wx) continue;
            const Iv* m = in + (size_t)(y * p.in.wx + x) * Ck;
            if (p.pool_scale != 0.0) {
                // average pooling: the weight 1/(kh*kw) is known as w_dn <= 1/(kh*kw) <= w_up, both positive
                const Iv a = m[c];
                const double w_dn = nextafter(p.pool_scale, 0.0), w_up = nextafter(p.pool_scale, 1.0);
                acc.lo = dn_add(acc.lo, a.lo >= 0.0 ? dn_mul(a.lo, w_dn) : dn_mul(a.lo, w_up));
                acc.hi = up_add(acc.hi, a.hi >= 0.0 ? up_mul(a.hi, w_up) : up_mul(a.hi, w_dn));
            } else {
                const float* w = p.wt + ((size_t)(f * p.kw + g) * p.Co + c) * Ck;
                for (int d = 0; d < Ck; ++d) {
                    const Iv a = m[d];
                    if (a.lo == 0.0 && a.hi == 0.0) continue;
                    acc_scaled(acc, a, (double)w[d]);
                }
            }
        }
    }
    if (p.add.data) {
        const int ay = A - clampi(p.add.Sy * ri.ys - p.add.Py, 0, p.add.H - p.add.wy);
        const int ax = B - clampi(p.add.Sx * ri.xs - p.add.Px, 0, p.add.W - p.add.wx);
        if (ay >= 0 && ay < p.add.wy && ax >= 0 && ax < p.add.wx) {
            const Iv a = reinterpret_cast<const Iv*>(p.add.data)[((size_t)r * p.add.wy * p.add.wx + (size_t)(ay * p.add.wx + ax)) * p.Co + c];
            acc.lo = dn_add(acc.lo, a.lo);
            acc.hi = up_add(acc.hi, a.hi);
        }
    }
    reinterpret_cast<Iv*>(p.out)[idx] = acc;
}

void launch_iv_init(const InitParams& p, hipStream_t s) {
    if (p.nrows > 0 && p.nelem > 0) hipLaunchKernelGGL(iv_init_kernel, dim3((p.nrows + 3) / 4), dim3(256), 0, s, p);
}
void launch_iv_cand(const IvRowParams& p, hipStream_t s) {
    if (p.nrows > 0) hipLaunchKernelGGL(iv_cand_kernel, dim3((p.nrows + 3) / 4), dim3(256), 0, s, p);
}
void launch_iv_relu(const IvRowParams& p, hipStream_t s) {
    if (p.nrows > 0) hipLaunchKernelGGL(iv_relu_kernel, dim3((p.nrows + 3) / 4), dim3(256), 0, s, p);
}
void launch_iv_bias(const IvRowParams& p, hipStream_t s) {
    if (p.nrows > 0) hipLaunchKernelGGL(iv_bias_kernel, dim3((p.nrows + 3) / 4), dim3(256), 0, s, p);
}
void launch_iv_cross(const CrossParams& p, hipStream_t s) {
    const long long total = (long long)p.nrows * p.owy * p.owx * p.Co;
    if (total > 0) hipLaunchKernelGGL(iv_cross_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p);
}

}  // namespace gp
